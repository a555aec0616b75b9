"""CPU oracle of the SPRINTER draft -> verifier -> conditional-target decode loop.

TEST INFRASTRUCTURE ONLY.  Plain NumPy in float64, written from the paper
(Sec. 3 "Algorithm", Alg. 1, Alg. 2 in App. "Full SPRINTER Algorithm") to be
checked against it by eye: no blocking, fusion or reordering.  It shares no code
with the HIP path; only tests, the smoke check and the benchmark's CPU-baseline
leg may import it.

Pins (tests/test_oracle_*.py): Philox known-answer vectors of the published
generator; Gumbel-max chi-square against softmax; transformer special cases
(one key, uniform scores, RoPE at position 0, norm statistics, GQA == MHA with
repeated heads, cached == uncached forward); the five loop invariants (accept
rule, target placement, lengths, tau=0 == pure draft, tau>1 == pure target);
run-length law and stopping time of Thm 3.2 / Thm 3.3 with an i.i.d. verifier;
output mixture law; brute-force compaction; for standard speculative decoding
(sd_baseline.py): tokens-per-round closed form, target-chain law, stream pattern
with identical models, uncached re-derivation of every committed token.
Parity unpinned: the FLOP counts of Table 5 and the latencies of Table 2 (the
paper does not state the accounting / hardware); they are not computed here.
"""
