// Runs a workload file written by dump_workload.py through the C ABI of libsprinter: prefill, warm-up steps,
// timed decode steps.  No Python in the process, so that hardware counters can be collected around it
// (rocprofv3 --pmc ... -- native_bench file --steps K --warmup W).  With --copy-calibration it first runs a plain
// copy kernel over 256 MiB (k_copy_calibration): the counters' scale on this machine follows from its known size.
#include "../../include/sprinter.h"
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 1; } } while (0)
#define SP(x) do { int rc_ = (x); if (rc_ != 0) { fprintf(stderr, "sprinter error %d: %s (%s:%d)\n", rc_, sprinter_last_error(ctx), __FILE__, __LINE__); return 1; } } while (0)

__global__ void k_copy_calibration(const float4* __restrict__ src, float4* __restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

struct Tensor { int which; std::string name; long long rows, cols; int es; long long off, nbytes; };

static bool read_model(FILE* f, sprinter_model_cfg* m) {
  return fscanf(f, "%d %d %d %d %d %d %d %d %f %f", &m->arch, &m->n_layer, &m->d_model, &m->n_head, &m->n_kv_head, &m->d_ff,
                &m->vocab, &m->max_pos, &m->norm_eps, &m->rope_theta) == 10;
}

int main(int argc, char** argv) {
  if (argc < 2) { fprintf(stderr, "usage: native_bench workload.sprw [--steps K] [--warmup W] [--copy-calibration]\n"); return 2; }
  int steps = 64, warmup = 16;
  bool calib = false;
  for (int i = 2; i < argc; ++i) {
    if (!strcmp(argv[i], "--steps") && i + 1 < argc) steps = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--warmup") && i + 1 < argc) warmup = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--copy-calibration")) calib = true;
    else { fprintf(stderr, "unknown argument %s\n", argv[i]); return 2; }
  }
  FILE* f = fopen(argv[1], "rb");
  if (!f) { perror(argv[1]); return 1; }
  char word[256];
  sprinter_cfg cfg;
  memset(&cfg, 0, sizeof cfg);
  int B = 0, P = 0;
  std::vector<int> plen;
  std::vector<Tensor> tensors;
  long long prompts_off = -1, prompts_bytes = 0;
  if (fscanf(f, "%255s", word) != 1 || strcmp(word, "SPRW1")) { fprintf(stderr, "not a workload file\n"); return 1; }
  while (fscanf(f, "%255s", word) == 1 && strcmp(word, "end")) {
    if (!strcmp(word, "draft")) { if (!read_model(f, &cfg.draft)) return 1; }
    else if (!strcmp(word, "target")) { if (!read_model(f, &cfg.target)) return 1; }
    else if (!strcmp(word, "cfg")) {
      unsigned long long seed;
      if (fscanf(f, "%d %d %d %d %d %f %f %llu %d %d", &cfg.ver_d_in, &cfg.ver_d_hidden, &cfg.dtype, &cfg.max_batch, &cfg.max_seq,
                 &cfg.tau, &cfg.temperature, &seed, &cfg.target_ctx_mode, &cfg.reject_mode) != 10) return 1;
      cfg.seed = seed;
    } else if (!strcmp(word, "batch")) { if (fscanf(f, "%d %d", &B, &P) != 2) return 1; }
    else if (!strcmp(word, "plen")) { plen.resize(B); for (int b = 0; b < B; ++b) if (fscanf(f, "%d", &plen[b]) != 1) return 1; }
    else if (!strcmp(word, "tensor")) {
      Tensor t; char name[128];
      if (fscanf(f, "%d %127s %lld %lld %d %lld %lld", &t.which, name, &t.rows, &t.cols, &t.es, &t.off, &t.nbytes) != 7) return 1;
      t.name = name; tensors.push_back(t);
    } else if (!strcmp(word, "prompts")) { if (fscanf(f, "%lld %lld", &prompts_off, &prompts_bytes) != 2) return 1; }
    else { fprintf(stderr, "unknown header record %s\n", word); return 1; }
  }
  long long data0 = (ftell(f) + 1 + 4095) / 4096 * 4096;      // header is padded to a multiple of 4096
  if (B < 1 || (int)plen.size() != B || prompts_off < 0) { fprintf(stderr, "incomplete header\n"); return 1; }

  hipStream_t stream;
  CK(hipStreamCreate(&stream));
  if (calib) {
    const size_t bytes = (size_t)256 << 20;
    float4 *src, *dst;
    CK(hipMalloc(&src, bytes)); CK(hipMalloc(&dst, bytes));
    CK(hipMemset(src, 1, bytes));
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(k_copy_calibration, dim3(4096), dim3(256), 0, stream, src, dst, bytes / 16);
    CK(hipStreamSynchronize(stream));
    CK(hipFree(src)); CK(hipFree(dst));
  }
  // tensors: file -> pinned staging -> device
  std::vector<void*> dev(tensors.size(), nullptr);
  size_t biggest = (size_t)prompts_bytes;
  for (const Tensor& t : tensors) if ((size_t)t.nbytes > biggest) biggest = (size_t)t.nbytes;
  void* stage;
  CK(hipHostMalloc(&stage, biggest, hipHostMallocDefault));
  for (size_t i = 0; i < tensors.size(); ++i) {
    const Tensor& t = tensors[i];
    CK(hipMalloc(&dev[i], (size_t)t.nbytes));
    if (fseek(f, data0 + t.off, SEEK_SET) || fread(stage, 1, (size_t)t.nbytes, f) != (size_t)t.nbytes) { fprintf(stderr, "short read of %s\n", t.name.c_str()); return 1; }
    CK(hipMemcpy(dev[i], stage, (size_t)t.nbytes, hipMemcpyHostToDevice));
  }
  int* d_prompts;
  CK(hipMalloc(&d_prompts, (size_t)prompts_bytes));
  if (fseek(f, data0 + prompts_off, SEEK_SET) || fread(stage, 1, (size_t)prompts_bytes, f) != (size_t)prompts_bytes) { fprintf(stderr, "short read of prompts\n"); return 1; }
  CK(hipMemcpy(d_prompts, stage, (size_t)prompts_bytes, hipMemcpyHostToDevice));
  fclose(f);

  sprinter_ctx* ctx = nullptr;
  size_t ws_bytes = 0;
  SP(sprinter_workspace_bytes(&cfg, &ws_bytes));
  void* ws;
  CK(hipMalloc(&ws, ws_bytes));
  SP(sprinter_create(&cfg, ws, ws_bytes, (void*)stream, &ctx));
  for (int which = 0; which < 3; ++which) {
    std::vector<const char*> names; std::vector<const void*> ptrs; std::vector<int64_t> shapes;
    for (size_t i = 0; i < tensors.size(); ++i)
      if (tensors[i].which == which) {
        names.push_back(tensors[i].name.c_str()); ptrs.push_back(dev[i]);
        shapes.push_back(tensors[i].rows); shapes.push_back(tensors[i].cols); shapes.push_back(0); shapes.push_back(0);
      }
    SP(sprinter_load_weights(ctx, which, names.data(), ptrs.data(), shapes.data(), (int)names.size()));
  }
  SP(sprinter_prefill(ctx, d_prompts, plen.data(), B, P));
  if (warmup > 0) SP(sprinter_generate(ctx, warmup, nullptr, nullptr, nullptr, nullptr));
  CK(hipStreamSynchronize(stream));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  CK(hipEventRecord(e0, stream));
  SP(sprinter_generate(ctx, steps, nullptr, nullptr, nullptr, nullptr));
  CK(hipEventRecord(e1, stream));
  CK(hipStreamSynchronize(stream));
  float ms = 0.f;
  CK(hipEventElapsedTime(&ms, e0, e1));
  sprinter_stats st;
  SP(sprinter_get_stats(ctx, &st, nullptr));
  printf("{\"steps\": %d, \"warmup\": %d, \"batch\": %d, \"ms_per_step\": %.4f, \"tokens_per_s\": %.1f, \"steps_total\": %lld, "
         "\"steps_with_target\": %lld, \"sum_rejected\": %lld}\n",
         steps, warmup, B, ms / steps, B * steps / (ms * 1e-3), (long long)st.steps, (long long)st.steps_with_target,
         (long long)st.sum_rejected);
  sprinter_destroy(ctx);
  return 0;
}
