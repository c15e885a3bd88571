// linear_bench: the benchmark's whole-image launch sequence driven from a plain C++ program through
// the C ABI (no Python, no PyTorch in the process), for runs under profilers that collect hardware
// counters: every library in the process then comes from one ROCm installation.  It times one
// whole image (decode steps of all layers, end-of-line evictions) with HIP events on the launch
// stream and, on request, first runs two kernels of known traffic -- a read-only pass and a copy
// -- as yardsticks for byte counters.
//   linear_bench <workload> [--full] [--calibrate-mib M] [--images R]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/linear_kv.h"
#include "../../include/linear_kv_diag.h"

#define CK(x)                                                                              \
  do {                                                                                     \
    hipError_t e_ = (x);                                                                   \
    if (e_ != hipSuccess) {                                                                \
      std::fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);  \
      return 1;                                                                            \
    }                                                                                      \
  } while (0)
#define LK(x)                                                                                        \
  do {                                                                                               \
    int rc_ = (x);                                                                                   \
    if (rc_ != LINEAR_OK) {                                                                          \
      std::fprintf(stderr, "%s failed: %s (line %d)\n", #x, linear_strerror(rc_), __LINE__);         \
      return 1;                                                                                      \
    }                                                                                                \
  } while (0)

struct Shape {
  const char* name;
  int layers, batch, heads, d, cond, n, h, budget, init, r, dtype;
};
static const Shape kShapes[] = {
    {"tiny-b", 1, 1, 4, 64, 8, 8, 8, 24, 4, 1, LINEAR_F32},
    {"llamagen-xl", 36, 64, 20, 64, 1, 24, 24, 96, 24, 1, LINEAR_BF16},
    {"janus-pro-1b", 24, 32, 16, 128, 64, 24, 24, 96, 24, 1, LINEAR_BF16},
    {"janus-pro-7b", 30, 32, 32, 128, 128, 24, 24, 96, 24, 1, LINEAR_BF16},
    {"lumina-mgpt-768", 32, 8, 32, 128, 256, 49, 48, 294, 49, 1, LINEAR_BF16},
};

// yardstick with known traffic: dst[i] = src[i] + 1 over 16-byte pieces
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    uint4 v = src[i];
    v.x += 1;
    dst[i] = v;
  }
}

int main(int argc, char** argv) {
  if (argc < 2) {
    std::fprintf(stderr, "usage: linear_bench <workload> [--full] [--calibrate-mib M] [--images R]\n");
    return 2;
  }
  const Shape* sh = nullptr;
  for (const Shape& s : kShapes)
    if (!std::strcmp(s.name, argv[1])) sh = &s;
  if (!sh) {
    std::fprintf(stderr, "unknown workload %s\n", argv[1]);
    return 2;
  }
  bool full = false;
  long calib_mib = 0;
  int images = 1;
  for (int i = 2; i < argc; ++i) {
    if (!std::strcmp(argv[i], "--full")) full = true;
    else if (!std::strcmp(argv[i], "--calibrate-mib") && i + 1 < argc) calib_mib = std::atol(argv[++i]);
    else if (!std::strcmp(argv[i], "--images") && i + 1 < argc) images = std::atoi(argv[++i]);
    else {
      std::fprintf(stderr, "unknown option %s\n", argv[i]);
      return 2;
    }
  }
  linear_cfg_t cfg = {};
  cfg.n_layers = sh->layers; cfg.batch = sh->batch; cfg.n_heads = sh->heads; cfg.head_dim = sh->d;
  cfg.n_cond = sh->cond; cfg.line_len = sh->n; cfg.n_lines = sh->h;
  cfg.budget = full ? sh->n * sh->h : sh->budget;
  cfg.n_init = sh->init; cfg.n_recent_lines = sh->r; cfg.dtype = sh->dtype;
  size_t cache_bytes = 0, scratch_bytes = 0;
  LK(linear_workspace_bytes(&cfg, &cache_bytes, &scratch_bytes));
  const int L = cfg.n_layers, P = cfg.batch * cfg.n_heads, N = cfg.line_len * cfg.n_lines;
  const size_t elem = cfg.dtype == LINEAR_BF16 ? 2 : 4, row = (size_t)cfg.head_dim * elem;
  hipStream_t stream;
  CK(hipStreamCreate(&stream));

  if (calib_mib > 0) {
    const size_t bytes = (size_t)calib_mib << 20;
    void *src, *dst;
    CK(hipMalloc(&src, bytes));
    CK(hipMalloc(&dst, bytes));
    CK(hipMemsetAsync(src, 1, bytes, stream));
    CK(hipStreamSynchronize(stream));
    const void* ks[1] = {src};
    const void* vs[1] = {dst};
    // read-only yardstick: reads `bytes` of src and `bytes` of dst, writes nothing
    LK(linear_probe_stream(ks, vs, 1, 1, (int32_t)(bytes / 4096), (int32_t)(bytes / 4096), 4096, stream));
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(4096), dim3(256), 0, stream, static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), bytes / 16);
    CK(hipGetLastError());
    CK(hipStreamSynchronize(stream));
    std::printf("calibration: stream_read_kernel read %zu bytes, wrote 0; calibration_copy_kernel read %zu, wrote %zu\n",
                2 * bytes, bytes, bytes);
    CK(hipFree(src));
    CK(hipFree(dst));
  }

  std::vector<void*> kc(L), vc(L), kcond(L), vcond(L);
  const size_t cond_bytes = (size_t)P * cfg.n_cond * row;
  for (int l = 0; l < L; ++l) {
    CK(hipMalloc(&kc[l], cache_bytes));
    CK(hipMalloc(&vc[l], cache_bytes));
    if (cond_bytes) {
      CK(hipMalloc(&kcond[l], cond_bytes));
      CK(hipMalloc(&vcond[l], cond_bytes));
      CK(hipMemsetAsync(kcond[l], 0x3c, cond_bytes, stream));   // finite values in either storage type
      CK(hipMemsetAsync(vcond[l], 0x3c, cond_bytes, stream));
    }
  }
  void *scratch, *q, *k, *v, *out;
  CK(hipMalloc(&scratch, scratch_bytes));
  const size_t step_bytes = (size_t)L * P * row;
  CK(hipMalloc(&q, step_bytes));
  CK(hipMalloc(&k, step_bytes));
  CK(hipMalloc(&v, step_bytes));
  CK(hipMalloc(&out, (size_t)L * P * cfg.head_dim * 4));
  CK(hipMemsetAsync(q, 0x3c, step_bytes, stream));
  CK(hipMemsetAsync(k, 0x3d, step_bytes, stream));
  CK(hipMemsetAsync(v, 0x3e, step_bytes, stream));
  CK(hipStreamSynchronize(stream));

  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  double keys = 0;
  float best_ms = 0;
  for (int img = 0; img <= images; ++img) {      // image 0 is the warm-up
    linear_kv_t* kv = nullptr;
    LK(kv_init(&cfg, kc.data(), vc.data(), scratch, cond_bytes ? kcond.data() : nullptr,
               cond_bytes ? vcond.data() : nullptr, stream, &kv));
    CK(hipStreamSynchronize(stream));
    CK(hipEventRecord(e0, stream));
    keys = 0;
    const int steps = img == 0 ? 2 * cfg.line_len : N;
    for (int s = 0; s < steps; ++s) {
      int32_t cached = 0;
      LK(kv_length(kv, 0, &cached, nullptr, nullptr));
      keys += cached + 1;
      LK(decode_step_layers(kv, 0, L, q, k, v, out, (size_t)P * row, (size_t)P * cfg.head_dim * 4, stream));
      if ((s + 1) % cfg.line_len == 0) LK(end_of_line_evict_layers(kv, 0, L, stream));
    }
    CK(hipEventRecord(e1, stream));
    CK(hipEventSynchronize(e1));
    float ms = 0;
    CK(hipEventElapsedTime(&ms, e0, e1));
    if (img > 0 && (best_ms == 0 || ms < best_ms)) best_ms = ms;
    LK(kv_free(kv));
  }
  const double bytes_per_launch = keys / N * 2.0 * P * row;
  std::printf("%s%s: %d decode steps x %d layers in %.3f ms: %.2f us/step, %.3f us per layer launch (evictions included), "
              "%.0f algorithmic K/V bytes per decode launch, %.1f GB/s\n",
              sh->name, full ? "-full" : "", N, L, best_ms, best_ms * 1e3 / N, best_ms * 1e3 / N / L, bytes_per_launch,
              bytes_per_launch * N * L / best_ms / 1e6);
  return 0;
}
