// phase_clock: where the time of a decode launch goes.  Compiles the library's decode kernel with
// its phase marks turned into wall-clock stamps (100 MHz counter, one stamp per wavefront and
// mark) and prints, for the last of a series of back-to-back launches cycling over 12 layers'
// caches, the distribution over wavefronts of each mark's time since the launch's first
// wavefront started.  The stamps cost time themselves (a launch takes about 30 % longer than in
// the library), so the figures show the order and the relative size of the phases, not absolute
// durations.  usage: phase_clock <pairs> <head_dim 64|128> <cache pitch in keys> <keys T> <wavefronts per pair>
#include <hip/hip_runtime.h>

__device__ unsigned long long g_phase_stamps[1 << 20];   // [pair][16 wavefronts][8 marks]
#define LINEAR_PHASE(i)                                                                                              \
  do {                                                                                                               \
    if ((threadIdx.x & 63) == 0)                                                                                     \
      g_phase_stamps[((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 16 + (threadIdx.x >> 6)) * 8 + (i)] = wall_clock64(); \
  } while (0)
#define LINEAR_PHASE_AFTER_STORES(i)                      \
  do {                                                    \
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      \
    LINEAR_PHASE(i);                                      \
  } while (0)

#include "decode_attn.hip"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

using namespace linear;
#define CK(x)                                                                             \
  do {                                                                                    \
    hipError_t e_ = (x);                                                                  \
    if (e_ != hipSuccess) {                                                               \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
      return 1;                                                                           \
    }                                                                                     \
  } while (0)

int main(int argc, char** argv) {
  if (argc < 6) {
    std::printf("usage: phase_clock <pairs> <head_dim> <pitch> <T> <wavefronts per pair>\n");
    return 2;
  }
  const int P = std::atoi(argv[1]), D = std::atoi(argv[2]), TMAX = std::atoi(argv[3]), T = std::atoi(argv[4]),
            nw = std::atoi(argv[5]);
  if (P < 1 || P > 8000 || (D != 64 && D != 128) || T < 2 || T > TMAX || nw < 1 || nw > 16) {
    std::printf("arguments out of range\n");
    return 2;
  }
  const int L = 12, RPG = 64 / (D / 8);
  const int groups = (T - 1 + RPG - 1) / RPG, per = (groups + nw - 1) / nw, depth = decode_depth_for(per);
  if (groups > 144 || !depth || nw > decode_max_waves(depth) || nw > groups) {
    std::printf("this many keys do not fit %d wavefronts of one workgroup\n", nw);
    return 2;
  }
  const size_t layer_elems = (size_t)P * TMAX * D, step_elems = (size_t)P * D;
  uint16_t *kc, *vc, *q, *k, *v;
  float *out, *part_o, *part_ml;
  CK(hipMalloc(&kc, layer_elems * 2 * L));
  CK(hipMalloc(&vc, layer_elems * 2 * L));
  CK(hipMemset(kc, 0x3c, layer_elems * 2 * L));
  CK(hipMemset(vc, 0x3c, layer_elems * 2 * L));
  CK(hipMalloc(&q, step_elems * 2 * L));
  CK(hipMalloc(&k, step_elems * 2 * L));
  CK(hipMalloc(&v, step_elems * 2 * L));
  CK(hipMemset(q, 0x3c, step_elems * 2 * L));
  CK(hipMemset(k, 0x3c, step_elems * 2 * L));
  CK(hipMemset(v, 0x3c, step_elems * 2 * L));
  CK(hipMalloc(&out, step_elems * 4 * L));
  CK(hipMalloc(&part_o, (size_t)P * 64 * D * 4));
  CK(hipMalloc(&part_ml, (size_t)P * 64 * 2 * 4));
  auto launch = [&](int l) {
    DecodeArgs a{};
    a.q = q + step_elems * l;
    a.k_new = k + step_elems * l;
    a.v_new = v + step_elems * l;
    a.kc = kc + layer_elems * l;
    a.vc = vc + layer_elems * l;
    a.out = out + step_elems * l;
    a.part_o = part_o;
    a.part_ml = part_ml;
    a.n_pairs = P;
    a.t = T;
    a.t_max = TMAX;
    a.rows_per_split = groups * RPG;
    a.n_split = 1;
    a.n_waves = nw;
    a.depth = depth;
    a.new_wave = groups % nw;
    a.max_split = 64;
    a.scale_log2e = 0.18f;
    return launch_decode(a, 1, D, 0);
  };
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  for (int l = 0; l < L; ++l) CK(launch(l));
  CK(hipDeviceSynchronize());
  const int REP = 20;
  CK(hipEventRecord(e0, 0));
  for (int r = 0; r < REP; ++r)
    for (int l = 0; l < L; ++l) CK(launch(l));
  CK(hipEventRecord(e1, 0));
  CK(hipEventSynchronize(e1));
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  std::printf("%d pairs, head_dim %d, T = %d keys, %d wavefronts of %d row groups per pair: %.2f us per launch with the stamps\n",
              P, D, T, nw, depth, ms * 1e3 / (REP * L));
  std::vector<unsigned long long> ts((size_t)P * 16 * 8);
  CK(hipMemcpyFromSymbol(ts.data(), HIP_SYMBOL(g_phase_stamps), ts.size() * 8));
  unsigned long long t0 = ~0ull;
  for (int p = 0; p < P; ++p)
    for (int w = 0; w < nw; ++w) t0 = std::min(t0, ts[((size_t)p * 16 + w) * 8]);
  const char* names[7] = {"wavefront started", "K rows arrived", "logits computed", "V rows consumed",
                          "pair's wavefronts met", "result store issued", "stores acknowledged"};
  for (int i = 0; i < 7; ++i) {
    std::vector<double> x;
    for (int p = 0; p < P; ++p)
      for (int w = 0; w < (i >= 5 ? 1 : nw); ++w) x.push_back((double)(ts[((size_t)p * 16 + w) * 8 + i] - t0) * 0.01);
    std::sort(x.begin(), x.end());
    std::printf("  %-22s min %6.2f  p10 %6.2f  median %6.2f  p90 %6.2f  max %6.2f us\n", names[i], x.front(),
                x[x.size() / 10], x[x.size() / 2], x[x.size() * 9 / 10], x.back());
  }
  return 0;
}
