// Split-K single-query decode attention over the compact LineAR cache, with the append
// of the new (k, v) (Eq. 2-4) and the per-query saliency term of Eq. 9 fused in.
//
// Shape of the work: per (sequence, head) pair one query attends to T keys of d
// elements; K and V rows are each read exactly once, there is no reuse between pairs,
// so the step is a pure HBM stream (1 flop per byte at bf16) and runs on the vector
// ALUs.  One workgroup (4 wavefronts) owns up to `rows_per_split` consecutive keys of
// one pair.  A key row is spread over LPR = d*sizeof(elem)/16 adjacent lanes, 16 bytes
// per lane, so every wave-wide load covers 1 KiB of contiguous cache.  All K and V
// loads of a 128-key tile are issued before the first use; logits are reduced across
// the LPR lanes of a row with lane shuffles; each wavefront keeps its own running
// (max, sum, numerator) in fp32 and the four are merged once through LDS.  With more
// than one split per pair the workgroup that finishes last (device-scope counter)
// merges the split partials, so a step is a single launch.
#include "kernels.h"

namespace linear {
namespace {

__device__ __forceinline__ float ninf() { return -__builtin_inff(); }
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

template <bool BF16>
struct Elems;
template <>
struct Elems<true> {
  static constexpr int kPerLane = 8;
  static __device__ __forceinline__ void unpack(const uint4& r, float (&f)[8]) {
    f[0] = __uint_as_float(r.x << 16);
    f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16);
    f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16);
    f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16);
    f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};
template <>
struct Elems<false> {
  static constexpr int kPerLane = 4;
  static __device__ __forceinline__ void unpack(const uint4& r, float (&f)[4]) {
    f[0] = __uint_as_float(r.x);
    f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z);
    f[3] = __uint_as_float(r.w);
  }
};

// Sum over the aligned group of W adjacent lanes.
template <int W>
__device__ __forceinline__ float sum_within(float x) {
#pragma unroll
  for (int o = W / 2; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
// Reductions over the lanes that share `lane % W` (one per row group of the wavefront).
template <int W>
__device__ __forceinline__ float sum_across(float x) {
#pragma unroll
  for (int o = 32; o >= W; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
template <int W>
__device__ __forceinline__ float max_across(float x) {
#pragma unroll
  for (int o = 32; o >= W; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}

// Adds this query's softmax probabilities on the mid keys to the line's accumulator
// (Eq. 9, one row of the softmax).  `mid` holds the logits in log2 units.  Mode 0
// normalises over the mid keys only; mode 1 uses the decode softmax's (m_all, l_all).
__device__ __forceinline__ void add_saliency(const float* mid, int mid_n, int mode, float m_all,
                                             float l_all, float* acc) {
  const int tid = threadIdx.x, lane = tid & 63;
  float mx = m_all, z = l_all;
  if (mode == 0) {
    float lm = ninf();
    for (int j = lane; j < mid_n; j += 64) lm = fmaxf(lm, mid[j]);
    lm = max_across<1>(lm);
    float ls = 0.f;
    for (int j = lane; j < mid_n; j += 64) ls += ex2(mid[j] - lm);
    ls = sum_across<1>(ls);
    mx = lm;
    z = ls;
  }
  const float inv = 1.0f / z;
  for (int j = tid; j < mid_n; j += kBlock) acc[j] += ex2(mid[j] - mx) * inv;
}

template <bool BF16, int D>
__global__ __launch_bounds__(kBlock) void decode_attn_kernel(const DecodeArgs a) {
  using E = Elems<BF16>;
  constexpr int EPL = E::kPerLane;        // elements per lane
  constexpr int LPR = D / EPL;            // lanes per key row
  constexpr int RPW = 64 / LPR;           // rows per wave-wide load
  constexpr int U = kRowsPerIter / (4 * RPW);  // loads per lane per tile, per matrix

  __shared__ float sm_o[4][D];
  __shared__ float sm_m[4];
  __shared__ float sm_l[4];
  __shared__ int sm_last;
  extern __shared__ float sm_mid[];       // mid logits when the pair is not split

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int seg = lane % LPR, sub = lane / LPR;
  const int pair = blockIdx.x % a.n_pairs, split = blockIdx.x / a.n_pairs;
  const int r0 = split * a.rows_per_split;
  const int r1 = min(a.t, r0 + a.rows_per_split);
  const int last_row = a.t - 1;

  const uint4* kc = reinterpret_cast<const uint4*>(a.kc) + (size_t)pair * a.t_max * LPR + seg;
  const uint4* vc = reinterpret_cast<const uint4*>(a.vc) + (size_t)pair * a.t_max * LPR + seg;
  const uint4* kn = reinterpret_cast<const uint4*>(a.k_new) + (size_t)pair * LPR + seg;
  const uint4* vn = reinterpret_cast<const uint4*>(a.v_new) + (size_t)pair * LPR + seg;

  float qf[EPL];
  {
    const uint4 qr = reinterpret_cast<const uint4*>(a.q)[(size_t)pair * LPR + seg];
    E::unpack(qr, qf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] *= a.scale_log2e;
  }

  const bool scoring = a.mid_n > 0;
  float* mid_dst = a.n_split == 1 ? sm_mid : a.mid_logit + (size_t)pair * a.mid_n;

  float m_run = ninf(), l_run = 0.f;
  float o[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) o[e] = 0.f;

  for (int base = r0; base < r1; base += kRowsPerIter) {
    uint4 kr[U], vr[U];
    // Row groups of RPW keys are dealt round-robin to the four wavefronts, so a short
    // tile still keeps all of them busy.
    const int row0 = base + wave * RPW + sub;
    constexpr int kStep = 4 * RPW;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + u * kStep;
      if (row < r1) {
        const bool is_new = row == last_row;
        kr[u] = *(is_new ? kn : kc + (size_t)row * LPR);
        vr[u] = *(is_new ? vn : vc + (size_t)row * LPR);
      } else {
        kr[u] = make_uint4(0, 0, 0, 0);
        vr[u] = make_uint4(0, 0, 0, 0);
      }
    }
    // Eq. 4: the new pair becomes the last row of the cache.
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + u * kStep;
      if (row == last_row && row < r1) {
        reinterpret_cast<uint4*>(a.kc)[((size_t)pair * a.t_max + row) * LPR + seg] = kr[u];
        reinterpret_cast<uint4*>(a.vc)[((size_t)pair * a.t_max + row) * LPR + seg] = vr[u];
        if (seg == 0) a.pos[(size_t)pair * a.t_max + row] = a.new_pos;
      }
    }
    float s[U];
    float m_it = ninf();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + u * kStep;
      float kf[EPL];
      E::unpack(kr[u], kf);
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) dot = __builtin_fmaf(qf[e], kf[e], dot);
      dot = sum_within<LPR>(dot);
      s[u] = row < r1 ? dot : ninf();
      m_it = fmaxf(m_it, s[u]);
      if (scoring && seg == 0 && row < r1) {
        const int j = row - a.mid_lo;
        if (j >= 0 && j < a.mid_n) mid_dst[j] = s[u];
      }
    }
    m_it = max_across<LPR>(m_it);
    const float m_new = fmaxf(m_run, m_it);
    if (m_new > ninf()) {                 // wave-uniform: this wavefront has seen a key
      const float corr = ex2(m_run - m_new);
      l_run *= corr;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[e] *= corr;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = ex2(s[u] - m_new);  // exp2(-inf) = 0 for rows past the end
        l_run += p;
        float vf[EPL];
        E::unpack(vr[u], vf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = __builtin_fmaf(p, vf[e], o[e]);
      }
      m_run = m_new;
    }
  }

  // Merge the row groups of the wavefront, then the four wavefronts.
  l_run = sum_across<LPR>(l_run);
#pragma unroll
  for (int e = 0; e < EPL; ++e) o[e] = sum_across<LPR>(o[e]);
  if (sub == 0) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) sm_o[wave][seg * EPL + e] = o[e];
  }
  if (lane == 0) {
    sm_m[wave] = m_run;
    sm_l[wave] = l_run;
  }
  __syncthreads();
  float m_blk = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));
  float l_blk = 0.f, o_blk = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float f = sm_m[w] > ninf() ? ex2(sm_m[w] - m_blk) : 0.f;   // wavefront without keys
    l_blk += sm_l[w] * f;
    if (tid < D) o_blk += sm_o[w][tid] * f;
  }

  if (a.n_split == 1) {
    if (tid < D) a.out[(size_t)pair * D + tid] = o_blk / l_blk;
    if (scoring) add_saliency(sm_mid, a.mid_n, a.score_mode, m_blk, l_blk, a.acc + (size_t)pair * a.mid_n);
    return;
  }

  const size_t pbase = (size_t)pair * a.max_split;
  if (tid < D) a.part_o[(pbase + split) * D + tid] = o_blk;
  if (tid == 0) {
    a.part_ml[(pbase + split) * 2 + 0] = m_blk;
    a.part_ml[(pbase + split) * 2 + 1] = l_blk;
  }
  __threadfence();                          // publish partials and mid logits device-wide
  __syncthreads();
  if (tid == 0) sm_last = atomicAdd(&a.counter[pair], 1) == a.n_split - 1;
  __syncthreads();
  if (!sm_last) return;
  __threadfence();                          // observe the other workgroups' partials

  float m_all = ninf();
  for (int sidx = 0; sidx < a.n_split; ++sidx)
    m_all = fmaxf(m_all, a.part_ml[(pbase + sidx) * 2]);
  float l_all = 0.f, o_all = 0.f;
  for (int sidx = 0; sidx < a.n_split; ++sidx) {
    const float ms = a.part_ml[(pbase + sidx) * 2];
    const float f = ms > ninf() ? ex2(ms - m_all) : 0.f;
    l_all += a.part_ml[(pbase + sidx) * 2 + 1] * f;
    if (tid < D) o_all += a.part_o[(pbase + sidx) * D + tid] * f;
  }
  if (tid < D) a.out[(size_t)pair * D + tid] = o_all / l_all;
  if (tid == 0) a.counter[pair] = 0;        // ready for the next launch
  if (scoring)
    add_saliency(a.mid_logit + (size_t)pair * a.mid_n, a.mid_n, a.score_mode, m_all, l_all,
                 a.acc + (size_t)pair * a.mid_n);
}

template <bool BF16, int D>
hipError_t launch_t(const DecodeArgs& a, hipStream_t s) {
  const size_t dyn = a.n_split == 1 ? (size_t)a.mid_n * sizeof(float) : 0;
  const dim3 grid((unsigned)a.n_pairs * (unsigned)a.n_split);
  hipLaunchKernelGGL((decode_attn_kernel<BF16, D>), grid, dim3(kBlock), dyn, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a, int dtype, int head_dim, hipStream_t s) {
  if (dtype == 1 && head_dim == 64) return launch_t<true, 64>(a, s);
  if (dtype == 1 && head_dim == 128) return launch_t<true, 128>(a, s);
  if (dtype == 0 && head_dim == 64) return launch_t<false, 64>(a, s);
  if (dtype == 0 && head_dim == 128) return launch_t<false, 128>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace linear
