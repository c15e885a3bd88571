// Single-query decode attention over the compact LineAR cache, with the append of the new
// (k, v) (Eq. 2-4) and the per-query saliency term of Eq. 9 fused in.
//
// Shape of the work: per (sequence, head) pair one query attends to T keys of d elements;
// every K and V row is read exactly once and nothing is shared between pairs, so the step
// is an HBM stream (1 flop per byte at bf16) that runs on the vector ALUs -- and at 8 TB/s
// the ALU budget is only a few hundred instructions per wavefront, so the kernel is built
// around instruction count as much as around bytes:
//   * a key row is spread over LPR = d*sizeof(elem)/16 adjacent lanes (16 bytes each), so a
//     wave-wide load covers 1 KiB of contiguous cache; a wavefront owns up to U such row
//     groups and issues all its K loads before the first use, and all its V loads as soon as
//     the K rows are there, so that the logits are computed under the V stream;
//   * q.k uses the packed bf16 dot instruction (fp32 accumulate) and a DPP butterfly over
//     the LPR lanes; no LDS, no ds_bpermute in the main phase;
//   * every group of LPR lanes is an independent softmax worker over its own rows (max and
//     sum stay in-lane); workers meet once, in LDS, where the first wavefront merges them;
//   * the new token is one extra row taken from the inputs; one wavefront counts it and
//     writes it to the cache (Eq. 4); its original position is implied by its row (only the
//     survivors of evictions need a position map, and the end-of-line kernel keeps it);
//   * on lines that end in an eviction the query joins the line's guide queue (Eq. 8): either
//     the query itself, stored with the new row, or -- for the modes that score decode-time
//     probabilities -- its logits on the scored keys, staged through LDS so that they leave as
//     one coalesced store; the softmax rows of Eq. 9 are evaluated once per line by the
//     end-of-line kernel, so a decode step carries no reduction for them;
//   * stores are few, early (the new row goes out right after the loads) and cover whole
//     aligned 128-byte lines: a kernel this short pays for every store instruction, for the
//     full latency of a late one and for the read-modify-write of a line written in part;
//   * what the loads need arrives as leading scalar kernel arguments (preloaded into SGPRs
//     where the firmware supports it), the rest of the arguments is fetched behind the loads;
//   * a pair whose keys fit one workgroup (up to 144 row groups) is a single launch with
//     no inter-workgroup traffic; longer ones are split over workgroups and merged by
//     a second, tiny kernel (a kernel boundary is cheaper here than device-scope fences).
#include "kernels.h"
#include "lanes.h"

// Phase stamps: nothing in the library; the instrumented timing program (phase_clock.hip) defines
// LINEAR_PHASE(i) to record a wall-clock stamp per wavefront at the marked points of the kernel.
#ifndef LINEAR_PHASE
#define LINEAR_PHASE(i)
#define LINEAR_PHASE_AFTER_STORES(i)
#endif

namespace linear {
namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Results are written once and read by a later kernel: nontemporal stores keep them from
// sitting dirty in L2 until the end-of-kernel write-back.
__device__ __forceinline__ void store_nt(float* p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void store_nt(uint4* p, const uint4& v) {
  __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(p));
}
// Element `idx` of the result, in single precision or rounded to bfloat16 (64 adjacent lanes
// write 256 or 128 contiguous bytes either way).
__device__ __forceinline__ void store_out(void* out, int bf16, size_t idx, float v) {
  if (bf16) {
    const __bf16 b = (__bf16)v;   // round to nearest even
    __builtin_nontemporal_store(__builtin_bit_cast(unsigned short, b), static_cast<unsigned short*>(out) + idx);
  } else {
    store_nt(static_cast<float*>(out) + idx, v);
  }
}
template <bool BF16>
struct Elems;
template <>
struct Elems<true> {
  static constexpr int kPerLane = 8;
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
    float r = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.x), __builtin_bit_cast(bf16x2, b.x), 0.f, false);
    r = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.y), __builtin_bit_cast(bf16x2, b.y), r, false);
    r = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.z), __builtin_bit_cast(bf16x2, b.z), r, false);
    r = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.w), __builtin_bit_cast(bf16x2, b.w), r, false);
    return r;
  }
  static __device__ __forceinline__ void axpy(float p, const uint4& r, float (&o)[8]) {
    o[0] = __builtin_fmaf(p, __uint_as_float(r.x << 16), o[0]);
    o[1] = __builtin_fmaf(p, __uint_as_float(r.x & 0xffff0000u), o[1]);
    o[2] = __builtin_fmaf(p, __uint_as_float(r.y << 16), o[2]);
    o[3] = __builtin_fmaf(p, __uint_as_float(r.y & 0xffff0000u), o[3]);
    o[4] = __builtin_fmaf(p, __uint_as_float(r.z << 16), o[4]);
    o[5] = __builtin_fmaf(p, __uint_as_float(r.z & 0xffff0000u), o[5]);
    o[6] = __builtin_fmaf(p, __uint_as_float(r.w << 16), o[6]);
    o[7] = __builtin_fmaf(p, __uint_as_float(r.w & 0xffff0000u), o[7]);
  }
};
template <>
struct Elems<false> {
  static constexpr int kPerLane = 4;
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
    float r = __uint_as_float(a.x) * __uint_as_float(b.x);
    r = __builtin_fmaf(__uint_as_float(a.y), __uint_as_float(b.y), r);
    r = __builtin_fmaf(__uint_as_float(a.z), __uint_as_float(b.z), r);
    r = __builtin_fmaf(__uint_as_float(a.w), __uint_as_float(b.w), r);
    return r;
  }
  static __device__ __forceinline__ void axpy(float p, const uint4& r, float (&o)[4]) {
    o[0] = __builtin_fmaf(p, __uint_as_float(r.x), o[0]);
    o[1] = __builtin_fmaf(p, __uint_as_float(r.y), o[1]);
    o[2] = __builtin_fmaf(p, __uint_as_float(r.z), o[2]);
    o[3] = __builtin_fmaf(p, __uint_as_float(r.w), o[3]);
  }
};

// Merge of n softmax partials (m[i], l[i], o[i][D]) by one wavefront, each partial being
// the plain sum of G consecutive rows of pl / po (already scaled to the common m[i]).
// Lane e (and e + 64) ends with the merged numerator; (m, l) are returned in every lane.
template <int D, int G>
__device__ __forceinline__ void merge_partials(const float* pm, const float* pl, const float* po,
                                               int n, float& m_all, float& l_all, float (&o)[D / 64]) {
  const int lane = threadIdx.x & 63;
  m_all = ninf();
  for (int i = 0; i < n; ++i) m_all = fmaxf(m_all, pm[i]);
  l_all = 0.f;
#pragma unroll
  for (int c = 0; c < D / 64; ++c) o[c] = 0.f;
  for (int i = 0; i < n; ++i) {
    const float mi = pm[i];
    const float f = mi > ninf() ? ex2(mi - m_all) : 0.f;   // a partial without keys
    float ls = 0.f, os[D / 64];
#pragma unroll
    for (int c = 0; c < D / 64; ++c) os[c] = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      ls += pl[i * G + g];
#pragma unroll
      for (int c = 0; c < D / 64; ++c) os[c] += po[(size_t)(i * G + g) * D + c * 64 + lane];
    }
    l_all = __builtin_fmaf(ls, f, l_all);
#pragma unroll
    for (int c = 0; c < D / 64; ++c) o[c] = __builtin_fmaf(os[c], f, o[c]);
  }
}

// Rotary embedding of one row held as LPR pieces of 16 bytes, element t paired with t + d/2:
// lane `seg` holds elements seg*EPL .. seg*EPL + EPL-1, its partner elements sit LPR/2 lanes
// away.  x' = x cos + sign * partner sin with sign -1 in the first half and +1 in the second,
// each product and the sum rounded to fp32 separately (no fused multiply-add) and the result
// rounded to the storage type, so that the rotated row has the bits an unfused fp32
// implementation produces.  `cs` points at this lane's EPL cosines, `sn` at its EPL sines.
template <int CTRL>
__device__ __forceinline__ unsigned dpp_u32(unsigned x) {
  return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}
template <int LPR>
__device__ __forceinline__ uint4 partner_piece(const uint4& r) {
  uint4 p;
  if (LPR == 8) {          // row_ror:4 -- every 16-lane row holds two copies of the 8-piece row
    p.x = dpp_u32<0x124>(r.x); p.y = dpp_u32<0x124>(r.y); p.z = dpp_u32<0x124>(r.z); p.w = dpp_u32<0x124>(r.w);
  } else if (LPR == 16) {  // row_ror:8
    p.x = dpp_u32<0x128>(r.x); p.y = dpp_u32<0x128>(r.y); p.z = dpp_u32<0x128>(r.z); p.w = dpp_u32<0x128>(r.w);
  } else {                 // 32 lanes per row: the partner is 16 lanes away
    p.x = __shfl_xor(r.x, 16); p.y = __shfl_xor(r.y, 16); p.z = __shfl_xor(r.z, 16); p.w = __shfl_xor(r.w, 16);
  }
  return p;
}
__device__ __forceinline__ float rot1(float x, float partner, float c, float s, float sign) {
#pragma clang fp contract(off)   // two rounded products, then a rounded sum: never a fused multiply-add
  const float xc = x * c;
  const float ps = partner * s;
  return xc + sign * ps;
}
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t v = {(__bf16)lo, (__bf16)hi};   // round to nearest even
  return __builtin_bit_cast(unsigned, v);
}
template <bool BF16, int LPR, int EPL>
__device__ __forceinline__ uint4 rotate_row(const uint4& r, const float (&cc)[EPL], const float (&ss)[EPL], float sign) {
  const uint4 p = partner_piece<LPR>(r);
  const unsigned rw[4] = {r.x, r.y, r.z, r.w}, pw[4] = {p.x, p.y, p.z, p.w};
  unsigned ow[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (BF16) {
      const float lo = rot1(__uint_as_float(rw[j] << 16), __uint_as_float(pw[j] << 16), cc[2 * j], ss[2 * j], sign);
      const float hi = rot1(__uint_as_float(rw[j] & 0xffff0000u), __uint_as_float(pw[j] & 0xffff0000u),
                            cc[(2 * j + 1) % EPL], ss[(2 * j + 1) % EPL], sign);
      ow[j] = pack_bf16(lo, hi);
    } else {
      ow[j] = __float_as_uint(rot1(__uint_as_float(rw[j]), __uint_as_float(pw[j]), cc[j % EPL], ss[j % EPL], sign));
    }
  }
  return make_uint4(ow[0], ow[1], ow[2], ow[3]);
}

template <int U>
struct MaxWaves {   // waves per workgroup the register budget of a U-deep wavefront allows
  static constexpr int value = U <= 8 ? 16 : 12;   // deeper than 8: three per SIMD, 170 registers each
};

// The first arguments are the ones the loads depend on, as scalars at the front of the kernel
// argument segment: with kernel-argument preloading (build flag) they arrive in SGPRs with the
// wavefront, so the first load does not wait for a scalar fetch of the arguments.  `t_nw` =
// keys visible to the query | wavefronts per workgroup << 24; `tmax_gps` = row pitch of the
// caches | row groups per workgroup << 21.  The rest is read from `a`, after the loads are out.
template <bool BF16, int D, int U, bool ROPE>
__global__ __launch_bounds__(64 * MaxWaves<U>::value) void decode_attn_kernel(
    const void* __restrict__ q_in, void* __restrict__ kc_in, void* __restrict__ vc_in,
    const void* __restrict__ k_in, const void* __restrict__ v_in, const float* __restrict__ cos_sin,
    const uint32_t t_nw, const uint32_t tmax_gps, const DecodeArgs a) {
  using E = Elems<BF16>;
  constexpr int EPL = E::kPerLane;   // elements per lane
  constexpr int LPR = D / EPL;       // lanes per key row
  constexpr int RPW = 64 / LPR;      // rows per wave-wide load = softmax workers per wavefront

  extern __shared__ float smem[];
  const int nw = (int)(t_nw >> 24);
  const int t = (int)(t_nw & 0xffffffu), t_max = (int)(tmax_gps & 0x1fffffu);
  const int rows_per_split = (int)(tmax_gps >> 21) * RPW;
  const int n_workers = nw * RPW;
  float* sm_o = smem;                        // [n_workers][D] numerators, scaled to the wave's max
  float* sm_l = sm_o + n_workers * D;        // [n_workers]    sums, likewise
  float* sm_m = sm_l + n_workers;            // [nw]           the waves' maxima
  float* sm_mid = sm_m + nw;                 // [mid_n]        logits of the mid keys

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int seg = lane % LPR, sub = lane / LPR;
  const int pair = blockIdx.x, split = blockIdx.y;
  LINEAR_PHASE(0);   // wavefront started
  const int r0 = split * rows_per_split;                 // cached rows [r0, r0 + n_rows)
  const int n_rows = min(t - 1, r0 + rows_per_split) - r0;

  // ---- loads: straight-line, so that every later wait counts exactly the loads behind it.
  // Addresses are a uniform base plus a 32-bit lane offset.  Row groups beyond the end
  // re-read the last row (served by the caches) and are masked.
  constexpr unsigned kRowBytes = LPR * 16;
  const char* kbase = static_cast<const char*>(kc_in) + ((size_t)pair * t_max + r0) * kRowBytes;
  const char* vbase = static_cast<const char*>(vc_in) + ((size_t)pair * t_max + r0) * kRowBytes;
  const unsigned in_off = (unsigned)seg * 16u;
  uint4 qr = *reinterpret_cast<const uint4*>(static_cast<const char*>(q_in) + (size_t)pair * kRowBytes + in_off);
  uint4 knr = *reinterpret_cast<const uint4*>(static_cast<const char*>(k_in) + (size_t)pair * kRowBytes + in_off);
  const uint4 vnr = *reinterpret_cast<const uint4*>(static_cast<const char*>(v_in) + (size_t)pair * kRowBytes + in_off);
  float rc[EPL], rs[EPL];   // this lane's rotary cosines and sines: requested ahead of the cache rows
  if (ROPE) {
    const float* cs = cos_sin + (seg * EPL) % (D / 2);
#pragma unroll
    for (int j = 0; j < EPL; j += 4) {
      const float4 c4 = *reinterpret_cast<const float4*>(cs + j), s4 = *reinterpret_cast<const float4*>(cs + D / 2 + j);
      rc[j] = c4.x; rc[j + 1] = c4.y; rc[j + 2] = c4.z; rc[j + 3] = c4.w;
      rs[j] = s4.x; rs[j + 1] = s4.y; rs[j + 2] = s4.z; rs[j + 3] = s4.w;
    }
  }
  uint4 kr[U], vr[U];
  int row[U];
  unsigned off[U];
  const unsigned last = (unsigned)max(n_rows - 1, 0);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    row[u] = (u * nw + wave) * RPW + sub;
    off[u] = min((unsigned)row[u], last) * kRowBytes + in_off;
    kr[u] = *reinterpret_cast<const uint4*>(kbase + off[u]);
  }
  __builtin_amdgcn_sched_barrier(0);   // all K requests go out before the first V request
  if (ROPE) {
    // q and k of the new token arrive unrotated: every lane rotates its piece of both (all
    // wavefronts need q; k is only used by the lane group that appends it, but rotating it
    // everywhere keeps the code straight-line and costs no memory traffic).  Done here, with
    // the K requests in flight and before the V requests, so that the table's registers are
    // free again when the V rows need theirs.
    const float sign = seg < LPR / 2 ? -1.0f : 1.0f;
    qr = rotate_row<BF16, LPR, EPL>(qr, rc, rs, sign);
    knr = rotate_row<BF16, LPR, EPL>(knr, rc, rs, sign);
  }
  // The V rows are requested when the K rows have arrived: two streams one after the other
  // instead of interleaved (measured faster, 250 -> 245 us/step at LlamaGen-XL); the logits and
  // the exponentials are then computed while the V rows are on their way.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  LINEAR_PHASE(1);   // K rows arrived
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < U; ++u) vr[u] = *reinterpret_cast<const uint4*>(vbase + off[u]);
  // Nothing below may be scheduled in front of the loads: a wait placed between them would
  // hold back the rest of the requests for a full memory round trip.
  __builtin_amdgcn_sched_barrier(0);

  const bool scoring = a.mid_n > 0;
  // The appended token is counted by sub-group 0 of one wavefront of the last split (the
  // host picks the one with the fewest row groups).
  const bool owner = split == a.n_split - 1 && wave == a.new_wave && sub == 0;
  // Stores go out as early as their data exists: a kernel ends only when its last store has
  // been acknowledged, so a store issued near the end adds its whole latency to the step.
  if (owner) {
    // Eq. 4: the new pair becomes row T-1 of the cache.
    const size_t dst = ((size_t)pair * t_max + (t - 1)) * LPR + seg;
    store_nt(&reinterpret_cast<uint4*>(kc_in)[dst], knr);
    store_nt(&reinterpret_cast<uint4*>(vc_in)[dst], vnr);
    // Eq. 8 as printed: the query joins the line's guide queue (one aligned row)
    if (a.qq) store_nt(reinterpret_cast<uint4*>(static_cast<char*>(a.qq) + (size_t)pair * a.qq_pitch) + seg, qr);
  }
  // ---- raw logits q.k and this worker's maximum (Eq. 2; the scale is applied with the shift)
  float s[U];
  float s_new = sum_within<LPR>(E::dot(knr, qr));
  s_new = owner ? s_new : ninf();
  float m = s_new;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const float d = sum_within<LPR>(E::dot(kr[u], qr));
    s[u] = row[u] < n_rows ? d : ninf();
    m = fmaxf(m, s[u]);
  }
  const float c = a.scale_log2e;          // > 0: scaling commutes with the maximum
  LINEAR_PHASE(2);   // logits computed (V rows requested before them)
  if (scoring) {
    // Eq. 8-9: the logits of the mid keys (log2 units) are staged in LDS: one 4-byte entry per
    // key from a few lanes each would cost a vector-memory instruction per row group, and the
    // memory system charges small scattered stores by the instruction.
    const int mid_first = a.mid_lo - r0, mid_end = min(mid_first + a.mid_n, n_rows);   // rows of this split
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int g0 = (u * nw + wave) * RPW;                     // wave-uniform: first row of the group
      if (g0 < mid_end && g0 + RPW > mid_first) {
        const int j = row[u] - mid_first;
        if (seg == 0 && row[u] >= mid_first && row[u] < mid_end) sm_mid[j] = s[u] * c;
      }
    }
    // accumulated attention also scores the appended token (row T-1) under its own query
    if (a.stage_new && owner && seg == 0 && t - 1 >= a.mid_lo) sm_mid[t - 1 - a.mid_lo] = s_new * c;
  }
  // ---- probabilities relative to the worker's own maximum, and its numerator
  const float m_ref = m > ninf() ? m : 0.f;
  const float shift = -m_ref * c;
  float o[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) o[e] = 0.f;
  float l = ex2(__builtin_fmaf(s_new, c, shift));   // exp2(-inf) = 0 where the row does not count
  E::axpy(l, vnr, o);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const float p = ex2(__builtin_fmaf(s[u], c, shift));
    l += p;
    E::axpy(p, vr[u], o);
  }
  // ---- the wavefront's workers move to a common maximum (log2 units) and meet in LDS
  const float m2 = m * c;
  const float m_wave = wave_max(m2);
  {
    const float f = m > ninf() ? ex2(m2 - m_wave) : 0.f;
    l *= f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] *= f;
    const int worker = wave * RPW + sub;
    float4* dst = reinterpret_cast<float4*>(sm_o + worker * D + seg * EPL);
    dst[0] = make_float4(o[0], o[1], o[2], o[3]);
    if constexpr (EPL == 8) dst[1] = make_float4(o[4], o[5], o[6], o[7]);
    if (seg == 0) sm_l[worker] = l;
    if (lane == 0) sm_m[wave] = m_wave;
  }
  LINEAR_PHASE(3);   // V rows consumed, partial written to LDS
  __syncthreads();
  LINEAR_PHASE(4);   // every wavefront of the pair is through
  // A query's guide-queue row (Eq. 8) occupies whole, aligned 128-byte lines and a workgroup that
  // holds all the keys writes all of them, padding included, in one coalesced store: lines
  // written in part cost a read-modify-write at the memory (measured: 0.3 us per launch).
  const int extra = a.stage_new && split == a.n_split - 1 ? 1 : 0;   // the appended token's entry
  const int j0 = max(r0 - a.mid_lo, 0), j1 = min(r0 + n_rows + extra - a.mid_lo, a.mid_n);
  float* qrow = a.guide + (size_t)pair * a.guide_pitch;
  if (scoring && wave == nw - 1 && (!a.store_ml || a.n_split > 1)) {
    // By the last wavefront while the first one merges; the softmax rows of Eq. 9 are evaluated
    // once, at the end of the line.  (Issuing it earlier, behind a barrier of its own between
    // the logits and the V phase, was measured slower.)
    if (a.n_split == 1) {
      for (int j = lane; j < a.guide_row; j += 64) store_nt(&qrow[j], j < j1 ? sm_mid[j] : 0.f);
    } else {
      for (int j = j0 + lane; j < j1; j += 64) store_nt(&qrow[j], sm_mid[j]);
    }
  }
  if (wave != 0) return;

  float m_all, l_all, o_all[D / 64];
  merge_partials<D, RPW>(sm_m, sm_l, sm_o, nw, m_all, l_all, o_all);
  if (a.n_split == 1) {
    const float inv = 1.0f / l_all;
#pragma unroll
    for (int c = 0; c < D / 64; ++c) store_out(a.out, a.out_bf16, (size_t)pair * D + c * 64 + lane, o_all[c] * inv);
    LINEAR_PHASE(5);   // merged and result store issued
    LINEAR_PHASE_AFTER_STORES(6);
    if (scoring && a.store_ml) {
      // the row together with the decode softmax's statistics, which only exist now
      for (int j = lane; j < a.guide_row; j += 64) {
        const float x = j < j1 ? sm_mid[j] : (j == a.guide_w ? m_all : (j == a.guide_w + 1 ? l_all : 0.f));
        store_nt(&qrow[j], x);
      }
    }
    return;
  }
  const size_t pidx = (size_t)pair * a.max_split + split;
#pragma unroll
  for (int c = 0; c < D / 64; ++c) a.part_o[pidx * D + c * 64 + lane] = o_all[c];
  if (lane == 0) {
    a.part_ml[pidx * 2 + 0] = m_all;
    a.part_ml[pidx * 2 + 1] = l_all;
  }
}

// Second kernel of a split step: merges the split partials of one pair.  One wavefront
// per pair.
template <int D>
__global__ __launch_bounds__(64) void decode_combine_kernel(const DecodeArgs a) {
  __shared__ float sm_m[kMaxSplit], sm_l[kMaxSplit];
  const int lane = threadIdx.x, pair = blockIdx.x;
  const size_t pbase = (size_t)pair * a.max_split;
  for (int i = lane; i < a.n_split; i += 64) {
    sm_m[i] = a.part_ml[(pbase + i) * 2 + 0];
    sm_l[i] = a.part_ml[(pbase + i) * 2 + 1];
  }
  __syncthreads();
  float m_all, l_all, o_all[D / 64];
  merge_partials<D, 1>(sm_m, sm_l, a.part_o + pbase * D, a.n_split, m_all, l_all, o_all);
  const float inv = 1.0f / l_all;
#pragma unroll
  for (int c = 0; c < D / 64; ++c) store_out(a.out, a.out_bf16, (size_t)pair * D + c * 64 + lane, o_all[c] * inv);
  if (a.mid_n > 0 && a.store_ml && lane == 0) {
    float* qrow = a.guide + (size_t)pair * a.guide_pitch;
    store_nt(&qrow[a.guide_w], m_all);
    store_nt(&qrow[a.guide_w + 1], l_all);
  }
}

template <bool BF16, int D, int U>
hipError_t launch_main(const DecodeArgs& a, hipStream_t s) {
  constexpr int RPW = 64 / (D / Elems<BF16>::kPerLane);
  const int workers = a.n_waves * RPW;
  const size_t dyn = ((size_t)workers * (D + 1) + a.n_waves + (size_t)a.mid_n) * sizeof(float);
  const dim3 grid((unsigned)a.n_pairs, (unsigned)a.n_split), block(64u * (unsigned)a.n_waves);
  const uint32_t t_nw = (uint32_t)a.t | ((uint32_t)a.n_waves << 24);
  const uint32_t tmax_gps = (uint32_t)a.t_max | ((uint32_t)(a.rows_per_split / RPW) << 21);
  if (a.cos_sin)
    hipLaunchKernelGGL((decode_attn_kernel<BF16, D, U, true>), grid, block, dyn, s, a.q, a.kc, a.vc, a.k_new,
                       a.v_new, a.cos_sin, t_nw, tmax_gps, a);
  else
    hipLaunchKernelGGL((decode_attn_kernel<BF16, D, U, false>), grid, block, dyn, s, a.q, a.kc, a.vc, a.k_new,
                       a.v_new, a.cos_sin, t_nw, tmax_gps, a);
  return hipGetLastError();
}

template <bool BF16, int D>
hipError_t launch_t(const DecodeArgs& a, hipStream_t s) {
  hipError_t e;
  switch (a.depth) {
    case 1: e = launch_main<BF16, D, 1>(a, s); break;
    case 2: e = launch_main<BF16, D, 2>(a, s); break;
    case 3: e = launch_main<BF16, D, 3>(a, s); break;
    case 4: e = launch_main<BF16, D, 4>(a, s); break;
    case 5: e = launch_main<BF16, D, 5>(a, s); break;
    case 6: e = launch_main<BF16, D, 6>(a, s); break;
    case 7: e = launch_main<BF16, D, 7>(a, s); break;
    case 8: e = launch_main<BF16, D, 8>(a, s); break;
    case 10: e = launch_main<BF16, D, 10>(a, s); break;
    case 12: e = launch_main<BF16, D, 12>(a, s); break;
    case 14: e = launch_main<BF16, D, 14>(a, s); break;
    case 16: e = launch_main<BF16, D, 16>(a, s); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess || a.n_split == 1) return e;
  hipLaunchKernelGGL((decode_combine_kernel<D>), dim3((unsigned)a.n_pairs), dim3(64), 0, s, a);
  return hipGetLastError();
}

}  // namespace

int decode_rows_per_group(int dtype, int head_dim) {
  const int lanes_per_row = head_dim / (dtype == 1 ? 8 : 4);
  return 64 / lanes_per_row;
}

int decode_max_waves(int depth) { return depth <= 8 ? 16 : 12; }

int decode_depth_for(int groups_per_wave) {
  static const int kDepths[] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16};
  for (int d : kDepths)
    if (d >= groups_per_wave) return d;
  return 0;
}

hipError_t launch_decode(const DecodeArgs& a, int dtype, int head_dim, hipStream_t s) {
  if (dtype == 1 && head_dim == 64) return launch_t<true, 64>(a, s);
  if (dtype == 1 && head_dim == 128) return launch_t<true, 128>(a, s);
  if (dtype == 0 && head_dim == 64) return launch_t<false, 64>(a, s);
  if (dtype == 0 && head_dim == 128) return launch_t<false, 128>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace linear
