// End-of-line work: saliency of the mid candidates from the line's guide queue (Eq. 9),
// BottomK selection (Eq. 10) and in-place gather-compaction (Eq. 5-7), plus the small
// copy / fill kernels of kv_init and kv_gather.
//
// One workgroup per (sequence, head) pair (and per layer, when layers share a launch).  The
// line's guide queue (Eq. 8) holds either the n queries themselves -- then Eq. 9's product
// Q_guide K_mid^T runs here on the matrix cores, for up to 64 mid keys entirely in the MFMA result
// registers (saliency_small), else tile by tile into LDS (fill_logits) -- or, for the modes that
// score decode-time probabilities, every query's logits on the scored keys as the decode step
// left them, which are copied to LDS.  Either way the workgroup takes every row's softmax
// statistics and adds the rows up column by column in a fixed order (so the result does not
// depend on timing).  The candidates are ranked by counting (stable: equal scores rank by age),
// the n lowest are dropped, the survivors and the r recent lines slide down over the holes.
// Rows only ever move to a lower or equal index and keep their order, so processing destination
// rows in ascending tiles -- load the tile's source rows into registers, barrier, store -- never
// overwrites a row that is still to be read.
#include "kernels.h"
#include "lanes.h"

namespace linear {
namespace {

constexpr int kPiecesPerThread = 4;   // 16-byte pieces of K (and of V) a thread holds per tile
constexpr int kMaxWaves = 16;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));


// Eq. 9's product for one pair when the guide queue holds the queries (Eq. 8 as printed):
// dst[r][j] = (q_r . k_(mid_lo + j)) * scale * log2(e) for the n_rows queued queries and the mid
// keys, on the matrix cores.  16 x 16 output tiles; a wavefront owns a tile column (16 keys,
// loaded once) and walks the query tiles MT at a time, all loads of a step issued before its
// products.  Operand layout of the 16x16 MFMA: lane l supplies row (l % 16) of its operand
// and the (l / 16)-th quarter of the step's k range -- here 16 bytes of the row, the same
// quarter for both operands, which is all a dot product needs; the result has column
// (l % 16) and rows 4 * (l / 16) .. + 3 in lane l.  Rows and columns past the end re-read
// the last one and are not written.  PPR = 16-byte pieces per row.
template <int PPR, bool BF16, int MT>
__device__ void fill_logits(const EvictArgs& a, int pair, float* dst, int dst_pitch) {
  constexpr int STEPS = PPR / 4;   // 64-byte slices of a row
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n_waves = blockDim.x >> 6;
  const int r16 = lane & 15, quarter = lane >> 4;
  const int n_rows = a.n_rows, n_keys = a.mid_n;
  const int tiles_m = (n_rows + 15) >> 4, tiles_n = (n_keys + 15) >> 4;
  const uint4* qq = reinterpret_cast<const uint4*>(a.qq) + (size_t)pair * a.line_len * PPR;
  const uint4* kc = reinterpret_cast<const uint4*>(a.kc) + ((size_t)pair * a.t_max + a.mid_lo) * PPR;
  for (int tn = wave; tn < tiles_n; tn += n_waves) {
    const int key = min(tn * 16 + r16, n_keys - 1);
    uint4 kb[STEPS];
#pragma unroll
    for (int s = 0; s < STEPS; ++s) kb[s] = kc[(size_t)key * PPR + s * 4 + quarter];
    for (int tm0 = 0; tm0 < tiles_m; tm0 += MT) {
      uint4 qa[MT][STEPS];
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const int row = min((tm0 + t) * 16 + r16, n_rows - 1);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) qa[t][s] = qq[(size_t)row * PPR + s * 4 + quarter];
      }
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
          if (BF16) {
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qa[t][s]),
                                                          __builtin_bit_cast(bf16x8, kb[s]), acc, 0, 0, 0);
          } else {
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[t][s].x), __uint_as_float(kb[s].x), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[t][s].y), __uint_as_float(kb[s].y), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[t][s].z), __uint_as_float(kb[s].z), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[t][s].w), __uint_as_float(kb[s].w), acc, 0, 0, 0);
          }
        }
        const int j = tn * 16 + r16;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = (tm0 + t) * 16 + quarter * 4 + i;
          if (r < n_rows && j < n_keys) dst[(size_t)r * dst_pitch + j] = acc[i] * a.scale_log2e;
        }
      }
    }
  }
}

// Eq. 9 in one pass for the common small case (score mode 0 with a queue of queries, at most
// 64 mid keys, at most 16 queries per wavefront of the workgroup): wavefront w takes query
// rows 16 w .. 16 w + 15 against all keys, so a row's logits sit in the MFMA result registers
// of one 16-lane row (lane l: key (l % 16) of each 16-key tile, queries 4 (l / 16) .. + 3) and
// its softmax statistics are DPP reductions over that row, no LDS and no barrier; the
// probabilities are added up over the wavefront's queries (in-lane, then across the four lane
// rows) and the wavefronts' partial column sums meet in LDS once, added in wavefront order.
// sc[j] = (1/n) sum over the queued queries of their softmax row at mid key j.  `part` is LDS
// space for 64 floats per wavefront.  All threads call it; it ends with a barrier.
constexpr int kSmallKeys = 64;
__host__ __device__ inline bool saliency_is_small(const EvictArgs& a, int n_threads) {
  return a.qq != nullptr && a.mid_n <= kSmallKeys && a.n_rows <= 16 * (n_threads / 64);
}
template <int PPR, bool BF16>
__device__ void saliency_small(const EvictArgs& a, int pair, float* part, float* sc) {
  constexpr int STEPS = PPR / 4;          // 64-byte slices of a row
  constexpr int NT = kSmallKeys / 16;     // key tiles
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n_waves = blockDim.x >> 6;
  const int r16 = lane & 15, quarter = lane >> 4;
  const int n_rows = a.n_rows, n_keys = a.mid_n;
  const uint4* qq = reinterpret_cast<const uint4*>(a.qq) + (size_t)pair * a.line_len * PPR;
  const uint4* kc = reinterpret_cast<const uint4*>(a.kc) + ((size_t)pair * a.t_max + a.mid_lo) * PPR;
  float col[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) col[t] = 0.f;
  if (wave * 16 < n_rows) {
    uint4 qa[STEPS], kb[NT][STEPS];
    const int row = min(wave * 16 + r16, n_rows - 1);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) qa[s] = qq[(size_t)row * PPR + s * 4 + quarter];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int key = min(t * 16 + r16, n_keys - 1);
#pragma unroll
      for (int s = 0; s < STEPS; ++s) kb[t][s] = kc[(size_t)key * PPR + s * 4 + quarter];
    }
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < STEPS; ++s) {
        if (BF16) {
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qa[s]),
                                                           __builtin_bit_cast(bf16x8, kb[t][s]), acc[t], 0, 0, 0);
        } else {
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[s].x), __uint_as_float(kb[t][s].x), acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[s].y), __uint_as_float(kb[t][s].y), acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[s].z), __uint_as_float(kb[t][s].z), acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(qa[s].w), __uint_as_float(kb[t][s].w), acc[t], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // query wave*16 + quarter*4 + i: logits in log2 units, keys past the end masked
      float x[NT], mx = ninf();
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        x[t] = t * 16 + r16 < n_keys ? acc[t][i] * a.scale_log2e : ninf();
        mx = fmaxf(mx, x[t]);
      }
      mx = max_within_row(mx);
      float sum = 0.f;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        x[t] = ex2(x[t] - mx);
        sum += x[t];
      }
      sum = sum_within<16>(sum);
      const float inv = wave * 16 + quarter * 4 + i < n_rows ? 1.0f / sum : 0.f;
#pragma unroll
      for (int t = 0; t < NT; ++t) col[t] = __builtin_fmaf(x[t], inv, col[t]);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {   // the four lane rows hold four queries each
      col[t] += __shfl_xor(col[t], 16);
      col[t] += __shfl_xor(col[t], 32);
    }
  }
  if (quarter == 0) {
#pragma unroll
    for (int t = 0; t < NT; ++t) part[wave * kSmallKeys + t * 16 + r16] = col[t];
  }
  __syncthreads();
  if (tid < n_keys) {
    float t = 0.f;
    for (int w = 0; w < n_waves; ++w) t += part[w * kSmallKeys + tid];
    sc[tid] = t * (1.0f / (float)a.line_len);
  }
  __syncthreads();
}

// Eq. 10 for at most 64 candidates by one wavefront, no barrier inside: lane j holds candidate
// j, ranks it against the others by lane broadcasts and takes its slot from the keep mask.
// Same outputs as select_survivors.  Called by the first wavefront only.
__device__ void select_small(const float* sc, int m, int n_evict, int* src, int* dst, int* first) {
  const int j = threadIdx.x & 63;
  const float sj = j < m ? sc[j] : 0.f;
  int rank = 0;
  for (int k = 0; k < m; ++k) {
    const float sk = lane_bcast(sj, k);
    rank += (sk < sj) || (sk == sj && k < j);
  }
  const bool kp = j < m && rank >= n_evict;
  const unsigned long long mask = __ballot(kp);
  const unsigned long long gone = ~mask & (m >= 64 ? ~0ull : (1ull << m) - 1ull);
  if (j < m) {
    const int slot = __popcll(mask & ((1ull << j) - 1ull));
    if (kp && src) src[slot] = j;
    if (dst) dst[j] = kp ? slot : -1;
  }
  if (j == 0) *first = gone ? __builtin_ctzll(gone) : m;
}

// Column sums of the line's softmax rows for one pair.
//   modes 0, 1 (Eq. 9): sc[j] = (1/n) sum over the queued queries of their softmax row at mid
//     key j; mode 0 normalises each row over the mid keys only, mode 1 uses the decode
//     softmax's (max, sum) stored behind the row's logits;
//   mode 2 (accumulated attention): sc[j] = sum over the queued queries of the decode-time
//     probability of scored key j; row r scores len0 + r * len_step keys (the line grows), the
//     rest of the row is not read.
// `g` is the pair's queue [n_rows][guide_row] in global memory (logits in log2 units);
// `qs_lds` is an LDS copy area of n_rows * (guide_w + 2) floats, or nullptr when the queue is
// too large for LDS (then the three passes read global memory, where it stays in L2); `st` is
// LDS space for 2 * n_rows floats.  With a queue of queries the logits are computed here
// instead of copied (into `qs_lds`, else into the pair's rows of `a.guide_out`).  All threads
// call it; it ends with a barrier.  Sums run in a fixed order, so the result does not depend
// on timing.
template <int PPR, int MT>
__device__ void block_saliency(const EvictArgs& a, int pair, float* qs_lds, float* st, float* sc) {
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int n_rows = a.n_rows, mode = a.score_mode;
  int pitch = a.guide_row;            // floats between queue rows where the passes read them
  const float* g = a.guide + (size_t)pair * a.line_len * a.guide_row;
  const float* qs = g;
  if (a.qq) {
    float* dst = qs_lds;
    if (qs_lds) {
      pitch = a.guide_w + 2;
    } else {
      dst = a.guide_out + (size_t)pair * a.line_len * a.guide_row;
    }
    if (a.elem_bf16) fill_logits<PPR, true, MT>(a, pair, dst, pitch);
    else fill_logits<PPR, false, MT>(a, pair, dst, pitch);
    qs = dst;
    __syncthreads();   // also orders the global writes of this workgroup before its reads
  } else if (qs_lds) {
    // the LDS copy drops the padding (and keeps the rows off a common bank)
    pitch = a.guide_w + 2;
    // rows are whole 128-byte lines and contiguous: 16-byte loads, four in flight per thread
    const int row4 = a.guide_row >> 2, total4 = n_rows * row4;
    const float4* g4 = reinterpret_cast<const float4*>(g);
    for (int i0 = tid; i0 < total4; i0 += 4 * nthreads) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * nthreads;
        if (i < total4) v[u] = g4[i];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * nthreads;
        if (i < total4) {
          const int r = i / row4, j = (i - r * row4) * 4;
          float* dst = qs_lds + r * pitch + j;
          if (j + 0 < pitch) dst[0] = v[u].x;
          if (j + 1 < pitch) dst[1] = v[u].y;
          if (j + 2 < pitch) dst[2] = v[u].z;
          if (j + 3 < pitch) dst[3] = v[u].w;
        }
      }
    }
    qs = qs_lds;
    __syncthreads();
  }
  // Row statistics: a power-of-two team of threads per row.
  int team = 1;
  while (team < 16 && team * 2 * n_rows <= nthreads) team *= 2;
  const int rows_per_pass = nthreads / team;
  const int tr = tid / team, tq = tid % team;
  for (int r0 = 0; r0 < n_rows; r0 += rows_per_pass) {
    const int r = r0 + tr;
    const bool on = r < n_rows;
    const float* row = qs + (on ? r : 0) * pitch;
    float mx, inv;
    if (mode == 0) {
      const int len = a.len0;
      float lm = ninf();
      for (int j = tq; j < len; j += team) lm = fmaxf(lm, row[j]);
      for (int o = team >> 1; o > 0; o >>= 1) lm = fmaxf(lm, __shfl_xor(lm, o));
      float ls = 0.f;
      for (int j = tq; j < len; j += team) ls += ex2(row[j] - lm);
      for (int o = team >> 1; o > 0; o >>= 1) ls += __shfl_xor(ls, o);
      mx = lm;
      inv = 1.0f / ls;
    } else {
      mx = row[a.guide_w];
      inv = 1.0f / row[a.guide_w + 1];
    }
    if (on && tq == 0) {
      st[2 * r] = mx;
      st[2 * r + 1] = inv;
    }
  }
  __syncthreads();
  const float weight = mode == 2 ? 1.0f : 1.0f / (float)a.line_len;
  for (int j = tid; j < a.n_cols; j += nthreads) {
    float t = 0.f;
    // rows whose scored length does not reach column j come first (lengths grow with r)
    int r_first = 0;
    if (a.len_step > 0 && j >= a.len0) r_first = (j - a.len0) / a.len_step + 1;
    else if (a.len_step == 0 && j >= a.len0) r_first = n_rows;
    for (int r = r_first; r < n_rows; ++r) t += ex2(qs[r * pitch + j] - st[2 * r]) * st[2 * r + 1];
    sc[j] = t * weight;
  }
  __syncthreads();
}

// Mode 3 (random eviction): sc[j] = the 24-bit hash of (seed, layer, sequence, head, line, original
// position of candidate j) as a float -- exact, so ranking by it is ranking the integers.  The
// position comes from the survivor map or, behind the mapped candidates, from the index.  Ends
// with a barrier.
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}
__device__ void random_scores(const EvictArgs& a, int pair, float* sc) {
  const int32_t* map = a.pos + (size_t)pair * a.pos_pitch;
  uint32_t h = mix32(a.seed ^ 0x9e3779b9u);
  h = mix32(h + (uint32_t)a.layer);
  h = mix32(h + (uint32_t)(pair / a.n_heads));
  h = mix32(h + (uint32_t)(pair % a.n_heads));
  h = mix32(h + (uint32_t)a.line);
  for (int j = threadIdx.x; j < a.mid_n; j += blockDim.x) {
    const int32_t pos = j < a.pos_mapped ? map[j] : a.pos_base + j - a.pos_mapped;
    sc[j] = (float)(mix32(h + (uint32_t)pos) >> 8);
  }
  __syncthreads();
}

// Mode 2: adds the pair's accumulators to the line's column sums; sc[0 .. n_cols) becomes the
// attention each scored slot has received so far, slots beyond n_cols read as zero.  Ends with
// a barrier.
__device__ void add_accumulated(const EvictArgs& a, int pair, float* sc) {
  const float* acc = a.acc + (size_t)pair * a.guide_w;
  for (int j = threadIdx.x; j < a.guide_w; j += blockDim.x) sc[j] = j < a.n_cols ? sc[j] + acc[j] : 0.f;
  __syncthreads();
}

// Mode 2, after a selection: the accumulators move with their tokens (survivors of mid, then
// everything behind mid n_evict slots down); the freed slots start from zero.
__device__ void compact_accumulated(const EvictArgs& a, int pair, const float* sc, const int* src) {
  float* acc = a.acc + (size_t)pair * a.guide_w;
  const int mid_after = a.mid_n - a.n_evict, moved = a.guide_w - a.n_evict;
  for (int d = threadIdx.x; d < a.guide_w; d += blockDim.x)
    acc[d] = d < mid_after ? sc[src[d]] : (d < moved ? sc[d + a.n_evict] : 0.f);
}

// Original positions of the survivors: slot d of the compacted mid region holds candidate
// src[d], whose position is in the map if it survived an earlier eviction and follows from its
// index otherwise (the candidates behind the mapped ones are one whole line of consecutive
// tokens).  Every entry must be read before any is written: the caller puts a barrier (the one
// its row moves need anyway) between the two calls.
template <int BLOCK>
struct SurvivorPositions {
  static constexpr int PER = (kMaxMid + BLOCK - 1) / BLOCK;
  int32_t pv[PER];
  __device__ __forceinline__ void load(const EvictArgs& a, int pair, const int* src) {
    const int32_t* map = a.pos + (size_t)pair * a.pos_pitch;
    const int mid_after = a.mid_n - a.n_evict;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int d = i * BLOCK + (int)threadIdx.x;
      if (d < mid_after) {
        const int s = src[d];
        pv[i] = s < a.pos_mapped ? map[s] : a.pos_base + s - a.pos_mapped;
      }
    }
  }
  // A pair's map is a whole number of aligned 128-byte lines and all of them are written
  // (padding included), so no line is written in part.
  __device__ __forceinline__ void store(const EvictArgs& a, int pair) const {
    int32_t* map = a.pos + (size_t)pair * a.pos_pitch;
    const int mid_after = a.mid_n - a.n_evict;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int d = i * BLOCK + (int)threadIdx.x;
      if (d < a.pos_pitch) __builtin_nontemporal_store(d < mid_after ? pv[i] : 0, &map[d]);
    }
  }
};

// LDS words block_saliency needs beyond sc[]: the row statistics, and the queue copy when the
// whole allocation stays within the 64 KiB every workgroup may use (`fixed_words` = what the
// calling kernel keeps besides).
// LDS a workgroup of the end-of-line kernels may allocate dynamically, in words: what the
// device reports (64 KiB on older parts, 160 KiB here), less the kernels' static arrays.
size_t lds_limit_words() {
  static const size_t words = [] {
    int dev = 0, bytes = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
      bytes = 0;
    if (bytes < 64 * 1024) bytes = 64 * 1024;
    if (bytes > 160 * 1024) bytes = 160 * 1024;
    return (size_t)(bytes - 256) / 4;
  }();
  return words;
}
inline bool queue_fits_lds(int n_rows, int guide_w, size_t fixed_words) {
  return fixed_words + 2 * (size_t)n_rows + (size_t)n_rows * (guide_w + 2) <= lds_limit_words();
}
inline size_t saliency_lds_words(const EvictArgs& a, int n_threads, size_t fixed_words, bool small_ok = true) {
  if (small_ok && saliency_is_small(a, n_threads)) return 2 * (size_t)a.n_rows + (size_t)kSmallKeys * (n_threads / 64);
  return 2 * (size_t)a.n_rows +
         (queue_fits_lds(a.n_rows, a.guide_w, fixed_words) ? (size_t)a.n_rows * (a.guide_w + 2) : 0);
}
// A kernel that asks for more than the 64 KiB every device grants must be told so first.
template <class K>
hipError_t allow_lds(K kernel, size_t dyn_bytes) {
  if (dyn_bytes <= 64 * 1024 - 256) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)dyn_bytes);
}

// Eq. 10 for one pair: a candidate's rank is the number of candidates evicted before it
// (lower score, or equal score and older); the n_evict lowest ranks go.  Survivors get their
// new slot from a prefix count over the keep flags, one workgroup-width of candidates at a
// time.  Writes src[new slot] = old index (if src) and dst[old index] = new slot or -1 (if
// dst); *first receives the smallest evicted index (it must hold mid_n on entry).  All
// threads call it; it ends with a barrier.
__device__ void select_survivors(const float* sc, int m, int n_evict, int* src, int* dst, int* first,
                                 unsigned long long* masks) {
  const int tid = threadIdx.x, nthreads = blockDim.x, wave = tid >> 6, lane = tid & 63;
  const int n_waves = nthreads >> 6;
  int running = 0;
  for (int base = 0; base < m; base += nthreads) {
    const int j = base + tid;
    bool kp = false;
    if (j < m) {
      const float sj = sc[j];
      int rank = 0;
      for (int k = 0; k < m; ++k) {
        const float sk = sc[k];
        rank += (sk < sj) || (sk == sj && k < j);
      }
      kp = rank >= n_evict;
      if (!kp) atomicMin(first, j);
    }
    const unsigned long long mask = __ballot(kp);
    if (lane == 0) masks[wave] = mask;
    __syncthreads();
    int before = running, all = 0;
    for (int w = 0; w < n_waves; ++w) {
      const int c = __popcll(masks[w]);
      if (w < wave) before += c;
      all += c;
    }
    if (j < m) {
      const int slot = before + __popcll(mask & ((1ull << lane) - 1ull));
      if (kp && src) src[slot] = j;
      if (dst) dst[j] = kp ? slot : -1;
    }
    running += all;
    __syncthreads();
  }
}

// The arguments of layer blockIdx.y of a launch that covers several layers.
__device__ __forceinline__ EvictArgs layer_args(const EvictArgs& a0, const EvictLayers& ly) {
  EvictArgs a = a0;
  const int i = blockIdx.y;
  a.kc = ly.kc[i];
  a.vc = ly.vc[i];
  a.guide += i * ly.guide_stride;
  a.guide_out += i * ly.guide_stride;
  if (a.qq) a.qq = static_cast<const char*>(a.qq) + i * ly.qq_stride;
  a.pos += i * ly.pos_stride;
  a.acc += i * ly.acc_stride;
  a.layer += i;
  return a;
}

template <int PPR>  // 16-byte pieces per key row
__global__ __launch_bounds__(kBlock) void evict_kernel(const EvictArgs a0, const EvictLayers ly) {
  const EvictArgs a = layer_args(a0, ly);
  extern __shared__ int sm_raw[];
  const int m = a.mid_n, w = a.guide_w;
  float* sc = reinterpret_cast<float*>(sm_raw);        // [guide_w] saliency (mid candidates first)
  int* src = sm_raw + w;                               // [mid_n] source index of survivor slot
  float* st = reinterpret_cast<float*>(sm_raw + w + m);   // [n_rows][2] row statistics
  float* qs = a.queue_in_lds ? st + 2 * a.n_rows : nullptr; // [n_rows][guide_w + 2] queue copy
  __shared__ int sm_first;
  __shared__ unsigned long long sm_mask[kMaxWaves];

  const int tid = threadIdx.x;
  const int pair = blockIdx.x;
  const int mid_after = m - a.n_evict;

  if (tid == 0) sm_first = m;
  if (saliency_is_small(a, kBlock)) {
    float* part = st + 2 * a.n_rows;
    if (a.elem_bf16) saliency_small<PPR, true>(a, pair, part, sc);
    else saliency_small<PPR, false>(a, pair, part, sc);
    if (tid < 64) select_small(sc, m, a.n_evict, src, nullptr, &sm_first);
    __syncthreads();
  } else {
    if (a.score_mode == 3) random_scores(a, pair, sc);
    else block_saliency<PPR, 2>(a, pair, qs, st, sc);
    if (a.score_mode == 2) add_accumulated(a, pair, sc);
    select_survivors(sc, m, a.n_evict, src, nullptr, &sm_first, sm_mask);
    if (a.score_mode == 2) compact_accumulated(a, pair, sc, src);
  }
  SurvivorPositions<kBlock> sp;
  sp.load(a, pair, src);   // its latency overlaps with the first tile's loads

  // Destination rows [first, mid_after + n_tail), relative to mid_lo; rows in front of the
  // first hole stay where they are.
  const int first = sm_first;
  const int n_move = mid_after + a.n_tail - first;
  const size_t row_base = (size_t)pair * a.t_max + a.mid_lo;
  uint4* kc = reinterpret_cast<uint4*>(a.kc) + row_base * PPR;
  uint4* vc = reinterpret_cast<uint4*>(a.vc) + row_base * PPR;

  constexpr int kTile = kBlock * kPiecesPerThread;
  const int n_pieces = n_move * PPR;
  for (int t0 = 0; t0 < n_pieces; t0 += kTile) {
    uint4 kr[kPiecesPerThread], vr[kPiecesPerThread];
#pragma unroll
    for (int i = 0; i < kPiecesPerThread; ++i) {
      const int piece = t0 + i * kBlock + tid;
      if (piece < n_pieces) {
        const int d = first + piece / PPR, c = piece % PPR;
        const int s = d < mid_after ? src[d] : d + a.n_evict;
        kr[i] = kc[(size_t)s * PPR + c];
        vr[i] = vc[(size_t)s * PPR + c];
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();   // every source row of the tile is in registers
    if (t0 == 0) sp.store(a, pair);
#pragma unroll
    for (int i = 0; i < kPiecesPerThread; ++i) {
      const int piece = t0 + i * kBlock + tid;
      if (piece < n_pieces) {
        const int d = first + piece / PPR, c = piece % PPR;
        // Moved rows are next read by a later kernel: nontemporal stores (measured: the
        // compaction's store phase takes 4 us instead of 10 at 1280 pairs).
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, kr[i]), reinterpret_cast<u32x4*>(&kc[(size_t)d * PPR + c]));
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, vr[i]), reinterpret_cast<u32x4*>(&vc[(size_t)d * PPR + c]));
      }
    }
  }
}

// The same end-of-line work when all rows that may move (the mid candidates and the r recent
// lines) fit the workgroup's registers: they are requested first, so their memory latency
// overlaps with the saliency and the selection, and they are written straight to their new
// slots afterwards -- one memory round trip instead of one per tile, and no ordering hazard
// at all because every source row has left memory before the first store.  Costs the read of
// the n rows that end up evicted.
template <int PPR, int PIECES, int BLOCK>
__global__ __launch_bounds__(BLOCK) void evict_fast_kernel(const EvictArgs a0, const EvictLayers ly) {
  const EvictArgs a = layer_args(a0, ly);
  extern __shared__ int sm_raw[];
  const int m = a.mid_n, w = a.guide_w;
  float* sc = reinterpret_cast<float*>(sm_raw);        // [guide_w] saliency (mid candidates first)
  int* dstmap = sm_raw + w;                            // [mid_n] new slot, -1 = evicted
  int* src = dstmap + m;                               // [mid_n] source index of survivor slot
  float* st = reinterpret_cast<float*>(src + m);       // [n_rows][2] row statistics
  float* qs = a.queue_in_lds ? st + 2 * a.n_rows : nullptr; // [n_rows][guide_w + 2] queue copy
  __shared__ int sm_first;
  __shared__ unsigned long long sm_mask[kMaxWaves];

  const int tid = threadIdx.x;
  const int pair = blockIdx.x;
  const size_t row_base = (size_t)pair * a.t_max + a.mid_lo;
  uint4* kc = reinterpret_cast<uint4*>(a.kc) + row_base * PPR;
  uint4* vc = reinterpret_cast<uint4*>(a.vc) + row_base * PPR;
  const int n_pieces = (m + a.n_tail) * PPR;           // host: <= BLOCK * PIECES

  uint4 kr[PIECES], vr[PIECES];
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    const int piece = i * BLOCK + tid;                 // rows are contiguous: piece = 16-byte index
    if (piece < n_pieces) {
      kr[i] = kc[piece];
      vr[i] = vc[piece];
    }
  }
  if (tid == 0) sm_first = m;
  if (PIECES <= 4 && saliency_is_small(a, BLOCK)) {   // (the 8-piece instance has no registers to spare)
    float* part = st + 2 * a.n_rows;
    if (a.elem_bf16) saliency_small<PPR, true>(a, pair, part, sc);
    else saliency_small<PPR, false>(a, pair, part, sc);
    if (tid < 64) select_small(sc, m, a.n_evict, src, dstmap, &sm_first);
    __syncthreads();
  } else {
    if (a.score_mode == 3) random_scores(a, pair, sc);
    else block_saliency<PPR, (PIECES > 4 ? 1 : 2)>(a, pair, qs, st, sc);
    if (a.score_mode == 2) add_accumulated(a, pair, sc);
    select_survivors(sc, m, a.n_evict, src, dstmap, &sm_first, sm_mask);
    if (a.score_mode == 2) compact_accumulated(a, pair, sc, src);
  }
  SurvivorPositions<BLOCK> sp;
  sp.load(a, pair, src);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();   // every row that may move, and every mapped position, is in registers
  sp.store(a, pair);
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    const int piece = i * BLOCK + tid;
    if (piece < n_pieces) {
      const int s = piece / PPR, c = piece % PPR;
      const int d = s < m ? dstmap[s] : s - a.n_evict;
      if (d >= 0 && d != s) {
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, kr[i]), reinterpret_cast<u32x4*>(&kc[(size_t)d * PPR + c]));
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4, vr[i]), reinterpret_cast<u32x4*>(&vc[(size_t)d * PPR + c]));
      }
    }
  }
}

// kv_scores: the saliency alone.  With fold != 0 (mode 2 at the end of a line that does not
// evict) the line's sums are added to the accumulators instead.
template <int PPR>
__global__ __launch_bounds__(kBlock) void saliency_kernel(const EvictArgs a, float* out, int fold) {
  extern __shared__ int sm_raw[];
  float* sc = reinterpret_cast<float*>(sm_raw);        // [guide_w]
  float* st = sc + a.guide_w;
  float* qs = a.queue_in_lds ? st + 2 * a.n_rows : nullptr;
  const int pair = blockIdx.x;
  if (saliency_is_small(a, kBlock)) {
    float* part = st + 2 * a.n_rows;
    if (a.elem_bf16) saliency_small<PPR, true>(a, pair, part, sc);
    else saliency_small<PPR, false>(a, pair, part, sc);
  } else if (a.score_mode == 3) {
    random_scores(a, pair, sc);
  } else {
    block_saliency<PPR, 2>(a, pair, qs, st, sc);
    if (a.score_mode == 2) add_accumulated(a, pair, sc);
  }
  if (fold) {
    float* acc = a.acc + (size_t)pair * a.guide_w;
    for (int j = threadIdx.x; j < a.n_cols; j += kBlock) acc[j] = sc[j];
  } else {
    for (int j = threadIdx.x; j < a.mid_n; j += kBlock) out[(size_t)pair * a.mid_n + j] = sc[j];
  }
}

__global__ __launch_bounds__(kBlock) void copy_rows_kernel(uint4* dst, int64_t dst_pitch,
                                                           const uint4* src, int64_t src_pitch,
                                                           int64_t pieces_per_pair, int64_t total) {
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kBlock) {
    const int64_t p = i / pieces_per_pair, r = i % pieces_per_pair;
    dst[p * dst_pitch + r] = src[p * src_pitch + r];
  }
}

__global__ __launch_bounds__(kBlock) void zero_rows_kernel(uint4* dst, int64_t dst_pitch,
                                                           int64_t pieces_per_pair, int64_t total) {
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kBlock) {
    const int64_t p = i / pieces_per_pair, r = i % pieces_per_pair;
    dst[p * dst_pitch + r] = make_uint4(0, 0, 0, 0);
  }
}

__global__ __launch_bounds__(kBlock) void positions_kernel(int32_t* out, const int32_t* map, int32_t map_pitch,
                                                           int32_t mid_lo, int32_t mapped, int32_t len,
                                                           int32_t newest, int64_t total) {
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kBlock) {
    const int64_t p = i / len;
    const int32_t j = (int32_t)(i % len);
    int32_t v = j;
    if (j >= mid_lo + mapped) v = newest - (len - 1 - j);
    else if (j >= mid_lo) v = map[p * map_pitch + (j - mid_lo)];
    out[i] = v;
  }
}

__global__ __launch_bounds__(kBlock) void fill_u32_kernel(uint32_t* dst, uint32_t v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
    dst[i] = v;
}

unsigned grid_for(size_t n) {
  size_t g = (n + kBlock - 1) / kBlock;
  if (g > 4096) g = 4096;
  if (g < 1) g = 1;
  return (unsigned)g;
}

}  // namespace

// Launch geometry of the end-of-line kernels for one configuration.
struct EvictShape {
  bool fast4, fast8, queue_in_lds, small;
  int threads;
  size_t dyn;
};
template <int PPR>
EvictShape evict_shape(const EvictArgs& a, int n_layers = 1) {
  EvictShape sh;
  const size_t fixed = (size_t)a.guide_w + 2 * (size_t)a.mid_n;
  sh.queue_in_lds = queue_fits_lds(a.n_rows, a.guide_w, fixed);
  const int64_t pieces = (int64_t)(a.mid_n + a.n_tail) * PPR;
  // Measured on the five workloads: with at least two pairs per compute unit the tiled
  // kernel wins (it never reads the evicted rows); with fewer pairs than that and more than
  // one tile of rows (Lumina: 256 pairs, 245 rows of 256 B) the register-resident kernel with
  // 16 wavefronts per pair is 1.5x faster.
  // Across the layers of a shared launch the same holds per workgroup count -- unless the
  // line's logits take so much LDS that fewer than three 4-wavefront workgroups fit a compute
  // unit (Lumina-mGPT-1024: 102 KB), where 16 wavefronts per workgroup keep it busy.
  const int64_t groups = (int64_t)a.n_pairs * n_layers;   // workgroups of the launch
  const size_t dyn_tiled = (fixed + saliency_lds_words(a, kBlock, fixed)) * sizeof(int);
  const bool few = groups <= 256 || dyn_tiled > 160 * 1024 / 3;
  sh.fast4 = few && pieces > kBlock * kPiecesPerThread && pieces <= 1024 * 4;
  sh.fast8 = few && pieces > 1024 * 4 && pieces <= 1024 * 8;
  sh.threads = sh.fast4 || sh.fast8 ? 1024 : kBlock;
  sh.small = !sh.fast8 && saliency_is_small(a, sh.threads);
  sh.dyn = (fixed + saliency_lds_words(a, sh.threads, fixed, !sh.fast8)) * sizeof(int);
  return sh;
}

template <int PPR>
hipError_t launch_evict_t(const EvictArgs& a0, const EvictLayers* ly0, hipStream_t s) {
  EvictArgs a = a0;
  EvictLayers ly;
  if (ly0) {
    ly = *ly0;
  } else {
    ly = EvictLayers{};
    ly.count = 1;
    ly.kc[0] = a.kc;
    ly.vc[0] = a.vc;
  }
  if (ly.count < 1 || ly.count > kMaxEvictLayers) return hipErrorInvalidValue;
  const EvictShape sh = evict_shape<PPR>(a, ly.count);
  a.queue_in_lds = sh.queue_in_lds;
  const dim3 grid((unsigned)a.n_pairs, (unsigned)ly.count);
  hipError_t e;
  if (sh.fast4) {
    if ((e = allow_lds(evict_fast_kernel<PPR, 4, 1024>, sh.dyn)) != hipSuccess) return e;
    hipLaunchKernelGGL((evict_fast_kernel<PPR, 4, 1024>), grid, dim3(1024), sh.dyn, s, a, ly);
  } else if (sh.fast8) {
    if ((e = allow_lds(evict_fast_kernel<PPR, 8, 1024>, sh.dyn)) != hipSuccess) return e;
    hipLaunchKernelGGL((evict_fast_kernel<PPR, 8, 1024>), grid, dim3(1024), sh.dyn, s, a, ly);
  } else {
    if ((e = allow_lds(evict_kernel<PPR>, sh.dyn)) != hipSuccess) return e;
    hipLaunchKernelGGL((evict_kernel<PPR>), grid, dim3(kBlock), sh.dyn, s, a, ly);
  }
  return hipGetLastError();
}

hipError_t launch_evict(const EvictArgs& a, const EvictLayers* ly, int dtype, int head_dim, hipStream_t s) {
  const int row_bytes = head_dim * (dtype == 1 ? 2 : 4);
  switch (row_bytes / 16) {
    case 8: return launch_evict_t<8>(a, ly, s);
    case 16: return launch_evict_t<16>(a, ly, s);
    case 32: return launch_evict_t<32>(a, ly, s);
    default: return hipErrorInvalidValue;
  }
}

bool evict_layers_may_share_launch(const EvictArgs& a, int n_layers, int dtype, int head_dim) {
  if (!a.qq) return true;   // a queue of logits has its own rows per layer
  const int row_bytes = head_dim * (dtype == 1 ? 2 : 4);
  EvictShape sh;
  switch (row_bytes / 16) {
    case 8: sh = evict_shape<8>(a, n_layers); break;
    case 16: sh = evict_shape<16>(a, n_layers); break;
    case 32: sh = evict_shape<32>(a, n_layers); break;
    default: return false;
  }
  return sh.small || sh.queue_in_lds;   // the logits never leave LDS / registers
}

template <int PPR>
hipError_t launch_saliency_t(const EvictArgs& a0, float* out, hipStream_t s) {
  EvictArgs a = a0;
  const size_t fixed = (size_t)a.guide_w;
  a.queue_in_lds = queue_fits_lds(a.n_rows, a.guide_w, fixed);
  const size_t dyn = (fixed + saliency_lds_words(a, kBlock, fixed)) * sizeof(int);
  const hipError_t e = allow_lds(saliency_kernel<PPR>, dyn);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(saliency_kernel<PPR>, dim3((unsigned)a.n_pairs), dim3(kBlock), dyn, s, a, out,
                     out == nullptr ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_saliency(const EvictArgs& a, int dtype, int head_dim, float* out, hipStream_t s) {
  const int row_bytes = head_dim * (dtype == 1 ? 2 : 4);
  switch (row_bytes / 16) {
    case 8: return launch_saliency_t<8>(a, out, s);
    case 16: return launch_saliency_t<16>(a, out, s);
    case 32: return launch_saliency_t<32>(a, out, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_copy_rows(void* dst, int64_t dst_pitch_rows, const void* src,
                            int64_t src_pitch_rows, int32_t rows, int32_t n_pairs,
                            int32_t row_bytes, hipStream_t s) {
  if (rows <= 0 || n_pairs <= 0) return hipSuccess;
  const int64_t ppr = row_bytes / 16;
  const int64_t per_pair = (int64_t)rows * ppr, total = per_pair * n_pairs;
  hipLaunchKernelGGL(copy_rows_kernel, dim3(grid_for((size_t)total)), dim3(kBlock), 0, s,
                     reinterpret_cast<uint4*>(dst), dst_pitch_rows * ppr,
                     reinterpret_cast<const uint4*>(src), src_pitch_rows * ppr, per_pair, total);
  return hipGetLastError();
}

hipError_t launch_zero_rows(void* dst, int64_t dst_pitch_rows, int32_t rows, int32_t n_pairs,
                            int32_t row_bytes, hipStream_t s) {
  if (rows <= 0 || n_pairs <= 0) return hipSuccess;
  const int64_t ppr = row_bytes / 16;
  const int64_t per_pair = (int64_t)rows * ppr, total = per_pair * n_pairs;
  hipLaunchKernelGGL(zero_rows_kernel, dim3(grid_for((size_t)total)), dim3(kBlock), 0, s,
                     reinterpret_cast<uint4*>(dst), dst_pitch_rows * ppr, per_pair, total);
  return hipGetLastError();
}

hipError_t launch_positions(int32_t* out, const int32_t* map, int32_t map_pitch, int32_t mid_lo,
                            int32_t mapped, int32_t len, int32_t newest, int32_t n_pairs, hipStream_t s) {
  if (len <= 0 || n_pairs <= 0) return hipSuccess;
  const int64_t total = (int64_t)len * n_pairs;
  hipLaunchKernelGGL(positions_kernel, dim3(grid_for((size_t)total)), dim3(kBlock), 0, s, out, map,
                     map_pitch, mid_lo, mapped, len, newest, total);
  return hipGetLastError();
}

hipError_t launch_fill_u32(void* dst, uint32_t value, size_t n_words, hipStream_t s) {
  if (n_words == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(n_words)), dim3(kBlock), 0, s,
                     reinterpret_cast<uint32_t*>(dst), value, n_words);
  return hipGetLastError();
}

}  // namespace linear
