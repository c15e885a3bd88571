// End-of-line eviction (Eq. 10) and in-place gather-compaction (Eq. 5-7), plus the small
// copy / fill kernels of kv_init and kv_gather.
//
// One workgroup per (sequence, head) pair.  The accumulated saliency of the mid candidates
// is ranked by counting (stable: equal scores rank by age), the n lowest are dropped, the
// survivors and the r recent lines slide down over the holes.  Rows only ever move to a
// lower or equal index and keep their order, so processing destination rows in ascending
// tiles -- load the tile's source rows into registers, barrier, store -- never overwrites
// a row that is still to be read.
#include "kernels.h"

namespace linear {
namespace {

constexpr int kPiecesPerThread = 4;   // 16-byte pieces of K (and of V) a thread holds per tile

template <int PPR>  // 16-byte pieces per key row
__global__ __launch_bounds__(kBlock) void evict_kernel(const EvictArgs a) {
  extern __shared__ int sm_raw[];
  float* sc = reinterpret_cast<float*>(sm_raw);        // [mid_n] scores
  int* keep = sm_raw + a.mid_n;                        // [mid_n] 1 = survives
  int* src = sm_raw + 2 * a.mid_n;                     // [mid_n] source index of survivor slot
  __shared__ int sm_first;

  const int tid = threadIdx.x;
  const int pair = blockIdx.x;
  float* acc = a.acc + (size_t)pair * a.mid_n;
  const int m = a.mid_n;
  const int mid_after = m - a.n_evict;

  if (tid == 0) sm_first = m;
  for (int j = tid; j < m; j += kBlock) {
    sc[j] = acc[j];
    acc[j] = 0.f;                                      // next line starts from zero
  }
  __syncthreads();
  // Eq. 10: rank = number of candidates that are evicted before this one.
  for (int j = tid; j < m; j += kBlock) {
    const float sj = sc[j];
    int rank = 0;
    for (int k = 0; k < m; ++k) {
      const float sk = sc[k];
      rank += (sk < sj) || (sk == sj && k < j);
    }
    const int kp = rank >= a.n_evict;
    keep[j] = kp;
    if (!kp) atomicMin(&sm_first, j);
  }
  __syncthreads();
  for (int j = tid; j < m; j += kBlock) {
    if (keep[j]) {
      int dst = 0;
      for (int k = 0; k < j; ++k) dst += keep[k];
      src[dst] = j;
    }
  }
  __syncthreads();

  // Destination rows [first, mid_after + n_tail), relative to mid_lo; rows in front of the
  // first hole stay where they are.
  const int first = sm_first;
  const int n_move = mid_after + a.n_tail - first;
  const size_t row_base = (size_t)pair * a.t_max + a.mid_lo;
  uint4* kc = reinterpret_cast<uint4*>(a.kc) + row_base * PPR;
  uint4* vc = reinterpret_cast<uint4*>(a.vc) + row_base * PPR;
  int32_t* pos = a.pos + row_base;

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
#pragma unroll
    for (int i = 0; i < kPiecesPerThread; ++i) {
      const int piece = t0 + i * kBlock + tid;
      if (piece < n_pieces) {
        const int d = first + piece / PPR, c = piece % PPR;
        kc[(size_t)d * PPR + c] = kr[i];
        vc[(size_t)d * PPR + c] = vr[i];
      }
    }
  }
  for (int t0 = 0; t0 < n_move; t0 += kBlock) {
    const int d = first + t0 + tid;
    int32_t p = 0;
    const bool on = t0 + tid < n_move;
    if (on) p = pos[d < mid_after ? src[d] : d + a.n_evict];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (on) pos[d] = p;
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

__global__ __launch_bounds__(kBlock) void iota_rows_kernel(int32_t* pos, int64_t pitch, int32_t rows,
                                                           int64_t total) {
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kBlock) {
    const int64_t p = i / rows, r = i % rows;
    pos[p * pitch + r] = (int32_t)r;
  }
}

__global__ __launch_bounds__(kBlock) void copy_i32_rows_kernel(int32_t* dst, int64_t dst_pitch,
                                                               const int32_t* src, int64_t src_pitch,
                                                               int32_t rows, int64_t total) {
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kBlock) {
    const int64_t p = i / rows, r = i % rows;
    dst[p * dst_pitch + r] = src[p * src_pitch + r];
  }
}

__global__ __launch_bounds__(kBlock) void fill_u32_kernel(uint32_t* dst, uint32_t v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
    dst[i] = v;
}

__global__ __launch_bounds__(kBlock) void scale_f32_kernel(float* out, const float* in, float f,
                                                           size_t n) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
    out[i] = in[i] * f;
}

unsigned grid_for(size_t n) {
  size_t g = (n + kBlock - 1) / kBlock;
  if (g > 4096) g = 4096;
  if (g < 1) g = 1;
  return (unsigned)g;
}

}  // namespace

hipError_t launch_evict(const EvictArgs& a, int dtype, int head_dim, hipStream_t s) {
  const int row_bytes = head_dim * (dtype == 1 ? 2 : 4);
  const size_t dyn = (size_t)a.mid_n * 3 * sizeof(int);
  const dim3 grid((unsigned)a.n_pairs), block(kBlock);
  switch (row_bytes / 16) {
    case 8: hipLaunchKernelGGL((evict_kernel<8>), grid, block, dyn, s, a); break;
    case 16: hipLaunchKernelGGL((evict_kernel<16>), grid, block, dyn, s, a); break;
    case 32: hipLaunchKernelGGL((evict_kernel<32>), grid, block, dyn, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
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

hipError_t launch_iota_rows(int32_t* pos, int64_t pitch, int32_t rows, int32_t n_pairs,
                            hipStream_t s) {
  if (rows <= 0 || n_pairs <= 0) return hipSuccess;
  const int64_t total = (int64_t)rows * n_pairs;
  hipLaunchKernelGGL(iota_rows_kernel, dim3(grid_for((size_t)total)), dim3(kBlock), 0, s, pos, pitch,
                     rows, total);
  return hipGetLastError();
}

hipError_t launch_copy_i32_rows(int32_t* dst, int64_t dst_pitch, const int32_t* src,
                                int64_t src_pitch, int32_t rows, int32_t n_pairs, hipStream_t s) {
  if (rows <= 0 || n_pairs <= 0) return hipSuccess;
  const int64_t total = (int64_t)rows * n_pairs;
  hipLaunchKernelGGL(copy_i32_rows_kernel, dim3(grid_for((size_t)total)), dim3(kBlock), 0, s, dst,
                     dst_pitch, src, src_pitch, rows, total);
  return hipGetLastError();
}

hipError_t launch_fill_u32(void* dst, uint32_t value, size_t n_words, hipStream_t s) {
  if (n_words == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(n_words)), dim3(kBlock), 0, s,
                     reinterpret_cast<uint32_t*>(dst), value, n_words);
  return hipGetLastError();
}

hipError_t launch_scale_f32(float* out, const float* in, float f, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(scale_f32_kernel, dim3(grid_for(n)), dim3(kBlock), 0, s, out, in, f, n);
  return hipGetLastError();
}

}  // namespace linear
