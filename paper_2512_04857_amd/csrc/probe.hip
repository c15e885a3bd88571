// Plain streaming read of cache rows and an empty kernel: the yardsticks the decode kernel is
// measured against (the same bytes with no arithmetic and no dependence between loads; the cost
// of a launch as such).
#include "kernels.h"

namespace linear {
namespace {

constexpr int kPieces = 8;   // 16-byte loads a thread has in flight

// Rows [0, rows) of every pair of up to two row-major tensors with `pitch` rows between pairs
// (K and V of one layer): the 16-byte pieces are dealt to threads in wave-contiguous runs, every
// thread issues kPieces loads before it uses any.  Nothing is written unless the exclusive-or of
// everything a thread read equals `never` (the caller passes a value that cannot occur, so the
// loads cannot be dropped and no store happens).
__global__ __launch_bounds__(kBlock) void stream_read_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                             int64_t pieces_per_pair, int64_t pitch_pieces,
                                                             int64_t total, uint32_t never, uint32_t* sink) {
  const int64_t tile = (int64_t)blockIdx.x * (kBlock * kPieces);
  uint4 r[kPieces];
#pragma unroll
  for (int i = 0; i < kPieces; ++i) {
    int64_t p = tile + (int64_t)i * kBlock + threadIdx.x;
    if (p >= total) p = total - 1;                       // re-read the last piece: straight-line loads
    const uint4* base = a;
    int64_t q = p;
    if (b != nullptr && p >= total / 2) {                // second half of the piece space: the other tensor
      base = b;
      q = p - total / 2;
    }
    const int64_t pair = q / pieces_per_pair, within = q - pair * pieces_per_pair;
    r[i] = base[pair * pitch_pieces + within];
  }
  uint32_t x = 0;
#pragma unroll
  for (int i = 0; i < kPieces; ++i) x ^= r[i].x ^ r[i].y ^ r[i].z ^ r[i].w;
  if (x == never && sink != nullptr) sink[0] = x;
}

__global__ void empty_kernel() {}

}  // namespace

hipError_t launch_stream_read(const void* a, const void* b, int64_t n_pairs, int64_t rows, int64_t pitch_rows,
                              int32_t row_bytes, uint32_t* sink, hipStream_t s) {
  if (n_pairs <= 0 || rows <= 0) return hipSuccess;
  const int64_t ppr = row_bytes / 16;
  const int64_t per_pair = rows * ppr;
  const int64_t total = per_pair * n_pairs * (b ? 2 : 1);
  const int64_t tiles = (total + kBlock * kPieces - 1) / (kBlock * kPieces);
  if (tiles > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)tiles), dim3(kBlock), 0, s, reinterpret_cast<const uint4*>(a),
                     reinterpret_cast<const uint4*>(b), per_pair, pitch_rows * ppr, total, 0x5bd1e995u, sink);
  return hipGetLastError();
}

hipError_t launch_empty(int32_t groups, int32_t threads, hipStream_t s) {
  hipLaunchKernelGGL(empty_kernel, dim3((unsigned)groups), dim3((unsigned)threads), 0, s);
  return hipGetLastError();
}

}  // namespace linear
