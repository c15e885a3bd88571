// Internal launch interface between the host-side state machine and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace linear {

constexpr int kBlock = 256;        // workgroup size of the eviction and copy kernels
constexpr int kMaxSplit = 64;      // workgroups one pair's keys may be split over
constexpr int kMaxMid = 2048;      // mid candidates the end-of-line kernels rank and map

// One decode step of one layer (Eq. 2-4 plus the per-query term of Eq. 9).
struct DecodeArgs {
  const void* q;      // [P, d] elem
  const void* k_new;  // [P, d] elem
  const void* v_new;  // [P, d] elem
  const float* cos_sin;  // null, or [d] floats: q and k_new arrive unrotated and are rotated here
                         //   (rotary embedding, element t paired with t + d/2): cos of the d/2
                         //   pair angles of the new token's position, then their sines
  void* kc;           // [P, t_max, d] elem
  void* vc;           // [P, t_max, d] elem
  void* out;          // [P, d] float, or bfloat16 when out_bf16 is set
  int32_t out_bf16;   // the result leaves in bfloat16 (round to nearest even)
  float* part_o;      // [P, max_split, d]   split partial numerators
  float* part_ml;     // [P, max_split, 2]   split partial (max, sum) in log2 units
  float* guide;       // [P, n, guide_row] guide queue of the layer, already advanced to this
                      //                   query's row: mid logits (log2 units), then (m, l), then padding
  int64_t guide_pitch;  // floats between the rows of consecutive pairs = n * guide_row
  int32_t guide_w;    // logits a queue row holds; the row's (m, l) sit behind them
  int32_t guide_row;  // floats per queue row in memory: guide_w + 2 rounded up to whole 128-byte lines
  void* qq;           // when not null: the query itself is queued (Eq. 8 as printed) at
                      //   qq + pair * qq_pitch bytes (the layer's [P, n, d] elem queue, already
                      //   advanced to this query's row) and mid_n is 0
  int64_t qq_pitch;   // bytes between consecutive pairs' queues = n * d * sizeof(elem)
  int32_t stage_new;  // the appended token's own logit is scored too (accumulated attention)
  int32_t store_ml;   // the decode softmax's (m, l) are needed (score modes 1 and 2)
  int32_t n_pairs;    // P = Bz * H
  int32_t t;          // keys visible to this query, the new one included
  int32_t t_max;      // row pitch of the caches, in keys
  int32_t rows_per_split;  // cached keys per workgroup (a multiple of the row-group size)
  int32_t n_split;    // workgroups per pair
  int32_t n_waves;    // wavefronts per workgroup
  int32_t new_wave;   // wavefront of the last split that counts the appended token
  int32_t depth;      // row groups a wavefront holds (an instantiated value, see decode_depth_for)
  int32_t max_split;  // pitch of the partial buffers
  int32_t mid_lo;     // first mid key (cache row index)
  int32_t mid_n;      // mid keys to score at this step (0: none)
  int32_t score_mode;
  float scale_log2e;  // logit scale times log2(e)
};

// End of line: saliency from the guide queue (Eq. 9), BottomK (Eq. 10), compaction (Eq. 5-7).
struct EvictArgs {
  void* kc;
  void* vc;
  int32_t* pos;        // [P, pos_pitch] original positions of the mid survivors (see pos_mapped)
  int32_t pos_pitch;
  int32_t pos_mapped;  // mid candidates 0 .. pos_mapped-1 have their position in the map; the
  int32_t pos_base;    //   others are consecutive tokens: candidate j sits at pos_base + j - pos_mapped
  const float* guide;  // [P, n, guide_row] of the layer
  float* guide_out;    // query queue only: where the logits go when the queue does not fit LDS
  const void* qq;      // [P, n, d] elem queue of the line's queries, or null (logits are queued)
  float scale_log2e;   // logit scale times log2(e) (query queue: applied at the end of the line)
  int32_t elem_bf16;   // element type of the caches and of the query queue
  float* acc;          // [P, guide_w] attention accumulated per cache slot behind the anchor (mode 2)
  int32_t n_rows;      // queries queued in the line (n at an end of line)
  int32_t line_len;    // n, the divisor of Eq. 9
  int32_t guide_w;     // logits per queue row
  int32_t guide_row;   // floats per queue row in memory (whole 128-byte lines)
  int32_t len0;        // scored keys of the first queued row ...
  int32_t len_step;    // ... and how many more every later row has (mode 2: 1, else 0)
  int32_t n_cols;      // columns to sum: mid_n, or every scored key of the line's last row (mode 2)
  int32_t do_evict;    // 0: only fold the line's queue into acc (mode 2 on lines that do not evict)
  int32_t score_mode;
  int32_t queue_in_lds;  // set by the launcher: the line's queue fits the workgroup's LDS
  int32_t n_pairs;
  int32_t t_max;
  int32_t mid_lo;
  int32_t mid_n;     // candidates
  int32_t n_evict;   // n
  int32_t n_tail;    // rows behind mid that slide down (r lines)
  // score mode 3 (random eviction): what the candidates' keys are hashed from
  uint32_t seed;
  int32_t layer;     // layer index (of the launch's first layer: grid.y is added)
  int32_t line;      // 1-based raster line that ends
  int32_t n_heads;   // pair = sequence * n_heads + head
};

// The layers one end-of-line launch covers (grid.y): layer i of the launch uses kc[i], vc[i] and
// the scratch parts of EvictArgs advanced by i strides.  All of them are in the same state.
constexpr int kMaxEvictLayers = 48;
struct EvictLayers {
  int32_t count;
  int64_t guide_stride;  // floats
  int64_t qq_stride;     // bytes
  int64_t pos_stride;    // int32 entries
  int64_t acc_stride;    // floats
  void* kc[kMaxEvictLayers];
  void* vc[kMaxEvictLayers];
};

hipError_t launch_decode(const DecodeArgs& a, int dtype, int head_dim, hipStream_t s);
int decode_rows_per_group(int dtype, int head_dim);   // keys one wave-wide load covers
int decode_max_waves(int depth);                      // wavefronts per workgroup at that depth
int decode_depth_for(int groups_per_wave);            // smallest instantiated depth >= the argument, 0 if none
// `ly` may be null (one layer: a.kc, a.vc).  False from evict_layers_may_share_launch means the
// launch would route every layer's logits through the one shared global scratch row set.
hipError_t launch_evict(const EvictArgs& a, const EvictLayers* ly, int dtype, int head_dim, hipStream_t s);
bool evict_layers_may_share_launch(const EvictArgs& a, int n_layers, int dtype, int head_dim);
// out[P, mid_n] = saliency of the mid candidates from the queue rows so far (Eq. 9; in mode 2
// the accumulated attention including the rows so far).
hipError_t launch_saliency(const EvictArgs& a, int dtype, int head_dim, float* out, hipStream_t s);

// dst[p, 0:rows, :] = src[p, 0:rows, :] for p < n_pairs; pitches in rows; row_bytes % 16 == 0.
hipError_t launch_copy_rows(void* dst, int64_t dst_pitch_rows, const void* src,
                            int64_t src_pitch_rows, int32_t rows, int32_t n_pairs,
                            int32_t row_bytes, hipStream_t s);
// dst[p, 0:rows, :] = 0.
hipError_t launch_zero_rows(void* dst, int64_t dst_pitch_rows, int32_t rows, int32_t n_pairs,
                            int32_t row_bytes, hipStream_t s);
// out[p, j] for j < len = original position of cache row j: j in front of mid_lo, the map's
// entry for the `mapped` rows from mid_lo on, and consecutive positions ending at `newest` behind.
hipError_t launch_positions(int32_t* out, const int32_t* map, int32_t map_pitch, int32_t mid_lo,
                            int32_t mapped, int32_t len, int32_t newest, int32_t n_pairs, hipStream_t s);
hipError_t launch_fill_u32(void* dst, uint32_t value, size_t n_words, hipStream_t s);
// Reads rows [0, rows) of every pair of `a` and (when not null) `b` and discards them: the plain
// streaming yardstick of the probe entry points.  `sink` receives nothing in practice.
hipError_t launch_stream_read(const void* a, const void* b, int64_t n_pairs, int64_t rows, int64_t pitch_rows,
                              int32_t row_bytes, uint32_t* sink, hipStream_t s);
hipError_t launch_empty(int32_t groups, int32_t threads, hipStream_t s);

}  // namespace linear
