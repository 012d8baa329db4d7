// Internal declarations shared by the host API and the HIP kernels of libcalvo.
// Not part of the public ABI (see include/calvo.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_plan.h"

namespace calvo {

// One request as the attention kernels see it (int32 x 4, device memory).
struct ReqDesc {
  int32_t table_off;  // offset of this request's block table inside the table array
  int32_t prefix_len; // P (tokens)
  int32_t suffix_len; // S (tokens)
  int32_t q_off;      // first row of this request inside q / out / k_suffix / v_suffix
};


struct AttnParams {
  const void* q;
  void* out;
  const void* pool_layer;   // this layer's [pool_blocks][2][B][Hkv][D]
  const ReqDesc* reqs;
  const WorkItem* items;
  const int32_t* item_index; // NULL, or n_items indices into items: the work items of this launch
  const int32_t* tables;    // per request: its block table, padded with copies of the last entry
  const int64_t* blk_offs;  // per request: slot * block_bytes of the even blocks, then of the odd blocks
  int32_t n_items;          // tiles over all requests
  int32_t n_q_heads, n_kv_heads, head_dim;
  int32_t heads_per_wg;     // MFMA kernel: 1, 2 or 4 query heads of one KV group per workgroup
  int32_t tile_tokens;      // suffix tokens per work item
  int32_t waves_per_wg;     // waves of an attention workgroup (8 or 4): layout of the split-KV partials
  float scale;              // softmax scale (natural-exponent units)
  // split-KV partial results, used by work items with n_splits > 1: per work item, head group, wave
  // (head of the group x 32-token half of the tile): part_o [32 rows][D] fp32 unnormalised,
  // part_ml [32 rows][2] = (softmax reference in exponent units, i.e. score * scale * log2 e, row sum)
  float* part_o;
  float* part_ml;
};

struct AppendParams {
  const void* k_suffix;
  const void* v_suffix;
  void* pool_layer;
  const ReqDesc* reqs;
  const int32_t* tables;
  int32_t n_reqs;
  int32_t total_tokens;
  int32_t row_chunks;       // 16-byte chunks in one token's K (or V) row: Hkv*D*elt/16
};

// Scatter n_blocks consecutive source blocks to the pool slots table[0..n_blocks).
hipError_t launch_scatter_blocks(const void* src, void* pool_layer, const int32_t* table, int64_t n_blocks,
                                 int32_t blk_bytes, int grid, hipStream_t stream);
hipError_t launch_suffix_append(const AppendParams& p, hipStream_t stream);
// test hook: occupies `stream` for about us microseconds (bounded), see kernels_ingest.hip
hipError_t launch_delay(int us, hipStream_t stream);
hipError_t launch_attn_simple(const AttnParams& p, int dtype, int total_tokens, hipStream_t stream);
// The pipelined bf16 / head-dim-128 kernels (attn_pipeline.h).  The *_prepare calls raise the
// kernels' dynamic LDS limit; once per device, before the first launch.
hipError_t attn_pipe_prepare();
hipError_t attn_duo_prepare();
hipError_t launch_attn_pipe(const AttnParams& p, hipStream_t stream);
hipError_t launch_attn_duo(const AttnParams& p, hipStream_t stream);
int attn_duo_tile_tokens(int heads_per_wg);
// combines the pieces of every split tile into out (bf16); n_split_tiles entries in split_tiles =
// indices of the first work item of each split tile
hipError_t launch_merge_splits(const AttnParams& p, const int32_t* split_tiles, int n_split_tiles, hipStream_t stream);
int attn_pipe_tile_tokens(int heads_per_wg);

constexpr int kBlockTokens = 16;
// Entries appended to every request's device-side block table (copies of its last entry): the
// pipelined attention kernel requests blocks up to 2 * (ring depth + 1) + 2 past the last one.
constexpr int kTablePad = 32;

}  // namespace calvo
