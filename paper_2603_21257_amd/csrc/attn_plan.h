// Host-side planning of an attention launch: which kernel, which tiles, how many split-KV pieces.
// No device types here: the file is shared by the HIP translation units and by plain C++.
#pragma once
#include <cstdint>
#include <vector>

namespace calvo {

// which shape of the pipelined MFMA kernel serves a batch with these suffix lengths (attn_plan.cpp);
// the other calls take its answer
constexpr int kAttnPipe = 3;   // 8-wave workgroups, 64-token tiles
constexpr int kAttnDuo = 4;    // two 4-wave workgroups per CU, 32-token tiles
int attn_mfma_choose(const int32_t* suffix_lens, int n_reqs, int heads_per_wg);
int attn_mfma_tile_tokens(int variant, int heads_per_wg);
int attn_mfma_waves_per_wg(int variant);

// query heads of one KV group that share a workgroup: 4, 2 or 1 (the largest that divides the group)
inline int attn_heads_per_wg(int n_q_heads, int n_kv_heads) {
  const int g = n_q_heads / n_kv_heads;
  return (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
}

struct PlanTile {
  int32_t req, tile;
  int32_t n_sub;      // 32-key sub-tiles its rows see (prefix + the suffix up to the tile's end)
};

struct PlanParams {
  int n_head_groups;  // workgroups per work item
  int wg_slots;       // workgroups resident on the device at a time
  int split_min;      // shortest piece of a cut tile, in sub-tiles
  int split_fill;     // cost of a workgroup's pipeline fill and drain, in sub-tile steps
  int force_splits;   // > 0: cut every tile into this many pieces (test knob)
};

// A work item is one workgroup's share of the attention of one request: a tile of suffix tokens
// (tile_tokens of them) over the sub-tile range [sub_begin, sub_end) of its context (32-key
// sub-tiles).  Normally a tile is one work item covering its whole context; a tile may be cut into
// n_splits > 1 pieces (split-KV), which then run as separate workgroups, write partial results
// (unnormalised O, running maximum, row sum) and are combined by a merge kernel; the pieces of one
// tile are consecutive work items.  The device reads this struct as it is.
struct WorkItem {
  int32_t req;
  int32_t q_tile;     // tile index inside the request's suffix
  int32_t sub_begin;  // first 32-key sub-tile of this piece
  int32_t sub_end;    // one past its last sub-tile (the last piece ends at the tile's causal limit)
  int32_t n_splits;   // pieces the tile is cut into; 1 = the kernel writes the final output itself
  int32_t first_item; // index of the tile's first piece
  int32_t pad0, pad1;
};

struct PlanItems {
  std::vector<WorkItem> items;
  std::vector<int32_t> split_tiles;              // first work item of every cut tile
  std::vector<std::vector<int32_t>> groups;      // chunk-granular layers: work item indices per launch; else empty
};

// the batch's tiles of tile_tokens suffix tokens, heaviest first
std::vector<PlanTile> plan_tiles(const int32_t* prefix_blocks, const int32_t* suffix_lens, int n_reqs, int tile_tokens);

// length of the pieces a tile of n_sub sub-tiles is cut into when `want` pieces are asked for
int plan_piece_len(int n_sub, int want, const PlanParams& p);

// pieces per tile to ask for (1 = no cut), from a replay of the launch
int plan_pieces(const std::vector<PlanTile>& tiles, const PlanParams& p);

// work items of a whole-layer launch: every tile cut into pieces of plan_piece_len(n_sub, want)
PlanItems plan_items(const std::vector<PlanTile>& tiles, int want, const PlanParams& p);

// Work items of a layer that was loaded in n_chunks chunks of chunk_blocks block indices (even): piece
// k of a tile covers the sub-tiles of chunk k that lie wholly inside the request's prefix and goes
// into launch k, which needs blocks below (k + 1) * chunk_blocks only; what is left of the tile (the
// end of the prefix that shares a sub-tile with the suffix, the suffix itself) is its last piece, in
// launch n_chunks, which needs the whole layer.
PlanItems plan_items_chunked(const std::vector<PlanTile>& tiles, const int32_t* prefix_blocks, int chunk_blocks, int n_chunks);

}  // namespace calvo
