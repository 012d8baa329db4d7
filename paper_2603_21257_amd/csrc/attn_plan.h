// Host-side planning of an attention launch: which kernel, which tiles, how many split-KV pieces.
// No device types here: the file is shared by the HIP translation units and by plain C++.
#pragma once
#include <cstdint>
#include <vector>

namespace calvo {

// which MFMA kernel serves a batch with these suffix lengths (see attn_mfma.hip); the other calls take its answer
int attn_mfma_choose(const int32_t* suffix_lens, int n_reqs, int heads_per_wg);
int attn_mfma_tile_tokens(int variant, int heads_per_wg);
bool attn_mfma_splits_context(int variant);   // whether that kernel handles work items with n_splits > 1
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

// the batch's tiles of tile_tokens suffix tokens, heaviest first
std::vector<PlanTile> plan_tiles(const int32_t* prefix_blocks, const int32_t* suffix_lens, int n_reqs, int tile_tokens);

// length of the pieces a tile of n_sub sub-tiles is cut into when `want` pieces are asked for
int plan_piece_len(int n_sub, int want, const PlanParams& p);

// pieces per tile to ask for (1 = no cut), from a replay of the launch
int plan_pieces(const std::vector<PlanTile>& tiles, const PlanParams& p);

}  // namespace calvo
