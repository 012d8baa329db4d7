// Planning of an attention launch on the host.  A tile of suffix tokens normally is one work item
// that walks its whole context.  Short suffixes over long contexts (the paper's main regime,
// Section 2.2 and Table 1) give too few tiles for the chip, and some batches give a workgroup
// count just above a whole number of rounds; in both cases every tile's context is cut into pieces
// that run as separate workgroups and are merged afterwards.  How many pieces is decided by
// replaying the launch: workgroups start in grid order on the first free workgroup slot, a piece
// costs its sub-tiles plus a fixed pipeline fill and drain, cut tiles pay the merge.
#include "attn_plan.h"

#include <algorithm>
#include <cstdlib>
#include <functional>

#include "../../include/calvo.h"

namespace calvo {

int attn_pipe_tile_tokens(int heads_per_wg);
int attn_duo_tile_tokens(int heads_per_wg);

// Two shapes of the pipelined kernel serve bf16 / head-dim-128 batches: kAttnPipe (8-wave workgroups,
// 64-token tiles for four heads: half the K/V traffic into LDS per query row) and kAttnDuo (two
// 4-wave workgroups per CU, 32-token tiles).  With the short queries of the paper's Table 1 half of
// a 64-token tile's waves would idle, so the smaller tiles win there.  The environment variable
// CALVO_ATTN_VARIANT (3 or 4, read per call: tests switch it inside one process) forces one.
int attn_mfma_choose(const int32_t* suffix_lens, int n_reqs, int heads_per_wg) {
  const char* e = getenv("CALVO_ATTN_VARIANT");
  if (e && (e[0] == '3' || e[0] == '4') && e[1] == 0) return e[0] - '0';
  // query rows the tiles of each kernel would hold, empty ones included
  const int t3 = attn_pipe_tile_tokens(heads_per_wg), t4 = attn_duo_tile_tokens(heads_per_wg);
  int64_t rows3 = 0, rows4 = 0;
  for (int r = 0; r < n_reqs; r++) {
    rows3 += (int64_t)((suffix_lens[r] + t3 - 1) / t3) * t3;
    rows4 += (int64_t)((suffix_lens[r] + t4 - 1) / t4) * t4;
  }
  return rows3 * 9 > rows4 * 10 ? kAttnDuo : kAttnPipe;       // the larger tiles would carry over 10 % more rows
}

int attn_mfma_waves_per_wg(int variant) { return variant == kAttnPipe ? 8 : 4; }

int attn_mfma_tile_tokens(int variant, int heads_per_wg) {
  return variant == kAttnDuo ? attn_duo_tile_tokens(heads_per_wg) : attn_pipe_tile_tokens(heads_per_wg);
}

std::vector<PlanTile> plan_tiles(const int32_t* prefix_blocks, const int32_t* suffix_lens, int n_reqs, int tile_tokens) {
  std::vector<PlanTile> tiles;
  for (int r = 0; r < n_reqs; r++) {
    const int nt = (suffix_lens[r] + tile_tokens - 1) / tile_tokens;
    for (int t = 0; t < nt; t++) {
      const int64_t keys = (int64_t)prefix_blocks[r] * 16 + std::min<int64_t>((int64_t)(t + 1) * tile_tokens, suffix_lens[r]);
      tiles.push_back({r, t, (int32_t)((keys + 31) / 32)});
    }
  }
  std::stable_sort(tiles.begin(), tiles.end(), [](const PlanTile& a, const PlanTile& b) { return a.n_sub > b.n_sub; });
  return tiles;
}

// The kernels run a piece of n sub-tiles as one fill step, unrolled steady iterations and a few
// slower drain steps; lengths of the form 8k + 2 leave two drain steps in either kernel.
int plan_piece_len(int n_sub, int want, const PlanParams& p) {
  const int n = std::max(1, std::min(want, p.force_splits ? n_sub : n_sub / p.split_min));
  int len = (n_sub + n - 1) / n;
  if (n > 1 && !p.force_splits) len = (len + 5) / 8 * 8 + 2;
  return len;
}

int plan_pieces(const std::vector<PlanTile>& tiles, const PlanParams& p) {
  if (p.force_splits) return p.force_splits;
  const int64_t wgs = (int64_t)tiles.size() * p.n_head_groups;
  if (wgs <= 0 || wgs > 16 * (int64_t)p.wg_slots) return 1;     // many rounds: the last one hardly matters
  const int cands[] = {1, 2, 3, 4, 5, 6, 8, 12, 16, 24, 32, 48, 64};
  int want = 1;
  double best = 0;
  std::vector<int64_t> heap;
  for (int n : cands) {
    if (n > 1 && wgs * n > 16 * (int64_t)p.wg_slots) break;
    heap.assign((size_t)p.wg_slots, 0);            // min-heap of the times at which workgroup slots become free
    auto cmp = std::greater<int64_t>();
    bool cut = false;
    int64_t end = 0;
    for (const PlanTile& t : tiles) {
      const int len = plan_piece_len(t.n_sub, n, p);
      const int np = (t.n_sub + len - 1) / len;
      cut |= np > 1;
      for (int k = 0; k < np; k++) {
        const int64_t cost = std::min(t.n_sub, (k + 1) * len) - k * len + p.split_fill;
        for (int h = 0; h < p.n_head_groups; h++) {
          std::pop_heap(heap.begin(), heap.end(), cmp);
          heap.back() += cost;
          end = std::max(end, heap.back());
          std::push_heap(heap.begin(), heap.end(), cmp);
        }
      }
    }
    const double span = (double)end + (cut ? p.split_fill : 0);
    if (n == 1 || span < best * 0.98) {            // a cut has to win by 2 % over what is chosen so far
      best = span;
      want = n;
    }
    if (!cut && n > 1) break;                       // longer cuts are refused by split_min: nothing changes
  }
  return want;
}

PlanItems plan_items(const std::vector<PlanTile>& tiles, int want, const PlanParams& p) {
  PlanItems out;
  for (const PlanTile& t : tiles) {
    const int len = plan_piece_len(t.n_sub, want, p);
    const int n = (t.n_sub + len - 1) / len;
    const int32_t first = (int32_t)out.items.size();
    if (n > 1) out.split_tiles.push_back(first);
    for (int k = 0; k < n; k++) out.items.push_back({t.req, t.tile, k * len, std::min(t.n_sub, (k + 1) * len), n, first, 0, 0});
  }
  return out;
}

PlanItems plan_items_chunked(const std::vector<PlanTile>& tiles, const int32_t* prefix_blocks, int chunk_blocks, int n_chunks) {
  PlanItems out;
  out.groups.assign((size_t)n_chunks + 1, {});
  const int sub_per_chunk = chunk_blocks / 2;
  for (const PlanTile& t : tiles) {
    const int full = prefix_blocks[t.req] / 2;                   // sub-tiles wholly inside the prefix
    const int32_t first = (int32_t)out.items.size();
    const int n = (full + sub_per_chunk - 1) / sub_per_chunk;    // pieces that follow the chunks
    const int cut_end = std::min(full, n * sub_per_chunk);
    const int total = n + (cut_end < t.n_sub ? 1 : 0);
    if (total > 1) out.split_tiles.push_back(first);
    for (int k = 0; k < n; k++) {
      out.groups[(size_t)std::min(k, n_chunks)].push_back((int32_t)out.items.size());
      out.items.push_back({t.req, t.tile, k * sub_per_chunk, std::min(full, (k + 1) * sub_per_chunk), total, first, 0, 0});
    }
    if (cut_end < t.n_sub) {
      out.groups[(size_t)n_chunks].push_back((int32_t)out.items.size());
      out.items.push_back({t.req, t.tile, cut_end, t.n_sub, total, first, 0, 0});
    }
  }
  return out;
}

}  // namespace calvo

extern "C" int calvo_attn_plan_items(int32_t n_q_heads, int32_t n_kv_heads, int32_t n_cus, const int32_t* prefix_blocks,
                                     const int32_t* suffix_lens, int32_t n_reqs, int32_t chunk_blocks, int32_t* items,
                                     int32_t capacity, int32_t* n_items) {
  using namespace calvo;
  if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || n_cus <= 0 || n_reqs < 0) return CALVO_EINVAL;
  if (n_reqs > 0 && (!prefix_blocks || !suffix_lens)) return CALVO_EINVAL;
  if (chunk_blocks < 0 || (chunk_blocks & 1) || capacity < 0 || (capacity > 0 && !items) || !n_items) return CALVO_EINVAL;
  int max_blocks = 0;
  for (int r = 0; r < n_reqs; r++) {
    if (prefix_blocks[r] < 0 || suffix_lens[r] < 0) return CALVO_EINVAL;
    max_blocks = std::max(max_blocks, prefix_blocks[r]);
  }
  const int hw = attn_heads_per_wg(n_q_heads, n_kv_heads);
  const int variant = attn_mfma_choose(suffix_lens, n_reqs, hw);
  const std::vector<PlanTile> tiles = plan_tiles(prefix_blocks, suffix_lens, n_reqs, attn_mfma_tile_tokens(variant, hw));
  const PlanParams p{n_q_heads / hw, n_cus * (8 / attn_mfma_waves_per_wg(variant)), 48, 30, 0};
  PlanItems pi;
  if (chunk_blocks > 0) {
    pi = plan_items_chunked(tiles, prefix_blocks, chunk_blocks, (max_blocks + chunk_blocks - 1) / chunk_blocks);
  } else {
    pi = plan_items(tiles, plan_pieces(tiles, p), p);
  }
  *n_items = (int32_t)pi.items.size();
  if ((int64_t)pi.items.size() > capacity) return CALVO_ENOMEM;
  std::vector<int32_t> launch(pi.items.size(), 0);
  for (size_t g = 0; g < pi.groups.size(); g++)
    for (int32_t i : pi.groups[g]) launch[(size_t)i] = (int32_t)g;
  for (size_t i = 0; i < pi.items.size(); i++) {
    const WorkItem& w = pi.items[i];
    int32_t* o = items + 6 * i;
    o[0] = w.req; o[1] = w.q_tile; o[2] = w.sub_begin; o[3] = w.sub_end; o[4] = w.n_splits; o[5] = launch[i];
  }
  return CALVO_OK;
}

extern "C" int calvo_attn_plan(int32_t n_q_heads, int32_t n_kv_heads, int32_t n_cus, const int32_t* prefix_blocks,
                               const int32_t* suffix_lens, int32_t n_reqs, int32_t* kernel, int32_t* tile_tokens,
                               int32_t* pieces, int32_t* n_workgroups) {
  using namespace calvo;
  if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || n_cus <= 0 || n_reqs < 0) return CALVO_EINVAL;
  if (n_reqs > 0 && (!prefix_blocks || !suffix_lens)) return CALVO_EINVAL;
  for (int r = 0; r < n_reqs; r++)
    if (prefix_blocks[r] < 0 || suffix_lens[r] < 0) return CALVO_EINVAL;
  const int hw = attn_heads_per_wg(n_q_heads, n_kv_heads);
  const int variant = attn_mfma_choose(suffix_lens, n_reqs, hw);
  const int tt = attn_mfma_tile_tokens(variant, hw);
  const std::vector<PlanTile> tiles = plan_tiles(prefix_blocks, suffix_lens, n_reqs, tt);
  PlanParams p{n_q_heads / hw, n_cus * (8 / attn_mfma_waves_per_wg(variant)), 48, 30, 0};
  const int want = plan_pieces(tiles, p);
  int64_t items = 0;
  for (const PlanTile& t : tiles) {
    const int len = plan_piece_len(t.n_sub, want, p);
    items += (t.n_sub + len - 1) / len;
  }
  if (kernel) *kernel = variant;
  if (tile_tokens) *tile_tokens = tt;
  if (pieces) *pieces = want;
  if (n_workgroups) *n_workgroups = (int32_t)(items * p.n_head_groups);
  return CALVO_OK;
}
