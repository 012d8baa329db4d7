// Planning of the loading stage's transfers (paper Section 3.1, L2 -> L1): every transfer boundary
// costs PCIe time, so blocks that follow each other in host memory travel together - across the
// requests of a batch, and across consecutive small layers.
#include "ingest_plan.h"

#include <algorithm>

#include "../../include/calvo.h"

namespace calvo {

std::vector<IngestRun> ingest_layer_runs(const IngestSrc* reqs, int n_reqs, int layer, size_t blk_bytes) {
  std::vector<IngestRun> runs;
  const int64_t bb = (int64_t)blk_bytes;
  for (int r = 0; r < n_reqs;) {
    if (reqs[r].nblk == reqs[r].first) { r++; continue; }
    int64_t j1 = reqs[r].nblk;
    int r2 = r + 1;
    for (; r2 < n_reqs; r2++) {
      const IngestSrc &a = reqs[r], &b = reqs[r2];
      if (b.nblk == b.first) continue;
      const uintptr_t end = a.base + (uintptr_t)((int64_t)layer * a.layer_stride + j1 * bb);
      const uintptr_t beg = b.base + (uintptr_t)((int64_t)layer * b.layer_stride + b.first * bb);
      if (end != beg || a.tab_off + j1 != b.tab_off + b.first) break;
      j1 += b.nblk - b.first;                       // request r's block numbering continues through b
    }
    const int64_t j0 = reqs[r].first;
    runs.push_back({r, j0, j1, reqs[r].base + (uintptr_t)((int64_t)layer * reqs[r].layer_stride + j0 * bb)});
    r = r2;
  }
  return runs;
}

int ingest_group_layers(const IngestSrc* reqs, int n_reqs, int layer, int layer_end, const int32_t* chunk_blocks,
                        int layer_begin, size_t blk_bytes, int64_t staging_blocks, size_t merge_bytes, int group_index) {
  auto chunk_of = [&](int l) { return chunk_blocks ? chunk_blocks[l - layer_begin] : 0; };
  if (chunk_of(layer) != 0 || staging_blocks <= 0) return 1;
  const std::vector<IngestRun> runs = ingest_layer_runs(reqs, n_reqs, layer, blk_bytes);
  if (runs.size() != 1) return 1;
  const int64_t nb = runs[0].j1 - runs[0].j0;
  const int64_t fit = std::min<int64_t>(staging_blocks / nb, (int64_t)(merge_bytes / ((size_t)nb * blk_bytes)));
  const int64_t kmax = std::min<int64_t>({fit, (int64_t)1 << std::min(std::max(group_index, 0), 16),
                                          ((int64_t)layer_end - layer + 2) / 3});
  int k = 1;
  while (k < kmax && chunk_of(layer + k) == 0) {
    const std::vector<IngestRun> next = ingest_layer_runs(reqs, n_reqs, layer + k, blk_bytes);
    if (next.size() != 1 || next[0].r != runs[0].r || next[0].j0 != runs[0].j0 || next[0].j1 != runs[0].j1 ||
        next[0].beg != runs[0].beg + (uintptr_t)((int64_t)k * nb * (int64_t)blk_bytes))
      break;
    k++;
  }
  return k;
}

}  // namespace calvo

extern "C" int calvo_ingest_plan(const calvo_request* reqs, int32_t n_reqs, int32_t layer_begin, int32_t layer_end,
                                 int64_t block_bytes, int64_t staging_blocks, int64_t merge_bytes,
                                 const int32_t* chunk_blocks, int32_t* transfer_of_layer, int32_t* runs_of_layer) {
  using namespace calvo;
  if (n_reqs < 0 || (n_reqs > 0 && !reqs) || layer_begin < 0 || layer_end < layer_begin || block_bytes <= 0 ||
      staging_blocks < 0 || merge_bytes < 0)
    return CALVO_EINVAL;
  std::vector<IngestSrc> src((size_t)n_reqs);
  int64_t n_tab = 0;
  for (int r = 0; r < n_reqs; r++) {
    const calvo_request& q = reqs[r];
    if (q.n_prefix_blocks < 0 || q.first_ingest_block < 0 || q.first_ingest_block > q.n_prefix_blocks) return CALVO_EINVAL;
    src[(size_t)r] = {(uintptr_t)q.host_kv, q.host_layer_stride, q.first_ingest_block, q.n_prefix_blocks,
                      n_tab - q.first_ingest_block};
    n_tab += q.n_prefix_blocks - q.first_ingest_block;
  }
  for (int l = layer_begin; l < layer_end; l++)
    if (chunk_blocks && (chunk_blocks[l - layer_begin] < 0 || (chunk_blocks[l - layer_begin] & 1))) return CALVO_EINVAL;
  int group = 0;
  for (int l = layer_begin; l < layer_end;) {
    const bool chunked = chunk_blocks && chunk_blocks[l - layer_begin] > 0;
    const int k = chunked ? 1 : ingest_group_layers(src.data(), n_reqs, l, layer_end, chunk_blocks, layer_begin,
                                                    (size_t)block_bytes, staging_blocks, (size_t)merge_bytes, group);
    const int32_t n_runs = (int32_t)ingest_layer_runs(src.data(), n_reqs, l, (size_t)block_bytes).size();
    for (int i = 0; i < k; i++) {
      if (transfer_of_layer) transfer_of_layer[l + i - layer_begin] = chunked ? -1 : group;
      if (runs_of_layer) runs_of_layer[l + i - layer_begin] = n_runs;
    }
    if (!chunked) group++;
    l += k;
  }
  return CALVO_OK;
}
