// Host-side planning of the L2 -> L1 loading stage: which blocks of a layer cross PCIe as one
// transfer, and which consecutive layers share a transfer.  Addresses are only compared and added,
// never dereferenced; no device types here.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace calvo {

struct IngestSrc {          // one request
  uintptr_t base;           // address of its host block 0 of layer 0
  int64_t layer_stride;     // bytes between layers
  int64_t first, nblk;      // blocks [first, nblk) are loaded
  int64_t tab_off;          // index of its block 0 in the device-side table of loaded blocks
};

// Blocks [j0, j1) in request r's numbering, continued through the requests that follow it: their
// host blocks and their table entries are consecutive, so one transfer and one scatter serve them.
struct IngestRun {
  int r;
  int64_t j0, j1;
  uintptr_t beg;            // host address of block j0 of this layer
};

std::vector<IngestRun> ingest_layer_runs(const IngestSrc* reqs, int n_reqs, int layer, size_t blk_bytes);

// How many consecutive layers, starting at `layer`, travel as one transfer (1 = this layer alone).
// More than one only if the layer is a single run that fits the staging buffer several times, the
// following layers are the same run right behind it in host memory and are loaded as a whole
// (chunk_of(l) == 0), and the bytes stay within merge_bytes.  The size is at most 2^group_index
// (ramp-up: the first layer arrives at once) and at most a third of the layers still to come,
// rounded up (ramp-down: the attention of a group's layers can only start when the whole group is
// in and must not pile up behind the last transfer).
int ingest_group_layers(const IngestSrc* reqs, int n_reqs, int layer, int layer_end, const int32_t* chunk_blocks,
                        int layer_begin, size_t blk_bytes, int64_t staging_blocks, size_t merge_bytes, int group_index);

}  // namespace calvo
