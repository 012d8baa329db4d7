// Byte-moving kernels of the L2->L1 loading stage (paper Section 3.1) and of the
// suffix KV write of prefill (Section 2.1).  gfx950 only.
//
// scatter_blocks: source blocks are consecutive (a host staging area read over
// PCIe, or a device staging buffer filled by the copy engine); block j goes to
// pool slot table[j].  The grid walks the source linearly in 16-byte units so the
// PCIe / HBM read stream is sequential; every lane keeps four loads in flight.
// A few workgroups saturate the host link, so the grid is kept small and the
// remaining compute units stay free for attention.
#include "calvo_internal.h"

namespace calvo {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Kept to a couple of dozen registers (32-bit chunk arithmetic, two loads in flight): its waves
// must fit into the 32 registers per SIMD lane that the attention kernel leaves free, otherwise
// the loading stage stalls whenever attention occupies every CU.
__global__ void __launch_bounds__(256)
scatter_blocks_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ pool_layer,
                      const int32_t* __restrict__ table, uint32_t n_chunks, uint32_t chunks_per_block) {
  const uint32_t stride = gridDim.x * 256u;
  uint32_t i = blockIdx.x * 256u + threadIdx.x;
  for (; i + stride < n_chunks; i += 2 * stride) {
    const uint32_t i1 = i + stride;
    const u32x4 v0 = __builtin_nontemporal_load(src + i);
    const u32x4 v1 = __builtin_nontemporal_load(src + i1);
    const uint32_t j0 = i / chunks_per_block, j1 = i1 / chunks_per_block;
    pool_layer[(uint64_t)(uint32_t)table[j0] * chunks_per_block + (i - j0 * chunks_per_block)] = v0;
    pool_layer[(uint64_t)(uint32_t)table[j1] * chunks_per_block + (i1 - j1 * chunks_per_block)] = v1;
  }
  if (i < n_chunks) {
    const uint32_t j = i / chunks_per_block;
    pool_layer[(uint64_t)(uint32_t)table[j] * chunks_per_block + (i - j * chunks_per_block)] =
        __builtin_nontemporal_load(src + i);
  }
}

// One launch moves at most 2^31 16-byte chunks (32 GiB); larger requests are split.
hipError_t launch_scatter_blocks(const void* src, void* pool_layer, const int32_t* table, int64_t n_blocks,
                                 int32_t blk_bytes, int grid, hipStream_t stream) {
  if (n_blocks <= 0) return hipSuccess;
  const int64_t cpb = blk_bytes / 16;
  const int64_t max_blocks = ((int64_t)1 << 31) / cpb;
  for (int64_t b0 = 0; b0 < n_blocks; b0 += max_blocks) {
    const int64_t nb = n_blocks - b0 < max_blocks ? n_blocks - b0 : max_blocks;
    const int64_t n_chunks = nb * cpb;
    int64_t need = (n_chunks + 511) / 512;
    int g = grid > need ? (int)need : grid;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(scatter_blocks_kernel, dim3(g), dim3(256), 0, stream,
                       (const u32x4*)((const unsigned char*)src + b0 * blk_bytes), (u32x4*)pool_layer, table + b0,
                       (uint32_t)n_chunks, (uint32_t)cpb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Test hook: keeps a stream busy for about `us` microseconds (one wave that sleeps in short naps until
// the constant 100 MHz counter has advanced; the nap count is bounded, so the wave always exits).
__global__ void __launch_bounds__(64) delay_kernel(unsigned ticks, unsigned max_naps) {
  const unsigned long long t0 = wall_clock64();
  for (unsigned i = 0; i < max_naps && wall_clock64() - t0 < ticks; i++) __builtin_amdgcn_s_sleep(64);
}

hipError_t launch_delay(int us, hipStream_t stream) {
  if (us <= 0) return hipSuccess;
  if (us > 20000) us = 20000;
  // a nap of s_sleep 64 lasts at least 64 * 64 cycles, i.e. more than 1.5 us at 2.4 GHz: the cap is never the limit
  hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, stream, (unsigned)us * 100u, (unsigned)us + 16u);
  return hipGetLastError();
}

// Suffix token i of request r sits at absolute position P_r + i: slot table_r[pos / 16],
// row pos % 16 of the K half and of the V half.  One lane per 16-byte chunk of a row.
__global__ void __launch_bounds__(256) suffix_append_kernel(AppendParams p) {
  const int64_t n = (int64_t)p.total_tokens * p.row_chunks;
  const int64_t half_chunks = (int64_t)kBlockTokens * p.row_chunks;   // one K (or V) half of a block
  const u32x4* ks = (const u32x4*)p.k_suffix;
  const u32x4* vs = (const u32x4*)p.v_suffix;
  u32x4* pool = (u32x4*)p.pool_layer;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int32_t tok = (int32_t)(i / p.row_chunks);
    const int32_t c = (int32_t)(i - (int64_t)tok * p.row_chunks);
    int r = 0;
    while (r + 1 < p.n_reqs && tok >= p.reqs[r + 1].q_off) r++;
    const ReqDesc rd = p.reqs[r];
    const int32_t pos = rd.prefix_len + (tok - rd.q_off);
    const int64_t slot = p.tables[rd.table_off + pos / kBlockTokens];
    const int64_t base = slot * 2 * half_chunks + (int64_t)(pos % kBlockTokens) * p.row_chunks + c;
    pool[base] = ks[i];
    pool[base + half_chunks] = vs[i];
  }
}

hipError_t launch_suffix_append(const AppendParams& p, hipStream_t stream) {
  const int64_t n = (int64_t)p.total_tokens * p.row_chunks;
  if (n <= 0) return hipSuccess;
  int grid = (int)((n + 255) / 256);
  if (grid > 2048) grid = 2048;
  hipLaunchKernelGGL(suffix_append_kernel, dim3(grid), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace calvo
