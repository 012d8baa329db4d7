// The 4-wave shape of the pipelined attention kernel (attn_pipeline.h): workgroup = 4 query heads
// of one KV group x one token tile of 32, two workgroups per CU (64 KiB of LDS each: K and V rings
// of four 8 KiB slots), so the two waves of a SIMD belong to different workgroups.  Tiles of 32 query tokens instead of 64: with the short queries of the paper's
// Table 1 (28 / 61 / 209 tokens) half of a 64-token tile's waves would idle.
#include "attn_pipeline.h"

namespace calvo {
namespace duo {

using namespace attn;
using Cfg = PipeCfg<4, 4>;

__global__ void __launch_bounds__(256, 2) __attribute__((amdgpu_num_vgpr(120))) attn_duo_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  attn_pipeline<Cfg>(p, smem);
}

}  // namespace duo

int attn_duo_tile_tokens(int heads_per_wg) { return 32 * (4 / heads_per_wg); }

hipError_t attn_duo_prepare() {
  return hipFuncSetAttribute((const void*)duo::attn_duo_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             duo::Cfg::LDS_BYTES);
}

hipError_t launch_attn_duo(const AttnParams& p, hipStream_t stream) {
  if (p.n_items <= 0) return hipSuccess;
  const unsigned grid = (unsigned)p.n_items * (unsigned)(p.n_q_heads / p.heads_per_wg);
  hipLaunchKernelGGL(duo::attn_duo_kernel, dim3(grid), dim3(256), duo::Cfg::LDS_BYTES, stream, p);
  return hipGetLastError();
}

}  // namespace calvo
