// The 8-wave shape of the pipelined attention kernel (attn_pipeline.h): workgroup = 4 query heads
// of one KV group x 2 token tiles of 32, one workgroup per CU, K and V rings of eight 8 KiB slots.
// Also the kernel that merges the partial results of tiles whose context was cut into pieces.
#include "attn_pipeline.h"

namespace calvo {
namespace pipe {

using namespace attn;
using Cfg = PipeCfg<8, 8>;

// 240 of the 256 registers a wave may have at two waves per SIMD (the attribute counts half of
// the unified VGPR+AGPR file on this target): the remaining 32 per SIMD lane let a wave of the
// ingest scatter kernel become resident next to the attention waves, so the loading stage keeps
// moving while attention occupies every CU.
__global__ void __launch_bounds__(512, 2) __attribute__((amdgpu_num_vgpr(120))) attn_pipe_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  attn_pipeline<Cfg>(p, smem);
}

// Combines the pieces of split tiles: for every row and head, with m = max_c m_c,
//     O = sum_c 2^(m_c - m) O_c  /  sum_c 2^(m_c - m) l_c
// (the pieces' O_c, l_c are sums of weights 2^(x - m_c), x the exponent of a score).  One workgroup of
// 256 threads per (split tile, head group, wave slot of the attention workgroup): thread = (row 0..31,
// 16-float chunk 0..7).  A piece in which a row saw no key has l_c = 0 and m_c = -inf and drops out.
__global__ void __launch_bounds__(256) merge_splits_kernel(AttnParams p, const int32_t* split_tiles) {
  const int NW = p.waves_per_wg;
  const int HW = p.heads_per_wg, NHG = p.n_q_heads / HW, TPW = NW / HW;
  const int wave_slot = blockIdx.x % NW;
  const int hg = (blockIdx.x / NW) % NHG;
  const int first = split_tiles[blockIdx.x / (NW * NHG)];
  const WorkItem wi = p.items[first];
  const ReqDesc rd = p.reqs[wi.req];
  const int row = threadIdx.x >> 3, chunk = threadIdx.x & 7;
  const int tokq = wi.q_tile * 32 * TPW + (wave_slot / HW) * 32 + row;
  if (tokq >= rd.suffix_len) return;
  const int hq = hg * HW + wave_slot % HW;
  float m = -INFINITY;
  for (int c = 0; c < wi.n_splits; c++) {
    const int64_t slot = ((int64_t)(first + c) * NHG + hg) * NW + wave_slot;
    m = fmaxf(m, p.part_ml[(slot * 32 + row) * 2]);
  }
  float acc[16], l = 0.f;
#pragma unroll
  for (int i = 0; i < 16; i++) acc[i] = 0.f;
  for (int c = 0; c < wi.n_splits; c++) {
    const int64_t slot = ((int64_t)(first + c) * NHG + hg) * NW + wave_slot;
    const float mc = p.part_ml[(slot * 32 + row) * 2], lc = p.part_ml[(slot * 32 + row) * 2 + 1];
    if (!(lc > 0.f)) continue;
    const float wgt = __builtin_amdgcn_exp2f(mc - m);
    l += wgt * lc;
    const f32x4* po = (const f32x4*)(p.part_o + (slot * 32 + row) * kD + 16 * chunk);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const f32x4 v = po[i];
      acc[4 * i] += wgt * v[0]; acc[4 * i + 1] += wgt * v[1]; acc[4 * i + 2] += wgt * v[2]; acc[4 * i + 3] += wgt * v[3];
    }
  }
  const float inv = 1.f / l;
  unsigned short* out = (unsigned short*)p.out + ((int64_t)(rd.q_off + tokq) * p.n_q_heads + hq) * kD + 16 * chunk;
  u32x4 w0, w1;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    bf16x2 a, b;
    a[0] = (__bf16)(acc[2 * i] * inv);
    a[1] = (__bf16)(acc[2 * i + 1] * inv);
    b[0] = (__bf16)(acc[8 + 2 * i] * inv);
    b[1] = (__bf16)(acc[8 + 2 * i + 1] * inv);
    w0[i] = __builtin_bit_cast(unsigned int, a);
    w1[i] = __builtin_bit_cast(unsigned int, b);
  }
  *(u32x4*)out = w0;
  *(u32x4*)(out + 8) = w1;
}

}  // namespace pipe

int attn_pipe_tile_tokens(int heads_per_wg) { return 32 * (8 / heads_per_wg); }

hipError_t attn_pipe_prepare() {
  return hipFuncSetAttribute((const void*)pipe::attn_pipe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             pipe::Cfg::LDS_BYTES);
}

hipError_t launch_attn_pipe(const AttnParams& p, hipStream_t stream) {
  if (p.n_items <= 0) return hipSuccess;
  const unsigned grid = (unsigned)p.n_items * (unsigned)(p.n_q_heads / p.heads_per_wg);
  hipLaunchKernelGGL(pipe::attn_pipe_kernel, dim3(grid), dim3(512), pipe::Cfg::LDS_BYTES, stream, p);
  return hipGetLastError();
}

hipError_t launch_merge_splits(const AttnParams& p, const int32_t* split_tiles, int n_split_tiles, hipStream_t stream) {
  if (n_split_tiles <= 0) return hipSuccess;
  const unsigned grid = (unsigned)n_split_tiles * (unsigned)(p.n_q_heads / p.heads_per_wg) * (unsigned)p.waves_per_wg;
  hipLaunchKernelGGL(pipe::merge_splits_kernel, dim3(grid), dim3(256), 0, stream, p, split_tiles);
  return hipGetLastError();
}

}  // namespace calvo
