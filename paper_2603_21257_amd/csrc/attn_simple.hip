// Generic paged causal GQA prefill attention: any head_dim <= 256 (multiple of 8),
// fp32 or bf16 storage, fp32 arithmetic on the vector ALUs.  One wavefront per
// (suffix token, query head).  This is the path for fp32 pools and for shapes the
// MFMA kernel does not cover; it is written for clarity, not speed.
//
// Per 64-key chunk: lane t scores key k0+t (dot product over D against the query
// held in LDS), the wave reduces max and sum for the online softmax, then the
// chunk's weights are broadcast one key at a time while lanes own output dims.
#include "calvo_internal.h"
#include "../../include/calvo.h"

namespace calvo {

__device__ inline float load_elem(const float* p) { return *p; }
__device__ inline float load_elem(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
__device__ inline void store_elem(float* p, float v) { *p = v; }
__device__ inline void store_elem(uint16_t* p, float v) {
  // round to nearest even; the result of a convex combination of finite values is finite
  uint32_t u = __float_as_uint(v);
  u += 0x7FFFu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <typename T>
__global__ void __launch_bounds__(64) attn_simple_kernel(AttnParams p, int total_tokens) {
  __shared__ float q_s[256];
  const int lane = threadIdx.x;
  const int tok = blockIdx.x / p.n_q_heads;
  const int h = blockIdx.x - tok * p.n_q_heads;
  if (tok >= total_tokens) return;
  int r = 0;
  while (r + 1 < p.n_items && tok >= p.reqs[r + 1].q_off) r++;   // n_items carries n_reqs here
  const ReqDesc rd = p.reqs[r];
  const int D = p.head_dim, Hkv = p.n_kv_heads;
  const int g = h / (p.n_q_heads / Hkv);
  const int pos = rd.prefix_len + (tok - rd.q_off);               // sees keys 0..pos
  const T* q = (const T*)p.q + ((int64_t)tok * p.n_q_heads + h) * D;
  for (int d = lane; d < D; d += 64) q_s[d] = load_elem(q + d);
  __syncthreads();
  const T* pool = (const T*)p.pool_layer;
  const int64_t half = (int64_t)kBlockTokens * Hkv * D;           // elements in the K half of a block
  const int32_t* table = p.tables + rd.table_off;

  float m = -INFINITY, l = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 <= pos; k0 += 64) {
    const int t = k0 + lane;
    float s = -INFINITY;
    int64_t row = 0;
    if (t <= pos) {
      row = (int64_t)table[t / kBlockTokens] * 2 * half + (int64_t)(t % kBlockTokens) * Hkv * D + (int64_t)g * D;
      const T* kr = pool + row;
      float dot = 0.f;
      for (int d = 0; d < D; d++) dot = fmaf(q_s[d], load_elem(kr + d), dot);
      s = dot * p.scale;
    }
    const float m_new = fmaxf(m, wave_max(s));
    const float w = (t <= pos) ? __expf(s - m_new) : 0.f;
    const float alpha = __expf(m - m_new);                        // exp(-inf) = 0 on the first chunk
    l = l * alpha + wave_sum(w);
    m = m_new;
#pragma unroll
    for (int i = 0; i < 4; i++) acc[i] *= alpha;
    const int nk = min(64, pos + 1 - k0);
    for (int j = 0; j < nk; j++) {
      const float wj = __shfl(w, j);
      const int64_t rj = __shfl(row, j);
      const T* vr = pool + rj + half;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int d = lane + 64 * i;
        if (d < D) acc[i] = fmaf(wj, load_elem(vr + d), acc[i]);
      }
    }
  }
  T* o = (T*)p.out + ((int64_t)tok * p.n_q_heads + h) * D;
  const float inv = 1.f / l;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int d = lane + 64 * i;
    if (d < D) store_elem(o + d, acc[i] * inv);
  }
}

hipError_t launch_attn_simple(const AttnParams& p, int dtype, int total_tokens, hipStream_t stream) {
  if (total_tokens <= 0) return hipSuccess;
  const unsigned grid = (unsigned)total_tokens * (unsigned)p.n_q_heads;
  if (dtype == CALVO_F32)
    hipLaunchKernelGGL(attn_simple_kernel<float>, dim3(grid), dim3(64), 0, stream, p, total_tokens);
  else
    hipLaunchKernelGGL(attn_simple_kernel<uint16_t>, dim3(grid), dim3(64), 0, stream, p, total_tokens);
  return hipGetLastError();
}

}  // namespace calvo
