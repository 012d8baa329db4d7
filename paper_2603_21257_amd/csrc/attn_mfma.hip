// Paged causal GQA prefill attention for gfx950 (CDNA4): bf16 storage, head_dim 128,
// bf16 MFMA (v_mfma_f32_32x32x16_bf16) for both contractions, fp32 online softmax.
//
// Work decomposition
//   workgroup = NW wavefronts = one tile of suffix tokens x up to 4 query heads that share
//   one KV head; the 64-key K/V tile it streams is staged once in LDS and used by all waves.
//   Each wave owns NT*32 query rows (one head) and keeps their Q, O and softmax state in
//   registers for the whole key loop.  Default: NW=4, NT=1, two workgroups per CU, so each
//   SIMD holds two waves of different workgroups and one wave's softmax (vector ALU) runs
//   under the other's MFMAs.
//
// Transposed formulation (so that every softmax statistic is lane-local):
//   S^T[key][query] = K[key][:] . Q[query][:]      A = K tile (LDS, d-contiguous), B = Q (registers)
//   O^T[d][query]  += V^T[d][key] * P^T[key][query] A = V^T, B = P^T
//   In the 32x32 accumulator layout a lane holds one query column and 16 keys, so row max /
//   row sum are reductions inside a lane plus one exchange with lane^32, the O rescale is a
//   per-lane scalar, and P^T is already the B operand of the second MFMA: the MFMA k index is
//   only a summation index, so the 8 keys a lane holds after QK^T (key = 8*(r/4)+4*(lane/32)+r%4)
//   are used as they are, and the V^T operand is fetched for exactly those keys.
//   V sits in LDS token-major (as in the pool); the d-major operand is produced by the
//   LDS transpose read ds_read_b64_tr_b16: inside a 16-lane group, lane i receives element
//   i%4 of the four 8-byte rows addressed by lanes i/4, i/4+4, i/4+8, i/4+12.
//
// LDS: two buffers of (K 64 rows x 272 B, V 64 rows x 320 B).  The row padding makes the
// operand reads conflict-free (K: 16 consecutive rows, same 16-byte column -> 16 distinct bank
// quads; V: 4 rows x 64 bytes -> 4 distinct bank sixteenths) while every operand address is
// one lane-constant base plus a compile-time offset, so the key loop spends no vector ALU
// instruction on addressing.
#include <stdlib.h>

#include "calvo_internal.h"

namespace calvo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kD = 128;                       // head_dim
constexpr int kKT = 64;                       // keys per LDS tile
constexpr int kKRow = 272;                    // padded K row stride in LDS (bytes)
constexpr int kVRow = 320;                    // padded V row stride in LDS (bytes)
constexpr int kKTileB = kKT * kKRow;          // 17408
constexpr int kVTileB = kKT * kVRow;          // 20480
constexpr int kBufB = kKTileB + kVTileB;      // one stage
constexpr int kLdsBytes = 2 * kBufB;          // 75776: two workgroups fit in a CU's 160 KiB

// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32 lanes
// of its second.  Fed two copies of one value it leaves (lower half, lower half) in the first and
// (upper half, upper half) in the second, so combining both gives every lane the reduction over
// lane and lane^32.  Written as inline asm: the compiler builtin returns its first result twice.
__device__ inline void half_swap(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ inline float half_swap_max(float v) {
  float a = v, b = v;
  half_swap(a, b);
  return fmaxf(a, b);
}
__device__ inline float half_swap_sum(float v) {
  float a = v, b = v;
  half_swap(a, b);
  return a + b;
}

// NT: 32-row query tiles per wave; NW: waves per workgroup (all share the staged K/V tile).
template <int NT, int NW>
__global__ void __launch_bounds__(64 * NW, (NT > 1) ? 1 : 2) attn_mfma_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31;       // query column inside a 32-wide tile
  const int lh = lane >> 5;       // which half of the k index this lane feeds

  // ---- which tile of which request, which head group (wave-uniform)
  const int HW = p.heads_per_wg;
  const int TPW = NW / HW;                        // token sub-tiles per workgroup
  const int NHG = p.n_q_heads / HW;
  int it, hg;
  {
    const int bid = blockIdx.x;
    if ((NHG & 7) == 0) {                         // keep one KV head's workgroups on one XCD
      const int per = NHG >> 3, rest = bid >> 3;
      hg = (bid & 7) * per + rest % per;
      it = rest / per;
    } else {
      hg = bid % NHG;
      it = bid / NHG;
    }
  }
  const WorkItem wi = p.items[it];
  const ReqDesc rd = p.reqs[wi.req];
  const int P = rd.prefix_len, S = rd.suffix_len;
  const int TQ = 32 * NT * TPW;
  const int q_base = wi.q_tile * TQ;
  const int hq = hg * HW + wave % HW;
  const int kv = hq / (p.n_q_heads / p.n_kv_heads);
  const int wq0 = q_base + (wave / HW) * 32 * NT;            // first suffix token of this wave
  const bool wave_active = wq0 < S;
  const int pq_min = P + wq0;
  const int pq_max = P + min(wq0 + 32 * NT, S) - 1;
  const int ctx_len = P + S;
  const int n_keys = P + min(q_base + TQ, S);
  const int n_tiles = (n_keys + kKT - 1) / kKT;
  const int last_blk = (ctx_len + kBlockTokens - 1) / kBlockTokens - 1;
  const int32_t* table = p.tables + rd.table_off;
  const int Hkv = p.n_kv_heads, Hq = p.n_q_heads;
  const float c2 = p.scale * 1.4426950408889634f;            // scores are exponentiated in base 2

  // ---- Q as the B operand of QK^T: lane (query ln, half lh) holds Q[query][16ks + 8lh .. +8]
  bf16x8 qB[NT][8];
  {
    const unsigned short* q = (const unsigned short*)p.q;
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
      const int tokq = wq0 + nt * 32 + ln;
      const bool ok = tokq < S;
      const unsigned short* row = q + ((int64_t)(rd.q_off + (ok ? tokq : 0)) * Hq + hq) * kD + 8 * lh;
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (ok) v = *(const u32x4*)(row + 16 * ks);
        qB[nt][ks] = __builtin_bit_cast(bf16x8, v);
      }
    }
  }

  f32x16 o[4][NT];
#pragma unroll
  for (int dt = 0; dt < 4; dt++)
#pragma unroll
    for (int nt = 0; nt < NT; nt++)
#pragma unroll
      for (int r = 0; r < 16; r++) o[dt][nt][r] = 0.f;
  float m_run[NT], l_run[NT];
#pragma unroll
  for (int nt = 0; nt < NT; nt++) { m_run[nt] = -INFINITY; l_run[nt] = 0.f; }

  // ---- global -> register -> LDS staging of one 64-key tile.  A wave stages 4 token rows x 16
  // chunks per pass; pass i covers tile row i*4*NW + tid/16.  The block (slot) of a pass is
  // wave-uniform, so the load address is a scalar base plus one loop-invariant lane offset.
  const unsigned char* pool = (const unsigned char*)p.pool_layer;
  const int64_t half_b = (int64_t)kBlockTokens * Hkv * kD * 2;        // bytes of the K half of a block
  constexpr int kPass = 16 / NW;
  const int ld_row = tid >> 4;                   // 0 .. 4*NW-1
  const int ld_chunk = tid & 15;
  const unsigned ld_voff = (unsigned)((ld_row & 15) * Hkv * kD * 2 + kv * kD * 2 + ld_chunk * 16);
  const int st_k = ld_row * kKRow + ld_chunk * 16;
  const int st_v = kKTileB + ld_row * kVRow + ld_chunk * 16;
  u32x4 kreg[kPass], vreg[kPass];

  auto load_tile = [&](int tile) {
#pragma unroll
    for (int i = 0; i < kPass; i++) {
      const int blk = min(tile * 4 + ((i * 4 * NW + ld_row) >> 4), last_blk);
      const int64_t slot = __builtin_amdgcn_readfirstlane(table[blk]);
      const unsigned char* sbase = pool + slot * 2 * half_b;
      kreg[i] = *(const u32x4*)(sbase + ld_voff);
      vreg[i] = *(const u32x4*)(sbase + half_b + ld_voff);
    }
    if (tile * kKT + kKT > ctx_len) {   // tokens past the context are undefined: keep them out of PV (0 * NaN)
#pragma unroll
      for (int i = 0; i < kPass; i++)
        if (tile * kKT + i * 4 * NW + ld_row >= ctx_len) vreg[i] = (u32x4){0u, 0u, 0u, 0u};
    }
  };
  auto store_tile = [&](int buf) {
    unsigned char* b = smem + buf * kBufB;
#pragma unroll
    for (int i = 0; i < kPass; i++) {
      *(u32x4*)(b + st_k + i * 4 * NW * kKRow) = kreg[i];
      *(u32x4*)(b + st_v + i * 4 * NW * kVRow) = vreg[i];
    }
  };

  // ---- lane-constant parts of the operand addresses
  // K operand: lane (key ln, half lh) reads 16 bytes at row ln, byte column 32*ks + 16*lh.
  const int k_rd = ln * kKRow + lh * 16;
  // V^T operand: 16-lane group g16 covers d = 16*(g16&1) .. +16 of a 32-wide d tile and 4 tokens
  // starting at 4*(g16>>1); source lane s16 points at token s16/4, d offset 4*(s16%4).
  const int g16 = lane >> 4, s16 = lane & 15;
  const int v_rd = kKTileB + (4 * (g16 >> 1) + (s16 >> 2)) * kVRow + (16 * (g16 & 1) + 4 * (s16 & 3)) * 2;

  bf16x2 ones;
  ones[0] = (__bf16)1.0f;
  ones[1] = (__bf16)1.0f;

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int tile = 0; tile < n_tiles; tile++) {
    const int buf = tile & 1;
    if (tile + 1 < n_tiles) load_tile(tile + 1);
    const unsigned char* kb = smem + buf * kBufB + k_rd;
    const unsigned char* vb = smem + buf * kBufB + v_rd;

#pragma unroll
    for (int sb = 0; sb < 2; sb++) {
      const int k0 = tile * kKT + sb * 32;
      if (wave_active && k0 <= pq_max) {
        // ---- S^T = K Q^T
        bf16x8 ka[8];
#pragma unroll
        for (int ks = 0; ks < 8; ks++) ka[ks] = *(const bf16x8*)(kb + sb * 32 * kKRow + ks * 32);
        f32x16 s[NT];
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
          f32x16 z;
#pragma unroll
          for (int r = 0; r < 16; r++) z[r] = 0.f;
          s[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0], qB[nt][0], z, 0, 0, 0);
        }
#pragma unroll
        for (int ks = 1; ks < 8; ks++) {
#pragma unroll
          for (int nt = 0; nt < NT; nt++)
            s[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qB[nt][ks], s[nt], 0, 0, 0);
        }
        // ---- causal mask (only near the diagonal)
        if (k0 + 31 > pq_min) {
#pragma unroll
          for (int nt = 0; nt < NT; nt++) {
            const int pq = pq_min + nt * 32 + ln;
#pragma unroll
            for (int r = 0; r < 16; r++) {
              const int kt = k0 + 8 * (r >> 2) + 4 * lh + (r & 3);
              if (kt > pq) s[nt][r] = -INFINITY;
            }
          }
        }
        // ---- online softmax, lane-local per query column
        bf16x8 pb[NT][2];
        float alpha[NT];
        bool changed = false;
#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
          float mx = fmaxf(s[nt][0], s[nt][1]);
#pragma unroll
          for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[nt][r]), s[nt][r + 1]);
          mx = half_swap_max(mx);
          const float m_new = fmaxf(m_run[nt], mx);
          alpha[nt] = __builtin_amdgcn_exp2f((m_run[nt] - m_new) * c2);
          changed |= (m_new != m_run[nt]);
          m_run[nt] = m_new;
          const float mc = m_new * c2;
          // weights are rounded to bf16 once; the row sum adds the rounded values (v_dot2 against
          // (1,1)), so numerator and denominator of the softmax use the same numbers
          float ps = 0.f;
          bf16x2 pk[8];
#pragma unroll
          for (int e = 0; e < 8; e++) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nt][2 * e], c2, -mc));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nt][2 * e + 1], c2, -mc));
            pk[e][0] = (__bf16)p0;
            pk[e][1] = (__bf16)p1;
            ps = __builtin_amdgcn_fdot2_f32_bf16(pk[e], ones, ps, false);
          }
          l_run[nt] = l_run[nt] * alpha[nt] + ps;
#pragma unroll
          for (int j = 0; j < 2; j++) {
            u32x4 w = {__builtin_bit_cast(unsigned, pk[4 * j]), __builtin_bit_cast(unsigned, pk[4 * j + 1]),
                       __builtin_bit_cast(unsigned, pk[4 * j + 2]), __builtin_bit_cast(unsigned, pk[4 * j + 3])};
            pb[nt][j] = __builtin_bit_cast(bf16x8, w);
          }
        }
        if (__builtin_amdgcn_ballot_w64(changed) != 0) {
#pragma unroll
          for (int dt = 0; dt < 4; dt++)
#pragma unroll
            for (int nt = 0; nt < NT; nt++)
#pragma unroll
              for (int r = 0; r < 16; r++) o[dt][nt][r] *= alpha[nt];
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int j = 0; j < 2; j++) {
#pragma unroll
          for (int dt = 0; dt < 4; dt++) {
            const unsigned char* va = vb + (sb * 32 + 16 * j) * kVRow + dt * 64;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(va));
            const s16x4 hi =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(va + 8 * kVRow));
            const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8 a = __builtin_bit_cast(bf16x8, both);
#pragma unroll
            for (int nt = 0; nt < NT; nt++)
              o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[nt][j], o[dt][nt], 0, 0, 0);
          }
        }
      }
    }

    if (tile + 1 < n_tiles) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- normalise and write O[token][head][d]; lane holds d = 32dt + 8(r/4) + 4lh + r%4
  if (wave_active) {
    unsigned short* out = (unsigned short*)p.out;
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
      const float lt = half_swap_sum(l_run[nt]);
      const float inv = 1.f / lt;
      const int tokq = wq0 + nt * 32 + ln;
      if (tokq < S) {
        unsigned short* row = out + ((int64_t)(rd.q_off + tokq) * Hq + hq) * kD + 4 * lh;
#pragma unroll
        for (int dt = 0; dt < 4; dt++)
#pragma unroll
          for (int rq = 0; rq < 4; rq++) {
            bf16x2 a, b;
            a[0] = (__bf16)(o[dt][nt][4 * rq + 0] * inv);
            a[1] = (__bf16)(o[dt][nt][4 * rq + 1] * inv);
            b[0] = (__bf16)(o[dt][nt][4 * rq + 2] * inv);
            b[1] = (__bf16)(o[dt][nt][4 * rq + 3] * inv);
            u32x2 w = {__builtin_bit_cast(unsigned int, a), __builtin_bit_cast(unsigned int, b)};
            *(u32x2*)(row + 32 * dt + 8 * rq) = w;
          }
      }
    }
  }
}

// Kernel choice.  Two pipelined kernels serve by default: variant 3, one 8-wave workgroup per CU
// with 64-token tiles (attn_pipe.hip), and variant 4, two independent 4-wave workgroups per CU with
// 32-token tiles (attn_duo.hip).  On long suffixes they run within 2 % of each other (the chip is
// power limited: what one gains in cycles it loses in clock) and variant 3 has half the K/V traffic
// into LDS; on short suffixes - 28 or 61 query tokens leave half of a 64-token tile empty -
// variant 4 wastes no waves.  attn_mfma_choose picks per call.  The environment variable
// CALVO_ATTN_VARIANT forces one: 3, 4, or the unpipelined kernel of this file for comparison runs
// (0 = 4 waves x 32 rows, two workgroups per CU; 1 = 4 waves x 64 rows, one wave per SIMD; 2 = 8
// waves x 32 rows).
static int forced_variant() {
  const char* e = getenv("CALVO_ATTN_VARIANT");      // read per call: tests switch it inside one process
  return (e && e[0] >= '0' && e[0] <= '4') ? e[0] - '0' : -1;
}

int attn_mfma_choose(const int32_t* suffix_lens, int n_reqs, int heads_per_wg) {
  const int f = forced_variant();
  if (f >= 0) return f;
  // query rows the tiles of each kernel would hold, empty ones included
  const int t3 = attn_pipe_tile_tokens(heads_per_wg), t4 = attn_duo_tile_tokens(heads_per_wg);
  int64_t rows3 = 0, rows4 = 0;
  for (int r = 0; r < n_reqs; r++) {
    rows3 += (int64_t)((suffix_lens[r] + t3 - 1) / t3) * t3;
    rows4 += (int64_t)((suffix_lens[r] + t4 - 1) / t4) * t4;
  }
  return rows3 * 9 > rows4 * 10 ? 4 : 3;       // the larger tiles would carry over 10 % more rows
}

bool attn_mfma_splits_context(int variant) { return variant >= 3; }

int attn_mfma_waves_per_wg(int variant) { return (variant == 3 || variant == 2) ? 8 : 4; }

int attn_mfma_tile_tokens(int variant, int heads_per_wg) {
  const int v = variant;
  if (v == 4) return attn_duo_tile_tokens(heads_per_wg);
  if (v == 3) return attn_pipe_tile_tokens(heads_per_wg);
  return v == 1 ? 64 * (4 / heads_per_wg) : v == 2 ? 32 * (8 / heads_per_wg) : 32 * (4 / heads_per_wg);
}

template <int NT, int NW>
static hipError_t launch_variant(const AttnParams& p, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_mfma_kernel<NT, NW>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const unsigned grid = (unsigned)p.n_items * (unsigned)(p.n_q_heads / p.heads_per_wg);
  hipLaunchKernelGGL((attn_mfma_kernel<NT, NW>), dim3(grid), dim3(64 * NW), kLdsBytes, stream, p);
  return hipGetLastError();
}

hipError_t launch_attn_mfma(int variant, const AttnParams& p, hipStream_t stream) {
  if (p.n_items <= 0) return hipSuccess;
  const int v = variant;
  if (v == 4) return launch_attn_duo(p, stream);
  if (v == 3) return launch_attn_pipe(p, stream);
  return v == 1 ? launch_variant<2, 4>(p, stream) : v == 2 ? launch_variant<1, 8>(p, stream)
                                                          : launch_variant<1, 4>(p, stream);
}

}  // namespace calvo
