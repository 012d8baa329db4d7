// Paged causal GQA prefill attention for gfx950 (CDNA4), two independent workgroups per CU:
// bf16 storage, head_dim 128, v_mfma_f32_32x32x16_bf16 for both contractions, fp32 online
// softmax, the transposed formulation and the software pipeline of attn_pipe.hip (S^T = K Q^T,
// O^T += V^T P^T; step t runs QK(t+1), softmax(t), PV(t-1); K and V go from the pool straight
// into LDS rings with global_load_lds_dwordx4; lazily raised softmax reference).
//
// What differs from attn_pipe.hip is who shares a SIMD.  There, the two waves of a SIMD belong
// to one workgroup and are held in opposite phases (one on the matrix pipe, one on the vector
// ALU) by a workgroup barrier every step; on this part an MFMA keeps the vector ALU of its SIMD
// from issuing for about half of its cycles, so each half step ends up bound by the slowed
// softmax and the wave that finishes early idles at the barrier.  Here a workgroup has four
// waves, one per SIMD, all running the same sequence - softmax(t), then the 16 MFMAs - and two
// such workgroups share a CU.  The two waves of a SIMD then belong to different workgroups:
// nothing synchronises them, they drift into whatever phase relation keeps both pipes fed, and a
// wave that is ahead simply goes on (free-running streams of this shape overlap 15 % better than
// barrier-coupled ones in the microbenchmark).  The barrier of a workgroup only joins four
// waves that execute the same code on four different SIMDs.
//
// Workgroup = 4 waves = heads_per_wg query heads of one KV group x 4/heads_per_wg token tiles of
// 32.  LDS: a K ring and a V ring of four 8 KiB slots each (64 KiB per workgroup, two workgroups
// per CU).  At step t a wave requests its share (8 of the 32 rows: two 1 KiB requests for K, two
// for V) of K(t+4) and V(t+2), reads K(t+1) and V(t-1), and ends with s_waitcnt vmcnt(8) + one
// barrier: everything requested two or more steps earlier has landed, i.e. K up to t+2 and V up
// to t.  The slots written at step t (those of K(t) and V(t-2)) were last read in step t-1.
#include "attn_common.h"

namespace calvo {
namespace duo {

using namespace attn;

constexpr int kRing = 4;
constexpr int kVBase = kRing * kSlot;          // V ring follows the K ring
// furthest sub-tile whose block offsets are fetched: n_pipe + 3 * kRing, with n_pipe at most
// half the number of real blocks (rounded up); each parity half of the padded table holds
// (real blocks + kTablePad) / 2 entries
static_assert(kTablePad >= 8 * kRing, "block table padding too small for the ring depth");
constexpr float kLazyBound = 65536.f;   // a lane's partial row sum of 16 weights may reach 2^16 before the reference is raised
constexpr int kLdsBytes = 2 * kRing * kSlot;   // 65536: two 4-wave workgroups per CU

// 240 of the 256 registers a wave may have at two waves per SIMD (the attribute counts half of
// the unified VGPR+AGPR file on this target): the remaining 32 per SIMD lane
// let a wave of the ingest scatter kernel become resident next to the attention waves, so the
// loading stage keeps moving while attention occupies every CU.
__global__ void __launch_bounds__(256, 2) __attribute__((amdgpu_num_vgpr(120))) attn_duo_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NW = 4;
  const lds_u8* lds = (const lds_u8*)smem;
  const unsigned lds0 = (unsigned)(size_t)lds;   // LDS byte address of the ring
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31;
  const int lh = lane >> 5;

  // ---- work item decode (wave-uniform)
  const int HW = p.heads_per_wg;
  const int TPW = NW / HW;
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
  if (p.item_index) it = p.item_index[it];       // this launch runs a subset of the work items
  const WorkItem wi = p.items[it];
  const ReqDesc rd = p.reqs[wi.req];
  const int P = rd.prefix_len, S = rd.suffix_len;
  const int TQ = 32 * TPW;
  const int q_base = wi.q_tile * TQ;
  const int hq = hg * HW + wave % HW;
  const int kv = hq / (p.n_q_heads / p.n_kv_heads);
  const int wq0 = q_base + (wave / HW) * 32;
  const bool wave_active = wq0 < S;
  const int pq_min = P + wq0;
  const int pq_max = P + min(wq0 + 32, S) - 1;
  const int ctx_len = P + S;
  // This work item covers the sub-tiles [jb, je) of the tile's context; t and j below count from jb.
  const int jb = wi.sub_begin;
  const int n_sub = wi.sub_end - jb;                           // sub-tiles this workgroup visits
  const int n_pipe = max(0, min(wi.sub_end, (P + q_base + 1) / kSK) - jb);   // ... fully visible to all its rows
  const int last_blk = (ctx_len + kBlockTokens - 1) / kBlockTokens - 1;
  // the block offsets are read-only for the whole launch: reading them through the constant address
  // space keeps the lookups on the scalar unit, outside the vmcnt accounting of the K/V requests
  typedef const __attribute__((address_space(4))) int64_t* const_i64p;
  const int n_blk_pad = last_blk + 1 + kTablePad + ((last_blk + 1) & 1);            // entries of the padded table
  // this wave's half of every sub-tile: block 2j + (wave >> 1); offsets of one parity are contiguous
  const const_i64p boffs = (const_i64p)(uintptr_t)(p.blk_offs + rd.table_off + (wave >> 1) * (n_blk_pad >> 1));
  const int Hkv = p.n_kv_heads, Hq = p.n_q_heads;
  const float c2 = p.scale * 1.4426950408889634f;

  // ---- Q as the B operand of QK^T: lane (query ln, half lh) holds Q[query][16ks + 8lh .. +8]
  bf16x8 qB[8];
  {
    const unsigned short* q = (const unsigned short*)p.q;
    const int tokq = wq0 + ln;
    const bool ok = tokq < S;
    const unsigned short* row = q + ((int64_t)(rd.q_off + (ok ? tokq : 0)) * Hq + hq) * kD + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ok) v = *(const u32x4*)(row + 16 * ks);
      qB[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[dt][r] = 0.f;
  // Softmax state per query: O and l_run are sums of weights 2^(c2 (score - m_run)).  In the
  // steady loop m_run is a reference that is only raised when a lane's partial row sum would
  // pass kLazyBound; it is always the exact maximum of some earlier sub-tile, so the largest
  // weight of a row is at least 1 and nothing underflows.
  float m_run = -INFINITY, l_run = 0.f;

  // ---- pool -> LDS.  Sub-tile j = blocks 2j and 2j+1.  Wave w fetches rows 8(w&1)..+7 of block
  // 2j + (w>>1): two instructions (4 rows x 256 B each) for K and two for V per sub-tile.  In
  // instruction h lane l owns row 8(w&1) + 4h + l/16 and LDS chunk position l%16, and fetches the
  // logical chunk that the swizzle maps there.
  const unsigned char* pool = (const unsigned char*)p.pool_layer;
  const int64_t half_b = (int64_t)kBlockTokens * Hkv * kD * 2;         // K half of a block, bytes
  const int wblk = wave >> 1;                                          // which block of the sub-tile
  // The second instruction's rows lie 4 rows further on: for V the swizzle (row & 3) is the same,
  // so the same lane offsets serve with the base moved by four rows; for K the swizzle (row & 15)
  // differs in bit 2 of the chunk index, i.e. bit 6 of the byte offset (row offsets are multiples
  // of 256).  One lane offset each is kept in registers.
  const int brow0 = 8 * (wave & 1) + (lane >> 4);                      // row inside the block, first instruction
  const unsigned rowoff = (unsigned)(brow0 * Hkv * kD * 2 + kv * kD * 2);
  const unsigned voff_k = rowoff + (((lane & 15) ^ (brow0 & 15)) << 4);
  const unsigned voff_v = rowoff + (((lane & 15) ^ ((brow0 & 3) << 2)) << 4);
  const int64_t rows4 = (int64_t)4 * Hkv * kD * 2;
  const unsigned dma_lds = lds0 + wave * 2048;                         // + h*1024 + slot*8192 (+ V ring)

  // byte offset of this wave's block of sub-tile j (the table is padded, so j may run past the end)
  auto fetch_off = [&](int j) -> int64_t { return boffs[jb + j]; };
  auto request_k_at = [&](int64_t off, int slot) {
    dma_1k(pool + off, voff_k, dma_lds + slot * kSlot);
    dma_1k(pool + off + rows4, voff_k ^ 64u, dma_lds + slot * kSlot + 1024);
  };
  auto request_v_at = [&](int64_t off, int slot) {
    dma_1k(pool + half_b + off, voff_v, dma_lds + kVBase + slot * kSlot);
    dma_1k(pool + half_b + off + rows4, voff_v, dma_lds + kVBase + slot * kSlot + 1024);
  };
  auto request_k = [&](int j) { request_k_at(fetch_off(j), j & (kRing - 1)); };
  auto request_v = [&](int j) { request_v_at(fetch_off(j), j & (kRing - 1)); };
  // synchronous variant for the sub-tiles at the end: rows past the context are not fetched,
  // their V is written as zeros so that undefined pool bytes cannot reach the PV product
  auto request_tail = [&](int j) {
    const int64_t boff = fetch_off(j);
#pragma unroll
    for (int h = 0; h < 2; h++) {
      const bool live = (jb + j) * kSK + wblk * 16 + brow0 + 4 * h < ctx_len;
      const unsigned l_k = dma_lds + (j & (kRing - 1)) * kSlot + h * 1024;
      if (live) {
        dma_1k(pool + boff + h * rows4, h ? voff_k ^ 64u : voff_k, l_k);
        dma_1k(pool + boff + half_b + h * rows4, voff_v, l_k + kVBase);
      } else {
        *(u32x4*)(smem + (l_k - lds0) + kVBase + (lane << 4)) = (u32x4){0u, 0u, 0u, 0u};
      }
    }
  };

  // ---- lane-constant operand addresses inside a slot
  // K operand: row ln, logical chunk 2ks+lh
  const lds_u8* ka_addr[8];
#pragma unroll
  for (int ks = 0; ks < 8; ks++) ka_addr[ks] = lds + ln * kRow + (((2 * ks + lh) ^ (ln & 15)) << 4);
  // V^T operand: 16-lane group g16 covers d = 16*(g16&1)..+16 of a 32-wide d tile and 4 tokens
  // starting at 4*(g16>>1); source lane s16 points at token s16/4, d offset 4*(s16%4)
  const int g16 = lane >> 4, s16 = lane & 15;
  const int v_row = 4 * (g16 >> 1) + (s16 >> 2);
  const int v_c0 = 2 * (g16 & 1) + ((s16 & 3) >> 1);
  const lds_u8* va_addr[4];
#pragma unroll
  for (int dt = 0; dt < 4; dt++)
    va_addr[dt] = lds + kVBase + v_row * kRow + ((4 * (dt ^ (v_row & 3)) + v_c0) << 4) + (s16 & 1) * 8;

  bf16x2 ones;
  ones[0] = (__bf16)1.0f;
  ones[1] = (__bf16)1.0f;

  // ---- pipeline registers: S and P of two consecutive sub-tiles
  f32x16 sbuf[2];
  bf16x8 pbuf[2][2];
  // Rescale of O that a raised reference asks for: al[b] per lane, needed[b] for the wave (a
  // scalar: the steady path sets it with one scalar move and spends no vector instruction on it).
  float al[2] = {1.f, 1.f};
  bool chg[2] = {false, false};
  bool needed[2] = {false, false};
  float nmc_run = INFINITY;     // -m_run * c2, kept beside m_run (m_run = -inf before the first sub-tile)

  auto rescale = [&](float a) {
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) o[dt][r] *= a;
  };
  auto qk = [&](int slot, f32x16& s) {
    bf16x8 ka[8];
#pragma unroll
    for (int ks = 0; ks < 8; ks++) ka[ks] = read_k(ka_addr[ks] + slot * kSlot);
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; r++) z[r] = 0.f;
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0], qB[0], z, 0, 0, 0);
#pragma unroll
    for (int ks = 1; ks < 8; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qB[ks], s, 0, 0, 0);
  };
  // statistics of one sub-tile: new running max, rescale factor, scaled max
  auto sm_head = [&](const f32x16& s, float& alpha, bool& changed, float& mc) {
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
    mx = half_swap_max(mx);
    const float m_new = fmaxf(m_run, mx);
    alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
    changed = (m_new != m_run);
    m_run = m_new;
    mc = m_new * c2;
    nmc_run = -mc;
  };
  // weights of accumulator registers 2e, 2e+1, rounded to bf16 once; the row sum adds the rounded
  // values (v_dot2 against (1,1)) so numerator and denominator use the same numbers
  auto sm_pair = [&](const f32x16& s, int e, float mc, float& ps) -> unsigned {
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e], c2, -mc));
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e + 1], c2, -mc));
    bf16x2 pk;
    pk[0] = (__bf16)p0;
    pk[1] = (__bf16)p1;
    ps = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, ps, false);
    return __builtin_bit_cast(unsigned, pk);
  };
  auto sm_all = [&](const f32x16& s, bf16x8 (&pb)[2], float& alpha, bool& changed) {
    float mc, ps = 0.f;
    sm_head(s, alpha, changed, mc);
    unsigned pk[8];
#pragma unroll
    for (int e = 0; e < 8; e++) pk[e] = sm_pair(s, e, mc, ps);
    l_run = l_run * alpha + ps;
    pb[0] = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
    pb[1] = __builtin_bit_cast(bf16x8, (u32x4){pk[4], pk[5], pk[6], pk[7]});
  };
  auto pv = [&](int slot, const bf16x8 (&pb)[2]) {
#pragma unroll
    for (int jj = 0; jj < 2; jj++)
#pragma unroll
      for (int dt = 0; dt < 4; dt++) {
        const bf16x8 a = read_vt(va_addr[dt] + slot * kSlot + 16 * jj * kRow);
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[jj], o[dt], 0, 0, 0);
      }
  };

  // ---- steady step t (t & 3 == T4): SM(t), then QK(t+1) and PV(t-1).
  // Block offsets for the requests of one unrolled iteration (steps t0 .. t0+3, t0 & 3 == 1):
  // off_cur[i] belongs to sub-tile t0 + 4 + i, off_prev2/3 to sub-tiles t0 + 2, t0 + 3.
  int64_t off_cur[4], off_prev2 = 0, off_prev3 = 0;
#ifdef CALVO_PHASE_PROF
  // One phase per build (CALVO_PHASE_PROF = phase index 0..5, or 6 for the whole step): two
  // scalar registers, so the instrumented kernel keeps the register allocation of the real one.
  unsigned prof_prev = 0, prof_acc = 0;
#define PROF(i)                                                                                  \
  {                                                                                              \
    if ((i) == (CALVO_PHASE_PROF + 5) % 6 && CALVO_PHASE_PROF < 6) prof_prev = (unsigned)clock64(); \
    if ((i) == CALVO_PHASE_PROF || ((i) == 5 && CALVO_PHASE_PROF == 6)) {                         \
      const unsigned tn_ = (unsigned)clock64();                                                  \
      prof_acc += tn_ - prof_prev;                                                               \
      prof_prev = tn_;                                                                           \
    }                                                                                            \
  }
#else
#define PROF(i)
#endif
  // first kPD MFMA operands of the coming MFMA half (see step_steady)
  bf16x8 pre[kPD];
  auto load_opnd = [&](auto idx, auto ks, auto vs) -> bf16x8 {
    constexpr int i = decltype(idx)::value, k = i >> 1;
    constexpr int KS = decltype(ks)::value, VS = decltype(vs)::value;
    if constexpr (i & 1) return read_vt(va_addr[k & 3] + VS * kSlot + 16 * (k >> 2) * kRow);
    else return read_k(ka_addr[k] + KS * kSlot);
  };
  auto prefetch = [&](auto ks, auto vs) {
    static_for<0, kPD>([&](auto idx) { pre[decltype(idx)::value] = load_opnd(idx, ks, vs); });
  };
  auto step_steady = [&](auto t4, int /*t*/) {
    constexpr int T4 = decltype(t4)::value;
    constexpr int I = (T4 + 3) & 3;                  // position inside the unrolled iteration
    constexpr int C = T4 & 1, N = C ^ 1;             // S/P of sub-tile t live in buffer C
    constexpr int KS = (T4 + 1) & 3, VS = (T4 + 3) & 3;   // ring slots of K(t+1), V(t-1)
    // K(t+4) and V(t+2) go into the ring slots of K(t) and V(t-2), which nobody reads after the
    // barrier that ended step t-1.
    request_k_at(off_cur[I], T4 & 3);
    request_v_at(I == 0 ? off_prev2 : I == 1 ? off_prev3 : off_cur[I - 2 >= 0 ? I - 2 : 0], (T4 + 2) & 3);
    PROF(0)
    auto valu_half = [&]() {
      pin(m_run);
      pin(nmc_run);
      const f32x16& s = sbuf[C];
      bool raised = false;
      float ps;
      unsigned pk[8];
      // weights of accumulator registers 2e, 2e+1, rounded to bf16 once; the row sum adds the
      // rounded values (v_dot2 against (1,1)) so numerator and denominator use the same numbers
      auto weights = [&]() {
        float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) {
          bf16x2 w;
          w[0] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e], c2, nmc_run));
          w[1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e + 1], c2, nmc_run));
          if (e & 1) ps1 = __builtin_amdgcn_fdot2_f32_bf16(w, ones, ps1, false);
          else ps0 = __builtin_amdgcn_fdot2_f32_bf16(w, ones, ps0, false);
          pk[e] = __builtin_bit_cast(unsigned, w);
        }
        ps = ps0 + ps1;
      };
      weights();
      // Accept unless a partial row sum is above the bound (or not a number).  Otherwise raise the
      // reference to this sub-tile's maximum, rescale the running sum (O is rescaled at the start
      // of the next MFMA half through al/chg) and compute the weights again: now all are <= 1.
      if (__builtin_amdgcn_ballot_w64(!(ps <= kLazyBound)) != 0) {
#if defined(CALVO_PHASE_PROF) && CALVO_PHASE_PROF == 7
        prof_acc += 1;                       // this build counts slow-path entries instead of cycles
#endif
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
        const float m_new = fmaxf(m_run, half_swap_max(mx));
        const float a_acc = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
        raised = __builtin_amdgcn_ballot_w64(m_new != m_run) != 0;
        m_run = m_new;
        nmc_run = -m_new * c2;
        l_run *= a_acc;
        al[C] = a_acc;
        weights();
      }
      l_run += ps;
      pbuf[C][0] = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
      pbuf[C][1] = __builtin_bit_cast(bf16x8, (u32x4){pk[4], pk[5], pk[6], pk[7]});
      needed[C] = raised;
      pin(pbuf[C][0]);
      pin(pbuf[C][1]);
      pin(l_run);
    };
    // The 16 MFMAs of a step alternate QK_k and PV_k (consecutive MFMAs never share an
    // accumulator); operand i is K chunk i/2 (i even) or V^T chunk i/2 (i odd), read from LDS
    // kPD operands ahead of the MFMA that consumes it.  The first kPD operands (pre[]) are read
    // by prefetch() well before the MFMA half starts, so no LDS latency is exposed.
    bf16x8 opnd[16];
    auto mfma_half = [&]() {
      pin(qB[0]);
      pin(pbuf[N][0]);
      pin(pbuf[N][1]);
      if (needed[N]) rescale(al[N]);
      f32x16 sn;
#pragma unroll
      for (int r = 0; r < 16; r++) sn[r] = 0.f;
      static_for<0, kPD>([&](auto idx) { opnd[decltype(idx)::value] = pre[decltype(idx)::value]; });
      static_for<0, 16>([&](auto idx) {
        constexpr int i = decltype(idx)::value, k = i >> 1;
        if constexpr (i & 1) o[k & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i], pbuf[N][k >> 2], o[k & 3], 0, 0, 0);
        else sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i], qB[k], sn, 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr (i + kPD < 16) {
          opnd[i + kPD] = load_opnd(Tag<i + kPD>{}, Tag<KS>{}, Tag<VS>{});
          __builtin_amdgcn_sched_group_barrier(0x100, ((i + kPD) & 1) ? 2 : 1, 0);
        }
      });
      sbuf[N] = sn;
      pin(sbuf[N]);
#pragma unroll
      for (int dt = 0; dt < 4; dt++) pin(o[dt]);
    };
    prefetch(Tag<KS>{}, Tag<VS>{});            // lands while the softmax runs
    valu_half();
    PROF(1)
    PROF(2)
    mfma_half();
    PROF(3)
    // End of the step: everything but the eight requests of the last two steps has landed, i.e.
    // K up to t+2 and V up to t: what step t+1 reads.  The barrier also separates the LDS reads
    // before it from the requests after it into the same ring slots.
    wait_vm<8>();
    PROF(4)
    __syncthreads();
    PROF(5)
  };

  // fill and drain of the pipeline: same three parts, each guarded, one after the other
  auto step_edge = [&](auto par, int t) {
    constexpr int C = decltype(par)::value, N = C ^ 1;
    request_k(t + 4);
    request_v(t + 2);
    if (t + 1 < n_pipe) qk((t + 1) & 3, sbuf[N]);
    if (t >= 1 && t <= n_pipe) {
      if (needed[N]) rescale(al[N]);
      pv((t - 1) & 3, pbuf[N]);
    }
    if (t < n_pipe) {
      sm_all(sbuf[C], pbuf[C], al[C], chg[C]);
      needed[C] = __builtin_amdgcn_ballot_w64(chg[C]) != 0;
    }
    wait_vm<8>();      // as in a steady step: K up to t+2 and V up to t have landed
    __syncthreads();
  };

  // ---- prologue: K(0..3), V(0..1) resident, S_0 computed.  From here on K(<= t+3) and V(<= t+1)
  // have been requested before step t starts.
#pragma unroll
  for (int j = 0; j < 4; j++) request_k(j);
#pragma unroll
  for (int j = 0; j < 2; j++) request_v(j);
  wait_vm<0>();
  __syncthreads();
  if (n_pipe > 0) qk(0, sbuf[0]);
  __syncthreads();   // all of QK(0) is done before any wave starts requesting into the ring again

  int t = 0;
  step_edge(Tag<0>{}, t++);                                   // t = 0: QK(1), SM(0)
  if (t + 4 < n_pipe) {
    // steady steps need 1 <= t and t + 1 < n_pipe; the unrolled loop is entered at t = 1 with the
    // block offsets of sub-tiles t+2 .. t+7 at hand; each iteration fetches the next four
    off_prev2 = fetch_off(t + 2);
    off_prev3 = fetch_off(t + 3);
#pragma unroll
    for (int i = 0; i < 4; i++) off_cur[i] = fetch_off(t + 4 + i);
    int64_t off_nxt[4];
#ifdef CALVO_PHASE_PROF
    prof_prev = (unsigned)clock64();
#endif
    for (; t + 4 < n_pipe; t += 4) {
#pragma unroll
      for (int i = 0; i < 4; i++) off_nxt[i] = fetch_off(t + 8 + i);
      step_steady(Tag<1>{}, t);
      step_steady(Tag<2>{}, t + 1);
      step_steady(Tag<3>{}, t + 2);
      step_steady(Tag<0>{}, t + 3);
      off_prev2 = off_cur[2];
      off_prev3 = off_cur[3];
#pragma unroll
      for (int i = 0; i < 4; i++) off_cur[i] = off_nxt[i];
    }
  }
#ifdef CALVO_PHASE_PROF
  if (lane == 0 && p.prof)
    p.prof[(long long)blockIdx.x * 4 + wave] = prof_acc;
#endif
  for (; t <= n_pipe; t++) {                                  // remaining pipelined steps and drain
    if (t & 1) step_edge(Tag<1>{}, t);
    else step_edge(Tag<0>{}, t);
  }

  // ---- sub-tiles on or past the diagonal: synchronous load, plain path.  The ring slots are
  // written again below (by requests and, for rows past the context, by plain LDS stores), so
  // every request of the pipelined part has to have landed first.
  wait_vm<0>();
  __syncthreads();
  for (int j = n_pipe; j < n_sub; j++) {
    request_tail(j);
    wait_vm<0>();
    __syncthreads();
    const int k0 = (jb + j) * kSK;
    if (wave_active && k0 <= pq_max) {
      f32x16 s;
      qk(j & (kRing - 1), s);
      if (k0 + 31 > pq_min) {
        const int pq = pq_min + ln;
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int kt = k0 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (kt > pq) s[r] = -INFINITY;
        }
      }
      bf16x8 pb[2];
      float alpha;
      bool changed;
      sm_all(s, pb, alpha, changed);
      if (__builtin_amdgcn_ballot_w64(changed) != 0) rescale(alpha);
      pv(j & (kRing - 1), pb);
    }
    __syncthreads();
  }

  // ---- one piece of a split tile: leave the unnormalised O, the reference and the row sum for
  // merge_splits_kernel.  Lane holds d = 32dt + 8(r/4) + 4lh + r%4 of query row ln.
  if (wi.n_splits > 1) {
    if (wave_active && wq0 + ln < S) {
      const int64_t slot = ((int64_t)it * NHG + hg) * NW + wave;
      float* po = p.part_o + (slot * 32 + ln) * kD + 4 * lh;
#pragma unroll
      for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int rq = 0; rq < 4; rq++)
          *(f32x4*)(po + 32 * dt + 8 * rq) = (f32x4){o[dt][4 * rq], o[dt][4 * rq + 1], o[dt][4 * rq + 2], o[dt][4 * rq + 3]};
      const float lt = half_swap_sum(l_run);
      if (lh == 0) {
        float* pm = p.part_ml + (slot * 32 + ln) * 2;
        pm[0] = m_run;
        pm[1] = lt;
      }
    }
    return;
  }

  // ---- normalise and write O[token][head][d]; lane holds d = 32dt + 8(r/4) + 4lh + r%4
  if (wave_active) {
    unsigned short* out = (unsigned short*)p.out;
    const float lt = half_swap_sum(l_run);
    const float inv = 1.f / lt;
    const int tokq = wq0 + ln;
    if (tokq < S) {
      unsigned short* row = out + ((int64_t)(rd.q_off + tokq) * Hq + hq) * kD + 4 * lh;
#pragma unroll
      for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int rq = 0; rq < 4; rq++) {
          bf16x2 a, b;
          a[0] = (__bf16)(o[dt][4 * rq + 0] * inv);
          a[1] = (__bf16)(o[dt][4 * rq + 1] * inv);
          b[0] = (__bf16)(o[dt][4 * rq + 2] * inv);
          b[1] = (__bf16)(o[dt][4 * rq + 3] * inv);
          u32x2 w = {__builtin_bit_cast(unsigned int, a), __builtin_bit_cast(unsigned int, b)};
          *(u32x2*)(row + 32 * dt + 8 * rq) = w;
        }
    }
  }
}

}  // namespace duo

int attn_duo_tile_tokens(int heads_per_wg) { return 32 * (4 / heads_per_wg); }

hipError_t launch_attn_duo(const AttnParams& p, hipStream_t stream) {
  if (p.n_items <= 0) return hipSuccess;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)duo::attn_duo_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, duo::kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const unsigned grid = (unsigned)p.n_items * (unsigned)(p.n_q_heads / p.heads_per_wg);
  hipLaunchKernelGGL(duo::attn_duo_kernel, dim3(grid), dim3(256), duo::kLdsBytes, stream, p);
  return hipGetLastError();
}

}  // namespace calvo
