// Paged causal GQA prefill attention for gfx950 (CDNA4), software-pipelined kernel:
// bf16 storage, head_dim 128, v_mfma_f32_32x32x16_bf16 for both contractions, fp32 online
// softmax.  Transposed formulation as in attn_mfma.hip (S^T = K Q^T, O^T += V^T P^T, all
// softmax statistics lane-local, V^T fetched with the LDS transpose read ds_read_b64_tr_b16).
//
// Schedule.  The key loop advances in 32-key sub-tiles.  For sub-tile j the stages
//     QK(j):  S_j = K_j Q^T                                     8 MFMA
//     SM(j):  P_j = 2^(c (S_j - m)), row sums                   ~55 vector-ALU instructions
//     PV(j):  O^T += V_j^T P_j^T                                8 MFMA
// depend on each other, but QK(t+1), SM(t) and PV(t-1) do not.  Step t runs exactly these three:
// the 16 MFMAs as one half of the step (QK_k and PV_k alternating, operands read from LDS four
// MFMAs ahead), the softmax as the other half.  S and P are double buffered in registers; the
// steady loop is unrolled by eight so that register buffers and LDS ring slots are named
// statically.
//
// Softmax.  A weight is one fused multiply-add (score * scale * log2(e) - m * scale * log2(e))
// and one v_exp_f32.  (Folding the factor into Q would save nothing - it replaces the multiply-add
// by a subtract - and re-rounding Q costs accuracy when scores are large.)  In the
// steady loop the reference m is raised lazily: the weights of a sub-tile are computed against
// the current m, and only if a lane's partial row sum passes 2^16 is the sub-tile's maximum
// taken, m raised, l and O rescaled and the weights computed again.  m is always the exact
// maximum of an earlier sub-tile, so the largest weight of a row is >= 1: nothing underflows, and
// with fp32 accumulation and bf16 weights (relative precision) the result is that of the
// textbook recurrence up to rounding.  Edge and diagonal sub-tiles use the textbook update.
//
// Data movement.  K and V go from the pool straight into LDS with global_load_lds_dwordx4
// (no register staging): each wave instruction deposits 4 token rows x 256 B.  Two rings of
// eight 8 KiB slots (K and V separately, because K_j is consumed two steps before V_j): at
// step t the workgroup requests K(t+7) and V(t+5), reads K(t+1) and V(t-1), and ends with
// s_waitcnt vmcnt(8) + one barrier, which guarantees K(t+3) and V(t+1) - requested at least four
// steps earlier - have landed.  The deep ring matters: all workgroups of an XCD walk the same
// K/V stream, whoever is first pays the full HBM latency, and only requests issued several
// steps ahead keep that latency off the critical path.  Rows are unpadded; 16-byte chunks are
// XOR-swizzled on the way in (the lane that owns LDS chunk position c fetches logical chunk
// c ^ f(row)) so that operand reads are bank-conflict free: K f = row & 15, V f = (row & 3) << 2.
// All operand addresses are lane constants (8 for K, 4 for V) plus compile-time offsets.
//
// Workgroup = 8 waves = 4 query heads of one KV group x 2 token tiles of 32; waves w and w+4
// share a SIMD.  Within a step waves 0-3 run softmax first and MFMAs second, waves 4-7 the
// other way round, so one wave of a SIMD feeds the matrix pipe while the other uses the vector
// ALU.  (Measured on MI355X: an MFMA keeps the vector ALU of its SIMD from issuing for about
// half its 32 cycles, whichever wave the vector instruction comes from, so the overlap is
// partial; a wave-level priority (s_setprio) changes nothing, and neither does dropping the
// per-step barrier in favour of per-wave progress counters.)
//
// Sub-tiles that touch the causal diagonal or the end of the context are not pipelined: they
// are at most a handful per workgroup and are loaded synchronously and run QK -> mask -> SM ->
// PV one after the other.
#include "attn_common.h"

namespace calvo {
namespace pipe {

using namespace attn;

constexpr int kRing = 8;
constexpr int kVBase = kRing * kSlot;          // V ring follows the K ring
// furthest sub-tile whose block offsets are fetched: n_pipe + 2 * kRing - 2, with n_pipe at most
// half the number of real blocks (rounded up); each parity half of the padded table holds
// (real blocks + kTablePad) / 2 entries
static_assert(kTablePad >= 4 * kRing, "block table padding too small for the ring depth");
constexpr float kLazyBound = 65536.f;   // a lane's partial row sum of 16 weights may reach 2^16 before the reference is raised
constexpr int kLdsBytes = 2 * kRing * kSlot;   // 131072: one 8-wave workgroup per CU

// 240 of the 256 registers a wave may have at two waves per SIMD (the attribute counts half of
// the unified VGPR+AGPR file on this target): the remaining 32 per SIMD lane
// let a wave of the ingest scatter kernel become resident next to the attention waves, so the
// loading stage keeps moving while attention occupies every CU.
__global__ void __launch_bounds__(512, 2) __attribute__((amdgpu_num_vgpr(120))) attn_pipe_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NW = 8;
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
  // this wave's half of every sub-tile: block 2j + (wave >> 2); offsets of one parity are contiguous
  const const_i64p boffs = (const_i64p)(uintptr_t)(p.blk_offs + rd.table_off + (wave >> 2) * (n_blk_pad >> 1));
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

  // ---- pool -> LDS.  Sub-tile j = blocks 2j and 2j+1.  Wave w fetches rows 4(w&3)..+3 of block
  // 2j + (w>>2): one instruction for K and one for V per sub-tile.  Lane l owns row 4(w&3) + l/16
  // and LDS chunk position l%16, and fetches the logical chunk that the swizzle maps there.
  const unsigned char* pool = (const unsigned char*)p.pool_layer;
  const int64_t half_b = (int64_t)kBlockTokens * Hkv * kD * 2;         // K half of a block, bytes
  const int wblk = wave >> 2;                                          // which block of the sub-tile
  const int brow = 4 * (wave & 3) + (lane >> 4);                       // row inside the block
  const unsigned rowoff = (unsigned)(brow * Hkv * kD * 2 + kv * kD * 2);
  const unsigned voff_k = rowoff + (((lane & 15) ^ (brow & 15)) << 4);
  const unsigned voff_v = rowoff + (((lane & 15) ^ ((brow & 3) << 2)) << 4);
  const unsigned dma_lds = lds0 + wave * 1024;                         // + slot*8192 (+ V ring)

  // byte offset of this wave's block of sub-tile j (the table is padded, so j may run past the end)
  auto fetch_off = [&](int j) -> int64_t { return boffs[jb + j]; };
  auto request_k_at = [&](int64_t off, int slot) { dma_1k(pool + off, voff_k, dma_lds + slot * kSlot); };
  auto request_v_at = [&](int64_t off, int slot) {
    dma_1k(pool + half_b + off, voff_v, dma_lds + kVBase + slot * kSlot);
  };
  auto request_k = [&](int j) { request_k_at(fetch_off(j), j & (kRing - 1)); };
  auto request_v = [&](int j) { request_v_at(fetch_off(j), j & (kRing - 1)); };
  // synchronous variant for the sub-tiles at the end: rows past the context are not fetched,
  // their V is written as zeros so that undefined pool bytes cannot reach the PV product
  auto request_tail = [&](int j) {
    const int64_t boff = fetch_off(j);
    const bool live = (jb + j) * kSK + wblk * 16 + brow < ctx_len;
    const unsigned l_k = dma_lds + (j & (kRing - 1)) * kSlot;
    if (live) {
      dma_1k(pool + boff, voff_k, l_k);
      dma_1k(pool + boff + half_b, voff_v, l_k + kVBase);
    } else {
      *(u32x4*)(smem + (l_k - lds0) + kVBase + (lane << 4)) = (u32x4){0u, 0u, 0u, 0u};
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

  // ---- steady step t (t & 7 == T8): QK(t+1), SM(t), PV(t-1).  MF selects the phase order.
  // Block offsets for the requests of one unrolled iteration (steps t0 .. t0+7, t0 & 7 == 1):
  // off_cur[i] belongs to sub-tile t0 + 8 + i, off_prev5/6/7 to sub-tiles t0 + 5, t0 + 6, t0 + 7.
  int64_t off_cur[8], off_prev5 = 0, off_prev6 = 0, off_prev7 = 0;
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
  auto step_steady = [&](auto t8, auto mf, int /*t*/) {
    constexpr int T8 = decltype(t8)::value;
    constexpr bool MF = decltype(mf)::value != 0;
    constexpr int I = (T8 + 7) & 7;                  // position inside the unrolled iteration
    constexpr int C = T8 & 1, N = C ^ 1;             // S/P of sub-tile t live in buffer C
    constexpr int KS = (T8 + 1) & 7, VS = (T8 + 7) & 7;   // ring slots of K(t+1), V(t-1)
    // K(t+7) and V(t+5) go into the ring slots of K(t-1) and V(t-3), which nobody reads after
    // the barrier that ended step t-1.  Waves 4-7 issue theirs after their MFMAs, which keeps the
    // requests out of the way of the matrix pipe at the start of the step.
    auto requests = [&]() {
      request_k_at(I == 0 ? off_prev7 : off_cur[(I + 7) & 7], (T8 + 7) & 7);
      request_v_at(I == 0 ? off_prev5 : I == 1 ? off_prev6 : I == 2 ? off_prev7 : off_cur[(I + 5) & 7], (T8 + 5) & 7);
    };
    if constexpr (!MF) requests();
    PROF(0)
    // The step has two halves.  Waves 0-3 run the softmax of
    // sub-tile t in the first half and the 16 MFMAs (QK(t+1), PV(t-1)) in the second; waves 4-7,
    // which share their SIMDs, do the opposite, so in each half one wave of a SIMD owns the
    // matrix pipe and the other the vector ALU.  The empty asm statements tie the inputs and
    // results of each half to its side of the barrier: the compiler may not move them across.
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
    if constexpr (!MF) {
      prefetch(Tag<KS>{}, Tag<VS>{});          // lands while the softmax runs
      valu_half();
      PROF(1)
      PROF(2)
      mfma_half();
      PROF(3)
    } else {
      mfma_half();                             // pre[] was read at the end of the previous step
      requests();
      PROF(1)
      PROF(2)
      valu_half();
      prefetch(Tag<(KS + 1) & 7>{}, Tag<(VS + 1) & 7>{});   // K(t+2), V(t): first operands of step t+1
      PROF(3)
    }
    // End of the step: everything but the eight requests of the last four steps has landed,
    // i.e. K up to t+3 and V up to t+1: what step t+1 reads, and what waves 4-7 prefetch at its
    // end for step t+2.  The barrier also separates the LDS reads before it from the requests
    // after it into the same ring slots.
    wait_vm<8>();
    PROF(4)
    __syncthreads();
    PROF(5)
  };

  // fill and drain of the pipeline: same three parts, each guarded, one after the other
  auto step_edge = [&](auto par, int t) {
    constexpr int C = decltype(par)::value, N = C ^ 1;
    request_k(t + 7);
    request_v(t + 5);
    if (t + 1 < n_pipe) qk((t + 1) & 7, sbuf[N]);
    if (t >= 1 && t <= n_pipe) {
      if (needed[N]) rescale(al[N]);
      pv((t - 1) & 7, pbuf[N]);
    }
    if (t < n_pipe) {
      sm_all(sbuf[C], pbuf[C], al[C], chg[C]);
      needed[C] = __builtin_amdgcn_ballot_w64(chg[C]) != 0;
    }
    wait_vm<8>();      // as in a steady step: K up to t+3 and V up to t+1 have landed
    __syncthreads();
  };

  // ---- prologue: K(0..6), V(0..4) resident, S_0 computed.  From here on K(<= t+6) and V(<= t+4)
  // have been requested before step t starts.
#pragma unroll
  for (int j = 0; j < 7; j++) request_k(j);
#pragma unroll
  for (int j = 0; j < 5; j++) request_v(j);
  wait_vm<0>();
  __syncthreads();
  if (n_pipe > 0) qk(0, sbuf[0]);
  __syncthreads();   // all of QK(0) is done before any wave starts requesting into the ring again

  int t = 0;
  step_edge(Tag<0>{}, t++);                                   // t = 0: QK(1), SM(0)
  if (t + 8 < n_pipe) {
    // steady steps need 1 <= t and t + 1 < n_pipe; the unrolled loop is entered at t = 1 with the
    // block offsets of sub-tiles t+6 .. t+15 at hand; each iteration fetches the next eight
    off_prev5 = fetch_off(t + 5);
    off_prev6 = fetch_off(t + 6);
    off_prev7 = fetch_off(t + 7);
#pragma unroll
    for (int i = 0; i < 8; i++) off_cur[i] = fetch_off(t + 8 + i);
    int64_t off_nxt[8];
    auto fetch_next = [&](int t0) {
#pragma unroll
      for (int i = 0; i < 8; i++) off_nxt[i] = fetch_off(t0 + 16 + i);
    };
    auto rotate = [&]() {
      off_prev5 = off_cur[5];
      off_prev6 = off_cur[6];
      off_prev7 = off_cur[7];
#pragma unroll
      for (int i = 0; i < 8; i++) off_cur[i] = off_nxt[i];
    };
#ifdef CALVO_PHASE_PROF
    prof_prev = (unsigned)clock64();
#endif
    if (wave < 4) {
      for (; t + 8 < n_pipe; t += 8) {
        fetch_next(t);
        step_steady(Tag<1>{}, Tag<0>{}, t);
        step_steady(Tag<2>{}, Tag<0>{}, t + 1);
        step_steady(Tag<3>{}, Tag<0>{}, t + 2);
        step_steady(Tag<4>{}, Tag<0>{}, t + 3);
        step_steady(Tag<5>{}, Tag<0>{}, t + 4);
        step_steady(Tag<6>{}, Tag<0>{}, t + 5);
        step_steady(Tag<7>{}, Tag<0>{}, t + 6);
        step_steady(Tag<0>{}, Tag<0>{}, t + 7);
        rotate();
      }
    } else {
      prefetch(Tag<2>{}, Tag<0>{});                          // K(2), V(0) for step 1
      for (; t + 8 < n_pipe; t += 8) {
        fetch_next(t);
        step_steady(Tag<1>{}, Tag<1>{}, t);
        step_steady(Tag<2>{}, Tag<1>{}, t + 1);
        step_steady(Tag<3>{}, Tag<1>{}, t + 2);
        step_steady(Tag<4>{}, Tag<1>{}, t + 3);
        step_steady(Tag<5>{}, Tag<1>{}, t + 4);
        step_steady(Tag<6>{}, Tag<1>{}, t + 5);
        step_steady(Tag<7>{}, Tag<1>{}, t + 6);
        step_steady(Tag<0>{}, Tag<1>{}, t + 7);
        rotate();
      }
    }
  }
#ifdef CALVO_PHASE_PROF
  if (lane == 0 && p.prof)
    p.prof[(long long)blockIdx.x * 8 + wave] = prof_acc;
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
      qk(j & 7, s);
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
      pv(j & 7, pb);
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

// Combines the pieces of split tiles: for every row and head, with m = max_c m_c,
//     O = sum_c 2^(c2 (m_c - m)) O_c  /  sum_c 2^(c2 (m_c - m)) l_c
// (the pieces' O_c, l_c are sums of weights 2^(c2 (score - m_c))).  One workgroup of 256 threads per
// (split tile, head group, wave slot of the attention workgroup): thread = (row 0..31, 16-float chunk 0..7).  A piece in which
// a row saw no key has l_c = 0 and m_c = -inf and drops out.
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
  const float c2 = p.scale * 1.4426950408889634f;
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
    const float wgt = __builtin_amdgcn_exp2f((mc - m) * c2);
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

hipError_t launch_attn_pipe(const AttnParams& p, hipStream_t stream) {
  if (p.n_items <= 0) return hipSuccess;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)pipe::attn_pipe_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, pipe::kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const unsigned grid = (unsigned)p.n_items * (unsigned)(p.n_q_heads / p.heads_per_wg);
  hipLaunchKernelGGL(pipe::attn_pipe_kernel, dim3(grid), dim3(512), pipe::kLdsBytes, stream, p);
  return hipGetLastError();
}

hipError_t launch_merge_splits(const AttnParams& p, const int32_t* split_tiles, int n_split_tiles, hipStream_t stream) {
  if (n_split_tiles <= 0) return hipSuccess;
  const unsigned grid = (unsigned)n_split_tiles * (unsigned)(p.n_q_heads / p.heads_per_wg) * (unsigned)p.waves_per_wg;
  hipLaunchKernelGGL(pipe::merge_splits_kernel, dim3(grid), dim3(256), 0, stream, p, split_tiles);
  return hipGetLastError();
}

}  // namespace calvo
