// Paged causal GQA prefill attention for gfx950 (CDNA4), software-pipelined kernel body shared by
// the 8-wave and the 4-wave workgroup shapes: bf16 storage, head_dim 128,
// v_mfma_f32_16x16x32_bf16 for both contractions, fp32 online softmax.
//
// Why the 16x16x32 shape: the part is power limited under matrix load, and on normally
// distributed operands this shape sustains 12 % more flop/s than 32x32x16 at the power limit
// (2010-2040 against 1800-1820 TFLOP/s with nothing but MFMAs on every SIMD: half the accumulator
// traffic per product).  It costs issue slots (twice the instructions; on all-zero data, where
// nothing limits the clock, the kernel is slower), and wins on real data.
//
// Transposed formulation (every softmax statistic stays in a lane's own registers):
//   S^T[key][query] = K[key][:] . Q[query][:]       A = K rows from LDS, B = Q in registers
//   O^T[d][query]  += V^T[d][key] * P^T[key][query]  A = V^T, B = P^T
// A wave owns 32 queries = two blocks of 16 (qb); a 32-key sub-tile is two blocks of 16 keys (kb).
// Lane (c = lane % 16, g = lane / 16) of a 16x16 accumulator tile (kb, qb) holds query 16qb + c and
// the keys 16kb + 4g + r, r = 0..3: a lane works on two query columns with 8 keys each, the four
// lanes c, c+16, c+32, c+48 share a query (row max and row sum cross them only in the rare slow
// path and at the end), the O rescale is one scalar per lane and query block, and the weights of a
// lane are exactly the eight k-slots 8g..8g+7 of the B operand of the second MFMA when the k-slot
// order is taken as (kb, r): slot 8g + 4kb + r <-> key 16kb + 4g + r.  V stays token-major in LDS
// (as in the pool); the d-major A operand in that key order comes from two LDS transpose reads
// (ds_read_b64_tr_b16: keys 4g..4g+3 and 16+4g..16+4g+3 for d = 16db + c).
//
// Schedule.  The key loop advances in 32-key sub-tiles.  For sub-tile j
//     QK(j):  S_j = K_j Q^T                                     16 MFMA
//     SM(j):  P_j = 2^(c (S_j - m)), row sums                   vector ALU
//     PV(j):  O^T += V_j^T P_j^T                                16 MFMA
// A wave runs the cycle  SM(j) -> MF(j) = {PV(j), QK(j+1)} -> SM(j+1) -> ...: MF(j) reads 16 A
// operands from LDS, alternately a K operand (16 keys x 32 d) and a V^T operand (16 d x 32 keys),
// each used by two MFMAs (one per query block), four operands ahead of the MFMAs that consume them.  S and P are single-buffered: S_j is dead once SM(j) has
// produced P_j, P_j is dead once MF(j) has consumed it.  The steady loop is unrolled by the ring
// depth so that LDS ring slots are immediates.
//
// Two workgroup shapes (PipeCfg):
//   8 waves, ring of 8 slots, one workgroup per CU: waves w and w+4 share a SIMD.  In a step
//     waves 0-3 run SM(t) then MF(t); waves 4-7 run MF(t) then SM(t+1) (they are half a cycle
//     ahead), so one wave of a SIMD feeds the matrix pipe while the other uses the vector ALU.
//   4 waves, ring of 4 slots, two workgroups per CU: every wave runs SM(t) then MF(t); the two
//     waves of a SIMD belong to different workgroups and nothing couples them.  Tiles of 32 query
//     tokens per head instead of 64: for short suffixes.
//
// (Measured alternatives on the 32x32x16 shape: running QK(t+1), SM(t), PV(t-1) as one interleaved stream in every wave
// keeps the matrix pipe 96 % busy in a microbenchmark where the two waves of a SIMD run free, but
// not behind the per-step barrier the shared K/V ring needs: the lower-numbered wave wins every
// arbitration, finishes its step in 1180 cycles and waits 480 for the other one.  Wave priorities
// (s_setprio) around either half change nothing.)
//
// Softmax with a lazily raised reference.  A weight is 2^(c s - c m) with c = scale * log2(e); the row
// sum adds the fp32 weights with v_add_f32, the PV product takes them rounded to bf16 (nearest even,
// unbiased; a row's result moves by at most 2^-9 relative, the size of the output's own rounding).
// The row sum must not use v_dot2_f32_bf16: measured on MI355X, a dot-product instruction waits for
// the matrix pipe (16 of them take 616 cycles beside another wave's MFMA stream against 104 alone),
// whereas v_exp_f32, v_fma_f32, v_add_f32 and v_cvt_pk_bf16_f32 issue in the shadow of MFMAs.  In the steady
// loop m is not the running maximum: the weights of a sub-tile are computed against the current m,
// and only if a lane's partial row sum passes 2^16 (or is not a number) is the sub-tile's maximum
// taken, m raised, l and O rescaled and the weights computed again.  m is always the exact maximum
// of an earlier sub-tile, so the largest weight of a row is >= 1: nothing underflows, and with
// fp32 accumulation and bf16 weights (relative precision) the result is that of the textbook
// recurrence up to rounding.  Fill / drain steps and diagonal sub-tiles use the textbook update.
//
// Data movement.  K and V go from the pool straight into LDS with global_load_lds_dwordx4 (no
// register staging), 1 KiB (4 token rows x 256 B) per wave instruction, into two rings (K and V)
// of RING 8 KiB slots.  Step t requests K(t+KD) and V(t+VD), reads K(t+1) and V(t), and ends with
// s_waitcnt vmcnt(8) + one barrier: everything requested more than 8 instructions ago has landed.
// Rows are unpadded; 16-byte chunks are XOR-swizzled on the way in (the lane that owns LDS chunk
// position c fetches logical chunk c ^ f(row)) so that operand reads are bank-conflict free:
// K f = row & 15 (a 16-lane group reads one chunk of 16 different rows), V f = (row & 7) << 1 (half
// a wave reads two chunks of 8 different rows).  Operand addresses are lane constants plus immediates.
//
// Sub-tiles that touch the causal diagonal or the end of the context are not pipelined: they are
// at most a handful per workgroup, are loaded synchronously and run QK -> mask -> SM -> PV.
#pragma once
#include "attn_common.h"

namespace calvo {
namespace attn {

template <int NW_, int RING_>
struct PipeCfg {
  static constexpr int NW = NW_;                       // waves per workgroup
  static constexpr int RING = RING_;                   // LDS ring slots per operand
  static constexpr int KD = RING_ == 8 ? 7 : 4;        // step t requests K(t + KD) ...
  static constexpr int VD = KD - 1;                    // ... and V(t + VD)
  static constexpr bool TWO_ROLES = NW_ == 8;          // waves NW/2.. run half a cycle ahead
  static constexpr int NI = 8 / NW_;                   // 1 KiB requests per wave, operand and sub-tile
  static constexpr int LDS_BYTES = 2 * RING_ * kSlot;
};

constexpr float kLazyBound = 65536.f;   // a lane's partial row sum of 16 weights may reach 2^16 before the reference is raised

template <class Cfg_>
__device__ __forceinline__ void attn_pipeline(const AttnParams& p, unsigned char* smem) {
  constexpr int NW = Cfg_::NW, RING = Cfg_::RING, KD = Cfg_::KD, VD = Cfg_::VD, NI = Cfg_::NI;
  constexpr int RM = RING - 1;
  constexpr int kVBase = RING * kSlot;                 // V ring follows the K ring
  // furthest sub-tile whose block offsets are fetched: n_pipe + 2 * RING - 2, with n_pipe at most
  // half the number of real blocks (rounded up); each parity half of the padded table holds
  // (real blocks + kTablePad) / 2 entries
  static_assert(kTablePad >= 4 * RING, "block table padding too small for the ring depth");
  const lds_u8* lds = (const lds_u8*)smem;
  const unsigned lds0 = (unsigned)(size_t)lds;         // LDS byte address of the ring
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15;                             // query column inside a block of 16 / row of an A operand
  const int g = lane >> 4;                             // k-slots 8g..8g+7 of an operand, rows 4g..4g+3 of a result tile

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
  // this wave's half of every sub-tile: block 2j + wblk; offsets of one parity are contiguous
  const int wblk = wave / (NW / 2);
  const const_i64p boffs = (const_i64p)(uintptr_t)(p.blk_offs + rd.table_off + wblk * (n_blk_pad >> 1));
  const int Hkv = p.n_kv_heads, Hq = p.n_q_heads;
  const float c2 = p.scale * 1.4426950408889634f;

  // ---- Q as the B operand of QK^T: lane (c, g) holds Q[query 16qb + c][32ks + 8g .. +8]
  bf16x8 qB[2][4];
  {
    const unsigned short* q = (const unsigned short*)p.q;
#pragma unroll
    for (int qb = 0; qb < 2; qb++) {
      const int tokq = wq0 + 16 * qb + c;
      const bool ok = tokq < S;
      const unsigned short* row = q + ((int64_t)(rd.q_off + (ok ? tokq : 0)) * Hq + hq) * kD + 8 * g;
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (ok) v = *(const u32x4*)(row + 32 * ks);
        qB[qb][ks] = __builtin_bit_cast(bf16x8, v);
      }
    }
  }

  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  f32x4 o[8][2];                                       // O^T tile (db, qb): d = 16db + 4g + r, query 16qb + c
#pragma unroll
  for (int db = 0; db < 8; db++) {
    o[db][0] = zero4;
    o[db][1] = zero4;
  }
  // Softmax state per query.  O and l_run are sums of weights 2^(x - m_run), x the exponent of a
  // score (c * score): m_run is kept in exponent units.  In the steady loop m_run
  // is a reference that is only raised when a lane's partial row sum would pass kLazyBound; it is
  // always the exact maximum of some earlier sub-tile, so the largest weight of a row is at least 1.
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};     // per query block
  // ---- pool -> LDS.  Sub-tile j = blocks 2j and 2j+1.  Wave w fetches 32 / NW rows of block
  // 2j + wblk with NI instructions of 4 rows for K and as many for V.  In instruction h lane l owns
  // row brow0 + 4h + l/16 and LDS chunk position l%16, and fetches the logical chunk that the
  // swizzle maps there.  The second instruction's rows lie 4 rows further on: bit 2 of the row
  // number flips, i.e. bit 2 of the chunk index for K (bit 6 of the byte offset) and bit 3 for V
  // (bit 7 of the byte offset).
  const unsigned char* pool = (const unsigned char*)p.pool_layer;
  const int64_t half_b = (int64_t)kBlockTokens * Hkv * kD * 2;         // K half of a block, bytes
  const int brow0 = (32 / NW) * (wave % (NW / 2)) + (lane >> 4);       // row inside the block, first instruction
  const unsigned rowoff = (unsigned)(brow0 * Hkv * kD * 2 + kv * kD * 2);
  const unsigned voff_k = rowoff + (((lane & 15) ^ (brow0 & 15)) << 4);
  const unsigned voff_v = rowoff + (((lane & 15) ^ ((brow0 & 7) << 1)) << 4);
  const int64_t rows4 = (int64_t)4 * Hkv * kD * 2;
  const unsigned dma_lds = lds0 + wave * (1024 * NI);                  // + h*1024 + slot*8192 (+ V ring)

  // byte offset of this wave's block of sub-tile j (the table is padded, so j may run past the end)
  auto fetch_off = [&](int j) -> int64_t { return boffs[jb + j]; };
  auto request_k_at = [&](int64_t off, int slot) {
    dma_1k(pool + off, voff_k, dma_lds + slot * kSlot);
    if constexpr (NI == 2) dma_1k(pool + off + rows4, voff_k ^ 64u, dma_lds + slot * kSlot + 1024);
  };
  auto request_v_at = [&](int64_t off, int slot) {
    dma_1k(pool + half_b + off, voff_v, dma_lds + kVBase + slot * kSlot);
    if constexpr (NI == 2) dma_1k(pool + half_b + off + rows4, voff_v ^ 128u, dma_lds + kVBase + slot * kSlot + 1024);
  };
  auto request_k = [&](int j) { request_k_at(fetch_off(j), j & RM); };
  auto request_v = [&](int j) { request_v_at(fetch_off(j), j & RM); };
  // synchronous variant for the sub-tiles at the end: rows past the context are not fetched,
  // their V is written as zeros so that undefined pool bytes cannot reach the PV product
  auto request_tail = [&](int j) {
    const int64_t boff = fetch_off(j);
#pragma unroll
    for (int h = 0; h < NI; h++) {
      const bool live = (jb + j) * kSK + wblk * 16 + brow0 + 4 * h < ctx_len;
      const unsigned l_k = dma_lds + (j & RM) * kSlot + h * 1024;
      if (live) {
        dma_1k(pool + boff + h * rows4, h ? voff_k ^ 64u : voff_k, l_k);
        dma_1k(pool + boff + half_b + h * rows4, h ? voff_v ^ 128u : voff_v, l_k + kVBase);
      } else {
        *(u32x4*)(smem + (l_k - lds0) + kVBase + (lane << 4)) = (u32x4){0u, 0u, 0u, 0u};
      }
    }
  };

  // ---- lane-constant operand addresses inside a slot
  // K operand (kb, ks): key row 16kb + c, logical chunk 4ks + g (d = 32ks + 8g .. +8); the key block
  // adds 16 rows, which leaves the swizzle alone
  const lds_u8* ka_addr[4];
#pragma unroll
  for (int ks = 0; ks < 4; ks++) ka_addr[ks] = lds + c * kRow + (((4 * ks + g) ^ c) << 4);
  // V^T operand db: the 16 lanes of group g read keys 4g..4g+3 (and, 16 rows further, 16+4g..) for
  // d = 16db..16db+15: source lane c points at key 4g + c/4, d offset 16db + 4*(c%4); after the
  // transpose lane c holds the four keys for d = 16db + c
  const int v_row = 4 * g + (c >> 2);
  const lds_u8* va_addr[8];
#pragma unroll
  for (int db = 0; db < 8; db++)
    va_addr[db] = lds + kVBase + v_row * kRow + ((2 * (db ^ (v_row & 7)) + ((c & 3) >> 1)) << 4) + (c & 1) * 8;

  // two weights rounded to bf16 (nearest even), packed
  auto pack_bf16 = [](float a, float b) -> unsigned {
    bf16x2 w;
    w[0] = (__bf16)a;
    w[1] = (__bf16)b;
    return __builtin_bit_cast(unsigned, w);
  };

  // ---- pipeline registers: S and P of the sub-tile in flight
  // S tile (kb, qb): keys 16kb + 4g + r of query 16qb + c.  P operand of query block qb: the lane's
  // eight weights in k-slot order (kb, r).
  struct STile { f32x4 t[2][2]; };
  STile sbuf;
  bf16x8 pbuf[2];
  // Rescale of O that a raised reference asks for before the next PV: al per lane and query block,
  // needed for the wave (a scalar: the steady path spends no vector instruction on it).
  float al[2] = {1.f, 1.f};
  bool needed = false;

  auto rescale = [&](const float (&a)[2]) {
#pragma unroll
    for (int db = 0; db < 8; db++) {
      o[db][0] *= a[0];
      o[db][1] *= a[1];
    }
  };
  // exponent of score s of query block qb against the current reference
  auto expo = [&](float s, int qb) -> float { return __builtin_fmaf(s, c2, -m_run[qb]); };
  auto qk = [&](int slot, STile& s) {
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
      bf16x8 ka[4];
#pragma unroll
      for (int ks = 0; ks < 4; ks++) ka[ks] = read_k(ka_addr[ks] + 16 * kb * kRow + slot * kSlot);
#pragma unroll
      for (int qb = 0; qb < 2; qb++) {
        f32x4 acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[0], qB[qb][0], zero4, 0, 0, 0);
#pragma unroll
        for (int ks = 1; ks < 4; ks++) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks], qB[qb][ks], acc, 0, 0, 0);
        s.t[kb][qb] = acc;
      }
    }
  };
  // largest score of the lane's query of block qb over the whole sub-tile (all four lanes of the query)
  auto row_max = [&](const STile& s, int qb) -> float {
    float mx = fmaxf(fmaxf(s.t[0][qb][0], s.t[0][qb][1]), fmaxf(s.t[0][qb][2], s.t[0][qb][3]));
    mx = fmaxf(mx, fmaxf(fmaxf(s.t[1][qb][0], s.t[1][qb][1]), fmaxf(s.t[1][qb][2], s.t[1][qb][3])));
    return quad_max(mx);
  };
  // weights of query block qb against the current reference: fp32 sum, bf16 operand
  auto weights_of = [&](const STile& s, int qb, float& ps, bf16x8& pb) {
    float w[8];
#pragma unroll
    for (int e = 0; e < 8; e++) w[e] = __builtin_amdgcn_exp2f(expo(s.t[e >> 2][qb][e & 3], qb));
    ps = ((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7]));
    pb = __builtin_bit_cast(bf16x8, (u32x4){pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3]), pack_bf16(w[4], w[5]), pack_bf16(w[6], w[7])});
  };
  // Textbook update for one sub-tile whose scores are in s (possibly masked with -inf): new
  // running maximum, rescale factor alpha for l and O, weights against the new maximum (summed in
  // fp32, rounded to bf16 once for the PV product).
  auto sm_textbook = [&](const STile& s, bf16x8 (&pb)[2], float (&alpha)[2], bool& changed) {
    changed = false;
#pragma unroll
    for (int qb = 0; qb < 2; qb++) {
      const float m_new = fmaxf(m_run[qb], row_max(s, qb) * c2);
      alpha[qb] = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
      changed |= (m_new != m_run[qb]);
      m_run[qb] = m_new;
      float ps;
      weights_of(s, qb, ps, pb[qb]);
      l_run[qb] = l_run[qb] * alpha[qb] + ps;
    }
  };
  auto pv = [&](int slot, const bf16x8 (&pb)[2]) {
#pragma unroll
    for (int db = 0; db < 8; db++) {
      const bf16x8 a = read_vt(va_addr[db] + slot * kSlot);
      o[db][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[0], o[db][0], 0, 0, 0);
      o[db][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[1], o[db][1], 0, 0, 0);
    }
  };

  // Block offsets for the requests of one unrolled iteration (steps t0 .. t0+RING-1, t0 & RM == 1):
  // off_cur[i] belongs to sub-tile t0 + RING + i, off_prev1 / off_prev2 to sub-tiles t0 + RING - 1
  // and t0 + RING - 2.
  int64_t off_cur[RING], off_prev1 = 0, off_prev2 = 0;
  // first kPD MFMA operands of the coming MFMA half (see step_steady)
  bf16x8 pre[kPD];
  // operand i of MF(j), k = i % 8: the K operand (key block k%2, d slice k/2) of K(j+1) for i < 8, the
  // V^T operand of d block k of V(j) for i >= 8
  auto load_opnd = [&](auto idx, auto ks, auto vs) -> bf16x8 {
    constexpr int i = decltype(idx)::value, k = i & 7;
    constexpr int KS = decltype(ks)::value, VS = decltype(vs)::value;
    if constexpr (i >= 8) return read_vt(va_addr[k] + VS * kSlot);
    else return read_k(ka_addr[k >> 1] + 16 * (k & 1) * kRow + KS * kSlot);
  };
  auto prefetch = [&](auto ks, auto vs) {
    static_for<0, kPD>([&](auto idx) { pre[decltype(idx)::value] = load_opnd(idx, ks, vs); });
  };

  // ---- steady step t (t & RM == TR).  ahead == false: SM(t), MF(t).  ahead == true: MF(t), SM(t+1).
  // One body serves both kinds of wave (the flag is wave-uniform: two scalar branches per step),
  // so that the register allocation of the loop is one and the same for all waves.
  auto step_steady = [&](auto tr, bool ahead) {
    constexpr int TR = decltype(tr)::value;
    constexpr int I = (TR + RM) & RM;                // position inside the unrolled iteration
    constexpr int KS = (TR + 1) & RM, VS = TR;       // ring slots of K(t+1), V(t)
    // K(t+KD) and V(t+VD) go into ring slots that nobody reads after the barrier that ended step
    // t-1.  The waves that run ahead issue theirs after their MFMAs, which keeps the requests out
    // of the way of the matrix pipe at the start of the step.
    auto requests = [&]() {
      constexpr int ik = I + KD - RING, iv = I + VD - RING;      // index into off_cur, negative: previous iteration
      request_k_at(ik == -1 ? off_prev1 : off_cur[ik < 0 ? 0 : ik], (TR + KD) & RM);
      request_v_at(iv == -2 ? off_prev2 : iv == -1 ? off_prev1 : off_cur[iv < 0 ? 0 : iv], (TR + VD) & RM);
    };
    // Softmax of the sub-tile in sbuf -> pbuf.  The empty asm statements tie the inputs and results
    // of each half to its side: the compiler may not move them across.
    auto valu_half = [&]() {
      pin(m_run[0]);
      pin(m_run[1]);
      const STile& s = sbuf;
      bool raised = false;
      float ps[2];
      weights_of(s, 0, ps[0], pbuf[0]);
      weights_of(s, 1, ps[1], pbuf[1]);
      // Accept unless a partial row sum is above the bound (or not a number).  Otherwise raise the
      // references to this sub-tile's maxima, rescale the running sums (O is rescaled at the start
      // of the next MFMA half through al / needed) and compute the weights again: now all are <= 1.
      if (__builtin_amdgcn_ballot_w64(!(ps[0] <= kLazyBound) || !(ps[1] <= kLazyBound)) != 0) {
#pragma unroll
        for (int qb = 0; qb < 2; qb++) {
          // this sub-tile's maximum, as an exponent relative to the current reference
          const float d = fmaxf(expo(row_max(s, qb), qb), 0.f);
          const float a_acc = __builtin_amdgcn_exp2f(-d);
          raised |= __builtin_amdgcn_ballot_w64(d > 0.f) != 0;
          l_run[qb] *= a_acc;
          al[qb] = a_acc;
          m_run[qb] += d;
          weights_of(s, qb, ps[qb], pbuf[qb]);
        }
      }
      l_run[0] += ps[0];
      l_run[1] += ps[1];
      needed = raised;
      pin(pbuf[0]);
      pin(pbuf[1]);
      pin(l_run[0]);
      pin(l_run[1]);
    };
    // Eight K operands, then eight V^T operands, two MFMAs each (query blocks 0 and 1): all of QK(t+1)
    // before all of PV(t).  Keeping the MFMAs of one contraction together is worth 2 % over alternating
    // them (measured; the B operands then change between Q and P once per step, not every instruction,
    // and the part is power limited).  Operand i is read from LDS kPD operands ahead of the MFMAs that
    // consume it; the first kPD operands (pre[]) are read by prefetch() well before the MFMA half
    // starts, so no LDS latency is exposed.
    bf16x8 opnd[16];
    auto mfma_half = [&]() {
      pin(qB[0][0]);
      pin(pbuf[0]);
      pin(pbuf[1]);
      if (needed) rescale(al);
      STile sn;
      static_for<0, kPD>([&](auto idx) { opnd[decltype(idx)::value] = pre[decltype(idx)::value]; });
      static_for<0, 16>([&](auto idx) {
        constexpr int i = decltype(idx)::value, k = i & 7;
        if constexpr (i >= 8) {
          o[k][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], pbuf[0], o[k][0], 0, 0, 0);
          o[k][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], pbuf[1], o[k][1], 0, 0, 0);
        } else {
          constexpr int kb = k & 1, ks = k >> 1;
          sn.t[kb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], qB[0][ks], ks == 0 ? zero4 : sn.t[kb][0], 0, 0, 0);
          sn.t[kb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], qB[1][ks], ks == 0 ? zero4 : sn.t[kb][1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        if constexpr (i + kPD < 16) {
          opnd[i + kPD] = load_opnd(Tag<i + kPD>{}, Tag<KS>{}, Tag<VS>{});
          __builtin_amdgcn_sched_group_barrier(0x100, (i + kPD >= 8) ? 2 : 1, 0);
        }
      });
      sbuf = sn;
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        pin(sbuf.t[kb][0]);
        pin(sbuf.t[kb][1]);
      }
#pragma unroll
      for (int db = 0; db < 8; db++) {
        pin(o[db][0]);
        pin(o[db][1]);
      }
    };
    if (!ahead) {
      requests();
      prefetch(Tag<KS>{}, Tag<VS>{});          // lands while the softmax runs
      valu_half();
    }
    mfma_half();                               // ahead: pre[] was read at the end of the previous step
    if (ahead) {
      requests();
      valu_half();
      prefetch(Tag<(KS + 1) & RM>{}, Tag<(VS + 1) & RM>{});   // K(t+2), V(t+1): first operands of step t+1
    }
    // End of the step: everything but the eight most recent requests of this wave has landed, i.e.
    // K up to t+2 and V up to t+1: what step t+1 reads, and what the waves that run ahead prefetch
    // at its end for step t+2.  The barrier also separates the LDS reads before it from the
    // requests after it into the same ring slots.
    wait_vm<8>();
    __syncthreads();
  };

  // fill and drain of the pipeline: the same parts one after the other, each guarded.  On entry
  // sbuf holds S(t) (if t < n_pipe); sm_done: SM(t) has already run (a wave that ran ahead).
  auto step_edge = [&](int t, bool sm_done) {
    request_k(t + KD);
    request_v(t + VD);
    if (t < n_pipe) {
      if (!sm_done) {
        bool chg;
        sm_textbook(sbuf, pbuf, al, chg);
        needed = __builtin_amdgcn_ballot_w64(chg) != 0;
      }
      if (needed) rescale(al);
      pv(t & RM, pbuf);
    }
    if (t + 1 < n_pipe) qk((t + 1) & RM, sbuf);
    wait_vm<8>();      // as in a steady step
    __syncthreads();
  };

  // ---- prologue: K(0..KD-1), V(0..VD-1) resident, S_0 computed.  From here on K(< t+KD) and
  // V(< t+VD) have been requested before step t starts.
#pragma unroll
  for (int j = 0; j < KD; j++) request_k(j);
#pragma unroll
  for (int j = 0; j < VD; j++) request_v(j);
  wait_vm<0>();
  __syncthreads();
  if (n_pipe > 0) qk(0, sbuf);
  __syncthreads();   // all of QK(0) is done before any wave starts requesting into the ring again

  int t = 0;
  step_edge(t++, false);                                      // t = 0: SM(0), PV(0), QK(1)
  bool ahead_sm = false;                                      // this wave has already run SM(t)
  if (t + RING < n_pipe) {
    // steady steps need 1 <= t and t + 1 < n_pipe; the unrolled loop is entered at t = 1 with the
    // block offsets of sub-tiles t+RING-2 .. t+2*RING-1 at hand; each iteration fetches the next RING
    off_prev2 = fetch_off(t + RING - 2);
    off_prev1 = fetch_off(t + RING - 1);
#pragma unroll
    for (int i = 0; i < RING; i++) off_cur[i] = fetch_off(t + RING + i);
    int64_t off_nxt[RING];
    auto fetch_next = [&](int t0) {
#pragma unroll
      for (int i = 0; i < RING; i++) off_nxt[i] = fetch_off(t0 + 2 * RING + i);
    };
    auto rotate = [&]() {
      off_prev2 = off_cur[RING - 2];
      off_prev1 = off_cur[RING - 1];
#pragma unroll
      for (int i = 0; i < RING; i++) off_cur[i] = off_nxt[i];
    };
    const bool ahead = Cfg_::TWO_ROLES && wave >= NW / 2;
    if (ahead) {
      // run half a cycle ahead: SM(1) now (textbook update: S(1) comes from the fill step), and the
      // first operands of MF(1) = {PV(1), QK(2)}
      bool chg;
      sm_textbook(sbuf, pbuf, al, chg);
      needed = __builtin_amdgcn_ballot_w64(chg) != 0;
      prefetch(Tag<2 & RM>{}, Tag<1>{});
    }
    for (; t + RING < n_pipe; t += RING) {
      fetch_next(t);
      static_for<0, RING>([&](auto idx) { step_steady(Tag<(decltype(idx)::value + 1) & RM>{}, ahead); });
      rotate();
    }
    ahead_sm = ahead;                                         // SM(t) of the first step after the loop is done
  }
  for (; t < n_pipe; t++) {                                   // remaining pipelined steps
    step_edge(t, ahead_sm);
    ahead_sm = false;
  }

  // ---- sub-tiles on or past the diagonal: loaded synchronously, plain path.  The ring slots are
  // written again below (by requests and, for rows past the context, by plain LDS stores), so
  // every request of the pipelined part has to have landed first.  There are at most
  // tile tokens / 32 + 1 of them, fewer than ring slots: they are requested together and computed
  // after one wait (a group of RING at a time, should there ever be more).
  wait_vm<0>();
  __syncthreads();
  for (int j0 = n_pipe; j0 < n_sub; j0 += RING) {
    const int j1 = min(n_sub, j0 + RING);
    for (int j = j0; j < j1; j++) request_tail(j);
    wait_vm<0>();
    __syncthreads();
    for (int j = j0; j < j1; j++) {
      const int k0 = (jb + j) * kSK;
      if (!(wave_active && k0 <= pq_max)) continue;
      STile s;
      qk(j & RM, s);
      if (k0 + 31 > pq_min) {
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int qb = 0; qb < 2; qb++)
#pragma unroll
            for (int r = 0; r < 4; r++)
              if (k0 + 16 * kb + 4 * g + r > pq_min + 16 * qb + c) s.t[kb][qb][r] = -INFINITY;
      }
      bf16x8 pb[2];
      float alpha[2];
      bool changed;
      sm_textbook(s, pb, alpha, changed);
      if (__builtin_amdgcn_ballot_w64(changed) != 0) rescale(alpha);
      pv(j & RM, pb);
    }
    if (j1 < n_sub) __syncthreads();      // the next group overwrites these slots
  }

  // ---- one piece of a split tile: leave the unnormalised O, the reference (exponent units) and
  // the row sum for merge_splits_kernel (32 rows x 128 floats per wave, row = 16qb + c).  Lane holds
  // d = 16db + 4g + r of the query rows 16qb + c.
  if (wi.n_splits > 1) {
    if (wave_active) {                       // wave-uniform: every lane takes part in the exchanges
      const int64_t slot = ((int64_t)it * NHG + hg) * NW + wave;
#pragma unroll
      for (int qb = 0; qb < 2; qb++) {
        const float lt = quad_sum(l_run[qb]);
        if (wq0 + 16 * qb + c < S) {
          float* po = p.part_o + (slot * 32 + 16 * qb + c) * kD + 4 * g;
#pragma unroll
          for (int db = 0; db < 8; db++) *(f32x4*)(po + 16 * db) = o[db][qb];
          if (g == 0) {
            float* pm = p.part_ml + (slot * 32 + 16 * qb + c) * 2;
            pm[0] = m_run[qb];
            pm[1] = lt;
          }
        }
      }
    }
    return;
  }

  // ---- normalise and write O[token][head][d]; lane holds d = 16db + 4g + r of the rows 16qb + c
  if (wave_active) {
    unsigned short* out = (unsigned short*)p.out;
#pragma unroll
    for (int qb = 0; qb < 2; qb++) {
      const float lt = quad_sum(l_run[qb]);
      const float inv = 1.f / lt;
      const int tokq = wq0 + 16 * qb + c;
      if (tokq < S) {
        unsigned short* row = out + ((int64_t)(rd.q_off + tokq) * Hq + hq) * kD + 4 * g;
#pragma unroll
        for (int db = 0; db < 8; db++) {
          bf16x2 a, b;
          a[0] = (__bf16)(o[db][qb][0] * inv);
          a[1] = (__bf16)(o[db][qb][1] * inv);
          b[0] = (__bf16)(o[db][qb][2] * inv);
          b[1] = (__bf16)(o[db][qb][3] * inv);
          u32x2 w = {__builtin_bit_cast(unsigned int, a), __builtin_bit_cast(unsigned int, b)};
          *(u32x2*)(row + 16 * db) = w;
        }
      }
    }
  }
}

}  // namespace attn
}  // namespace calvo
