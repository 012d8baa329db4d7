// Microbenchmark: how the two instruction streams of the pipelined attention kernels share one
// SIMD of gfx950.  Stream M = bursts of 16 LDS-fed v_mfma_f32_32x32x16_bf16 (the QK/PV half of
// a step, operands read four MFMAs ahead with the kernel's swizzled addresses); stream S = the
// 32-key softmax of a step (16 fused multiply-adds, 16 v_exp_f32, 8 bf16 packs, 8 v_dot2 row
// sums).  Waves w and w + 4 of a 512-thread workgroup share a SIMD; every wave times itself with
// s_memtime.  Not part of the library; build and run by hand:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         paper_2603_21257_amd/csrc/probe_coissue.hip -o probe_coissue && ./probe_coissue
// Compile-time variants:
//   -DPRIO=1 / -DPRIO=2   raise the wave priority (s_setprio 3) around the softmax / around the MFMA burst
//   -DM16                 the burst uses 32 v_mfma_f32_16x16x32_bf16 instead of 16 of the 32x32x16 shape
//   -DLEAN                the softmax adds its row sum straight into the running sum (one dependent chain)
//   -DNOLDS               the MFMA operands come from registers instead of LDS (what the LDS reads cost)
//   -DW12                 twelve waves per workgroup (three per SIMD, at most 168 registers each); waves 4-11 take the second role
//   -DACCO                the O accumulators of the burst live in accumulation registers (a[..]) instead of v[..]
// The "fused" runs interleave the softmax instructions between the MFMAs of the same wave.
#include <hip/hip_runtime.h>
#ifndef PRIO
#define PRIO 0
#endif
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((address_space(3))) unsigned char lds_u8;
template <int V> struct Tag { static constexpr int value = V; };
template <int B, int E, typename F> __device__ inline void static_for(F&& f) { if constexpr (B < E) { f(Tag<B>{}); static_for<B + 1, E>(f); } }
__device__ inline bf16x8 rd128(const lds_u8* a) { return *(const __attribute__((address_space(3))) bf16x8*)a; }
__device__ inline bf16x8 rdtr(const lds_u8* a) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a + 2048));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
constexpr int PD = 4;
enum Role { IDLE = 0, MFMA = 1, SOFTMAX = 2, ALTERNATE = 3, FUSED = 4 };
// sync (ALTERNATE only): 0 no barrier, 1 one barrier per step, 2 one per half step
#ifdef W12
constexpr int kThreads = 768;    // twelve waves: three per SIMD; waves 4-11 take role B
#else
constexpr int kThreads = 512;
#endif
template <int NVT>
__global__ void __launch_bounds__(kThreads, kThreads == 512 ? 2 : 1) k_mix(float* out, long long* cyc, int iters, int roleA, int roleB, int sync, int nvsel) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const lds_u8* lds = (const lds_u8*)smem;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int role = wave < 4 ? roleA : roleB;
  for (int i = threadIdx.x; i < 131072 / 4; i += kThreads) ((unsigned*)smem)[i] = 0x3c003c00u + i % 7;
  __syncthreads();
  bf16x8 qB[8], pb[2];
  for (int k = 0; k < 8; k++) for (int j = 0; j < 8; j++) qB[k][j] = (__bf16)(0.01f * (k + j + lane % 3));
  for (int k = 0; k < 2; k++) for (int j = 0; j < 8; j++) pb[k][j] = (__bf16)(0.02f * (k + j));
  f32x16 o[4]; for (int d = 0; d < 4; d++) for (int r = 0; r < 16; r++) o[d][r] = 0.f;
  f32x16 sprev; for (int r = 0; r < 16; r++) sprev[r] = 0.01f * r + lane;
  const int ln = lane & 31, lh = lane >> 5, g16 = lane >> 4, s16 = lane & 15;
  const int v_row = 4 * (g16 >> 1) + (s16 >> 2), v_c0 = 2 * (g16 & 1) + ((s16 & 3) >> 1);
  const lds_u8* ka_addr[8]; const lds_u8* va_addr[4];
  for (int ks = 0; ks < 8; ks++) ka_addr[ks] = lds + ln * 256 + (((2 * ks + lh) ^ (ln & 15)) << 4);
  for (int dt = 0; dt < 4; dt++) va_addr[dt] = lds + 65536 + v_row * 256 + ((4 * (dt ^ (v_row & 3)) + v_c0) << 4) + (s16 & 1) * 8;
  float m_run = 0.5f, l_run = 0.f; const float c2 = 0.1275f; float nmc = -m_run * c2;
  bf16x2 ones; ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;
  bf16x8 pre[PD];
  auto operand = [&](auto idx, int slot) -> bf16x8 {
    constexpr int i = decltype(idx)::value, k = i >> 1;
#ifdef NOLDS
    return qB[i & 7];                          // operands from registers: the burst reads no LDS
#endif
    if constexpr (i & 1) return rdtr(va_addr[k & 3] + slot + 16 * (k >> 2) * 256);
    else return rd128(ka_addr[k] + slot);
  };
  auto prefetch = [&](int slot) { static_for<0, PD>([&](auto idx) { pre[decltype(idx)::value] = operand(idx, slot); }); };
  // 16 MFMAs on the operands of `slot`; stream == true also requests the first operands of `next`
#ifdef M16
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  f32x4 o16[16]; for (int d = 0; d < 16; d++) for (int r = 0; r < 4; r++) o16[d][r] = 0.f;
  auto burst = [&](int slot, int next, bool stream) {
    bf16x8 opnd[16];
    static_for<0, PD>([&](auto idx) { opnd[decltype(idx)::value] = pre[decltype(idx)::value]; });
    f32x4 sn4[4]; for (int d = 0; d < 4; d++) for (int r = 0; r < 4; r++) sn4[d][r] = 0.f;
    static_for<0, 16>([&](auto idx) {
      constexpr int i = decltype(idx)::value, k = i >> 1;
      if constexpr (i & 1) {
        o16[(2 * k) & 15] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], pb[0], o16[(2 * k) & 15], 0, 0, 0);
        o16[(2 * k + 1) & 15] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], pb[1], o16[(2 * k + 1) & 15], 0, 0, 0);
      } else {
        sn4[k & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], qB[k], sn4[k & 1], 0, 0, 0);
        sn4[2 + (k & 1)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(opnd[i], qB[(k + 1) & 7], sn4[2 + (k & 1)], 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      if constexpr (i + PD < 16) {
        opnd[i + PD] = operand(Tag<i + PD>{}, slot);
        __builtin_amdgcn_sched_group_barrier(0x100, ((i + PD) & 1) ? 2 : 1, 0);
      } else if (stream) {
        pre[i + PD - 16] = operand(Tag<i + PD - 16>{}, next);
        __builtin_amdgcn_sched_group_barrier(0x100, ((i + PD) & 1) ? 2 : 1, 0);
      }
    });
    for (int d = 0; d < 4; d++) for (int r = 0; r < 4; r++) sprev[4 * d + r] = sn4[d][r];
  };
#else
  auto burst = [&](int slot, int next, bool stream) {
    bf16x8 opnd[16];
    static_for<0, PD>([&](auto idx) { opnd[decltype(idx)::value] = pre[decltype(idx)::value]; });
    f32x16 sn; for (int r = 0; r < 16; r++) sn[r] = 0.f;
    static_for<0, 16>([&](auto idx) {
      constexpr int i = decltype(idx)::value, k = i >> 1;
#ifdef ACCO
      // accumulators named by register file: O in accumulation registers, S in ordinary ones
      if constexpr (i & 1) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o[k & 3]) : "v"(opnd[i]), "v"(pb[k >> 2]));
      else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(sn) : "v"(opnd[i]), "v"(qB[k]));
      if constexpr (i + PD < 16) opnd[i + PD] = operand(Tag<i + PD>{}, slot);
      else if (stream) pre[i + PD - 16] = operand(Tag<i + PD - 16>{}, next);
#else
      if constexpr (i & 1) o[k & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i], pb[k >> 2], o[k & 3], 0, 0, 0);
      else sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i], qB[k], sn, 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if constexpr (i + PD < 16) {
        opnd[i + PD] = operand(Tag<i + PD>{}, slot);
        __builtin_amdgcn_sched_group_barrier(0x100, ((i + PD) & 1) ? 2 : 1, 0);
      } else if (stream) {
        pre[i + PD - 16] = operand(Tag<i + PD - 16>{}, next);
        __builtin_amdgcn_sched_group_barrier(0x100, ((i + PD) & 1) ? 2 : 1, 0);
      }
#endif
    });
    sprev = sn;
  };
#endif
  auto softmax = [&]() {
    f32x16 s = sprev;
    asm volatile("" : "+v"(s));
#ifdef LEAN
    const float l_old = l_run;
    unsigned pk[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
      bf16x2 w;
      w[0] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e], c2, nmc));
      w[1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e + 1], c2, nmc));
      l_run = __builtin_amdgcn_fdot2_f32_bf16(w, ones, l_run, false);
      pk[e] = __builtin_bit_cast(unsigned, w);
    }
    if (__builtin_amdgcn_ballot_w64(!(l_run <= 1.15e18f)) != 0) { m_run += 1.f; nmc = -m_run * c2; l_run = l_old * 0.5f; }
#else
    const float mc = m_run * c2;
    float ps0 = 0.f, ps1 = 0.f; unsigned pk[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
      bf16x2 w;
      w[0] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e], c2, -mc));
      w[1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * e + 1], c2, -mc));
      if (e & 1) ps1 = __builtin_amdgcn_fdot2_f32_bf16(w, ones, ps1, false); else ps0 = __builtin_amdgcn_fdot2_f32_bf16(w, ones, ps0, false);
      pk[e] = __builtin_bit_cast(unsigned, w);
    }
    const float ps = ps0 + ps1;
    if (__builtin_amdgcn_ballot_w64(!(ps <= 65536.f)) != 0) { m_run += 1.f; l_run *= 0.5f; }
    l_run += ps;
#endif
    pb[0] = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
    pb[1] = __builtin_bit_cast(bf16x8, (u32x4){pk[4], pk[5], pk[6], pk[7]});
  };
  // one step with the softmax of the previous scores interleaved between the 16 MFMAs: NV vector
  // instructions after every MFMA
  auto fused = [&](int slot, int next, auto nv) {
    constexpr int NV = decltype(nv)::value;   // 3: fma/exp + cvt|dot per packet; 4: two packets of softmax per MFMA pair ...
    bf16x8 opnd[16];
    static_for<0, PD>([&](auto idx) { opnd[decltype(idx)::value] = pre[decltype(idx)::value]; });
    f32x16 sn; for (int r = 0; r < 16; r++) sn[r] = 0.f;
    f32x16 s = sprev;
    const float mc = m_run * c2;
    float ps0 = 0.f, ps1 = 0.f; unsigned pk[8]; float ex[16];
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, 16>([&](auto idx) {
      constexpr int i = decltype(idx)::value, k = i >> 1;
      if constexpr (i & 1) o[k & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i], pb[k >> 2], o[k & 3], 0, 0, 0);
      else sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[i], qB[k], sn, 0, 0, 0);
      if constexpr (i + PD < 16) opnd[i + PD] = operand(Tag<i + PD>{}, slot);
      else pre[i + PD - 16] = operand(Tag<i + PD - 16>{}, next);
      ex[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], c2, -mc));
      if constexpr (i & 1) {
        bf16x2 w; w[0] = (__bf16)ex[i - 1]; w[1] = (__bf16)ex[i];
        pk[k] = __builtin_bit_cast(unsigned, w);
      } else if constexpr (i >= 2) {
        const bf16x2 w = __builtin_bit_cast(bf16x2, pk[k - 1]);
        if ((k - 1) & 1) ps1 = __builtin_amdgcn_fdot2_f32_bf16(w, ones, ps1, false); else ps0 = __builtin_amdgcn_fdot2_f32_bf16(w, ones, ps0, false);
      }
      if constexpr (NV == 3 || (i & 1)) __builtin_amdgcn_sched_barrier(0);
    });
    ps1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk[7]), ones, ps1, false);
    const float ps = ps0 + ps1;
    __builtin_amdgcn_sched_barrier(0);
    if (__builtin_amdgcn_ballot_w64(!(ps <= 65536.f)) != 0) { m_run += 1.f; l_run *= 0.5f; }
    l_run += ps;
    pb[0] = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
    pb[1] = __builtin_bit_cast(bf16x8, (u32x4){pk[4], pk[5], pk[6], pk[7]});
    sprev = sn;
  };
  const long long t0 = clock64();
  if (role == MFMA) {
    prefetch(0);
    for (int it = 0; it < iters; it++) burst((it & 7) * 8192, ((it + 1) & 7) * 8192, true);
  } else if (role == SOFTMAX) {
    for (int it = 0; it < iters; it++) { softmax(); sprev[it & 15] += l_run * 1e-12f; }
  } else if (role == FUSED) {
    prefetch(0);
    for (int it = 0; it < iters; it++) {
      fused((it & 7) * 8192, ((it + 1) & 7) * 8192, Tag<NVT>{});
      if (sync != 0) __builtin_amdgcn_s_barrier();
    }
  } else if (role == ALTERNATE) {
    if (wave < 4) {                               // softmax first, MFMAs second
      for (int it = 0; it < iters; it++) {
        const int slot = (it & 7) * 8192;
        prefetch(slot);
        __builtin_amdgcn_sched_barrier(0);
#if PRIO == 1
        __builtin_amdgcn_s_setprio(3);
#endif
        softmax();
        __builtin_amdgcn_sched_barrier(0);
#if PRIO == 1
        __builtin_amdgcn_s_setprio(0);
#endif
        if (sync == 2) __builtin_amdgcn_s_barrier();
#if PRIO == 2
        __builtin_amdgcn_s_setprio(3);
#endif
        burst(slot, 0, false);
#if PRIO == 2
        __builtin_amdgcn_s_setprio(0);
#endif
        __builtin_amdgcn_sched_barrier(0);
        if (sync != 0) __builtin_amdgcn_s_barrier();
      }
    } else {                                      // MFMAs first, softmax second
      prefetch(0);
      for (int it = 0; it < iters; it++) {
#if PRIO == 2
        __builtin_amdgcn_s_setprio(3);
#endif
        burst((it & 7) * 8192, 0, false);
        __builtin_amdgcn_sched_barrier(0);
#if PRIO == 2
        __builtin_amdgcn_s_setprio(0);
#endif
        if (sync == 2) __builtin_amdgcn_s_barrier();
#if PRIO == 1
        __builtin_amdgcn_s_setprio(3);
#endif
        softmax();
        __builtin_amdgcn_sched_barrier(0);
#if PRIO == 1
        __builtin_amdgcn_s_setprio(0);
#endif
        prefetch(((it + 1) & 7) * 8192);
        __builtin_amdgcn_sched_barrier(0);
        if (sync != 0) __builtin_amdgcn_s_barrier();
      }
    }
  }
  const long long t1 = clock64();
  float acc = l_run + m_run;
#ifdef M16
  for (int d = 0; d < 16; d++) for (int r = 0; r < 4; r++) acc += o16[d][r];
#endif
  for (int d = 0; d < 4; d++) for (int r = 0; r < 16; r++) acc += o[d][r] + sprev[r];
  out[blockIdx.x * kThreads + threadIdx.x] = acc;
  if (lane == 0) cyc[blockIdx.x * 16 + wave] = t1 - t0;
}

static void run(const char* name, int roleA, int roleB, int sync, int nvsel = 4) {
  const int nblk = 256, iters = 2000;
  float* out; long long* cyc;
  CK(hipMalloc(&out, nblk * kThreads * 4)); CK(hipMalloc(&cyc, nblk * 16 * 8));
  auto kern = nvsel == 3 ? k_mix<3> : nvsel == 5 ? k_mix<5> : k_mix<4>;
  CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms = 0;
  for (int rep = 0; rep < 3; rep++) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(nblk), dim3(kThreads), 131072, 0, out, cyc, iters, roleA, roleB, sync, nvsel);
    CK(hipEventRecord(e1)); CK(hipDeviceSynchronize()); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  long long h[16]; CK(hipMemcpy(h, cyc, 128, hipMemcpyDeviceToHost));
  printf("%-58s waves 0-3 %5.0f ticks/iter, waves 4-7 %5.0f ticks/iter, kernel %.3f ms", name, (double)h[0] / iters, (double)h[4] / iters, ms);
  if (kThreads == 768) printf(", waves 8-11 %5.0f ticks/iter", (double)h[8] / iters);
  printf("\n");
  CK(hipFree(out)); CK(hipFree(cyc));
}

int main() {
  run("MFMA bursts alone (one wave per SIMD)", MFMA, IDLE, 0);
  run("softmax alone (one wave per SIMD)", SOFTMAX, IDLE, 0);
  run("MFMA + MFMA", MFMA, MFMA, 0);
  run("softmax + softmax", SOFTMAX, SOFTMAX, 0);
  run("MFMA on waves 0-3, softmax on waves 4-7", MFMA, SOFTMAX, 0);
  run("softmax on waves 0-3, MFMA on waves 4-7", SOFTMAX, MFMA, 0);
  run("alternating as the 8-wave kernel does, no barrier", ALTERNATE, ALTERNATE, 0);
  run("alternating as the 8-wave kernel does, one barrier per step", ALTERNATE, ALTERNATE, 1);
  run("alternating as the 8-wave kernel does, barrier per half step", ALTERNATE, ALTERNATE, 2);
  run("fused: softmax between the MFMAs of the same wave, one wave per SIMD", FUSED, IDLE, 0, 3);
  run("fused, both waves, no barrier", FUSED, FUSED, 0, 3);
  run("fused, both waves, one barrier per step", FUSED, FUSED, 1, 3);
  return 0;
}
