// Microbenchmark: how the two instruction streams of the pipelined attention kernel share one
// SIMD of gfx950.  Stream M = bursts of 16 LDS-fed v_mfma_f32_32x32x16_bf16 (the QK/PV half of
// a step, operands read four MFMAs ahead with the kernel's swizzled addresses); stream S = the
// 32-key softmax of a step (16 fused multiply-adds, 16 v_exp_f32, 8 bf16 packs, 8 v_dot2 row
// sums).  Waves w and w + 4 of a 512-thread workgroup share a SIMD; every wave times itself with
// s_memtime.  Not part of the library; build and run by hand:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         paper_2603_21257_amd/csrc/probe_coissue.hip -o probe_coissue && ./probe_coissue
#include <hip/hip_runtime.h>
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
enum Role { IDLE = 0, MFMA = 1, SOFTMAX = 2, ALTERNATE = 3 };
// sync (ALTERNATE only): 0 no barrier, 1 one barrier per step, 2 one per half step
__global__ void __launch_bounds__(512, 2) k_mix(float* out, long long* cyc, int iters, int roleA, int roleB, int sync) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const lds_u8* lds = (const lds_u8*)smem;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int role = wave < 4 ? roleA : roleB;
  for (int i = threadIdx.x; i < 131072 / 4; i += 512) ((unsigned*)smem)[i] = 0x3c003c00u + i % 7;
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
  float m_run = 0.5f, l_run = 0.f; const float c2 = 0.1275f;
  bf16x2 ones; ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;
  bf16x8 pre[PD];
  auto operand = [&](auto idx, int slot) -> bf16x8 {
    constexpr int i = decltype(idx)::value, k = i >> 1;
    if constexpr (i & 1) return rdtr(va_addr[k & 3] + slot + 16 * (k >> 2) * 256);
    else return rd128(ka_addr[k] + slot);
  };
  auto prefetch = [&](int slot) { static_for<0, PD>([&](auto idx) { pre[decltype(idx)::value] = operand(idx, slot); }); };
  // 16 MFMAs on the operands of `slot`; stream == true also requests the first operands of `next`
  auto burst = [&](int slot, int next, bool stream) {
    bf16x8 opnd[16];
    static_for<0, PD>([&](auto idx) { opnd[decltype(idx)::value] = pre[decltype(idx)::value]; });
    f32x16 sn; for (int r = 0; r < 16; r++) sn[r] = 0.f;
    static_for<0, 16>([&](auto idx) {
      constexpr int i = decltype(idx)::value, k = i >> 1;
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
    });
    sprev = sn;
  };
  auto softmax = [&]() {
    f32x16 s = sprev;
    asm volatile("" : "+v"(s));
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
    pb[0] = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
    pb[1] = __builtin_bit_cast(bf16x8, (u32x4){pk[4], pk[5], pk[6], pk[7]});
  };
  const long long t0 = clock64();
  if (role == MFMA) {
    prefetch(0);
    for (int it = 0; it < iters; it++) burst((it & 7) * 8192, ((it + 1) & 7) * 8192, true);
  } else if (role == SOFTMAX) {
    for (int it = 0; it < iters; it++) { softmax(); sprev[it & 15] += l_run * 1e-12f; }
  } else if (role == ALTERNATE) {
    if (wave < 4) {                               // softmax first, MFMAs second
      for (int it = 0; it < iters; it++) {
        const int slot = (it & 7) * 8192;
        prefetch(slot);
        __builtin_amdgcn_sched_barrier(0);
        softmax();
        __builtin_amdgcn_sched_barrier(0);
        if (sync == 2) __builtin_amdgcn_s_barrier();
        burst(slot, 0, false);
        __builtin_amdgcn_sched_barrier(0);
        if (sync != 0) __builtin_amdgcn_s_barrier();
      }
    } else {                                      // MFMAs first, softmax second
      prefetch(0);
      for (int it = 0; it < iters; it++) {
        burst((it & 7) * 8192, 0, false);
        __builtin_amdgcn_sched_barrier(0);
        if (sync == 2) __builtin_amdgcn_s_barrier();
        softmax();
        __builtin_amdgcn_sched_barrier(0);
        prefetch(((it + 1) & 7) * 8192);
        __builtin_amdgcn_sched_barrier(0);
        if (sync != 0) __builtin_amdgcn_s_barrier();
      }
    }
  }
  const long long t1 = clock64();
  float acc = l_run + m_run;
  for (int d = 0; d < 4; d++) for (int r = 0; r < 16; r++) acc += o[d][r] + sprev[r];
  out[blockIdx.x * 512 + threadIdx.x] = acc;
  if (lane == 0) cyc[blockIdx.x * 8 + wave] = t1 - t0;
}

static void run(const char* name, int roleA, int roleB, int sync) {
  const int nblk = 256, iters = 2000;
  float* out; long long* cyc;
  CK(hipMalloc(&out, nblk * 512 * 4)); CK(hipMalloc(&cyc, nblk * 8 * 8));
  CK(hipFuncSetAttribute((const void*)k_mix, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms = 0;
  for (int rep = 0; rep < 3; rep++) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(k_mix, dim3(nblk), dim3(512), 131072, 0, out, cyc, iters, roleA, roleB, sync);
    CK(hipEventRecord(e1)); CK(hipDeviceSynchronize()); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  long long h[8]; CK(hipMemcpy(h, cyc, 64, hipMemcpyDeviceToHost));
  printf("%-58s waves 0-3 %5.0f ticks/iter, waves 4-7 %5.0f ticks/iter, kernel %.3f ms\n", name, (double)h[0] / iters, (double)h[4] / iters, ms);
  CK(hipFree(out)); CK(hipFree(cyc));
}

int main() {
  run("MFMA bursts alone (one wave per SIMD)", MFMA, IDLE, 0);
  run("softmax alone (one wave per SIMD)", SOFTMAX, IDLE, 0);
  run("MFMA + MFMA", MFMA, MFMA, 0);
  run("softmax + softmax", SOFTMAX, SOFTMAX, 0);
  run("MFMA on waves 0-3, softmax on waves 4-7", MFMA, SOFTMAX, 0);
  run("softmax on waves 0-3, MFMA on waves 4-7", SOFTMAX, MFMA, 0);
  run("alternating as the kernel does, no barrier", ALTERNATE, ALTERNATE, 0);
  run("alternating as the kernel does, one barrier per step", ALTERNATE, ALTERNATE, 1);
  run("alternating as the kernel does, barrier per half step", ALTERNATE, ALTERNATE, 2);
  return 0;
}
