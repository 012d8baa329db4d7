// Microbenchmark: issue cost of the vector instructions the attention kernels' softmax is made of,
// on gfx950.  Every wave runs a loop of 16 independent instructions of one kind (or a fixed mix of
// v_exp_f32 and multiply-adds) and times itself with s_memtime; waves w and w + 4 of a 512-thread
// workgroup share a SIMD, so a run with two roles shows how two streams share the vector ALU and
// the transcendental pipe.  The printed figure is ticks per loop iteration / 16: ticks per
// instruction for the single-kind loops, 1/16 of an iteration for the mixes (8 exp + 8, 16 or 24
// multiply-adds per iteration).  Not part of the library; build and run by hand:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         paper_2603_21257_amd/csrc/probe_valu_issue.hip -o probe_valu_issue && ./probe_valu_issue
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) _Float16 h2;
enum { FMA = 0, EXP, CVTPK, DOT2, EXPH, MAXF, PKFMAH, MOV, NOPS, P_EF, P_EFF, P_EFFF, P_GROUP, P_EEFF };
template <int OP>
__device__ inline void body(float (&x)[16], float c, int iters) {
  bf16x2 ones; ones[0] = (__bf16)1.f; ones[1] = (__bf16)1.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int r = 0; r < 16; r++) {
      if constexpr (OP == FMA) x[r] = __builtin_fmaf(x[r], c, 0.25f);
      else if constexpr (OP == EXP) x[r] = __builtin_amdgcn_exp2f(x[r]);
      else if constexpr (OP == CVTPK) { bf16x2 w; w[0] = (__bf16)x[r]; w[1] = (__bf16)x[(r + 1) & 15]; x[r] = __builtin_bit_cast(float, w); }
      else if constexpr (OP == DOT2) x[r] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x[(r + 1) & 15]), ones, x[r], false);
      else if constexpr (OP == EXPH) { _Float16 h = __builtin_bit_cast(h2, x[r])[0]; _Float16 e; asm volatile("v_exp_f16 %0, %1" : "=v"(e) : "v"(h)); h2 o; o[0] = e; o[1] = e; x[r] = __builtin_bit_cast(float, o); }
      else if constexpr (OP == MAXF) x[r] = fmaxf(x[r], x[(r + 1) & 15] );
      else if constexpr (OP == PKFMAH) { h2 a = __builtin_bit_cast(h2, x[r]); h2 b = __builtin_bit_cast(h2, c); a = a * b + b; x[r] = __builtin_bit_cast(float, a); }
      else if constexpr (OP == MOV) { asm volatile("v_mov_b32 %0, %1" : "=v"(x[r]) : "v"(x[(r + 1) & 15])); }
    }
#pragma unroll
    for (int r = 0; r < 16; r++) asm volatile("" : "+v"(x[r]));
  }
}
// mixed streams: x[0..7] carry exponentials, y[0..23] multiply-adds; all chains independent
template <int NF, bool GROUP, bool PAIRS = false>
__device__ inline void pattern(float (&x)[16], float c, int iters) {
  float y[24];
  for (int r = 0; r < 24; r++) y[r] = x[r & 15] + r;
  for (int it = 0; it < iters; it++) {
    if constexpr (GROUP) {
#pragma unroll
      for (int r = 0; r < 8; r++) x[r] = __builtin_amdgcn_exp2f(x[r]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 0; r < 8 * NF; r++) y[r] = __builtin_fmaf(y[r], c, 0.25f);
      __builtin_amdgcn_sched_barrier(0);
    } else if constexpr (PAIRS) {
#pragma unroll
      for (int r = 0; r < 8; r += 2) {
        x[r] = __builtin_amdgcn_exp2f(x[r]);
        x[r + 1] = __builtin_amdgcn_exp2f(x[r + 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < 2 * NF; f++) y[r * NF + f] = __builtin_fmaf(y[r * NF + f], c, 0.25f);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 8; r++) {
        x[r] = __builtin_amdgcn_exp2f(x[r]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < NF; f++) y[r * NF + f] = __builtin_fmaf(y[r * NF + f], c, 0.25f);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int r = 0; r < 16; r++) asm volatile("" : "+v"(x[r]));
#pragma unroll
    for (int r = 0; r < 24; r++) asm volatile("" : "+v"(y[r]));
  }
  for (int r = 0; r < 24; r++) x[r & 15] += y[r];
}
__global__ void __launch_bounds__(512, 2) k_ops(float* out, long long* cyc, int iters, int opA, int opB) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int op = wave < 4 ? opA : opB;
  float x[16];
  for (int r = 0; r < 16; r++) x[r] = 0.001f * (r + lane);
  const float c = 0.5f + 0.001f * lane;
  __syncthreads();
  const long long t0 = clock64();
  switch (op) {
    case FMA: body<FMA>(x, c, iters); break;
    case EXP: body<EXP>(x, c, iters); break;
    case CVTPK: body<CVTPK>(x, c, iters); break;
    case DOT2: body<DOT2>(x, c, iters); break;
    case EXPH: body<EXPH>(x, c, iters); break;
    case MAXF: body<MAXF>(x, c, iters); break;
    case PKFMAH: body<PKFMAH>(x, c, iters); break;
    case MOV: body<MOV>(x, c, iters); break;
    case P_EF: pattern<1, false>(x, c, iters); break;
    case P_EFF: pattern<2, false>(x, c, iters); break;
    case P_EFFF: pattern<3, false>(x, c, iters); break;
    case P_GROUP: pattern<2, true>(x, c, iters); break;
    case P_EEFF: pattern<2, false, true>(x, c, iters); break;
    default: break;
  }
  const long long t1 = clock64();
  float acc = 0.f;
  for (int r = 0; r < 16; r++) acc += x[r];
  out[blockIdx.x * 512 + threadIdx.x] = acc;
  if (lane == 0) cyc[blockIdx.x * 8 + wave] = t1 - t0;
}
static const char* names[] = {"v_fma_f32", "v_exp_f32", "v_cvt_pk_bf16_f32", "v_dot2_f32_bf16", "v_exp_f16", "v_max_f32", "v_pk_fma_f16", "v_mov_b32", "idle", "8x[exp,fma]", "8x[exp,fma,fma]", "8x[exp,3 fma]", "8 exp then 16 fma", "4x[2 exp,4 fma]"};
static void run(int a, int b) {
  const int nblk = 256, iters = 2000;
  float* out; long long* cyc;
  CK(hipMalloc(&out, nblk * 512 * 4)); CK(hipMalloc(&cyc, nblk * 8 * 8));
  for (int rep = 0; rep < 2; rep++) { hipLaunchKernelGGL(k_ops, dim3(nblk), dim3(512), 0, 0, out, cyc, iters, a, b); CK(hipDeviceSynchronize()); }
  long long h[8]; CK(hipMemcpy(h, cyc, 64, hipMemcpyDeviceToHost));
  printf("waves 0-3 %-18s %6.2f ticks/instr | waves 4-7 %-18s %6.2f ticks/instr\n", names[a], (double)h[0] / iters / 16, names[b], (double)h[4] / iters / 16);
  CK(hipFree(out)); CK(hipFree(cyc));
}
int main() {
  for (int a = 0; a < NOPS; a++) run(a, NOPS);
  for (int a = P_EF; a <= P_EEFF; a++) run(a, NOPS);
  run(P_EFF, P_EFF); run(P_GROUP, P_GROUP);
  run(EXP, EXP); run(FMA, FMA); run(EXP, FMA); run(FMA, EXP); run(EXP, CVTPK); run(EXP, DOT2); run(CVTPK, DOT2);
  return 0;
}
