// Measurement helper: what the matrix pipes of this GPU sustain on nothing but bf16 MFMAs of one
// shape (v_mfma_f32_16x16x32_bf16, the attention kernels' shape, or v_mfma_f32_32x32x16_bf16) with
// caller-supplied operand data.  The published bf16 peak assumes the top clock; under matrix load
// the part is power limited and the sustained rate depends on how much the operand bits toggle
// (all-zero operands run at the top clock, normally distributed ones 20-30 % slower) and on the
// shape (16x16x32 sustains about 12 % more than 32x32x16 on normally distributed operands), so the
// attention kernel's rate is also reported against this measured ceiling.
#include <hip/hip_runtime.h>

#include "../../include/calvo.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kMfmaPerIter = 16;
constexpr int kWaves = 8;            // two waves per SIMD, as the attention kernel runs

// Every wave keeps eight A and eight B operands (taken from `tab`, 1024 x 16 bytes) and four
// accumulators and issues nothing but MFMAs; consecutive MFMAs use different accumulators.
__global__ void __launch_bounds__(64 * kWaves, 2) mfma_peak_kernel(const u32x4* tab, float* sink, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; i++) {
    a[i] = __builtin_bit_cast(bf16x8, tab[(i * 64 + lane) & 1023]);
    b[i] = __builtin_bit_cast(bf16x8, tab[(512 + i * 64 + lane) & 1023]);
  }
  f32x16 o[4];
  for (int d = 0; d < 4; d++)
    for (int r = 0; r < 16; r++) o[d][r] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < kMfmaPerIter; i++)
      o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 7], b[(i >> 1) & 7], o[i & 3], 0, 0, 0);
  }
  float acc = 0.f;
  for (int d = 0; d < 4; d++)
    for (int r = 0; r < 16; r++) acc += o[d][r];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

// The same with the 16x16x32 shape: two MFMAs for every one above (the same products per iteration),
// eight accumulator tiles, consecutive MFMAs on different accumulators.
__global__ void __launch_bounds__(64 * kWaves, 2) mfma_peak16_kernel(const u32x4* tab, float* sink, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; i++) {
    a[i] = __builtin_bit_cast(bf16x8, tab[(i * 64 + lane) & 1023]);
    b[i] = __builtin_bit_cast(bf16x8, tab[(512 + i * 64 + lane) & 1023]);
  }
  f32x4 o[8];
  for (int d = 0; d < 8; d++)
    for (int r = 0; r < 4; r++) o[d][r] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 2 * kMfmaPerIter; i++)
      o[i & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 7], b[(i >> 1) & 7], o[i & 7], 0, 0, 0);
  }
  float acc = 0.f;
  for (int d = 0; d < 8; d++)
    for (int r = 0; r < 4; r++) acc += o[d][r];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

}  // namespace

extern "C" int calvo_mfma_peak(const void* operands, void* sink, int iters, int repeats, int shape, double* tflops, double* ms_out) {
  if (!operands || !sink || iters <= 0 || iters > (1 << 20) || repeats <= 0 || repeats > 64 || !tflops) return CALVO_EINVAL;
  if (shape != CALVO_MFMA_16x16x32 && shape != CALVO_MFMA_32x32x16) return CALVO_EINVAL;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    return CALVO_EHIP;
  }
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    if (e0) (void)hipEventDestroy(e0);
    (void)hipGetLastError();
    return CALVO_EHIP;
  }
  float best = 0.f;
  int rc = CALVO_OK;
  for (int r = 0; r < repeats + 1 && rc == CALVO_OK; r++) {             // the first launch warms up
    float ms = 0.f;
    if (hipEventRecord(e0, nullptr) != hipSuccess) rc = CALVO_EHIP;
    if (shape == CALVO_MFMA_32x32x16)
      hipLaunchKernelGGL(mfma_peak_kernel, dim3(cus), dim3(64 * kWaves), 0, nullptr, (const u32x4*)operands, (float*)sink, iters);
    else
      hipLaunchKernelGGL(mfma_peak16_kernel, dim3(cus), dim3(64 * kWaves), 0, nullptr, (const u32x4*)operands, (float*)sink, iters);
    if (rc == CALVO_OK && (hipGetLastError() != hipSuccess || hipEventRecord(e1, nullptr) != hipSuccess ||
                           hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
      rc = CALVO_EHIP;
    if (rc == CALVO_OK && r > 0 && (best == 0.f || ms < best)) best = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != CALVO_OK) { (void)hipGetLastError(); return rc; }
  const double flop = (double)cus * kWaves * (double)iters * kMfmaPerIter * 32768.0;   // 32 x 32 x 16 x 2 (or 2 x 16 x 16 x 32 x 2) per wave
  *tflops = flop / ((double)best * 1e-3) / 1e12;
  if (ms_out) *ms_out = best;
  return CALVO_OK;
}
