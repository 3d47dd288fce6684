// Measured ceilings of the device, to set beside the datasheet peaks: what the
// MFMA pipes deliver from registers alone, and what a plain streaming read of HBM
// delivers.  Both matter here: with Gaussian bf16 operands the chip clocks down
// under MFMA load, and a pure read stream stays below the nominal HBM rate.
#include <stdio.h>

#include <string>

#include "mfma_common.h"

namespace hyp {
namespace {

// independent accumulator chains per wave, operands loaded once: no LDS, no memory traffic.
// SHAPE 16: v_mfma_f32_16x16x32_bf16 (the prefill GEMM's), 32: v_mfma_f32_32x32x16_bf16 (the attention kernels').
// Both do the same FLOPs per pass of the inner loop.
template <int SHAPE>
__global__ void __launch_bounds__(256) k_mfma_only(const bf16x8_t *__restrict__ src, float *__restrict__ out, int iters) {
  bf16x8_t a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = src[(threadIdx.x * 8 + i) & 4095];
    b[i] = src[(threadIdx.x * 8 + 4 + i) & 4095];
  }
  float s = 0.f;
  if constexpr (SHAPE == 32) {
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[(i + u) & 3], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][r];
  } else {
    f32x4_t acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[((i >> 2) + u) & 3], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) s += acc[i][r];
  }
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// operands: N(0,1) rounded to bf16 (Box-Muller on a counter hash), or the constant 1.0
__global__ void k_fill_operands(bf16_t *dst, int n, int gaussian) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  unsigned h = (unsigned)i * 2654435761u;
  h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
  unsigned g = h * 3266489917u; g ^= g >> 16;
  float u1 = ((h >> 8) + 1.0f) * (1.0f / 16777217.0f), u2 = (g >> 8) * (1.0f / 16777216.0f);
  float z = sqrtf(-2.0f * logf(u1)) * cosf(6.2831853f * u2);
  dst[i] = f32_to_bf16(gaussian ? z : 1.0f);
}

// Every workgroup owns a contiguous span and reads it 4 KiB (its four waves' 1 KiB each) at a
// time, 16 such reads in flight per wave: the pattern HBM serves best here (7.2 TB/s; a
// grid-stride loop over the same buffer reaches 6.4).
__global__ void __launch_bounds__(256) k_stream_read(const f32x4_t *__restrict__ p, float *__restrict__ out, size_t n16) {
  const size_t per = n16 / 256 / gridDim.x;  // 4 KiB rows per workgroup (the rest of the buffer is left out)
  const f32x4_t *q = p + (size_t)blockIdx.x * per * 256 + threadIdx.x;
  f32x4_t a = {0.f, 0.f, 0.f, 0.f};
  size_t t = 0;
  for (; t + 16 <= per; t += 16) {
    f32x4_t v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = __builtin_nontemporal_load(q + (t + u) * 256);
#pragma unroll
    for (int u = 0; u < 16; ++u) a += v[u];
  }
  for (; t < per; ++t) a += __builtin_nontemporal_load(q + t * 256);
  if (a[0] + a[1] + a[2] + a[3] == 1.2345e-30f) out[0] = 1.f;  // keeps the loads alive
}

}  // namespace
}  // namespace hyp

using namespace hyp;

extern "C" {

hyp_status_t hyp_measure_mfma_ceiling(void *scratch, size_t scratch_bytes, int32_t mode, void *hip_stream,
                                      double *tflops_out) {
  const int gaussian = mode & 1;
  const bool shape32 = (mode & 2) != 0;
  const int n_wg = 2048, iters = 20000;
  const size_t need = 4096 * 16 + (size_t)n_wg * 256 * sizeof(float);
  if (!scratch || !tflops_out || scratch_bytes < need || (uintptr_t)scratch % 16) return HYP_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  bf16_t *src = (bf16_t *)scratch;
  float *out = (float *)((char *)scratch + 4096 * 16);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return HYP_EDEVICE;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return HYP_EDEVICE; }
  k_fill_operands<<<(4096 * 8 + 255) / 256, 256, 0, s>>>(src, 4096 * 8, gaussian);
  auto launch = [&](int n) {
    if (shape32) k_mfma_only<32><<<n_wg, 256, 0, s>>>((const bf16x8_t *)src, out, n);
    else k_mfma_only<16><<<n_wg, 256, 0, s>>>((const bf16x8_t *)src, out, n);
  };
  launch(400);  // warm-up, clocks settle
  float best = 0.f;
  hipError_t err = hipSuccess;
  for (int rep = 0; rep < 3 && err == hipSuccess; ++rep) {
    (void)hipEventRecord(e0, s);
    launch(iters);
    (void)hipEventRecord(e1, s);
    err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    double tf = (double)n_wg * 4 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12;
    if (rep > 0 && tf > best) best = (float)tf;  // sustained: skip the first timed launch
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess) return HYP_EDEVICE;
  *tflops_out = best;
  return HYP_OK;
}

hyp_status_t hyp_measure_hbm_read_ceiling(const void *buffer, size_t bytes, void *hip_stream, double *gbs_out) {
  if (!buffer || !gbs_out || bytes < ((size_t)1 << 30) || (uintptr_t)buffer % 16) return HYP_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return HYP_EDEVICE;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return HYP_EDEVICE; }
  // the flag word lives in the first 16 bytes' shadow: reuse the buffer tail as output sink
  float *sink = (float *)((char *)const_cast<void *>(buffer) + (bytes / 16 - 1) * 16);
  size_t n16 = bytes / 16 - 1;
  k_stream_read<<<8192, 256, 0, s>>>((const f32x4_t *)buffer, sink, n16);
  double best = 0;
  hipError_t err = hipSuccess;
  for (int rep = 0; rep < 3 && err == hipSuccess; ++rep) {
    (void)hipEventRecord(e0, s);
    k_stream_read<<<8192, 256, 0, s>>>((const f32x4_t *)buffer, sink, n16);
    (void)hipEventRecord(e1, s);
    err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    double gbs = (double)(n16 / 256 / 8192) * 256 * 8192 * 16 / (ms * 1e-3) / 1e9;
    if (gbs > best) best = gbs;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess) return HYP_EDEVICE;
  *gbs_out = best;
  return HYP_OK;
}

}  // extern "C"
