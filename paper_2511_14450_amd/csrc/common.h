// Internal declarations shared by the translation units of the stage library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hyp_stage.h"

namespace hyp {

// ----------------------------------------------------------------------------
// bf16 <-> fp32 (bit patterns; round to nearest even)
// ----------------------------------------------------------------------------
typedef uint16_t bf16_t;

__host__ __device__ inline float bf16_to_f32(bf16_t v) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)v << 16;
  return c.f;
}

__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> __device__ inline float load_f32(const T *p);
template <> __device__ inline float load_f32<float>(const float *p) { return *p; }
template <> __device__ inline float load_f32<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void store_f32(T *p, float v);
template <> __device__ inline void store_f32<float>(float *p, float v) { *p = v; }
template <> __device__ inline void store_f32<bf16_t>(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// ----------------------------------------------------------------------------
// Geometry of one block, as the kernels see it
// ----------------------------------------------------------------------------
struct Dims {
  int H, nq, nkv, d, I;
  int qd, kvd;       // nq*d, nkv*d
  int max_batch, max_seq;
  float eps;
};

// ----------------------------------------------------------------------------
// Plain (shape-generic) kernels, T = float or bf16_t storage, fp32 arithmetic.
// Every launcher enqueues on `s` and returns the launch status.
// ----------------------------------------------------------------------------
template <typename T>
hipError_t plain_load_hidden(const T *in, float *xres, size_t n, hipStream_t s);
template <typename T>
hipError_t plain_store_hidden(const float *xres, T *out, size_t n, hipStream_t s);
template <typename T>
hipError_t plain_rmsnorm(const float *xres, const T *g, T *y, int rows, int H, float eps,
                         hipStream_t s);
// C[M,N] (+)= A[M,K] * B[N,K]^T ; OutT = T or float
template <typename T, typename OutT>
hipError_t plain_gemm_nt(const T *A, const T *B, OutT *C, int M, int N, int K, bool accumulate,
                         hipStream_t s);
// rotate q and k of qkv[T, qd+2kvd] in place; write k, v to the cache
// cache layout: [request][kv_head][max_seq][d]
template <typename T>
hipError_t plain_rope_cache(T *qkv, const int *tok_req, const int *tok_pos, const float *cos_tab,
                            const float *sin_tab, T *Kc, T *Vc, int rows, const Dims &dm,
                            hipStream_t s);
template <typename T>
hipError_t plain_attention(const T *qkv, const int *tok_req, const int *tok_pos, const T *Kc,
                           const T *Vc, T *out, int rows, const Dims &dm, hipStream_t s);
template <typename T>
hipError_t plain_swiglu(const T *gu, T *m, int rows, int I, hipStream_t s);
hipError_t advance_lens(int *lens, int batch, hipStream_t s);
template <typename T>
hipError_t plain_export_kv(const T *Kc, const T *Vc, T *k_out, T *v_out, int request, int len,
                           const Dims &dm, hipStream_t s);

}  // namespace hyp
