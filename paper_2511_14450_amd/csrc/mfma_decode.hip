// Decode-step kernels of the MFMA path: the weight-streaming skinny GEMM
// (<= 32 tokens against a [N, K] matrix, bandwidth-bound) and the small kernels
// that finish its split-K partial sums (RoPE + cache append, SwiGLU), for the
// KV-cached generation phase of the decoder block of Sec. III-A.
#include "mfma_common.h"
#include "mfma_kernels.h"

namespace hyp {

namespace {

// ----------------------------------------------------------------------------
// partial[ks][token][n] = sum over the K slice ks of W[n, k] x[token, k]
// W = P(N, K): the 1 KiB tiles of one 32-row block are contiguous along K, and a
// tile is the MFMA A fragment as it stands, so every wave streams its slice
// with 1 KiB fully coalesced loads straight into registers (no LDS on the way
// in).  x = P(32, K) is tiny and stays in L2.  A workgroup owns FBW feature
// blocks; its NW waves split the K slice and are reduced through LDS in wave
// order (deterministic).
// ----------------------------------------------------------------------------
constexpr int FBW = 2, NW = 8, UNROLL = 5;

__global__ void __launch_bounds__(NW * 64) k_gemv(const bf16_t *__restrict__ W,
                                                  const bf16_t *__restrict__ x,
                                                  float *__restrict__ partial, int N, int KT,
                                                  int tiles_per_wave, int batch) {
  extern __shared__ __attribute__((aligned(16))) float red_raw[];
  float (*red)[FBW][16][64] = (float (*)[FBW][16][64])red_raw;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int fb0 = blockIdx.x * FBW, ks = blockIdx.y;
  const int kt0 = (ks * NW + wave) * tiles_per_wave;
  f32x16_t acc[FBW];
#pragma unroll
  for (int i = 0; i < FBW; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  const bf16_t *xp = x + (size_t)kt0 * kTileElems + lane * 8;
  const bf16_t *wp[FBW];
#pragma unroll
  for (int i = 0; i < FBW; ++i) wp[i] = W + ((size_t)(fb0 + i) * KT + kt0) * kTileElems + lane * 8;
  int t = 0;
  for (; t + UNROLL <= tiles_per_wave; t += UNROLL) {
    bf16x8_t xf[UNROLL], wf[FBW][UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
      for (int i = 0; i < FBW; ++i) wf[i][u] = __builtin_nontemporal_load((const bf16x8_t *)(wp[i] + (size_t)(t + u) * kTileElems));
      xf[u] = *(const bf16x8_t *)(xp + (size_t)(t + u) * kTileElems);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int i = 0; i < FBW; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i][u], xf[u], acc[i], 0, 0, 0);
  }
  for (; t < tiles_per_wave; ++t) {
    bf16x8_t xf = *(const bf16x8_t *)(xp + (size_t)t * kTileElems);
#pragma unroll
    for (int i = 0; i < FBW; ++i) {
      bf16x8_t wf = __builtin_nontemporal_load((const bf16x8_t *)(wp[i] + (size_t)t * kTileElems));
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[i], 0, 0, 0);
    }
  }
#pragma unroll
  for (int i = 0; i < FBW; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][i][r][lane] = acc[i][r];
  __syncthreads();
  // thread -> (token, feature f of the FBW*32 this workgroup owns): consecutive threads
  // write consecutive features of one token row
  for (int idx = threadIdx.x; idx < FBW * 32 * 32; idx += NW * 64) {
    int f = idx % (FBW * 32), token = idx / (FBW * 32);
    if (token >= batch) break;
    int i = f >> 5, fl = f & 31;
    int r = ((fl >> 3) << 2) + (fl & 3), l = (((fl >> 2) & 1) << 5) + token;
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += red[w][i][r][l];
    partial[((size_t)ks * 32 + token) * N + fb0 * 32 + f] = sum;
  }
}

__device__ inline int packed_row_qkv(int head, int d) {
  return head * 128 + ((d & 63) >> 5) * 64 + (d >> 6) * 32 + (d & 31);
}

// grid (batch, nq + 2 nkv), 64 threads: thread i owns the RoPE pair (i, i + 64)
__global__ void __launch_bounds__(64) k_dec_qkv_finish(const float *__restrict__ partial, int ksplit,
                                                       int N, const int *__restrict__ lens,
                                                       const float *__restrict__ cos_tab,
                                                       const float *__restrict__ sin_tab,
                                                       bf16_t *__restrict__ qdec, bf16_t *__restrict__ Kc,
                                                       bf16_t *__restrict__ Vc, CacheGeom geom, int nq,
                                                       int nkv) {
  const int b = blockIdx.x, head = blockIdx.y, i = threadIdx.x;
  const int pos = lens[b];
  float a = 0.f, c = 0.f;
  int r0 = packed_row_qkv(head, i), r1 = packed_row_qkv(head, i + 64);
  for (int s = 0; s < ksplit; ++s) {
    a += partial[((size_t)s * 32 + b) * N + r0];
    c += partial[((size_t)s * 32 + b) * N + r1];
  }
  if (head < nq + nkv) {
    float cs = cos_tab[(size_t)pos * 64 + i], sn = sin_tab[(size_t)pos * 64 + i];
    float lo = a * cs - c * sn, hi = c * cs + a * sn;
    if (head < nq) {
      int G = nq / nkv;
      bf16_t *dst = qdec + ((size_t)b * nkv + head / G) * (32 * 128);
      dst[frag_offset(head % G, i, 128)] = f2bf_dev(lo);
      dst[frag_offset(head % G, i + 64, 128)] = f2bf_dev(hi);
    } else {
      bf16_t *dst = Kc + geom.off(b, head - nq, pos >> 5);
      dst[frag_offset(pos & 31, i, 128)] = f2bf_dev(lo);
      dst[frag_offset(pos & 31, i + 64, 128)] = f2bf_dev(hi);
    }
  } else {
    bf16_t *dst = Vc + geom.off(b, head - nq - nkv, pos >> 5);
    int m, khh;
    int e = vtile_slot_of_key(pos & 31, &m, &khh);
    dst[(size_t)(m * 4 + (i >> 5)) * kTileElems + (khh * 32 + (i & 31)) * 8 + e] = f2bf_dev(a);
    dst[(size_t)(m * 4 + ((i + 64) >> 5)) * kTileElems + (khh * 32 + (i & 31)) * 8 + e] = f2bf_dev(c);
  }
}

// grid (I / 256, batch), 256 threads: one FFN feature per thread
__global__ void __launch_bounds__(256) k_dec_swiglu(const float *__restrict__ partial, int ksplit, int I,
                                                    bf16_t *__restrict__ m) {
  const int f = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
  const int N = 2 * I;
  int rg = (f >> 7) * 256 + ((f & 127) >> 5) * 64 + (f & 31), ru = rg + 32;
  float g = 0.f, u = 0.f;
  for (int s = 0; s < ksplit; ++s) {
    g += partial[((size_t)s * 32 + b) * N + rg];
    u += partial[((size_t)s * 32 + b) * N + ru];
  }
  m[frag_offset(b, f, I)] = f2bf_dev(g / (1.0f + __expf(-g)) * u);
}

__global__ void k_export_kv(const bf16_t *__restrict__ Kc, const bf16_t *__restrict__ Vc, CacheGeom geom,
                            bf16_t *__restrict__ k_out, bf16_t *__restrict__ v_out, int request, int len,
                            int nkv) {
  size_t n = (size_t)len * nkv * 128;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int pos = (int)(i / (nkv * 128)), e = (int)(i % (nkv * 128));
    int h = e >> 7, d = e & 127;
    size_t blk = geom.off(request, h, pos >> 5);
    k_out[i] = Kc[blk + frag_offset(pos & 31, d, 128)];
    int m, khh;
    int slot = vtile_slot_of_key(pos & 31, &m, &khh);
    v_out[i] = Vc[blk + (size_t)(m * 4 + (d >> 5)) * kTileElems + (khh * 32 + (d & 31)) * 8 + slot];
  }
}

__global__ void k_fill_zero(uint4 *p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  uint4 z = {0, 0, 0, 0};
  for (; i < n16; i += stride) p[i] = z;
}

}  // namespace

constexpr int GEMV_LDS = NW * FBW * 16 * 64 * 4;

hipError_t mfma_gemv_init() {
  return hipFuncSetAttribute((const void *)k_gemv, hipFuncAttributeMaxDynamicSharedMemorySize, GEMV_LDS);
}

hipError_t mfma_gemv(const bf16_t *W, const bf16_t *x, float *partial, int N, int K, int ksplit,
                     int batch, hipStream_t s) {
  int KT = K / 16;
  int tiles_per_wave = KT / (ksplit * NW);
  k_gemv<<<dim3(N / (32 * FBW), ksplit), NW * 64, GEMV_LDS, s>>>(W, x, partial, N, KT, tiles_per_wave, batch);
  return hipGetLastError();
}

// K slices across workgroups: enough workgroups to fill the chip, few enough
// that the fp32 partial sums stay a small fraction of the weight bytes
int mfma_gemv_ksplit(int N, int K) {
  int KT = K / 16, groups = N / (32 * FBW);
  int want = (1024 + groups - 1) / groups;
  int best = 1;
  for (int ks = 1; ks <= want; ++ks)
    if (KT % (ks * NW) == 0) best = ks;
  return best;
}

hipError_t mfma_dec_qkv_finish(const float *partial, int ksplit, int N, const int *lens,
                               const float *cos_tab, const float *sin_tab, bf16_t *qdec, bf16_t *Kc,
                               bf16_t *Vc, CacheGeom geom, int nq, int nkv, int batch, hipStream_t s) {
  k_dec_qkv_finish<<<dim3(batch, nq + 2 * nkv), 64, 0, s>>>(partial, ksplit, N, lens, cos_tab, sin_tab, qdec, Kc, Vc, geom, nq, nkv);
  return hipGetLastError();
}

hipError_t mfma_dec_swiglu(const float *partial, int ksplit, int I, bf16_t *m, int batch, hipStream_t s) {
  k_dec_swiglu<<<dim3(I / 256, batch), 256, 0, s>>>(partial, ksplit, I, m);
  return hipGetLastError();
}

hipError_t mfma_export_kv(const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom, bf16_t *k_out,
                          bf16_t *v_out, int request, int len, int nkv, hipStream_t s) {
  if (len == 0) return hipSuccess;
  size_t n = (size_t)len * nkv * 128;
  int grid = (int)((n + 255) / 256 > 4096 ? 4096 : (n + 255) / 256);
  k_export_kv<<<grid, 256, 0, s>>>(Kc, Vc, geom, k_out, v_out, request, len, nkv);
  return hipGetLastError();
}

hipError_t mfma_fill_zero(void *p, size_t bytes, hipStream_t s) {
  size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  int grid = (int)((n16 + 255) / 256 > 16384 ? 16384 : (n16 + 255) / 256);
  k_fill_zero<<<grid, 256, 0, s>>>((uint4 *)p, n16);
  return hipGetLastError();
}

}  // namespace hyp
