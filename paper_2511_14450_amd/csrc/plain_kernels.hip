// Shape-generic HIP kernels of the decoder block (Sec. III-A of the paper):
// fp32 arithmetic on float or bf16 storage.  They are the whole fp32 path and
// serve bf16 stages whose shape the MFMA kernels do not cover.
#include "common.h"

namespace hyp {

namespace {

constexpr int kWave = 64;

__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

template <typename T>
__global__ void k_load_hidden(const T *__restrict__ in, float *__restrict__ xres, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) xres[i] = load_f32(in + i);
}

template <typename T>
__global__ void k_store_hidden(const float *__restrict__ xres, T *__restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) store_f32(out + i, xres[i]);
}

// one 256-thread block per row: y = x * rsqrt(mean(x^2) + eps) * g
template <typename T>
__global__ void __launch_bounds__(256) k_rmsnorm(const float *__restrict__ xres,
                                                 const T *__restrict__ g, T *__restrict__ y, int H,
                                                 float eps) {
  __shared__ float part[4];
  const float *x = xres + (size_t)blockIdx.x * H;
  float ss = 0.f;
  for (int i = threadIdx.x; i < H; i += 256) ss += x[i] * x[i];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = part[0] + part[1] + part[2] + part[3];
  float r = 1.0f / sqrtf(tot / (float)H + eps);
  T *yr = y + (size_t)blockIdx.x * H;
  for (int i = threadIdx.x; i < H; i += 256) store_f32(yr + i, x[i] * r * load_f32(g + i));
}

// C[M,N] (+)= A[M,K] B[N,K]^T, 64x64 tile, 16-deep LDS stages, 4x4 per thread
template <typename T, typename OutT>
__global__ void __launch_bounds__(256) k_gemm_nt(const T *__restrict__ A, const T *__restrict__ B,
                                                 OutT *__restrict__ C, int M, int N, int K,
                                                 int accumulate) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int e = threadIdx.x; e < 64 * 16; e += 256) {
      int r = e >> 4, kk = e & 15;
      int gm = m0 + r, gn = n0 + r, gk = k0 + kk;
      As[kk][r] = (gm < M && gk < K) ? load_f32(A + (size_t)gm * K + gk) : 0.f;
      Bs[kk][r] = (gn < N && gk < K) ? load_f32(B + (size_t)gn * K + gk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
      for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      OutT *c = C + (size_t)gm * N + gn;
      float v = acc[i][j];
      if (accumulate) v += load_f32(c);
      store_f32(c, v);
    }
  }
}

// one block per token: rotate q heads in place, rotate k heads into the cache,
// copy v heads into the cache
template <typename T>
__global__ void __launch_bounds__(256) k_rope_cache(T *__restrict__ qkv,
                                                    const int *__restrict__ tok_req,
                                                    const int *__restrict__ tok_pos,
                                                    const float *__restrict__ cos_tab,
                                                    const float *__restrict__ sin_tab,
                                                    T *__restrict__ Kc, T *__restrict__ Vc, Dims dm) {
  int t = blockIdx.x;
  int req = tok_req[t], pos = tok_pos[t];
  int half = dm.d / 2;
  int ld = dm.qd + 2 * dm.kvd;
  T *row = qkv + (size_t)t * ld;
  const float *ct = cos_tab + (size_t)pos * half, *st = sin_tab + (size_t)pos * half;
  for (int e = threadIdx.x; e < dm.nq * half; e += 256) {
    int h = e / half, i = e % half;
    T *p = row + h * dm.d;
    float a = load_f32(p + i), b = load_f32(p + i + half);
    float c = ct[i], s = st[i];
    store_f32(p + i, a * c - b * s);
    store_f32(p + i + half, b * c + a * s);
  }
  for (int e = threadIdx.x; e < dm.nkv * half; e += 256) {
    int h = e / half, i = e % half;
    const T *p = row + dm.qd + h * dm.d;
    T *kdst = Kc + (((size_t)req * dm.nkv + h) * dm.max_seq + pos) * dm.d;
    float a = load_f32(p + i), b = load_f32(p + i + half);
    float c = ct[i], s = st[i];
    store_f32(kdst + i, a * c - b * s);
    store_f32(kdst + i + half, b * c + a * s);
  }
  for (int e = threadIdx.x; e < dm.kvd; e += 256) {
    int h = e / dm.d, i = e % dm.d;
    Vc[(((size_t)req * dm.nkv + h) * dm.max_seq + pos) * dm.d + i] = row[dm.qd + dm.kvd + e];
  }
}

// one wave per (token, query head); keys in chunks of kChunk with a running
// (max, sum, accumulator) so that any context length fits
constexpr int kChunk = 1024;
constexpr int kMaxDimPerLane = 4;  // head_dim <= 256

template <typename T>
__global__ void __launch_bounds__(64) k_attention(const T *__restrict__ qkv,
                                                  const int *__restrict__ tok_req,
                                                  const int *__restrict__ tok_pos,
                                                  const T *__restrict__ Kc, const T *__restrict__ Vc,
                                                  T *__restrict__ out, Dims dm) {
  __shared__ float q_s[256];
  __shared__ float sc[kChunk];
  int t = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  int req = tok_req[t], nkeys = tok_pos[t] + 1;
  int kh = h / (dm.nq / dm.nkv);
  int ld = dm.qd + 2 * dm.kvd;
  float scale = 1.0f / sqrtf((float)dm.d);
  for (int i = lane; i < dm.d; i += 64) q_s[i] = load_f32(qkv + (size_t)t * ld + h * dm.d + i);
  __syncthreads();
  const T *Kh = Kc + ((size_t)req * dm.nkv + kh) * dm.max_seq * dm.d;
  const T *Vh = Vc + ((size_t)req * dm.nkv + kh) * dm.max_seq * dm.d;
  float m_run = -INFINITY, l_run = 0.f;
  float acc[kMaxDimPerLane] = {0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < nkeys; c0 += kChunk) {
    int n = min(kChunk, nkeys - c0);
    float lmax = -INFINITY;
    for (int j = lane; j < n; j += 64) {
      const T *kr = Kh + (size_t)(c0 + j) * dm.d;
      float s = 0.f;
      for (int i = 0; i < dm.d; ++i) s = fmaf(q_s[i], load_f32(kr + i), s);
      s *= scale;
      sc[j] = s;
      lmax = fmaxf(lmax, s);
    }
    float m_new = fmaxf(m_run, wave_max(lmax));
    float lsum = 0.f;
    for (int j = lane; j < n; j += 64) {
      float p = expf(sc[j] - m_new);
      sc[j] = p;
      lsum += p;
    }
    lsum = wave_sum(lsum);
    float corr = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    l_run = l_run * corr + lsum;
    m_run = m_new;
    __syncthreads();
    for (int c = 0; c < kMaxDimPerLane; ++c) {
      int dim = lane + 64 * c;
      if (dim >= dm.d) break;
      float a = acc[c] * corr;
      for (int j = 0; j < n; ++j) a = fmaf(sc[j], load_f32(Vh + (size_t)(c0 + j) * dm.d + dim), a);
      acc[c] = a;
    }
    __syncthreads();
  }
  for (int c = 0; c < kMaxDimPerLane; ++c) {
    int dim = lane + 64 * c;
    if (dim >= dm.d) break;
    store_f32(out + (size_t)t * dm.qd + h * dm.d + dim, acc[c] / l_run);
  }
}

template <typename T>
__global__ void k_swiglu(const T *__restrict__ gu, T *__restrict__ m, int rows, int I) {
  size_t n = (size_t)rows * I;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    size_t r = i / I, c = i % I;
    float g = load_f32(gu + r * 2 * I + c), u = load_f32(gu + r * 2 * I + I + c);
    store_f32(m + i, g / (1.0f + expf(-g)) * u);
  }
}

__global__ void k_advance_lens(int *lens, int batch) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < batch) lens[i] += 1;
}

template <typename T>
__global__ void k_export_kv(const T *__restrict__ Kc, const T *__restrict__ Vc, T *__restrict__ k_out,
                            T *__restrict__ v_out, int request, int len, Dims dm) {
  size_t n = (size_t)len * dm.kvd;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int pos = (int)(i / dm.kvd), e = (int)(i % dm.kvd);
    int h = e / dm.d, dd = e % dm.d;
    size_t src = (((size_t)request * dm.nkv + h) * dm.max_seq + pos) * dm.d + dd;
    k_out[i] = Kc[src];
    v_out[i] = Vc[src];
  }
}

inline int grid_for(size_t n, int block) {
  size_t g = (n + block - 1) / block;
  if (g > 65536) g = 65536;
  if (g < 1) g = 1;
  return (int)g;
}

}  // namespace

template <typename T>
hipError_t plain_load_hidden(const T *in, float *xres, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  k_load_hidden<T><<<grid_for(n, 256), 256, 0, s>>>(in, xres, n);
  return hipGetLastError();
}
template <typename T>
hipError_t plain_store_hidden(const float *xres, T *out, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  k_store_hidden<T><<<grid_for(n, 256), 256, 0, s>>>(xres, out, n);
  return hipGetLastError();
}
template <typename T>
hipError_t plain_rmsnorm(const float *xres, const T *g, T *y, int rows, int H, float eps,
                         hipStream_t s) {
  if (rows == 0) return hipSuccess;
  k_rmsnorm<T><<<rows, 256, 0, s>>>(xres, g, y, H, eps);
  return hipGetLastError();
}
template <typename T, typename OutT>
hipError_t plain_gemm_nt(const T *A, const T *B, OutT *C, int M, int N, int K, bool accumulate,
                         hipStream_t s) {
  if (M == 0 || N == 0) return hipSuccess;
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  k_gemm_nt<T, OutT><<<grid, 256, 0, s>>>(A, B, C, M, N, K, accumulate ? 1 : 0);
  return hipGetLastError();
}
template <typename T>
hipError_t plain_rope_cache(T *qkv, const int *tok_req, const int *tok_pos, const float *cos_tab,
                            const float *sin_tab, T *Kc, T *Vc, int rows, const Dims &dm,
                            hipStream_t s) {
  if (rows == 0) return hipSuccess;
  k_rope_cache<T><<<rows, 256, 0, s>>>(qkv, tok_req, tok_pos, cos_tab, sin_tab, Kc, Vc, dm);
  return hipGetLastError();
}
template <typename T>
hipError_t plain_attention(const T *qkv, const int *tok_req, const int *tok_pos, const T *Kc,
                           const T *Vc, T *out, int rows, const Dims &dm, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  // grid.x carries the token index (up to 2^31-1), grid.y the head
  k_attention<T><<<dim3(rows, dm.nq), 64, 0, s>>>(qkv, tok_req, tok_pos, Kc, Vc, out, dm);
  return hipGetLastError();
}
template <typename T>
hipError_t plain_swiglu(const T *gu, T *m, int rows, int I, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  k_swiglu<T><<<grid_for((size_t)rows * I, 256), 256, 0, s>>>(gu, m, rows, I);
  return hipGetLastError();
}
hipError_t advance_lens(int *lens, int batch, hipStream_t s) {
  k_advance_lens<<<(batch + 63) / 64, 64, 0, s>>>(lens, batch);
  return hipGetLastError();
}
template <typename T>
hipError_t plain_export_kv(const T *Kc, const T *Vc, T *k_out, T *v_out, int request, int len,
                           const Dims &dm, hipStream_t s) {
  if (len == 0) return hipSuccess;
  k_export_kv<T><<<grid_for((size_t)len * dm.kvd, 256), 256, 0, s>>>(Kc, Vc, k_out, v_out, request,
                                                                    len, dm);
  return hipGetLastError();
}

#define HYP_INSTANTIATE(T)                                                                          \
  template hipError_t plain_load_hidden<T>(const T *, float *, size_t, hipStream_t);                \
  template hipError_t plain_store_hidden<T>(const float *, T *, size_t, hipStream_t);               \
  template hipError_t plain_rmsnorm<T>(const float *, const T *, T *, int, int, float, hipStream_t); \
  template hipError_t plain_gemm_nt<T, T>(const T *, const T *, T *, int, int, int, bool,           \
                                          hipStream_t);                                             \
  template hipError_t plain_rope_cache<T>(T *, const int *, const int *, const float *,             \
                                          const float *, T *, T *, int, const Dims &, hipStream_t); \
  template hipError_t plain_attention<T>(const T *, const int *, const int *, const T *, const T *, \
                                         T *, int, const Dims &, hipStream_t);                      \
  template hipError_t plain_swiglu<T>(const T *, T *, int, int, hipStream_t);                       \
  template hipError_t plain_export_kv<T>(const T *, const T *, T *, T *, int, int, const Dims &,    \
                                         hipStream_t);
HYP_INSTANTIATE(float)
HYP_INSTANTIATE(bf16_t)
template hipError_t plain_gemm_nt<bf16_t, float>(const bf16_t *, const bf16_t *, float *, int, int,
                                                 int, bool, hipStream_t);

}  // namespace hyp
