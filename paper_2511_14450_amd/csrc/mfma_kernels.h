// Host-side launchers of the MFMA path (bf16 stages with head_dim 128).
#pragma once

#include "mfma_common.h"

namespace hyp {

enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATEUP = 2 };
enum { EPI_STORE = 0, EPI_SWIGLU = 1, EPI_QKV = 2 };

struct QkvEpilogue {
  bf16_t *Kc, *Vc;  // caches of the layer
  CacheGeom geom;
  int qd, kvd;
  const float *cos_tab, *sin_tab;  // [position][64]
  const int *row_pos, *row_req;    // per internal row
};

// dst = P(N, K) of the row-permuted concatenation [src0; src1; src2]
hipError_t mfma_pack_weight(const bf16_t *src0, const bf16_t *src1, const bf16_t *src2, int rows0,
                            int rows1, bf16_t *dst, int N, int K, int mode, int I, hipStream_t s);

hipError_t mfma_add_norm(const bf16_t *hidden_in, float *xres, const bf16_t *delta_bf,
                         const float *delta_part, int n_part, size_t part_stride, const bf16_t *gain,
                         bf16_t *y, bf16_t *hidden_out, const int *row_ext, int rows, int H, float eps,
                         bool final_mode, hipStream_t s);

hipError_t mfma_gemm_init();
hipError_t mfma_gemv_init();
// out^T[N, rows] = W[N,K] X[rows,K]^T with the epilogue `epi`; rows % 32 == 0,
// N % 256 == 0, K % 32 == 0, K >= 128
hipError_t mfma_gemm(int epi, const bf16_t *X, const bf16_t *W, int rows, int N, int K, bf16_t *out,
                     int out_K, const QkvEpilogue *qkv, hipStream_t s);

// Causal GQA attention over the prompt (flash-style, scores never stored).
//   q P(rows, nq*128) ; caches of the layer ; out P(rows, nq*128)
//   work items: (request, first internal row, query blocks) per 64-row query tile
struct PrefillTile { int req, row0, qblk0; };  // qblk0: index of the tile's first 32-row block in the request
hipError_t mfma_attn_prefill(const bf16_t *q, const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom,
                             bf16_t *out, const PrefillTile *tiles, int n_tiles, const int *req_len,
                             int nq, int nkv, hipStream_t s);

// ------------------------------------------------------------------ decode
// partial[ks][32][N] (fp32) = x[32 rows, K-slice ks] W[N, K-slice]^T, token rows < batch only
hipError_t mfma_gemv(const bf16_t *W, const bf16_t *x, float *partial, int N, int K, int ksplit,
                     int batch, hipStream_t s);
int mfma_gemv_ksplit(int N, int K);

// sum the QKV partials, rotate q and k at position lens[b], write q into the
// decode query buffer and k, v into the caches
hipError_t mfma_dec_qkv_finish(const float *partial, int ksplit, int N, const int *lens,
                               const float *cos_tab, const float *sin_tab, bf16_t *qdec, bf16_t *Kc,
                               bf16_t *Vc, CacheGeom geom, int nq, int nkv, int batch, hipStream_t s);
// split-KV decode attention + fixed-order merge; out row b of P(32, nq*128)
hipError_t mfma_attn_decode(const bf16_t *qdec, const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom,
                            const int *lens, float *part, bf16_t *out, int nq, int nkv, int batch,
                            int max_chunks, hipStream_t s);
size_t mfma_attn_decode_part_floats(int nq, int batch, int max_chunks);
constexpr int kDecodeChunkKeys = 128;
// m = silu(gate) * up from the gate/up partials -> P(32, I)
hipError_t mfma_dec_swiglu(const float *partial, int ksplit, int I, bf16_t *m, int batch, hipStream_t s);

// cache -> plain [len, nkv*128] rows
hipError_t mfma_export_kv(const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom, bf16_t *k_out,
                          bf16_t *v_out, int request, int len, int nkv, hipStream_t s);
hipError_t mfma_fill_zero(void *p, size_t bytes, hipStream_t s);

}  // namespace hyp
