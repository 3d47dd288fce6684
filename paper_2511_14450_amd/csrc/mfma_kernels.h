// Host-side launchers of the MFMA path (bf16 stages with head_dim 128).
#pragma once

#include "mfma_common.h"

namespace hyp {

enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATEUP = 2 };
enum { EPI_STORE = 0, EPI_SWIGLU = 1, EPI_QKV = 2, EPI_RESID = 3 };

// What the epilogue of a prefill GEMM needs besides its output; fields an epilogue does
// not use stay null.
struct GemmEpilogue {
  // EPI_QKV
  bf16_t *Kc = nullptr, *Vc = nullptr;  // caches of the layer
  CacheGeom geom = {};
  int qd = 0, kvd = 0;
  const float *cos_tab = nullptr, *sin_tab = nullptr;  // [position][64]
  const int *row_pos = nullptr, *row_req = nullptr;    // per internal row
  // EPI_QKV, EPI_SWIGLU: RMS Norm factor of every input row (the rows carry the gain only)
  const float *rstd = nullptr;
  // EPI_RESID: residual stream A(T', N), gains of the following norm, padding map,
  // sums of squares out [N / 64][T']
  float *xres = nullptr;
  const bf16_t *gain = nullptr;
  const int *row_ext = nullptr;
  float *ssq_part = nullptr;
  // any epilogue: scratch for GEMMs whose K loop is split across workgroups (few output tiles)
  float *split_ws = nullptr;          // mfma_gemm_split_ws_bytes()
  unsigned *split_counters = nullptr;  // kGemmSplitMaxTiles, zero between launches
};

constexpr int kGemmSplitMaxTiles = 255;  // GEMMs with at least a round of output tiles are never split
size_t mfma_gemm_split_ws_bytes();

// dst = P(N, K) of the row-permuted concatenation [src0; src1; src2]
hipError_t mfma_pack_weight(const bf16_t *src0, const bf16_t *src1, const bf16_t *src2, int rows0,
                            int rows1, bf16_t *dst, int N, int K, int mode, int I, hipStream_t s);

// first block's input: x = hidden_in (external rows) -> residual A(T', H), y' = x * gain -> P(T', H), rstd
hipError_t mfma_prefill_begin(const bf16_t *hidden_in, float *xres, const bf16_t *gain, bf16_t *y, float *rstd,
                              const int *row_ext, int rows, int H, float eps, hipStream_t s);
// stage output: hidden_out (external rows) = residual + delta
hipError_t mfma_prefill_end(const float *xres, const bf16_t *delta_bf, bf16_t *hidden_out, const int *row_ext,
                            int rows, int H, hipStream_t s);
// rstd[row] from the per-group sums of squares of EPI_RESID
hipError_t mfma_rstd(const float *ssq_part, float *rstd, const int *row_ext, int rows, int H, float eps, hipStream_t s);

hipError_t mfma_gemm_init();
// out^T[N, rows] = W[N,K] X[rows,K]^T with the epilogue `epi`; rows % 32 == 0,
// N % 256 == 0, K % 32 == 0, K >= 128
// `cls` (a hyp_kernel_class_t) names the GEMM of the block; it selects a kernel symbol, not behaviour
hipError_t mfma_gemm(int epi, int cls, const bf16_t *X, const bf16_t *W, int rows, int N, int K, bf16_t *out,
                     int out_K, const GemmEpilogue &ep, hipStream_t s);

// Causal GQA attention over the prompt (flash-style, scores never stored).
//   q P(rows, nq*128) ; caches of the layer ; out P(rows, nq*128)
//   work items: (request, first internal row, query blocks) per 64-row query tile
struct PrefillTile { int req, row0, qblk0; };  // qblk0: index of the tile's first 32-row block in the request
hipError_t mfma_attn_init();  // kernel attributes, once per process and device
hipError_t mfma_attn_prefill(const bf16_t *q, const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom,
                             bf16_t *out, const PrefillTile *tiles, int n_tiles, const int *req_len,
                             int nq, int nkv, hipStream_t s);

// ------------------------------------------------------------------ decode
enum { DEC_QKV = 0, DEC_SWIGLU = 1, DEC_RESID = 2, DEC_FINAL = 3 };

// One skinny GEMM of a decode step, sum[token, n] = W[n, :] . x[token, :], with
// its consumer fused in (see k_dec_gemv).  Fields a given epilogue does not use
// stay null / 0.
// how a skinny GEMM is cut into workgroups (see mfma_gemv_plan)
struct GemvPlan { int fbw = 2, nw = 4, ksplit = 1, tail = 1; };  // tail: how many times finer the row groups of a thin second round are cut

struct DecGemv {
  const bf16_t *W = nullptr, *x = nullptr;  // P(N, K), P(32, K)
  float *partial = nullptr;                 // partial sums of the K slices, mfma_gemv_partial_floats(plan, N, K) floats
  unsigned *counters = nullptr;             // [N / 32], zero between launches
  int N = 0, K = 0, batch = 0;
  GemvPlan plan;                            // plan.fbw also sets the granularity of ssq_out (sums of squares per 32 or 64 rows)
  size_t partial_floats = 0;                // room behind `partial`
  const float *ssq_in = nullptr;            // [n_ssq][32] sums of squares of the normalised input
  int n_ssq = 0;
  float eps = 0.f;
  const int *lens = nullptr;
  const float *cos_tab = nullptr, *sin_tab = nullptr;
  bf16_t *qdec = nullptr, *Kc = nullptr, *Vc = nullptr;
  CacheGeom geom = {};
  int nq = 0, nkv = 0;
  bf16_t *m_out = nullptr;
  int I = 0;
  float *xres = nullptr;
  const bf16_t *gain = nullptr;
  bf16_t *y_out = nullptr;
  float *ssq_out = nullptr;
  bf16_t *hidden_out = nullptr;
  int H = 0;
  int *lens_advance = nullptr;  // DEC_FINAL: lengths to increment at the end of the step
};
hipError_t mfma_dec_gemv(int epi, int cls, const DecGemv &a, hipStream_t s);  // cls: as for mfma_gemm
GemvPlan mfma_gemv_plan(int cls, int N, int K, int batch);  // cls: HYP_K_GEMV_*
size_t mfma_gemv_partial_floats(const GemvPlan &plan, int N, int K);
hipError_t mfma_gemv_init();  // kernel attributes, once per process and device
// x = hidden_in ; xres = x ; y' = x * gain -> P(32, H) ; ssq_out[H/64][32]
hipError_t mfma_dec_begin(const bf16_t *hidden_in, float *xres, const bf16_t *gain, bf16_t *y_out, float *ssq_out,
                          int H, int batch, hipStream_t s);

// split-KV decode attention + fixed-order merge; out row b of P(32, nq*128)
hipError_t mfma_attn_decode(const bf16_t *qdec, const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom,
                            const int *lens, float *part, bf16_t *out, int nq, int nkv, int batch,
                            int max_chunks, int chunk_keys, hipStream_t s);
size_t mfma_attn_decode_part_floats(int nq, int batch, int max_chunks);
// keys per decode-attention chunk (one wave each, one wave per SIMD): the largest power-of-two
// multiple of 128 up to 1024 that still gives the longest context about 512 waves over all
// (request, KV head) pairs - chunks of 256 for 8 x 10 pairs at 2K keys, 1024 for 32 x 10
// pairs at 1K - 4K and for 8 x 10 pairs at 9K (measured over 128 .. 1408 keys per chunk:
// fewer, longer waves beat more rounds of short ones until a wave's own serial time shows),
// doubled until a context has at most 64 chunks
inline int mfma_decode_chunk_keys(int max_seq, int heads_in_flight) {
  int c = 1024;
  while (c > 128 && (long)heads_in_flight * ((max_seq + c - 1) / c) < 512) c /= 2;
  while ((max_seq + c - 1) / c > 64) c *= 2;
  return c;
}
// cache -> plain [len, nkv*128] rows
hipError_t mfma_export_kv(const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom, bf16_t *k_out,
                          bf16_t *v_out, int request, int len, int nkv, hipStream_t s);
hipError_t mfma_fill_zero(void *p, size_t bytes, hipStream_t s);

}  // namespace hyp
