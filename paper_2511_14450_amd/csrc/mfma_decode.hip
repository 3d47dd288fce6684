// Decode-step kernels of the MFMA path: the weight-streaming skinny GEMM
// (<= 32 tokens against a [N, K] matrix, bandwidth-bound) with its consumers fused
// into the workgroup that finishes a row group (RoPE + cache append, SwiGLU,
// residual + next norm), and the kernel that opens a step, for the KV-cached
// generation phase of the decoder block of Sec. III-A.
#include "mfma_common.h"
#include "mfma_kernels.h"

namespace hyp {

namespace {

// ----------------------------------------------------------------------------
// Skinny GEMM of a decode step with its consumer fused in.
//
//   sum[token, n] = sum_k W[n, k] x[token, k]        (<= 32 tokens, W streamed once)
//
// W = P(N, K): the 1 KiB tiles of one 32-row block are contiguous along K and a
// tile is the MFMA A fragment as it stands, so every wave streams its slice
// with fully coalesced 1 KiB loads straight into registers.  x = P(32, K) is
// tiny and stays in L2.  A workgroup owns 64 packed rows (2 blocks; 32 rows in the
// unsplit form of the O / down projections); its NW waves (4, 8 or 16) split the
// workgroup's K slice and are reduced through LDS in wave order; the
// `ksplit` workgroups of one row group (two or four times as many for the row groups that would
// otherwise form a thin second round of the launch) write fp32 partial sums, and the one that
// arrives last (a counter per row group) adds them up in slice order - so the
// result does not depend on which one that is - and runs the epilogue.  The
// partial sums are written with device-scope (write-through) stores that have
// completed before the counter is bumped, which keeps cache write-backs and
// invalidations out of the protocol.  Epilogues:
//   DEC_QKV    scale by the RMS Norm factor, RoPE at position lens[b], write q
//              to the decode query buffer and k, v into the cache
//   DEC_SWIGLU scale, m = silu(gate) * up -> P(32, I)
//   DEC_RESID  x += sum ; xres = x ; y' = x * gain -> P(32, H) ; per-token sum of
//              squares of this row group -> ssq_out   (RMS Norm of the next
//              sub-layer, applied by that sub-layer's epilogue as a scale:
//              W (x * rstd * g) = rstd * W (x * g))
//   DEC_FINAL  x += sum ; hidden_out = x ; the finisher of row group 0 also counts the
//              step's token into the cached lengths (every reader of them in this
//              step ran in an earlier kernel)
// ----------------------------------------------------------------------------
// A wave keeps 10 weight loads of 1 KiB in flight (a window of 5 k-tiles of two row blocks, or 10 of
// one); 16 such waves per CU (124 registers) measured better than 20 loads in flight at 12 waves.
constexpr int kWavesPerCu = 16;  // 4 per SIMD: NW waves per workgroup, kWavesPerCu / NW workgroups per CU
constexpr int kBeginRows = 64;  // rows per workgroup of the kernel that opens a step (and per sum of squares it writes)

struct DecGemvParams {
  const bf16_t *W, *x;
  float *partial;
  unsigned *counters;
  int N, KT, ksplit, tiles_per_wave, batch;
  // row groups from `groups1` on are split `tail` times as fine (they run last and keep the launch's tail short)
  int groups1, n_groups, tail;
  const float *ssq_in;  // [n_ssq][32]
  int n_ssq;
  float inv_H, eps;
  const int *lens;
  const float *cos_tab, *sin_tab;
  bf16_t *qdec, *Kc, *Vc;
  CacheGeom geom;
  int nq, nkv;
  bf16_t *m_out;
  int I;
  float *xres;
  const bf16_t *gain;
  bf16_t *y_out;
  float *ssq_out;
  bf16_t *hidden_out;
  int H;
  int *lens_advance;  // DEC_FINAL: cached lengths to bump once the step's last kernel finishes
};

// FBW row blocks of 32 per workgroup: 2 where an epilogue pairs rows of two blocks (RoPE partners,
// gate and up) and for long K; 1 for the residual epilogues at short K, where 32-row workgroups with
// a 10-tile window give as many waves with as much in flight as two slices of 64-row workgroups
// would, without partial sums, counter and gather at the end.
// CLS (a hyp_kernel_class_t) only gives each GEMM of a block its own kernel name in a trace.
// NW waves per workgroup share the k-tiles of the workgroup's K slice: more waves per workgroup mean
// fewer K slices across workgroups (fewer partial sums in memory, or none) for the same number of
// waves in flight.
template <int EPI, int FBW, int NW, int CLS>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(4))) k_dec_gemv(DecGemvParams p) {
  constexpr int UNROLL = FBW == 1 ? 10 : 5;
  constexpr int kGroupRows = FBW * 32;
  constexpr int kRedStride = kGroupRows + 4;  // keeps 16-byte alignment, spreads tokens over banks
  constexpr int kSsqParts = NW * 2;  // interleaved partial sums of the row groups' sums of squares (one per 32 threads)
  // the waves' sums as [wave][token][row], tokens of the batch only: rows contiguous so that the
  // cross-wave add reads without bank conflicts; reused as fin[token][kGroupRows + 1] once reduced
  extern __shared__ __attribute__((aligned(16))) float red_raw[];
  float (*red)[kRedStride] = (float (*)[kRedStride])red_raw;  // red[wave * batch + token][row]
  __shared__ float rstd_s[32];
  __shared__ unsigned is_last;
  float (*fin)[kGroupRows + 1] = (float (*)[kGroupRows + 1])red_raw;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // 1-D grid: first the `ksplit` slices of row groups [0, groups1), slice-major, then the
  // tail * ksplit slices of the remaining groups
  int group, ks, ksplit = p.ksplit, tiles_per_wave = p.tiles_per_wave;
  {
    const int first = p.groups1 * p.ksplit, id = blockIdx.x;
    if (id < first) { group = id % p.groups1; ks = id / p.groups1; }
    else {
      const int g2 = p.n_groups - p.groups1, id2 = id - first;
      group = p.groups1 + id2 % g2; ks = id2 / g2; ksplit *= p.tail; tiles_per_wave /= p.tail;
    }
  }
  const int fb0 = group * FBW;
  // partial sums [slice][32 tokens][rows]: the finely cut last groups have a narrow array of their own behind the
  // main one (rows of those groups only), so their extra slices do not cost room over all N rows
  const bool fine = group >= p.groups1;
  float *const part = fine ? p.partial + (size_t)p.ksplit * 32 * p.N : p.partial;
  const int part_n = fine ? (p.n_groups - p.groups1) * kGroupRows : p.N;        // rows per token
  const int part_r0 = fine ? (group - p.groups1) * kGroupRows : fb0 * 32;       // this group's first row
  // positions of the step's tokens (the QKV epilogue's rotary angles depend on them): fetched under the streaming loop
  // (ahead of time for the first kPf * 8 tokens, which covers the usual batch; the rest is loaded in place)
  constexpr int kPf = 2;
  int pos_pf[kPf] = {0, 0};
  if (EPI == DEC_QKV) {
#pragma unroll
    for (int j = 0; j < kPf; ++j) {
      int idx = threadIdx.x + j * NW * 64;
      if (idx < p.batch * 32) pos_pf[j] = p.lens[idx >> 5];
    }
  }
  // the workgroup's NW waves take the k-tiles of its slice in turn, so that each step of
  // the workgroup reads NW KiB contiguous per row block (HBM serves that pattern ~10 % faster
  // than separate 1 KiB streams)
  const int kt0 = ks * NW * tiles_per_wave + wave;
  constexpr size_t kStep = (size_t)NW * kTileElems;
  f32x16_t acc[FBW];
#pragma unroll
  for (int i = 0; i < FBW; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  // token columns beyond the batch feed output columns nobody reads: their lanes all read
  // token 0's chunk, so the x tile costs one cache line more instead of a whole tile
  const bf16_t *xp = p.x + (size_t)kt0 * kTileElems + ((lane & 31) < p.batch ? lane : (lane & 32)) * 8;
  const bf16_t *wp[FBW];
#pragma unroll
  for (int i = 0; i < FBW; ++i) wp[i] = p.W + ((size_t)(fb0 + i) * p.KT + kt0) * kTileElems + lane * 8;
  // A window of UNROLL k-tiles lives in registers; as soon as a tile has gone through the
  // MFMAs its registers are reloaded with the tile UNROLL further on, so the wave keeps
  // about 2 (UNROLL - 1) KiB of weights in flight all the time.
  bf16x8_t xf[UNROLL], wf[FBW][UNROLL];
  auto load_tile = [&](int u, int tile) {
#pragma unroll
    for (int i = 0; i < FBW; ++i) wf[i][u] = __builtin_nontemporal_load((const bf16x8_t *)(wp[i] + (size_t)tile * kStep));
    xf[u] = *(const bf16x8_t *)(xp + (size_t)tile * kStep);
  };
  auto use_tile = [&](int u) {
#pragma unroll
    for (int i = 0; i < FBW; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i][u], xf[u], acc[i], 0, 0, 0);
  };
  const int n_win = tiles_per_wave / UNROLL, rem = tiles_per_wave - n_win * UNROLL;
  if (n_win > 0) {
    int t = 0;
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) load_tile(u, u);
    for (int wi = 1; wi < n_win; ++wi, t += UNROLL) {
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        use_tile(u);
        load_tile(u, t + UNROLL + u);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // last full window; the rem (< UNROLL) tiles left over move into its registers as they free up
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      use_tile(u);
      if (u < rem) load_tile(u, t + UNROLL + u);
    }
  } else {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (u < rem) load_tile(u, u);
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u)
    if (u < rem) use_tile(u);
  // accumulator register r of lane l of block i is packed row 32 i + 8 (r/4) + 4 (l/32) + r%4 of
  // token l % 32: four consecutive rows per 16-byte store; token columns beyond the batch stay home
  if ((lane & 31) < p.batch) {
#pragma unroll
    for (int i = 0; i < FBW; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4_t v = {acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]};
        *(f32x4_t *)&red[wave * p.batch + (lane & 31)][32 * i + 8 * q + 4 * (lane >> 5)] = v;
      }
  }
  __syncthreads();
  // sums of the 64 rows of this group, at most 8 (token, row) pairs per thread
  const int n_pairs = p.batch * kGroupRows;
  float mine[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int idx = threadIdx.x + j * NW * 64;
    mine[j] = 0.f;
    if (idx < n_pairs) {
      int f = idx % kGroupRows, token = idx / kGroupRows;
#pragma unroll
      for (int w = 0; w < NW; ++w) mine[j] += red[w * p.batch + token][f];
    }
  }
  __syncthreads();  // `red` is free from here on
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int idx = threadIdx.x + j * NW * 64;
    if (idx < n_pairs) {
      int f = idx % kGroupRows, token = idx / kGroupRows;
      if (ksplit > 1)  // write-through store: visible to the other XCDs once it has completed
        __hip_atomic_store(&part[((size_t)ks * 32 + token) * part_n + part_r0 + f], mine[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else fin[token][f] = mine[j];
    }
  }
  if (ksplit > 1) {
    __builtin_amdgcn_s_waitcnt(0);  // this thread's partial sums have completed ...
    __syncthreads();
    if (threadIdx.x == 0) {  // ... before it is counted
      unsigned old = atomicAdd(&p.counters[group], 1u);
      is_last = (old == (unsigned)ksplit - 1) ? 1u : 0u;
      if (is_last) p.counters[group] = 0;  // ready for the next launch
    }
    __syncthreads();
    if (!is_last) return;
  }
  // The finishing workgroup.  Its loads are issued together so that their round trips
  // overlap: first the sums of squares behind the RMS Norm factor (16 row groups per
  // thread at once), then the partial sums.
  // what the epilogues need from memory besides the partial sums is requested first, so that
  // all of a finisher's loads share one round trip
  float cos_pf[kPf] = {0.f, 0.f}, sin_pf[kPf] = {0.f, 0.f};
  if (EPI == DEC_QKV) {
#pragma unroll
    for (int j = 0; j < kPf; ++j) {
      int idx = threadIdx.x + j * NW * 64;
      if (idx < p.batch * 32) {
        int d0 = ((fb0 >> 1) & 1) * 32 + (idx & 31);
        cos_pf[j] = p.cos_tab[(size_t)pos_pf[j] * 64 + d0];
        sin_pf[j] = p.sin_tab[(size_t)pos_pf[j] * 64 + d0];
      }
    }
  }
  constexpr int kPfR = 4;  // (token, row) pairs per thread fetched ahead: 16 tokens' worth
  float xres_pf[kPfR], gain_pf[kPfR];  // residual stream and next norm's gain
  if (EPI == DEC_RESID || EPI == DEC_FINAL) {
#pragma unroll
    for (int j = 0; j < kPfR; ++j) {
      int idx = threadIdx.x + j * NW * 64;
      xres_pf[j] = 0.f; gain_pf[j] = 0.f;
      if (idx < n_pairs) {
        int f = idx % kGroupRows, b = idx / kGroupRows;
        xres_pf[j] = p.xres[(size_t)b * p.H + fb0 * 32 + f];
        if (EPI == DEC_RESID) gain_pf[j] = bf16_to_f32(p.gain[fb0 * 32 + f]);
      }
    }
  }
  float ssq_v[16];
  const int ssq_tkn = threadIdx.x & 31, ssq_part_id = threadIdx.x >> 5;
  if (EPI == DEC_QKV || EPI == DEC_SWIGLU) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      int g = ssq_part_id + kSsqParts * u;
      ssq_v[u] = g < p.n_ssq ? p.ssq_in[g * 32 + ssq_tkn] : 0.f;
    }
  }
  if (ksplit > 1) {
    // Plain loads are enough here: every 256-byte run of `partial` has exactly one
    // writer in this launch, this XCD's L2 was invalidated when the launch began,
    // and nothing in this launch read these lines before, so a line is either
    // absent (fetched from memory, where the writer's store has completed) or was
    // put there by a writer on this very XCD.  With more than four slices, two (token, row)
    // pairs per thread and GW slices of each are in flight at once; slices beyond ksplit are masked
    // rather than peeled, so the gather costs ceil(ksplit / GW) round trips.
    constexpr int GW = EPI == DEC_QKV ? 8 : 16;
    if (ksplit <= 4) {
      // few slices: four of the thread's pairs at once (16 tokens' worth per round trip)
      for (int j0 = 0; j0 * NW * 64 < n_pairs; j0 += 4) {
        float v[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int idx = threadIdx.x + (j0 + j) * NW * 64;
          const bool has = idx < n_pairs;
          const unsigned off = has ? (unsigned)((idx / kGroupRows) * part_n + part_r0 + idx % kGroupRows) : 0u;
#pragma unroll
          for (int u = 0; u < 4; ++u) v[j][u] = has && u < ksplit ? (part + (size_t)u * 32 * part_n)[off] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int idx = threadIdx.x + (j0 + j) * NW * 64;
          if (idx < n_pairs) fin[idx / kGroupRows][idx % kGroupRows] = ((v[j][0] + v[j][1]) + v[j][2]) + v[j][3];
        }
      }
    } else {
      for (int idx0 = threadIdx.x; idx0 < n_pairs; idx0 += 2 * NW * 64) {
        const int idx1 = idx0 + NW * 64;
        const bool has1 = idx1 < n_pairs;
        // slice bases are uniform (scalar registers); one 32-bit offset per pair serves every slice
        const unsigned off0 = (unsigned)((idx0 / kGroupRows) * part_n + part_r0 + idx0 % kGroupRows);
        const unsigned off1 = (unsigned)(((has1 ? idx1 : idx0) / kGroupRows) * part_n + part_r0 + (has1 ? idx1 : idx0) % kGroupRows);
        float sum0 = 0.f, sum1 = 0.f;
        for (int s = 0; s < ksplit; s += GW) {
          float v0[GW], v1[GW];
#pragma unroll
          for (int u = 0; u < GW; ++u) {
            const bool in = s + u < ksplit;
            const float *slice = part + (size_t)(s + u) * 32 * part_n;
            v0[u] = in ? slice[off0] : 0.f;
            v1[u] = in && has1 ? slice[off1] : 0.f;
          }
#pragma unroll
          for (int u = 0; u < GW; ++u) { sum0 += v0[u]; sum1 += v1[u]; }
        }
        fin[idx0 / kGroupRows][idx0 % kGroupRows] = sum0;
        if (has1) fin[idx1 / kGroupRows][idx1 % kGroupRows] = sum1;
      }
    }
  }
  if (EPI == DEC_QKV || EPI == DEC_SWIGLU) {
    // RMS Norm factor of every token: the row groups' sums of squares, added in a
    // fixed order (kSsqParts interleaved partial sums, then those in order)
    __shared__ float ssq_part[kSsqParts][32];
    {
      float ss = 0.f;
#pragma unroll
      for (int u = 0; u < 16; ++u) ss += ssq_v[u];
      for (int g = ssq_part_id + kSsqParts * 16; g < p.n_ssq; g += kSsqParts) ss += p.ssq_in[g * 32 + ssq_tkn];
      ssq_part[ssq_part_id][ssq_tkn] = ss;
    }
    __syncthreads();
    if (threadIdx.x < 32) {
      float ss = 0.f;
      for (int i = 0; i < kSsqParts; ++i) ss += ssq_part[i][threadIdx.x];
      rstd_s[threadIdx.x] = 1.0f / sqrtf(ss * p.inv_H + p.eps);
    }
  }
  __syncthreads();

  if (EPI == DEC_QKV) {
    const int r0 = fb0 * 32;
    const int head = r0 >> 7, w = (r0 >> 6) & 1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int idx = threadIdx.x + j * NW * 64;
      if (idx >= p.batch * 32) break;
      int x = idx & 31, b = idx >> 5;
      float a = fin[b][x] * rstd_s[b], c = fin[b][32 + x] * rstd_s[b];
      int d0 = w * 32 + x, d1 = d0 + 64;
      int pos = j < kPf ? pos_pf[j] : p.lens[b];
      if (head < p.nq + p.nkv) {
        float cs = j < kPf ? cos_pf[j] : p.cos_tab[(size_t)pos * 64 + d0];
        float sn = j < kPf ? sin_pf[j] : p.sin_tab[(size_t)pos * 64 + d0];
        float lo = a * cs - c * sn, hi = c * cs + a * sn;
        if (head < p.nq) {
          int G = p.nq / p.nkv;
          bf16_t *dst = p.qdec + ((size_t)b * p.nkv + head / G) * (32 * 128);
          dst[frag_offset(head % G, d0, 128)] = f2bf_dev(lo);
          dst[frag_offset(head % G, d1, 128)] = f2bf_dev(hi);
        } else {
          bf16_t *dst = p.Kc + p.geom.off(b, head - p.nq, pos >> 5);
          dst[frag_offset(pos & 31, d0, 128)] = f2bf_dev(lo);
          dst[frag_offset(pos & 31, d1, 128)] = f2bf_dev(hi);
        }
      } else {
        bf16_t *dst = p.Vc + p.geom.off(b, head - p.nq - p.nkv, pos >> 5);
        int m, khh;
        int e = vtile_slot_of_key(pos & 31, &m, &khh);
        dst[(size_t)(m * 4 + (d0 >> 5)) * kTileElems + (khh * 32 + (d0 & 31)) * 8 + e] = f2bf_dev(a);
        dst[(size_t)(m * 4 + (d1 >> 5)) * kTileElems + (khh * 32 + (d1 & 31)) * 8 + e] = f2bf_dev(c);
      }
    }
  } else if (EPI == DEC_SWIGLU) {
    const int f0 = (fb0 >> 3) * 128 + ((fb0 >> 1) & 3) * 32;
    for (int idx = threadIdx.x; idx < p.batch * 32; idx += NW * 64) {
      int x = idx & 31, b = idx >> 5;
      float g = fin[b][x] * rstd_s[b], u = fin[b][32 + x] * rstd_s[b];
      p.m_out[frag_offset(b, f0 + x, p.I)] = f2bf_dev(g / (1.0f + __expf(-g)) * u);
    }
  } else {
    const int n0 = fb0 * 32;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int idx = threadIdx.x + j * NW * 64;
      if (idx >= n_pairs) break;
      int f = idx % kGroupRows, b = idx / kGroupRows;
      float xn = (j < kPfR ? xres_pf[j] : p.xres[(size_t)b * p.H + n0 + f]) + fin[b][f];
      if (EPI == DEC_RESID) {
        p.xres[(size_t)b * p.H + n0 + f] = xn;
        p.y_out[frag_offset(b, n0 + f, p.H)] = f2bf_dev(xn * (j < kPfR ? gain_pf[j] : bf16_to_f32(p.gain[n0 + f])));
        fin[b][f] = xn * xn;
      } else {
        p.hidden_out[(size_t)b * p.H + n0 + f] = f2bf_dev(xn);
      }
    }
    if (EPI == DEC_FINAL && group == 0 && p.lens_advance && threadIdx.x < p.batch) p.lens_advance[threadIdx.x] += 1;
    if (EPI == DEC_RESID) {
      __syncthreads();
      if (threadIdx.x < p.batch) {
        float ss = 0.f;
        for (int f = 0; f < kGroupRows; ++f) ss += fin[threadIdx.x][f];
        p.ssq_out[group * 32 + threadIdx.x] = ss;
      }
    }
  }
}

// first kernel of a decode step: x = hidden_in ; xres = x ; y' = x * gain ; ssq
// grid H / 64, 256 threads
__global__ void __launch_bounds__(256) k_dec_begin(const bf16_t *__restrict__ hidden_in, float *__restrict__ xres,
                                                   const bf16_t *__restrict__ gain, bf16_t *__restrict__ y_out,
                                                   float *__restrict__ ssq_out, int H, int batch) {
  __shared__ float sq[32][kBeginRows + 1];
  const int n0 = blockIdx.x * kBeginRows;
  for (int idx = threadIdx.x; idx < batch * kBeginRows; idx += 256) {
    int f = idx % kBeginRows, b = idx / kBeginRows;
    float x = bf16_to_f32(hidden_in[(size_t)b * H + n0 + f]);
    xres[(size_t)b * H + n0 + f] = x;
    y_out[frag_offset(b, n0 + f, H)] = f2bf_dev(x * bf16_to_f32(gain[n0 + f]));
    sq[b][f] = x * x;
  }
  __syncthreads();
  if (threadIdx.x < batch) {
    float ss = 0.f;
    for (int f = 0; f < kBeginRows; ++f) ss += sq[threadIdx.x][f];
    ssq_out[blockIdx.x * 32 + threadIdx.x] = ss;
  }
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

// How one skinny GEMM of a decode step is cut into workgroups.
//   fbw     32-row blocks per workgroup: 2 where the epilogue pairs rows of two blocks (RoPE partners,
//           gate and up) and for long K; 1 for the residual GEMMs at short K, which then run as
//           unsplit 4-wave workgroups with a 10-tile window
//   nw      waves per workgroup; they share the k-tiles of the workgroup's K slice.  8 for the
//           64-row workgroups: the same waves in flight with half the K slices of 4-wave workgroups
//   ksplit  K slices across workgroups (partial sums in memory, the last to arrive adds them up):
//           the fewest that put a wave on every slot of the chip (16 per CU), as long as a wave
//           keeps at least 20 k-tiles (four windows of the streaming loop) and the fp32 partial sums
//           (written and read once per slice and token) stay a few percent of the weight bytes.
//           Phi-3-medium shapes: gate/up unsplit (560 workgroups), QKV 2 slices, down 7 slices;
//           measured against every other admissible cut of each GEMM at batch 8 and 32, this rule's
//           choices were the fastest or within 1 % of it.
GemvPlan mfma_gemv_plan(int cls, int N, int K, int batch) {
  GemvPlan g;
  const int KT = K / 16;
  if ((cls == HYP_K_GEMV_O || cls == HYP_K_GEMV_DOWN) && KT / 4 <= 112 && KT % 4 == 0) {
    g.fbw = 1; g.nw = 4; g.ksplit = 1;
    return g;
  }
  g.fbw = 2; g.nw = 8; g.ksplit = 1;
  if (KT % g.nw != 0) g.nw = 4;
  const int groups = N / 64, wave_slots = kWavesPerCu * 256;
  int cap = (int)(0.025 * K / (batch > 0 ? batch : 1));
  if (cap < 1) cap = 1;
  for (int ks = 1; ks <= 64 && ks <= cap; ++ks) {
    if (KT % (ks * g.nw) != 0 || KT / (ks * g.nw) < 20) continue;
    g.ksplit = ks;
    if (groups * ks * g.nw >= wave_slots) break;
  }
  // More workgroups than fit the chip at once, but fewer than two rounds: the groups beyond the first round
  // are cut finer, for what would otherwise be a thin second round of long workgroups.  A CU serves its waves'
  // loads oldest first, so the late workgroups stream last whatever their size: they should be many (bytes
  // in flight on every CU to the end) and short.  Four times finer where a wave keeps two windows of
  // the streaming loop (gate/up: 62.3 -> 59.6 us), else twice.
  const int units = groups * g.ksplit, slots = wave_slots / g.nw, tpw = KT / (g.ksplit * g.nw);
  if (units > slots && units < 2 * slots) {
    if (tpw % 4 == 0 && tpw / 4 >= 10) g.tail = 4;
    else if (tpw % 2 == 0 && tpw / 2 >= 10) g.tail = 2;
  }
  return g;
}

// Row groups [0, groups1) run as plan.ksplit workgroups each, the rest (beyond the first round of the launch, if the plan
// cuts those finer) as plan.ksplit * tail.
static void gemv_cut(const GemvPlan &g, int N, int K, int *groups1, int *tail) {
  const int groups = N / (g.fbw * 32), slots = kWavesPerCu / g.nw * 256, tpw = K / 16 / (g.ksplit * g.nw);
  *groups1 = groups; *tail = 1;
  if (g.tail > 1 && groups * g.ksplit > slots && tpw % g.tail == 0) { *groups1 = slots / g.ksplit; *tail = g.tail; }
}

// floats of partial sums a GEMM cut this way needs: [ksplit][32][N], then [ksplit * tail][32][rows of the finely cut groups]
size_t mfma_gemv_partial_floats(const GemvPlan &g, int N, int K) {
  int groups1, tail;
  gemv_cut(g, N, K, &groups1, &tail);
  const int fine_rows = (N / (g.fbw * 32) - groups1) * g.fbw * 32;
  return (size_t)g.ksplit * 32 * N + (size_t)g.ksplit * tail * 32 * fine_rows;
}

// the (epilogue, blocks per workgroup, waves per workgroup, class) combinations a plan may ask for
#define HYP_GEMV_VARIANTS(X, NW)                                                                         \
  X(DEC_QKV, 2, NW, HYP_K_GEMV_QKV) X(DEC_SWIGLU, 2, NW, HYP_K_GEMV_GATEUP)                              \
  X(DEC_RESID, 1, NW, HYP_K_GEMV_O) X(DEC_RESID, 2, NW, HYP_K_GEMV_O)                                    \
  X(DEC_RESID, 1, NW, HYP_K_GEMV_DOWN) X(DEC_RESID, 2, NW, HYP_K_GEMV_DOWN)                              \
  X(DEC_FINAL, 1, NW, HYP_K_GEMV_DOWN) X(DEC_FINAL, 2, NW, HYP_K_GEMV_DOWN)

// the waves' sums of 32 tokens can pass the 64 KiB a workgroup gets by default
hipError_t mfma_gemv_init() {
  hipError_t e = hipSuccess;
#define X(EPI, FBW, NW, CLS)                                                                                     \
  if (e == hipSuccess)                                                                                           \
    e = hipFuncSetAttribute((const void *)k_dec_gemv<EPI, FBW, NW, CLS>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                            (int)(sizeof(float) * NW * 32 * (FBW * 32 + 4)));
  HYP_GEMV_VARIANTS(X, 8)
  HYP_GEMV_VARIANTS(X, 16)
#undef X
  return e;
}

hipError_t mfma_dec_gemv(int epi, int cls, const DecGemv &a, hipStream_t s) {
  DecGemvParams p = {};
  const int fbw = a.plan.fbw, nw = a.plan.nw, ksplit = a.plan.ksplit;
  p.W = a.W; p.x = a.x; p.partial = a.partial; p.counters = a.counters;
  p.N = a.N; p.KT = a.K / 16; p.ksplit = ksplit; p.tiles_per_wave = p.KT / (ksplit * nw); p.batch = a.batch;
  if (p.tiles_per_wave * ksplit * nw != p.KT || a.N % (fbw * 32) != 0 || kWavesPerCu % nw != 0) return hipErrorInvalidValue;
  p.ssq_in = a.ssq_in; p.n_ssq = a.n_ssq; p.inv_H = a.n_ssq ? 1.0f / (float)a.K : 0.f; p.eps = a.eps;
  p.lens = a.lens; p.cos_tab = a.cos_tab; p.sin_tab = a.sin_tab; p.qdec = a.qdec; p.Kc = a.Kc; p.Vc = a.Vc;
  p.geom = a.geom; p.nq = a.nq; p.nkv = a.nkv; p.m_out = a.m_out; p.I = a.I; p.xres = a.xres; p.gain = a.gain;
  p.y_out = a.y_out; p.ssq_out = a.ssq_out; p.hidden_out = a.hidden_out; p.H = a.H; p.lens_advance = a.lens_advance;
  // the plan's finer cut of the row groups beyond the first round
  const int groups = a.N / (fbw * 32);
  p.n_groups = groups;
  gemv_cut(a.plan, a.N, a.K, &p.groups1, &p.tail);
  if (mfma_gemv_partial_floats(a.plan, a.N, a.K) > a.partial_floats) return hipErrorInvalidValue;
  dim3 grid(p.groups1 * ksplit + (groups - p.groups1) * p.tail * ksplit);
  const size_t lds = sizeof(float) * nw * a.batch * (fbw * 32 + 4);  // the waves' sums of the live tokens
  bool launched = false;
#define X(EPI, FBW, NW, CLS)                                                 \
  if (!launched && epi == EPI && fbw == FBW && nw == NW && cls == CLS) {      \
    k_dec_gemv<EPI, FBW, NW, CLS><<<grid, NW * 64, lds, s>>>(p);             \
    launched = true;                                                         \
  }
  HYP_GEMV_VARIANTS(X, 4)
  HYP_GEMV_VARIANTS(X, 8)
  HYP_GEMV_VARIANTS(X, 16)
#undef X
  if (!launched) return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t mfma_dec_begin(const bf16_t *hidden_in, float *xres, const bf16_t *gain, bf16_t *y_out, float *ssq_out,
                          int H, int batch, hipStream_t s) {
  k_dec_begin<<<H / kBeginRows, 256, 0, s>>>(hidden_in, xres, gain, y_out, ssq_out, H, batch);
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
