// MFMA kernels of the prefill path of a bf16 stage: weight repacking, the kernels
// at the two ends of the residual stream, the LDS-staged GEMM with its four
// epilogues (RoPE + KV-cache write, SwiGLU, residual add + next RMS Norm's gain
// and statistics, plain), for the decoder block of Sec. III-A.
#include <type_traits>
#include "mfma_common.h"
#include "mfma_kernels.h"

namespace hyp {

namespace {

// ----------------------------------------------------------------------------
// Row permutations applied when a weight matrix is repacked, chosen so that the
// two values an epilogue has to combine land in the same lane and register of
// two accumulator blocks of one wave (a wave owns 64 packed rows = 2 blocks):
//   QKV:     inside every head, block 0 of a wave holds d in [ib, ib+32) and
//            block 1 holds d + 64 -> the RoPE partner (i, i + 64);
//   gate/up: block 0 holds gate rows f..f+31, block 1 the up rows of the same f.
// ----------------------------------------------------------------------------
__device__ inline int src_row_qkv(int r) {  // packed row -> row of [wq; wk; wv]
  int head = r >> 7, w = (r >> 6) & 1, i = (r >> 5) & 1, x = r & 31;
  return head * 128 + w * 32 + i * 64 + x;
}
__device__ inline int src_row_gateup(int r, int I) {  // packed row -> row of [gate; up]
  int tile = r >> 8, w = (r >> 6) & 3, i = (r >> 5) & 1, x = r & 31;
  int f = tile * 128 + w * 32 + x;
  return i ? I + f : f;
}

// one thread per 16-byte chunk of the destination
__global__ void __launch_bounds__(256) k_pack_weight(const bf16_t *__restrict__ src0,
                                                     const bf16_t *__restrict__ src1,
                                                     const bf16_t *__restrict__ src2, int rows0,
                                                     int rows1, bf16_t *__restrict__ dst, int N, int K,
                                                     int mode, int I) {
  size_t chunk = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t total = (size_t)N * K / 8;
  if (chunk >= total) return;
  size_t tile = chunk >> 6;
  int lane = chunk & 63;
  int rb = (int)(tile / (K >> 4)), kt = (int)(tile % (K >> 4));
  int r = rb * 32 + (lane & 31), k = kt * 16 + (lane >> 5) * 8;
  int sr = mode == PACK_QKV ? src_row_qkv(r) : mode == PACK_GATEUP ? src_row_gateup(r, I) : r;
  const bf16_t *s;
  if (sr < rows0) s = src0 + (size_t)sr * K;
  else if (sr < rows0 + rows1) s = src1 + (size_t)(sr - rows0) * K;
  else s = src2 + (size_t)(sr - rows0 - rows1) * K;
  *(u16x8_t *)(dst + chunk * 8) = *(const u16x8_t *)(s + k);
}

// ----------------------------------------------------------------------------
// The two ends of a prefill over internal rows (everything between them happens in
// GEMM epilogues).
//   MODE 0  x = hidden_in[row_ext] ; residual = x (accumulator order) ;
//           y' = x * g -> P(rows, H) ; rstd = rsqrt(mean(x^2) + eps)
//           (the norm factor is applied by the consuming GEMM's epilogue)
//   MODE 1  hidden_out[row_ext] = residual + delta, delta = P(rows, H) bf16 of the last GEMM
// A 256-thread block owns RPW consecutive rows (8, or 1 when there are only a few
// rows so that more workgroups share the work); thread t works on row t % RPW.
// ----------------------------------------------------------------------------
template <int MODE, int RPW>  // MODE 0: first block's input ; 1: stage output
__global__ void __launch_bounds__(256) k_add_norm(const bf16_t *__restrict__ hidden_in,
                                                  float *__restrict__ xres,
                                                  const bf16_t *__restrict__ delta_bf,
                                                  const bf16_t *__restrict__ gain,
                                                  bf16_t *__restrict__ y, float *__restrict__ rstd,
                                                  bf16_t *__restrict__ hidden_out,
                                                  const int *__restrict__ row_ext, int H, float eps) {
  constexpr int CPR = 256 / RPW;  // threads per row
  __shared__ float red[RPW][CPR + 1];
  int r8 = threadIdx.x % RPW, cg = threadIdx.x / RPW;
  int row = blockIdx.x * RPW + r8;
  int ext = row_ext[row];
  int nchunk = H >> 3;
  float ss = 0.f;
  for (int c = cg; c < nchunk; c += CPR) {
    float v[8];
    float *xa = xres + acc_offset(row, c * 8, H), *xb = xres + acc_offset(row, c * 8 + 4, H);
    if (ext < 0) {
      for (int e = 0; e < 8; ++e) v[e] = 0.f;
    } else if (MODE == 0) {
      u16x8_t h = *(const u16x8_t *)(hidden_in + (size_t)ext * H + c * 8);
      for (int e = 0; e < 8; ++e) v[e] = bf16_to_f32(h.v[e]);
    } else {
      f32x4_t a = *(const f32x4_t *)xa, b = *(const f32x4_t *)xb;
      u16x8_t d = *(const u16x8_t *)(delta_bf + frag_offset(row, c * 8, H));
      for (int e = 0; e < 4; ++e) { v[e] = a[e] + bf16_to_f32(d.v[e]); v[4 + e] = b[e] + bf16_to_f32(d.v[4 + e]); }
    }
    if (MODE == 0) {
      f32x4_t a, b;
      for (int e = 0; e < 4; ++e) { a[e] = v[e]; b[e] = v[4 + e]; }
      *(f32x4_t *)xa = a;
      *(f32x4_t *)xb = b;
      u16x8_t gg = *(const u16x8_t *)(gain + c * 8), o;
      for (int e = 0; e < 8; ++e) {
        ss += v[e] * v[e];
        o.v[e] = f2bf_dev(v[e] * bf16_to_f32(gg.v[e]));
      }
      *(u16x8_t *)(y + frag_offset(row, c * 8, H)) = o;
    } else if (ext >= 0) {
      u16x8_t o;
      for (int e = 0; e < 8; ++e) o.v[e] = f2bf_dev(v[e]);
      *(u16x8_t *)(hidden_out + (size_t)ext * H + c * 8) = o;
    }
  }
  if (MODE == 1) return;
  red[r8][cg] = ss;
  __syncthreads();
  if (cg == 0) {
    float tot = 0.f;
    for (int i = 0; i < CPR; ++i) tot += red[r8][i];
    rstd[row] = ext < 0 ? 0.f : 1.0f / sqrtf(tot / (float)H + eps);  // padding rows stay zero also when eps == 0
  }
}

// rstd[row] = 1 / sqrt(mean square + eps) from the sums of squares the residual
// epilogue left per 64-feature group: ssq_part[group][row], added in group order.
__global__ void __launch_bounds__(256) k_rstd(const float *__restrict__ ssq_part, float *__restrict__ rstd,
                                              const int *__restrict__ row_ext, int rows, int groups, float inv_H, float eps) {
  int row = blockIdx.x * 256 + threadIdx.x;
  if (row >= rows) return;
  const bool live = row_ext[row] >= 0;
  float tot = 0.f;
  for (int g0 = 0; g0 < groups; g0 += 16) {  // 16 loads in flight, added in group order
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = g0 + u < groups ? ssq_part[(size_t)(g0 + u) * rows + row] : 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) tot += v[u];
  }
  rstd[row] = live ? 1.0f / sqrtf(tot * inv_H + eps) : 0.f;  // a padding row's sum is 0: no 1/0 when eps == 0
}

// ----------------------------------------------------------------------------
// GEMM  C^T[N, T] = W[N, K] X[T, K]^T  on fragment-order operands.
//
// Workgroup tile 256 features x 256 tokens, 8 waves (4 along features x 2 along
// tokens), each wave 64 x 128 = 2 x 4 blocks of 32 x 32, every block four 16 x 16
// outputs of v_mfma_f32_16x16x32_bf16 (128 fp32 registers).  That shape, not
// 32x32x16: on Gaussian operands the chip sustains 2.06 PFLOP/s of it from registers
// against 1.78 of the 32x32x16 form (it is power-limited, and the deeper, narrower
// product costs less per FLOP), and this kernel got 6 - 8 % faster by the change.
// K advances in stages of 32 (2 k-tiles = one MFMA's depth); 4 stages of 32 KiB rotate
// through LDS and are filled by direct global->LDS wave loads issued three stages
// ahead, 4 per wave and stage.  Fragments are read from LDS with conflict-free
// ds_read_b128 (16 lanes on 256 contiguous bytes) well ahead of the MFMAs that use
// them.  Every LDS read and every global->LDS load is pinned behind one particular
// MFMA of the stage: left to the compiler they bunch up and the matrix pipe waits
// for the burst to issue.
// One barrier per stage.  Workgroups are numbered so that the ones
// that run together on an XCD (id % 8) cover a band of `gm` token tiles times
// consecutive feature tiles and share operand panels in that XCD's L2.  A GEMM of 64
// rounds or more leaves its last rounds to workgroups that draw a tile each from a counter.
// ----------------------------------------------------------------------------
constexpr int WF = 4, WT = 2, FB = 2, TB = 4, KTS = 2, NST = 4;
constexpr int XB = WT * TB, NBK = WF * FB;           // 8 token blocks, 8 feature blocks
constexpr int STAGE_BYTES = (XB + NBK) * KTS * 1024;  // 32 KiB
constexpr int LPW = (XB + NBK) * KTS / (WF * WT);     // 4 wave loads per wave and stage
constexpr int GEMM_LDS = STAGE_BYTES * NST;           // 128 KiB

struct GemmParams {
  const bf16_t *X;   // P(T', K)
  const bf16_t *W;   // P(N, K)
  int KT;            // K / 16
  int tok_blocks;    // T' / 32
  int feat_blocks;   // N / 32 (multiple of 8)
  int gm;            // token tiles per band
  int n_tiles;
  // epilogue
  bf16_t *out;       // EPI_STORE: P(T', N); EPI_SWIGLU: P(T', N/2); EPI_QKV: q as P(T', qd); EPI_RESID: y' as P(T', N)
  int out_K;         // row length of `out`
  bf16_t *Kc, *Vc;   // EPI_QKV: caches of this layer
  CacheGeom geom;
  int qd, kvd;
  const float *cos_tab, *sin_tab;  // [pos][64]
  const int *row_pos, *row_req;    // per internal row
  const float *rstd;               // EPI_QKV / EPI_SWIGLU: RMS Norm factor of every row of X
  // EPI_RESID: residual stream A(T', N), gains of the next norm, padding map, statistics out
  float *xres;
  const bf16_t *gain;
  const int *row_ext;
  float *ssq_part;                 // [N / 64][T']
  // K loop split over `ksplit` workgroups per tile (GEMMs with few tiles): fp32 partial tiles and arrival counters
  int ksplit, tiles_grid;
  int n_static, pool_wgs;          // unsplit GEMMs of many rounds: tiles assigned by position / workgroups that draw the rest
  float *split_ws;
  unsigned *split_counters;
};

// Accumulators.  A wave's 32 x 32 block (features x tokens) is four 16 x 16 outputs of v_mfma_f32_16x16x32_bf16,
// indexed [fh][th] (feature half, token half); lane l holds, in the four registers e of output [fh][th],
// features 16 fh + 4 (l / 16) + e of token 16 th + l % 16.
struct AccLane {
  int q, t16;  // l / 16, l % 16
};
// four consecutive features f0 .. f0+3 (f0 a multiple of 4) of internal row `row` into P(T', out_K): one 8-byte store
__device__ __forceinline__ void store4(bf16_t *out, int out_K, int row, int f0, f32x4_t v) {
  // non-temporal, like all epilogue traffic: nothing of it is read again before it has left L2 anyway, and it
  // should not push the operand panels out (O projection 5 % faster, gate/up 1.5 %)
  typedef __attribute__((__vector_size__(2 * sizeof(unsigned)))) unsigned u32x2_t;
  const bf16x4_t pk = pack4(v[0], v[1], v[2], v[3]);
  __builtin_nontemporal_store(__builtin_bit_cast(u32x2_t, pk), (u32x2_t *)(out + frag_offset(row, f0, out_K)));
}

// CLS (a hyp_kernel_class_t) does not change the code: it gives each GEMM of a block a kernel name of its
// own, so that a trace tells the O projection from the down projection, which share an epilogue.
template <int EPI, int CLS>
__global__ void __launch_bounds__(WF * WT * 64) k_gemm(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;  // wave-uniform: scalar registers
  const int wf = wave / WT, wt = wave % WT;
  // tile of this workgroup
  __shared__ unsigned split_last;
  const int nwg = p.tiles_grid, id = blockIdx.x % p.tiles_grid, slice = blockIdx.x / p.tiles_grid;
  int q;
  if (p.pool_wgs == 0) {
    q = (id % 8) * (nwg / 8) + id / 8;
  } else if (id < p.n_static) {
    // a large unsplit GEMM: most tiles belong to an XCD by position, as above ...
    q = (id % 8) * (p.n_static / 8) + id / 8;
  } else {
    // ... and the last ones go to whoever gets to them: the XCDs of one chip differ by a few percent in how fast
    // they get through their tiles (which ones are slow changes from box to box), workgroups reach them strictly
    // round-robin, and a GEMM ends with its slowest XCD.  Every workgroup of this tail draws exactly once, so the
    // last draw can leave the counter at zero for the next launch; which XCD computes a tile does not change it.
    if (threadIdx.x == 0) {
      const unsigned t = atomicAdd(p.split_counters, 1u);
      if (t == (unsigned)p.pool_wgs - 1) *p.split_counters = 0;
      split_last = t;
    }
    __syncthreads();
    q = p.n_static + (int)split_last;
  }
  if (q >= p.n_tiles) return;
  const int tiles_n = p.feat_blocks / NBK;
  const int tiles_t = (p.tok_blocks + XB - 1) / XB;
  int band = q / (p.gm * tiles_n);
  int in_band = q - band * p.gm * tiles_n;
  int rows_in_band = min(p.gm, tiles_t - band * p.gm);
  int tile_n = in_band / rows_in_band, tile_t = band * p.gm + in_band % rows_in_band;
  const int tb0 = tile_t * XB, nb0 = tile_n * NBK;
  const int KT = p.KT;

  f32x4_t acc[FB][2][TB][2];  // [feature block][feature half][token block][token half]
#pragma unroll
  for (int i = 0; i < FB; ++i)
#pragma unroll
    for (int fh = 0; fh < 2; ++fh)
#pragma unroll
      for (int j = 0; j < TB; ++j)
#pragma unroll
        for (int th = 0; th < 2; ++th)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][fh][j][th][e] = 0.f;

  const int nsteps = KT / KTS / p.ksplit;  // stages of this workgroup's K slice, >= NST guaranteed by the host
  const size_t k_first = (size_t)slice * nsteps * KTS * kTileElems;
  const bf16_t *src[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    int lid = wave * LPW + i;
    int blk = lid / KTS, kt = lid % KTS;
    if (blk >= XB) {
      src[i] = p.W + ((size_t)(nb0 + blk - XB) * KT + kt) * kTileElems + lane * 8 + k_first;
    } else {
      int tb = min(tb0 + blk, p.tok_blocks - 1);  // tail tile: reread the last block
      src[i] = p.X + ((size_t)tb * KT + kt) * kTileElems + lane * 8 + k_first;
    }
  }
  auto issue1 = [&](int i, int step, int buf) {
    __builtin_amdgcn_global_load_lds((gbl_ptr_t *)(src[i] + (size_t)step * KTS * kTileElems),
                                     (lds_ptr_t *)(lds + buf * STAGE_BYTES + (wave * LPW + i) * 1024), 16, 0, 0);
  };
#pragma unroll
  for (int s = 0; s < NST; ++s)
#pragma unroll
    for (int i = 0; i < LPW; ++i) issue1(i, s, s);
  __builtin_amdgcn_s_waitcnt(0x0F70 | (((NST - 1) * LPW) & 15) | ((((NST - 1) * LPW) >> 4) << 14));
  __builtin_amdgcn_s_barrier();

  // Fragments.  A stage holds, per 32-row block, its two k-tiles back to back (2 KiB); the operand of a
  // 16x16x32 MFMA for rows 16 h .. 16 h + 15 of the block takes from lane l rows' 16 bytes k-chunk l / 16 of
  // row 16 h + l % 16: byte (l / 16) * 512 + h * 256 + (l % 16) * 16 of the block - 16 lanes read 256 contiguous
  // bytes, no bank conflicts.  The four feature fragments of a stage (a = 2 i + fh) stay in registers for the
  // whole stage (double-buffered); the eight token fragments (b = 2 j + th) pass through four slots, each read
  // three groups of four MFMAs ahead of its use.
  const char *frag_base = lds + (lane >> 4) * 512 + (lane & 15) * 16;
  bf16x8_t afr[2][2 * FB], bfr[4];
  auto read_a = [&](int which, int buf, int a) {
    afr[which][a] = *(const bf16x8_t *)(frag_base + buf * STAGE_BYTES + (XB + wf * FB + (a >> 1)) * (KTS * 1024) + (a & 1) * 256);
  };
  auto read_b = [&](int buf, int b) {
    bfr[b & 3] = *(const bf16x8_t *)(frag_base + buf * STAGE_BYTES + (wt * TB + (b >> 1)) * (KTS * 1024) + (b & 1) * 256);
  };
  auto mfma_group = [&](int which, int b, int a) {
    acc[a >> 1][a & 1][b >> 1][b & 1] =
        __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[which][a], bfr[b & 3], acc[a >> 1][a & 1][b >> 1][b & 1], 0, 0, 0);
  };
#pragma unroll
  for (int a = 0; a < 2 * FB; ++a) read_a(0, 0, a);
#pragma unroll
  for (int b = 0; b < 3; ++b) read_b(0, b);
  int buf = 0;
  // One stage = 8 groups (token fragments b) of 4 MFMAs (feature fragments a).  Groups 0 - 4 each request the
  // token fragment three groups ahead; then every LDS read of the stage is out, the barrier says stage s + 1 has
  // landed everywhere, and groups 5 - 7 request the next stage's feature fragments and first three token fragments
  // and refill this stage's buffer - every request pinned behind one particular MFMA.
  auto stage = [&](auto cur_tag, int s) {
    constexpr int cur = decltype(cur_tag)::value, nxt = cur ^ 1;
    const int nbuf = buf + 1 == NST ? 0 : buf + 1;
    const int lstep = s + NST < nsteps ? s + NST : nsteps - 1;  // tail refills land in buffers nobody reads again
#pragma unroll
    for (int b = 0; b < 2 * TB; ++b) {
      if (b == 5) {
        // my part of stage s+1 has landed and all my LDS reads of stage s are done
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0x0070 | (((NST - 2) * LPW) & 15) | ((((NST - 2) * LPW) >> 4) << 14));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int a = 0; a < 2 * FB; ++a) {
        mfma_group(cur, b, a);
        __builtin_amdgcn_sched_barrier(0);
        if (b < 5) {
          if (a == 0) read_b(buf, b + 3);
        } else {
          const int m = (b - 5) * 4 + a;  // 0 .. 11 behind the barrier
          if (m == 0) read_a(nxt, nbuf, 0);
          if (m == 1) issue1(0, lstep, buf);
          if (m == 2) read_a(nxt, nbuf, 1);
          if (m == 3) read_b(nbuf, 0);      // slot 0 held fragment 4
          if (m == 4) read_a(nxt, nbuf, 2);
          if (m == 5) issue1(1, lstep, buf);
          if (m == 6) read_a(nxt, nbuf, 3);
          if (m == 7) read_b(nbuf, 1);      // slot 1 held fragment 5
          if (m == 8) issue1(2, lstep, buf);
          if (m == 9) read_b(nbuf, 2);      // slot 2 held fragment 6
          if (m == 10) issue1(3, lstep, buf);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    buf = nbuf;
  };
  static_assert(LPW == 4 && FB == 2 && TB == 4, "the pinned slots above assume 4 loads, 4 + 8 fragments per stage");
  // Stages run in pairs (the feature fragments alternate between two register sets); an odd count starts with a
  // single stage and one copy of its set.  The very last stage requests nothing beyond itself.
  {
    int s = 0;
    if (nsteps & 1) {
      stage(std::integral_constant<int, 0>(), 0);
#pragma unroll
      for (int a = 0; a < 2 * FB; ++a) afr[0][a] = afr[1][a];
      s = 1;
    }
    for (; s + 2 < nsteps; s += 2) {
      stage(std::integral_constant<int, 0>(), s);
      stage(std::integral_constant<int, 1>(), s + 1);
    }
    stage(std::integral_constant<int, 0>(), s);
#pragma unroll
    for (int b = 0; b < 2 * TB; ++b)
#pragma unroll
      for (int a = 0; a < 2 * FB; ++a) {
        mfma_group(1, b, a);
        if (a == 0 && b < 5) read_b(buf, b + 3);
      }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // drain the tail refills before the wave ends

  constexpr int kAccRegs = FB * 2 * TB * 2 * 4;  // 128
  // ------------------------------------------------------------------ split K: the last workgroup of a tile adds up
  if (p.ksplit > 1) {
    // Every workgroup of a tile leaves its fp32 accumulators of the live token blocks in the
    // scratch area (write-through stores, completed before its arrival is counted); the one
    // that arrives last reads all slices back in slice order - so the sum does not depend on
    // which one that is - and goes on to the epilogue.  Plain loads suffice: every line has one
    // writer in this launch and no reader before the counter says so.
    float *mine = p.split_ws + (((size_t)q * p.ksplit + slice) * (WF * WT) + wave) * (kAccRegs * 64);
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      if (tb0 + wt * TB + j >= p.tok_blocks) continue;
#pragma unroll
      for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int h = 0; h < 4; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            __hip_atomic_store(mine + (((i * TB + j) * 4 + h) * 4 + e) * 64 + lane, acc[i][h >> 1][j][h & 1][e], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
      unsigned old = atomicAdd(&p.split_counters[q], 1u);
      split_last = old == (unsigned)p.ksplit - 1 ? 1u : 0u;
      if (split_last) p.split_counters[q] = 0;  // ready for the next launch
    }
    __syncthreads();
    if (!split_last) return;
    const float *tile_ws = p.split_ws + ((size_t)q * p.ksplit * (WF * WT) + wave) * (kAccRegs * 64);
    const size_t slice_stride = (size_t)(WF * WT) * (kAccRegs * 64);
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      if (tb0 + wt * TB + j >= p.tok_blocks) continue;
#pragma unroll
      for (int i = 0; i < FB; ++i) {
        float sum[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[r] = 0.f;
        for (int s0 = 0; s0 < p.ksplit; s0 += 4) {  // 4 slices x 16 values in flight
          float v[4][16];
#pragma unroll
          for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              v[u][r] = s0 + u < p.ksplit ? tile_ws[(size_t)(s0 + u) * slice_stride + ((i * TB + j) * 16 + r) * 64 + lane] : 0.f;
#pragma unroll
          for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) sum[r] += v[u][r];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][(r >> 3) & 1][j][(r >> 2) & 1][r & 3] = sum[r];
      }
    }
  }

  // ------------------------------------------------------------------ epilogue
  // lane l: features 4 q .. 4 q + 3 of a 16-feature half, token t16 of a 16-token half
  const int q4 = (lane >> 4) * 4, t16 = lane & 15;
  if (EPI == EPI_STORE) {
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      int tb = tb0 + wt * TB + j;
      if (tb >= p.tok_blocks) continue;
#pragma unroll
      for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int fh = 0; fh < 2; ++fh)
#pragma unroll
          for (int th = 0; th < 2; ++th)
            store4(p.out, p.out_K, tb * 32 + 16 * th + t16, (nb0 + wf * FB + i) * 32 + 16 * fh + q4, acc[i][fh][j][th]);
    }
  } else if (EPI == EPI_SWIGLU) {
    // block 0 = gate, block 1 = up of FFN features [(tile_n*4 + wf)*32, +32)
    float rs_all[TB][2];  // requested together: one round trip for the whole epilogue
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int th = 0; th < 2; ++th) rs_all[j][th] = p.rstd[min(tb0 + wt * TB + j, p.tok_blocks - 1) * 32 + 16 * th + t16];
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      int tb = tb0 + wt * TB + j;
      if (tb >= p.tok_blocks) continue;
#pragma unroll
      for (int th = 0; th < 2; ++th) {
        const int row = tb * 32 + 16 * th + t16;
        const float rs = rs_all[j][th];  // the input rows carry gain only: W (x g r) = r W (x g)
#pragma unroll
        for (int fh = 0; fh < 2; ++fh) {
          f32x4_t v;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float g = acc[0][fh][j][th][e] * rs, u = acc[1][fh][j][th][e] * rs;
            v[e] = g / (1.0f + __expf(-g)) * u;
          }
          store4(p.out, p.out_K, row, (tile_n * 4 + wf) * 32 + 16 * fh + q4, v);
        }
      }
    }
  } else if (EPI == EPI_RESID) {
    // x += W a ; y' = x * gain of the next norm ; sum of squares of these 64 features per token.
    // Padding rows stay zero.  The residual of a token block (8 loads of 1 KiB per wave) is requested one block
    // ahead of the arithmetic that needs it: the epilogue is a chain of memory round trips otherwise.
    f32x4_t old[2][2][FB][2];  // [parity of j][th][i][fh]
    auto xres_at = [&](int tb, int i, int fh, int th) {
      // the residual stream's accumulator order: group [fh][th] of the block, 64 lanes x 4 floats
      return p.xres + (((size_t)tb * p.feat_blocks + (nb0 + wf * FB + i)) * 4 + fh * 2 + th) * 256 + lane * 4;
    };
    auto fetch = [&](int j) {
      const int tb = min(tb0 + wt * TB + j, p.tok_blocks - 1);  // a block past the end rereads the last one (unused)
#pragma unroll
      for (int th = 0; th < 2; ++th)
#pragma unroll
        for (int i = 0; i < FB; ++i)
#pragma unroll
          for (int fh = 0; fh < 2; ++fh) old[j & 1][th][i][fh] = __builtin_nontemporal_load((const f32x4_t *)xres_at(tb, i, fh, th));
    };
    bf16x4_t gg[FB][2];
#pragma unroll
    for (int i = 0; i < FB; ++i)
#pragma unroll
      for (int fh = 0; fh < 2; ++fh) gg[i][fh] = *(const bf16x4_t *)(p.gain + (nb0 + wf * FB + i) * 32 + 16 * fh + q4);
    fetch(0);
    fetch(1);
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      int tb = tb0 + wt * TB + j;
      if (tb >= p.tok_blocks) continue;
#pragma unroll
      for (int th = 0; th < 2; ++th) {
        const int row = tb * 32 + 16 * th + t16;
        const bool live = p.row_ext[row] >= 0;
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < FB; ++i) {
          const int fb = nb0 + wf * FB + i;
#pragma unroll
          for (int fh = 0; fh < 2; ++fh) {
            f32x4_t nw, v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float xn = live ? old[j & 1][th][i][fh][e] + acc[i][fh][j][th][e] : 0.f;
              nw[e] = xn;
              ss += xn * xn;
              v[e] = xn * bf16_to_f32(gg[i][fh].v[e]);
            }
            __builtin_nontemporal_store(nw, (f32x4_t *)xres_at(tb, i, fh, th));
            store4(p.out, p.out_K, row, fb * 32 + 16 * fh + q4, v);
          }
        }
        // the token's 64 features of this wave sit in the four lanes l % 16 == t16
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (lane < 16) p.ssq_part[(size_t)((nb0 + wf * FB) >> 1) * (p.tok_blocks * 32) + row] = ss;
      }
      if (j + 2 < TB) fetch(j + 2);  // into the set this block has just left
    }
  } else {  // EPI_QKV
    const int n0 = tile_n * 256;              // first packed row of this tile
    const int head_in_tile = wf >> 1, ib = (wf & 1) * 32;
    const bool rotary = n0 < p.qd + p.kvd;
    // what the epilogue needs per token is requested up front (one round trip), the rotary table's entries - which
    // wait for the positions - one token half ahead of their use
    int pos_all[TB][2], req_all[TB][2];
    float rs_all[TB][2];
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int th = 0; th < 2; ++th) {
        const int row = min(tb0 + wt * TB + j, p.tok_blocks - 1) * 32 + 16 * th + t16;
        pos_all[j][th] = p.row_pos[row]; req_all[j][th] = p.row_req[row]; rs_all[j][th] = p.rstd[row];
      }
    f32x4_t cs[2][2][2];  // [parity of the token half][fh][cos, sin]
    auto fetch_cs = [&](int h) {  // h = 2 j + th
      if (!rotary) return;
#pragma unroll
      for (int fh = 0; fh < 2; ++fh) {
        const size_t at = (size_t)pos_all[h >> 1][h & 1] * 64 + ib + 16 * fh + q4;
        cs[h & 1][fh][0] = *(const f32x4_t *)(p.cos_tab + at);
        cs[h & 1][fh][1] = *(const f32x4_t *)(p.sin_tab + at);
      }
    };
    fetch_cs(0);
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      int tb = tb0 + wt * TB + j;
#pragma unroll
      for (int th = 0; th < 2; ++th) {
        if (2 * j + th + 1 < 2 * TB) fetch_cs(2 * j + th + 1);
        if (tb >= p.tok_blocks) continue;
        const int row = tb * 32 + 16 * th + t16;
        const int pos = pos_all[j][th], req = req_all[j][th];
        const float rs = rs_all[j][th];
        if (rotary) {
          // q or k: rotate the pair (d, d + 64) by the angle of this position; block 0 holds d, block 1 d + 64
#pragma unroll
          for (int fh = 0; fh < 2; ++fh) {
            const int d0 = ib + 16 * fh + q4;  // d0 .. d0 + 3 and their partners d0 + 64 ..
            const f32x4_t c4 = cs[(2 * j + th) & 1][fh][0], s4 = cs[(2 * j + th) & 1][fh][1];
            f32x4_t lo, hi;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float a = acc[0][fh][j][th][e] * rs, b = acc[1][fh][j][th][e] * rs;
              lo[e] = a * c4[e] - b * s4[e];
              hi[e] = b * c4[e] + a * s4[e];
            }
            if (n0 < p.qd) {
              const int head = (n0 >> 7) + head_in_tile;
              store4(p.out, p.out_K, row, head * 128 + d0, lo);
              store4(p.out, p.out_K, row, head * 128 + 64 + d0, hi);
            } else {
              const int kvh = ((n0 - p.qd) >> 7) + head_in_tile;
              bf16_t *kb = p.Kc + p.geom.off(req, kvh, pos >> 5);  // P(32, 128) of this key block
              *(bf16x4_t *)(kb + frag_offset(pos & 31, d0, 128)) = pack4(lo[0], lo[1], lo[2], lo[3]);
              *(bf16x4_t *)(kb + frag_offset(pos & 31, 64 + d0, 128)) = pack4(hi[0], hi[1], hi[2], hi[3]);
            }
          }
        } else {
          // v: feature d of kv head, key `pos` -> value tile slot
          const int kvh = ((n0 - p.qd - p.kvd) >> 7) + head_in_tile;
          bf16_t *vb = p.Vc + p.geom.off(req, kvh, pos >> 5);
          int m, khh;
          const int e = vtile_slot_of_key(pos & 31, &m, &khh);
#pragma unroll
          for (int i = 0; i < FB; ++i)
#pragma unroll
            for (int fh = 0; fh < 2; ++fh)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int d = ib + i * 64 + 16 * fh + q4 + r;
                vb[(size_t)(m * 4 + (d >> 5)) * kTileElems + (khh * 32 + (d & 31)) * 8 + e] = f2bf_dev(acc[i][fh][j][th][r] * rs);
              }
        }
      }
    }
  }
}

}  // namespace

// ----------------------------------------------------------------------------
// host launchers
// ----------------------------------------------------------------------------
hipError_t mfma_pack_weight(const bf16_t *src0, const bf16_t *src1, const bf16_t *src2, int rows0,
                            int rows1, bf16_t *dst, int N, int K, int mode, int I, hipStream_t s) {
  size_t chunks = (size_t)N * K / 8;
  k_pack_weight<<<(unsigned)((chunks + 255) / 256), 256, 0, s>>>(src0, src1, src2, rows0, rows1, dst, N, K, mode, I);
  return hipGetLastError();
}

hipError_t mfma_prefill_begin(const bf16_t *hidden_in, float *xres, const bf16_t *gain, bf16_t *y, float *rstd,
                              const int *row_ext, int rows, int H, float eps, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (rows <= 64) k_add_norm<0, 1><<<rows, 256, 0, s>>>(hidden_in, xres, nullptr, gain, y, rstd, nullptr, row_ext, H, eps);
  else k_add_norm<0, 8><<<rows / 8, 256, 0, s>>>(hidden_in, xres, nullptr, gain, y, rstd, nullptr, row_ext, H, eps);
  return hipGetLastError();
}

hipError_t mfma_prefill_end(const float *xres, const bf16_t *delta_bf, bf16_t *hidden_out, const int *row_ext,
                            int rows, int H, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  float *x = const_cast<float *>(xres);
  if (rows <= 64) k_add_norm<1, 1><<<rows, 256, 0, s>>>(nullptr, x, delta_bf, nullptr, nullptr, nullptr, hidden_out, row_ext, H, 0.f);
  else k_add_norm<1, 8><<<rows / 8, 256, 0, s>>>(nullptr, x, delta_bf, nullptr, nullptr, nullptr, hidden_out, row_ext, H, 0.f);
  return hipGetLastError();
}

hipError_t mfma_rstd(const float *ssq_part, float *rstd, const int *row_ext, int rows, int H, float eps, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  k_rstd<<<(rows + 255) / 256, 256, 0, s>>>(ssq_part, rstd, row_ext, rows, H / 64, 1.0f / (float)H, eps);
  return hipGetLastError();
}

constexpr int kGemmSplitCus = 256;    // workgroups that run at once (one per CU)
constexpr int kGemmSplitUnits = 512;  // most (tile, slice) pairs of a split GEMM

// largest scratch a split GEMM can use: kGemmSplitUnits partial tiles of 256 x 256 fp32
size_t mfma_gemm_split_ws_bytes() { return (size_t)kGemmSplitUnits * (WF * WT) * (FB * TB * 16 * 64) * sizeof(float); }

// the (epilogue, class) pairs a block uses
#define HYP_GEMM_VARIANTS(X)                                                                        \
  X(EPI_QKV, HYP_K_GEMM_QKV) X(EPI_RESID, HYP_K_GEMM_O) X(EPI_SWIGLU, HYP_K_GEMM_GATEUP)            \
  X(EPI_RESID, HYP_K_GEMM_DOWN) X(EPI_STORE, HYP_K_GEMM_DOWN)

hipError_t mfma_gemm_init() {
  hipError_t e = hipSuccess;
#define X(EPI, CLS) \
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_gemm<EPI, CLS>, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS);
  HYP_GEMM_VARIANTS(X)
#undef X
  return e;
}

hipError_t mfma_gemm(int epi, int cls, const bf16_t *X, const bf16_t *W, int rows, int N, int K, bf16_t *out,
                     int out_K, const GemmEpilogue &ep, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  GemmParams p = {};
  p.X = X; p.W = W; p.KT = K / 16; p.tok_blocks = rows / 32; p.feat_blocks = N / 32;
  int tiles_t = (p.tok_blocks + XB - 1) / XB, tiles_n = p.feat_blocks / NBK;
  p.gm = tiles_t < 8 ? tiles_t : 8;
  p.n_tiles = tiles_t * tiles_n;
  p.out = out; p.out_K = out_K;
  p.Kc = ep.Kc; p.Vc = ep.Vc; p.geom = ep.geom; p.qd = ep.qd; p.kvd = ep.kvd;
  p.cos_tab = ep.cos_tab; p.sin_tab = ep.sin_tab; p.row_pos = ep.row_pos; p.row_req = ep.row_req;
  p.rstd = ep.rstd; p.xres = ep.xres; p.gain = ep.gain; p.row_ext = ep.row_ext; p.ssq_part = ep.ssq_part;
  p.tiles_grid = (p.n_tiles + 7) / 8 * 8;
  // Few output tiles (short prompts): split the K loop over c workgroups per tile when a simple
  // model says it pays.  Rounds of 256 workgroups times the share of a tile's K loop each one
  // runs, against what the slices then write and read back (the token blocks that exist, fp32,
  // at the ~3 TB/s write-through stores and the gather reach) plus the extra round trips.
  // Slices are whole numbers of stages, at least 2 NST of them each.
  p.ksplit = 1;
  if (ep.split_ws && ep.split_counters && p.n_tiles <= kGemmSplitMaxTiles) {
    const int nsteps = p.KT / KTS;
    const double tile_us = K * 0.0267;  // 256 x 256 x K on one CU at the rate the big GEMMs run at
    const int live_blocks = p.tok_blocks < XB ? p.tok_blocks : XB;
    double best = 0.9 * (double)((p.n_tiles + kGemmSplitCus - 1) / kGemmSplitCus) * tile_us;  // a split has to win clearly
    for (int c = 2; c <= 32 && p.n_tiles * c <= kGemmSplitUnits; ++c) {
      if (nsteps % c != 0 || nsteps / c < 2 * NST) continue;
      double rounds = (double)((p.n_tiles * c + kGemmSplitCus - 1) / kGemmSplitCus);
      double partial_mb = (double)p.n_tiles * c * live_blocks * NBK * 4096.0 * 2 / 1e6;
      double t = rounds * tile_us / c + partial_mb / 3.0 + 5.0;
      if (t < best) { best = t; p.ksplit = c; }
    }
  }
  p.split_ws = ep.split_ws; p.split_counters = ep.split_counters;
  // 64 rounds of 256 tiles or more: the last sixteenth of the rounds is drawn from a counter by twice as many
  // workgroups as it has tiles, so that an XCD can take up to a quarter of it.  (Gate/up at 64 K tokens, 140 rounds:
  // 2.3 % faster.  With 20 - 30 rounds the drawn tiles' lost L2 neighbourhood and the tile granularity cost more than
  // the balance brings: down projection 1.7 % slower.)
  p.n_static = 0; p.pool_wgs = 0;
  if (p.ksplit == 1 && ep.split_counters && p.n_tiles >= 64 * kGemmSplitCus) {
    const int rounds = p.n_tiles / kGemmSplitCus;
    const int pool_rounds = (rounds + 8) / 16;
    p.n_static = (rounds - pool_rounds) * kGemmSplitCus;
    p.pool_wgs = (2 * (p.n_tiles - p.n_static) + 7) / 8 * 8;
    p.tiles_grid = p.n_static + p.pool_wgs;
  }
  int grid = p.tiles_grid * p.ksplit;
  bool launched = false;
#define X(EPI, CLS) \
  if (!launched && epi == EPI && cls == CLS) { k_gemm<EPI, CLS><<<grid, WF * WT * 64, GEMM_LDS, s>>>(p); launched = true; }
  HYP_GEMM_VARIANTS(X)
#undef X
  if (!launched) return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace hyp
