// Attention kernels of the MFMA path: causal grouped-query attention over the
// prompt (flash-style: the score matrix is never written), and split-KV
// attention of one new token per request against the cache (bandwidth-bound).
// Both follow the GQA-with-RoPE sub-layer of Sec. III-A; RoPE was already
// applied to q and to the cached keys by the QKV epilogue.
#include <type_traits>
#include "mfma_common.h"
#include "mfma_kernels.h"

namespace hyp {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// The two halves of a wave exchanged in the vector ALU (v_permlane32_swap: lanes 32..63 of its first operand
// trade places with lanes 0..31 of its second), not through the LDS crossbar and its wait: with both operands v
// the first result holds v's lower half in both halves, the second its upper half.
struct HalfPair { float lo, hi; };
__device__ __forceinline__ HalfPair both_halves(float v) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return {__uint_as_float(r[0]), __uint_as_float(r[1])};
}
__device__ __forceinline__ float xhalf_max(float v) { const HalfPair h = both_halves(v); return fmaxf(h.lo, h.hi); }
__device__ __forceinline__ float xhalf_sum(float v) { const HalfPair h = both_halves(v); return h.lo + h.hi; }

__device__ __forceinline__ bf16x8_t probs_operand(const float *p /*16*/, int m) {
  // MFMA step m of the P V product contracts keys 16m + 8(e/4) + 4hh + e%4: registers 8m .. 8m+7
  bf16x8_t r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (__bf16)p[8 * m + e];
  return r;
}

// ----------------------------------------------------------------------------
// Prefill.  One workgroup = one KV head x one tile of 64 query rows.  It has two
// waves per query head of the group (32 query rows each), so a K / V stage of 64
// keys (32 KiB, already in fragment order) is fetched once into LDS by direct
// loads and read by all 2G waves.  Per wave: S^T = K Q^T (keys on the MFMA M axis,
// so a lane owns one query column and the softmax reductions stay inside a lane
// plus one cross-half exchange), online softmax in fp32, O^T += V^T P^T.
//
// The loop is software-pipelined over stages: the scores of stage s + 1 are
// formed (MFMA) in the same straight-line block in which the probabilities of
// stage s are exponentiated, summed and rounded (VALU), so the matrix pipe works
// under the softmax arithmetic, which is the longer of the two; three LDS buffers
// keep stage s (values), s + 1 (keys, then values) and s + 2 (arriving) apart.
// The running maximum is only moved - and the accumulators rescaled - when it has
// grown by more than 2^8 in some row: probabilities stay below 256, sums and
// outputs are formed against the same reference, and the rescale leaves the loop's
// steady state.  Only the last stage of a tile touches the diagonal and is masked.
// ----------------------------------------------------------------------------
constexpr int kKvStageKeys = 64;
constexpr int kKvStageBytes = 2 * 16384;  // per 32 keys: 8 K tiles + 8 V tiles
constexpr int kKvBufs = 3;
constexpr int kAttnPrefillLds = kKvBufs * kKvStageBytes;
constexpr float kRescaleLog2 = 8.0f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// max of three: one v_max3_f32, because this file is compiled with -fno-honor-nans (scores are never
// NaN; otherwise the compiler puts a canonicalising self-maximum in front of every fmaxf operand).
// Not inline assembly: the compiler's hazard logic must see that the operands come out of MFMAs.
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <int G>
__global__ void __launch_bounds__(128 * G) k_attn_prefill(const bf16_t *__restrict__ q,
                                                      const bf16_t *__restrict__ Kc,
                                                      const bf16_t *__restrict__ Vc, CacheGeom geom,
                                                      bf16_t *__restrict__ out,
                                                      const PrefillTile *__restrict__ tiles,
                                                      const int *__restrict__ req_len, int nq) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  // wave-uniform values in scalar registers: the LDS destination of a direct load has to be uniform, and a wave index
  // the compiler takes for divergent turns every such load into a loop over lanes
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, hh = lane >> 5, tl = lane & 31;
  constexpr int nw = 2 * G;  // waves per workgroup
  const PrefillTile tile = tiles[blockIdx.x];
  const int kvh = blockIdx.y;
  const int head = kvh * G + (wave >> 1);
  const int tq = wave & 1;                 // which 32-row block of the tile
  const int qblk = tile.qblk0 + tq;        // its index inside the request
  const int qd = nq * 128;
  const int len = req_len[tile.req];
  const int n_kb = min(tile.qblk0 + 2, (len + 31) >> 5);  // 32-key blocks the tile needs
  const int n_st = (n_kb + 1) >> 1;                        // 64-key stages; every wave of the tile needs all of them
  const int rb = (tile.row0 >> 5) + tq;
  const float c = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)
  const int qpos = qblk * 32 + tl;

  bf16x8_t qf[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt)
    qf[dt] = *(const bf16x8_t *)(q + ((size_t)rb * (qd >> 4) + head * 8 + dt) * kTileElems + lane * 8);

  f32x16_t o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // A stage is the pair of key blocks 2 st, 2 st + 1: 16 KiB contiguous in either cache layout
  // (the block count of a request is even and a page holds four blocks).  Its offset is uniform
  // over the workgroup and, with a paged cache, costs a table lookup: it is formed one stage
  // before the loads that use it are issued.
  auto stage_off = [&](int st) { return geom.off(tile.req, kvh, min(st * 2, geom.key_blocks - 2)); };
  auto issue = [&](size_t off, int buf) {
    // 32 tiles of 1 KiB: [key block 0: 8 K, 8 V][key block 1: 8 K, 8 V]; the second
    // block of the last stage may lie past the tile's need but is inside the cache
    // wave w fetches tiles w, w + nw, ...; with 2, 4 or 8 waves everything about a tile but w itself is known at
    // compile time, and the loop unrolls into straight scalar address arithmetic
    if constexpr (nw == 2 || nw == 4 || nw == 8) {
      constexpr int per8 = 8 / nw;
#pragma unroll
      for (int j = 0; j < 32 / nw; ++j) {
        const int hi = j / per8, lo = nw * (j % per8);  // tile t = 8 hi + lo + wave
        const bf16_t *src = ((hi & 1) ? Vc : Kc) + off + (size_t)(hi >> 1) * (32 * 128) + (size_t)(lo + wave) * kTileElems + lane * 8;
        __builtin_amdgcn_global_load_lds((gbl_ptr_t *)src, (lds_ptr_t *)(lds + buf * kKvStageBytes + (8 * hi + lo + wave) * 1024), 16, 0, 0);
      }
    } else {
      for (int t = wave; t < 32; t += nw) {
        const bf16_t *src = ((t & 8) ? Vc : Kc) + off + (size_t)(t >> 4) * (32 * 128) + (size_t)(t & 7) * kTileElems + lane * 8;
        __builtin_amdgcn_global_load_lds((gbl_ptr_t *)src, (lds_ptr_t *)(lds + buf * kKvStageBytes + t * 1024), 16, 0, 0);
      }
    }
  };
  // scores of both 32-key blocks of the stage in `buf`: two independent accumulator chains
  auto scores = [&](int buf, f32x16_t &a0, f32x16_t &a1) {
    const char *base = lds + buf * kKvStageBytes + lane * 16;
#pragma unroll
    for (int r = 0; r < 16; ++r) { a0[r] = 0.f; a1[r] = 0.f; }
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      bf16x8_t k0 = *(const bf16x8_t *)(base + dt * 1024);
      bf16x8_t k1 = *(const bf16x8_t *)(base + 16384 + dt * 1024);
      a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[dt], a0, 0, 0, 0);
      a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[dt], a1, 0, 0, 0);
    }
  };
  // move the running maximum when some row's has grown by more than 2^kRescaleLog2 (always on the
  // first stage, where the old maximum is -inf and the factor 0)
  auto follow_max = [&](float mx) {
    float m_new = fmaxf(m_run, xhalf_max(mx));  // finite from the first stage on: key 0 is visible to every row
    if (__any((m_new - m_run) * c > kRescaleLog2)) {
      float alpha = fast_exp2((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      m_run = m_new;
    }
  };
  // O^T += V^T P^T for the stage in `buf`
  auto values = [&](int buf, const bf16x8_t *pf) {
    const char *base = lds + buf * kKvStageBytes + lane * 16;
#pragma unroll
    for (int h2 = 0; h2 < 4; ++h2)   // (key block, MFMA step) pairs
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        bf16x8_t vf = *(const bf16x8_t *)(base + (h2 >> 1) * 16384 + (8 + (h2 & 1) * 4 + db) * 1024);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[h2], o[db], 0, 0, 0);
      }
  };

  issue(stage_off(0), 0);
  if (n_st > 1) issue(stage_off(1), 1);
  size_t off_next = stage_off(2);
  __builtin_amdgcn_s_waitcnt(0x0070);  // my loads of the first two stages have landed
  __syncthreads();
  f32x16_t s0, s1;
  scores(0, s0, s1);
  float mx = max3(s0[0], s1[0], -INFINITY);
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = max3(mx, s0[r], s1[r]);

  // A wave issues in order: an MFMA that finds the matrix pipe still busy with the previous one
  // holds up the arithmetic behind it.  So each iteration is laid out as two phases in which
  // every MFMA (32 cycles) is followed by about as many cycles of independent VALU work:
  //   phase 1   scores of stage st + 1 (16 MFMAs)  |  exponentials and rounding of stage st
  //   phase 2   P V of stage st (16 MFMAs)         |  row sums of stage st, maxima of stage st + 1
  // The scheduling-group builtins fix that interleaving; left alone the compiler bunches the MFMAs.
  bf16x8_t pf[4];
  int buf = 0;  // buffer of stage st
  // one stage of the loop: consumes the scores c0, c1 of stage st, leaves those of stage st + 1 in n0, n1
  auto stage = [&](int st, const f32x16_t &c0, const f32x16_t &c1, f32x16_t &n0, f32x16_t &n1) {
    const int buf1 = buf + 1 == kKvBufs ? 0 : buf + 1, buf2 = buf1 + 1 == kKvBufs ? 0 : buf1 + 1;
    if (st + 2 < n_st) issue(off_next, buf2);  // over stage st - 1, which every wave has left
    // Fragments come from LDS in batches of four, each batch requested one group of four MFMAs ahead
    // (while LDS-direct loads are in flight the compiler only emits full LDS waits, so a batch is
    // awaited as a whole, long after it was requested).
    const char *kbase = lds + buf1 * kKvStageBytes + lane * 16;
    const char *vbase = lds + buf * kKvStageBytes + lane * 16 + 8 * 1024;
    auto kfrag = [&](int i) { return *(const bf16x8_t *)(kbase + (i & 1) * 16384 + (i >> 1) * 1024); };  // i = 2 dt + key block
    auto vfrag = [&](int i) { return *(const bf16x8_t *)(vbase + (i >> 3) * 16384 + (i & 7) * 1024); };  // i = 8 key block + 4 step + d block
    bf16x8_t fr[2][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) fr[0][u] = kfrag(u);
    __builtin_amdgcn_sched_barrier(0);
    follow_max(mx);
    const float mc = m_run * c;
    // ---- phase 1: scores of stage st + 1 | probabilities of stage st
#pragma unroll
    for (int r = 0; r < 16; ++r) { n0[r] = 0.f; n1[r] = 0.f; }
    float p[32];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int g = i >> 2, u = i & 3;
      if (i & 1) n1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][u], qf[i >> 1], n1, 0, 0, 0);
      else n0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][u], qf[i >> 1], n0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (u == 0) {  // the next batch: keys of the next group, or the first values of phase 2
#pragma unroll
        for (int w = 0; w < 4; ++w) fr[(g + 1) & 1][w] = g < 3 ? kfrag(4 * (g + 1) + w) : vfrag(w);
      }
      // two probabilities and their rounding per MFMA: registers 2 i and 2 i + 1 of the 32 scores
      {
        const int r0 = 2 * i, r1 = 2 * i + 1;
        p[r0] = fast_exp2((r0 < 16 ? c0[r0] : c1[r0 - 16]) * c - mc);
        p[r1] = fast_exp2((r1 < 16 ? c0[r1] : c1[r1 - 16]) * c - mc);
        pf[r0 >> 3][r0 & 7] = (__bf16)p[r0];
        pf[r0 >> 3][r1 & 7] = (__bf16)p[r1];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- phase 2: P V of stage st | row sums of stage st, maxima of stage st + 1
    float rowsum = 0.f;
    mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int g = i >> 2, u = i & 3;
      o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][u], pf[i >> 2], o[i & 3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (u == 0 && g < 3) {
#pragma unroll
        for (int w = 0; w < 4; ++w) fr[(g + 1) & 1][w] = vfrag(4 * (g + 1) + w);
      }
      rowsum += p[2 * i];
      rowsum += p[2 * i + 1];
      mx = max3(mx, n0[i], n1[i]);
      // an empty statement that "uses" both: without it the two chains are sunk as a whole below the loop's last
      // MFMA (they are only needed there), and the matrix pipe runs phase 2 alone
      asm volatile("" : "+v"(rowsum), "+v"(mx));
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += rowsum;
    buf = buf1;
    // a paged cache answers this with a scalar load; issued here, it completes under the wait below -
    // outstanding during the phases it would turn every LDS wait into a full one
    off_next = stage_off(st + 3);
    __builtin_amdgcn_s_waitcnt(0x0070);  // my loads of stage st + 2 landed, my LDS reads of stage st done
    __syncthreads();
  };
  // two stages per trip with the roles of the two accumulator pairs swapped, so that no stage ends by copying
  // the next scores into the current ones; an odd stage count starts with a single stage (one copy per tile)
  {
    f32x16_t t0, t1;
    int st = 0;
    if ((n_st - 1) & 1) {
      stage(0, s0, s1, t0, t1);
      s0 = t0; s1 = t1;
      st = 1;
    }
    for (; st + 1 < n_st; st += 2) {
      stage(st, s0, s1, t0, t1);
      stage(st + 1, t0, t1, s0, s1);
    }
  }
  // last stage: the only one that touches the diagonal (a block past the tile's need is fully
  // masked here: its keys lie after every row)
  {
    const int kb0 = (n_st - 1) * 2;
    float p[32];
    mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      int koff = 8 * (r >> 2) + 4 * hh + (r & 3);
      p[r] = (kb0 * 32 + koff > qpos) ? -INFINITY : s0[r];
      p[16 + r] = (kb0 * 32 + 32 + koff > qpos) ? -INFINITY : s1[r];
      mx = fmaxf(mx, fmaxf(p[r], p[16 + r]));
    }
    follow_max(mx);
    const float mc = m_run * c;
    float rowsum = 0.f;
#pragma unroll
    for (int r = 0; r < 32; ++r) {
      p[r] = fast_exp2(p[r] * c - mc);
      rowsum += p[r];
    }
    l_run += rowsum;
    pf[0] = probs_operand(p, 0); pf[1] = probs_operand(p, 1); pf[2] = probs_operand(p + 16, 0); pf[3] = probs_operand(p + 16, 1);
    values(buf, pf);
  }

  // normalise and store into P(rows, qd): lane owns query tl, features 8g + 4hh + e of each d block
  float inv = 1.0f / xhalf_sum(l_run);
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      int f0 = head * 128 + db * 32;
      size_t off = ((size_t)rb * (qd >> 4) + ((f0 + 8 * g) >> 4)) * kTileElems + (((g & 1) << 5) + tl) * 8 + hh * 4;
      *(bf16x4_t *)(out + off) = pack4(o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv,
                                       o[db][4 * g + 3] * inv);
    }
}

// ----------------------------------------------------------------------------
// Decode.  The query buffer holds, per (request, KV head), the G query heads as
// rows 0..G-1 of a P(32, 128) block (other rows zero), so the same MFMA shape
// serves: S^T[key, head] = K q^T.  K and V fragments go straight from HBM into
// registers (fragment order = operand order), 16 wave loads of 1 KiB per 32-key
// block, no LDS.  One wave owns a chunk of chunk_keys keys of one
// (request, KV head).  Every chunk
// writes (max, sum, unnormalised output) and a second small kernel merges the
// chunks of a head in index order, so the result does not depend on scheduling.
// part layout: [request][head][chunk][130] = {m, l, o[128]}
// ----------------------------------------------------------------------------
constexpr int kPartStride = 130;

template <int NSETS>
__global__ void __launch_bounds__(64) k_attn_decode(const bf16_t *__restrict__ qdec,
                                                    const bf16_t *__restrict__ Kc,
                                                    const bf16_t *__restrict__ Vc, CacheGeom geom,
                                                    const int *__restrict__ lens, float *__restrict__ part,
                                                    int nq, int G, int max_chunks, int chunk_keys) {
  const int lane = threadIdx.x, hh = lane >> 5, tl = lane & 31;
  const int chunk = blockIdx.x, kvh = blockIdx.y, req = blockIdx.z;
  const int nkeys = lens[req] + 1;  // the new token's key is already in the cache
  const int k0 = chunk * chunk_keys;
  if (k0 >= nkeys) return;
  const int kb_begin = k0 >> 5;
  const int kb_end = min((k0 + chunk_keys) >> 5, (nkeys + 31) >> 5);
  const float c = kLog2e * 0.08838834764831845f;
  const int key_limit = nkeys;

  bf16x8_t qf[8];
  const bf16_t *qb = qdec + ((size_t)req * geom.nkv + kvh) * (32 * 128);
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) qf[dt] = *(const bf16x8_t *)(qb + dt * kTileElems + lane * 8);

  f32x16_t o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  bf16x8_t kS[NSETS][8], vS[NSETS][8];
  auto load_block = [&](int kb, bf16x8_t *kf, bf16x8_t *vf) {
    const bf16_t *kblk = Kc + geom.off(req, kvh, kb) + lane * 8;
    const bf16_t *vblk = Vc + geom.off(req, kvh, kb) + lane * 8;
#pragma unroll
    for (int t = 0; t < 8; ++t) kf[t] = __builtin_nontemporal_load((const bf16x8_t *)(kblk + t * kTileElems));
#pragma unroll
    for (int t = 0; t < 8; ++t) vf[t] = __builtin_nontemporal_load((const bf16x8_t *)(vblk + t * kTileElems));
  };
  auto compute_block = [&](int kb, const bf16x8_t *kf, const bf16x8_t *vf) {
    f32x16_t s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[dt], qf[dt], s, 0, 0, 0);
    float p[16];
    float mx = -INFINITY;
    if ((kb + 1) * 32 > key_limit) {  // only the last block of a chunk can hold keys past the end
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int kpos = kb * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
        p[r] = kpos < key_limit ? s[r] : -INFINITY;
        mx = fmaxf(mx, p[r]);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = s[r];
        mx = fmaxf(mx, p[r]);
      }
    }
    mx = xhalf_max(mx);
    float m_new = fmaxf(m_run, mx);  // finite: the first key of a chunk is always valid and comes first
    float mc = m_new * c, rowsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      p[r] = fast_exp2(p[r] * c - mc);
      rowsum += p[r];
    }
    if (__any(m_new > m_run)) {  // the accumulators are rescaled only when some maximum moved
      float alpha = fast_exp2((m_run - m_new) * c);  // 0 on the first block
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      m_run = m_new;
    }
    l_run += rowsum;
    bf16x8_t pf0 = probs_operand(p, 0), pf1 = probs_operand(p, 1);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db], pf0, o[db], 0, 0, 0);
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[4 + db], pf1, o[db], 0, 0, 0);
    }
  };
  // NSETS register sets: the loads of the next NSETS - 1 blocks are in flight while one is used.
  // Block kb_begin + j lives in set j % NSETS.  No load sits under a condition between two
  // uses: the compiler counts outstanding loads per path, and a load that may or may not have
  // been issued makes it wait for everything.  So: a steady loop of whole groups of NSETS
  // blocks, then one of NSETS straight-line endings chosen by the number of loads still to issue.
  const int n = kb_end - kb_begin;
  if (n < NSETS - 1) {
    for (int j = 0; j < n; ++j) {
      load_block(kb_begin + j, kS[0], vS[0]);
      compute_block(kb_begin + j, kS[0], vS[0]);
    }
  } else {
#pragma unroll
    for (int u = 0; u < NSETS - 1; ++u) load_block(kb_begin + u, kS[u], vS[u]);
    int i = 0;
    for (; i + 2 * NSETS - 1 <= n; i += NSETS) {
#pragma unroll
      for (int u = 0; u < NSETS; ++u) {
        load_block(kb_begin + i + u + NSETS - 1, kS[(u + NSETS - 1) % NSETS], vS[(u + NSETS - 1) % NSETS]);
        __builtin_amdgcn_sched_barrier(0);
        compute_block(kb_begin + i + u, kS[u], vS[u]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    const int r = n - (i + NSETS - 1);  // loads still to issue, 0 .. NSETS - 1
    auto ending = [&](auto R) {
      constexpr int kR = decltype(R)::value;
#pragma unroll
      for (int u = 0; u < kR + NSETS - 1; ++u) {
        if (u < kR) load_block(kb_begin + i + u + NSETS - 1, kS[(u + NSETS - 1) % NSETS], vS[(u + NSETS - 1) % NSETS]);
        __builtin_amdgcn_sched_barrier(0);
        compute_block(kb_begin + i + u, kS[u % NSETS], vS[u % NSETS]);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (r == 0) ending(std::integral_constant<int, 0>());
    else if (r == 1) ending(std::integral_constant<int, 1>());
    else if (r == 2 || NSETS < 4) ending(std::integral_constant<int, NSETS < 3 ? 1 : 2>());
    else ending(std::integral_constant<int, NSETS < 4 ? 1 : 3>());
  }
  // lanes tl < G hold real heads
  float l_tot = xhalf_sum(l_run);
  if (tl < G) {
    int head = kvh * G + tl;
    float *dst = part + (((size_t)req * nq + head) * max_chunks + chunk) * kPartStride;
    if (hh == 0) { dst[0] = m_run; dst[1] = l_tot; }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[2 + db * 32 + 8 * (r >> 2) + 4 * hh + (r & 3)] = o[db][r];
  }
}

// One 128-thread block per (request, query head): combine its chunks in chunk
// order.  Lane i of the first wave takes chunk i (max, sum -> weight); then thread
// d accumulates output feature d over all chunks, eight loads in flight at a time.
__global__ void __launch_bounds__(128) k_attn_decode_merge(const float *__restrict__ part,
                                                           const int *__restrict__ lens,
                                                           bf16_t *__restrict__ out, int nq,
                                                           int max_chunks, int chunk_keys) {
  __shared__ float wgt[64];
  __shared__ float lsum;
  const int head = blockIdx.x, req = blockIdx.y, d = threadIdx.x;
  const int n_chunks = (lens[req] + 1 + chunk_keys - 1) / chunk_keys;  // <= 64 by the host's choice of chunk_keys
  const float c = kLog2e * 0.08838834764831845f;
  const float *src = part + ((size_t)req * nq + head) * max_chunks * kPartStride;
  // One round trip: the first 16 chunks' outputs, the maxima and the sums are requested for every
  // chunk slot the buffer has, without waiting for the request's length; slots past n_chunks hold
  // whatever an earlier step left there and are dropped below without entering any arithmetic.
  float v0[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) v0[u] = u < max_chunks ? src[u * kPartStride + 2 + d] : 0.f;
  float mi_raw = 0.f, li_raw = 0.f;
  if (d < 64 && d < max_chunks) { mi_raw = src[d * kPartStride]; li_raw = src[d * kPartStride + 1]; }
  if (d < 64) {
    float mi = d < n_chunks ? mi_raw : -INFINITY;
    float li = d < n_chunks ? li_raw : 0.f;
    float m = mi;
    for (int o2 = 32; o2 > 0; o2 >>= 1) m = fmaxf(m, __shfl_xor(m, o2, 64));
    float w = d < n_chunks ? exp2f((mi - m) * c) : 0.f;
    wgt[d] = w;
    float wl = w * li, tot = 0.f;
    for (int i = 0; i < n_chunks; ++i) tot += __shfl(wl, i, 64);  // chunk order
    if (d == 0) lsum = tot;
  }
  __syncthreads();
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < 16; ++u)
    if (u < n_chunks) acc += wgt[u] * v0[u];
  int i = 16;
  for (; i + 8 <= n_chunks; i += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[(i + u) * kPartStride + 2 + d];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += wgt[i + u] * v[u];
  }
  for (; i < n_chunks; ++i) acc += wgt[i] * src[i * kPartStride + 2 + d];
  out[frag_offset(req, head * 128 + d, nq * 128)] = f2bf_dev(acc / lsum);
}

}  // namespace

hipError_t mfma_attn_prefill(const bf16_t *q, const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom,
                             bf16_t *out, const PrefillTile *tiles, int n_tiles, const int *req_len,
                             int nq, int nkv, hipStream_t s) {
  if (n_tiles == 0) return hipSuccess;
  const int G = nq / nkv;
  const dim3 grid(n_tiles, nkv);
  switch (G) {
    case 1: k_attn_prefill<1><<<grid, 128, kAttnPrefillLds, s>>>(q, Kc, Vc, geom, out, tiles, req_len, nq); break;
    case 2: k_attn_prefill<2><<<grid, 256, kAttnPrefillLds, s>>>(q, Kc, Vc, geom, out, tiles, req_len, nq); break;
    case 3: k_attn_prefill<3><<<grid, 384, kAttnPrefillLds, s>>>(q, Kc, Vc, geom, out, tiles, req_len, nq); break;
    case 4: k_attn_prefill<4><<<grid, 512, kAttnPrefillLds, s>>>(q, Kc, Vc, geom, out, tiles, req_len, nq); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t mfma_attn_init() {
  hipError_t e = hipFuncSetAttribute((const void *)k_attn_prefill<1>, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnPrefillLds);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_attn_prefill<2>, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnPrefillLds);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_attn_prefill<3>, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnPrefillLds);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_attn_prefill<4>, hipFuncAttributeMaxDynamicSharedMemorySize, kAttnPrefillLds);
  return e;
}

size_t mfma_attn_decode_part_floats(int nq, int batch, int max_chunks) {
  return (size_t)batch * nq * max_chunks * kPartStride;
}

hipError_t mfma_attn_decode(const bf16_t *qdec, const bf16_t *Kc, const bf16_t *Vc, CacheGeom geom,
                            const int *lens, float *part, bf16_t *out, int nq, int nkv, int batch,
                            int max_chunks, int chunk_keys, hipStream_t s) {
  int G = nq / nkv;
  k_attn_decode<2><<<dim3(max_chunks, nkv, batch), 64, 0, s>>>(qdec, Kc, Vc, geom, lens, part, nq, G, max_chunks, chunk_keys);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_attn_decode_merge<<<dim3(nq, batch), 128, 0, s>>>(part, lens, out, nq, max_chunks, chunk_keys);
  return hipGetLastError();
}

}  // namespace hyp
