// Data layout and small device helpers shared by the MFMA kernels (bf16 stages).
//
// Every matrix operand of an MFMA contraction lives in HBM in *fragment order*:
// a [R, K] matrix (K = contraction index) is cut into tiles of 32 rows x 16 k;
// a tile is 1 KiB = 64 lanes x 16 bytes, and lane l holds row (l % 32),
// k = (l / 32) * 8 .. + 8.  That is exactly the register fragment that
// v_mfma_f32_32x32x16_bf16 wants from lane l for either operand, so a tile
// moves HBM -> (LDS ->) registers as one fully coalesced 1 KiB wave access with
// no shuffles, swizzles or bank conflicts.  Tiles of one 32-row block are
// contiguous along K.  "P(R,K)" below names this layout.
//
// Accumulator blocks are kept with *features on the MFMA M axis and tokens on
// the N axis*: lane l of a 32x32 block then owns token (l % 32) and the features
// 8g + 4(l/32) + j (g, j = 0..3) in register 4g + j, so four consecutive
// features of one token sit in one lane -> an 8-byte store straight into the
// fragment-order activation of the next GEMM, 512 contiguous bytes per wave
// store.
#pragma once

#include "common.h"

namespace hyp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((address_space(3))) void lds_ptr_t;
typedef __attribute__((address_space(1))) const void gbl_ptr_t;

struct __attribute__((aligned(8))) bf16x4_t { bf16_t v[4]; };
struct __attribute__((aligned(16))) u16x8_t { bf16_t v[8]; };

constexpr int kTileElems = 512;  // 32 rows x 16 k

// element offset of (row, k) in P(R, K)
__host__ __device__ inline size_t frag_offset(size_t row, size_t k, size_t K) {
  return ((row >> 5) * (K >> 4) + (k >> 4)) * kTileElems + ((((k & 15) >> 3) << 5) + (row & 31)) * 8 +
         (k & 7);
}

// The fp32 residual stream of a prefill is kept in *accumulator order*, "A(T', H)":
// blocks of 32 tokens x 32 features of 4 KiB, stored as 4 groups [fh][th] (feature half,
// token half) of 64 lanes x 4 floats - lane l of group [fh][th] holds token 16 th + l % 16,
// features 16 fh + 4 (l / 16) + 0..3, i.e. the four registers of that lane's 16 x 16 MFMA
// output [fh][th] of the block.  A GEMM epilogue then reads and writes the residual with
// 1 KiB contiguous wave accesses.
__host__ __device__ inline size_t acc_offset(size_t row, size_t col, size_t H) {
  const size_t f = col & 31, t = row & 31;
  const size_t group = ((f >> 4) << 1) | (t >> 4), lane = (((f >> 2) & 3) << 4) | (t & 15);
  return (((row >> 5) * (H >> 5) + (col >> 5)) * 4 + group) * 256 + lane * 4 + (f & 3);
}

// Value tile of the KV cache: 32 feature rows (d) x 16 keys, contraction over
// keys.  Inside a 32-key block, MFMA step m (0/1), lane half hh and slot e read
// key 16m + 8(e/4) + 4hh + e%4, which is the order in which the probabilities
// come out of the score accumulators.
__host__ __device__ inline int vtile_slot_of_key(int key_in_block, int *m, int *hh) {
  int w = key_in_block & 15;
  *m = key_in_block >> 4;
  *hh = (w & 7) >> 2;
  return ((w >> 3) << 2) + (w & 3);
}

// Geometry of the caches of one layer.  Contiguous form: [request][kv_head][key_block][8 KiB].
// Paged form (page_table != nullptr): the cache is a pool of pages of kPageKeys keys,
// [page][kv_head][kPageBlocks][8 KiB], and page_table[request * pages_per_req + i] names the page
// that holds keys [kPageKeys * i, kPageKeys * (i + 1)) of that request.  Either way a 32-key block
// of one KV head is 8 KiB contiguous and a page keeps a head's blocks together, so the kernels
// stream the same tiles; only the block address differs.
constexpr int kPageKeys = 128, kPageBlocks = kPageKeys / 32;
struct CacheGeom {
  int nkv;
  int key_blocks;  // ceil(max_seq / 32)
  const int *page_table;
  int pages_per_req;
  __host__ __device__ size_t block_elems() const { return 32 * 128; }
  __host__ __device__ size_t off(int req, int kvh, int kb) const {
    if (page_table) {
      const int page = page_table[req * pages_per_req + kb / kPageBlocks];
      return (((size_t)page * nkv + kvh) * kPageBlocks + kb % kPageBlocks) * (32 * 128);
    }
    return (((size_t)req * nkv + kvh) * key_blocks + kb) * (32 * 128);
  }
};

__device__ inline bf16_t f2bf_dev(float f) { return f32_to_bf16(f); }

__device__ inline bf16x4_t pack4(float a, float b, float c, float d) {
  bf16x4_t r;
  r.v[0] = f2bf_dev(a); r.v[1] = f2bf_dev(b); r.v[2] = f2bf_dev(c); r.v[3] = f2bf_dev(d);
  return r;
}

}  // namespace hyp
