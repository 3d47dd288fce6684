// Host runtime behind the C ABI of hyp_stage.h: argument checking, workspace
// carving, weight repacking, the block loop (Eq. 1) over the stage's range
// (Eq. 6) for prefill and for KV-cached decode steps.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <string>
#include <unordered_set>
#include <vector>

#include "common.h"
#include "mfma_kernels.h"

using namespace hyp;

// Per-step temporaries of stage_decode_step_noalloc(): one array per GPU, shared by every
// stage and every call on that GPU until the process ends.  Host code never uses this name as
// an address; it uses what hipGetSymbolAddress() returns for the current device.
constexpr size_t kNoAllocScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

namespace {

thread_local std::string g_create_error = "";

// device address of `scratch` on each GPU, looked up once per device by stage_create
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch_of_current_device(void **out) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct LayerPtrs {
  size_t g1, wqkv, wo, g2, wgu, wd;  // offsets into the workspace
};

// Where everything lives inside the caller's workspace.
struct Layout {
  std::vector<LayerPtrs> layers;
  size_t Kc = 0, Vc = 0, kv_layer_stride = 0;  // per-layer stride in bytes
  size_t cos_tab = 0, sin_tab = 0;
  size_t xres = 0, y = 0, qkv = 0, attn = 0, gu = 0, m = 0;
  size_t tok_req = 0, tok_pos = 0, lens = 0, iota = 0;
  // MFMA path only
  size_t q = 0, delta = 0, row_ext = 0, row_pos = 0, row_req = 0, tiles = 0, req_len = 0, row_ext_dec = 0, qdec = 0,
         partial = 0, attn_part = 0, counters = 0, gemm_counters = 0, ssq = 0, rstd = 0, ssq_part = 0, gemm_ws = 0;
  size_t kv_bytes = 0;  // bytes of each of Kc, Vc over all layers
  int rows_cap = 0;     // internal rows the scratch holds
  int key_blocks = 0;   // 32-key blocks per (request, kv head)
  int max_chunks = 0;   // decode attention chunks per head
  int chunk_keys = 128; // keys per chunk
  GemvPlan g_qkv, g_o, g_gu, g_d;  // how the four skinny GEMMs of a decode step are cut into workgroups
  size_t partial_bytes = 0, attn_part_bytes = 0, counters_bytes = 0;
  // paged KV cache (HYP_FLAG_PAGED_KV): pages per layer of the pool, table entries per request
  size_t page_table = 0;
  int pool_pages = 0, pages_per_req = 0;
  size_t total = 0;
};

// The temporaries one decode step of the MFMA path works in (everything but weights, caches,
// position tables and cached lengths): either carved from the stage's workspace or from the
// per-GPU static array.
struct DecScratch {
  float *xres = nullptr, *ssq = nullptr, *partial = nullptr, *attn_part = nullptr;
  unsigned *counters = nullptr;
  bf16_t *y = nullptr, *attn = nullptr, *m = nullptr, *qdec = nullptr;
};

// The MFMA kernels cover bf16 stages shaped like the models of Table I: head_dim
// 128, at most 4 query heads per KV head, even head counts and widths that tile
// by 256; at most 32 resident requests (one token block per decode step).
bool mfma_applies(const hyp_stage_config_t &c) {
  if (c.dtype != HYP_BF16 || (c.flags & HYP_FLAG_PLAIN_KERNELS)) return false;
  if (c.head_dim != 128) return false;
  int G = c.n_q_heads / c.n_kv_heads;
  if (G > 4) return false;
  if (c.n_q_heads % 2 || c.n_kv_heads % 2) return false;
  if (c.hidden % 256 || c.ffn_dim % 256) return false;
  if (c.max_batch > 32) return false;
  return true;
}

int round_up(int v, int m) { return (v + m - 1) / m * m; }

size_t elem_size(const hyp_stage_config_t &c) { return c.dtype == HYP_BF16 ? 2 : 4; }

int64_t max_rows(const hyp_stage_config_t &c) {
  return c.max_prefill_tokens > c.max_batch ? c.max_prefill_tokens : (int64_t)c.max_batch;
}

hyp_status_t check_config(const hyp_stage_config_t *c, int32_t l_start, int32_t l_end,
                          std::string &err) {
  if (!c) { err = "config is NULL"; return HYP_EINVAL; }
  if (l_start < 0 || l_start >= l_end) { err = "need 0 <= l_start < l_end"; return HYP_EINVAL; }
  if (c->dtype != HYP_F32 && c->dtype != HYP_BF16) { err = "dtype must be HYP_F32 or HYP_BF16"; return HYP_EINVAL; }
  if (c->kv_pool_pages != 0 && !(c->flags & HYP_FLAG_PAGED_KV)) { err = "kv_pool_pages must be 0 unless HYP_FLAG_PAGED_KV is set"; return HYP_EINVAL; }
  if (c->flags & ~(HYP_FLAG_PLAIN_KERNELS | HYP_FLAG_NO_GRAPH | HYP_FLAG_PAGED_KV)) { err = "unknown flag"; return HYP_EINVAL; }
  if (c->hidden < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 || c->ffn_dim < 1 ||
      c->max_batch < 1 || c->max_seq < 1 || c->max_prefill_tokens < 1) {
    err = "sizes must be positive"; return HYP_ESHAPE;
  }
  if (c->n_q_heads % c->n_kv_heads != 0) { err = "n_kv_heads must divide n_q_heads"; return HYP_ESHAPE; }
  if (c->head_dim % 2 != 0) { err = "head_dim must be even (RoPE pairs)"; return HYP_ESHAPE; }
  if (c->head_dim > 256) { err = "head_dim above 256 is not supported"; return HYP_ESHAPE; }
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) { err = "rms_eps must be >= 0 and rope_base > 0"; return HYP_ESHAPE; }
  if (c->max_prefill_tokens > (int64_t)c->max_batch * c->max_seq) {
    err = "max_prefill_tokens exceeds max_batch * max_seq"; return HYP_ESHAPE;
  }
  if (c->max_prefill_tokens > (int64_t)1 << 30) { err = "max_prefill_tokens too large"; return HYP_ESHAPE; }
  if ((c->flags & HYP_FLAG_PAGED_KV) && !mfma_applies(*c)) {
    err = "HYP_FLAG_PAGED_KV needs a stage that runs the MFMA kernels (bf16, head_dim 128, widths in multiples of 256)";
    return HYP_ESHAPE;
  }
  if ((uint64_t)c->kv_pool_pages > (uint64_t)1 << 24) { err = "kv_pool_pages too large"; return HYP_ESHAPE; }
  return HYP_OK;
}

void make_layout(const hyp_stage_config_t &c, int n_layers, Layout &L) {
  size_t es = elem_size(c);
  size_t H = c.hidden, qd = (size_t)c.n_q_heads * c.head_dim, kvd = (size_t)c.n_kv_heads * c.head_dim;
  size_t I = c.ffn_dim, R = (size_t)max_rows(c);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.layers.resize(n_layers);
  for (int l = 0; l < n_layers; ++l) {
    LayerPtrs &p = L.layers[l];
    p.g1 = take(es * H);
    p.wqkv = take(es * (qd + 2 * kvd) * H);
    p.wo = take(es * H * qd);
    p.g2 = take(es * H);
    p.wgu = take(es * 2 * I * H);
    p.wd = take(es * H * I);
  }
  if (mfma_applies(c)) {
    // every request's rows are padded to a multiple of 64 (one query tile)
    L.rows_cap = round_up((int)c.max_prefill_tokens + 63 * c.max_batch, 64);
    if (L.rows_cap < 64) L.rows_cap = 64;
    R = L.rows_cap;
    L.key_blocks = round_up(c.max_seq, 64) / 32;
    if (c.flags & HYP_FLAG_PAGED_KV) {
      L.pages_per_req = (L.key_blocks + kPageBlocks - 1) / kPageBlocks;
      L.pool_pages = c.kv_pool_pages ? (int)c.kv_pool_pages : c.max_batch * L.pages_per_req;
      L.kv_layer_stride = align_up(es * (size_t)L.pool_pages * c.n_kv_heads * kPageBlocks * 32 * 128);
    } else {
      L.kv_layer_stride = align_up(es * (size_t)c.max_batch * c.n_kv_heads * L.key_blocks * 32 * 128);
    }
    L.kv_bytes = L.kv_layer_stride * n_layers;
    L.Kc = take(L.kv_bytes);
    L.Vc = take(L.kv_bytes);
    size_t tab = sizeof(float) * (size_t)L.key_blocks * 32 * 64;
    L.cos_tab = take(tab);
    L.sin_tab = take(tab);
    L.xres = take(sizeof(float) * R * H);
    L.y = take(es * R * H);
    L.q = take(es * R * qd);
    L.attn = take(es * R * qd);
    L.m = take(es * R * I);
    L.delta = take(es * R * H);
    L.rstd = take(sizeof(float) * R);
    L.ssq_part = take(sizeof(float) * R * (H / 64));
    L.row_ext = take(sizeof(int) * R);
    L.row_pos = take(sizeof(int) * R);
    L.row_req = take(sizeof(int) * R);
    L.tiles = take(sizeof(PrefillTile) * (R / 64));
    L.req_len = take(sizeof(int) * c.max_batch);
    L.lens = take(sizeof(int) * c.max_batch);
    L.row_ext_dec = take(sizeof(int) * 32);
    L.qdec = take(es * (size_t)c.max_batch * c.n_kv_heads * 32 * 128);
    L.g_qkv = mfma_gemv_plan(HYP_K_GEMV_QKV, (int)(qd + 2 * kvd), (int)H, c.max_batch);
    L.g_o = mfma_gemv_plan(HYP_K_GEMV_O, (int)H, (int)qd, c.max_batch);
    L.g_gu = mfma_gemv_plan(HYP_K_GEMV_GATEUP, (int)(2 * I), (int)H, c.max_batch);
    L.g_d = mfma_gemv_plan(HYP_K_GEMV_DOWN, (int)H, (int)I, c.max_batch);
    // fp32 partial sums of the K slices: room for the GEMM with the most of them
    const size_t pf = std::max(std::max(mfma_gemv_partial_floats(L.g_qkv, (int)(qd + 2 * kvd), (int)H), mfma_gemv_partial_floats(L.g_o, (int)H, (int)qd)),
                               std::max(mfma_gemv_partial_floats(L.g_gu, (int)(2 * I), (int)H), mfma_gemv_partial_floats(L.g_d, (int)H, (int)I)));
    L.partial_bytes = sizeof(float) * pf;
    L.partial = take(L.partial_bytes);
    L.chunk_keys = mfma_decode_chunk_keys(c.max_seq, c.max_batch * c.n_kv_heads);
    L.max_chunks = (c.max_seq + L.chunk_keys - 1) / L.chunk_keys;
    L.attn_part_bytes = sizeof(float) * mfma_attn_decode_part_floats(c.n_q_heads, c.max_batch, L.max_chunks);
    L.attn_part = take(L.attn_part_bytes);
    L.counters_bytes = sizeof(unsigned) * (2 * I / 64 + (qd + 2 * kvd) / 64 + H / 32);
    L.counters = take(L.counters_bytes);
    L.gemm_counters = take(sizeof(unsigned) * kGemmSplitMaxTiles);  // zeroed together with `counters`
    L.ssq = take(sizeof(float) * 32 * (H / 32));
    L.gemm_ws = take(mfma_gemm_split_ws_bytes());
    if (L.pages_per_req) L.page_table = take(sizeof(int) * (size_t)c.max_batch * L.pages_per_req);
    L.total = off;
    return;
  }
  L.kv_layer_stride = align_up(es * (size_t)c.max_batch * kvd * c.max_seq);
  L.Kc = take(L.kv_layer_stride * n_layers);
  L.Vc = take(L.kv_layer_stride * n_layers);
  size_t tab = sizeof(float) * (size_t)c.max_seq * (c.head_dim / 2);
  L.cos_tab = take(tab);
  L.sin_tab = take(tab);
  L.xres = take(sizeof(float) * R * H);
  L.y = take(es * R * H);
  L.qkv = take(es * R * (qd + 2 * kvd));
  L.attn = take(es * R * qd);
  L.gu = take(es * R * 2 * I);
  L.m = take(es * R * I);
  L.tok_req = take(sizeof(int) * R);
  L.tok_pos = take(sizeof(int) * R);
  L.lens = take(sizeof(int) * c.max_batch);
  L.iota = take(sizeof(int) * c.max_batch);
  L.total = off;
}

}  // namespace

struct hyp_stage {
  hyp_stage_config_t cfg;
  int l_start, l_end, n_layers;
  Dims dm;
  hipStream_t stream;
  bool bf16, mfma;
  char *ws;
  Layout L;
  // pinned host staging for the per-call index arrays, and the event that says
  // the previous upload has been consumed
  int *h_stage;
  size_t h_stage_ints;
  hipEvent_t upload_done;
  bool upload_pending;
  std::vector<int> lens;  // host mirror of the cached lengths
  std::vector<int> pages;  // paged cache: host mirror of the page table [max_batch][pages_per_req], -1 = none
  // optional per-kernel-class timing with HIP events on the stage's stream
  struct ProfSlot { hipEvent_t a, b; int cls; };
  std::vector<ProfSlot> prof;
  size_t prof_used = 0;
  uint32_t prof_mask = 0;
  bool prof_off = false;  // set around calls that must not create events
  // recorded decode steps (kernel arguments baked in), replayed when they match
  struct DecGraph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    int batch = 0;
    void *out = nullptr;
  };
  std::vector<DecGraph> dec_graphs;
  hipStream_t cap_stream = nullptr;  // recording only (the null stream cannot be captured); nothing runs on it
  // MFMA path: where a decode step keeps its temporaries - in the workspace, or (for
  // stage_decode_step_noalloc) in the GPU's static array when `static_bytes` of it suffice
  DecScratch dec_ws, dec_static;
  size_t static_bytes = 0;
  int batch;
  bool prefilled;
  std::string err;
};

namespace {

hyp_status_t fail(hyp_stage *st, hyp_status_t code, const std::string &msg) {
  if (st) st->err = msg; else g_create_error = msg;
  return code;
}

#define HIP_TRY(st, expr)                                                                        \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess)                                                                        \
      return fail(st, HYP_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_));           \
  } while (0)

// Launch `expr`; when kernel class `cls` is being profiled, bracket it with a
// pair of events recorded on the stage's stream.
hipError_t prof_begin(hyp_stage *st, int cls, int *slot) {
  *slot = -1;
  if (!(st->prof_mask & (1u << cls)) || st->prof_off) return hipSuccess;
  if (st->prof_used == st->prof.size()) {
    hyp_stage::ProfSlot ps;
    hipError_t e = hipEventCreate(&ps.a);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&ps.b);
    if (e != hipSuccess) { (void)hipEventDestroy(ps.a); return e; }
    st->prof.push_back(ps);
  }
  *slot = (int)st->prof_used++;
  st->prof[*slot].cls = cls;
  return hipEventRecord(st->prof[*slot].a, st->stream);
}
hipError_t prof_end(hyp_stage *st, int slot) {
  return slot < 0 ? hipSuccess : hipEventRecord(st->prof[slot].b, st->stream);
}
#define PROF(st, cls, expr)                         \
  do {                                              \
    int slot_;                                      \
    HIP_TRY(st, prof_begin(st, cls, &slot_));       \
    HIP_TRY(st, expr);                              \
    HIP_TRY(st, prof_end(st, slot_));               \
  } while (0)

template <typename T> T *at(hyp_stage *st, size_t off) { return reinterpret_cast<T *>(st->ws + off); }

// Copy the caller's matrices into the workspace: wq|wk|wv stacked into one
// [qd+2kvd, H] matrix and gate|up into one [2I, H] matrix.
hyp_status_t copy_weights(hyp_stage *st, const hyp_layer_weights_t *layers) {
  size_t es = st->bf16 ? 2 : 4;
  const Dims &d = st->dm;
  for (int l = 0; l < st->n_layers; ++l) {
    const hyp_layer_weights_t &w = layers[l];
    const void *ptrs[] = {w.attn_norm_g, w.wq, w.wk, w.wv, w.wo, w.ffn_norm_g, w.w_gate, w.w_up, w.w_down};
    for (const void *p : ptrs)
      if (!p) return fail(st, HYP_EINVAL, "a weight pointer of layer " + std::to_string(l) + " is NULL");
    const LayerPtrs &p = st->L.layers[l];
    auto cp = [&](size_t dst, const void *src, size_t bytes) {
      return hipMemcpyAsync(st->ws + dst, src, bytes, hipMemcpyDeviceToDevice, st->stream);
    };
    size_t H = d.H;
    HIP_TRY(st, cp(p.g1, w.attn_norm_g, es * H));
    HIP_TRY(st, cp(p.wqkv, w.wq, es * d.qd * H));
    HIP_TRY(st, cp(p.wqkv + es * d.qd * H, w.wk, es * d.kvd * H));
    HIP_TRY(st, cp(p.wqkv + es * (d.qd + d.kvd) * H, w.wv, es * d.kvd * H));
    HIP_TRY(st, cp(p.wo, w.wo, es * H * d.qd));
    HIP_TRY(st, cp(p.g2, w.ffn_norm_g, es * H));
    HIP_TRY(st, cp(p.wgu, w.w_gate, es * (size_t)d.I * H));
    HIP_TRY(st, cp(p.wgu + es * (size_t)d.I * H, w.w_up, es * (size_t)d.I * H));
    HIP_TRY(st, cp(p.wd, w.w_down, es * H * (size_t)d.I));
  }
  return HYP_OK;
}

// MFMA path: repack every matrix into fragment order (with the row permutations
// its epilogue relies on); gains are copied as they are.
hyp_status_t pack_weights_mfma(hyp_stage *st, const hyp_layer_weights_t *layers) {
  const Dims &d = st->dm;
  hipStream_t s = st->stream;
  for (int l = 0; l < st->n_layers; ++l) {
    const hyp_layer_weights_t &w = layers[l];
    const void *ptrs[] = {w.attn_norm_g, w.wq, w.wk, w.wv, w.wo, w.ffn_norm_g, w.w_gate, w.w_up, w.w_down};
    for (const void *p : ptrs)
      if (!p) return fail(st, HYP_EINVAL, "a weight pointer of layer " + std::to_string(l) + " is NULL");
    const LayerPtrs &p = st->L.layers[l];
    HIP_TRY(st, hipMemcpyAsync(st->ws + p.g1, w.attn_norm_g, 2 * (size_t)d.H, hipMemcpyDeviceToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + p.g2, w.ffn_norm_g, 2 * (size_t)d.H, hipMemcpyDeviceToDevice, s));
    HIP_TRY(st, mfma_pack_weight((const bf16_t *)w.wq, (const bf16_t *)w.wk, (const bf16_t *)w.wv, d.qd, d.kvd,
                                 at<bf16_t>(st, p.wqkv), d.qd + 2 * d.kvd, d.H, PACK_QKV, 0, s));
    HIP_TRY(st, mfma_pack_weight((const bf16_t *)w.wo, nullptr, nullptr, d.H, 0, at<bf16_t>(st, p.wo), d.H, d.qd,
                                 PACK_PLAIN, 0, s));
    HIP_TRY(st, mfma_pack_weight((const bf16_t *)w.w_gate, (const bf16_t *)w.w_up, nullptr, d.I, d.I,
                                 at<bf16_t>(st, p.wgu), 2 * d.I, d.H, PACK_GATEUP, d.I, s));
    HIP_TRY(st, mfma_pack_weight((const bf16_t *)w.w_down, nullptr, nullptr, d.H, 0, at<bf16_t>(st, p.wd), d.H, d.I,
                                 PACK_PLAIN, 0, s));
  }
  // Cache blocks are read 32 keys at a time; slots that were never written must
  // hold finite numbers because a masked probability of 0 still multiplies them.
  HIP_TRY(st, mfma_fill_zero(st->ws + st->L.Kc, st->L.kv_bytes, s));
  HIP_TRY(st, mfma_fill_zero(st->ws + st->L.Vc, st->L.kv_bytes, s));
  HIP_TRY(st, mfma_fill_zero(st->ws + st->L.qdec, 2 * (size_t)d.max_batch * d.nkv * 32 * 128, s));
  HIP_TRY(st, mfma_fill_zero(st->ws + st->L.counters, st->L.ssq - st->L.counters, s));
  return HYP_OK;
}

CacheGeom cache_geom(const hyp_stage *st) {
  CacheGeom g;
  g.nkv = st->dm.nkv;
  g.key_blocks = st->L.key_blocks;
  g.pages_per_req = st->L.pages_per_req;
  g.page_table = st->L.pages_per_req ? reinterpret_cast<const int *>(st->ws + st->L.page_table) : nullptr;
  return g;
}

// prefill through the MFMA kernels; `rows` internal rows (multiple of 64)
hyp_status_t run_prefill_mfma(hyp_stage *st, const void *hidden_in, void *hidden_out, int rows, int n_tiles) {
  const Dims &d = st->dm;
  hipStream_t s = st->stream;
  const Layout &L = st->L;
  float *xres = at<float>(st, L.xres);
  bf16_t *y = at<bf16_t>(st, L.y), *q = at<bf16_t>(st, L.q), *attn = at<bf16_t>(st, L.attn);
  bf16_t *m = at<bf16_t>(st, L.m), *delta = at<bf16_t>(st, L.delta);
  const int *row_ext = at<int>(st, L.row_ext);
  CacheGeom geom = cache_geom(st);
  float *rstd = at<float>(st, L.rstd), *ssq_part = at<float>(st, L.ssq_part);
  PROF(st, HYP_K_ADD_NORM, mfma_prefill_begin((const bf16_t *)hidden_in, xres, at<bf16_t>(st, L.layers[0].g1), y, rstd,
                                               row_ext, rows, d.H, d.eps, s));
  GemmEpilogue split;  // scratch of GEMMs that split their K loop (short prompts leave few output tiles)
  split.split_ws = at<float>(st, L.gemm_ws); split.split_counters = at<unsigned>(st, L.gemm_counters);
  for (int l = 0; l < st->n_layers; ++l) {
    const LayerPtrs &p = L.layers[l];
    const bool last = l + 1 == st->n_layers;
    GemmEpilogue e = split;
    e.Kc = at<bf16_t>(st, L.Kc + L.kv_layer_stride * l);
    e.Vc = at<bf16_t>(st, L.Vc + L.kv_layer_stride * l);
    e.geom = geom; e.qd = d.qd; e.kvd = d.kvd;
    e.cos_tab = at<float>(st, L.cos_tab); e.sin_tab = at<float>(st, L.sin_tab);
    e.row_pos = at<int>(st, L.row_pos); e.row_req = at<int>(st, L.row_req);
    e.rstd = rstd;
    PROF(st, HYP_K_GEMM_QKV, mfma_gemm(EPI_QKV, HYP_K_GEMM_QKV, y, at<bf16_t>(st, p.wqkv), rows, d.qd + 2 * d.kvd, d.H, q, d.qd, e, s));
    PROF(st, HYP_K_ATTN_PREFILL, mfma_attn_prefill(q, e.Kc, e.Vc, geom, attn, at<PrefillTile>(st, L.tiles), n_tiles,
                                  at<int>(st, L.req_len), d.nq, d.nkv, s));
    // residual add, the next norm's gain and its statistics all happen in the epilogue
    GemmEpilogue r = split;
    r.xres = xres; r.row_ext = row_ext; r.ssq_part = ssq_part;
    r.gain = at<bf16_t>(st, p.g2);
    PROF(st, HYP_K_GEMM_O, mfma_gemm(EPI_RESID, HYP_K_GEMM_O, attn, at<bf16_t>(st, p.wo), rows, d.H, d.qd, y, d.H, r, s));
    PROF(st, HYP_K_ADD_NORM, mfma_rstd(ssq_part, rstd, row_ext, rows, d.H, d.eps, s));
    GemmEpilogue g = split;
    g.rstd = rstd;
    PROF(st, HYP_K_GEMM_GATEUP, mfma_gemm(EPI_SWIGLU, HYP_K_GEMM_GATEUP, y, at<bf16_t>(st, p.wgu), rows, 2 * d.I, d.H, m, d.I, g, s));
    if (!last) {
      r.gain = at<bf16_t>(st, L.layers[l + 1].g1);
      PROF(st, HYP_K_GEMM_DOWN, mfma_gemm(EPI_RESID, HYP_K_GEMM_DOWN, m, at<bf16_t>(st, p.wd), rows, d.H, d.I, y, d.H, r, s));
      PROF(st, HYP_K_ADD_NORM, mfma_rstd(ssq_part, rstd, row_ext, rows, d.H, d.eps, s));
    } else {
      PROF(st, HYP_K_GEMM_DOWN, mfma_gemm(EPI_STORE, HYP_K_GEMM_DOWN, m, at<bf16_t>(st, p.wd), rows, d.H, d.I, delta, d.H, split, s));
      PROF(st, HYP_K_ADD_NORM, mfma_prefill_end(xres, delta, (bf16_t *)hidden_out, row_ext, rows, d.H, s));
    }
  }
  return HYP_OK;
}

// One decode step through the MFMA kernels (a single block of 32 token rows):
// 1 + 5 launches per block, every reduction finished inside the kernel that
// produced it.
hyp_status_t decode_step_mfma(hyp_stage *st, hipStream_t s, const DecScratch &sc, const void *hidden_in, void *hidden_out,
                              bool begin, bool layers) {
  const Dims &d = st->dm;
  const Layout &L = st->L;
  DecGemv base;
  base.partial = sc.partial;
  base.partial_floats = L.partial_bytes / sizeof(float);
  base.counters = sc.counters;
  base.batch = st->batch;
  base.eps = d.eps;
  base.H = d.H;
  base.xres = sc.xres;
  float *ssq = sc.ssq;
  bf16_t *y = sc.y, *attn = sc.attn, *m = sc.m;
  CacheGeom geom = cache_geom(st);
  if (begin)
    PROF(st, HYP_K_ADD_NORM, mfma_dec_begin((const bf16_t *)hidden_in, base.xres, at<bf16_t>(st, L.layers[0].g1), y, ssq,
                                             d.H, st->batch, s));
  for (int l = 0; layers && l < st->n_layers; ++l) {
    const LayerPtrs &p = L.layers[l];
    bf16_t *Kc = at<bf16_t>(st, L.Kc + L.kv_layer_stride * l), *Vc = at<bf16_t>(st, L.Vc + L.kv_layer_stride * l);
    DecGemv a = base;
    a.W = at<bf16_t>(st, p.wqkv); a.x = y; a.N = d.qd + 2 * d.kvd; a.K = d.H; a.plan = L.g_qkv;
    a.ssq_in = ssq; a.n_ssq = d.H / (l == 0 ? 64 : 32 * L.g_d.fbw);  // written by the opening kernel / the previous down GEMM
    a.lens = at<int>(st, L.lens); a.cos_tab = at<float>(st, L.cos_tab); a.sin_tab = at<float>(st, L.sin_tab);
    a.qdec = sc.qdec; a.Kc = Kc; a.Vc = Vc; a.geom = geom; a.nq = d.nq; a.nkv = d.nkv;
    PROF(st, HYP_K_GEMV_QKV, mfma_dec_gemv(DEC_QKV, HYP_K_GEMV_QKV, a, s));
    PROF(st, HYP_K_ATTN_DECODE, mfma_attn_decode(a.qdec, Kc, Vc, geom, a.lens, sc.attn_part,
                                                 attn, d.nq, d.nkv, st->batch,
                                                 L.max_chunks, L.chunk_keys, s));
    DecGemv o = base;
    o.W = at<bf16_t>(st, p.wo); o.x = attn; o.N = d.H; o.K = d.qd; o.plan = L.g_o;
    o.gain = at<bf16_t>(st, p.g2); o.y_out = y; o.ssq_out = ssq;
    PROF(st, HYP_K_GEMV_O, mfma_dec_gemv(DEC_RESID, HYP_K_GEMV_O, o, s));
    DecGemv g = base;
    g.W = at<bf16_t>(st, p.wgu); g.x = y; g.N = 2 * d.I; g.K = d.H; g.plan = L.g_gu;
    g.ssq_in = ssq; g.n_ssq = d.H / (32 * L.g_o.fbw); g.m_out = m; g.I = d.I;
    PROF(st, HYP_K_GEMV_GATEUP, mfma_dec_gemv(DEC_SWIGLU, HYP_K_GEMV_GATEUP, g, s));
    DecGemv w = base;
    w.W = at<bf16_t>(st, p.wd); w.x = m; w.N = d.H; w.K = d.I; w.plan = L.g_d;
    if (l + 1 < st->n_layers) {
      w.gain = at<bf16_t>(st, L.layers[l + 1].g1); w.y_out = y; w.ssq_out = ssq;
      PROF(st, HYP_K_GEMV_DOWN, mfma_dec_gemv(DEC_RESID, HYP_K_GEMV_DOWN, w, s));
    } else {
      w.hidden_out = (bf16_t *)hidden_out;
      w.lens_advance = at<int>(st, L.lens);
      PROF(st, HYP_K_GEMV_DOWN, mfma_dec_gemv(DEC_FINAL, HYP_K_GEMV_DOWN, w, s));
    }
  }
  return HYP_OK;
}

void drop_decode_graph(hyp_stage::DecGraph &g) {
  if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (g.graph) (void)hipGraphDestroy(g.graph);
  g.exec = nullptr;
  g.graph = nullptr;
}

// The launches of a decode step are latency-bound next to ~0.1 ms of streaming
// per block, so the step is recorded into a HIP graph (kernel nodes only) the
// first time a (batch, output buffer) pair is seen and replayed afterwards;
// while kernel classes are being timed, or when the caller is itself capturing
// the stream, it is launched kernel by kernel instead.
hyp_status_t run_decode_mfma(hyp_stage *st, const void *hidden_in, void *hidden_out) {
  hipStream_t s = st->stream;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  HIP_TRY(st, hipStreamIsCapturing(s, &cap));
  bool use_graph = st->prof_mask == 0 && cap == hipStreamCaptureStatusNone && !(st->cfg.flags & HYP_FLAG_NO_GRAPH);
  if (!use_graph) return decode_step_mfma(st, s, st->dec_ws, hidden_in, hidden_out, true, true);
  // the first kernel reads the caller's input and stays outside the recording, so a
  // new input address every step does not force a new graph
  hyp_status_t rc0 = decode_step_mfma(st, s, st->dec_ws, hidden_in, hidden_out, true, false);
  if (rc0 != HYP_OK) return rc0;
  // a few recorded graphs, keyed by what is baked into their kernel arguments
  hyp_stage::DecGraph *g = nullptr;
  for (auto &c : st->dec_graphs)
    if (c.batch == st->batch && c.out == hidden_out) g = &c;
  if (!g) {
    if (st->dec_graphs.size() >= 4) {
      drop_decode_graph(st->dec_graphs.front());
      st->dec_graphs.erase(st->dec_graphs.begin());
    }
    hyp_stage::DecGraph n;
    n.batch = st->batch; n.out = hidden_out;
    if (!st->cap_stream) HIP_TRY(st, hipStreamCreateWithFlags(&st->cap_stream, hipStreamNonBlocking));
    HIP_TRY(st, hipStreamBeginCapture(st->cap_stream, hipStreamCaptureModeThreadLocal));
    hyp_status_t rc = decode_step_mfma(st, st->cap_stream, st->dec_ws, hidden_in, hidden_out, false, true);
    hipError_t e = hipStreamEndCapture(st->cap_stream, &n.graph);
    if (rc != HYP_OK) { drop_decode_graph(n); return rc; }
    if (e != hipSuccess) { drop_decode_graph(n); return fail(st, HYP_EDEVICE, std::string("hipStreamEndCapture: ") + hipGetErrorString(e)); }
    e = hipGraphInstantiate(&n.exec, n.graph, nullptr, nullptr, 0);
    if (e != hipSuccess) { drop_decode_graph(n); return fail(st, HYP_EDEVICE, std::string("hipGraphInstantiate: ") + hipGetErrorString(e)); }
    st->dec_graphs.push_back(n);
    g = &st->dec_graphs.back();
  }
  HIP_TRY(st, hipGraphLaunch(g->exec, s));
  return HYP_OK;
}

// rows tokens through every block with the shape-generic kernels
template <typename T>
hyp_status_t run_plain(hyp_stage *st, const void *hidden_in, void *hidden_out, int rows,
                       const int *tok_req, const int *tok_pos) {
  const Dims &d = st->dm;
  hipStream_t s = st->stream;
  float *xres = at<float>(st, st->L.xres);
  T *y = at<T>(st, st->L.y), *qkv = at<T>(st, st->L.qkv), *attn = at<T>(st, st->L.attn);
  T *gu = at<T>(st, st->L.gu), *m = at<T>(st, st->L.m);
  const float *ct = at<float>(st, st->L.cos_tab), *sn = at<float>(st, st->L.sin_tab);
  HIP_TRY(st, plain_load_hidden<T>((const T *)hidden_in, xres, (size_t)rows * d.H, s));
  for (int l = 0; l < st->n_layers; ++l) {
    const LayerPtrs &p = st->L.layers[l];
    T *Kc = at<T>(st, st->L.Kc + st->L.kv_layer_stride * l);
    T *Vc = at<T>(st, st->L.Vc + st->L.kv_layer_stride * l);
    HIP_TRY(st, plain_rmsnorm<T>(xres, at<T>(st, p.g1), y, rows, d.H, d.eps, s));
    HIP_TRY(st, (plain_gemm_nt<T, T>(y, at<T>(st, p.wqkv), qkv, rows, d.qd + 2 * d.kvd, d.H, false, s)));
    HIP_TRY(st, plain_rope_cache<T>(qkv, tok_req, tok_pos, ct, sn, Kc, Vc, rows, d, s));
    HIP_TRY(st, plain_attention<T>(qkv, tok_req, tok_pos, Kc, Vc, attn, rows, d, s));
    HIP_TRY(st, (plain_gemm_nt<T, float>(attn, at<T>(st, p.wo), xres, rows, d.H, d.qd, true, s)));
    HIP_TRY(st, plain_rmsnorm<T>(xres, at<T>(st, p.g2), y, rows, d.H, d.eps, s));
    HIP_TRY(st, (plain_gemm_nt<T, T>(y, at<T>(st, p.wgu), gu, rows, 2 * d.I, d.H, false, s)));
    HIP_TRY(st, plain_swiglu<T>(gu, m, rows, d.I, s));
    HIP_TRY(st, (plain_gemm_nt<T, float>(m, at<T>(st, p.wd), xres, rows, d.H, d.I, true, s)));
  }
  HIP_TRY(st, plain_store_hidden<T>(xres, (T *)hidden_out, (size_t)rows * d.H, s));
  return HYP_OK;
}

// paged cache: the first key of request b in [0, n_keys) that has no page, or -1
int first_key_without_page(const hyp_stage *st, int b, int n_keys) {
  const int ppr = st->L.pages_per_req;
  for (int i = 0; i * kPageKeys < n_keys; ++i)
    if (i >= ppr || st->pages[(size_t)b * ppr + i] < 0) return i * kPageKeys;
  return -1;
}

hyp_status_t upload_page_table(hyp_stage *st) {
  HIP_TRY(st, hipMemcpyAsync(st->ws + st->L.page_table, st->pages.data(), sizeof(int) * st->pages.size(),
                             hipMemcpyHostToDevice, st->stream));
  HIP_TRY(st, hipStreamSynchronize(st->stream));  // the host mirror may change right after
  return HYP_OK;
}

hyp_status_t wait_upload(hyp_stage *st) {
  if (st->upload_pending) {
    HIP_TRY(st, hipEventSynchronize(st->upload_done));
    st->upload_pending = false;
  }
  return HYP_OK;
}

// Handles this library has created and not yet destroyed.  Every entry point looks its
// argument up here first, so a stale or foreign pointer (a stage destroyed twice, say) is
// refused with HYP_EINVAL instead of being dereferenced.
std::mutex g_live_mu;
std::unordered_set<const hyp_stage *> g_live;
bool is_live(const hyp_stage *st) {
  std::lock_guard<std::mutex> lock(g_live_mu);
  return g_live.count(st) != 0;
}
#define LIVE_OR_RETURN(st)                                                         \
  do {                                                                             \
    if (!(st)) return fail(nullptr, HYP_EINVAL, "stage is NULL");                  \
    if (!is_live(st)) return fail(nullptr, HYP_EINVAL, "not a live stage handle"); \
  } while (0)


size_t do_stage_workspace_bytes(const hyp_stage_config_t *cfg, int32_t l_start, int32_t l_end) {
  std::string err;
  if (check_config(cfg, l_start, l_end, err) != HYP_OK) { g_create_error = err; return 0; }
  Layout L;
  make_layout(*cfg, l_end - l_start, L);
  return L.total;
}

hyp_status_t do_stage_create(const hyp_stage_config_t *cfg, int32_t l_start, int32_t l_end,
                          const hyp_layer_weights_t *layers, void *workspace, size_t workspace_bytes,
                          void *hip_stream, hyp_stage_t **out) {
  if (out) *out = nullptr;
  std::string err;
  hyp_status_t rc = check_config(cfg, l_start, l_end, err);
  if (rc != HYP_OK) return fail(nullptr, rc, err);
  if (!layers || !workspace || !out) return fail(nullptr, HYP_EINVAL, "layers, workspace and out must not be NULL");
  if ((uintptr_t)workspace % kAlign != 0) return fail(nullptr, HYP_ENOMEM, "workspace must be 256-byte aligned");

  hyp_stage *st = new (std::nothrow) hyp_stage();
  if (!st) return fail(nullptr, HYP_ENOMEM, "host allocation failed");
  st->cfg = *cfg;
  st->l_start = l_start; st->l_end = l_end; st->n_layers = l_end - l_start;
  st->stream = (hipStream_t)hip_stream;
  st->bf16 = cfg->dtype == HYP_BF16;
  st->mfma = mfma_applies(*cfg);
  st->ws = (char *)workspace;
  st->h_stage = nullptr; st->upload_done = nullptr; st->upload_pending = false;
  st->batch = 0; st->prefilled = false;
  Dims &d = st->dm;
  d.H = cfg->hidden; d.nq = cfg->n_q_heads; d.nkv = cfg->n_kv_heads; d.d = cfg->head_dim;
  d.I = cfg->ffn_dim; d.qd = d.nq * d.d; d.kvd = d.nkv * d.d;
  d.max_batch = cfg->max_batch; d.max_seq = cfg->max_seq; d.eps = cfg->rms_eps;
  make_layout(*cfg, st->n_layers, st->L);
  if (workspace_bytes < st->L.total) {
    std::string m = "workspace too small: need " + std::to_string(st->L.total) + " bytes";
    delete st;
    return fail(nullptr, HYP_ENOMEM, m);
  }

  auto bail = [&](hyp_status_t code) {
    g_create_error = st->err;
    if (st->upload_done) (void)hipEventDestroy(st->upload_done);
    if (st->h_stage) (void)hipHostFree(st->h_stage);
    delete st;
    return code;
  };

  st->h_stage_ints = st->mfma ? 3 * (size_t)st->L.rows_cap + 3 * ((size_t)st->L.rows_cap / 64) + 2 * (size_t)cfg->max_batch + 32
                              : 2 * (size_t)max_rows(*cfg) + 2 * (size_t)cfg->max_batch;
  if (hipHostMalloc((void **)&st->h_stage, sizeof(int) * st->h_stage_ints, hipHostMallocDefault) != hipSuccess) {
    st->h_stage = nullptr; st->err = "hipHostMalloc failed";
    return bail(HYP_ENOMEM);
  }
  if (hipEventCreateWithFlags(&st->upload_done, hipEventDisableTiming) != hipSuccess) {
    st->upload_done = nullptr; st->err = "hipEventCreate failed";
    return bail(HYP_EDEVICE);
  }

  if (st->mfma) {
    hipError_t e = mfma_gemm_init();
    if (e == hipSuccess) e = mfma_gemv_init();
    if (e == hipSuccess) e = mfma_attn_init();
    if (e != hipSuccess) { st->err = std::string("kernel attributes: ") + hipGetErrorString(e); return bail(HYP_EDEVICE); }
    // where a decode step keeps its temporaries: in the workspace ...
    const Layout &L = st->L;
    DecScratch &w = st->dec_ws;
    w.xres = at<float>(st, L.xres); w.ssq = at<float>(st, L.ssq); w.partial = at<float>(st, L.partial);
    w.attn_part = at<float>(st, L.attn_part); w.counters = at<unsigned>(st, L.counters);
    w.y = at<bf16_t>(st, L.y); w.attn = at<bf16_t>(st, L.attn); w.m = at<bf16_t>(st, L.m); w.qdec = at<bf16_t>(st, L.qdec);
    // ... or, for stage_decode_step_noalloc, in this GPU's static array, if that is large enough
    void *sbase = nullptr;
    e = static_scratch_of_current_device(&sbase);
    if (e != hipSuccess) { st->err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e); return bail(HYP_EDEVICE); }
    {
      const size_t es = 2, H = d.H;
      size_t off = 0;
      auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
      const size_t o_cnt = take(L.counters_bytes), o_xres = take(sizeof(float) * 32 * H), o_ssq = take(sizeof(float) * 32 * (H / 32)),
                   o_y = take(es * 32 * H), o_attn = take(es * 32 * (size_t)d.qd), o_m = take(es * 32 * (size_t)d.I),
                   o_q = take(es * (size_t)d.max_batch * d.nkv * 32 * 128), o_part = take(L.partial_bytes),
                   o_ap = take(L.attn_part_bytes);
      st->static_bytes = off;
      if (off <= kNoAllocScratchBytes) {
        char *b = (char *)sbase;
        DecScratch &t = st->dec_static;
        t.counters = (unsigned *)(b + o_cnt); t.xres = (float *)(b + o_xres); t.ssq = (float *)(b + o_ssq);
        t.y = (bf16_t *)(b + o_y); t.attn = (bf16_t *)(b + o_attn); t.m = (bf16_t *)(b + o_m); t.qdec = (bf16_t *)(b + o_q);
        t.partial = (float *)(b + o_part); t.attn_part = (float *)(b + o_ap);
      }
    }
    rc = pack_weights_mfma(st, layers);
    if (rc == HYP_OK && st->L.pages_per_req) {
      // until stage_set_page_table says otherwise: request r owns pages r * ppr .. if the pool has that many
      const int ppr = st->L.pages_per_req;
      st->pages.assign((size_t)cfg->max_batch * ppr, -1);
      if (st->L.pool_pages >= cfg->max_batch * ppr)
        for (size_t i = 0; i < st->pages.size(); ++i) st->pages[i] = (int)i;
      rc = upload_page_table(st);
    }
  } else {
    rc = copy_weights(st, layers);
  }
  if (rc != HYP_OK) return bail(rc);

  // RoPE tables: angle = pos * base^(-2i/d), formed in double on the host
  {
    int half = d.d / 2;
    int n_pos = st->mfma ? st->L.key_blocks * 32 : d.max_seq;  // the MFMA path also rotates padding rows
    std::vector<float> ct((size_t)n_pos * half), sn((size_t)n_pos * half);
    for (int i = 0; i < half; ++i) {
      double theta = pow((double)cfg->rope_base, -2.0 * (double)i / (double)d.d);
      for (int p = 0; p < n_pos; ++p) {
        double a = (double)p * theta;
        ct[(size_t)p * half + i] = (float)cos(a);
        sn[(size_t)p * half + i] = (float)sin(a);
      }
    }
    hipError_t e = hipMemcpyAsync(st->ws + st->L.cos_tab, ct.data(), sizeof(float) * ct.size(), hipMemcpyHostToDevice, st->stream);
    if (e == hipSuccess)
      e = hipMemcpyAsync(st->ws + st->L.sin_tab, sn.data(), sizeof(float) * sn.size(), hipMemcpyHostToDevice, st->stream);
    std::vector<int> iota(cfg->max_batch);
    for (int i = 0; i < cfg->max_batch; ++i) iota[i] = i;
    if (e == hipSuccess && !st->mfma)
      e = hipMemcpyAsync(st->ws + st->L.iota, iota.data(), sizeof(int) * iota.size(), hipMemcpyHostToDevice, st->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(st->stream);  // host vectors die here
    if (e != hipSuccess) { st->err = std::string("table upload: ") + hipGetErrorString(e); return bail(HYP_EDEVICE); }
  }
  {
    std::lock_guard<std::mutex> lock(g_live_mu);
    g_live.insert(st);
  }
  *out = st;
  return HYP_OK;
}

hyp_status_t do_stage_prefill(hyp_stage_t *st, const void *hidden_in, const int32_t *seq_lens,
                           int32_t batch, void *hidden_out) {
  LIVE_OR_RETURN(st);
  if (!hidden_in || !seq_lens || !hidden_out) return fail(st, HYP_EINVAL, "NULL argument");
  if (batch < 1 || batch > st->cfg.max_batch) return fail(st, HYP_ECAPACITY, "batch outside 1..max_batch");
  int64_t total = 0;
  for (int b = 0; b < batch; ++b) {
    if (seq_lens[b] < 1 || seq_lens[b] > st->cfg.max_seq)
      return fail(st, HYP_ECAPACITY, "seq_lens[" + std::to_string(b) + "] outside 1..max_seq");
    total += seq_lens[b];
  }
  if (total > st->cfg.max_prefill_tokens) return fail(st, HYP_ECAPACITY, "sum(seq_lens) exceeds max_prefill_tokens");
  if (st->L.pages_per_req)
    for (int b = 0; b < batch; ++b) {  // the padded rows of a prompt are written to the cache as well
      int k = first_key_without_page(st, b, round_up(seq_lens[b], 64));
      if (k >= 0)
        return fail(st, HYP_ECAPACITY, "request " + std::to_string(b) + " has no cache page for key " + std::to_string(k));
    }
  int rows = (int)total;

  hyp_status_t rc = wait_upload(st);
  if (rc != HYP_OK) return rc;
  hipStream_t s = st->stream;
  if (st->mfma) {
    // internal rows: every request starts at a multiple of 64 and is padded to one
    const Layout &L = st->L;
    int R = 0;
    for (int b = 0; b < batch; ++b) R += round_up(seq_lens[b], 64);
    int *h_ext = st->h_stage, *h_pos = h_ext + R, *h_req = h_pos + R;
    PrefillTile *h_tiles = (PrefillTile *)(h_req + R);
    int n_tiles = R / 64;
    int *h_len = (int *)(h_tiles + n_tiles), *h_ext_dec = h_len + batch;
    int row = 0, ext = 0, nt = 0;
    for (int b = 0; b < batch; ++b) {
      int padded = round_up(seq_lens[b], 64);
      for (int p = 0; p < padded; ++p, ++row) {
        h_ext[row] = p < seq_lens[b] ? ext + p : -1;
        h_pos[row] = p;
        h_req[row] = b;
      }
      for (int qb = 0; qb < padded / 32; qb += 2) h_tiles[nt++] = PrefillTile{b, row - padded + qb * 32, qb};
      ext += seq_lens[b];
      h_len[b] = seq_lens[b];
    }
    // causal attention work grows with a tile's position in its request: longest tiles first,
    // so that the launch ends on short ones
    std::sort(h_tiles, h_tiles + nt, [](const PrefillTile &a, const PrefillTile &b) {
      return a.qblk0 != b.qblk0 ? a.qblk0 > b.qblk0 : a.row0 < b.row0;  // total order, in place
    });
    for (int i = 0; i < 32; ++i) h_ext_dec[i] = i < batch ? i : -1;
    HIP_TRY(st, hipMemcpyAsync(st->ws + L.row_ext, h_ext, sizeof(int) * R, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + L.row_pos, h_pos, sizeof(int) * R, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + L.row_req, h_req, sizeof(int) * R, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + L.tiles, h_tiles, sizeof(PrefillTile) * n_tiles, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + L.req_len, h_len, sizeof(int) * batch, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + L.lens, h_len, sizeof(int) * batch, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + L.row_ext_dec, h_ext_dec, sizeof(int) * 32, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipEventRecord(st->upload_done, s));
    st->upload_pending = true;
    rc = run_prefill_mfma(st, hidden_in, hidden_out, R, n_tiles);
  } else {
    int *h_req = st->h_stage, *h_pos = st->h_stage + rows, *h_len = st->h_stage + 2 * (size_t)rows;
    {
      int t = 0;
      for (int b = 0; b < batch; ++b)
        for (int p = 0; p < seq_lens[b]; ++p, ++t) { h_req[t] = b; h_pos[t] = p; }
      for (int b = 0; b < batch; ++b) h_len[b] = seq_lens[b];
    }
    HIP_TRY(st, hipMemcpyAsync(st->ws + st->L.tok_req, h_req, sizeof(int) * rows, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + st->L.tok_pos, h_pos, sizeof(int) * rows, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipMemcpyAsync(st->ws + st->L.lens, h_len, sizeof(int) * batch, hipMemcpyHostToDevice, s));
    HIP_TRY(st, hipEventRecord(st->upload_done, s));
    st->upload_pending = true;
    const int *tok_req = at<int>(st, st->L.tok_req), *tok_pos = at<int>(st, st->L.tok_pos);
    rc = st->bf16 ? run_plain<bf16_t>(st, hidden_in, hidden_out, rows, tok_req, tok_pos)
                  : run_plain<float>(st, hidden_in, hidden_out, rows, tok_req, tok_pos);
  }
  if (rc != HYP_OK) return rc;
  st->lens.assign(seq_lens, seq_lens + batch);
  st->batch = batch;
  st->prefilled = true;
  return HYP_OK;
}

hyp_status_t check_decode_args(hyp_stage *st, const void *hidden_in, void *hidden_out) {
  if (!hidden_in || !hidden_out) return fail(st, HYP_EINVAL, "NULL argument");
  if (!st->prefilled) return fail(st, HYP_ESTATE, "stage_decode_step before stage_prefill");
  for (int b = 0; b < st->batch; ++b)
    if (st->lens[b] >= st->cfg.max_seq)
      return fail(st, HYP_ECAPACITY, "request " + std::to_string(b) + " already holds max_seq tokens");
  if (st->L.pages_per_req)
    for (int b = 0; b < st->batch; ++b) {
      const int i = st->lens[b] / kPageKeys;
      if (st->pages[(size_t)b * st->L.pages_per_req + i] < 0)
        return fail(st, HYP_ECAPACITY, "request " + std::to_string(b) + " has no cache page for key " + std::to_string(st->lens[b]));
    }
  return HYP_OK;
}

hyp_status_t do_stage_decode_step(hyp_stage_t *st, const void *hidden_in, void *hidden_out) {
  LIVE_OR_RETURN(st);
  hyp_status_t rc = check_decode_args(st, hidden_in, hidden_out);
  if (rc != HYP_OK) return rc;
  const int *iota = at<int>(st, st->L.iota), *lens = at<int>(st, st->L.lens);
  rc = st->mfma   ? run_decode_mfma(st, hidden_in, hidden_out)
       : st->bf16 ? run_plain<bf16_t>(st, hidden_in, hidden_out, st->batch, iota, lens)
                  : run_plain<float>(st, hidden_in, hidden_out, st->batch, iota, lens);
  if (rc != HYP_OK) return rc;
  if (!st->mfma) HIP_TRY(st, advance_lens(at<int>(st, st->L.lens), st->batch, st->stream));  // the MFMA path's last kernel does it
  for (int b = 0; b < st->batch; ++b) st->lens[b] += 1;
  return HYP_OK;
}

// The same step with its temporaries in the GPU's static array: kernel launches only - no
// device or host allocation, no graph objects, no events.
hyp_status_t do_stage_decode_step_noalloc(hyp_stage_t *st, const void *hidden_in, void *hidden_out) {
  LIVE_OR_RETURN(st);
  if (!st->mfma) return fail(st, HYP_ESHAPE, "stage_decode_step_noalloc serves stages that run the MFMA kernels");
  if (st->static_bytes > kNoAllocScratchBytes)
    return fail(st, HYP_ECAPACITY, "a decode step of this stage needs " + std::to_string(st->static_bytes) +
                                       " bytes of temporaries; the static array holds " + std::to_string(kNoAllocScratchBytes));
  hyp_status_t rc = check_decode_args(st, hidden_in, hidden_out);
  if (rc != HYP_OK) return rc;
  // the array keeps whatever the last call on this GPU left: the arrival counters must start at zero
  // (a fill kernel, not a memset node, so that the call can be captured into a graph)
  HIP_TRY(st, mfma_fill_zero(st->dec_static.counters, align_up(st->L.counters_bytes), st->stream));
  st->prof_off = true;
  rc = decode_step_mfma(st, st->stream, st->dec_static, hidden_in, hidden_out, true, true);
  st->prof_off = false;
  if (rc != HYP_OK) return rc;
  for (int b = 0; b < st->batch; ++b) st->lens[b] += 1;
  return HYP_OK;
}

hyp_status_t do_stage_set_page_table(hyp_stage_t *st, const int32_t *table, int32_t n_requests, int32_t pages_per_request) {
  LIVE_OR_RETURN(st);
  const int ppr = st->L.pages_per_req;
  if (!ppr) return fail(st, HYP_ESTATE, "the stage was not created with HYP_FLAG_PAGED_KV");
  if (!table || n_requests < 1 || pages_per_request < 1) return fail(st, HYP_EINVAL, "NULL table or non-positive count");
  if (n_requests > st->cfg.max_batch) return fail(st, HYP_ECAPACITY, "more requests than max_batch");
  std::vector<int> next((size_t)st->cfg.max_batch * ppr, -1);
  std::vector<char> used((size_t)st->L.pool_pages, 0);
  for (int r = 0; r < n_requests; ++r)
    for (int i = 0; i < pages_per_request; ++i) {
      const int page = table[(size_t)r * pages_per_request + i];
      if (page < 0) continue;  // no page for these keys
      if (i >= ppr) return fail(st, HYP_ECAPACITY, "a page beyond max_seq");
      if (page >= st->L.pool_pages) return fail(st, HYP_EINVAL, "page " + std::to_string(page) + " is outside the pool");
      if (used[page]) return fail(st, HYP_EINVAL, "page " + std::to_string(page) + " is assigned twice");
      used[page] = 1;
      next[(size_t)r * ppr + i] = page;
    }
  // requests that are resident keep what they hold: their keys must stay where they are
  if (st->prefilled)
    for (int b = 0; b < st->batch; ++b)
      for (int i = 0; i * kPageKeys < st->lens[b]; ++i)
        if (next[(size_t)b * ppr + i] != st->pages[(size_t)b * ppr + i])
          return fail(st, HYP_ESTATE, "the table moves a page that holds cached keys of request " + std::to_string(b));
  st->pages.swap(next);
  return upload_page_table(st);
}

hyp_status_t do_stage_export_kv(hyp_stage_t *st, int32_t layer, int32_t request, void *k_out, void *v_out) {
  LIVE_OR_RETURN(st);
  if (!k_out || !v_out) return fail(st, HYP_EINVAL, "NULL argument");
  if (layer < 0 || layer >= st->n_layers) return fail(st, HYP_EINVAL, "layer outside the stage");
  if (!st->prefilled || request < 0 || request >= st->batch) return fail(st, HYP_ESTATE, "no such request");
  size_t off = st->L.kv_layer_stride * layer;
  int len = st->lens[request];
  if (st->mfma)
    HIP_TRY(st, mfma_export_kv(at<bf16_t>(st, st->L.Kc + off), at<bf16_t>(st, st->L.Vc + off), cache_geom(st),
                               (bf16_t *)k_out, (bf16_t *)v_out, request, len, st->dm.nkv, st->stream));
  else if (st->bf16)
    HIP_TRY(st, plain_export_kv<bf16_t>(at<bf16_t>(st, st->L.Kc + off), at<bf16_t>(st, st->L.Vc + off),
                                        (bf16_t *)k_out, (bf16_t *)v_out, request, len, st->dm, st->stream));
  else
    HIP_TRY(st, plain_export_kv<float>(at<float>(st, st->L.Kc + off), at<float>(st, st->L.Vc + off),
                                       (float *)k_out, (float *)v_out, request, len, st->dm, st->stream));
  return HYP_OK;
}

hyp_status_t do_stage_context_len(const hyp_stage_t *st, int32_t request, int32_t *len_out) {
  if (!st || !len_out || !is_live(st)) return HYP_EINVAL;
  if (!st->prefilled || request < 0 || request >= st->batch) return HYP_ESTATE;
  *len_out = st->lens[request];
  return HYP_OK;
}

hyp_status_t do_stage_profile(hyp_stage_t *st, uint32_t class_mask) {
  LIVE_OR_RETURN(st);
  HIP_TRY(st, hipStreamSynchronize(st->stream));
  st->prof_mask = class_mask;
  st->prof_used = 0;
  return HYP_OK;
}

hyp_status_t do_stage_profile_read(hyp_stage_t *st, int32_t kernel_class, double *total_ms, int64_t *launches) {
  LIVE_OR_RETURN(st);
  if (!total_ms || !launches || kernel_class < 0 || kernel_class >= HYP_K_COUNT) return fail(st, HYP_EINVAL, "bad argument");
  HIP_TRY(st, hipStreamSynchronize(st->stream));
  double tot = 0;
  int64_t n = 0;
  for (size_t i = 0; i < st->prof_used; ++i) {
    if (st->prof[i].cls != kernel_class) continue;
    float ms = 0.f;
    HIP_TRY(st, hipEventElapsedTime(&ms, st->prof[i].a, st->prof[i].b));
    tot += ms;
    ++n;
  }
  *total_ms = tot;
  *launches = n;
  return HYP_OK;
}

hyp_status_t do_stage_destroy(hyp_stage_t *st) {
  {
    if (!st) return fail(nullptr, HYP_EINVAL, "stage is NULL");
    std::lock_guard<std::mutex> lock(g_live_mu);
    if (g_live.erase(st) == 0) return fail(nullptr, HYP_EINVAL, "not a live stage handle (destroyed twice?)");
  }
  if (st->upload_done) (void)hipEventDestroy(st->upload_done);
  if (st->h_stage) (void)hipHostFree(st->h_stage);
  for (auto &ps : st->prof) { (void)hipEventDestroy(ps.a); (void)hipEventDestroy(ps.b); }
  for (auto &g : st->dec_graphs) drop_decode_graph(g);
  if (st->cap_stream) (void)hipStreamDestroy(st->cap_stream);
  delete st;
  return HYP_OK;
}

const char *do_stage_last_error(const hyp_stage_t *st) {
  if (st && !is_live(st)) return "not a live stage handle";
  return st ? st->err.c_str() : g_create_error.c_str();
}

int32_t do_stage_uses_mfma(const hyp_stage_t *st) { return st && is_live(st) && st->mfma ? 1 : 0; }

// No C++ exception may cross the C ABI: every entry point runs its body under this guard
// (the bodies allocate host memory through std::string / std::vector).
template <typename F> hyp_status_t guarded(F &&body) {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    return HYP_ENOMEM;
  } catch (...) {
    return HYP_EDEVICE;
  }
}

}  // namespace

extern "C" {

size_t stage_workspace_bytes(const hyp_stage_config_t *cfg, int32_t l_start, int32_t l_end) {
  try {
    return do_stage_workspace_bytes(cfg, l_start, l_end);
  } catch (...) {
    return 0;
  }
}

hyp_status_t stage_create(const hyp_stage_config_t *cfg, int32_t l_start, int32_t l_end,
                          const hyp_layer_weights_t *layers, void *workspace, size_t workspace_bytes,
                          void *hip_stream, hyp_stage_t **out) {
  return guarded([&] { return do_stage_create(cfg, l_start, l_end, layers, workspace, workspace_bytes, hip_stream, out); });
}

hyp_status_t stage_prefill(hyp_stage_t *st, const void *hidden_in, const int32_t *seq_lens, int32_t batch,
                           void *hidden_out) {
  return guarded([&] { return do_stage_prefill(st, hidden_in, seq_lens, batch, hidden_out); });
}

hyp_status_t stage_decode_step(hyp_stage_t *st, const void *hidden_in, void *hidden_out) {
  return guarded([&] { return do_stage_decode_step(st, hidden_in, hidden_out); });
}

hyp_status_t stage_decode_step_noalloc(hyp_stage_t *st, const void *hidden_in, void *hidden_out) {
  return guarded([&] { return do_stage_decode_step_noalloc(st, hidden_in, hidden_out); });
}

hyp_status_t stage_set_page_table(hyp_stage_t *st, const int32_t *table, int32_t n_requests, int32_t pages_per_request) {
  return guarded([&] { return do_stage_set_page_table(st, table, n_requests, pages_per_request); });
}

hyp_status_t stage_export_kv(hyp_stage_t *st, int32_t layer, int32_t request, void *k_out, void *v_out) {
  return guarded([&] { return do_stage_export_kv(st, layer, request, k_out, v_out); });
}

hyp_status_t stage_context_len(const hyp_stage_t *st, int32_t request, int32_t *len_out) {
  return guarded([&] { return do_stage_context_len(st, request, len_out); });
}

hyp_status_t stage_profile(hyp_stage_t *st, uint32_t class_mask) {
  return guarded([&] { return do_stage_profile(st, class_mask); });
}

hyp_status_t stage_profile_read(hyp_stage_t *st, int32_t kernel_class, double *total_ms, int64_t *launches) {
  return guarded([&] { return do_stage_profile_read(st, kernel_class, total_ms, launches); });
}

hyp_status_t stage_destroy(hyp_stage_t *st) {
  return guarded([&] { return do_stage_destroy(st); });
}

const char *stage_last_error(const hyp_stage_t *st) {
  try {
    return do_stage_last_error(st);
  } catch (...) {
    return "";
  }
}

int32_t stage_uses_mfma(const hyp_stage_t *st) {
  try {
    return do_stage_uses_mfma(st);
  } catch (...) {
    return 0;
  }
}

}  // extern "C"
