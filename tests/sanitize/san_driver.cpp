// Driver for the CPU sanitizer build (-fsanitize=address,undefined) of the host-only code:
// the planner of hyp_plan.h and the C oracle.  It reads cases from stdin, calls the entry
// points and prints their results; tests/test_sanitized_host_code.py feeds it and compares
// the output with the regular builds.  Any sanitizer report ends the process with an error.
//
//   split N T eps | f[N] | m[N] | C[T] | M[T]
//   sched K F_new m_act | C[K] | M_avail[K] | available[K] | F_run_rem[K] | F_wait[K]
//   sim n T has_avail | arrivals[n] | F[T] | m_act[T] | nodes[T] | C[sum] | M[sum] | available[sum]? | transfer[T-1]
//   stage <file>   binary: int32 H nq nkv d I n_layers B steps, float64 eps base, int32 lens[B],
//                  float32 weights of every layer (attn_norm_g wq wk wv wo ffn_norm_g w_gate w_up w_down),
//                  float32 x[sum(lens)][H], float32 xd[steps][B][H]
#include <cstdint>
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "hyp_plan.h"

extern "C" {
typedef struct { int hidden, n_q_heads, n_kv_heads, head_dim, ffn_dim; double rms_eps, rope_base; } orc_shape;
typedef struct { const float *attn_norm_g, *wq, *wk, *wv, *wo, *ffn_norm_g, *w_gate, *w_up, *w_down; } orc_layer;
void orc_stage_forward(const orc_shape *c, const orc_layer *layers, int n_layers, const float *x, const int *seq_lens,
                       const int *pos0, int batch, float *K, float *V, int cap, float *out);
}

template <typename T> static std::vector<T> read_n(int n) {
  std::vector<T> v(n);
  for (auto &x : v) {
    double d;
    std::cin >> d;
    x = (T)d;
  }
  return v;
}

static int run_stage(const std::string &path) {
  FILE *fp = fopen(path.c_str(), "rb");
  if (!fp) return 1;
  int32_t h[8];
  double de[2];
  if (fread(h, 4, 8, fp) != 8 || fread(de, 8, 2, fp) != 2) return 1;
  const int H = h[0], nq = h[1], nkv = h[2], d = h[3], I = h[4], n_layers = h[5], B = h[6], steps = h[7];
  std::vector<int32_t> lens(B);
  if (fread(lens.data(), 4, B, fp) != (size_t)B) return 1;
  const size_t qd = (size_t)nq * d, kvd = (size_t)nkv * d;
  const size_t sizes[9] = {(size_t)H, qd * H, kvd * H, kvd * H, H * qd, (size_t)H, (size_t)I * H, (size_t)I * H, (size_t)H * I};
  std::vector<std::vector<float>> store;
  std::vector<orc_layer> layers(n_layers);
  for (int l = 0; l < n_layers; ++l) {
    const float *ptr[9];
    for (int t = 0; t < 9; ++t) {
      store.emplace_back(sizes[t]);
      if (fread(store.back().data(), 4, sizes[t], fp) != sizes[t]) return 1;
      ptr[t] = store.back().data();
    }
    layers[l] = orc_layer{ptr[0], ptr[1], ptr[2], ptr[3], ptr[4], ptr[5], ptr[6], ptr[7], ptr[8]};
  }
  int T = 0, cap = 0;
  for (int b = 0; b < B; ++b) { T += lens[b]; cap = lens[b] > cap ? lens[b] : cap; }
  cap += steps;
  std::vector<float> x((size_t)T * H), xd((size_t)steps * B * H), out((size_t)T * H), outd((size_t)B * H);
  if (fread(x.data(), 4, x.size(), fp) != x.size() || fread(xd.data(), 4, xd.size(), fp) != xd.size()) return 1;
  fclose(fp);
  orc_shape sh{H, nq, nkv, d, I, de[0], de[1]};
  std::vector<float> K((size_t)n_layers * B * cap * kvd, 0.f), V(K.size(), 0.f);
  std::vector<int> pos(B, 0), one(B, 1), len(lens.begin(), lens.end());
  orc_stage_forward(&sh, layers.data(), n_layers, x.data(), len.data(), pos.data(), B, K.data(), V.data(), cap, out.data());
  printf("stage prefill");
  for (float v : out) printf(" %.9g", v);
  printf("\n");
  for (int s = 0; s < steps; ++s) {
    for (int b = 0; b < B; ++b) pos[b] = lens[b] + s;
    orc_stage_forward(&sh, layers.data(), n_layers, xd.data() + (size_t)s * B * H, one.data(), pos.data(), B, K.data(),
                      V.data(), cap, outd.data());
    printf("stage decode");
    for (float v : outd) printf(" %.9g", v);
    printf("\n");
  }
  return 0;
}

int main() {
  std::string cmd;
  while (std::cin >> cmd) {
    if (cmd == "split") {
      int N, T;
      double eps;
      std::cin >> N >> T >> eps;
      auto f = read_n<double>(N), m = read_n<double>(N), C = read_n<double>(T), M = read_n<double>(T);
      std::vector<int32_t> p(T > 1 ? T - 1 : 1, -1);
      double tau = 0;
      int32_t ok = 0;
      int rc = hypsplit_dp(N, T, f.data(), m.data(), C.data(), M.data(), eps, p.data(), &tau, &ok);
      printf("split %d %d %.17g", rc, ok, tau);
      for (int j = 0; ok && j + 1 < T; ++j) printf(" %d", p[j]);
      printf("\n");
    } else if (cmd == "sched") {
      int K;
      double F_new, m_act;
      std::cin >> K >> F_new >> m_act;
      auto C = read_n<double>(K), Ma = read_n<double>(K);
      auto av = read_n<uint8_t>(K);
      auto Fr = read_n<double>(K), Fw = read_n<double>(K);
      int32_t k = -2;
      int rc = hypsched_rt(K, C.data(), Ma.data(), av.data(), Fr.data(), Fw.data(), F_new, m_act, &k);
      printf("sched %d %d\n", rc, k);
    } else if (cmd == "sim") {
      int n, T, has_av;
      std::cin >> n >> T >> has_av;
      auto arr = read_n<double>(n), F = read_n<double>(T), ma = read_n<double>(T);
      auto nodes = read_n<int32_t>(T);
      int tot = 0;
      for (int v : nodes) tot += v;
      auto C = read_n<double>(tot), M = read_n<double>(tot);
      std::vector<uint8_t> av;
      if (has_av) av = read_n<uint8_t>(tot);
      auto tr = read_n<double>(T > 1 ? T - 1 : 0);
      std::vector<int32_t> node((size_t)n * T);
      std::vector<double> fin((size_t)n * T);
      int rc = hypsched_simulate(n, arr.data(), T, F.data(), ma.data(), nodes.data(), C.data(), M.data(),
                                 has_av ? av.data() : nullptr, T > 1 ? tr.data() : nullptr, node.data(), fin.data());
      printf("sim %d", rc);
      for (size_t i = 0; i < node.size(); ++i) printf(" %d %.17g", node[i], fin[i]);
      printf("\n");
    } else if (cmd == "stage") {
      std::string path;
      std::cin >> path;
      if (run_stage(path) != 0) { fprintf(stderr, "bad stage file\n"); return 2; }
    } else {
      fprintf(stderr, "unknown case %s\n", cmd.c_str());
      return 2;
    }
  }
  return 0;
}
