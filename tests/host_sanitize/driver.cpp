// Host-code driver for the sanitizer build: calls the planning entry points and the decode
// step's plan builder on inputs it draws itself, and prints every input and result as text, so
// that the test can repeat each call against the regular library and compare.  No GPU call.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "spotshard.h"
#include "spotshard_debug.h"
#include "spotshard_plan.h"

static uint64_t g_state = 0x2311155660ull;
static uint64_t draw() {  // splitmix64
  uint64_t z = (g_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}
static int64_t below(int64_t n) { return (int64_t)(draw() % (uint64_t)n); }

template <typename T> static void print_list(const char *tag, const std::vector<T> &v) {
  printf("%s", tag);
  for (auto x : v) printf(" %lld", (long long)x);
  printf("\n");
}

static void match_case(int n) {
  std::vector<uint64_t> w((size_t)n * n);
  for (auto &x : w) x = (uint64_t)below(n <= 4 ? 4 : 1000);  // small ranges: many ties
  std::vector<int32_t> pos(n);
  uint64_t total = 0;
  const ss_status st = ss_match_devices(n, w.data(), pos.data(), &total);
  printf("match %d\n", n);
  print_list("in", w);
  printf("status %d total %llu\n", (int)st, (unsigned long long)total);
  print_list("out", pos);
}

static void order_case(int L, int I) {
  std::vector<int64_t> delta((size_t)L * I);
  for (auto &x : delta) x = below(2001) - 1000;
  const int64_t u_max = below(1500);
  std::vector<int32_t> order(L), stage(L), kind(1 + L + 8), arg(1 + L + 8);
  const ss_status st = ss_migration_order(L, I, delta.data(), u_max, order.data());
  printf("order %d %d %lld\n", L, I, (long long)u_max);
  print_list("in", delta);
  printf("status %d\n", (int)st);
  print_list("out", order);
  const int n_stages = 1 + (int)below(L < 8 ? L : 8);
  for (int l = 0; l < L; ++l) stage[l] = (int)((int64_t)l * n_stages / L);
  kind.resize(1 + L + n_stages), arg.resize(1 + L + n_stages);
  const ss_status sp = ss_progressive_plan(L, order.data(), stage.data(), n_stages, kind.data(), arg.data());
  printf("plan %d %d\n", L, n_stages);
  print_list("in", stage);
  printf("status %d\n", (int)sp);
  print_list("kind", kind);
  print_list("arg", arg);
}

static void keep_case(int rows, int n_dst) {
  std::vector<int32_t> lens(rows), map(n_dst);
  for (auto &x : lens) x = (int32_t)below(6) * (int32_t)below(40);
  const int keep = (int)below(n_dst + 1);
  const ss_status st = ss_rows_to_keep(rows, lens.data(), keep, n_dst, map.data());
  printf("keep %d %d %d\n", rows, keep, n_dst);
  print_list("in", lens);
  printf("status %d\n", (int)st);
  print_list("out", map);
}

static void cost_case() {
  const int nb = 1 + (int)below(4);
  std::vector<ss_cost_sample> dec, pre;
  for (int b = 0; b < nb; ++b) {
    const int batch = 1 << b;
    const int nd = 1 + (int)below(5), np = (int)below(4);
    for (int i = 0; i < nd; ++i) dec.push_back({batch, 16 + (int)below(2000), 0.5 + 0.001 * (double)below(4000)});
    for (int i = 0; i < np; ++i) pre.push_back({batch, 1 + (int)below(1024), 1.0 + 0.01 * (double)below(20000)});
  }
  ss_cost_model m;
  memset(&m, 0, sizeof m);
  const ss_status st = ss_cost_fit(dec.data(), (int)dec.size(), pre.empty() ? nullptr : pre.data(), (int)pre.size(), &m);
  printf("cost %d %d\n", (int)dec.size(), (int)pre.size());
  for (auto &s : dec) printf("d %d %d %.17g\n", s.batch, s.length, s.ms);
  for (auto &s : pre) printf("p %d %d %.17g\n", s.batch, s.length, s.ms);
  printf("status %d n %d\n", (int)st, m.n_batches);
  for (int i = 0; i < m.n_batches; ++i)
    printf("m %d %.17g %.17g %.17g %.17g\n", m.batch[i], m.dec_base_ms[i], m.dec_per_row_ms[i], m.pre_base_ms[i], m.pre_per_token_ms[i]);
  if (st != SS_OK) return;
  const int batch = 1 + (int)below(12), s_in = 1 + (int)below(512), s_out = (int)below(200);
  std::vector<double> l(s_out + 1);
  const ss_status sl = ss_cost_l_exe(&m, batch, s_in, s_out, l.data());
  const double t_grace = 30.0 + (double)below(2000), t_mig = (double)below(500);
  const int acq = (int)below(2);
  const int jit = sl == SS_OK ? ss_jit_iterations(acq, s_out, l.data(), t_grace, t_mig) : -1;
  printf("lexe %d %d %d status %d last %.17g jit %d %.17g %.17g %d\n", batch, s_in, s_out, (int)sl, l[s_out], acq, t_grace, t_mig, jit);
}

// "plan" lines on stdin: 15 descriptor fields, 6 slice fields, max_batch max_seq B
static void plan_cases() {
  char line[1024];
  while (fgets(line, sizeof line, stdin)) {
    ss_model_desc d;
    ss_slice s;
    int mb, ms, B;
    if (sscanf(line, "plan %d %d %d %d %d %d %d %d %d %d %d %d %d %f %f %d %d %d %d %d %d %d %d %d", &d.n_layers, &d.d_model, &d.n_heads,
               &d.head_dim, &d.ffn, &d.vocab, &d.max_pos, &d.norm, &d.act, &d.pos, &d.has_bias, &d.dtype, &d.kv_dtype, &d.norm_eps,
               &d.rope_theta, &s.layer_lo, &s.layer_hi, &s.head_lo, &s.head_hi, &s.ffn_lo, &s.ffn_hi, &mb, &ms, &B) != 24)
      continue;
    uint64_t total = 0, sz = 0;
    std::vector<unsigned char> buf;
    int n = ss_debug_plan(&d, &s, mb, ms, B, 1ull << 40, nullptr, 0, &total, &sz);  // sizes only
    if (sz) buf.resize((size_t)sz * 256);
    if (sz) n = ss_debug_plan(&d, &s, mb, ms, B, 1ull << 40, buf.data(), 256, &total, &sz);
    const size_t bytes = ss_shard_device_bytes(&d, &s, mb, ms);
    uint64_t model = 0, cache = 0;
    const ss_status so = ss_context_overlap(&d, 0, &s, &s, (uint64_t)B * 17, &model, &cache);
    printf("planned %d total %llu bytes %llu overlap %d %llu %llu\n", n, (unsigned long long)total, (unsigned long long)bytes, (int)so,
           (unsigned long long)model, (unsigned long long)cache);
  }
}

int main() {
  for (int n : {1, 2, 3, 4, 5, 8, 13, 32, 64}) match_case(n);
  for (int rep = 0; rep < 6; ++rep) order_case(1 + (int)below(40), 1 + (int)below(9));
  for (int rep = 0; rep < 8; ++rep) keep_case(1 + (int)below(32), 1 + (int)below(32));
  for (int rep = 0; rep < 8; ++rep) cost_case();
  // refusals: every argument check on the way out
  int32_t one = 0;
  uint64_t t = 0;
  printf("refuse %d %d %d %d\n", (int)ss_match_devices(0, nullptr, &one, &t), (int)ss_migration_order(0, 1, nullptr, 0, &one),
         (int)ss_rows_to_keep(-1, &one, 0, 1, &one), (int)ss_cost_fit(nullptr, 0, nullptr, 0, nullptr));
  plan_cases();
  printf("done\n");
  return 0;
}
