// Host logic of the library under AddressSanitizer and UndefinedBehaviorSanitizer (CPU build, no GPU call is made):
// the batch former and its virtual-clock run over seeded traces under memory pressure, the launch planners over
// seeded random batches, and the validation paths with bad input.  Any sanitizer report aborts the program; the
// program also checks a few invariants of its own.  Built and run by tests/test_host_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "ps.h"

static uint64_t rng_state = 88172645463325252ull;
static uint64_t rnd() {  // xorshift64
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return rng_state;
}
static int64_t rnd_in(int64_t lo, int64_t hi) { return lo + (int64_t)(rnd() % (uint64_t)(hi - lo + 1)); }

#define CHECK(cond)                                                       \
  do {                                                                    \
    if (!(cond)) {                                                        \
      fprintf(stderr, "host_checks: %s failed at line %d (%s)\n", #cond, __LINE__, ps_last_error()); \
      return 1;                                                           \
    }                                                                     \
  } while (0)

static ps_sched_cfg sched_cfg(int layers) {
  const int64_t MS = 1000000000ll, US = 1000000ll, NS = 1000ll;
  ps_sched_cfg c = {};
  c.n_classes = 3;
  c.block_tokens = 16;
  c.class_weight[0] = 4; c.class_weight[1] = 2; c.class_weight[2] = 1;
  c.w_first = 4; c.w_decode = 1;
  c.ttft_slo_ps = 2000 * MS; c.tpot_slo_ps = 100 * MS;
  c.a_p = 13 * layers / 2; c.b_p = 13 * layers; c.c_p = 50 * NS * layers;
  c.a_d = 730 * layers; c.b_d = US * layers; c.t_c = 2 * MS;
  c.eta_ps = 10 * MS; c.tau_ps = 3000 * MS;
  c.gamma_num = 9; c.gamma_den = 10; c.beta_num = 2; c.beta_den = 1; c.rho_num = 9; c.rho_den = 10;
  c.t_block_ps = 1200 * NS * layers;
  c.n_off_base = 8;
  return c;
}

static int run_scheduler() {
  for (int variant = 0; variant < 4; ++variant) {
    ps_sched_cfg cfg = sched_cfg(36);
    if (variant == 1) cfg.order_policy = PS_ORDER_FCFS;
    if (variant == 2) { cfg.t_block_ps *= 40; cfg.n_off_base = 2; }
    if (variant == 3) { cfg.gamma_num = 1000000; cfg.tau_ps = 200 * 1000000000ll; }
    const int M = 300, Mh = 600, N = 250;
    std::vector<int32_t> dev(M), host(Mh);
    for (int i = 0; i < M; ++i) dev[i] = i;
    for (int i = 0; i < Mh; ++i) host[i] = Mh - 1 - i;
    for (int i = M - 1; i > 0; --i) std::swap(dev[i], dev[rnd() % (i + 1)]);
    std::vector<ps_trace_req> tr(N);
    int64_t t = 0, total_out = 0;
    for (int i = 0; i < N; ++i) {
      t += rnd_in(0, 10000000000ll);  // up to 10 ms apart
      tr[i] = ps_trace_req{(int64_t)i, t, (int32_t)rnd_in(1, 3), (int32_t)rnd_in(1, 3000), (int32_t)rnd_in(1, 200), 0};
      total_out += tr[i].out_len;
    }
    std::vector<int64_t> times((size_t)total_out);
    std::vector<int32_t> delivered(N);
    ps_sim_result res;
    CHECK(ps_sched_simulate(&cfg, dev.data(), M, host.data(), Mh, tr.data(), N, 1500, times.data(), delivered.data(), &res) == PS_OK);
    CHECK(res.steps > 100 && res.gain <= res.ideal_gain && res.finished <= N && res.slo_attained <= res.finished);
    // the same trace step by step through ps_form_batch, reporting offloads two rounds late
    ps_sched* s = nullptr;
    CHECK(ps_sched_create(&cfg, dev.data(), M, host.data(), Mh, &s) == PS_OK);
    int64_t now = 0;
    int nxt = 0;
    for (int step = 0; step < 600; ++step) {
      while (nxt < N && tr[nxt].arrival_ps <= now) {
        CHECK(ps_sched_add_request(s, tr[nxt].rid, tr[nxt].arrival_ps, tr[nxt].prio, tr[nxt].prompt_len, tr[nxt].out_len) == PS_OK);
        ++nxt;
      }
      if (step > 2) CHECK(ps_sched_offloads_done(s, step - 2) == PS_OK);
      ps_batch_out fb;
      CHECK(ps_form_batch(s, now, &fb) == PS_OK);
      CHECK(fb.round == step + 1 && fb.n_swap_in <= fb.copy_budget);
      int64_t blocks = 0;
      for (int r = 0; r < fb.batch.n_req; ++r) {
        const int lq = fb.batch.q_start[r + 1] - fb.batch.q_start[r];
        CHECK(lq >= 1 && lq <= fb.batch.kv_len[r]);
        CHECK(fb.batch.bt_start[r + 1] - fb.batch.bt_start[r] == (fb.batch.kv_len[r] + 15) / 16);
        blocks += fb.batch.bt_start[r + 1] - fb.batch.bt_start[r];
      }
      for (int64_t i = 0; i < blocks; ++i) CHECK(fb.batch.block_ids[i] >= 0 && fb.batch.block_ids[i] < M);
      int32_t nq = 0, nd = 0, nh = 0;
      CHECK(ps_sched_counts(s, &nq, &nd, &nh) == PS_OK && nd >= 0 && nd <= M && nh >= 0 && nh <= Mh);
      now += fb.t_batch_ps > 0 ? fb.t_batch_ps : cfg.eta_ps;
    }
    CHECK(ps_sched_offloads_done(s, 100000) == PS_EINVAL);  // a round that has not been formed
    ps_sched_destroy(s);
  }
  // bad configurations and requests are errors, not crashes
  ps_sched_cfg bad = sched_cfg(1);
  bad.eta_ps = bad.t_c;
  ps_sched* s = nullptr;
  int32_t one = 0;
  CHECK(ps_sched_create(&bad, &one, 1, &one, 1, &s) == PS_EINVAL && s == nullptr);
  CHECK(ps_sched_create(nullptr, nullptr, 0, nullptr, 0, &s) == PS_EINVAL);
  ps_sched_cfg ok = sched_cfg(1);
  CHECK(ps_sched_create(&ok, nullptr, 0, nullptr, 0, &s) == PS_OK);  // no blocks at all: nothing can ever be admitted
  CHECK(ps_sched_add_request(s, 1, 0, 1, 100, 5) == PS_OK);
  CHECK(ps_sched_add_request(s, 1, 0, 1, 100, 5) == PS_EINVAL);
  CHECK(ps_sched_add_request(s, 2, 0, 9, 100, 5) == PS_EINVAL);
  ps_batch_out fb;
  CHECK(ps_form_batch(s, 10, &fb) == PS_OK && fb.batch.n_req == 0 && fb.t_batch_ps == 0);
  ps_sched_destroy(s);
  int64_t g = 0, ideal = 0;
  int32_t ok_slo = 0;
  const int64_t tt[3] = {1, 2, 3};
  CHECK(ps_tdg_score(&ok, 1, 3, tt, 3, &g, &ideal, &ok_slo) == PS_OK && g == ideal && ok_slo == 1);
  CHECK(ps_tdg_score(&ok, 0, 3, tt, 3, &g, &ideal, &ok_slo) == PS_EINVAL);
  return 0;
}

static int run_planners() {
  for (int iter = 0; iter < 300; ++iter) {
    ps_layer_cfg cfg = {};
    const int shapes[4][2] = {{32, 8}, {64, 8}, {8, 2}, {16, 1}};
    cfg.n_q_heads = shapes[iter % 4][0];
    cfg.n_kv_heads = shapes[iter % 4][1];
    cfg.head_dim = 128;
    cfg.block_tokens = 16;
    cfg.n_device_blocks = 200000;
    if (iter % 7 == 3) cfg.decode_chunk = 512;
    if (iter % 5 == 2) cfg.prefill_split_tiles = (int32_t)rnd_in(-1, 9);
    cfg.mixed_launch = iter % 3;
    const int n_dec = (int)rnd_in(0, 300), n_pre = (int)rnd_in(n_dec ? 0 : 1, 4);
    std::vector<int32_t> q_start(1, 0), kv_len, bt_start(1, 0), ids;
    for (int r = 0; r < n_dec + n_pre; ++r) {
      const int lq = r < n_dec ? 1 : (int)rnd_in(2, 3000);
      const int L = lq + (int)rnd_in(0, iter % 3 == 0 ? 40000 : 3000);
      q_start.push_back(q_start.back() + lq);
      kv_len.push_back(L);
      for (int b = 0; b < (L + 15) / 16; ++b) ids.push_back((int32_t)rnd_in(0, cfg.n_device_blocks - 1));
      bt_start.push_back((int32_t)ids.size());
    }
    ps_batch b = {n_dec + n_pre, q_start.back(), q_start.data(), kv_len.data(), bt_start.data(), ids.data(), nullptr};
    int32_t out6[6];
    const int n_cus = iter % 2 ? 256 : (int)rnd_in(1, 400);
    CHECK(ps_plan_launch(&cfg, &b, n_cus, out6) == PS_OK);
    CHECK(out6[0] >= 0 && out6[2] >= 0 && out6[3] >= 0 && out6[5] >= 0 && out6[0] == out6[1] * cfg.n_kv_heads);
    if (n_dec == 0) CHECK(out6[2] == 0);
    std::vector<int32_t> seg((size_t)(n_dec * 100 + 8192) * 5);
    int32_t n_seg = 0, n_slots = 0;
    const int waves = (int)rnd_in(cfg.n_kv_heads, 4096);
    CHECK(ps_plan_decode(&cfg, &b, waves, seg.data(), (int32_t)(seg.size() / 5), &n_seg, &n_slots) == PS_OK);
    int64_t covered = 0, want = 0;
    for (int i = 0; i < n_seg; ++i) covered += seg[5 * i + 2] - seg[5 * i + 1];
    for (int r = 0; r < n_dec; ++r) want += kv_len[r];
    CHECK(covered == want);
    // a broken description is refused
    if (b.n_req > 0) {
      kv_len[0] += 16;
      CHECK(ps_plan_launch(&cfg, &b, 256, out6) == PS_EINVAL);
      kv_len[0] -= 16;
      if (!ids.empty()) {
        const int32_t keep = ids[0];
        ids[0] = cfg.n_device_blocks;
        CHECK(ps_plan_launch(&cfg, &b, 256, out6) == PS_EINVAL);
        ids[0] = keep;
      }
    }
  }
  ps_layer_cfg bad = {};
  ps_ctx* ctx = nullptr;
  CHECK(ps_create(&bad, &ctx) == PS_EINVAL && ctx == nullptr);
  return 0;
}

int main() {
  if (run_scheduler() != 0) return 1;
  if (run_planners() != 0) return 1;
  printf("host_checks ok\n");
  return 0;
}
