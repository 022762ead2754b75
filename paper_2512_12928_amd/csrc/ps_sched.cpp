// Host-only batch former behind ps_sched_* / ps_form_batch: SlideBatching (Alg. 1) with the
// eviction, offload and copy-budget rules of Sec. 4.3.  Integer picoseconds, exact arithmetic.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/ps.h"

// defined next to ps_last_error(): stores the thread-local error text
extern "C" void ps_internal_set_error(const char* text);

namespace {

typedef __int128 i128;

int sched_fail(int code, const char* fmt, ...);

struct Req {
  int64_t rid, arrival;
  int32_t prio, prompt_len, out_len;
  int64_t computed = 0;   // tokens whose KV exists (on the device, or on the host if evicted)
  int64_t generated = 0;  // output tokens delivered
  int64_t last_sched = 0;
  std::vector<int32_t> dev_blocks;  // logical order
  std::vector<int32_t> host_slots;  // host copies of logical blocks 0..n-1 (issued, maybe still in flight)
  std::vector<int64_t> host_round;  // the scheduling round that issued each of them
  // per-round scratch
  int64_t exec = 0, remain = 0, weight = 0;
  bool urgent = false, starving = false, in_batch = false, evicted_now = false;

  int64_t need() const { return (int64_t)prompt_len + generated; }
  int64_t b_miss() const {  // max(0, b_host - b_device)
    const int64_t d = (int64_t)host_slots.size() - (int64_t)dev_blocks.size();
    return d > 0 ? d : 0;
  }
};

}  // namespace

struct ps_sched {
  ps_sched_cfg cfg;
  std::vector<int32_t> dev_free, host_free;  // LIFO: back() is handed out next
  std::unordered_map<int64_t, Req*> by_id;
  std::vector<Req*> reqs;  // active requests
  int64_t round = 0;        // ps_form_batch calls so far
  int64_t done_upto = 0;    // offloads issued in rounds <= this have completed (ps_sched_offloads_done)
  // result storage
  std::vector<int32_t> q_start, kv_len, bt_start, block_ids, si_host, si_dev, so_dev, so_host, emitted_index;
  std::vector<uint8_t> prio;
  std::vector<int64_t> req_ids, order, urgent, evicted, emitted_req, finished;
};

namespace {

inline int64_t t_prefill(const ps_sched_cfg& c, int64_t lq, int64_t lkv) {
  return c.a_p * lq * lq + c.b_p * lq * lkv + c.c_p * lq;
}
inline int64_t t_decode(const ps_sched_cfg& c, int64_t lkv) { return c.a_d * lkv + c.b_d; }

// GetMaxChunk: largest c in [0, lq] with T~_p(c, lkv) <= T (the cost is non-decreasing in c).
int64_t max_chunk(const ps_sched_cfg& c, int64_t lq, int64_t lkv, int64_t T) {
  if (lq <= 0 || T < 0) return 0;
  int64_t lo = 0, hi = lq;  // cost(lo) <= T always holds for lo = 0
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo + 1) / 2;
    if (t_prefill(c, mid, lkv) <= T)
      lo = mid;
    else
      hi = mid - 1;
  }
  return lo;
}

// Adaptive copy-budget control (Sec. 4.3).  Case 2(ii): transfer time B * t_block rises with B,
// the batch latency T_fwd^min + (B_missing - B) * s_blk * c_p falls (blocks not copied are
// recomputed); the answer is the largest B with transfer <= latency, found by bisection.
int64_t copy_budget(const ps_sched_cfg& c, int64_t t_budget, int64_t t_fwd_min, int64_t b_missing) {
  if (t_fwd_min >= t_budget) return t_budget / c.t_block_ps;
  if ((i128)t_fwd_min >= (i128)b_missing * c.t_block_ps) return b_missing;
  auto ok = [&](int64_t B) {
    return (i128)B * c.t_block_ps <= (i128)t_fwd_min + (i128)(b_missing - B) * c.block_tokens * c.c_p;
  };
  int64_t lo = 0, hi = b_missing;  // ok(0) holds: 0 <= t_fwd_min + ...
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo + 1) / 2;
    if (ok(mid))
      lo = mid;
    else
      hi = mid - 1;
  }
  return lo;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

namespace {
int sched_fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  ps_internal_set_error(buf);
  return code;
}
}  // namespace

extern "C" {

int ps_sched_create(const ps_sched_cfg* cfg, const int32_t* dev_free_order, int32_t n_dev,
                    const int32_t* host_free_order, int32_t n_host, ps_sched** out) {
  if (!cfg || !out) return sched_fail(PS_EINVAL, "ps_sched_create: NULL argument");
  *out = nullptr;
  if (cfg->n_classes < 1 || cfg->n_classes > 8) return sched_fail(PS_EINVAL, "n_classes must be in 1..8");
  if (cfg->block_tokens < 1) return sched_fail(PS_EINVAL, "block_tokens must be positive");
  if (cfg->eta_ps <= cfg->t_c) return sched_fail(PS_EINVAL, "eta must exceed t_c (denominator of Eq. 8)");
  if (cfg->gamma_den <= 0 || cfg->beta_den <= 0 || cfg->rho_den <= 0 || cfg->gamma_num < 0 || cfg->beta_num < 0 ||
      cfg->rho_num < 0)
    return sched_fail(PS_EINVAL, "gamma / beta / rho must be non-negative fractions with positive denominators");
  if (cfg->t_block_ps <= 0) return sched_fail(PS_EINVAL, "t_block must be positive");
  if (cfg->order_policy != PS_ORDER_SLIDEBATCHING && cfg->order_policy != PS_ORDER_FCFS)
    return sched_fail(PS_EINVAL, "order_policy must be PS_ORDER_SLIDEBATCHING or PS_ORDER_FCFS");
  if (cfg->a_p < 0 || cfg->b_p < 0 || cfg->c_p < 0 || cfg->a_d < 0 || cfg->b_d < 0 || cfg->t_c < 0)
    return sched_fail(PS_EINVAL, "estimator coefficients must be non-negative");
  if (n_dev < 0 || n_host < 0 || (n_dev > 0 && !dev_free_order) || (n_host > 0 && !host_free_order))
    return sched_fail(PS_EINVAL, "bad pool description");
  for (int p = 0; p < cfg->n_classes; ++p)
    if (cfg->class_weight[p] <= 0) return sched_fail(PS_EINVAL, "class weights must be positive");
  for (int pass = 0; pass < 2; ++pass) {
    std::vector<int32_t> v(pass == 0 ? dev_free_order : host_free_order,
                           (pass == 0 ? dev_free_order : host_free_order) + (pass == 0 ? n_dev : n_host));
    std::sort(v.begin(), v.end());
    if (std::adjacent_find(v.begin(), v.end()) != v.end()) return sched_fail(PS_EINVAL, "duplicate block id in a pool");
  }
  ps_sched* s = new (std::nothrow) ps_sched();
  if (!s) return sched_fail(PS_ENOMEM, "out of host memory");
  s->cfg = *cfg;
  s->dev_free.assign(dev_free_order, dev_free_order + n_dev);
  std::reverse(s->dev_free.begin(), s->dev_free.end());
  s->host_free.assign(host_free_order, host_free_order + n_host);
  std::reverse(s->host_free.begin(), s->host_free.end());
  *out = s;
  return PS_OK;
}

void ps_sched_destroy(ps_sched* s) {
  if (!s) return;
  for (Req* r : s->reqs) delete r;
  delete s;
}

int ps_sched_add_request(ps_sched* s, int64_t rid, int64_t arrival_ps, int32_t prio, int32_t prompt_len,
                         int32_t out_len) {
  if (!s) return sched_fail(PS_EINVAL, "NULL scheduler");
  if (prio < 1 || prio > s->cfg.n_classes) return sched_fail(PS_EINVAL, "priority class %d outside 1..%d", prio, s->cfg.n_classes);
  if (prompt_len < 1 || out_len < 1) return sched_fail(PS_EINVAL, "prompt_len and out_len must be >= 1");
  if (s->by_id.count(rid)) return sched_fail(PS_EINVAL, "request %lld already queued", (long long)rid);
  Req* r = new (std::nothrow) Req();
  if (!r) return sched_fail(PS_ENOMEM, "out of host memory");
  r->rid = rid;
  r->arrival = arrival_ps;
  r->prio = prio;
  r->prompt_len = prompt_len;
  r->out_len = out_len;
  r->last_sched = arrival_ps;  // "waiting time" counts from arrival until first scheduled
  s->reqs.push_back(r);
  s->by_id[rid] = r;
  return PS_OK;
}

int ps_sched_counts(const ps_sched* s, int32_t* n_queued, int32_t* n_dev_free, int32_t* n_host_free) {
  if (!s) return sched_fail(PS_EINVAL, "NULL scheduler");
  if (n_queued) *n_queued = (int32_t)s->reqs.size();
  if (n_dev_free) *n_dev_free = (int32_t)s->dev_free.size();
  if (n_host_free) *n_host_free = (int32_t)s->host_free.size();
  return PS_OK;
}

int ps_sched_offloads_done(ps_sched* s, int64_t upto_round) {
  if (!s) return sched_fail(PS_EINVAL, "NULL scheduler");
  if (upto_round > s->round) return sched_fail(PS_EINVAL, "round %lld has not been formed yet", (long long)upto_round);
  if (upto_round > s->done_upto) s->done_upto = upto_round;
  return PS_OK;
}

int ps_form_batch(ps_sched* s, int64_t now, ps_batch_out* out) {
  if (!s || !out) return sched_fail(PS_EINVAL, "ps_form_batch: NULL argument");
  s->round += 1;
  const ps_sched_cfg& c = s->cfg;
  const int64_t blk = c.block_tokens;
  for (auto* v : {&s->q_start, &s->kv_len, &s->bt_start, &s->block_ids, &s->si_host, &s->si_dev, &s->so_dev,
                  &s->so_host, &s->emitted_index})
    v->clear();
  for (auto* v : {&s->req_ids, &s->order, &s->urgent, &s->evicted, &s->emitted_req, &s->finished}) v->clear();
  s->prio.clear();
  std::memset(out, 0, sizeof *out);

  // queue = requests that have arrived
  std::vector<Req*> Q;
  for (Req* r : s->reqs)
    if (r->arrival <= now) Q.push_back(r);

  int64_t t_budget = 0, phi = 0, b_copy = 0, t_batch = 0;
  std::vector<std::pair<Req*, int64_t>> members;
  if (!Q.empty()) {
    // Alg. 1 lines 1-6: exec, remain, density (as weight / exec), t_min
    int64_t t_min = INT64_MAX, sum_exec = 0, b_missing = 0;
    for (Req* r : Q) {
      const int64_t lq = r->need() - r->computed;
      const bool dec = r->generated >= 1 && lq == 1;
      r->exec = dec ? t_decode(c, r->need()) : t_prefill(c, lq, r->computed);
      const int64_t i = r->generated + 1;  // index of the next token to deliver
      r->remain = c.ttft_slo_ps + (i - 1) * c.tpot_slo_ps - (now - r->arrival);
      r->weight = (i == 1 ? c.w_first : c.w_decode) * c.class_weight[r->prio - 1];
      r->in_batch = r->evicted_now = false;
      t_min = std::min(t_min, r->remain);
      sum_exec += r->exec;
      b_missing += r->b_miss();
    }
    // line 7
    t_budget = std::max(t_min, c.eta_ps);
    // Eq. 8 and lines 8-12
    phi = (int64_t)(((i128)t_budget * sum_exec) / (t_budget - c.t_c));
    for (Req* r : Q) {
      r->urgent = (i128)r->remain * c.gamma_den < (i128)c.gamma_num * phi;
      r->starving = now - r->last_sched > c.tau_ps;
    }
    // line 13 and the starvation rule: starving (longest wait first), URGENT by density
    // descending, NORMAL by remaining time ascending; ties by arrival, then id
    const bool fcfs = c.order_policy == PS_ORDER_FCFS;  // comparison arm: arrival order, nothing else
    auto group = [&](const Req* r) { return fcfs ? 3 : (r->starving ? 0 : (r->urgent ? 1 : 2)); };
    std::sort(Q.begin(), Q.end(), [&](const Req* a, const Req* b) {
      const int ga = group(a), gb = group(b);
      if (ga != gb) return ga < gb;
      if (ga == 0) {
        const int64_t wa = now - a->last_sched, wb = now - b->last_sched;
        if (wa != wb) return wa > wb;
      } else if (ga == 1) {
        const i128 da = (i128)a->weight * std::max<int64_t>(b->exec, 1);  // a.w/a.exec vs b.w/b.exec
        const i128 db = (i128)b->weight * std::max<int64_t>(a->exec, 1);
        if (da != db) return da > db;
      } else if (ga == 2) {
        if (a->remain != b->remain) return a->remain < b->remain;
      }
      if (a->arrival != b->arrival) return a->arrival < b->arrival;
      return a->rid < b->rid;
    });
    for (Req* r : Q) {
      s->order.push_back(r->rid);
      if (r->urgent) s->urgent.push_back(r->rid);
    }
    // line 14
    b_copy = copy_budget(c, t_budget, c.t_c + sum_exec, b_missing);
    int64_t b_rem = b_copy;
    // lines 15-23
    t_batch = c.t_c;
    size_t idx = 0;
    while (idx < Q.size() && t_batch < t_budget) {
      Req* r = Q[idx++];
      if (r->evicted_now) continue;
      const int64_t T = t_budget - t_batch;
      const int64_t miss = r->b_miss();
      int64_t k = 0, comp = r->computed;
      if (miss > 0) {
        k = b_rem >= miss ? miss : b_rem;
        comp = k * blk;  // what is not reloaded is recomputed
      }
      const bool partial = miss > 0 && k < miss;
      const int64_t lq = r->need() - comp;
      const bool dec = r->generated >= 1 && lq == 1;
      int64_t chunk, t;
      if (dec) {
        chunk = 1;  // a decode token is atomic
        t = t_decode(c, r->need());
      } else {
        chunk = max_chunk(c, lq, comp, T);
        if (chunk == 0) continue;
        t = t_prefill(c, chunk, comp);
      }
      if (partial) {
        const bool ok = chunk == lq || (i128)chunk * c.beta_den > (i128)c.beta_num * (miss - k) * blk;
        if (!ok) continue;
      }
      const int64_t held = (int64_t)r->dev_blocks.size();
      int64_t want = ceil_div(comp + chunk, blk) - held;
      if (want > (int64_t)s->dev_free.size()) {
        // victims from the tail of the sorted queue, behind r, never a near-starved request
        for (size_t j = Q.size(); j-- > idx && want > (int64_t)s->dev_free.size();) {
          Req* v = Q[j];
          if (v->in_batch || v->evicted_now || v->dev_blocks.empty()) continue;
          if ((i128)(now - v->last_sched) * c.rho_den >= (i128)c.rho_num * c.tau_ps) continue;
          for (int32_t b : v->dev_blocks) s->dev_free.push_back(b);
          v->dev_blocks.clear();
          // host copies still in flight are discarded with the eviction (Sec. 4.3, Asynchronous
          // Offloading): only completed ones keep their tokens from being recomputed
          size_t conf = 0;
          while (conf < v->host_round.size() && v->host_round[conf] <= s->done_upto) ++conf;
          for (size_t b = conf; b < v->host_slots.size(); ++b) s->host_free.push_back(v->host_slots[b]);
          v->host_slots.resize(conf);
          v->host_round.resize(conf);
          v->computed = std::min<int64_t>(v->computed, (int64_t)conf * blk);
          v->evicted_now = true;
          s->evicted.push_back(v->rid);
        }
      }
      if (want > (int64_t)s->dev_free.size()) {
        const int64_t fit = (held + (int64_t)s->dev_free.size()) * blk - comp;
        if (dec || fit <= 0) break;  // memory is not enough
        chunk = std::min(chunk, fit);
        t = t_prefill(c, chunk, comp);
        want = ceil_div(comp + chunk, blk) - held;
      }
      // admit
      if (miss > 0) {
        std::vector<int32_t> fresh;
        for (int64_t b = 0; b < k; ++b) {
          fresh.push_back(s->dev_free.back());
          s->dev_free.pop_back();
        }
        for (int64_t b = 0; b < k; ++b) {
          s->si_host.push_back(r->host_slots[(size_t)b]);
          s->si_dev.push_back(fresh[(size_t)b]);
        }
        for (size_t b = (size_t)k; b < r->host_slots.size(); ++b) s->host_free.push_back(r->host_slots[b]);
        r->host_slots.resize((size_t)k);
        r->host_round.resize((size_t)k);
        r->dev_blocks = fresh;
        r->computed = comp;
        b_rem -= k;
        want -= k;
      }
      for (int64_t b = 0; b < want; ++b) {
        r->dev_blocks.push_back(s->dev_free.back());
        s->dev_free.pop_back();
      }
      r->computed += chunk;
      r->last_sched = now;
      r->in_batch = true;
      t_batch += t;
      members.emplace_back(r, chunk);
    }
    if (members.empty()) t_batch = 0;
  }

  // the batch as the attention layer takes it, in admission order
  s->q_start.push_back(0);
  s->bt_start.push_back(0);
  for (auto& mc : members) {
    Req* r = mc.first;
    s->req_ids.push_back(r->rid);
    s->q_start.push_back(s->q_start.back() + (int32_t)mc.second);
    s->kv_len.push_back((int32_t)r->computed);
    const int64_t nb = ceil_div(r->computed, blk);
    for (int64_t b = 0; b < nb; ++b) s->block_ids.push_back(r->dev_blocks[(size_t)b]);
    s->bt_start.push_back((int32_t)s->block_ids.size());
    s->prio.push_back((uint8_t)r->prio);
  }
  // token delivery at now + T_pd(B), completion
  for (auto& mc : members) {
    Req* r = mc.first;
    if (r->computed != r->need()) continue;
    r->generated += 1;
    s->emitted_req.push_back(r->rid);
    s->emitted_index.push_back((int32_t)r->generated);
    if (r->generated == r->out_len) {
      for (int32_t b : r->dev_blocks) s->dev_free.push_back(b);
      for (int32_t h : r->host_slots) s->host_free.push_back(h);
      r->dev_blocks.clear();
      r->host_slots.clear();
      r->host_round.clear();
      s->finished.push_back(r->rid);
    }
  }
  // asynchronous offload: every n_off^r newly completed full blocks of r get a host copy
  for (auto& mc : members) {
    Req* r = mc.first;
    if (r->generated == r->out_len && r->dev_blocks.empty()) continue;  // finished above
    const int64_t full = r->computed / blk;
    const int64_t pending = full - (int64_t)r->host_slots.size();
    int64_t n_off = (int64_t)c.n_off_base >> (r->prio - 1);
    if (n_off < 1) n_off = 1;
    if (pending >= n_off && (int64_t)s->host_free.size() >= pending) {
      for (int64_t b = (int64_t)r->host_slots.size(); b < full; ++b) {
        const int32_t h = s->host_free.back();
        s->host_free.pop_back();
        r->host_slots.push_back(h);
        r->host_round.push_back(s->round);
        s->so_dev.push_back(r->dev_blocks[(size_t)b]);
        s->so_host.push_back(h);
      }
    }
  }
  for (int64_t rid : s->finished) {
    Req* r = s->by_id[rid];
    s->by_id.erase(rid);
    s->reqs.erase(std::find(s->reqs.begin(), s->reqs.end(), r));
    delete r;
  }

  out->batch.n_req = (int32_t)members.size();
  out->batch.n_tokens = s->q_start.back();
  out->batch.q_start = s->q_start.data();
  out->batch.kv_len = s->kv_len.data();
  out->batch.bt_start = s->bt_start.data();
  out->batch.block_ids = s->block_ids.data();
  out->batch.prio = s->prio.data();
  out->req_ids = s->req_ids.data();
  out->t_budget_ps = t_budget;
  out->phi_ps = phi;
  out->t_batch_ps = t_batch;
  out->copy_budget = b_copy;
  out->n_order = (int32_t)s->order.size();
  out->order = s->order.data();
  out->n_urgent = (int32_t)s->urgent.size();
  out->urgent = s->urgent.data();
  out->n_swap_in = (int32_t)s->si_host.size();
  out->swap_in_host_slots = s->si_host.data();
  out->swap_in_dev_blocks = s->si_dev.data();
  out->n_swap_out = (int32_t)s->so_dev.size();
  out->swap_out_dev_blocks = s->so_dev.data();
  out->swap_out_host_slots = s->so_host.data();
  out->n_evicted = (int32_t)s->evicted.size();
  out->evicted = s->evicted.data();
  out->n_emitted = (int32_t)s->emitted_req.size();
  out->emitted_req = s->emitted_req.data();
  out->emitted_index = s->emitted_index.data();
  out->n_finished = (int32_t)s->finished.size();
  out->finished = s->finished.data();
  out->round = s->round;
  return PS_OK;
}

// Eq. 3 and the two metrics of Sec. 5.1 for one request.
int ps_tdg_score(const ps_sched_cfg* cfg, int32_t prio, int32_t out_len, const int64_t* token_times, int32_t n_times,
                 int64_t* gain, int64_t* ideal_gain, int32_t* slo_attained) {
  if (!cfg || (n_times > 0 && !token_times)) return sched_fail(PS_EINVAL, "ps_tdg_score: NULL argument");
  if (prio < 1 || prio > cfg->n_classes || cfg->n_classes > 8 || out_len < 0 || n_times < 0)
    return sched_fail(PS_EINVAL, "ps_tdg_score: bad class, out_len or n_times");
  const int64_t wc = cfg->class_weight[prio - 1];
  int64_t g = 0;
  for (int32_t i = 1; i <= n_times; ++i) {
    const int64_t deadline = cfg->ttft_slo_ps + (int64_t)(i - 1) * cfg->tpot_slo_ps;
    if (token_times[i - 1] < deadline) g += (i == 1 ? cfg->w_first : cfg->w_decode) * wc;
  }
  if (gain) *gain = g;
  if (ideal_gain) *ideal_gain = out_len > 0 ? (cfg->w_first + (int64_t)(out_len - 1) * cfg->w_decode) * wc : 0;
  if (slo_attained) {
    bool ok = n_times > 0 && token_times[0] < cfg->ttft_slo_ps;
    if (ok && n_times > 1)
      ok = (i128)(token_times[n_times - 1] - token_times[0]) < (i128)cfg->tpot_slo_ps * (n_times - 1);
    *slo_attained = ok ? 1 : 0;
  }
  return PS_OK;
}

// Virtual-clock run of the batch former over an arrival trace.
int ps_sched_simulate(const ps_sched_cfg* cfg, const int32_t* dev_free_order, int32_t n_dev, const int32_t* host_free_order,
                      int32_t n_host, const ps_trace_req* trace, int32_t n_trace, int32_t max_steps, int64_t* token_times,
                      int32_t* n_delivered, ps_sim_result* out) {
  if (!cfg || !out || (n_trace > 0 && !trace) || n_trace < 0 || max_steps < 0)
    return sched_fail(PS_EINVAL, "ps_sched_simulate: bad argument");
  std::memset(out, 0, sizeof *out);
  ps_sched* s = nullptr;
  int rc = ps_sched_create(cfg, dev_free_order, n_dev, host_free_order, n_host, &s);
  if (rc != PS_OK) return rc;
  // arrival order (ties by id); where each request's token times go
  std::vector<int32_t> by_arrival((size_t)n_trace);
  std::vector<int64_t> t_off((size_t)n_trace + 1, 0);
  std::unordered_map<int64_t, int32_t> index_of;
  for (int32_t i = 0; i < n_trace; ++i) {
    by_arrival[(size_t)i] = i;
    t_off[(size_t)i + 1] = t_off[(size_t)i] + std::max(trace[i].out_len, 0);
    if (!index_of.emplace(trace[i].rid, i).second) {
      ps_sched_destroy(s);
      return sched_fail(PS_EINVAL, "ps_sched_simulate: duplicate request id %lld", (long long)trace[i].rid);
    }
  }
  std::sort(by_arrival.begin(), by_arrival.end(), [&](int32_t a, int32_t b) {
    if (trace[a].arrival_ps != trace[b].arrival_ps) return trace[a].arrival_ps < trace[b].arrival_ps;
    return trace[a].rid < trace[b].rid;
  });
  std::vector<int64_t> own_times;
  std::vector<int32_t> own_counts;
  if (!token_times) {
    own_times.assign((size_t)t_off[(size_t)n_trace], 0);
    token_times = own_times.data();
  }
  if (!n_delivered) {
    own_counts.assign((size_t)n_trace, 0);
    n_delivered = own_counts.data();
  }
  for (int32_t i = 0; i < n_trace; ++i) n_delivered[i] = 0;
  // the offload thread on the same clock: a round's copies start when its batch has been computed and
  // the earlier copies are through, and take t_block per block
  std::vector<std::pair<int64_t, int64_t>> inflight;  // (round, completion time), oldest first
  size_t inflight_head = 0;
  int64_t copy_free_at = 0, now = 0;
  int32_t nxt = 0, steps = 0;
  ps_batch_out fb;
  while (steps < max_steps) {
    while (nxt < n_trace && trace[by_arrival[(size_t)nxt]].arrival_ps <= now) {
      const ps_trace_req& p = trace[by_arrival[(size_t)nxt]];
      rc = ps_sched_add_request(s, p.rid, p.arrival_ps, p.prio, p.prompt_len, p.out_len);
      if (rc != PS_OK) {
        ps_sched_destroy(s);
        return rc;
      }
      ++nxt;
    }
    if (s->reqs.empty()) {
      if (nxt >= n_trace) break;
      now = trace[by_arrival[(size_t)nxt]].arrival_ps;
      continue;
    }
    while (inflight_head < inflight.size() && inflight[inflight_head].second <= now)
      (void)ps_sched_offloads_done(s, inflight[inflight_head++].first);
    rc = ps_form_batch(s, now, &fb);
    if (rc != PS_OK) {
      ps_sched_destroy(s);
      return rc;
    }
    ++steps;
    if (fb.n_swap_out > 0) {
      copy_free_at = std::max(copy_free_at, now + fb.t_batch_ps) + (int64_t)fb.n_swap_out * cfg->t_block_ps;
      inflight.emplace_back(fb.round, copy_free_at);
    }
    for (int32_t e = 0; e < fb.n_emitted; ++e) {  // tokens are delivered when the batch ends
      const int32_t i = index_of[fb.emitted_req[e]];
      token_times[t_off[(size_t)i] + n_delivered[i]] = now + fb.t_batch_ps - trace[i].arrival_ps;
      n_delivered[i] += 1;
    }
    for (int32_t f = 0; f < fb.n_finished; ++f) {
      const int32_t i = index_of[fb.finished[f]];
      int64_t g = 0, ideal = 0;
      int32_t ok = 0;
      (void)ps_tdg_score(cfg, trace[i].prio, trace[i].out_len, token_times + t_off[(size_t)i], n_delivered[i], &g, &ideal, &ok);
      out->gain += g;
      out->ideal_gain += ideal;
      out->slo_attained += ok;
      out->finished += 1;
    }
    now += fb.t_batch_ps > 0 ? fb.t_batch_ps : cfg->eta_ps;
  }
  out->steps = steps;
  out->end_ps = now;
  ps_sched_destroy(s);
  return PS_OK;
}

}  // extern "C"
