// Host side of the C ABI declared in include/ps.h: argument validation, work-list
// construction, metadata staging, kernel launches, swap tickets.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <functional>
#include <new>
#include <string>
#include <vector>

#include "ps_internal.h"

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define PS_HIP(call)                                                                          \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess) return fail(PS_EHIP, "%s: %s", #call, hipGetErrorString(e_));       \
  } while (0)

constexpr int kStepSlots = 4;     // pinned staging buffers for ps_step metadata
constexpr int kSwapSlots = 8;     // id staging for swaps
constexpr int kMaxSwap = 16384;   // blocks per swap call
constexpr int kTicketRing = 64;
constexpr int kStagingBlocks = 1024;  // blocks a swap staging buffer holds (64 MiB at 64 KiB per block)

struct StageSlot {
  void* pinned = nullptr;
  size_t cap = 0;
  hipEvent_t ev = nullptr;
  bool in_flight = false;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

// ---- device memory of ps_step_static: one fixed array per GPU, held until the process ends.
// [0, 2 * kStaticMeta): two copies of the batch description, used alternately; the rest: split-K partials.
constexpr size_t kStaticMeta = (size_t)2 << 20;
constexpr size_t kStaticBytes = (size_t)PS_STATIC_SCRATCH_BYTES;
constexpr size_t kStaticPartials = kStaticBytes - 2 * kStaticMeta;
constexpr size_t kStepStaging = kStaticMeta;  // pinned staging per slot, allocated at ps_create
static __device__ __align__(256) unsigned char scratch[kStaticBytes];
constexpr int kMaxDevices = 64;
struct StaticScratch {
  unsigned char* ptr = nullptr;   // device address of `scratch` on this GPU (hipGetSymbolAddress)
  int next = 0;                   // which of the two description copies the next call takes
  hipEvent_t done[2] = {nullptr, nullptr};
  hipStream_t last_stream[2] = {nullptr, nullptr};
  bool used[2] = {false, false};
};
static StaticScratch g_static[kMaxDevices];

// The decode work list of a step (and the merge items of the step: decode's first, prefill's appended).
struct DecodePlan {
  std::vector<ps::DecodeItem> ditems;
  std::vector<int32_t> dslots;  // slot x owns ditems[dslots[x] .. dslots[x+1])
  std::vector<ps::MergeItem> mitems;
};

struct ps_ctx {
  ps_layer_cfg cfg;
  int device = 0;
  int G = 1;
  size_t block_bytes = 0;
  float scale_log2 = 0.f;
  StageSlot step_slot[kStepSlots];
  int step_next = 0;
  StageSlot swap_slot[kSwapSlots];
  int swap_next = 0;
  hipEvent_t ticket_ev[kTicketRing];
  uint64_t ticket_id[kTicketRing];
  uint64_t next_ticket = 1;
  // Device copies of the batch description, double-buffered so that the upload of step n+1 (on the
  // context's copy stream) runs while the kernels of step n still read theirs.
  struct MetaBuf {
    char* dev = nullptr;
    size_t cap = 0;
    hipEvent_t uploaded = nullptr;  // on the copy stream, after the upload
    hipEvent_t done = nullptr;      // on the launching stream, after the last kernel that reads it
    hipStream_t last_stream = nullptr;  // the stream `done` was last recorded on
    bool used = false;
  } meta[2];
  int meta_next = 0;
  hipStream_t copy = nullptr;
  int n_cus = 256;
  int profiling = 0;  // 0 off, 1 phases as they run, 2 decode and prefill roles in launches of their own
  // profiling: the events of the last kProfRing profiled steps; step number prof_n records into slot prof_n % kProfRing
  // (slot 0 exists from ps_create on, the others from the first ps_set_profiling that switches profiling on)
  static constexpr int kProfRing = 64;
  hipEvent_t prof_ring[kProfRing][6];
  uint64_t prof_n = 0;       // profiled steps enqueued since ps_set_profiling
  uint64_t prof_read = 0;    // of which ps_get_step_times has reported
  ps_step_times prof_last;   // its last report
  hipEvent_t* prof_ev_now() { return prof_ring[prof_n % kProfRing]; }
  unsigned long long* clocks_dev = nullptr;  // profiling: clock counters of the attention workgroups (ps_set_profiling allocates)
  int prof_wgs[2] = {0, 0};                  // decode / prefill workgroups of the last profiled step
  bool prof_valid = false;
  int prof_mode = 0;
  DecodePlan plan;
  bool plan_fused = false;  // the plan's decode slots are laid out for the launch whose workgroups carry both kinds of work
  std::vector<ps::PrefillTile> ptiles;
  std::vector<ps::AppendItem> aitems;
  // What ps_step_next_layer needs of the last ps_step: where its batch description sits on the device
  // (offsets of the lists inside the buffer), the pinned slot it was staged in, the partials it needs.
  struct LastStep {
    bool valid = false;
    char* meta_dev = nullptr;       // device copy of the batch description
    MetaBuf* mb = nullptr;          // the context's buffer it lives in (NULL: the static array)
    int slot = 0;
    size_t off[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};  // q_start, kv_len, bt_start, block_ids, aitems, ditems, dslots, mitems, ptiles
    size_t part_bytes = 0;
    bool has_new_kv = false;
  } last;
  // Device staging of the copy-engine swap path, one buffer per direction ([0] out, [1] in), allocated at ps_create
  // when there is a host pool; `done`: the last call that used it, `last_stream`: where.
  struct Staging {
    char* dev = nullptr;
    int blocks = 0;
    hipEvent_t done = nullptr;
    hipStream_t last_stream = nullptr;
    bool used = false;
  } staging[2];
  std::vector<int32_t> seen;  // duplicate detection in swap lists
  std::vector<int64_t> cover;  // scratch of the decode work-list check
};

namespace {

// The planner's picture of the machine: cfg value, or the MI355X default.
struct PlanTuning {
  double stream_TBps, tile_step_us, merge_launch_steps, merge_row_steps, decode_share;
  int knee_cus;
};
PlanTuning tuning_of(const ps_layer_cfg& c) {
  PlanTuning t;
  t.stream_TBps = c.plan_stream_TBps > 0.f ? c.plan_stream_TBps : 6.3;
  t.tile_step_us = c.plan_tile_step_us > 0.f ? c.plan_tile_step_us : 1.78;
  t.merge_launch_steps = c.plan_merge_launch_steps > 0.f ? c.plan_merge_launch_steps : 4.0;
  t.merge_row_steps = c.plan_merge_row_steps > 0.f ? c.plan_merge_row_steps : 0.0047;
  t.decode_share = c.plan_decode_share > 0.f ? c.plan_decode_share : 0.95;
  t.knee_cus = c.plan_decode_knee_cus > 0 ? c.plan_decode_knee_cus : 176;
  return t;
}

// A prefill work item while the launch is being planned: `reach` = its length in 64-token KV tiles.
struct TileKey {
  int64_t reach;
  ps::PrefillTile t;
};

// Prefill: a query tile walks `reach` KV tiles.  In a small launch the longest walks decide when
// it ends; they can be cut into partitions whose partial results the merge kernel combines.
// In:  tiles, one per query tile of every prefill chunk, with its full walk [0, reach).
// Out: tiles replaced by the launch's work items (partitions of the walks, not yet ordered), merge
//      items and partial slots for split rows appended; returns the price of the prefill work with the
//      whole chip, in KV tile steps per CU.
// The time (in KV tile steps) at which a launch ends when `busy` of the n_cus compute units are taken
// until `busy_until` (by the decode workgroups, dispatched first) and the prefill workgroups, `per_tile`
// for each entry of `tiles` (sorted longest first), are handed one by one to whichever unit is free next.
double mixed_makespan(const std::vector<TileKey>& tiles, int per_tile, int n_cus, int busy, double busy_until,
                      std::vector<double>& bins) {
  bins.assign((size_t)n_cus, 0.0);
  for (int i = 0; i < busy && i < n_cus; ++i) bins[(size_t)i] = busy_until;
  auto later = std::greater<double>();
  std::make_heap(bins.begin(), bins.end(), later);
  double end = busy > 0 ? busy_until : 0.0;
  for (auto& t : tiles)
    for (int w = 0; w < per_tile; ++w) {
      std::pop_heap(bins.begin(), bins.end(), later);
      bins.back() += (double)t.reach;
      end = std::max(end, bins.back());
      std::push_heap(bins.begin(), bins.end(), later);
    }
  return end;
}

// A prefill row's KV range is cut into at most this many partitions.
constexpr int kMaxPrefillParts = 32;
// Partial slots a batch of n_tokens may spend on prefill rows whose KV range is split: two per batch token, and 8192 on
// top for small batches (a lone chunk over a long prefix is a handful of workgroups that walk the whole prefix each
// unless every one of its query tiles can be cut), never more than the split can use.
static int64_t prefill_partial_budget(int64_t n_tokens) {
  return std::min<int64_t>((int64_t)kMaxPrefillParts * n_tokens, 2 * n_tokens + 8192);
}

double plan_prefill(ps_ctx* c, const ps_batch* b, std::vector<TileKey>& tiles, int TT, size_t workspace_bytes, int& n_parts) {
  double prefill_steps = 0;
  const PlanTuning tune = tuning_of(c->cfg);
  const int wg_per_tile = c->cfg.n_kv_heads * (c->G / ps::prefill_heads_per_wg(c->G));
  int64_t longest = 0;
  for (auto& t : tiles) longest = std::max(longest, t.reach);
  int64_t split = 0;  // partition length in KV tiles; 0 = none
  bool priced = false;
  {  // default price of the prefill work, in KV tile steps per CU: an even spread
    int64_t total = 0;
    for (auto& t : tiles) total += t.reach;
    prefill_steps = (double)total * wg_per_tile / c->n_cus;
  }
  if (c->cfg.prefill_split_tiles > 0) {
    split = c->cfg.prefill_split_tiles;
  } else if (c->cfg.prefill_split_tiles == 0 && !tiles.empty()) {
    // Candidates: the longest walk cut into k = 1..8, 12, 16, 24 or 32 equal parts.  Each is priced in units of one
    // KV tile step of a workgroup (measured on workload-sized launches): the time the launch
    // ends when workgroups are handed, longest first, to whichever CU is free next, plus the merge
    // (a kernel launch worth 4 steps, and 0.0047 steps per partial row of 32 heads).  Launches of
    // more than 1024 workgroups balance well enough without a cut and are not priced.
    std::vector<int64_t> sizes, bins;
    double best = 0;
    for (int k : {1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 24, 32}) {
      const int64_t cand = (longest + k - 1) / k;
      if (k > 1 && cand < 8) break;
      sizes.clear();
      int64_t rows = 0;
      for (auto& t : tiles) {
        int np = k == 1 ? 1 : (int)std::min<int64_t>((t.reach + cand - 1) / cand, kMaxPrefillParts);
        const int64_t len = (t.reach + np - 1) / np;
        np = (int)((t.reach + len - 1) / len);
        for (int q = 0; q < np; ++q) sizes.push_back(std::min<int64_t>((int64_t)(q + 1) * len, t.reach) - q * len);
        if (np > 1) rows += (int64_t)std::min(TT, b->q_start[t.t.req + 1] - b->q_start[t.t.req] - t.t.q0) * np;
      }
      if (sizes.size() * (size_t)wg_per_tile > 1024) break;
      std::sort(sizes.begin(), sizes.end(), std::greater<int64_t>());
      bins.assign((size_t)c->n_cus, 0);  // min-heap of CU finish times
      auto later = std::greater<int64_t>();
      for (int64_t sz : sizes)
        for (int w = 0; w < wg_per_tile; ++w) {
          std::pop_heap(bins.begin(), bins.end(), later);
          bins.back() += sz;
          std::push_heap(bins.begin(), bins.end(), later);
        }
      const int64_t makespan = *std::max_element(bins.begin(), bins.end());
      const double cost = (double)makespan + (rows > 0 ? tune.merge_launch_steps : 0.0) +
                          tune.merge_row_steps * (c->cfg.n_q_heads / 32.0) * (double)rows;
      if (k == 1 || cost < best) {
        best = cost;
        split = k == 1 ? 0 : cand;
      }
    }
    if (best > 0) {
      prefill_steps = best;
      priced = true;
    }
  }
  // partial slots: the budget above, and whatever the caller's workspace holds; the longest walks are served first
  const size_t slot_bytes = (size_t)c->cfg.n_q_heads * ps::kPartStride * sizeof(float);
  int64_t budget = std::min<int64_t>(prefill_partial_budget(b->n_tokens), (int64_t)(workspace_bytes / slot_bytes) - n_parts);
  if (split > 0) std::stable_sort(tiles.begin(), tiles.end(), [](const TileKey& x, const TileKey& y) { return x.reach > y.reach; });
  std::vector<TileKey> cut;
  for (auto& t : tiles) {
    const int qs = b->q_start[t.t.req], lq = b->q_start[t.t.req + 1] - qs;
    const int rows = std::min(TT, lq - t.t.q0);
    int np = split > 0 ? (int)std::min<int64_t>((t.reach + split - 1) / split, kMaxPrefillParts) : 1;
    if (np > 1 && (int64_t)rows * np > budget) np = 1;
    if (np == 1) {
      t.t.tile_end = (int32_t)t.reach;
      cut.push_back(t);
      continue;
    }
    const int len = (int)((t.reach + np - 1) / np);
    np = (int)((t.reach + len - 1) / len);  // no empty partition: every one starts inside the reach
    budget -= (int64_t)rows * np;
    for (int k = 0; k < np; ++k) {
      ps::PrefillTile q = t.t;
      q.tile_begin = k * len;
      q.tile_end = (int32_t)std::min<int64_t>((int64_t)(k + 1) * len, t.reach);
      q.part = n_parts;
      q.n_parts = np;
      q.k = k;
      cut.push_back(TileKey{q.tile_end - q.tile_begin, q});
    }
    for (int row = 0; row < rows; ++row) c->plan.mitems.push_back(ps::MergeItem{qs + t.t.q0 + row, n_parts + row * np, np, 0});
    n_parts += rows * np;
  }
  tiles.swap(cut);
  if (!priced && !tiles.empty()) {  // forced partition length, or a launch too large to simulate: a bound instead
    int64_t longest_part = 0, rows = 0;
    for (auto& t : tiles) {
      longest_part = std::max(longest_part, t.reach);
      if (t.t.part >= 0 && t.t.k == 0)
        rows += (int64_t)std::min(TT, b->q_start[t.t.req + 1] - b->q_start[t.t.req] - t.t.q0) * t.t.n_parts;
    }
    prefill_steps = std::max(prefill_steps, (double)longest_part) + (rows > 0 ? tune.merge_launch_steps : 0.0) +
                    tune.merge_row_steps * (c->cfg.n_q_heads / 32.0) * (double)rows;
  }
  return prefill_steps;
}

// The checks on a batch description that need no device: PS_EINVAL with a message, or PS_OK and the
// number of cached tokens the decode requests read.  Arrays must be non-NULL and n_req > 0.
int check_batch(const ps_batch* b, int M, int64_t* decode_kv_out) {
  const int n_req = b->n_req;
  if (b->q_start[0] != 0 || b->bt_start[0] != 0) return fail(PS_EINVAL, "q_start[0] and bt_start[0] must be 0");
  int64_t decode_kv = 0;
  for (int r = 0; r < n_req; ++r) {
    const int64_t lq = (int64_t)b->q_start[r + 1] - b->q_start[r];
    const int64_t L = b->kv_len[r];
    if (lq < 1) return fail(PS_EINVAL, "request %d: l_q = %lld < 1", r, (long long)lq);
    if (L < lq) return fail(PS_EINVAL, "request %d: l_q = %lld exceeds kv_len = %lld", r, (long long)lq, (long long)L);
    const int64_t nb = (int64_t)b->bt_start[r + 1] - b->bt_start[r];
    if (nb != (L + ps::kBlockTokens - 1) / ps::kBlockTokens)
      return fail(PS_EINVAL, "request %d: block table has %lld entries, kv_len %lld needs %lld", r, (long long)nb,
                  (long long)L, (long long)((L + ps::kBlockTokens - 1) / ps::kBlockTokens));
    if (lq == 1) decode_kv += L;
  }
  if (b->q_start[n_req] != b->n_tokens) return fail(PS_EINVAL, "q_start[n_req] != n_tokens");
  const int64_t n_table = b->bt_start[n_req];
  for (int64_t i = 0; i < n_table; ++i)
    if ((uint32_t)b->block_ids[i] >= (uint32_t)M)
      return fail(PS_EINVAL, "block_ids[%lld] = %d outside [0, %d)", (long long)i, b->block_ids[i], M);
  *decode_kv_out = decode_kv;
  return PS_OK;
}

// A balanced decode slot holds at least this many 32-token tiles.  Small batches are latency-bound (a wave
// takes its tiles one after the other, about 2 us each): with 4 instead of 16 a layer over 16 requests of
// 1 k tokens takes 20 us instead of 31; large batches have more tiles per slot than that anyway.
constexpr int kMinSlotTiles = 4;

// Decode work list.  Every decode request is cut into segments, and the segments are dealt to
// slots; the decode kernel runs one wave per (slot, kv-head) which walks its slot's segments.
//  - cfg.decode_chunk > 0: fixed partitions of that many tokens, one per slot, longest first.
//  - otherwise: the requests' 32-token tiles, laid end to end in batch order, are cut into S slots
//    of equal length (to within a tile), S chosen so that all waves of the launch are resident at
//    once (cfg.decode_waves, default one per SIMD: measured best) and a slot is not shorter than
//    kMinSlotTiles.  At most S - 1 requests are cut, so there are at most n_req + S segments.
// A request with several segments gets one partials slot per segment and a merge item.
void build_decode_slots(DecodePlan* c, int n_kv_heads, int decode_chunk, const ps_batch* b, const std::vector<int>& reqs,
                        int& n_parts, int waves) {
  c->ditems.clear();
  c->dslots.clear();
  c->dslots.push_back(0);
  auto close_slot = [&]() {
    if ((int)c->ditems.size() > c->dslots.back()) c->dslots.push_back((int32_t)c->ditems.size());
  };
  auto item = [&](int r, int t0, int t1, int part) {
    const int L = b->kv_len[r];
    return ps::DecodeItem{b->bt_start[r], b->q_start[r], t0, t1, part, (L + ps::kBlockTokens - 1) / ps::kBlockTokens, {0, 0}};
  };
  if (decode_chunk > 0) {
    const int CH = decode_chunk;
    for (int r : reqs) {
      const int L = b->kv_len[r], np = (L + CH - 1) / CH;
      if (np == 1) {
        c->ditems.push_back(item(r, 0, L, -1));
      } else {
        c->mitems.push_back(ps::MergeItem{b->q_start[r], n_parts, np, 0});
        for (int k = 0; k < np; ++k) c->ditems.push_back(item(r, k * CH, std::min((k + 1) * CH, L), n_parts++));
      }
    }
    // longest partitions first, so that the tail of the launch is made of short ones
    std::stable_sort(c->ditems.begin(), c->ditems.end(),
                     [](const ps::DecodeItem& a, const ps::DecodeItem& b2) { return a.t1 - a.t0 > b2.t1 - b2.t0; });
    for (size_t i = 1; i <= c->ditems.size(); ++i) c->dslots.push_back((int32_t)i);
    return;
  }
  int64_t T = 0;
  for (int r : reqs) T += (b->kv_len[r] + ps::kTileTokens - 1) / ps::kTileTokens;
  const int64_t S = std::max<int64_t>(1, std::min<int64_t>(waves / n_kv_heads, T / kMinSlotTiles));
  auto boundary = [&](int64_t x) { return ((x + 1) * T + S - 1) / S; };  // nominal end of slot x, in tiles
  int64_t off = 0, x = 0;
  std::vector<int> cuts;  // tile indices inside one request at which a slot ends
  for (int r : reqs) {
    const int L = b->kv_len[r];
    const int n = (L + ps::kTileTokens - 1) / ps::kTileTokens;
    while (x < S - 1 && boundary(x) <= off) {  // slot ends at or before the start of this request
      close_slot();
      ++x;
    }
    cuts.clear();
    while (x < S - 1 && boundary(x) < off + n) cuts.push_back((int)(boundary(x++) - off));  // in (0, n), increasing
    if (cuts.empty()) {
      c->ditems.push_back(item(r, 0, L, -1));
    } else {
      c->mitems.push_back(ps::MergeItem{b->q_start[r], n_parts, (int)cuts.size() + 1, 0});
      int t0 = 0;
      for (int cu : cuts) {
        c->ditems.push_back(item(r, t0, cu * ps::kTileTokens, n_parts++));
        close_slot();
        t0 = cu * ps::kTileTokens;
      }
      c->ditems.push_back(item(r, t0, L, n_parts++));
    }
    off += n;
  }
  close_slot();
}

// Decode work list for the launch whose workgroups carry both kinds of work.  Slot x is walked by a decode wave of
// the prefill workgroups of work item x / slots_per_item, and lasts as long as they do if its share of the decode
// tiles is that of its work item in the prefill work: weight[x] = length of that item's tile walk.  The requests'
// 32-token tiles, laid end to end in batch order, are cut at the cumulative weights (rounded up to kMinSlotTiles
// tiles: short slots are latency-bound); a slot may come out empty, and is kept as an empty range so that slot
// numbers still name their workgroups.  Requests cut by a boundary get one partials slot per segment and a merge item.
void build_weighted_decode_slots(DecodePlan* c, const ps_batch* b, const std::vector<int>& reqs, int& n_parts,
                                 const std::vector<int64_t>& weight) {
  c->ditems.clear();
  c->dslots.assign(1, 0);
  const size_t S = weight.size();
  int64_t T = 0, wtot = 0;
  for (int r : reqs) T += (b->kv_len[r] + ps::kTileTokens - 1) / ps::kTileTokens;
  for (int64_t w : weight) wtot += std::max<int64_t>(w, 0);
  if (wtot < 1) wtot = 1;
  std::vector<int64_t> end(S);  // one past the last tile of slot x, non-decreasing
  {
    int64_t wc = 0;
    for (size_t x = 0; x < S; ++x) {
      wc += std::max<int64_t>(weight[x], 0);
      const int64_t e = (int64_t)(((__int128)T * wc + wtot - 1) / wtot);
      end[x] = x + 1 == S ? T : std::min<int64_t>((e + kMinSlotTiles - 1) / kMinSlotTiles * kMinSlotTiles, T);
    }
  }
  auto item = [&](int r, int t0, int t1, int part) {
    const int L = b->kv_len[r];
    return ps::DecodeItem{b->bt_start[r], b->q_start[r], t0, t1, part, (L + ps::kBlockTokens - 1) / ps::kBlockTokens, {0, 0}};
  };
  auto close_slot = [&]() { c->dslots.push_back((int32_t)c->ditems.size()); };
  int64_t off = 0;  // tiles before the current request
  size_t x = 0;     // the slot the next tile falls into
  for (int r : reqs) {
    const int L = b->kv_len[r];
    const int64_t n = (L + ps::kTileTokens - 1) / ps::kTileTokens;
    while (x + 1 < S && end[x] <= off) {  // slots that end at or before the start of this request (some of them empty)
      close_slot();
      ++x;
    }
    int nseg = 1;
    {
      int64_t pos = off;
      for (size_t y = x; y + 1 < S && end[y] < off + n; ++y)
        if (end[y] > pos) {
          ++nseg;
          pos = end[y];
        }
    }
    if (nseg == 1) {
      c->ditems.push_back(item(r, 0, L, -1));
      // slots that end inside the request without taking a tile of it (their end is its start) were closed above
    } else {
      c->mitems.push_back(ps::MergeItem{b->q_start[r], n_parts, nseg, 0});
      int64_t pos = off;
      while (x + 1 < S && end[x] < off + n) {
        if (end[x] > pos) {
          c->ditems.push_back(item(r, (int)((pos - off) * ps::kTileTokens), (int)((end[x] - off) * ps::kTileTokens), n_parts++));
          pos = end[x];
        }
        close_slot();
        ++x;
      }
      c->ditems.push_back(item(r, (int)((pos - off) * ps::kTileTokens), L, n_parts++));
    }
    off += n;
  }
  while (c->dslots.size() < S + 1) close_slot();
}

// Host-side check of the decode work list before anything is launched from it: every slot a
// non-empty range of items (an empty one only where empty_ok says so), every item inside its request, the segments of a request tiling
// [0, kv_len) exactly.  A mistake here would otherwise become an out-of-bounds access on the GPU.
bool decode_slots_ok(const DecodePlan* c, const ps_batch* b, const std::vector<int>& reqs, std::vector<int64_t>& cover,
                     bool empty_ok = false) {
  const size_t n = c->ditems.size();
  if (c->dslots.empty() || c->dslots.front() != 0 || (size_t)c->dslots.back() != n) return false;
  for (size_t i = 1; i < c->dslots.size(); ++i)
    if (c->dslots[i] < c->dslots[i - 1] || (!empty_ok && c->dslots[i] == c->dslots[i - 1])) return false;
  if (reqs.empty()) return n == 0 && (empty_ok || c->dslots.size() == 1);
  cover.assign((size_t)b->n_tokens, 0);
  std::vector<int> req_of((size_t)b->n_tokens, -1);
  for (int r : reqs) req_of[(size_t)b->q_start[r]] = r;
  for (const ps::DecodeItem& it : c->ditems) {
    if (it.tok < 0 || it.tok >= b->n_tokens || req_of[(size_t)it.tok] < 0) return false;
    const int r = req_of[(size_t)it.tok], L = b->kv_len[r];
    if (it.bt_off != b->bt_start[r] || it.nblk != (L + ps::kBlockTokens - 1) / ps::kBlockTokens) return false;
    if (it.t0 < 0 || it.t0 >= it.t1 || it.t1 > L || it.t0 % ps::kTileTokens != 0) return false;
    if (it.t1 != L && it.t1 % ps::kTileTokens != 0) return false;
    cover[(size_t)it.tok] += it.t1 - it.t0;
  }
  for (int r : reqs)
    if (cover[(size_t)b->q_start[r]] != b->kv_len[r]) return false;
  return true;
}

// Bytes of the metadata block for given sizes (also the layout used by ps_step).
struct MetaLayout {
  size_t q_start, kv_len, bt_start, block_ids, aitems, ditems, dslots, mitems, ptiles, total;
};

MetaLayout meta_layout(int n_req, size_t n_aitems, int64_t n_table, size_t n_ditems, size_t n_dslots,
                       size_t n_mitems, size_t n_ptiles) {
  MetaLayout m;
  size_t o = 0;
  auto put = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes, 256);
    return at;
  };
  m.q_start = put((size_t)(n_req + 1) * 4);
  m.kv_len = put((size_t)n_req * 4);
  m.bt_start = put((size_t)(n_req + 1) * 4);
  m.block_ids = put((size_t)n_table * 4);
  m.aitems = put((size_t)n_aitems * sizeof(ps::AppendItem));
  m.ditems = put(n_ditems * sizeof(ps::DecodeItem));
  m.dslots = put(n_dslots * 4);
  m.mitems = put(n_mitems * sizeof(ps::MergeItem));
  m.ptiles = put(n_ptiles * sizeof(ps::PrefillTile));
  m.total = o;
  return m;
}

constexpr int kMinChunk = 32;

int acquire_slot(StageSlot& s, size_t bytes) {
  if (s.in_flight) {
    PS_HIP(hipEventSynchronize(s.ev));
    s.in_flight = false;
  }
  if (s.cap < bytes) {
    if (s.pinned) PS_HIP(hipHostFree(s.pinned));
    s.pinned = nullptr;
    s.cap = 0;
    size_t cap = align_up(bytes + bytes / 2, 4096);
    PS_HIP(hipHostMalloc(&s.pinned, cap, hipHostMallocDefault));
    s.cap = cap;
  }
  return PS_OK;
}

}  // namespace

extern "C" {

const char* ps_last_error(void) { return g_err.c_str(); }

// used by the host-only scheduler translation unit
void ps_internal_set_error(const char* text) { g_err = text ? text : ""; }

int ps_mixed_launch_faults(uint32_t* out) {
  if (!out) return fail(PS_EINVAL, "ps_mixed_launch_faults: NULL argument");
  unsigned int n = 0;
  if (ps::fused_gave_up_count(&n) != 0) return fail(PS_EHIP, "ps_mixed_launch_faults: reading the device counter failed");
  *out = n;
  return PS_OK;
}

static int check_cfg(const ps_layer_cfg* cfg) {
  if (cfg->head_dim != ps::kHeadDim) return fail(PS_EINVAL, "head_dim must be 128 (got %d)", cfg->head_dim);
  if (cfg->block_tokens != ps::kBlockTokens)
    return fail(PS_EINVAL, "block_tokens must be 16 (got %d)", cfg->block_tokens);
  if (cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads != 0)
    return fail(PS_EINVAL, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", cfg->n_q_heads,
                cfg->n_kv_heads);
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  if (G > 16) return fail(PS_EINVAL, "group size Hq/Hkv = %d exceeds 16", G);
  if (cfg->n_device_blocks < 1 || cfg->n_host_blocks < 0)
    return fail(PS_EINVAL, "n_device_blocks must be >= 1 and n_host_blocks >= 0");
  if ((int64_t)cfg->n_device_blocks * 2 * cfg->n_kv_heads > INT32_MAX / 2)
    return fail(PS_EINVAL, "n_device_blocks * n_kv_heads too large");
  if (cfg->out_dtype != PS_BF16 && cfg->out_dtype != PS_F32) return fail(PS_EINVAL, "bad out_dtype");
  if (cfg->decode_chunk != 0 &&
      (cfg->decode_chunk < kMinChunk || cfg->decode_chunk > 65536 || cfg->decode_chunk % 32 != 0))
    return fail(PS_EINVAL, "decode_chunk must be 0 or a multiple of 32 in [32, 65536]");
  if (cfg->swap_workgroups < 0 || cfg->swap_workgroups > 65536) return fail(PS_EINVAL, "bad swap_workgroups");
  if (cfg->swap_dma_runs < 0 || cfg->swap_dma_runs > 65536) return fail(PS_EINVAL, "swap_dma_runs must be in [0, 65536]");
  if (cfg->own_streams != 0 && cfg->own_streams != 1) return fail(PS_EINVAL, "own_streams must be 0 or 1");
  if (cfg->prefill_split_tiles < -1 || cfg->prefill_split_tiles > 65536)
    return fail(PS_EINVAL, "prefill_split_tiles must be -1, 0 or a positive tile count");
  if (cfg->decode_waves < 0 || cfg->decode_waves > 65536)
    return fail(PS_EINVAL, "decode_waves must be in [0, 65536]");
  if (!(cfg->softmax_scale >= 0.f) || std::isinf(cfg->softmax_scale))
    return fail(PS_EINVAL, "softmax_scale must be finite and >= 0");
  for (float v : {cfg->plan_stream_TBps, cfg->plan_tile_step_us, cfg->plan_merge_launch_steps, cfg->plan_merge_row_steps,
                  cfg->plan_decode_share})
    if (!(v >= 0.f) || std::isinf(v)) return fail(PS_EINVAL, "planner constants must be finite and >= 0 (0 = default)");
  if (cfg->plan_decode_share > 1.f) return fail(PS_EINVAL, "plan_decode_share must be at most 1");
  if (cfg->plan_decode_knee_cus < 0) return fail(PS_EINVAL, "plan_decode_knee_cus must be >= 0");
  if (cfg->mixed_launch < 0 || cfg->mixed_launch > 2) return fail(PS_EINVAL, "mixed_launch must be 0, 1 or 2");
  return PS_OK;
}

int ps_create(const ps_layer_cfg* cfg, ps_ctx** out) {
  if (!cfg || !out) return fail(PS_EINVAL, "ps_create: NULL argument");
  *out = nullptr;
  {
    int rc = check_cfg(cfg);
    if (rc != PS_OK) return rc;
  }
  ps_ctx* c = new (std::nothrow) ps_ctx();
  if (!c) return fail(PS_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  c->G = cfg->n_q_heads / cfg->n_kv_heads;
  c->block_bytes = (size_t)2 * cfg->n_kv_heads * ps::kSliceElems * 2;
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  c->scale_log2 = scale * 1.4426950408889634f;
  for (auto& e : c->ticket_ev) e = nullptr;
  for (auto& slot_ev : c->prof_ring)
    for (auto& e : slot_ev) e = nullptr;
  for (auto& t : c->ticket_id) t = 0;
  hipError_t e = hipGetDevice(&c->device);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, c->device);
  if (e == hipSuccess && c->n_cus < 1) c->n_cus = 1;
  for (int i = 0; i < kStepSlots && e == hipSuccess; ++i) {
    e = hipEventCreateWithFlags(&c->step_slot[i].ev, hipEventDisableTiming);
    // staging for the batch description, large enough for every batch ps_step_static accepts, so that a step
    // only allocates when a batch is larger than that
    if (e == hipSuccess) e = hipHostMalloc(&c->step_slot[i].pinned, kStepStaging, hipHostMallocDefault);
    if (e == hipSuccess) c->step_slot[i].cap = kStepStaging;
  }
  for (int i = 0; i < kSwapSlots && e == hipSuccess; ++i)
    e = hipEventCreateWithFlags(&c->swap_slot[i].ev, hipEventDisableTiming);
  for (int i = 0; i < kTicketRing && e == hipSuccess; ++i)
    e = hipEventCreateWithFlags(&c->ticket_ev[i], hipEventDisableTiming);
  for (int i = 0; i < 6 && e == hipSuccess; ++i) e = hipEventCreate(&c->prof_ring[0][i]);
  if (cfg->own_streams) {
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->copy, hipStreamNonBlocking);
  }
  for (int i = 0; i < 2 && e == hipSuccess; ++i) {
    e = hipEventCreateWithFlags(&c->meta[i].uploaded, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->meta[i].done, hipEventDisableTiming);
  }
  if (cfg->n_host_blocks > 0 && cfg->swap_dma_runs > 0) {
    for (int i = 0; i < 2 && e == hipSuccess; ++i) {
      ps_ctx::Staging& st = c->staging[i];
      st.blocks = std::min(cfg->n_host_blocks, kStagingBlocks);
      e = hipMalloc((void**)&st.dev, (size_t)st.blocks * c->block_bytes);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&st.done, hipEventDisableTiming);
    }
  }
  if (e != hipSuccess) {
    int rc = fail(PS_EHIP, "ps_create: %s", hipGetErrorString(e));
    ps_destroy(c);
    return rc;
  }
  *out = c;
  return PS_OK;
}

void ps_destroy(ps_ctx* c) {
  if (!c) return;
  (void)hipDeviceSynchronize();
  for (auto& s : c->step_slot) {
    if (s.pinned) (void)hipHostFree(s.pinned);
    if (s.ev) (void)hipEventDestroy(s.ev);
  }
  for (auto& s : c->swap_slot) {
    if (s.pinned) (void)hipHostFree(s.pinned);
    if (s.ev) (void)hipEventDestroy(s.ev);
  }
  for (auto& e : c->ticket_ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& slot_ev : c->prof_ring)
    for (auto& e : slot_ev)
      if (e) (void)hipEventDestroy(e);
  if (c->copy) (void)hipStreamDestroy(c->copy);
  if (c->clocks_dev) (void)hipFree(c->clocks_dev);
  for (auto& st : c->staging) {
    if (st.dev) (void)hipFree(st.dev);
    if (st.done) (void)hipEventDestroy(st.done);
  }
  for (auto& mb : c->meta) {
    if (mb.dev) (void)hipFree(mb.dev);
    if (mb.uploaded) (void)hipEventDestroy(mb.uploaded);
    if (mb.done) (void)hipEventDestroy(mb.done);
  }
  delete c;
}

int ps_workspace_bytes(const ps_ctx* c, int32_t max_req, int32_t max_tokens, int64_t max_table_entries,
                       size_t* out_bytes) {
  if (!c || !out_bytes) return fail(PS_EINVAL, "ps_workspace_bytes: NULL argument");
  if (max_req < 0 || max_tokens < 0 || max_table_entries < 0) return fail(PS_EINVAL, "negative size");
  // decode partials: one per segment.  Fixed partitions: every request a decode split at that size;
  // balanced slots: at most one extra segment per slot; a slot holds at least kMinSlotTiles tiles (a
  // request of n table entries has at most (n + 1) / 2 tiles) and there are no more slots than one per
  // decode wave and kv-head.
  const size_t slots_by_tiles = (size_t)((max_table_entries + max_req) / (2 * kMinSlotTiles)) + 1;
  size_t slots_by_waves =
      (size_t)((c->cfg.decode_waves > 0 ? c->cfg.decode_waves : ps::decode_waves_per_wg() * c->n_cus) / c->cfg.n_kv_heads) + 1;
  if (c->cfg.mixed_launch != 1)  // the layout with two decode slots per prefill work item (a query tile, or one of its partitions) may be picked
    slots_by_waves = std::max(slots_by_waves, (size_t)ps::fused_decode_slots(1, c->G) * kMaxPrefillParts *
                                                  ((size_t)max_tokens / ps::prefill_tile_tokens(c->G) + (size_t)max_req) + 1);
  const size_t max_parts = (size_t)max_req + (c->cfg.decode_chunk > 0
                                                 ? (size_t)(max_table_entries * ps::kBlockTokens / c->cfg.decode_chunk)
                                                 : std::min(slots_by_tiles, slots_by_waves));
  // + the partial slots of prefill rows whose KV range is split
  *out_bytes = align_up((max_parts + (size_t)prefill_partial_budget(max_tokens)) * c->cfg.n_q_heads * ps::kPartStride * sizeof(float), 256) + 256;
  return PS_OK;
}

int ps_plan_decode(const ps_layer_cfg* cfg, const ps_batch* b, int32_t waves, int32_t* seg, int32_t seg_cap,
                   int32_t* n_seg, int32_t* n_slots) {
  if (!cfg || !b || !n_seg || !n_slots || (!seg && seg_cap > 0)) return fail(PS_EINVAL, "ps_plan_decode: NULL argument");
  if (cfg->n_kv_heads < 1 || cfg->n_device_blocks < 1 || waves < 1 || seg_cap < 0)
    return fail(PS_EINVAL, "ps_plan_decode: bad n_kv_heads / n_device_blocks / waves / seg_cap");
  if (cfg->decode_chunk != 0 && (cfg->decode_chunk < kMinChunk || cfg->decode_chunk > 65536 || cfg->decode_chunk % 32 != 0))
    return fail(PS_EINVAL, "decode_chunk must be 0 or a multiple of 32 in [32, 65536]");
  *n_seg = *n_slots = 0;
  if (b->n_req < 0 || b->n_tokens < 0) return fail(PS_EINVAL, "negative n_req / n_tokens");
  if (b->n_req == 0) return b->n_tokens == 0 ? PS_OK : fail(PS_EINVAL, "n_tokens != 0 with n_req == 0");
  if (!b->q_start || !b->kv_len || !b->bt_start || !b->block_ids) return fail(PS_EINVAL, "ps_plan_decode: NULL batch array");
  int64_t decode_kv = 0;
  int rc = check_batch(b, cfg->n_device_blocks, &decode_kv);
  if (rc != PS_OK) return rc;
  std::vector<int> reqs;
  for (int r = 0; r < b->n_req; ++r)
    if (b->q_start[r + 1] - b->q_start[r] == 1) reqs.push_back(r);
  DecodePlan plan;
  int n_parts = 0;
  std::vector<int64_t> cover;
  build_decode_slots(&plan, cfg->n_kv_heads, cfg->decode_chunk, b, reqs, n_parts, waves);
  if (!decode_slots_ok(&plan, b, reqs, cover)) return fail(PS_ESTATE, "ps_plan_decode: inconsistent decode work list (library bug)");
  *n_seg = (int32_t)plan.ditems.size();
  *n_slots = (int32_t)plan.dslots.size() - 1;
  if (*n_seg > seg_cap) return fail(PS_ENOMEM, "ps_plan_decode: %d segments, room for %d", *n_seg, seg_cap);
  std::vector<int> req_of((size_t)b->n_tokens, -1);
  for (int r : reqs) req_of[(size_t)b->q_start[r]] = r;
  for (int x = 0; x + 1 < (int)plan.dslots.size(); ++x)
    for (int i = plan.dslots[x]; i < plan.dslots[x + 1]; ++i) {
      const ps::DecodeItem& it = plan.ditems[(size_t)i];
      int32_t* o = seg + (size_t)i * 5;
      o[0] = req_of[(size_t)it.tok];
      o[1] = it.t0;
      o[2] = it.t1;
      o[3] = x;
      o[4] = it.part;
    }
  return PS_OK;
}

int ps_set_profiling(ps_ctx* c, int enabled) {
  if (!c) return fail(PS_EINVAL, "NULL ctx");
  if (enabled < 0 || enabled > 2) return fail(PS_EINVAL, "ps_set_profiling: mode must be 0, 1 or 2");
  if (enabled && !c->clocks_dev) {
    const size_t bytes = (size_t)2 * ps::kClockSlots * 4 * sizeof(unsigned long long);
    PS_HIP(hipMalloc((void**)&c->clocks_dev, bytes));
    PS_HIP(hipMemset(c->clocks_dev, 0, bytes));
  }
  if (enabled)
    for (auto& slot_ev : c->prof_ring)
      for (auto& e : slot_ev)
        if (!e) PS_HIP(hipEventCreate(&e));
  c->profiling = enabled;
  c->prof_valid = false;
  c->prof_n = c->prof_read = 0;
  return PS_OK;
}

int ps_get_step_times(ps_ctx* c, ps_step_times* out) {
  if (!c || !out) return fail(PS_EINVAL, "NULL argument");
  std::memset(out, 0, sizeof *out);
  if (!c->prof_valid) return fail(PS_ESTATE, "no profiled step");
  // the mean over the profiled steps enqueued since the last report (the most recent kProfRing of them): a caller
  // that asks after every step gets that step, one that runs many steps back to back and asks once gets their mean
  // with no host synchronisation in between
  const uint64_t fresh = std::min<uint64_t>(c->prof_n - c->prof_read, ps_ctx::kProfRing);
  if (fresh == 0) {
    *out = c->prof_last;
    return PS_OK;
  }
  double sum[6] = {0, 0, 0, 0, 0, 0};
  for (uint64_t k = c->prof_n - fresh; k < c->prof_n; ++k) {
    hipEvent_t* ev = c->prof_ring[k % ps_ctx::kProfRing];
    PS_HIP(hipEventSynchronize(ev[5]));
    float t = 0.f;
    for (int i = 0; i < 5; ++i) {
      PS_HIP(hipEventElapsedTime(&t, ev[i], ev[i + 1]));
      sum[i] += t;
    }
    PS_HIP(hipEventElapsedTime(&t, ev[0], ev[5]));
    sum[5] += t;
  }
  c->prof_read = c->prof_n;
  const double inv = 1.0 / (double)fresh;
  out->upload_ms = (float)(sum[0] * inv);
  out->append_ms = (float)(sum[1] * inv);
  const float att = (float)(sum[2] * inv), pre = (float)(sum[3] * inv);
  out->merge_ms = (float)(sum[4] * inv);
  if (c->prof_mode == 2) {
    out->decode_ms = att;
    out->prefill_ms = pre;
  }
  out->attention_ms = att + pre;
  out->total_ms = (float)(sum[5] * inv);
  // shader clock of each role's workgroups: the median over the recorded ones of (shader-clock ticks) / (100 MHz ticks)
  if (c->clocks_dev) {
    std::vector<unsigned long long> rec((size_t)2 * ps::kClockSlots * 4);
    PS_HIP(hipMemcpy(rec.data(), c->clocks_dev, rec.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
    std::vector<float> mhz;
    for (int role = 0; role < 2; ++role) {
      mhz.clear();
      const int n = std::min(c->prof_wgs[role], ps::kClockSlots);
      for (int i = 0; i < n; ++i) {
        const unsigned long long* r = &rec[((size_t)role * ps::kClockSlots + i) * 4];
        if (r[3] > r[1] + 20 && r[2] > r[0]) mhz.push_back((float)((double)(r[2] - r[0]) / (double)(r[3] - r[1]) * 100.0));  // at least 0.2 us of life
      }
      float med = 0.f;
      if (!mhz.empty()) {
        std::nth_element(mhz.begin(), mhz.begin() + mhz.size() / 2, mhz.end());
        med = mhz[mhz.size() / 2];
      }
      (role == 0 ? out->decode_mhz : out->prefill_mhz) = med;
    }
  }
  c->prof_last = *out;
  return PS_OK;
}

static int find_ticket(ps_ctx* c, uint64_t ticket, hipEvent_t* ev, bool* done) {
  *done = false;
  if (ticket == 0 || ticket >= c->next_ticket) return fail(PS_ESTATE, "unknown ticket %llu", (unsigned long long)ticket);
  const int slot = (int)(ticket % kTicketRing);
  if (c->ticket_id[slot] != ticket) {  // slot recycled: the older copy finished before reuse
    *done = true;
    return PS_OK;
  }
  *ev = c->ticket_ev[slot];
  return PS_OK;
}

// The work lists of one step (append items, decode slots, prefill tiles, merge items) into c->plan, c->ptiles
// and c->aitems; n_parts = partial slots they use.  Host work only: c needs cfg, G, block_bytes, n_cus and
// profiling set, nothing of the device.
static int plan_batch(ps_ctx* c, const ps_batch* b, bool has_new_kv, size_t workspace_bytes, int64_t decode_kv,
                      int& n_parts_out, int64_t* prefill_split_out) {
  const int n_req = b->n_req;
  const int TT = ps::prefill_tile_tokens(c->G);
  c->plan.ditems.clear();
  c->plan.dslots.assign(1, 0);
  c->plan.mitems.clear();
  c->ptiles.clear();
  c->aitems.clear();
  int n_parts = 0;
  std::vector<TileKey> tiles;
  std::vector<int> decode_reqs;
  for (int r = 0; r < n_req; ++r) {
    const int qs = b->q_start[r], lq = b->q_start[r + 1] - qs, L = b->kv_len[r];
    if (has_new_kv)
      for (int lb = (L - lq) / ps::kBlockTokens; lb * ps::kBlockTokens < L; ++lb) {
        const int b0 = lb * ps::kBlockTokens;
        const int lo = std::max(L - lq, b0), hi = std::min(L, b0 + ps::kBlockTokens);  // new positions in this block
        c->aitems.push_back(ps::AppendItem{b->block_ids[b->bt_start[r] + lb], qs + lo - (L - lq), lo - b0, hi - lo});
      }
    if (lq == 1) {
      decode_reqs.push_back(r);
    } else {
      const int p = L - lq;
      for (int q0 = 0; q0 < lq; q0 += TT) {
        const int last = std::min(q0 + TT, lq) - 1;  // KV tiles (64 tokens) any query of the tile can see
        tiles.push_back(TileKey{(p + last) / 64 + 1, ps::PrefillTile{r, q0, 0, 0, -1, 1, 0, 0}});
      }
    }
  }
  const double prefill_steps = plan_prefill(c, b, tiles, TT, workspace_bytes, n_parts);
  // launch order of the prefill work items: heaviest partitions first, so the tail of the launch is made of short ones
  std::stable_sort(tiles.begin(), tiles.end(), [](const TileKey& a, const TileKey& b2) { return a.reach > b2.reach; });

  // Decode slots.  With prefill work in the same launch the decode workgroups get the share of the
  // CUs that makes both kinds of work end together (each priced at its full-chip speed: 6.3 TB/s
  // for the cache stream, 1.78 us per KV tile step of a prefill workgroup; the decode share is cut
  // by 5 %: prefill workgroups inherit CUs that decode leaves early, never the other way round).
  {
    int waves = c->cfg.decode_waves > 0 ? c->cfg.decode_waves : ps::decode_waves_per_wg() * c->n_cus;
    // Every workgroup carries both kinds of work (two decode slots per prefill work item and z-split).  Forced by
    // cfg.mixed_launch = 2; picked by the library when neither kind of work dwarfs the other and there is at least one
    // prefill workgroup per compute unit: the prefill work priced at no more than 8 times the decode work, and at no less
    // than 0.65 times it when the walks are long (64 KV tiles or more per workgroup on average), no less than it when they
    // are of 32 tiles or more, no less than 1.6 times it when they are shorter.
    // Measured on an MI355X against disjoint units, by that ratio.  Launches of 2048 workgroups with walks of 72 tiles
    // on average: 10, the same; 7.2, -2 %; 5.8, -3 %; 4.2, -5 %; 3.3, -6 %; 1.8, -11 %; 1.2, -14 %; 0.9, -10 %; 0.7, -4 %;
    // 0.59 and 0.43, 2 % slower; 0.28, 8 % slower.  Launches of 256 to 512 workgroups: long walks 2.9, -5 %; 1.7, -16 %;
    // 1.3, -18 %; 0.93, -9 %; 0.73, -10 %; walks of 24 to 34 tiles 1.4, -4 to -21 %; 1.1, 2 % slower; 0.85, 6 % slower;
    // 0.79, -9 %; 0.71, 3 % slower; 0.64, 14 % slower; 0.43, 3 to 21 % slower; walks of 12 to 20 tiles 1.9, -10 %;
    // 1.8, -12 %; 1.3, 19 % slower; 1.15, 16 to 26 % slower.
    const bool fusable = c->cfg.decode_waves == 0 && c->cfg.decode_chunk == 0 && c->profiling != 2 && !decode_reqs.empty() &&
                         !tiles.empty() && ps::fused_supports(c->G) &&
                         (int64_t)ps::fused_decode_slots((int)tiles.size(), c->G) * c->cfg.n_kv_heads <= INT32_MAX;
    c->plan_fused = fusable && c->cfg.mixed_launch == 2;
    if (fusable && c->cfg.mixed_launch == 0) {
      const PlanTuning tune = tuning_of(c->cfg);
      const double t_d = (double)decode_kv * (double)(c->block_bytes / ps::kBlockTokens) / (tune.stream_TBps * 1e6);  // us
      const double t_p = prefill_steps * tune.tile_step_us;
      const int64_t wgs = (int64_t)tiles.size() * c->cfg.n_kv_heads * (c->G / ps::prefill_heads_per_wg(c->G));
      int64_t walk_sum = 0;
      for (auto& t : tiles) walk_sum += t.reach;
      const double lo = walk_sum >= 64 * (int64_t)tiles.size() ? 0.65 : walk_sum >= 32 * (int64_t)tiles.size() ? 1.0 : 1.6;
      c->plan_fused = t_p >= lo * t_d && t_p <= 8.0 * t_d && wgs >= (int64_t)c->n_cus;
    }
    if (c->plan_fused) {
      waves = ps::fused_decode_slots((int)tiles.size(), c->G) * c->cfg.n_kv_heads;
    } else if (c->cfg.decode_waves == 0 && c->profiling != 2 && !decode_reqs.empty() && !tiles.empty()) {
      const PlanTuning tune = tuning_of(c->cfg);
      const double t_d = (double)decode_kv * (double)(c->block_bytes / ps::kBlockTokens) / (tune.stream_TBps * 1e6);  // us
      const double t_p = prefill_steps * tune.tile_step_us;
      const int lo = std::min(8, c->n_cus), hi = c->n_cus - 8;
      int cus = (int)(tune.decode_share * c->n_cus * t_d / (t_d + t_p));
      cus = std::max(lo, std::min(cus, hi));
      // Few, equally long prefill workgroups (one long chunk that outweighs the decode work) pack badly
      // next to a small decode share:
      // they run in rounds, and the decode units come free in the middle of one.  Larger shares are
      // priced too: the decode workgroups on n units last t_d stretched by 176/n below 176 units
      // (above, HBM is the limit) and by 5 % for the prefill traffic next to them; the launch ends when
      // the prefill workgroups, handed to whichever unit is free next, are through.  A larger share
      // wins only if it ends the launch 2 % sooner.
      const int wg_per_tile = c->cfg.n_kv_heads * (c->G / ps::prefill_heads_per_wg(c->G));
      if (t_p > t_d && tiles.size() * (size_t)wg_per_tile <= 1024) {
        std::vector<TileKey> sorted(tiles);
        std::stable_sort(sorted.begin(), sorted.end(), [](const TileKey& a, const TileKey& b2) { return a.reach > b2.reach; });
        std::vector<double> bins;
        auto ends = [&](int n) {
          const double d = t_d / tune.tile_step_us * 1.05 * std::max(1.0, (double)tune.knee_cus / n);
          return mixed_makespan(sorted, wg_per_tile, c->n_cus, n, d, bins);
        };
        double best = ends(cus);
        for (int n = std::max(128, (cus / 32 + 1) * 32); n <= hi; n += 32) {
          const double e = ends(n);
          if (e < 0.98 * best) {
            best = e;
            cus = n;
          }
        }
      }
      waves = ps::decode_waves_per_wg() * cus;
    }
    if (c->plan_fused) {
      // slot x goes with the workgroups of work item (x / slots per item) of the launch order fixed above
      const int per_item = ps::fused_decode_slots(1, c->G);
      std::vector<int64_t> weight((size_t)per_item * tiles.size());
      for (size_t x = 0; x < weight.size(); ++x) weight[x] = tiles[x / (size_t)per_item].reach;
      build_weighted_decode_slots(&c->plan, b, decode_reqs, n_parts, weight);
    } else {
      build_decode_slots(&c->plan, c->cfg.n_kv_heads, c->cfg.decode_chunk, b, decode_reqs, n_parts, waves);
    }
    if (!decode_slots_ok(&c->plan, b, decode_reqs, c->cover, c->plan_fused))
      return fail(PS_ESTATE, "ps_step: inconsistent decode work list (library bug)");
  }

  for (auto& t : tiles) c->ptiles.push_back(t.t);
  n_parts_out = n_parts;
  if (prefill_split_out) {
    *prefill_split_out = 0;
    for (auto& t : c->ptiles)
      if (t.part >= 0) *prefill_split_out = std::max<int64_t>(*prefill_split_out, t.tile_end - t.tile_begin);
  }
  return PS_OK;
}

// The launches of one step over the batch description that c->last points to: prologue (upload of
// `upload_bytes` from the pinned slot `h`, if any, and the append of the new K/V rows), attention,
// merge.
static int launch_phases(ps_ctx* c, const char* h, size_t upload_bytes, const ps::AppendItem* aitems_src, const void* q,
                         const void* k_new, const void* v_new, void* kv_cache, void* out, void* workspace,
                         hipStream_t stream) {
  StageSlot& slot = c->step_slot[c->last.slot];
  const size_t* off = c->last.off;
  const int prof = c->profiling;
  char* w = c->last.meta_dev;

  ps::StepParams P;
  P.q_start = (const int32_t*)(w + off[0]);
  P.kv_len = (const int32_t*)(w + off[1]);
  P.bt_start = (const int32_t*)(w + off[2]);
  P.block_ids = (const int32_t*)(w + off[3]);
  P.ditems = (const ps::DecodeItem*)(w + off[5]);
  P.dslots = (const int32_t*)(w + off[6]);
  P.mitems = (const ps::MergeItem*)(w + off[7]);
  P.ptiles = (const ps::PrefillTile*)(w + off[8]);
  P.partials = (float*)workspace;
  P.clocks = prof ? c->clocks_dev : nullptr;
  P.q = (const uint16_t*)q;
  P.k_new = (const uint16_t*)k_new;
  P.v_new = (const uint16_t*)v_new;
  P.cache = (uint16_t*)kv_cache;
  P.out = out;
  P.Hq = c->cfg.n_q_heads;
  P.Hkv = c->cfg.n_kv_heads;
  P.G = c->G;
  P.out_f32 = c->cfg.out_dtype == PS_F32;
  P.scale_log2 = c->scale_log2;

  // Prologue: one launch.  It appends the new K/V rows and, unless the context's copy stream has
  // already brought the batch description over, uploads it with a kernel that reads the pinned slot
  // over the host link (a third of the latency of a DMA copy).
  PS_HIP(ps::launch_prologue(P, h, w, upload_bytes, aitems_src, k_new ? (int)c->aitems.size() : 0, stream));
  if (h && (upload_bytes > 0 || k_new)) PS_HIP(hipEventRecord(slot.ev, stream));  // last reader of the pinned slot
  if (prof) PS_HIP(hipEventRecord(c->prof_ev_now()[2], stream));
  // Attention: one launch for the decode slots and the prefill tiles (decode streams the cache at
  // HBM speed and leaves the matrix pipes idle, prefill is the opposite: they run side by side on
  // disjoint CUs).  Profiling mode 2 gives each its own launch instead.
  const int n_slots = (int)c->plan.dslots.size() - 1;
  if (prof == 2) {
    PS_HIP(ps::launch_attention(P, n_slots, 0, stream, &c->prof_wgs[0], nullptr));
    PS_HIP(hipEventRecord(c->prof_ev_now()[3], stream));
    PS_HIP(ps::launch_attention(P, 0, (int)c->ptiles.size(), stream, nullptr, &c->prof_wgs[1]));
    PS_HIP(hipEventRecord(c->prof_ev_now()[4], stream));
  } else {
    if (c->plan_fused) {
      PS_HIP(ps::launch_fused(P, n_slots, (int)c->ptiles.size(), stream, &c->prof_wgs[1]));
      c->prof_wgs[0] = c->prof_wgs[1];
    } else {
      PS_HIP(ps::launch_attention(P, n_slots, (int)c->ptiles.size(), stream, &c->prof_wgs[0], &c->prof_wgs[1]));
    }
    if (prof) {
      PS_HIP(hipEventRecord(c->prof_ev_now()[3], stream));
      PS_HIP(hipEventRecord(c->prof_ev_now()[4], stream));
    }
  }
  PS_HIP(ps::launch_merge(P, 0, (int)c->plan.mitems.size(), stream));
  if (prof) {
    PS_HIP(hipEventRecord(c->prof_ev_now()[5], stream));
    ++c->prof_n;
    c->prof_valid = true;
    c->prof_mode = prof;
  }
  // whoever writes this copy of the batch description next (two steps on, maybe from another stream) waits for this
  if (c->last.mb) {
    PS_HIP(hipEventRecord(c->last.mb->done, stream));
    c->last.mb->last_stream = stream;
  } else {
    StaticScratch& ss = g_static[c->device];
    const int which = w == (char*)ss.ptr ? 0 : 1;
    PS_HIP(hipEventRecord(ss.done[which], stream));
    ss.last_stream[which] = stream;
  }
  return PS_OK;
}

// Brings the address of this GPU's `scratch` array into g_static (once per device, with that device current).
static int static_scratch(ps_ctx* c, StaticScratch** out) {
  int cur = -1;
  PS_HIP(hipGetDevice(&cur));
  if (cur != c->device) return fail(PS_ESTATE, "ps_step_static: the context was created on device %d, current is %d", c->device, cur);
  if (cur < 0 || cur >= kMaxDevices) return fail(PS_EINVAL, "ps_step_static: device index %d not supported", cur);
  StaticScratch& ss = g_static[cur];
  if (!ss.ptr) {
    void* p = nullptr;
    PS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(PS_EHIP, "hipGetSymbolAddress returned NULL");
    for (int i = 0; i < 2; ++i) PS_HIP(hipEventCreateWithFlags(&ss.done[i], hipEventDisableTiming));
    ss.ptr = (unsigned char*)p;
  }
  *out = &ss;
  return PS_OK;
}

static int step_impl(ps_ctx* c, const ps_batch* b, const void* q, const void* k_new, const void* v_new, void* kv_cache,
                     void* out, void* workspace, size_t workspace_bytes, void* hip_stream, uint64_t wait_ticket,
                     bool use_static) {
  if (!c || !b) return fail(PS_EINVAL, "ps_step: NULL ctx or batch");
  c->last.valid = false;  // the work lists are rebuilt below; set again once this step is enqueued
  if (b->n_req < 0 || b->n_tokens < 0) return fail(PS_EINVAL, "negative n_req / n_tokens");
  hipStream_t stream = (hipStream_t)hip_stream;
  hipEvent_t wait_ev = nullptr;
  if (wait_ticket != 0) {
    bool done = false;
    int rc = find_ticket(c, wait_ticket, &wait_ev, &done);
    if (rc != PS_OK) return rc;
    if (done) wait_ev = nullptr;
  }
  if (b->n_req == 0) {
    if (b->n_tokens != 0) return fail(PS_EINVAL, "n_tokens != 0 with n_req == 0");
    if (wait_ev) PS_HIP(hipStreamWaitEvent(stream, wait_ev, 0));
    return PS_OK;
  }
  if (!b->q_start || !b->kv_len || !b->bt_start || !b->block_ids)
    return fail(PS_EINVAL, "ps_step: NULL batch array");
  StaticScratch* ss = nullptr;
  if (use_static) {  // the library's fixed array takes the place of the caller's workspace
    int rc = static_scratch(c, &ss);
    if (rc != PS_OK) return rc;
    workspace = ss->ptr + 2 * kStaticMeta;
    workspace_bytes = kStaticPartials;
  }
  if (!q || !kv_cache || !out || !workspace) return fail(PS_EINVAL, "ps_step: NULL tensor pointer");
  if ((k_new == nullptr) != (v_new == nullptr)) return fail(PS_EINVAL, "k_new and v_new must be given together");
  if (((uintptr_t)workspace & 255) != 0) return fail(PS_EINVAL, "workspace must be 256-byte aligned");
  if ((((uintptr_t)q | (uintptr_t)kv_cache | (uintptr_t)out | (uintptr_t)k_new | (uintptr_t)v_new) & 15) != 0)
    return fail(PS_EINVAL, "tensor pointers must be 16-byte aligned");

  // ---- validation, O(batch description)
  const int n_req = b->n_req;
  int64_t decode_kv = 0;
  {
    int rc = check_batch(b, c->cfg.n_device_blocks, &decode_kv);
    if (rc != PS_OK) return rc;
  }
  const int64_t n_table = b->bt_start[n_req];

  // ---- work lists
  int n_parts = 0;
  {
    int rc = plan_batch(c, b, k_new != nullptr, workspace_bytes, decode_kv, n_parts, nullptr);
    if (rc != PS_OK) return rc;
  }

  const MetaLayout ml = meta_layout(n_req, c->aitems.size(), n_table, c->plan.ditems.size(), c->plan.dslots.size(),
                                     c->plan.mitems.size(), c->ptiles.size());
  const size_t part_bytes = align_up((size_t)n_parts * c->cfg.n_q_heads * ps::kPartStride * sizeof(float), 256);
  if (part_bytes > workspace_bytes)
    return fail(PS_ENOMEM, use_static ? "ps_step_static: the batch needs %zu bytes of split-K partials, the fixed array holds %zu"
                                      : "workspace too small: need %zu bytes, have %zu", part_bytes, workspace_bytes);
  if (use_static && ml.total > kStaticMeta)
    return fail(PS_ENOMEM, "ps_step_static: the batch description takes %zu bytes, the fixed array holds %zu per step", ml.total,
                kStaticMeta);

  // ---- stage + upload metadata
  StageSlot& slot = c->step_slot[c->step_next];
  if (use_static && slot.cap < ml.total)  // cannot happen while kStepStaging >= kStaticMeta; never allocate here
    return fail(PS_ENOMEM, "ps_step_static: staging slot of %zu bytes too small for %zu", slot.cap, ml.total);
  c->step_next = (c->step_next + 1) % kStepSlots;
  int rc = acquire_slot(slot, ml.total);
  if (rc != PS_OK) return rc;
  char* h = (char*)slot.pinned;
  std::memcpy(h + ml.q_start, b->q_start, (size_t)(n_req + 1) * 4);
  std::memcpy(h + ml.kv_len, b->kv_len, (size_t)n_req * 4);
  std::memcpy(h + ml.bt_start, b->bt_start, (size_t)(n_req + 1) * 4);
  std::memcpy(h + ml.block_ids, b->block_ids, (size_t)n_table * 4);
  if (!c->aitems.empty()) std::memcpy(h + ml.aitems, c->aitems.data(), c->aitems.size() * sizeof(ps::AppendItem));
  if (!c->plan.ditems.empty()) std::memcpy(h + ml.ditems, c->plan.ditems.data(), c->plan.ditems.size() * sizeof(ps::DecodeItem));
  if (!c->plan.dslots.empty()) std::memcpy(h + ml.dslots, c->plan.dslots.data(), c->plan.dslots.size() * 4);
  if (!c->plan.mitems.empty()) std::memcpy(h + ml.mitems, c->plan.mitems.data(), c->plan.mitems.size() * sizeof(ps::MergeItem));
  if (!c->ptiles.empty()) std::memcpy(h + ml.ptiles, c->ptiles.data(), c->ptiles.size() * sizeof(ps::PrefillTile));

  const int prof = c->profiling;
  if (use_static) {
    // the copy of the batch description that the call before last used; if that call ran on another stream this
    // one waits for it (calls that overlap on one GPU share the array: the caller keeps them ordered)
    const int which = ss->next;
    ss->next ^= 1;
    if (wait_ev) PS_HIP(hipStreamWaitEvent(stream, wait_ev, 0));
    if (ss->used[which] && ss->last_stream[which] != stream) PS_HIP(hipStreamWaitEvent(stream, ss->done[which], 0));
    ss->used[which] = true;
    if (prof) {
      PS_HIP(hipEventRecord(c->prof_ev_now()[0], stream));
      PS_HIP(hipEventRecord(c->prof_ev_now()[1], stream));
    }
    slot.in_flight = true;
    c->last.valid = false;
    c->last.meta_dev = (char*)ss->ptr + (size_t)which * kStaticMeta;
    c->last.mb = nullptr;
    c->last.slot = (int)(&slot - c->step_slot);
    const size_t offs[9] = {ml.q_start, ml.kv_len, ml.bt_start, ml.block_ids, ml.aitems, ml.ditems, ml.dslots, ml.mitems, ml.ptiles};
    for (int i = 0; i < 9; ++i) c->last.off[i] = offs[i];
    c->last.part_bytes = part_bytes;
    c->last.has_new_kv = k_new != nullptr;
    // ps_step_next_layer does not follow a static step: last.valid stays false
    return launch_phases(c, h, ml.total, (const ps::AppendItem*)(h + ml.aitems), q, k_new, v_new, kv_cache, out, workspace, stream);
  }
  // upload on the copy stream into the buffer that step n-2 used, once that step is done with it
  ps_ctx::MetaBuf& mb = c->meta[c->meta_next];
  c->meta_next ^= 1;
  if (mb.cap < ml.total) {  // grow (rare): nothing may still be reading the old buffer
    if (mb.dev) {
      PS_HIP(hipDeviceSynchronize());
      PS_HIP(hipFree(mb.dev));
      mb.dev = nullptr;
      mb.cap = 0;
    }
    const size_t cap = align_up(ml.total + ml.total / 2, 1 << 16);
    PS_HIP(hipMalloc((void**)&mb.dev, cap));
    mb.cap = cap;
    mb.used = false;
  }
  if (c->copy) {  // own copy stream: the upload does not wait for the caller's earlier work
    if (mb.used) PS_HIP(hipStreamWaitEvent(c->copy, mb.done, 0));
    PS_HIP(hipMemcpyAsync(mb.dev, h, ml.total, hipMemcpyHostToDevice, c->copy));
    PS_HIP(hipEventRecord(slot.ev, c->copy));
    PS_HIP(hipEventRecord(mb.uploaded, c->copy));
    if (wait_ev) PS_HIP(hipStreamWaitEvent(stream, wait_ev, 0));
    if (prof) PS_HIP(hipEventRecord(c->prof_ev_now()[0], stream));
    PS_HIP(hipStreamWaitEvent(stream, mb.uploaded, 0));
  } else {  // everything on the caller's stream (the two buffers still alternate)
    if (wait_ev) PS_HIP(hipStreamWaitEvent(stream, wait_ev, 0));
    // the step before last read this copy of the description; on the same stream it is over by order, on another
    // stream this one waits for it before the prologue overwrites the lists
    if (mb.used && mb.last_stream != stream) PS_HIP(hipStreamWaitEvent(stream, mb.done, 0));
    if (prof) PS_HIP(hipEventRecord(c->prof_ev_now()[0], stream));
    // the upload is part of the prologue kernel launched below
  }
  slot.in_flight = true;
  mb.used = true;
  if (prof) PS_HIP(hipEventRecord(c->prof_ev_now()[1], stream));
  c->last.valid = false;
  c->last.meta_dev = mb.dev;
  c->last.mb = &mb;
  c->last.slot = (int)(&slot - c->step_slot);
  const size_t offs[9] = {ml.q_start, ml.kv_len, ml.bt_start, ml.block_ids, ml.aitems, ml.ditems, ml.dslots, ml.mitems, ml.ptiles};
  for (int i = 0; i < 9; ++i) c->last.off[i] = offs[i];
  c->last.part_bytes = part_bytes;
  c->last.has_new_kv = k_new != nullptr;
  rc = launch_phases(c, h, c->copy ? 0 : ml.total, (const ps::AppendItem*)(h + ml.aitems), q, k_new, v_new, kv_cache, out,
                     workspace, stream);
  if (rc == PS_OK) c->last.valid = true;
  return rc;
}

int ps_step(ps_ctx* c, const ps_batch* b, const void* q, const void* k_new, const void* v_new, void* kv_cache,
            void* out, void* workspace, size_t workspace_bytes, void* hip_stream, uint64_t wait_ticket) {
  return step_impl(c, b, q, k_new, v_new, kv_cache, out, workspace, workspace_bytes, hip_stream, wait_ticket, false);
}

int ps_step_static(ps_ctx* c, const ps_batch* b, const void* q, const void* k_new, const void* v_new, void* kv_cache,
                   void* out, void* hip_stream, uint64_t wait_ticket) {
  return step_impl(c, b, q, k_new, v_new, kv_cache, out, nullptr, 0, hip_stream, wait_ticket, true);
}

int ps_step_next_layer(ps_ctx* c, const void* q, const void* k_new, const void* v_new, void* kv_cache, void* out,
                       void* workspace, size_t workspace_bytes, void* hip_stream, uint64_t wait_ticket) {
  if (!c) return fail(PS_EINVAL, "ps_step_next_layer: NULL ctx");
  if (!c->last.valid) return fail(PS_ESTATE, "ps_step_next_layer: no batch from an earlier ps_step on this context");
  hipStream_t stream = (hipStream_t)hip_stream;
  hipEvent_t wait_ev = nullptr;
  if (wait_ticket != 0) {
    bool done = false;
    int rc = find_ticket(c, wait_ticket, &wait_ev, &done);
    if (rc != PS_OK) return rc;
    if (done) wait_ev = nullptr;
  }
  if (!q || !kv_cache || !out || !workspace) return fail(PS_EINVAL, "ps_step_next_layer: NULL tensor pointer");
  if ((k_new == nullptr) != (v_new == nullptr)) return fail(PS_EINVAL, "k_new and v_new must be given together");
  if ((k_new != nullptr) != c->last.has_new_kv)
    return fail(PS_EINVAL, "ps_step_next_layer: k_new/v_new must be given exactly when the ps_step it follows had them");
  if (((uintptr_t)workspace & 255) != 0) return fail(PS_EINVAL, "workspace must be 256-byte aligned");
  if ((((uintptr_t)q | (uintptr_t)kv_cache | (uintptr_t)out | (uintptr_t)k_new | (uintptr_t)v_new) & 15) != 0)
    return fail(PS_EINVAL, "tensor pointers must be 16-byte aligned");
  if (c->last.part_bytes > workspace_bytes)
    return fail(PS_ENOMEM, "workspace too small: need %zu bytes, have %zu", c->last.part_bytes, workspace_bytes);
  if (wait_ev) PS_HIP(hipStreamWaitEvent(stream, wait_ev, 0));
  if (c->profiling) {
    PS_HIP(hipEventRecord(c->prof_ev_now()[0], stream));
    PS_HIP(hipEventRecord(c->prof_ev_now()[1], stream));
  }
  // the append items are taken from the device copy of the batch description this time
  const char* w = c->last.meta_dev;
  // a call on another stream than the one the batch was uploaded on: ordered by the caller (see ps.h), but the wait is cheap
  if (c->last.mb && c->last.mb->last_stream != stream) PS_HIP(hipStreamWaitEvent(stream, c->last.mb->done, 0));
  return launch_phases(c, nullptr, 0, (const ps::AppendItem*)(w + c->last.off[4]), q, k_new, v_new, kv_cache, out, workspace,
                       stream);
}

int ps_plan_launch(const ps_layer_cfg* cfg, const ps_batch* b, int32_t n_cus, int32_t* out6) {
  if (!cfg || !b || !out6) return fail(PS_EINVAL, "ps_plan_launch: NULL argument");
  for (int i = 0; i < 6; ++i) out6[i] = 0;
  {
    int rc = check_cfg(cfg);
    if (rc != PS_OK) return rc;
  }
  if (n_cus < 1 || n_cus > 65536) return fail(PS_EINVAL, "ps_plan_launch: n_cus must be in [1, 65536]");
  if (b->n_req < 0 || b->n_tokens < 0) return fail(PS_EINVAL, "negative n_req / n_tokens");
  if (b->n_req == 0) return b->n_tokens == 0 ? PS_OK : fail(PS_EINVAL, "n_tokens != 0 with n_req == 0");
  if (!b->q_start || !b->kv_len || !b->bt_start || !b->block_ids) return fail(PS_EINVAL, "ps_plan_launch: NULL batch array");
  int64_t decode_kv = 0;
  {
    int rc = check_batch(b, cfg->n_device_blocks, &decode_kv);
    if (rc != PS_OK) return rc;
  }
  ps_ctx c;  // host fields only: nothing of the device is created or touched
  c.cfg = *cfg;
  c.G = cfg->n_q_heads / cfg->n_kv_heads;
  c.block_bytes = (size_t)2 * cfg->n_kv_heads * ps::kSliceElems * 2;
  c.n_cus = n_cus;
  int n_parts = 0;
  int64_t split = 0;
  int rc = plan_batch(&c, b, false, (size_t)1 << 62, decode_kv, n_parts, &split);
  if (rc != PS_OK) return rc;
  const int n_slots = (int)c.plan.dslots.size() - 1;
  const int dw = ps::decode_waves_per_wg();
  out6[0] = n_slots * cfg->n_kv_heads;
  out6[1] = n_slots;
  out6[2] = c.plan_fused ? 0 : (n_slots > 0 ? (n_slots + dw - 1) / dw * cfg->n_kv_heads : 0);
  out6[3] = (int32_t)c.ptiles.size() * cfg->n_kv_heads * (c.G / ps::prefill_heads_per_wg(c.G));
  out6[4] = (int32_t)split;
  out6[5] = n_parts;
  return PS_OK;
}

static int swap_common(ps_ctx* c, bool out_dir, const int32_t* dev_ids, const int32_t* host_ids, int32_t n,
                       int32_t copy_budget, const void* kv_cache, const void* host_pool, void* side_stream,
                       int32_t* n_done, uint64_t* ticket) {
  const char* fn = out_dir ? "ps_swap_out" : "ps_swap_in";
  if (!c || !n_done || !ticket) return fail(PS_EINVAL, "%s: NULL ctx / n_done / ticket", fn);
  *n_done = 0;
  *ticket = 0;
  if (n < 0) return fail(PS_EINVAL, "%s: n < 0", fn);
  const int m = copy_budget < 0 ? n : std::min(n, copy_budget);
  if (n > 0 && (!dev_ids || !host_ids)) return fail(PS_EINVAL, "%s: NULL id list", fn);
  // the whole list is validated, also the part the budget leaves for a later step
  const int M = c->cfg.n_device_blocks, Mh = c->cfg.n_host_blocks;
  for (int pass = 0; pass < 2; ++pass) {
    const int32_t* ids = pass == 0 ? dev_ids : host_ids;
    const int lim = pass == 0 ? M : Mh;
    c->seen.assign((size_t)lim, 0);
    for (int k = 0; k < n; ++k) {
      if ((uint32_t)ids[k] >= (uint32_t)lim)
        return fail(PS_EINVAL, "%s: %s id %d at %d outside [0, %d)", fn, pass == 0 ? "device block" : "host slot",
                    ids[k], k, lim);
      if (c->seen[(size_t)ids[k]]++) return fail(PS_EINVAL, "%s: duplicate %s id %d", fn, pass == 0 ? "device block" : "host slot", ids[k]);
    }
  }
  if (m == 0) return PS_OK;
  if (!kv_cache || !host_pool) return fail(PS_EINVAL, "%s: NULL pool pointer", fn);
  if ((((uintptr_t)kv_cache | (uintptr_t)host_pool) & 15) != 0) return fail(PS_EINVAL, "%s: pools must be 16-byte aligned", fn);
  if (m > kMaxSwap) return fail(PS_EINVAL, "%s: at most %d blocks per call (got %d)", fn, kMaxSwap, m);
  hipStream_t stream = (hipStream_t)side_stream;

  const int si = c->swap_next;
  (void)si;
  c->swap_next = (c->swap_next + 1) % kSwapSlots;
  StageSlot& slot = c->swap_slot[si];
  int rc = acquire_slot(slot, (size_t)3 * kMaxSwap * sizeof(int32_t));
  if (rc != PS_OK) return rc;
  int32_t* h = (int32_t*)slot.pinned;
  std::memcpy(h, dev_ids, (size_t)m * 4);
  std::memcpy(h + m, host_ids, (size_t)m * 4);
  // The kernel reads the ids straight from the pinned staging slot (one small read over the host
  // link in its prologue).  A separate host-to-device copy of the ids in front of every kernel put
  // a link round trip, queued behind the bulk traffic, between consecutive copy kernels.
  int32_t* d = h;
  // Runs of consecutive host slots in list order: few runs => the copy engines move the bytes, one DMA per run,
  // between the host pool and a device staging buffer that a kernel packs from / unpacks into the listed blocks.
  int runs = 1;
  for (int k = 1; k < m; ++k) runs += host_ids[k] != host_ids[k - 1] + 1;
  ps_ctx::Staging& st = c->staging[out_dir ? 0 : 1];
  if (st.dev && runs <= c->cfg.swap_dma_runs && m <= st.blocks) {
    if (st.used && st.last_stream != stream) PS_HIP(hipStreamWaitEvent(stream, st.done, 0));  // the buffer's last user
    for (int k = 0; k < m; ++k) h[2 * m + k] = k;  // positions in the staging buffer
    const size_t bb = c->block_bytes;
    char* hp = (char*)const_cast<void*>(host_pool);
    if (out_dir) {
      PS_HIP(ps::launch_block_copy(d, d + 2 * m, m, kv_cache, st.dev, bb, 64, stream));
      for (int k0 = 0; k0 < m;) {
        int k1 = k0 + 1;
        while (k1 < m && host_ids[k1] == host_ids[k1 - 1] + 1) ++k1;
        PS_HIP(hipMemcpyAsync(hp + (size_t)host_ids[k0] * bb, st.dev + (size_t)k0 * bb, (size_t)(k1 - k0) * bb,
                              hipMemcpyDeviceToHost, stream));
        k0 = k1;
      }
    } else {
      for (int k0 = 0; k0 < m;) {
        int k1 = k0 + 1;
        while (k1 < m && host_ids[k1] == host_ids[k1 - 1] + 1) ++k1;
        PS_HIP(hipMemcpyAsync(st.dev + (size_t)k0 * bb, hp + (size_t)host_ids[k0] * bb, (size_t)(k1 - k0) * bb,
                              hipMemcpyHostToDevice, stream));
        k0 = k1;
      }
      PS_HIP(ps::launch_block_copy(d + 2 * m, d, m, st.dev, const_cast<void*>(kv_cache), bb, 64, stream));
    }
    PS_HIP(hipEventRecord(st.done, stream));
    st.last_stream = stream;
    st.used = true;
  } else {
    // measured next to a running attention step: 8 workgroups move more than 32 or 128 do
    const int wgs = c->cfg.swap_workgroups > 0 ? c->cfg.swap_workgroups : 8;
    if (out_dir)
      PS_HIP(ps::launch_block_copy(d, d + m, m, kv_cache, const_cast<void*>(host_pool), c->block_bytes, wgs, stream));
    else
      PS_HIP(ps::launch_block_copy(d + m, d, m, host_pool, const_cast<void*>(kv_cache), c->block_bytes, wgs, stream));
  }
  PS_HIP(hipEventRecord(slot.ev, stream));
  slot.in_flight = true;

  const uint64_t id = c->next_ticket++;
  const int ts = (int)(id % kTicketRing);
  if (c->ticket_id[ts] != 0) PS_HIP(hipEventSynchronize(c->ticket_ev[ts]));  // recycled: older copy must be over
  PS_HIP(hipEventRecord(c->ticket_ev[ts], stream));
  c->ticket_id[ts] = id;
  *n_done = m;
  *ticket = id;
  return PS_OK;
}

int ps_swap_out(ps_ctx* c, const int32_t* dev_block_ids, const int32_t* host_slot_ids, int32_t n, int32_t copy_budget,
                const void* kv_cache, void* host_pool, void* side_stream, int32_t* n_done, uint64_t* ticket) {
  return swap_common(c, true, dev_block_ids, host_slot_ids, n, copy_budget, kv_cache, host_pool, side_stream, n_done,
                     ticket);
}

int ps_swap_in(ps_ctx* c, const int32_t* host_slot_ids, const int32_t* dev_block_ids, int32_t n, int32_t copy_budget,
               const void* host_pool, void* kv_cache, void* side_stream, int32_t* n_done, uint64_t* ticket) {
  return swap_common(c, false, dev_block_ids, host_slot_ids, n, copy_budget, kv_cache, host_pool, side_stream, n_done,
                     ticket);
}

int ps_ticket_query(ps_ctx* c, uint64_t ticket) {
  if (!c) return fail(PS_EINVAL, "NULL ctx");
  hipEvent_t ev = nullptr;
  bool done = false;
  int rc = find_ticket(c, ticket, &ev, &done);
  if (rc != PS_OK) return rc;
  if (done) return PS_OK;
  hipError_t e = hipEventQuery(ev);
  if (e == hipSuccess) return PS_OK;
  if (e == hipErrorNotReady) return PS_EBUSY;
  return fail(PS_EHIP, "hipEventQuery: %s", hipGetErrorString(e));
}

int ps_ticket_wait(ps_ctx* c, uint64_t ticket) {
  if (!c) return fail(PS_EINVAL, "NULL ctx");
  hipEvent_t ev = nullptr;
  bool done = false;
  int rc = find_ticket(c, ticket, &ev, &done);
  if (rc != PS_OK) return rc;
  if (done) return PS_OK;
  PS_HIP(hipEventSynchronize(ev));
  return PS_OK;
}

}  // extern "C"
