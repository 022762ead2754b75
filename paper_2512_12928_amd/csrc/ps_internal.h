// Internal declarations shared by the host-side API code and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ps.h"

namespace ps {

constexpr int kHeadDim = 128;
constexpr int kBlockTokens = 16;
constexpr int kSliceElems = kBlockTokens * kHeadDim;  // one (block, K|V, kv-head) slice: 4 KiB
constexpr int kTileTokens = 32;                       // KV tokens per MFMA tile (two blocks)
constexpr int kPartStride = 132;                      // fp32 per split-K partial: o[128], m, l, pad
constexpr int kClockSlots = 2048;                     // workgroups per role whose clock counters a profiled step records

// One split-K partition (segment) of one decode token: KV tokens [t0, t1) of its request, for all
// G query heads of the kv-head that blockIdx.y selects.  A decode workgroup walks the segments
// dslots[x] .. dslots[x+1] of its slot x one after the other.
struct DecodeItem {
  int32_t bt_off;  // first block-table entry of the request
  int32_t tok;     // batch token index (row of q / out)
  int32_t t0;      // first cached token of the segment (multiple of 32)
  int32_t t1;      // one past the last cached token (kv_len for the final segment)
  int32_t part;    // slot in the partials buffer, or -1: the only segment, write out directly
  int32_t nblk;    // block-table entries of the request
  int32_t pad[2];
};

struct MergeItem {
  int32_t tok;
  int32_t part0;
  int32_t n_parts;
  int32_t pad;
};

// The new rows of one request that fall into one of its blocks (all fields resolved on the host, so
// that the kernel's loads depend on nothing but the item).
struct AppendItem {
  int32_t block;  // physical block
  int32_t row0;   // batch token index (row of k_new / v_new) of the first new row of the block
  int32_t slot0;  // its slot in the block
  int32_t n;      // number of new rows, 1..16
};

// One tile of consecutive query tokens of a prefill chunk, over one range of its KV tiles.
struct PrefillTile {
  int32_t req;
  int32_t q0;          // chunk-relative index of the tile's first query token
  int32_t tile_begin;  // first 64-token KV tile of this partition
  int32_t tile_end;    // one past its last KV tile (the kernel also stops at the causal reach)
  int32_t part;        // -1: the only partition, write the output; else first partials slot of the tile
  int32_t n_parts;     // partitions of this query tile
  int32_t k;           // index of this partition: token t of the tile uses slot part + t*n_parts + k
  int32_t pad;
};

struct StepParams {
  // batch description (device copies)
  const int32_t* q_start;
  const int32_t* kv_len;
  const int32_t* bt_start;
  const int32_t* block_ids;
  const DecodeItem* ditems;
  const int32_t* dslots;  // n_slots + 1 offsets into ditems
  const MergeItem* mitems;
  const PrefillTile* ptiles;
  float* partials;
  unsigned long long* clocks;  // profiling: 2 * kClockSlots records of 4 counters (see clock_record), else NULL
  // tensors
  const uint16_t* q;
  const uint16_t* k_new;
  const uint16_t* v_new;
  uint16_t* cache;
  void* out;
  int32_t Hq, Hkv, G;
  int32_t out_f32;
  float scale_log2;  // softmax_scale * log2(e)
};

// Launchers (ps_kernels.hip). Each checks its own launch and returns the hipError_t.
// Uploads the batch description, dst (device) <- src_pinned (pinned host memory, read over the host
// link by the kernel; bytes a multiple of 16), and in the same launch appends the step's new K/V
// rows (n_items append items, read from aitems_pinned, which lies in the same pinned block).
hipError_t launch_prologue(const StepParams& p, const void* src_pinned, void* dst, size_t bytes,
                           const AppendItem* aitems_pinned, int n_items, hipStream_t s);
// merges items [first, first + n_merge) of the merge list
hipError_t launch_merge(const StepParams& p, int first, int n_merge, hipStream_t s);
// One launch for the decode slots and the prefill tiles of the batch (either may be 0).
// n_decode_wgs_out / n_prefill_wgs_out (may be NULL): the workgroups of each role in the launch.
hipError_t launch_attention(const StepParams& p, int n_slots, int n_tiles, hipStream_t s, int* n_decode_wgs_out,
                            int* n_prefill_wgs_out);
// The same batch with every workgroup carrying both kinds of work (ps_fused.hip): n_tiles prefill work items as
// above, whose workgroup bid also walks the decode slots (bid / Hkv) * 3 + 0..2 for kv-head bid % Hkv, so
// n_slots <= fused_decode_slots(n_tiles, G).  Needs fused_supports(G).
hipError_t launch_fused(const StepParams& p, int n_slots, int n_tiles, hipStream_t s, int* n_wgs_out);
int fused_decode_slots(int n_tiles, int G);
bool fused_supports(int G);
int fused_gave_up_count(unsigned int* out);
int decode_waves_per_wg();
// tile_tokens: query tokens per workgroup tile as returned by prefill_tile_tokens(G).
int prefill_tile_tokens(int G);
int prefill_heads_per_wg(int G);
hipError_t launch_block_copy(const int32_t* src_ids, const int32_t* dst_ids, int n, const void* src_pool,
                             void* dst_pool, size_t block_bytes, int workgroups, hipStream_t s);

}  // namespace ps
