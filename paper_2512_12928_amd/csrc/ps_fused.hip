// gfx950 kernel for a mixed batch in which every workgroup carries both kinds of work: a prefill
// workgroup's tile walk on eight waves that do nothing but matrix and softmax arithmetic, and four
// memory waves: two that fetch the walk's K/V tiles into LDS and two that walk decode slots.
//
// Why the split.  When prefill waves share a compute unit with decode waves and issue their own tile
// loads, every load instruction they issue stands in the unit's in-order vector memory path behind the
// decode waves' HBM misses, and it is the issuing wave that waits: two loads per tile cost a prefill wave
// 250 cycles alone and 650 to 1000 next to decode waves, during which its MFMAs stand still.  Here only
// the memory waves ever issue a load; what they wait for delays nothing but themselves, and the ring of
// tiles between them and the MFMA waves rides it out.
//
// Workgroup = 12 waves, three per SIMD (168 registers each), one workgroup per compute unit (LDS).
//   waves 0..7   MFMA waves: the prefill role on 32-token KV tiles (v_mfma_f32_32x32x16_bf16), operands
//                from an LDS ring of eight tiles that is handed over in pairs of tiles (64 tokens): a wave
//                waits for the pair's `ready` flag ahead of its first tile and counts itself into the
//                pair's `consumed` counter once its last read of the second tile has been issued.
//   waves 8, 9   feeders: wave 8 + f fetches the pairs p = f (mod 2) of the walk in order, up to three tiles in
//                flight (16 global->LDS loads each: every load one contiguous KiB of a block's K or V slice,
//                addressed by a scalar base and a per-lane offset that never changes), a pair's first tile
//                once all eight MFMA waves have consumed the previous pair in those slots; when a tile's loads
//                are back it zeroes V slots past the end of the request, and behind a pair's last tile it sets
//                `ready`.
//   waves 10, 11 decode waves: wave 10 + k walks decode slot (bid / Hkv) * 2 + k of the launch for the
//                workgroup's kv-head, one 32-token tile at a time (16x16x32 MFMA, the G query heads of the
//                kv-head in 16 columns, no LDS), and ends when the slot does.
// Nobody waits at a barrier after the start: MFMA waves wait only for `ready`, feeders only for memory
// and for `consumed`, decode waves only for memory; pair p's `ready` needs `consumed` of pair p - 4 only,
// which needs `ready` of p - 4: every wait is for something earlier in that order, so the walk drains.
// What it buys (MI355X), against the two kinds of work on disjoint compute units: 2 to 14 % off a launch in
// which neither kind dwarfs the other (the prefill work 0.65 to 8 times the decode work); outside that
// range the two layouts take the same time or this one more.  It stops there because every load on a
// unit, hit or miss, returns at the pace of the misses in front of it, and because a load issued next to
// MFMA waves costs its wave some 90 cycles (160 with a 64-bit address per lane).
#include <type_traits>

#include "ps_device.h"

namespace ps {

constexpr int kFusedMfmaWaves = 8;
constexpr int kFusedMemWaves = 4;     // kFusedFeeders feeders and kFusedDecodeWaves decode waves
constexpr int kFusedFeeders = 2;
constexpr int kFusedDecodeWaves = kFusedMemWaves - kFusedFeeders;
constexpr int kFusedThreads = (kFusedMfmaWaves + kFusedMemWaves) * 64;
constexpr int kFusedRows = 32;      // query tokens per MFMA wave
constexpr int kFusedKV = 32;        // KV tokens per ring tile
constexpr int kFusedRing = 8;       // tiles in the LDS ring
constexpr int kFusedPairs = kFusedRing / 2;  // handed over in pairs: tiles 2p and 2p + 1 in ring slots (2p) % 8 and (2p + 1) % 8
constexpr int kHostTileKV = 64;     // unit of PrefillTile::tile_begin / tile_end

struct FusedStage {
  uint4 k[2][256]; // block u of the tile as it lies in the cache: [dim/8][token][8 dims], 16 bytes per (dim group, token)
  uint4 v[8][64];  // fragment 4u+n: dims 32n..32n+31 of block u, in MFMA A-operand lane order
};
struct FusedLds {
  FusedStage ring[kFusedRing];
  uint32_t ready[kFusedRing];     // ready[p % 4] = 1 + index of the last pair that landed in pair slot p % 4 (entries 4.. unused)
  uint32_t consumed[kFusedRing];  // MFMA waves that are through with pair slot p % 4, counted over the whole walk
};
static_assert(sizeof(FusedLds) <= 160 * 1024, "one workgroup's LDS");

__device__ __forceinline__ uint32_t lds_peek(const uint32_t* f) {
  return __builtin_amdgcn_readfirstlane(*(const volatile uint32_t*)f);
}

// Every wait of this kernel is bounded: a wave that has waited this many sleeps for a flag stops waiting for
// flags altogether (its results are then wrong, and the count below says so), so that whatever goes wrong in
// the hand-over the launch still drains.  By the ordering argument at the top of this file no wait ever gets
// near the bound.
constexpr int kFusedSpinLimit = 1 << 18;
__device__ unsigned int g_fused_gave_up;

// Two block-table entries through the scalar cache.
__device__ __forceinline__ void load_ids2(const int* p0, const int* p1, int (&id)[2]) {
  asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %3, 0x0\n\ts_waitcnt lgkmcnt(0)"
               : "=&s"(id[0]), "=&s"(id[1])
               : "s"(p0), "s"(p1));
}

__global__ __launch_bounds__(kFusedThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void fused_kernel(
    StepParams P, const DecodeItem* __restrict__ ditems, const int32_t* __restrict__ dslots,
    const int32_t* __restrict__ block_ids, int n_slots, int HW, int n_zsplit) {
  __shared__ __attribute__((aligned(16))) FusedLds sm;
  const int bid = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = lane & 31;   // row of the K operand / query column of Q, P, O
  const int h2 = lane >> 5;  // k-group
  const int Hkv = P.Hkv, G = P.G;
  const int g = bid % Hkv;
  const int z = (bid / Hkv) % n_zsplit;
  const PrefillTile t = P.ptiles[bid / (Hkv * n_zsplit)];
  const int r = t.req;
  const int qs = P.q_start[r];
  const int lq = P.q_start[r + 1] - qs;
  const int L = P.kv_len[r];
  const int p = L - lq;
  const int* table = block_ids + P.bt_start[r];
  const int nblk = (L + kBlockTokens - 1) >> 4;
  const int SUB = kFusedMfmaWaves / HW;
  const int wg_last = (t.q0 + SUB * kFusedRows < lq ? t.q0 + SUB * kFusedRows : lq) - 1;
  const int reach = (p + wg_last) / kFusedKV + 1;  // ring tiles any query of the workgroup can see
  const int tile0 = t.tile_begin * (kHostTileKV / kFusedKV);  // this partition: tiles [tile0, tile1)
  const int tile1 = t.tile_end * (kHostTileKV / kFusedKV) < reach ? t.tile_end * (kHostTileKV / kFusedKV) : reach;
  const int ntiles = tile1 - tile0;  // workgroup-uniform; the host never makes it < 1

  if (bid < kClockSlots) {
    clock_record(P, kClockSlots + bid, 0);
    if (P.clocks != nullptr && threadIdx.x == (kFusedMfmaWaves + kFusedFeeders) * 64) {
      P.clocks[bid * 4 + 0] = __builtin_amdgcn_s_memtime();
      P.clocks[bid * 4 + 1] = __builtin_amdgcn_s_memrealtime();
    }
  }
  if (threadIdx.x < kFusedRing) {
    sm.ready[threadIdx.x] = 0;
    sm.consumed[threadIdx.x] = 0;
  }
  __syncthreads();  // the only workgroup barrier

  if (wave < kFusedMfmaWaves) {
    // ------------------------------------------------------------------------------- MFMA waves
    const int head = g * G + z * HW + wave % HW;
    const int q0 = t.q0 + (wave / HW) * kFusedRows;  // this wave's first query token
    const bool active = q0 < lq;
    // Q^T operand: lane (query j, k-group h2) holds dims (c*2+h2)*8 .. +7 for chunk c.
    bf16x8 qop[8];
    {
      int row = q0 + j;
      row = row < lq ? row : lq - 1;
      const uint16_t* qrow = P.q + ((size_t)(qs + row) * P.Hq + head) * kHeadDim;
#pragma unroll
      for (int c = 0; c < 8; ++c) qop[c] = as_bf16x8(*(const uint4*)(qrow + (c * 2 + h2) * 8));
    }
    float m = PS_NEG_INF, l = 0.f;
    float m_use = 0.f;  // what the exponentials subtract: m, or 0 while m = -inf; renewed where m is
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;
    const int my_last = p + (q0 + kFusedRows < lq ? q0 + kFusedRows : lq) - 1;  // last visible key
    const int qpos = p + q0 + j;
    // K row j of a score tile is token pi(j) of the ring tile: block j>>4, slot 8*bit2(j) + 4*bit3(j) + (j&3)
    const int kslot = 8 * ((j >> 2) & 1) + 4 * ((j >> 3) & 1) + (j & 3);
    // byte offsets of this lane's first K fragment and of its V fragments inside a ring slot (the chunks follow at 512 B,
    // the V fragments at 1 KiB): one addition per tile instead of the index arithmetic
    uint32_t k_lane = (uint32_t)((j >> 4) * sizeof(uint4) * 256 + (h2 * 16 + kslot) * sizeof(uint4));
    uint32_t v_lane = (uint32_t)(sizeof(uint4) * 512 + lane * sizeof(uint4));
    asm("" : "+v"(k_lane), "+v"(v_lane));  // kept in a register each: left alone, the compiler rebuilds them from j and h2 every tile
    static_assert(offsetof(FusedStage, v) == sizeof(uint4) * 512 && sizeof(FusedStage::k[0]) == sizeof(uint4) * 256, "ring slot layout");

    bool gave_up = false;
    bool track = true;  // wave-uniform: the next tile's maximum is taken (see PS_RESCALE_SLACK)
    // The walk is handed over in pairs of tiles (64 tokens): one wait for the pair's flag ahead of its first tile, one
    // count behind the wave's last read of its second (or only) tile.
    for (int it = 0; it < ntiles; ++it) {
      const int slot = it & (kFusedRing - 1);
      const int pslot = (it >> 1) & (kFusedPairs - 1);
      const int ts = (tile0 + it) * kFusedKV;
      const bool last_of_pair = (it & 1) || it + 1 == ntiles;
      if (!(it & 1) && !gave_up) {
        int spins = 0;
        while (lds_peek(&sm.ready[pslot]) < (uint32_t)((it >> 1) + 1)) {
          __builtin_amdgcn_s_sleep(1);
          if (++spins > kFusedSpinLimit) {
            gave_up = true;
            if (lane == 0) atomicAdd(&g_fused_gave_up, 1u);
            break;
          }
        }
        // The eight waves drift apart, and a pair's slots come free only when the last of them is through: a wave that
        // finds its pair waiting is behind the others and goes first on its SIMD (wave priority 2) until it has to wait
        // for a pair itself (priority 0, that of the memory waves).  2.5 % off the launch.
        if (spins == 0)
          __builtin_amdgcn_s_setprio(2);
        else
          __builtin_amdgcn_s_setprio(0);
      }
      asm volatile("" ::: "memory");  // no read of the pair moves above the flag
      if (active && ts <= my_last) {
        const FusedStage& S = sm.ring[slot];
        // all 8 K fragments are requested from LDS before the first MFMA needs one, the first 4 V fragments
        // right behind the score MFMAs and the other 4 behind the softmax arithmetic, so that LDS latency is
        // paid once per tile and no more than 8 fragments are held at a time
        // K operand of dim chunk c: row j is token pi(j) of the tile (block j>>4, slot kslot), this lane's 8 dims are dim
        // group 2c + h2; the 16 lanes of a quarter wave read 16 consecutive slots of one group: no bank conflict
        bf16x8 kf[8], vf[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) kf[c] = as_bf16x8(*(const uint4*)((const char*)&S + k_lane + c * 512));
        __builtin_amdgcn_sched_barrier(0);
        f32x16 s;
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c], qop[c], s, 0, 0, 0);
#pragma unroll
        for (int f = 0; f < 4; ++f) vf[f] = as_bf16x8(*(const uint4*)((const char*)&S + v_lane + f * 1024));
        __builtin_amdgcn_sched_barrier(0);
        // s[e]: token ts + 16*(e/8) + 8*h2 + e%8, query q0 + j (raw dot products)
        if (ts + kFusedKV - 1 > p + q0) {  // diagonal tile (wave-uniform test)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int tok = ts + 16 * (e >> 3) + 8 * h2 + (e & 7);
            if (tok > qpos) s[e] = PS_NEG_INF;
          }
        }
        const bool tracked = track;
        if (tracked) {
          float tmax = max16<true>(s);  // starts with the wait states an MFMA result needs
          tmax = xor32_max(tmax) * P.scale_log2;
          if (__builtin_amdgcn_ballot_w64(tmax > m + PS_RESCALE_SLACK) != 0) {  // some row outgrew its reference
            const float m_new = fmaxf(m, tmax);
            const float alpha = m_new == PS_NEG_INF ? 1.f : __builtin_amdgcn_exp2f(m - m_new);
            l *= alpha;
            m = m_new;
#pragma unroll
            for (int n = 0; n < 4; ++n) acc[n] *= alpha;
          }
          track = __builtin_amdgcn_ballot_w64(m == PS_NEG_INF) != 0;  // rows that have seen nothing yet have no reference
          m_use = m == PS_NEG_INF ? 0.f : m;  // all scores of such a row are -inf: exp2 gives 0
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], P.scale_log2, -m_use));
        uint4 pv[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
          pv[u] = make_uint4(pack_bf16x2(s[8 * u + 0], s[8 * u + 1]), pack_bf16x2(s[8 * u + 2], s[8 * u + 3]),
                             pack_bf16x2(s[8 * u + 4], s[8 * u + 5]), pack_bf16x2(s[8 * u + 6], s[8 * u + 7]));
        const float psum = sum_bf16x16(pv[0], pv[1]);  // of the rounded probabilities: what the output MFMAs multiply by
        // Without the maximum nothing bounds the probabilities but the row sum itself: one beyond 2^40 (or infinite)
        // says that a row's scores have left the range its reference covers, and the tile is done once more, this time
        // with its maximum taken.  Nothing of the tile has gone into l or the accumulators yet, and the pair's count
        // has not been touched; at the pair's first tile the flag is looked at again, which costs a read.
        if (!tracked && __builtin_amdgcn_ballot_w64(!(psum <= PS_ROWSUM_LIMIT)) != 0) {
          track = true;
          --it;
          continue;
        }
        l += psum;
        bf16x8 pop[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) pop[u] = as_bf16x8(pv[u]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 4; f < 8; ++f) vf[f] = as_bf16x8(*(const uint4*)((const char*)&S + v_lane + f * 1024));
        // the wave's last read of the tile is issued: LDS serves a wave's instructions in order, so the count
        // may follow at once
        asm volatile("" ::: "memory");
        if (last_of_pair && lane == 0)
          __hip_atomic_fetch_add(&sm.consumed[pslot], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u * 4 + n], pop[u], acc[n], 0, 0, 0);
      } else if (last_of_pair) {
        asm volatile("" ::: "memory");
        if (lane == 0) __hip_atomic_fetch_add(&sm.consumed[pslot], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
    if (bid < kClockSlots) clock_record(P, kClockSlots + bid, 2);

    if (!active) return;
    const float ls = l + __shfl_xor(l, 32);
    const int row = q0 + j;
    if (row >= lq) return;
    if (t.part < 0) {
      const float inv = 1.f / ls;
      const size_t ob = ((size_t)(qs + row) * P.Hq + head) * kHeadDim;
#pragma unroll
      for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const int x = n * 32 + a * 8 + h2 * 4;  // acc[n][4a+b] is dim x + b
          const float o0 = acc[n][4 * a + 0] * inv, o1 = acc[n][4 * a + 1] * inv;
          const float o2 = acc[n][4 * a + 2] * inv, o3 = acc[n][4 * a + 3] * inv;
          if (P.out_f32) {
            *(f32x4*)((float*)P.out + ob + x) = (f32x4){o0, o1, o2, o3};
          } else {
            uint2 w = {pack_bf16x2(o0, o1), pack_bf16x2(o2, o3)};
            *(uint2*)((uint16_t*)P.out + ob + x) = w;
          }
        }
    } else {  // one of several KV partitions of this row: unnormalised partial for the merge kernel
      const int pslot = t.part + (row - t.q0) * t.n_parts + t.k;
      float* dst = P.partials + ((size_t)pslot * P.Hq + head) * kPartStride;
#pragma unroll
      for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int a = 0; a < 4; ++a)
          *(f32x4*)(dst + n * 32 + a * 8 + h2 * 4) =
              (f32x4){acc[n][4 * a], acc[n][4 * a + 1], acc[n][4 * a + 2], acc[n][4 * a + 3]};
      if (h2 == 0) {
        dst[128] = m;
        dst[129] = ls;
      }
    }
    return;
  }

  // ---------------------------------------------------------------------------------- memory waves
  const int mw = wave - kFusedMfmaWaves;
  if (mw < kFusedFeeders) {
    // ---- a feeder: fetches the pairs of tiles p = mw (mod kFusedFeeders) of the walk in order, up to three tiles in
    // flight, as their ring slots come free
    const uint32_t ring_base = (uint32_t)(uintptr_t)(&sm.ring[0]);  // LDS byte address of the ring
    const uint32_t k_voff = (uint32_t)lane * 16u;                       // K slice: straight copy
    const uint32_t v_voff = (uint32_t)(j * kBlockTokens + 8 * h2) * 2u;  // V slice: dim row j of a 32-dim group, tokens 8*h2..
    // The previous occupants of pair pr's two ring slots have been read by all eight MFMA waves.
    auto pair_free = [&](int pr) {
      return pr < kFusedPairs || lds_peek(&sm.consumed[pr & (kFusedPairs - 1)]) >= (uint32_t)(kFusedMfmaWaves * (pr >> 2));
    };
    // The 16 loads of tile ti: K fragments 0..7 (dim chunks), V fragments 0..7 (block f/4, dims 32*(f%4)..).
    auto issue_tile = [&](int ti) {
      // the tile's two block ids come through the scalar cache (an absent second block repeats the first and is
      // fully masked): a feeder keeps away from the LDS, which the MFMA waves' operand reads keep busy
      const int b0 = (tile0 + ti) * (kFusedKV / kBlockTokens);
      const int last = nblk - 1;
      int id[2];
      load_ids2(table + (b0 < last ? b0 : last), table + (b0 + 1 < last ? b0 + 1 : last), id);
      const int idA = id[0], idB = id[1];
      const uint32_t st = ring_base + (uint32_t)(ti & (kFusedRing - 1)) * (uint32_t)sizeof(FusedStage);
      // Every load is one contiguous KiB of one block's K or V slice: a wave-uniform base (scalar arithmetic only), a
      // per-lane offset that never changes, and an instruction offset that counts on the LDS side as well.
      const uint16_t* kA = k_slice(P.cache, idA, Hkv, g);
      const uint16_t* kB = k_slice(P.cache, idB, Hkv, g);
      const uint16_t* vA = v_slice(P.cache, idA, Hkv, g);
      const uint16_t* vB = v_slice(P.cache, idB, Hkv, g);
      load_to_lds16_sbase<0>(kA, k_voff, st);
      load_to_lds16_sbase<1024>(kA, k_voff, st);
      load_to_lds16_sbase<2048>(kA, k_voff, st);
      load_to_lds16_sbase<3072>(kA, k_voff, st);
      load_to_lds16_sbase<0>(kB, k_voff, st + 4096u);
      load_to_lds16_sbase<1024>(kB, k_voff, st + 4096u);
      load_to_lds16_sbase<2048>(kB, k_voff, st + 4096u);
      load_to_lds16_sbase<3072>(kB, k_voff, st + 4096u);
      load_to_lds16_sbase<0>(vA, v_voff, st + 8192u);
      load_to_lds16_sbase<1024>(vA, v_voff, st + 8192u);
      load_to_lds16_sbase<2048>(vA, v_voff, st + 8192u);
      load_to_lds16_sbase<3072>(vA, v_voff, st + 8192u);
      load_to_lds16_sbase<0>(vB, v_voff, st + 12288u);
      load_to_lds16_sbase<1024>(vB, v_voff, st + 12288u);
      load_to_lds16_sbase<2048>(vB, v_voff, st + 12288u);
      load_to_lds16_sbase<3072>(vB, v_voff, st + 12288u);
    };
    // Pair pr has landed (the caller has waited for its loads): zero what must not be read and hand it to the MFMA waves.
    auto publish = [&](int pr) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int ti = 2 * pr + h;
        const int ts = (tile0 + ti) * kFusedKV;
        if (ti < ntiles && ts + kFusedKV > L) {
          // Last tile of the request: slots past kv_len may hold anything, and 0 * NaN is NaN: zero them in V.
          const int slot = ti & (kFusedRing - 1);
#pragma unroll
          for (int f = 0; f < 8; ++f) {
            const int first = ts + 16 * (f >> 2) + 8 * h2;
            const uint4 vv = sm.ring[slot].v[f][lane];
            const uint2 lo = zero_from(make_uint2(vv.x, vv.y), first, L);
            const uint2 hi = zero_from(make_uint2(vv.z, vv.w), first + 4, L);
            sm.ring[slot].v[f][lane] = make_uint4(lo.x, lo.y, hi.x, hi.y);
          }
        }
      }
      asm volatile("" ::: "memory");  // the flag is written after the tiles, in program order (LDS keeps it)
      if (lane == 0) *(volatile uint32_t*)&sm.ready[pr & (kFusedPairs - 1)] = (uint32_t)(pr + 1);
    };
    // One pass per pair, and one look at the LDS per pass: wait until the pair's slots are free, issue its first tile,
    // hand over the pair before (loads return in issue order: with at most the 16 loads just issued still out, it has
    // landed), issue the second tile.  At most three tiles are in flight (the load counter holds 63).
    int prev = -1;  // the pair in flight
    for (int pr = mw; 2 * pr < ntiles; pr += kFusedFeeders) {
      int spins = 0;
      while (!pair_free(pr)) {
        if (prev >= 0) {  // do not sit on a pair that has landed meanwhile
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          publish(prev);
          prev = -1;
          continue;
        }
        __builtin_amdgcn_s_sleep(1);
        if (++spins > kFusedSpinLimit) {  // nothing of this wave is in flight here: prev was handed over above
          if (lane == 0) atomicAdd(&g_fused_gave_up, 1u);
          return;
        }
      }
      issue_tile(2 * pr);
      if (prev >= 0) {
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        publish(prev);
      }
      if (2 * pr + 1 < ntiles) issue_tile(2 * pr + 1);
      prev = pr;
    }
    if (prev >= 0) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      publish(prev);
    }
    return;
  }

  // ---- decode waves: slot (bid / Hkv) * kFusedDecodeWaves + mw - kFusedFeeders of the launch, for this workgroup's kv-head
  const int dslot = (bid / Hkv) * kFusedDecodeWaves + mw - kFusedFeeders;
  if (dslot >= n_slots) return;
  {
    const int i = lane & 15;   // row of the K operand / dim row of the V operand / query-head column of Q, P, O
    const int kg = lane >> 4;  // k-group of the MFMA operands
    // per-lane element offsets inside a (block, head) slice
    const int k_off = kg * (kBlockTokens * 8) + (8 * ((i >> 2) & 1) + (i & 3)) * 8;  // T0; T1: + 4 slots; chunk c: + 4c groups
    const bool k_in_b = i >= 8;
    const int v_off = i * kBlockTokens + 8 * (kg & 1);  // + 16n dims
    const bool v_in_b = kg >= 2;
    const int qhead = g * G + (i < G ? i : 0);  // columns G..15 repeat head g*G: computed, never written
    // No branches around loads anywhere below: at a branch the compiler waits for every load in flight.
    // Q^T operand: lane (head i, k-group kg) holds dims 32c + 8kg .. +7 for chunk c.
    auto fetch_q = [&](int tok, bf16x8 (&v)[4]) {
      const uint16_t* qrow = P.q + ((size_t)tok * P.Hq + qhead) * kHeadDim + kg * 8;
#pragma unroll
      for (int c = 0; c < 4; ++c) v[c] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + c * 32));
    };
    // block ids of the 32-token tile that starts at token ts (an absent second block repeats the first
    // and is masked by the token test)
    auto tile_ids = [&](const DecodeItem& d, int ts, int& a, int& b2) {
      const int32_t* tb = block_ids + d.bt_off;
      const int bA = ts >> 4;
      a = tb[bA];
      b2 = tb[bA + 1 < d.nblk ? bA + 1 : bA];
    };
    const int seg_end = dslots[dslot + 1];
    int seg = dslots[dslot];
    if (seg >= seg_end) return;  // a slot may be empty (its workgroup's share of the decode tiles rounded to nothing)
    DecodeItem it = ditems[seg];
    int nextA, nextB;
    tile_ids(it, it.t0, nextA, nextB);
    bf16x8 qop[4];
    fetch_q(it.tok, qop);
    for (; seg < seg_end; ++seg) {
      const DecodeItem itn = ditems[seg + 1 < seg_end ? seg + 1 : seg];  // the last one repeats itself
      float m = PS_NEG_INF, l = 0.f;
      f32x4 acc[8];
#pragma unroll
      for (int n = 0; n < 8; ++n) acc[n] = (f32x4){0.f, 0.f, 0.f, 0.f};
      bf16x8 qn[4];
      // One 32-token tile.  In the last tile of the segment (LAST) the next segment's Q is requested ahead of the
      // tile's own loads, and the ids fetched one tile ahead are those of the next segment's first tile.
      auto tile = [&](int ts, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        if (LAST) fetch_q(itn.tok, qn);
        const int idA = nextA, idB = nextB;
        if (LAST)
          tile_ids(itn, itn.t0, nextA, nextB);
        else
          tile_ids(it, ts + kTileTokens, nextA, nextB);
        const uint16_t* kp = k_slice(P.cache, k_in_b ? idB : idA, Hkv, g) + k_off;
        const uint16_t* vp = v_slice(P.cache, v_in_b ? idB : idA, Hkv, g) + v_off;
        bf16x8 kf[2][4], vf[8];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          kf[0][c] = load_stream16(kp + c * 4 * (kBlockTokens * 8));
          kf[1][c] = load_stream16(kp + c * 4 * (kBlockTokens * 8) + 4 * 8);
        }
#pragma unroll
        for (int n = 0; n < 8; ++n) vf[n] = load_stream16(vp + n * 16 * kBlockTokens);
        // all 16 loads are in flight before anything waits for the first
        __builtin_amdgcn_sched_barrier(0);
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][c], qop[c], s0, 0, 0, 0);
          s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][c], qop[c], s1, 0, 0, 0);
        }
        // s0[e]: token ts + 8kg + e, s1[e]: token ts + 8kg + 4 + e, head i
        float tmax = PS_NEG_INF;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int tok = ts + 8 * kg + e;
          s0[e] = (!LAST || tok < it.t1) ? s0[e] * P.scale_log2 : PS_NEG_INF;  // only the last tile is ragged
          s1[e] = (!LAST || tok + 4 < it.t1) ? s1[e] * P.scale_log2 : PS_NEG_INF;
          tmax = fmaxf(tmax, fmaxf(s0[e], s1[e]));
        }
        if (LAST) {  // slots past the segment's end may hold anything
#pragma unroll
          for (int n = 0; n < 8; ++n) vf[n] = zero_from8(vf[n], ts + 8 * kg, it.t1);
        }
        tmax = xor32_max(xor16_max(tmax));
        const float m_new = fmaxf(m, tmax);  // finite: every tile holds at least one valid token
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          s0[e] = __builtin_amdgcn_exp2f(s0[e] - m_new);
          s1[e] = __builtin_amdgcn_exp2f(s1[e] - m_new);
        }
        const uint4 pv = {pack_bf16x2(s0[0], s0[1]), pack_bf16x2(s0[2], s0[3]), pack_bf16x2(s1[0], s1[1]), pack_bf16x2(s1[2], s1[3])};
        l = l * alpha + sum_bf16x8(pv);  // of the rounded probabilities, the ones the output MFMAs multiply by
        m = m_new;
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[n] *= alpha;
        const bf16x8 pop = as_bf16x8(pv);
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[n], pop, acc[n], 0, 0, 0);
      };
      int ts = it.t0;
      for (; ts + kTileTokens < it.t1; ts += kTileTokens) tile(ts, std::false_type{});
      tile(ts, std::true_type{});
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      // acc[n][e] is dim 16n + 4kg + e of head i
      if (i < G) {
        const int head = g * G + i;
        if (it.part < 0) {
          const float inv = 1.f / l;
          const size_t ob = ((size_t)it.tok * P.Hq + head) * kHeadDim + 4 * kg;
#pragma unroll
          for (int n = 0; n < 8; ++n) {
            const f32x4 o = acc[n] * inv;
            if (P.out_f32) {
              *(f32x4*)((float*)P.out + ob + 16 * n) = o;
            } else {
              uint2 w = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
              *(uint2*)((uint16_t*)P.out + ob + 16 * n) = w;
            }
          }
        } else {  // unnormalised partial for the merge kernel
          float* dst = P.partials + ((size_t)it.part * P.Hq + head) * kPartStride;
#pragma unroll
          for (int n = 0; n < 8; ++n) *(f32x4*)(dst + 16 * n + 4 * kg) = acc[n];
          if (kg == 0) {
            dst[128] = m;
            dst[129] = l;
          }
        }
      }
      it = itn;
#pragma unroll
      for (int c = 0; c < 4; ++c) qop[c] = qn[c];
    }
  }
  if (bid < kClockSlots && P.clocks != nullptr && threadIdx.x == (kFusedMfmaWaves + kFusedFeeders) * 64) {
    P.clocks[bid * 4 + 2] = __builtin_amdgcn_s_memtime();
    P.clocks[bid * 4 + 3] = __builtin_amdgcn_s_memrealtime();
  }
}

// Waves that gave up a wait since the library was loaded (0 unless something is broken); host call, synchronises.
int fused_gave_up_count(unsigned int* out) {
  return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_fused_gave_up), sizeof(unsigned int)) == hipSuccess ? 0 : -1;
}


int fused_decode_slots(int n_tiles, int G) { return n_tiles * (G / prefill_heads_per_wg(G)) * kFusedDecodeWaves; }
bool fused_supports(int G) { return G <= 16; }

hipError_t launch_fused(const StepParams& p, int n_slots, int n_tiles, hipStream_t s, int* n_wgs_out) {
  const int HW = prefill_heads_per_wg(p.G);
  const int nz = p.G / HW;
  const long long grid = (long long)n_tiles * p.Hkv * nz;
  if (n_wgs_out) *n_wgs_out = (int)std::min<long long>(grid, 0x7fffffffLL);
  if (grid <= 0 || grid > 0x7fffffffLL || p.G > 16 || n_slots > fused_decode_slots(n_tiles, p.G)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fused_kernel, dim3((unsigned)grid), dim3(kFusedThreads), 0, s, p, p.ditems, p.dslots, p.block_ids, n_slots, HW, nz);
  return hipGetLastError();
}

}  // namespace ps
