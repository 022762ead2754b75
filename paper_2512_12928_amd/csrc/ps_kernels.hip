// gfx950 (CDNA4) kernels for one mixed-batch attention layer over a paged bf16 KV cache and for
// KV block copies.  Wave64; bf16 MFMA with fp32 accumulation.
//
// Operand plan shared by the decode and prefill kernels.  Scores are produced transposed,
//   S^T[token][qrow] = K[token][:] . Q[qrow][:]        (A = K tile, B = Q^T)
// so that in the MFMA result layout each lane owns ONE query row and several tokens.  The
// probabilities that lane computes are then, without any cross-lane movement, exactly the
// B operand of the second product
//   O^T[dim][qrow] += V^T[dim][token] . P^T[token][qrow]   (A = V^T tile, B = P^T)
// and the per-row rescale factors of the online softmax are per-lane scalars.  Inside a block K
// is stored [dim/8][token][8 dims] and V [dim][token], so every A-operand lane is one 16-byte
// load and the lanes of one load instruction cover runs of 256 bytes or more.
#include <type_traits>

#include "ps_device.h"

namespace ps {

// ------------------------------------------------------------------------------------ prologue
// One launch, 256 threads per workgroup, two kinds of workgroup:
//  - the first n_up copy the step's batch description to the device: dst <- src, n16 units of
//    16 bytes.  src is pinned host memory read over the host link; every lane has its loads in
//    flight before the first store.
//  - the rest write this step's new K/V rows into the paged cache, two (item, kv-head) pairs per
//    workgroup (128 threads each).  An item is the new rows of one request that fall into one
//    block; the items are read from the pinned copy (the device copy is being written by the
//    other workgroups of this launch).  K goes to [dim/8][token][8]: a thread moves 16-byte groups
//    (token, 8 dims).  V is dim-major inside a block: thread x owns dim x; when the chunk covers
//    the whole block it gathers its dim from the 16 rows and writes one full 32-byte run,
//    otherwise (a decode token, the ragged ends of a chunk) it writes 2-byte elements.  All loads
//    of a thread are issued before its first store.
__global__ __launch_bounds__(256) void prologue_kernel(StepParams P, const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                       int n16, int n_up, const AppendItem* __restrict__ aitems_pinned,
                                                       int n_pairs) {
  if ((int)blockIdx.x < n_up) {
    const int stride = n_up * 256;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n16; i += 4 * stride) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = src[i + u * stride < n16 ? i + u * stride : i];  // no branch around a load
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i + u * stride < n16) dst[i + u * stride] = v[u];
    }
    return;
  }
  const int pair = ((int)blockIdx.x - n_up) * 2 + (threadIdx.x >> 7);  // item * Hkv + kv-head
  if (pair >= n_pairs) return;
  const AppendItem it = aitems_pinned[pair / P.Hkv];
  const int g = pair % P.Hkv, x = threadIdx.x & 127;
  uint16_t* kd = const_cast<uint16_t*>(k_slice(P.cache, it.block, P.Hkv, g));
  uint16_t* vd = const_cast<uint16_t*>(v_slice(P.cache, it.block, P.Hkv, g));
  const size_t rstride = (size_t)P.Hkv * kHeadDim;
  const uint16_t* ks = P.k_new + ((size_t)it.row0 * P.Hkv + g) * kHeadDim;
  const uint16_t* vs = P.v_new + ((size_t)it.row0 * P.Hkv + g) * kHeadDim + x;
  // rows past the item's last are replaced by its last row: the loads are unconditional (a
  // branch around a load would make the compiler wait for every load before it)
  const int last = it.n - 1;
  u32x4 kv[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int tt = (x + 128 * h) >> 4, grp = x & 15;
    kv[h] = *(const u32x4*)(ks + (size_t)(tt < last ? tt : last) * rstride + grp * 8);
  }
  uint16_t vv[kBlockTokens];
#pragma unroll
  for (int tt = 0; tt < kBlockTokens; ++tt) vv[tt] = vs[(size_t)(tt < last ? tt : last) * rstride];
  asm volatile("" : "+v"(kv[0]), "+v"(kv[1]));  // keeps the K loads up here, out of the branches below
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int tt = (x + 128 * h) >> 4, grp = x & 15;
    if (tt < it.n) *(u32x4*)(kd + grp * (kBlockTokens * 8) + (it.slot0 + tt) * 8) = kv[h];
  }
  if (it.n == kBlockTokens) {
    uint4* dst2 = (uint4*)(vd + x * kBlockTokens);
    dst2[0] = make_uint4(vv[0] | ((uint32_t)vv[1] << 16), vv[2] | ((uint32_t)vv[3] << 16), vv[4] | ((uint32_t)vv[5] << 16),
                         vv[6] | ((uint32_t)vv[7] << 16));
    dst2[1] = make_uint4(vv[8] | ((uint32_t)vv[9] << 16), vv[10] | ((uint32_t)vv[11] << 16),
                         vv[12] | ((uint32_t)vv[13] << 16), vv[14] | ((uint32_t)vv[15] << 16));
  } else {
#pragma unroll
    for (int tt = 0; tt < kBlockTokens; ++tt)
      if (tt < it.n) vd[x * kBlockTokens + it.slot0 + tt] = vv[tt];
  }
}

// ------------------------------------------------------------------------------------ decode
// Split-K decode attention, HBM-bound.  grid (ceil(n_slots / 4), Hkv), 256 threads: four waves
// that work independently (one slot each; a workgroup only pins them to the four SIMDs of one
// CU), no barriers, no cross-wave combine.  A wave walks the segments of its slot one after the
// other; a segment is KV tokens [t0, t1) of one request, handled for one kv-head and all G query
// heads of that head (padded to the 32 columns of a 32x32x16 MFMA: the matrix pipe has ten times
// the throughput this kernel can feed it), so every K/V byte is read once.  The host cuts the
// batch's decode tokens into slots of equal length, as many as the chip runs at once, so that
// all waves end together: measured on the same access pattern, a launch whose workgroups all
// run at once reads 6.7 TB/s, one with a second, partly filled round 5.7.  Per 32-token tile
// the wave issues 16 non-temporal 16-byte loads per lane (8 KiB K + 8 KiB V; the cache is read
// once, nothing is worth keeping in L2), 8 MFMAs for S^T and 8 for O^T.  At the end of a
// segment the lanes write their accumulators straight out: the final output (the request's
// only segment) or an unnormalised partial for the merge kernel.  The next segment's
// description, first block ids and Q are requested before that, so a segment boundary costs
// about one tile step.
//
// Operand order (same as the prefill kernel): row i of the K operand is token pi(i) of the tile
// (bits 2 and 3 of i swapped; rows 0..15 block A, 16..31 block B).  One K load instruction then
// covers, per 8-dim group, all 16 slots of a block: runs of 256 bytes.  In the 32x32 result
// layout lane (head j, k-group h2) holds, for MFMA step u, the 8 consecutive tokens
// 16u + 8*h2 .. +7: its V operand is one 16-byte run of the dim-major V block.

// The work lists and the block tables come as separate restrict-qualified kernel parameters: only
// then does the compiler know that the kernel's own stores cannot change them, and fetches them
// through the scalar cache instead of with vector loads it waits for on the spot.
typedef uint4 DecodeQ[2][8][64];  // one wave's two copies of its Q^T operand in LDS (16 KiB)

// wg: index of the decode workgroup in the launch; its kv-head is wg % Hkv and its waves 0 .. kDecodeWaves-1
// take the slots (wg / Hkv) * kDecodeWaves + wave (one wave per SIMD; further waves of the workgroup idle).
constexpr int kDecodeWaves = 4;
__device__ __forceinline__ void decode_role(const StepParams& P, const DecodeItem* __restrict__ ditems,
                                            const int32_t* __restrict__ dslots, const int32_t* __restrict__ block_ids,
                                            int n_slots, int wg, DecodeQ* q_all) {
  // Q^T operand: lane (head j, k-group h2) holds dims (c*2+h2)*8 .. +7 for chunk c.  Kept in LDS
  // rather than in 32 registers (every lane reads back exactly what it wrote: no barrier); two
  // copies, so that the next segment's Q can be stored while this one is still in use.
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int Hkv = P.Hkv, G = P.G;
  const int slot = (wg / Hkv) * kDecodeWaves + wave;  // the waves of a workgroup work independently
  if (wave >= kDecodeWaves || slot >= n_slots) return;
  uint4 (*q_lds)[8][64] = q_all[wave];
  const int j = lane & 31;   // row of the K operand / query-head column of Q, P, O
  const int h2 = lane >> 5;  // k-group of the MFMA operands
  const int g = wg % Hkv;

  // per-lane element offsets inside a (block, head) slice
  const int k_off = h2 * (kBlockTokens * 8) + (8 * ((j >> 2) & 1) + 4 * ((j >> 3) & 1) + (j & 3)) * 8;  // + c*2 groups
  const bool k_in_b = j >= 16;
  const int v_off = j * kBlockTokens + 8 * h2;  // + n*32 dims
  const int qhead = g * G + (j < G ? j : 0);
  const uint32_t qmask = j < G ? 0xFFFFFFFFu : 0u;  // columns G..31 of the MFMA tile are zero

  // No branches around loads anywhere below: at a branch the compiler waits for every load in flight.
  auto fetch_q = [&](int tok, u32x4 (&v)[8]) {
    const uint16_t* qrow = P.q + ((size_t)tok * P.Hq + qhead) * kHeadDim;
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = *(const u32x4*)(qrow + (c * 2 + h2) * 8);
  };
  auto store_q = [&](const u32x4 (&v)[8], int buf) {
#pragma unroll
    for (int c = 0; c < 8; ++c)
      q_lds[buf][c][lane] = make_uint4(v[c][0] & qmask, v[c][1] & qmask, v[c][2] & qmask, v[c][3] & qmask);
  };
  // block ids of the 32-token tile that starts at token ts (an absent second block repeats the
  // first and is masked by the token test)
  auto tile_ids = [&](const DecodeItem& d, int ts, int& a, int& b2) {
    const int32_t* table = block_ids + d.bt_off;
    const int bA = ts >> 4;
    a = table[bA];
    b2 = table[bA + 1 < d.nblk ? bA + 1 : bA];
  };

  const int seg_end = dslots[slot + 1];
  int seg = dslots[slot];
  DecodeItem it = ditems[seg];
  int nextA, nextB;
  tile_ids(it, it.t0, nextA, nextB);
  {
    u32x4 q0[8];
    fetch_q(it.tok, q0);
    store_q(q0, 0);
  }
  for (int buf = 0; seg < seg_end; ++seg, buf ^= 1) {
    const DecodeItem itn = ditems[seg + 1 < seg_end ? seg + 1 : seg];  // the last one repeats itself

    float m = PS_NEG_INF, l = 0.f;
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;

    // One 32-token tile.  In the last tile of the segment (LAST) the next segment's Q is requested
    // ahead of the tile's own loads and stored to LDS behind its arithmetic, and the ids fetched one
    // tile ahead are those of the next segment's first tile: a segment boundary costs no extra
    // memory round trip.
    auto tile = [&](int ts, auto last_tag) {
      constexpr bool LAST = decltype(last_tag)::value;
      u32x4 qn[8];
      if (LAST) fetch_q(itn.tok, qn);
      const int idA = nextA, idB = nextB;
      if (LAST)
        tile_ids(itn, itn.t0, nextA, nextB);
      else
        tile_ids(it, ts + kTileTokens, nextA, nextB);
      const uint16_t* kp = k_slice(P.cache, k_in_b ? idB : idA, Hkv, g) + k_off;
      const uint16_t* vA = v_slice(P.cache, idA, Hkv, g) + v_off;
      const uint16_t* vB = v_slice(P.cache, idB, Hkv, g) + v_off;

      bf16x8 kf[8], vf[2][4];
#pragma unroll
      for (int c = 0; c < 8; ++c) kf[c] = load_stream16(kp + c * 2 * (kBlockTokens * 8));
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        vf[0][n] = load_stream16(vA + n * 32 * kBlockTokens);
        vf[1][n] = load_stream16(vB + n * 32 * kBlockTokens);
      }
      // all 16 loads are in flight before anything waits for the first (left alone, the scheduler
      // holds the V loads back until the K registers are free again: two round trips per tile)
      __builtin_amdgcn_sched_barrier(0);

      f32x16 s;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c], as_bf16x8(q_lds[buf][c][lane]), s, 0, 0, 0);
      // s[e]: token ts + 16*(e/8) + 8*h2 + e%8, head j
      float tmax = PS_NEG_INF;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int tok = ts + 16 * (e >> 3) + 8 * h2 + (e & 7);
        s[e] = (!LAST || tok < it.t1) ? s[e] * P.scale_log2 : PS_NEG_INF;  // only the last tile is ragged
        tmax = fmaxf(tmax, s[e]);
      }
      if (LAST) {  // slots past the segment's end may hold anything
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int n = 0; n < 4; ++n) vf[u][n] = zero_from8(vf[u][n], ts + 16 * u + 8 * h2, it.t1);
      }
      tmax = xor32_max(tmax);
      const float m_new = fmaxf(m, tmax);  // finite: every tile holds at least one valid token
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = __builtin_amdgcn_exp2f(s[e] - m_new);
      uint4 pv[2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
        pv[u] = make_uint4(pack_bf16x2(s[8 * u + 0], s[8 * u + 1]), pack_bf16x2(s[8 * u + 2], s[8 * u + 3]),
                           pack_bf16x2(s[8 * u + 4], s[8 * u + 5]), pack_bf16x2(s[8 * u + 6], s[8 * u + 7]));
      l = l * alpha + sum_bf16x16(pv[0], pv[1]);  // of the rounded probabilities, the ones the output MFMAs multiply by
      m = m_new;
#pragma unroll
      for (int n = 0; n < 4; ++n) acc[n] *= alpha;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 pop = as_bf16x8(pv[u]);
#pragma unroll
        for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u][n], pop, acc[n], 0, 0, 0);
      }
      if (LAST) store_q(qn, buf ^ 1);
    };
    int ts = it.t0;
    for (; ts + kTileTokens < it.t1; ts += kTileTokens) tile(ts, std::false_type{});
    tile(ts, std::true_type{});
    l += __shfl_xor(l, 32);

    // acc[n][4a+b] is dim 32n + 8a + 4*h2 + b of head j
    if (j < G) {
      const int head = g * G + j;
      if (it.part < 0) {
        const float inv = 1.f / l;
        const size_t ob = ((size_t)it.tok * P.Hq + head) * kHeadDim;
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
          for (int a = 0; a < 4; ++a) {
            const int x = n * 32 + a * 8 + h2 * 4;
            const float o0 = acc[n][4 * a + 0] * inv, o1 = acc[n][4 * a + 1] * inv;
            const float o2 = acc[n][4 * a + 2] * inv, o3 = acc[n][4 * a + 3] * inv;
            if (P.out_f32) {
              *(f32x4*)((float*)P.out + ob + x) = (f32x4){o0, o1, o2, o3};
            } else {
              uint2 w = {pack_bf16x2(o0, o1), pack_bf16x2(o2, o3)};
              *(uint2*)((uint16_t*)P.out + ob + x) = w;
            }
          }
      } else {  // unnormalised partial for the merge kernel
        float* dst = P.partials + ((size_t)it.part * P.Hq + head) * kPartStride;
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
          for (int a = 0; a < 4; ++a)
            *(f32x4*)(dst + n * 32 + a * 8 + h2 * 4) =
                (f32x4){acc[n][4 * a], acc[n][4 * a + 1], acc[n][4 * a + 2], acc[n][4 * a + 3]};
        if (h2 == 0) {
          dst[128] = m;
          dst[129] = l;
        }
      }
    }
    it = itn;
  }
  if (wg < kClockSlots) clock_record(P, wg, 2);
}

// Combines the split-K partials of one token (decode, or a prefill row whose KV range was split).
// grid (n_merge, ceil(Hq/8)), 256 threads: 32 lanes per (token, head), 4 dims per lane.  The
// partials of up to 8 partitions are loaded at once (nothing but the item is on their address
// path); longer lists are folded in 8 at a time with a running maximum.
__global__ __launch_bounds__(256) void merge_kernel(StepParams P, int first) {
  const MergeItem it = P.mitems[first + blockIdx.x];
  const int head = blockIdx.y * 8 + (threadIdx.x >> 5);
  if (head >= P.Hq) return;
  const int x = (threadIdx.x & 31) * 4;
  const float* base = P.partials + ((size_t)it.part0 * P.Hq + head) * kPartStride;
  const size_t stride = (size_t)P.Hq * kPartStride;
  float mstar = PS_NEG_INF, L = 0.f;
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < it.n_parts; k0 += 8) {
    float mk[8], lk[8];
    f32x4 ok[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = k0 + i < it.n_parts ? k0 + i : it.n_parts - 1;
      const float* p = base + (size_t)k * stride;
      mk[i] = p[128];
      lk[i] = p[129];
      ok[i] = *(const f32x4*)(p + x);
    }
    float m_new = mstar;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (k0 + i >= it.n_parts) mk[i] = PS_NEG_INF;  // a repeat of the last partition: weight 0
      m_new = fmaxf(m_new, mk[i]);
    }
    // a partition whose row saw no key has m = -inf (and l = 0, o = 0): weight 0
    const float f0 = mstar == PS_NEG_INF ? 0.f : __builtin_amdgcn_exp2f(mstar - m_new);
    L *= f0;
    o *= f0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float f = mk[i] == PS_NEG_INF ? 0.f : __builtin_amdgcn_exp2f(mk[i] - m_new);
      L += lk[i] * f;
      o += ok[i] * f;
    }
    mstar = m_new;
  }
  const size_t oi = ((size_t)it.tok * P.Hq + head) * kHeadDim + x;
  const float inv = 1.f / L;
  if (P.out_f32) {
    *(f32x4*)((float*)P.out + oi) = o * inv;
  } else {
    uint2 w = {pack_bf16x2(o[0] * inv, o[1] * inv), pack_bf16x2(o[2] * inv, o[3] * inv)};
    *(uint2*)((uint16_t*)P.out + oi) = w;
  }
}

// ------------------------------------------------------------------------------------ prefill
// Causal attention of prefill chunks on 32x32x16 bf16 MFMA.  1-D grid, 512 threads = 8 waves,
// i.e. two waves per SIMD: on this chip a wave cannot overlap its own VALU work (softmax) with
// its own MFMAs, two waves sharing a SIMD can, so each wave keeps its state within 256
// registers.  A workgroup owns a tile of query tokens of one request for one kv-head and HW of
// its G query heads; wave w owns 32 consecutive query tokens (one 32-column B tile) of head
// z*HW + w % HW, token sub-tile w / HW.  All eight waves walk the same 64-token KV tiles.
//
// KV tiles go from the cache straight into LDS (global_load_lds_dwordx4, no VGPR round trip), every load one
// contiguous KiB of one block's K or V slice (scalar base, fixed per-lane offset, instruction offset).  A 64-token
// tile is two halves of 32 tokens (two blocks each).  The K of a block lies in LDS as it lies in the cache,
// [dim/8][token][8 dims]; a wave gathers its A operand of dim chunk c from it with one 16-byte ds_read per lane
// (row j of the operand = slot kslot(j) of block j>>4, dim group 2c + h2: the 16 lanes of a quarter wave read the 16
// consecutive slots of one group, so no bank conflict).  V arrives in MFMA operand order: a fragment is the 1 KiB
// that the 64 lanes feed to one MFMA, lane after lane (fragment 4u+n = dims 32n.. of block u), read back with one
// conflict-free 16-byte ds_read per lane.  Wave w fetches two KiB of K and two of V of block w >> 1 of the tile.
// The LDS ring holds kStages tiles; loads run kStages-1 tiles ahead of the compute, one barrier per tile.
//
// Row j of a K operand is token pi(j) of its half (bits 2 and 3 of j swapped).  With the
// 32x32 result layout this makes the 8 probabilities a lane holds for MFMA step u the 8
// consecutive tokens 16u + 8*h2 .. +7, so its V operand is one contiguous 16-byte run of the
// dim-major V block.
//
// Workgroup -> work mapping: consecutive workgroup ids go to consecutive XCDs (8 of them, each
// with its own L2), so the kv-head is taken from the low bits of the id: the workgroups that
// share one XCD's L2 then walk the same K/V stream.
constexpr int kPrefillWaves = 8;
constexpr int kPrefillRows = 32;    // query tokens per wave
constexpr int kPrefillKV = 64;      // KV tokens per pipeline step
constexpr int kStages = 4;
constexpr int kLoadsPerTile = 4;
constexpr int kIdTiles = 512;       // block ids of up to this many KV tiles (32k tokens) are kept in LDS    // global->LDS loads each wave issues per tile

// Four block-table entries through the scalar cache.  Written as asm because the compiler will
// not use scalar loads next to the memory-clobbering LDS loads above, and its vector-load
// fallback would wait for vmcnt(0), i.e. for every tile still in flight.
__device__ __forceinline__ void load_ids(const int* p0, const int* p1, const int* p2, const int* p3, int (&id)[4]) {
  asm volatile(
      "s_load_dword %0, %4, 0x0\n\ts_load_dword %1, %5, 0x0\n\ts_load_dword %2, %6, 0x0\n\t"
      "s_load_dword %3, %7, 0x0\n\ts_waitcnt lgkmcnt(0)"
      : "=&s"(id[0]), "=&s"(id[1]), "=&s"(id[2]), "=&s"(id[3])
      : "s"(p0), "s"(p1), "s"(p2), "s"(p3));
}

struct PrefillHalf {
  uint4 k[2][256];  // block u of the half as it lies in the cache: [dim/8][token][8 dims], 16 bytes per (dim group, token)
  uint4 v[8][64];   // fragment 4u+n: dims 32n..32n+31 of block u, in MFMA A-operand lane order
};
struct PrefillStage {
  PrefillHalf h[2];
};

// bid: index of the prefill workgroup in the launch; sm: the LDS ring of kStages tiles; id_lds: kIdTiles * 4 ints.
__device__ __forceinline__ void prefill_role(const StepParams& P, int bid, int HW, int n_zsplit, PrefillStage* sm, int* id_lds) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = lane & 31;   // row of the K operand / query column of Q, P, O
  const int h2 = lane >> 5;  // k-group
  const int Hkv = P.Hkv, G = P.G;
  const int g = bid % Hkv;
  const int z = (bid / Hkv) % n_zsplit;
  const PrefillTile t = P.ptiles[bid / (Hkv * n_zsplit)];
  const int head = g * G + z * HW + wave % HW;
  const int SUB = kPrefillWaves / HW;
  const int r = t.req;
  const int qs = P.q_start[r];
  const int lq = P.q_start[r + 1] - qs;
  const int L = P.kv_len[r];
  const int p = L - lq;
  const int q0 = t.q0 + (wave / HW) * kPrefillRows;  // this wave's first query token
  const bool active = q0 < lq;
  const int* table = P.block_ids + P.bt_start[r];
  const int nblk = (L + kBlockTokens - 1) >> 4;

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
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;

  const int wg_last = (t.q0 + SUB * kPrefillRows < lq ? t.q0 + SUB * kPrefillRows : lq) - 1;
  const int reach = (p + wg_last) / kPrefillKV + 1;  // KV tiles any query of the workgroup can see
  const int tile0 = t.tile_begin;                    // this partition: tiles [tile0, tile1)
  const int tile1 = t.tile_end < reach ? t.tile_end : reach;
  const int ntiles = tile1 - tile0;                  // workgroup-uniform; the host never makes it < 1
  const int nt_ids = ntiles > 1 ? ntiles : 1;        // tiles whose block ids are looked up (never none)
  const int my_last = p + (q0 + kPrefillRows < lq ? q0 + kPrefillRows : lq) - 1;  // last visible key
  const int qpos = p + q0 + j;

  // K row j of a fragment is token pi(j) of its half: block j>>4, slot 8*bit2(j) + 4*bit3(j) + (j&3)
  const int kslot = 8 * ((j >> 2) & 1) + 4 * ((j >> 3) & 1) + (j & 3);
  const uint32_t sm_base = (uint32_t)(uintptr_t)(&sm[0]);  // LDS byte address of the ring

  // Block ids of the i-th tile of the partition (clamped to its last tile; absent blocks repeat the
  // last present one and are fully masked).  For partitions of up to kIdTiles tiles the ids sit in
  // LDS (filled below, before the ring starts): the read is issued one iteration before its use
  // and costs no wait.  Longer partitions read them through the scalar cache and wait for it.
  const bool ids_in_lds = nt_ids <= kIdTiles;
  auto lookup = [&](int i, int4& idv) {
    i = i < nt_ids ? i : nt_ids - 1;
    if (ids_in_lds) {
      idv = *(const int4*)&id_lds[i * 4];
    } else {
      const int b0 = (tile0 + i) * (kPrefillKV / kBlockTokens);
      const int last = nblk - 1;
      int id[4];
      load_ids(table + b0, table + (b0 + 1 < last ? b0 + 1 : last), table + (b0 + 2 < last ? b0 + 2 : last),
               table + (b0 + 3 < last ? b0 + 3 : last), id);
      idv = make_int4(id[0], id[1], id[2], id[3]);
    }
  };
  // Issues this wave's loads of one tile into ring slot `stage`.  Wave w fetches from block (w >> 1) of the tile's
  // four (half w >> 2, block u = (w >> 1) & 1 of the half) the two KiB 2(w & 1), 2(w & 1) + 1 of its K slice (dim
  // groups 8(w & 1) .. +7, a straight copy) and of its V slice (dims 64(w & 1) .. +63, as two operand fragments).
  // Every load is one contiguous KiB addressed by a wave-uniform base, a per-lane offset that never changes and an
  // instruction offset (which counts on the LDS side too): next to busy MFMA waves this form is taken far faster than
  // one with a 64-bit address per lane.  Every call issues exactly kLoadsPerTile loads (past the end the last tile
  // is fetched again): the vmcnt bookkeeping below counts on it.
  const int my_hf = wave >> 2, my_u = (wave >> 1) & 1, my_qp = wave & 1;
  const uint32_t k_voff = (uint32_t)lane * 16u;
  const uint32_t v_voff = (uint32_t)(j * kBlockTokens + 8 * h2) * 2u;
  auto issue = [&](int stage, const int4& idv) {
    const int id[4] = {__builtin_amdgcn_readfirstlane(idv.x), __builtin_amdgcn_readfirstlane(idv.y),
                       __builtin_amdgcn_readfirstlane(idv.z), __builtin_amdgcn_readfirstlane(idv.w)};
    const int blk = my_hf ? (my_u ? id[3] : id[2]) : (my_u ? id[1] : id[0]);
    const uint32_t st = sm_base + (uint32_t)stage * (uint32_t)sizeof(PrefillStage) + (uint32_t)my_hf * 16384u;
    const char* kb = (const char*)k_slice(P.cache, blk, Hkv, g) + my_qp * 2048;
    const char* vb = (const char*)v_slice(P.cache, blk, Hkv, g) + my_qp * 2048;
    const uint32_t kd = st + (uint32_t)my_u * 4096u + (uint32_t)my_qp * 2048u;
    const uint32_t vd = st + 8192u + (uint32_t)(my_u * 4 + my_qp * 2) * 1024u;
    load_to_lds16_sbase<0>(kb, k_voff, kd);
    load_to_lds16_sbase<1024>(kb, k_voff, kd);
    load_to_lds16_sbase<0>(vb, v_voff, vd);
    load_to_lds16_sbase<1024>(vb, v_voff, vd);
  };

  if (ids_in_lds) {
    const int last = nblk - 1;
    for (int e = threadIdx.x; e < nt_ids * 4; e += kPrefillWaves * 64) {
      const int bi = tile0 * (kPrefillKV / kBlockTokens) + e;
      id_lds[e] = table[bi < last ? bi : last];
    }
    __syncthreads();
  }

  // The Q loads above must be complete, and known to the compiler to be complete, before the ring
  // starts: otherwise its own vmcnt bookkeeping makes every MFMA in the loop wait for vmcnt(0),
  // which also waits for every tile in flight.
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(PS_VMCNT(0));
  asm volatile("" ::: "memory");

  int4 id;
#pragma unroll
  for (int i = 0; i < kStages - 1; ++i) {
    lookup(i, id);
    issue(i, id);
  }
  lookup(kStages - 1, id);  // ids of the tile the first iteration will issue

  for (int it = 0; it < ntiles; ++it) {
    const int stage = it % kStages;
    const int ts = (tile0 + it) * kPrefillKV;
    // own loads of this tile have landed (the younger ones may still fly) ...
    __builtin_amdgcn_s_waitcnt(PS_VMCNT(kLoadsPerTile * (kStages - 2)));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();  // ... and so have everybody's; everyone is done with tile-1
    asm volatile("" ::: "memory");
    issue((it + kStages - 1) % kStages, id);  // tile it + kStages-1 refills the slot of tile it-1
    lookup(it + kStages, id);                  // ids for the next iteration's issue

    if (ts + kPrefillKV > L) {
      // Last tile of the request: slots past kv_len may hold anything.  The wave that fetched a V
      // fragment zeroes those slots in LDS before anyone multiplies by them (0 * NaN is NaN).
      const int first = ts + 32 * my_hf + 16 * my_u + 8 * h2;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int f = my_u * 4 + my_qp * 2 + k;
        const uint4 vv = sm[stage].h[my_hf].v[f][lane];
        const uint2 lo = zero_from(make_uint2(vv.x, vv.y), first, L);
        const uint2 hi = zero_from(make_uint2(vv.z, vv.w), first + 4, L);
        sm[stage].h[my_hf].v[f][lane] = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
      __syncthreads();  // workgroup-uniform branch
    }

    if (active && ts <= my_last) {
      const PrefillStage& S = sm[stage];
      // all 16 K fragments of the tile are requested from LDS before the first MFMA needs one,
      // and the 16 V fragments right behind them, so that LDS latency is paid once per tile, not
      // once per MFMA (left alone, the compiler sinks every ds_read next to its MFMA)
      bf16x8 kf[2][8], vf[2][8];
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int c = 0; c < 8; ++c) kf[hf][c] = as_bf16x8(S.h[hf].k[j >> 4][(2 * c + h2) * 16 + kslot]);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 s[2];
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[hf][e] = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c)
          s[hf] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[hf][c], qop[c], s[hf], 0, 0, 0);
      }
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int f = 0; f < 8; ++f) vf[hf][f] = as_bf16x8(S.h[hf].v[f][lane]);
      __builtin_amdgcn_sched_barrier(0);
      // s[hf][e]: token ts + 32*hf + 16*(e/8) + 8*h2 + e%8, query q0 + j (raw dot products)
      if (ts + kPrefillKV - 1 > p + q0) {  // diagonal tile (wave-uniform test)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int tok = ts + 32 * hf + 16 * (e >> 3) + 8 * h2 + (e & 7);
            if (tok > qpos) s[hf][e] = PS_NEG_INF;
          }
      }
      // max16 starts with the wait states an MFMA result needs before a vector instruction may read it
      float tmax = max2(max16<true>(s[0]), max16<false>(s[1]));
      tmax = xor32_max(tmax) * P.scale_log2;
      // a row that sees nothing in this tile keeps its m; a row that has seen nothing yet in this
      // partition has m = -inf, l = 0 and all-zero accumulators
      if (__builtin_amdgcn_ballot_w64(tmax > m + PS_RESCALE_SLACK) != 0) {  // some row outgrew its reference
        const float m_new = fmaxf(m, tmax);
        const float alpha = m_new == PS_NEG_INF ? 1.f : __builtin_amdgcn_exp2f(m - m_new);
        l *= alpha;
        m = m_new;
#pragma unroll
        for (int n = 0; n < 4; ++n) acc[n] *= alpha;
      }
      const float m_use = m == PS_NEG_INF ? 0.f : m;  // all scores of such a row are -inf: exp2 gives 0
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[hf][e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[hf][e], P.scale_log2, -m_use));
        uint4 pv[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
          pv[u] = make_uint4(pack_bf16x2(s[hf][8 * u + 0], s[hf][8 * u + 1]), pack_bf16x2(s[hf][8 * u + 2], s[hf][8 * u + 3]),
                             pack_bf16x2(s[hf][8 * u + 4], s[hf][8 * u + 5]), pack_bf16x2(s[hf][8 * u + 6], s[hf][8 * u + 7]));
        // the row sum is that of the rounded probabilities, the ones the output MFMAs multiply by: numerator and
        // denominator then carry the same rounding, and a row that one key dominates comes out as that key's value
        l += sum_bf16x16(pv[0], pv[1]);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 pop = as_bf16x8(pv[u]);
#pragma unroll
          for (int n = 0; n < 4; ++n)
            acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[hf][u * 4 + n], pop, acc[n], 0, 0, 0);
        }
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(PS_VMCNT(0));  // no load may still be writing LDS when the wave ends
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
    const int slot = t.part + (row - t.q0) * t.n_parts + t.k;
    float* dst = P.partials + ((size_t)slot * P.Hq + head) * kPartStride;
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
}

// ------------------------------------------------------------------------------------ attention
// One launch for the whole mixed batch.  The first n_decode_wgs workgroups take the decode role,
// the rest the prefill role.  Every workgroup claims the LDS of a whole CU (the prefill ring),
// so the workgroups are resident one per CU: the decode workgroups, first in dispatch order,
// settle on n_decode_wgs CUs and stay there for the length of the launch (their slots are cut to
// last that long), streaming the cache at HBM speed with one wave per SIMD; the prefill
// workgroups go through the remaining CUs, heaviest first, and keep the matrix pipes busy; they
// also inherit the decode CUs as those finish.  Measured on the mixed workloads, side by side
// the two take 5 to 18 % less time than one after the other.  n_decode_wgs is a multiple of the
// XCD count (padded with workgroups that exit at once), so that the prefill workgroups keep their
// kv-head to XCD mapping.
__global__ __launch_bounds__(kPrefillWaves * 64) void attention_kernel(StepParams P, const DecodeItem* __restrict__ ditems,
                                                                       const int32_t* __restrict__ dslots,
                                                                       const int32_t* __restrict__ block_ids, int n_slots,
                                                                       int n_decode_wgs, int HW, int n_zsplit) {
  __shared__ __attribute__((aligned(16))) char lds[sizeof(PrefillStage) * kStages + kIdTiles * 4 * sizeof(int)];
  static_assert(sizeof(DecodeQ) * kDecodeWaves <= sizeof(PrefillStage) * kStages, "decode Q copies fit the prefill ring");
  {
    const int role_idx = (int)blockIdx.x < n_decode_wgs ? (int)blockIdx.x : (int)blockIdx.x - n_decode_wgs;
    if (role_idx < kClockSlots) clock_record(P, ((int)blockIdx.x < n_decode_wgs ? 0 : kClockSlots) + role_idx, 0);
  }
  if ((int)blockIdx.x < n_decode_wgs)
    decode_role(P, ditems, dslots, block_ids, n_slots, blockIdx.x, (DecodeQ*)lds);
  else
    prefill_role(P, (int)blockIdx.x - n_decode_wgs, HW, n_zsplit, (PrefillStage*)lds,
                 (int*)(lds + sizeof(PrefillStage) * kStages));
}

// ------------------------------------------------------------------------------------ block copy
// dst_pool[dst_ids[k]] <- src_pool[src_ids[k]] for k < n, whole blocks.  Either pool may be
// pinned host memory addressed over the host link.  A workgroup moves one unit of LPL * 4 KiB per
// pass (LPL 16-byte loads in flight per lane, then LPL stores); grid-stride over units.  Few
// workgroups with many loads in flight each: next to an attention kernel that saturates HBM the
// copy's own read latency grows several-fold, and it is bytes in flight that keep the link busy.
template <int LPL>
__global__ __launch_bounds__(256) void block_copy_kernel(const int32_t* __restrict__ src_ids,
                                                         const int32_t* __restrict__ dst_ids, int n,
                                                         const char* __restrict__ src_pool,
                                                         char* __restrict__ dst_pool, size_t block_bytes) {
  constexpr size_t kUnit = (size_t)LPL * 4096;
  const int upb = (int)(block_bytes / kUnit);
  const long total = (long)n * upb;
  for (long u = blockIdx.x; u < total; u += gridDim.x) {
    const int k = (int)(u / upb);
    const size_t off = (size_t)(u % upb) * kUnit + threadIdx.x * 16;
    const char* s = src_pool + (size_t)src_ids[k] * block_bytes + off;
    char* d = dst_pool + (size_t)dst_ids[k] * block_bytes + off;
    u32x4 v[LPL];
#pragma unroll
    for (int i = 0; i < LPL; ++i) v[i] = __builtin_nontemporal_load((const u32x4*)(s + i * 4096));
#pragma unroll
    for (int i = 0; i < LPL; ++i) __builtin_nontemporal_store(v[i], (u32x4*)(d + i * 4096));
  }
}

// ------------------------------------------------------------------------------------ launchers
hipError_t launch_prologue(const StepParams& p, const void* src_pinned, void* dst, size_t bytes,
                           const AppendItem* aitems_pinned, int n_items, hipStream_t s) {
  const int n16 = (int)(bytes / 16);
  const int n_up = std::min((n16 + 1023) / 1024, 64);  // 4 loads per lane in flight
  const int n_pairs = n_items * p.Hkv;
  const int grid = n_up + (n_pairs + 1) / 2;
  if (grid <= 0) return hipSuccess;
  hipLaunchKernelGGL(prologue_kernel, dim3(grid), dim3(256), 0, s, p, (const uint4*)src_pinned, (uint4*)dst, n16, n_up,
                     aitems_pinned, n_pairs);
  return hipGetLastError();
}

hipError_t launch_merge(const StepParams& p, int first, int n_merge, hipStream_t s) {
  if (n_merge <= 0) return hipSuccess;
  hipLaunchKernelGGL(merge_kernel, dim3(n_merge, (p.Hq + 7) / 8), dim3(256), 0, s, p, first);
  return hipGetLastError();
}

int prefill_heads_per_wg(int G) { return G % 8 == 0 ? 8 : (G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1)); }
int prefill_tile_tokens(int G) { return (kPrefillWaves / prefill_heads_per_wg(G)) * kPrefillRows; }

int decode_waves_per_wg() { return kDecodeWaves; }

hipError_t launch_attention(const StepParams& p, int n_slots, int n_tiles, hipStream_t s, int* n_decode_wgs_out,
                            int* n_prefill_wgs_out) {
  const int HW = prefill_heads_per_wg(p.G);
  const int nz = p.G / HW;
  const long long n_prefill_wgs = (long long)n_tiles * p.Hkv * nz;
  // decode workgroups: one per kDecodeWaves slots and kv-head, rounded up to a multiple of 8 (XCDs)
  const long long n_decode_wgs = n_slots > 0 ? (((long long)(n_slots + kDecodeWaves - 1) / kDecodeWaves * p.Hkv + 7) / 8 * 8) : 0;
  const long long grid = n_decode_wgs + n_prefill_wgs;
  if (n_decode_wgs_out) *n_decode_wgs_out = (int)std::min<long long>(n_decode_wgs, 0x7fffffffLL);
  if (n_prefill_wgs_out) *n_prefill_wgs_out = (int)std::min<long long>(n_prefill_wgs, 0x7fffffffLL);
  if (grid <= 0) return hipSuccess;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attention_kernel, dim3((unsigned)grid), dim3(kPrefillWaves * 64), 0, s, p, p.ditems, p.dslots, p.block_ids,
                     n_slots, (int)n_decode_wgs, HW, nz);
  return hipGetLastError();
}

hipError_t launch_block_copy(const int32_t* src_ids, const int32_t* dst_ids, int n, const void* src_pool,
                             void* dst_pool, size_t block_bytes, int workgroups, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const bool big = block_bytes % 32768 == 0;  // else a block is an odd multiple of 8 KiB
  const long total = (long)n * (long)(block_bytes / (big ? 32768 : 8192));
  int grid = (int)(total < workgroups ? total : workgroups);
  if (grid < 1) grid = 1;
  if (big)
    hipLaunchKernelGGL(block_copy_kernel<8>, dim3(grid), dim3(256), 0, s, src_ids, dst_ids, n,
                       (const char*)src_pool, (char*)dst_pool, block_bytes);
  else
    hipLaunchKernelGGL(block_copy_kernel<2>, dim3(grid), dim3(256), 0, s, src_ids, dst_ids, n,
                       (const char*)src_pool, (char*)dst_pool, block_bytes);
  return hipGetLastError();
}

}  // namespace ps
