// What this GPU gives the two kinds of work of an attention step, measured with bare kernels (no attention
// arithmetic): the numbers behind the launch planner's machine constants (ps_layer_cfg.plan_*) and behind the
// question how far the matrix pipes and HBM can be driven at once.  A stand-alone program:
//
//   ps_machine_probe            all sections
//   ps_machine_probe mfma       matrix-pipe rate and shader clock against the operand bits
//   ps_machine_probe stream     cache-streaming rate of one CU and of the chip against the waves per CU
//   ps_machine_probe share      an MFMA wave set and a streaming wave set in one workgroup, alone and together
//   ps_machine_probe loads      what a 16-byte-per-lane load costs the wave that issues it, by destination and source
//
// Sections
//  mfma    two waves per SIMD issue v_mfma_f32_32x32x16_bf16 back to back, four independent accumulators each,
//          the A operand of every MFMA freshly read from LDS (1 KiB per MFMA, as in the prefill role), with or
//          without the vector arithmetic of an online softmax between them (per MFMA: multiply-add, exponential,
//          add, and a bf16 conversion every other one).  Operands: all zero, or random bf16 of magnitude about 1.
//          Every workgroup reads the shader-clock counter and the constant 100 MHz counter at its start and end;
//          the ratio is the clock the chip ran it at.  The published peak, 2.5 PFLOP/s, is 1024 SIMDs x one MFMA
//          of 32768 FLOP per 32 cycles at 2400 MHz.
//  stream  every lane keeps 16 non-temporal 16-byte loads in flight (a wave: 16 KiB, one decode tile), nothing is
//          reused; 4 or 8 waves per CU, on 32 CUs (HBM far from its limit: what one CU can take) and on all CUs.
//  share   workgroups of 12 waves, one per CU: 8 waves as in `mfma` (random operands, softmax arithmetic), 4
//          waves as in `stream` over 4 GiB.  Timed with only the first kind active, only the second, and both.
//  loads   one workgroup per CU of 1, 2, 4 or 8 waves; a wave issues rounds of 16 loads of 16 bytes per lane (1 KiB
//          per instruction) and waits for each round.  Destination LDS (global_load_lds_dwordx4, M0 written before
//          every load) or registers; source a region every workgroup shares (1 MiB: served by the L2s) or 128 KiB of
//          its own per wave out of 256 MiB (served by HBM and the memory-side cache).  Reported: shader cycles per
//          load the wave spends issuing, cycles per load overall, and the rate per CU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                       \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) {                                                         \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      exit(1);                                                                      \
    }                                                                               \
  } while (0)

namespace {

constexpr int kLdsVec = 8192;  // uint4 elements: 128 KiB, so that one workgroup fills a CU
constexpr double kMfmaFlop = 2.0 * 32 * 32 * 16;

__device__ __forceinline__ unsigned hash32(unsigned x) {
  x ^= x >> 16;
  x *= 0x7feb352dU;
  x ^= x >> 15;
  x *= 0x846ca68bU;
  x ^= x >> 16;
  return x;
}
// two random bf16 values with sign and mantissa from the hash and an exponent of 2^-1 or 2^0
__device__ __forceinline__ unsigned random_bf16x2(unsigned i) {
  const unsigned h = hash32(i);
  return (h & 0x807F807Fu) | 0x3F003F00u | ((h >> 3) & 0x00800080u);
}

struct Clocks {
  unsigned long long shader0, ref0, shader1, ref1;
};

// The MFMA wave set: `iters` rounds of 8 MFMAs per wave.  VALU: the softmax-like vector work between MFMAs.
template <bool VALU>
__device__ __forceinline__ float mfma_waves(const uint4* lds, int wave, int lane, int iters) {
  bf16x8 b = __builtin_bit_cast(bf16x8, lds[lane + 64 * wave]);
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  float x0 = lane * 1e-3f, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4;
  const float k0 = 0.25f, k1 = -1.f;
  bf16x8 f[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) f[i] = __builtin_bit_cast(bf16x8, lds[i * 64 + lane]);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      f32x16& c = (s & 3) == 0 ? c0 : (s & 3) == 1 ? c1 : (s & 3) == 2 ? c2 : c3;
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(f[s]), "v"(b));
      f[s] = __builtin_bit_cast(bf16x8, lds[wave * 1024 + ((it & 1) * 8 + s) * 64 + lane]);  // the next round's operand
      if (VALU) {
        asm volatile("v_fma_f32 %0, %0, %5, %6\n v_exp_f32 %3, %3\n v_add_f32 %1, %1, %2"
                     : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3), "+v"(x4)
                     : "v"(k0), "v"(k1));
        if (s & 1) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(x4) : "v"(x1), "v"(x2));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if ((it & 63) == 63) {  // keep the accumulators finite
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        c0[i] *= 1e-30f;
        c1[i] *= 1e-30f;
        c2[i] *= 1e-30f;
        c3[i] *= 1e-30f;
      }
    }
  }
  float s = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  return s + x0 + x1 + x2 + x3 + x4;
}

// The streaming wave: tiles of 16 KiB (16 loads of 1 KiB per wave), tile t of wave w at ((t * n_waves + w) * 16) KiB.
__device__ __forceinline__ unsigned stream_wave(const u32x4* __restrict__ src, size_t tiles, size_t n_waves, size_t w, int lane) {
  u32x4 acc = {0, 0, 0, 0};
  for (size_t t = 0; t < tiles; ++t) {
    const u32x4* p = src + ((t * n_waves + w) * 16) * 64 + lane;
    u32x4 v[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) v[c] = __builtin_nontemporal_load(p + c * 64);
    __builtin_amdgcn_sched_barrier(0);  // all 16 in flight before the first is waited for
#pragma unroll
    for (int c = 0; c < 16; ++c) acc ^= v[c];
  }
  return acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// role bit 0: waves 0..7 run the MFMA set; bit 1: waves 8..8+stream_waves-1 stream.  Block = (8 + stream_waves) * 64.
template <bool VALU>
__global__ __launch_bounds__(1024) void probe_kernel(int roles, int zero_operands, int iters, const u32x4* __restrict__ src,
                                                     size_t tiles, size_t n_stream_waves, int stream_waves, float* sink,
                                                     Clocks* clocks) {
  __shared__ uint4 lds[kLdsVec];
  for (int i = threadIdx.x; i < kLdsVec; i += blockDim.x)
    lds[i] = zero_operands ? make_uint4(0, 0, 0, 0)
                           : make_uint4(random_bf16x2(4 * i), random_bf16x2(4 * i + 1), random_bf16x2(4 * i + 2), random_bf16x2(4 * i + 3));
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) {
    clocks[blockIdx.x].shader0 = __builtin_amdgcn_s_memtime();
    clocks[blockIdx.x].ref0 = __builtin_amdgcn_s_memrealtime();
  }
  float r = 0.f;
  if (wave < 8) {
    if (roles & 1) r = mfma_waves<VALU>(lds, wave, lane, iters);
    if (threadIdx.x == 0) {
      clocks[blockIdx.x].shader1 = __builtin_amdgcn_s_memtime();
      clocks[blockIdx.x].ref1 = __builtin_amdgcn_s_memrealtime();
    }
  } else if ((roles & 2) && wave - 8 < stream_waves) {
    r = (float)stream_wave(src, tiles, n_stream_waves, (size_t)blockIdx.x * stream_waves + (wave - 8), lane);
  }
  if (r == 12345.678f) sink[0] = r;  // keeps the work alive
}

struct Result {
  float ms;
  double mhz;
};

template <bool VALU>
Result launch(int grid, int roles, int zero_operands, int iters, const u32x4* src, size_t tiles, int stream_waves, float* sink,
              Clocks* clocks_dev) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  float best = 1e30f;
  for (int rep = 0; rep < 3; ++rep) {
    float ms = 0;
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(probe_kernel<VALU>, dim3(grid), dim3((8 + stream_waves) * 64), 0, 0, roles, zero_operands, iters, src, tiles,
                       (size_t)grid * stream_waves, stream_waves, sink, clocks_dev);
    CK(hipGetLastError());
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms, e0, e1));
    best = std::min(best, ms);
  }
  std::vector<Clocks> c((size_t)grid);
  CK(hipMemcpy(c.data(), clocks_dev, sizeof(Clocks) * (size_t)grid, hipMemcpyDeviceToHost));
  std::vector<double> mhz;
  for (auto& x : c)
    if (x.ref1 > x.ref0 + 20) mhz.push_back((double)(x.shader1 - x.shader0) / (double)(x.ref1 - x.ref0) * 100.0);
  std::sort(mhz.begin(), mhz.end());
  CK(hipEventDestroy(e0));
  CK(hipEventDestroy(e1));
  return Result{best, mhz.empty() ? 0.0 : mhz[mhz.size() / 2]};
}

// `loads` section.  DST 0: to LDS, 1: to registers.  shared != 0: every workgroup reads the same 1 MiB.
template <int DST>
__global__ __launch_bounds__(512) void loads_kernel(const char* __restrict__ src, int shared, int rounds, unsigned long long* out,
                                                    float* sink) {
  __shared__ __attribute__((aligned(16))) char lds[128 * 1024];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const char* p = src + (size_t)(shared ? wave : blockIdx.x * nw + wave) * (8 * 16384) + lane * 16;
  const unsigned base = (unsigned)(uintptr_t)lds + wave * 16384;
  unsigned long long t_issue = 0, t_all = __builtin_amdgcn_s_memtime();
  u32x4 acc = {0, 0, 0, 0};
  for (int r = 0; r < rounds; ++r) {
    const char* q = p + (size_t)(r & 7) * 16384;
    const unsigned long long t0 = __builtin_amdgcn_s_memtime();
    if (DST == 0) {
#pragma unroll
      for (int f = 0; f < 16; ++f) {
        unsigned saved;
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved)
                     : "v"(q + f * 1024), "s"(base + f * 1024)
                     : "memory");
      }
      t_issue += __builtin_amdgcn_s_memtime() - t0;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
      u32x4 v[16];
#pragma unroll
      for (int f = 0; f < 16; ++f) asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v[f]) : "v"(q + f * 1024) : "memory");
      t_issue += __builtin_amdgcn_s_memtime() - t0;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int f = 0; f < 16; ++f) {
        asm volatile("" : "+v"(v[f]));
        acc += v[f];
      }
    }
  }
  t_all = __builtin_amdgcn_s_memtime() - t_all;
  if (lane == 0) {
    atomicAdd(&out[0], t_issue);
    atomicAdd(&out[1], t_all);
  }
  if (acc.x == 0x12345u) sink[0] = (float)acc.y;
  if (lds[threadIdx.x] == 77) sink[1] = 1.f;
}

void section_loads(int n_cus, const u32x4* buf, float* sink, Clocks* clocks) {
  printf("== loads: one workgroup per CU, rounds of 16 loads of 16 bytes per lane, each round waited for (%d CUs)\n", n_cus);
  unsigned long long* out = (unsigned long long*)clocks;  // two counters; the clock records are not used here
  for (int shared = 1; shared >= 0; --shared)
    for (int dst = 0; dst < 2; ++dst)
      for (int waves : {1, 2, 4, 8}) {
        const int rounds = shared ? 256 : 64;
        unsigned long long z[2] = {0, 0}, o[2];
        hipEvent_t a, b;
        CK(hipEventCreate(&a));
        CK(hipEventCreate(&b));
        for (int pass = 0; pass < 2; ++pass) {  // the first pass warms the caches
          CK(hipMemcpy(out, z, sizeof(z), hipMemcpyHostToDevice));
          CK(hipEventRecord(a));
          if (dst == 0)
            hipLaunchKernelGGL(loads_kernel<0>, dim3(n_cus), dim3(waves * 64), 0, 0, (const char*)buf, shared, pass ? rounds : 8, out, sink);
          else
            hipLaunchKernelGGL(loads_kernel<1>, dim3(n_cus), dim3(waves * 64), 0, 0, (const char*)buf, shared, pass ? rounds : 8, out, sink);
          CK(hipGetLastError());
          CK(hipEventRecord(b));
          CK(hipDeviceSynchronize());
        }
        float ms = 0.f;
        CK(hipEventElapsedTime(&ms, a, b));
        CK(hipMemcpy(o, out, sizeof(o), hipMemcpyDeviceToHost));
        CK(hipEventDestroy(a));
        CK(hipEventDestroy(b));
        const double loads = (double)n_cus * waves * rounds * 16;
        printf("  %-30s %-12s %d waves per CU: %4.0f cycles per load issuing, %4.0f overall, %6.1f GB/s per CU\n",
               shared ? "1 MiB shared by all (L2):" : "128 KiB per wave of 256 MiB:", dst ? "to registers," : "to LDS,", waves, o[0] / loads,
               o[1] / loads, loads * 1024 / n_cus / (ms * 1e6));
        fflush(stdout);
      }
  CK(hipMemset(clocks, 0, sizeof(Clocks) * 1024));
}

void section_mfma(int n_cus, const u32x4* buf, float* sink, Clocks* clocks) {
  printf("== mfma: 8 waves per CU (two per SIMD), one LDS operand fragment per MFMA, %d CUs\n", n_cus);
  const int iters = 6000;
  const double flop = (double)n_cus * 8 * iters * 8 * kMfmaFlop;
  for (int valu = 0; valu < 2; ++valu)
    for (int zero = 1; zero >= 0; --zero) {
      const Result r = valu ? launch<true>(n_cus, 1, zero, iters, buf, 0, 0, sink, clocks) : launch<false>(n_cus, 1, zero, iters, buf, 0, 0, sink, clocks);
      const double pf = flop / (r.ms * 1e-3) / 1e15;
      printf("  %-18s %-26s %7.3f ms  %5.2f PFLOP/s = %.2f of 2.5  shader clock %4.0f MHz  (%.2f of the peak at that clock)\n",
             zero ? "all-zero operands," : "random operands,", valu ? "MFMA + softmax arithmetic:" : "MFMA only:", r.ms, pf, pf / 2.5, r.mhz,
             pf / (2.5 * r.mhz / 2400.0));
      fflush(stdout);
    }
}

void section_stream(int n_cus, const u32x4* buf, size_t buf_bytes, float* sink, Clocks* clocks) {
  printf("== stream: 16 non-temporal 16-byte loads in flight per lane, nothing reused\n");
  for (int cus : {32, n_cus})
    for (int waves : {4, 8}) {
      size_t tiles = 256;  // 4 MiB per wave
      while (tiles * cus * waves * 16384 > buf_bytes) tiles /= 2;
      const Result r = launch<false>(cus, 2, 1, 0, buf, tiles, waves, sink, clocks);
      const double bytes = (double)tiles * cus * waves * 16384;
      printf("  %3d CUs x %d waves: %6.2f TB/s, %5.1f GB/s per CU\n", cus, waves, bytes / (r.ms * 1e-3) / 1e12, bytes / (r.ms * 1e-3) / 1e9 / cus);
      fflush(stdout);
    }
}

void section_share(int n_cus, const u32x4* buf, size_t buf_bytes, float* sink, Clocks* clocks) {
  printf("== share: per CU one workgroup of 8 MFMA waves (random operands, softmax arithmetic) + 4 streaming waves\n");
  size_t tiles = 256;
  while (tiles * n_cus * 4 * 16384 > buf_bytes) tiles /= 2;
  const double bytes = (double)tiles * n_cus * 4 * 16384;
  for (int iters : {3000, 6000}) {
    const Result m = launch<true>(n_cus, 1, 0, iters, buf, tiles, 4, sink, clocks);
    const Result s = launch<true>(n_cus, 2, 0, iters, buf, tiles, 4, sink, clocks);
    const Result b = launch<true>(n_cus, 3, 0, iters, buf, tiles, 4, sink, clocks);
    printf("  MFMA waves alone %.3f ms | streaming waves alone %.3f ms (%.2f TB/s) | both %.3f ms = %.2f x the longer, %.2f x the sum\n", m.ms, s.ms,
           bytes / (s.ms * 1e-3) / 1e12, b.ms, b.ms / std::max(m.ms, s.ms), b.ms / (m.ms + s.ms));
    fflush(stdout);
  }
}

}  // namespace

int main(int argc, char** argv) {
  const char* what = argc > 1 ? argv[1] : "all";
  int dev = 0, n_cus = 0;
  CK(hipGetDevice(&dev));
  CK(hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (n_cus < 32 || n_cus > 1024) {
    fprintf(stderr, "unexpected compute-unit count %d\n", n_cus);
    return 1;
  }
  const size_t buf_bytes = (size_t)4 << 30;
  u32x4* buf = nullptr;
  float* sink = nullptr;
  Clocks* clocks = nullptr;
  CK(hipMalloc((void**)&buf, buf_bytes));
  CK(hipMemset(buf, 0x5a, buf_bytes));
  CK(hipMalloc((void**)&sink, 256));
  CK(hipMalloc((void**)&clocks, sizeof(Clocks) * 1024));
  CK(hipMemset(clocks, 0, sizeof(Clocks) * 1024));
  const bool all = !strcmp(what, "all");
  if (all || !strcmp(what, "mfma")) section_mfma(n_cus, buf, sink, clocks);
  if (all || !strcmp(what, "stream")) section_stream(n_cus, buf, buf_bytes, sink, clocks);
  if (all || !strcmp(what, "share")) section_share(n_cus, buf, buf_bytes, sink, clocks);
  if (all || !strcmp(what, "loads")) section_loads(n_cus, buf, sink, clocks);
  CK(hipFree(buf));
  CK(hipFree(sink));
  CK(hipFree(clocks));
  return 0;
}
