// Benchmark-only study (its own executable, paper_2511_11062_amd/bench_issue_mix; nothing of the attention library
// links it): what rate does the INSTRUCTION MIX of the fused attention kernel allow on gfx950, and what does each
// ingredient of the kernel's stage structure cost?  A register-resident loop issues, per "step", one bf16 MFMA
// 32x32x16, one 16-byte LDS fragment read and a slice of vector-ALU work (1 transcendental + VS-1 fused multiply-adds:
// the count the online softmax needs per MFMA), fenced the way the kernel fences its steps; a "stage" is 32 steps.
// Ingredients that can be switched on: the dependent accumulator chains of S^T = K Q^T (CHAIN), the barrier that ends
// a stage (BAR), the K/V global -> LDS DMA of a stage (DMA pieces of 1 KB per wave, L2-resident source), extra
// instructions per step (EXTRA kind/count), one wave per SIMD with two MFMAs per LDS fragment (QB = 2: 64 Q rows per
// wave), and for those the order "MFMA, slice, MFMA, slice" against "MFMA, MFMA, slice, slice" (GROUPED).
// Operands are either all 1.0 (the clock stays near nominal: issue structure alone) or pseudo-random bf16 N(0,1)
// values (the matrix cores run power-limited: what the attention kernel meets on real data).
//
//   bench_issue_mix [stages per launch, default 30000]
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <utility>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T) const __attribute__((address_space(3))) T*

struct Cfg {
  static constexpr int kNone = 0, kNop = 1, kWaitcnt = 2, kSalu = 3, kValu = 4;
};

// WPS waves per SIMD (workgroups of 4 waves: WPS workgroups per CU); QB MFMAs per LDS fragment; VS vector instructions
// per MFMA; CHAIN/BAR/DMA/GROUPED as above; XK/XN kind and number of extra instructions per step
template <int WPS, int QB, int VS, int CHAIN, int BAR, int DMA, int GROUPED, int XK, int XN>
__global__ __launch_bounds__(256, WPS) void mix_kernel(const uint4* __restrict__ data, const char* __restrict__ big,
                                                       float* out, int stages) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 65536 / 16; i += blockDim.x) ((uint4*)smem)[i] = data[(i + 64 * blockIdx.x) & 4095];
  __syncthreads();
  const int lq = lane & 31, hi = lane >> 5;
  const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)smem;
  uint32_t kread[8];  // swizzled fragment addresses as in the attention kernel: conflict-free 16-byte reads
  for (int kk = 0; kk < 8; ++kk) kread[kk] = lds0 + lq * 256 + ((32 * kk) ^ (16 * (hi ^ (lq & 15))));
  bf16x8 b[QB][8];
  for (int q = 0; q < QB; ++q)
    for (int x = 0; x < 8; ++x) {
      const uint4 t = data[(tid + 256 * (8 * q + x) + 1024) & 4095];
      b[q][x] = __builtin_bit_cast(bf16x8, t);
    }
  f32x16 acc[QB][4], sa[QB][2];
  for (int q = 0; q < QB; ++q) {
    for (int n = 0; n < 4; ++n)
      for (int r = 0; r < 16; ++r) acc[q][n][r] = 0.f;
    for (int n = 0; n < 2; ++n)
      for (int r = 0; r < 16; ++r) sa[q][n][r] = 0.f;
  }
  float v[QB][8];
  for (int q = 0; q < QB; ++q)
    for (int i = 0; i < 8; ++i) v[q][i] = __uint_as_float((data[(tid + i + 8 * q) & 4095].x & 0x007fffffu) | 0x3f000000u);
  bf16x8 frag[3];
  for (int i = 0; i < 3; ++i) frag[i] = *reinterpret_cast<LDS_PTR(bf16x8)>(kread[i]);
  const uint64_t a64 = (uint64_t)big + (size_t)(blockIdx.x % 64) * 65536;
  const u32x4 rsrc = {(uint32_t)a64, (uint32_t)(a64 >> 32) & 0xffffu, 65536u, 0x00020000u};
  const uint32_t voff = lane * 16 + wave * 4096;
  const uint32_t ldsw = __builtin_amdgcn_readfirstlane(lds0 + 4096 * wave);
  float sink = 0.f, vdummy = 1.f;
  uint32_t sdummy = 0;

  auto slice = [&](int q, int u) __attribute__((always_inline)) {
#pragma unroll
    for (int w = 0; w < VS; ++w) {
      float x = v[q][(w + u) & 7];
      if (w == 0)
        x = __builtin_amdgcn_exp2f(x);
      else
        x = __builtin_fmaf(x, 0.9990234375f, 0.0009765625f);
      asm volatile("" : "+v"(x));
      v[q][(w + u) & 7] = x;
    }
  };
  auto extra = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int x = 0; x < XN; ++x) {
      if (XK == Cfg::kNop) asm volatile("s_nop 0");
      if (XK == Cfg::kWaitcnt) asm volatile("s_waitcnt lgkmcnt(15)");
      if (XK == Cfg::kSalu) asm volatile("s_add_u32 %0, %0, 1" : "+s"(sdummy)::"scc");
      if (XK == Cfg::kValu) asm volatile("v_mov_b32 %0, %0" : "+v"(vdummy));
    }
  };
  auto stage = [&](auto parc, int it) __attribute__((always_inline)) {
    constexpr int par = decltype(parc)::value;  // half of LDS read in this stage; the DMA fills the other half
#pragma unroll
    for (int u = 0; u < 32; ++u) {
      const bf16x8 a = frag[u % 3];
      auto mfma = [&](int q) __attribute__((always_inline)) {
        if (CHAIN && u >= 16) {
          const int c = (u - 16) >> 3;
          sa[q][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[q][u & 7], sa[q][c], 0, 0, 0);
        } else {
          acc[q][u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[q][(u >> 2) & 7], acc[q][u & 3], 0, 0, 0);
        }
      };
      auto memory = [&]() __attribute__((always_inline)) {
        frag[u % 3] = *reinterpret_cast<LDS_PTR(bf16x8)>(
            kread[(u + 3) & 7] +
            (uint32_t)(8192 * (((u + 3) >> 3) & 1) + 16384 * (((u + 3) >> 4) & 1) + 32768 * (par ^ 1)));
        if (DMA && u % 2 == 0 && u / 2 < DMA) {
          const int x = u / 2;
          asm volatile("s_add_u32 m0, %2, %3\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
                       :
                       : "v"(voff + 1024 * (x & 3) + 16384 * (x >> 2)), "s"(rsrc), "s"(ldsw), "n"(32768 * par)
                       : "memory", "m0", "scc");
        }
        extra();
      };
      if (!GROUPED) {
#pragma unroll
        for (int q = 0; q < QB; ++q) {
          mfma(q);
          if (q == 0) memory();
          __builtin_amdgcn_sched_barrier(0);
          slice(q, u);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int q = 0; q < QB; ++q) mfma(q);
        memory();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < QB; ++q) slice(q, u);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (CHAIN)
      for (int q = 0; q < QB; ++q) sink += sa[q][0][it & 15] + sa[q][1][it & 15];
    if (DMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (BAR) __syncthreads();
  };
  for (int it = 0; it < stages; it += 2) {
    stage(std::integral_constant<int, 0>{}, it);
    stage(std::integral_constant<int, 1>{}, it);
  }
  float s = sink + (float)sdummy + vdummy;
  for (int q = 0; q < QB; ++q) {
    for (int n = 0; n < 4; ++n)
      for (int r = 0; r < 16; ++r) s += acc[q][n][r];
    for (int n = 0; n < 2; ++n)
      for (int r = 0; r < 16; ++r) s += sa[q][n][r];
    for (int i = 0; i < 8; ++i) s += v[q][i];
  }
  out[blockIdx.x * blockDim.x + tid] = s;
}

static uint4* g_data[2];
static char* g_big;
static int g_stages = 30000;

#define CHECK(x)                                                                    \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) {                                                         \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                       \
      exit(1);                                                                      \
    }                                                                               \
  } while (0)

template <int WPS, int QB, int VS, int CHAIN, int BAR, int DMA, int GROUPED = 0, int XK = 0, int XN = 0>
static void run(const char* name) {
  auto kern = mix_kernel<WPS, QB, VS, CHAIN, BAR, DMA, GROUPED, XK, XN>;
  const int blocks = 256 * WPS, threads = 256, stages = g_stages / QB;
  float* d = nullptr;
  CHECK(hipMalloc(&d, (size_t)blocks * threads * 4));
  CHECK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  double frac[2];
  for (int rnd = 0; rnd < 2; ++rnd) {
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 65536, 0, g_data[rnd], g_big, d, 64);  // warm-up
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 65536, 0, g_data[rnd], g_big, d, stages);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double mfmas = 1024.0 * WPS * stages * 32.0 * QB;  // on the whole device: 1024 SIMDs
    frac[rnd] = mfmas * 32768.0 / (ms * 1e-3) / 2.5e15;
  }
  printf("%-58s %6.3f %6.3f\n", name, frac[0], frac[1]);
  fflush(stdout);
  CHECK(hipFree(d));
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
}

int main(int argc, char** argv) {
  if (argc > 1) g_stages = atoi(argv[1]);
  uint4* h = (uint4*)malloc(4096 * 16);
  for (int r = 0; r < 2; ++r) {  // 0: every bf16 value 1.0; 1: roughly N(0,1) (sum of four uniforms)
    unsigned short* p = (unsigned short*)h;
    for (int i = 0; i < 4096 * 8; ++i) {
      float f = 1.0f;
      if (r) {
        f = 0;
        for (int t = 0; t < 4; ++t) f += (rand() / (float)RAND_MAX) - 0.5f;
        f *= 1.7f;
      }
      unsigned u;
      memcpy(&u, &f, 4);
      p[i] = (unsigned short)(u >> 16);
    }
    CHECK(hipMalloc(&g_data[r], 4096 * 16));
    CHECK(hipMemcpy(g_data[r], h, 4096 * 16, hipMemcpyHostToDevice));
  }
  CHECK(hipMalloc(&g_big, 64 * 65536));
  CHECK(hipMemset(g_big, 0x3c, 64 * 65536));
  printf("fraction of the published dense bf16 peak (2.5 PFLOP/s); %d stages of 32 steps per launch\n", g_stages);
  printf("%-58s %6s %6s\n", "configuration (2 waves per SIMD unless said)", "ones", "random");
  run<2, 1, 0, 0, 0, 0>("warm-up (discard)");
  run<2, 1, 0, 0, 0, 0>("MFMA + LDS fragment read");
  run<2, 1, 3, 0, 0, 0>("+ 3 vector instructions per MFMA");
  run<2, 1, 4, 0, 0, 0>("+ 4 vector instructions per MFMA (the softmax's share)");
  run<2, 1, 4, 1, 0, 0>("  + dependent QK accumulator chains");
  run<2, 1, 4, 0, 1, 0>("  + barrier per stage");
  run<2, 1, 4, 0, 0, 8>("  + K/V DMA, 8 KB per wave per stage");
  run<2, 1, 4, 1, 1, 8>("  + chains + barrier + DMA = the kernel's stage structure");
  run<2, 1, 4, 1, 1, 4>("    same with half the DMA (two Q tiles per workgroup)");
  run<2, 1, 0, 1, 1, 8>("    same without the vector instructions");
  run<2, 1, 4, 1, 1, 8, 0, Cfg::kNop, 1>("    + 1 s_nop per step");
  run<2, 1, 4, 1, 1, 8, 0, Cfg::kWaitcnt, 1>("    + 1 satisfied s_waitcnt per step");
  run<2, 1, 4, 1, 1, 8, 0, Cfg::kSalu, 1>("    + 1 scalar instruction per step");
  run<2, 1, 4, 1, 1, 8, 0, Cfg::kValu, 1>("    + 1 vector instruction per step");
  run<1, 1, 4, 0, 0, 0>("1 wave per SIMD, 1 MFMA per fragment, 4 vector");
  run<1, 2, 4, 0, 0, 0>("1 wave per SIMD, 2 MFMAs per fragment, MFMA slice MFMA slice");
  run<1, 2, 4, 0, 0, 0, 1>("1 wave per SIMD, 2 MFMAs per fragment, MFMA MFMA slice slice");
  return 0;
}
