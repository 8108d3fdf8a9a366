// gfx950 (CDNA4) kernels of the LiteAttention forward path.
//
//   clear_state_kernel   : zero the Skip-Mask and the statistics (step 0)
//   compact_skiplist     : Skip-Mask row -> packed ascending list of live K/V tile indices
//                          (Implementation, "Producer and Skip-List Optimization")
//   lite_attn_fwd_kernel : fused tiled forward over the live tiles with the skip predicate
//                          (Algorithm 2; eq. sparge_cond; tile recurrences of the Preliminaries)
//
// Layout of the fused kernel (one workgroup = one Q tile = one Skip-Mask row, 4 wave64s):
//   * wave w owns Q rows [32w, 32w+32) of the tile; lane l owns Q row (l & 31) of them.
//   * the kernel works on S^T = K Q^T: with v_mfma_f32_32x32x16_bf16 the K rows are the A operand (from
//     LDS) and the Q rows the B operand (registers, loaded once), so a lane's 16 accumulator values per
//     32x32 block all belong to ONE Q row.  Row max and row sum are then in-lane reductions plus one
//     exchange with lane^32, and exp(S^T) in accumulator layout IS the B operand of O^T = V^T P^T:
//     P never moves between lanes.
//   * a 128-column mask tile is streamed as two 64-column stages; K is stored row-major (padded) in LDS,
//     V is transposed in registers on its way into LDS so that V^T fragments are single 16-byte reads.
//   * LDS is double-buffered (2 x 35 KB), one barrier per stage, two workgroups per CU.
//   * the predicate of a tile is reduced per wave with a ballot; the four per-wave results meet through
//     LDS at the barrier that ends the tile and one lane ORs the bit into the global mask row.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lite_attn_kernels.h"

namespace la {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;           // head dimension
constexpr int kTile = 128;        // Skip-Mask tile: 128 Q rows x 128 K/V columns
constexpr int kSub = 64;          // K/V columns per pipeline stage
constexpr int kThreads = 256;
constexpr int kKRow = 272;        // bytes per K row in LDS: 128 bf16 + 16 B pad (conflict-free 16 B reads)
constexpr int kVtRow = 144;       // bytes per V^T row in LDS: 64 bf16 + 16 B pad
constexpr int kKBytes = kSub * kKRow;      // 17408
constexpr int kVtBytes = kD * kVtRow;      // 18432
constexpr int kStage = kKBytes + kVtBytes; // 35840
constexpr int kFlagsOff = 2 * kStage;      // 8 ints: [tile parity][wave]
constexpr int kORow = 272;        // bytes per O row in the epilogue staging (reuses the stage buffers)

__global__ void clear_state_kernel(uint64_t* bits, size_t words, unsigned long long* stats, size_t nstats) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t x = i; x < words; x += stride) bits[x] = 0;
  for (size_t x = i; x < nstats; x += stride) stats[x] = 0;
}

// One wave per Q-tile row: ballot + prefix popcount packs the indices of clear bits.
__global__ __launch_bounds__(256) void compact_skiplist(const uint64_t* __restrict__ bits, int rows, int Tk, int W,
                                                         uint16_t* __restrict__ live_idx,
                                                         uint32_t* __restrict__ live_cnt,
                                                         unsigned long long* __restrict__ stat_skipped_in) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const uint64_t* mrow = bits + (size_t)row * W;
  uint16_t* out = live_idx + (size_t)row * Tk;
  uint32_t n = 0;
  for (int w = 0; w < W; ++w) {
    const uint64_t word = mrow[w];
    const int j = w * 64 + lane;
    const bool live = (j < Tk) && !((word >> lane) & 1ull);
    const uint64_t bal = __ballot(live);
    const uint32_t pre = __popcll(bal & ((1ull << lane) - 1ull));
    if (live) out[n + pre] = (uint16_t)j;
    n += __popcll(bal);
  }
  if (lane == 0) {
    live_cnt[row] = n;
    if (stat_skipped_in && (uint32_t)Tk > n) atomicAdd(stat_skipped_in, (unsigned long long)(Tk - n));
  }
}

__device__ __forceinline__ uint4 ld16(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return *reinterpret_cast<uint32_t*>(&h);
}

struct StageRegs {
  uint4 k[4];
  uint4 v[4];
};

// Global -> registers for one 64-column stage.  Rows past the end of the sequence read as zero.
__device__ __forceinline__ void load_stage(StageRegs& r, const uint16_t* kb, const uint16_t* vb, int64_t stride_n,
                                           int kv0, int N, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const uint4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int row = kv0 + (tid >> 4) + 16 * t;
    r.k[t] = (row < N) ? ld16(kb + (int64_t)row * stride_n + 8 * (tid & 15)) : zero;
  }
  const int kg = lane & 15, dg = 4 * wave + (lane >> 4);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int row = kv0 + 4 * kg + t;
    r.v[t] = (row < N) ? ld16(vb + (int64_t)row * stride_n + 8 * dg) : zero;
  }
}

// Registers -> LDS.  K goes in row-major; V is transposed 4x8 -> 8x4 in registers and written as V^T with the
// K/V index permuted inside each group of 16 so that a lane's 8 contraction values are contiguous.
__device__ __forceinline__ void store_stage(const StageRegs& r, char* stage, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  char* sK = stage;
  char* sVt = stage + kKBytes;
#pragma unroll
  for (int t = 0; t < 4; ++t)
    *reinterpret_cast<uint4*>(sK + ((tid >> 4) + 16 * t) * kKRow + 16 * (tid & 15)) = r.k[t];
  const int kg = lane & 15, dg = 4 * wave + (lane >> 4);
  const int g = kg & 3;
  const int pos = 32 * (kg >> 2) + ((g & 1) << 4) + ((g & 2) << 2);  // bytes: {0,16,8,24}[g]
  const uint32_t v0[4] = {r.v[0].x, r.v[0].y, r.v[0].z, r.v[0].w};
  const uint32_t v1[4] = {r.v[1].x, r.v[1].y, r.v[1].z, r.v[1].w};
  const uint32_t v2[4] = {r.v[2].x, r.v[2].y, r.v[2].z, r.v[2].w};
  const uint32_t v3[4] = {r.v[3].x, r.v[3].y, r.v[3].z, r.v[3].w};
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    uint2 lo, hi;
    lo.x = __builtin_amdgcn_perm(v1[w], v0[w], 0x05040100u);
    lo.y = __builtin_amdgcn_perm(v3[w], v2[w], 0x05040100u);
    hi.x = __builtin_amdgcn_perm(v1[w], v0[w], 0x07060302u);
    hi.y = __builtin_amdgcn_perm(v3[w], v2[w], 0x07060302u);
    *reinterpret_cast<uint2*>(sVt + (8 * dg + 2 * w) * kVtRow + pos) = lo;
    *reinterpret_cast<uint2*>(sVt + (8 * dg + 2 * w + 1) * kVtRow + pos) = hi;
  }
}

__global__ __launch_bounds__(kThreads, 2) void lite_attn_fwd_kernel(const FwdParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, hi = lane >> 5;

  // Consecutive workgroup ids land on different XCDs; give each XCD a contiguous range of rows so that the
  // workgroups sharing one L2 stream the K/V of the same head.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  if (slot >= p.rows_per_xcd) return;
  const int row = xcd * p.rows_per_xcd + slot;
  if (row >= p.rows_total) return;
  const int i = row % p.Tq;
  const int bh = row / p.Tq;
  const int64_t base = (int64_t)(bh / p.H) * p.stride_b + (int64_t)(bh % p.H) * p.stride_h;
  const uint16_t* qb = p.q + base;
  const uint16_t* kb = p.k + base;
  const uint16_t* vb = p.v + base;
  uint16_t* ob = p.out + base;
  const int N = p.N;
  const int cnt = (int)p.live_cnt[row];
  const uint16_t* live = p.live_idx + (size_t)row * p.Tk;
  int* flags = reinterpret_cast<int*>(smem + kFlagsOff);

  const int qrow = i * kTile + wave * 32 + lq;
  const bool qvalid = qrow < N;
  const bool q_pinned = p.protect_len > 0 && i * kTile < p.protect_start + p.protect_len &&
                        p.protect_start < min(N, (i + 1) * kTile);

  // Q^T fragments: B operand of S^T = K Q^T, kept for the whole row.
  bf16x8 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    uint4 raw = {0u, 0u, 0u, 0u};
    if (qvalid) raw = ld16(qb + (int64_t)qrow * p.stride_n + 16 * kk + 8 * hi);
    qf[kk] = *reinterpret_cast<bf16x8*>(&raw);
  }

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -INFINITY;  // running row max of the raw dot products (m_{i,j-1} * sqrt(d))
  float l_run = 0.f;        // this lane's half of the row sum
  float mloc_tile = -INFINITY;
  const float c = p.scale * 1.4426950408889634f;  // exp(x*scale) = exp2(x*c)
  unsigned newly = 0;

  const int nsub = 2 * cnt;
  StageRegs regs;
  if (nsub > 0) {
    load_stage(regs, kb, vb, p.stride_n, (int)live[0] * kTile, N, tid);
    store_stage(regs, smem, tid);
  }
  __syncthreads();

  for (int s = 0; s < nsub; ++s) {
    const int j = (int)live[s >> 1];
    const int half = s & 1;
    const int kv0 = j * kTile + half * kSub;
    char* stage = smem + (s & 1) * kStage;
    const bool more = (s + 1) < nsub;
    if (more) {
      const int jn = (int)live[(s + 1) >> 1];
      load_stage(regs, kb, vb, p.stride_n, jn * kTile + ((s + 1) & 1) * kSub, N, tid);
    }

    // ---- S^T = K Q^T for 64 K/V columns (raw dot products; the 1/sqrt(d) is folded into c) ----
    f32x16 sacc[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[blk][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(stage + (32 * blk + lq) * kKRow + 32 * kk + 16 * hi);
        sacc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], sacc[blk], 0, 0, 0);
      }
    }
    // columns past the end of the sequence do not exist: exclude them from max and sum
    if (kv0 + kSub > N) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int col = kv0 + 32 * blk + 8 * (r >> 2) + 4 * hi + (r & 3);
          if (col >= N) sacc[blk][r] = -INFINITY;
        }
    }

    // ---- online softmax: m_local, m_ij, P~ ----
    float mx = sacc[0][0];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[blk][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    mloc_tile = half ? fmaxf(mloc_tile, mx) : mx;
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
    const float mc = m_new * c;
    float lsum = 0.f;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pexp = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[blk][r], c, -mc));
        sacc[blk][r] = pexp;
        lsum += pexp;
      }
    l_run = l_run * alpha + lsum;
    if (__any(m_new > m_run)) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    m_run = m_new;

    // ---- skip predicate of the whole 128-column tile, once its second half is in ----
    if (half) {
      const float g = (mloc_tile - m_run) * p.scale;  // max over rows is the ballot below
      const bool ok = !qvalid || (g <= p.thr);
      const bool wave_all = __all(ok);
      if (lane == 0) flags[((s >> 1) & 1) * 4 + wave] = wave_all ? 1 : 0;
    }

    // ---- P~ in accumulator layout is the B operand of O^T += V^T P~^T ----
    bf16x8 pf[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      const int blk = cc >> 1, r0 = 8 * (cc & 1);
      uint4 raw;
      raw.x = pack_bf16x2(sacc[blk][r0 + 0], sacc[blk][r0 + 1]);
      raw.y = pack_bf16x2(sacc[blk][r0 + 2], sacc[blk][r0 + 3]);
      raw.z = pack_bf16x2(sacc[blk][r0 + 4], sacc[blk][r0 + 5]);
      raw.w = pack_bf16x2(sacc[blk][r0 + 6], sacc[blk][r0 + 7]);
      pf[cc] = *reinterpret_cast<bf16x8*>(&raw);
    }
    const char* sVt = stage + kKBytes;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(sVt + (32 * db + lq) * kVtRow + 32 * cc + 16 * hi);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[cc], oacc[db], 0, 0, 0);
      }

    if (more) store_stage(regs, smem + ((s + 1) & 1) * kStage, tid);
    __syncthreads();

    // ---- the four per-wave results of the finished tile meet here; one lane updates the mask ----
    if (half && tid == 0) {
      const int* f = flags + ((s >> 1) & 1) * 4;
      const bool k_pinned = p.protect_len > 0 && j * kTile < p.protect_start + p.protect_len &&
                            p.protect_start < min(N, (j + 1) * kTile);
      if ((f[0] & f[1] & f[2] & f[3]) && !q_pinned && !k_pinned) {
        atomicOr(reinterpret_cast<unsigned long long*>(p.bits + (size_t)row * p.W + (j >> 6)), 1ull << (j & 63));
        ++newly;
      }
    }
  }
  if (tid == 0 && newly) atomicAdd(p.stat_newly, (unsigned long long)newly);

  // ---- epilogue: O = acc / l, transposed through LDS so that global stores are 16 B and row-contiguous ----
  const float l = l_run + __shfl_xor(l_run, 32);
  const float inv = (l > 0.f) ? 1.f / l : 0.f;
  char* sO = smem;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      uint2 w;
      w.x = pack_bf16x2(oacc[db][4 * rg + 0] * inv, oacc[db][4 * rg + 1] * inv);
      w.y = pack_bf16x2(oacc[db][4 * rg + 2] * inv, oacc[db][4 * rg + 3] * inv);
      *reinterpret_cast<uint2*>(sO + (32 * wave + lq) * kORow + 2 * (32 * db + 8 * rg + 4 * hi)) = w;
    }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int r = (tid >> 4) + 16 * t;
    const int grow = i * kTile + r;
    if (grow < N)
      *reinterpret_cast<uint4*>(ob + (int64_t)grow * p.stride_n + 8 * (tid & 15)) =
          *reinterpret_cast<const uint4*>(sO + r * kORow + 16 * (tid & 15));
  }
}

int fwd_lds_bytes() { return kFlagsOff + 32; }

hipError_t launch_clear(uint64_t* bits, size_t words, unsigned long long* stats, size_t nstats, hipStream_t st) {
  size_t n = words > nstats ? words : nstats;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(clear_state_kernel, dim3(blocks), dim3(256), 0, st, bits, words, stats, nstats);
  return hipGetLastError();
}

hipError_t launch_compact(const uint64_t* bits, int rows, int Tk, int W, uint16_t* live_idx, uint32_t* live_cnt,
                          unsigned long long* stat_skipped_in, hipStream_t st) {
  hipLaunchKernelGGL(compact_skiplist, dim3((rows + 3) / 4), dim3(256), 0, st, bits, rows, Tk, W, live_idx, live_cnt,
                     stat_skipped_in);
  return hipGetLastError();
}

hipError_t prepare_fwd() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(lite_attn_fwd_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, fwd_lds_bytes());
}

hipError_t launch_fwd(const FwdParams& p, hipStream_t st) {
  const int grid = 8 * p.rows_per_xcd;
  hipLaunchKernelGGL(lite_attn_fwd_kernel, dim3(grid), dim3(kThreads), fwd_lds_bytes(), st, p);
  return hipGetLastError();
}

}  // namespace la
