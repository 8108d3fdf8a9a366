// gfx950 (CDNA4) kernels of the LiteAttention forward path.
//
//   clear_state_kernel   : zero the Skip-Mask and the statistics (step 0)
//   compact_skiplist     : Skip-Mask row -> run-length list of its live K/V tiles, (start,end) per run
//                          (Implementation, "Producer and Skip-List Optimization"); only at the start of a trajectory
//                          or after a mask import: the fused kernel's epilogue builds the next call's Skip-Lists
//   order_rows_kernel    : per head, Q-tile rows ranked by Skip-List length (the launch order of the fused kernel)
//   transpose_v_kernel   : V -> V^T scratch, so that the PV operand is read from LDS like the QK operand
//   lite_attn_fwd_kernel : fused tiled forward over the live tiles with the skip predicate
//                          (Algorithm 2; eq. sparge_cond; tile recurrences of the Preliminaries)
//
// Fused kernel, one workgroup (4 wave64) = one Q tile = one Skip-Mask row:
//   * wave w owns Q rows [32w, 32w+32); lane l owns Q row (l & 31) of them.
//   * it works on S^T = K Q^T with v_mfma_f32_32x32x16_bf16: K rows are the A operand (LDS), Q rows the B
//     operand (registers, loaded once), so the 16 accumulator values a lane holds per 32x32 block all belong
//     to ONE Q row: row max / row sum are in-lane reductions plus one v_permlane32_swap, and exp(S^T) in
//     accumulator layout IS the B operand of O^T = V^T P^T -- P never moves between lanes.
//   * a 128-column mask tile is streamed as two 64-column stages.  K and V stages go global -> LDS with
//     buffer_load ... lds (no registers, rows past the end of the sequence arrive as zeros through the buffer
//     descriptor's range check); both are stored unpadded with an XOR swizzle applied on the global-address
//     side.  V is transposed once per call into a scratch (transpose_v_kernel), so that K and V^T fragments are
//     both plain 16-byte LDS reads.
//   * software pipeline: in stage s the matrix cores run S(s+1) = K(s+1) Q^T and O += V(s-1) P(s-1) while the
//     vector ALU runs the online softmax of stage s; LDS holds two K and two V stages (64 KB), one barrier per
//     stage, two workgroups per CU.
//   * the predicate of a tile is reduced per wave with a ballot; the four per-wave results meet through LDS
//     at the barrier that ends the tile and one lane ORs the bit into the global mask row.
//   * IMM variant (Algorithm 2 taken literally: a tile that fires contributes nothing in the step that marks it):
//     O += V(s-2) P(s-2) runs two stages behind instead of one, so that the verdict on a tile is known before the
//     first of its two PV products is issued; a fired tile's PV MFMAs and row sums are then dropped.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <stdint.h>

#include <utility>

#include "lite_attn_kernels.h"

namespace la {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define LA_LDS __attribute__((address_space(3)))

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ... : a loop whose index is a constant expression
template <int... Ks, class F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, Ks...>, F&& f) {
  (f(std::integral_constant<int, Ks>{}), ...);
}

constexpr int kTile = 128;        // Skip-Mask tile: 128 Q rows x 128 K/V columns
constexpr int kSub = 64;          // K/V columns per pipeline stage
constexpr int kStageBytes = kSub * 256;  // one K or V stage: 64 rows x 128 bf16, unpadded
constexpr int kKOff = 0;                 // K stage p at kKOff + p * kStageBytes
constexpr int kVOff = 2 * kStageBytes;   // V stage p at kVOff + p * kStageBytes
constexpr int kFlagsOff = 4 * kStageBytes;  // 8 ints [tile parity][wave] + 64 dummy ints
constexpr int kFiredOff = kFlagsOff + 8 * 4 + 64 * 4;  // W uint64: mask bits this workgroup set during the call
constexpr int kMaxMaskWords = 256;                     // ceil(16383 / 64)
constexpr int kLdsBytes = kFiredOff + 8 * kMaxMaskWords;
constexpr int kORow = 272;        // bytes per O row in the epilogue staging (reuses the stage buffers)

constexpr int kRowsPerWave = 8;  // Q-tile rows compacted by one wave of compact_skiplist

__global__ void clear_state_kernel(uint64_t* bits, size_t words, unsigned long long* stats, size_t nstats) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t x = i; x < words; x += stride) bits[x] = 0;
  for (size_t x = i; x < nstats; x += stride) stats[x] = 0;
}

// Skip-List of ONE Q-tile row, built by one wave (all 64 lanes call this).  The list is run-length encoded as the
// paper describes: one entry (start | end << 16) per maximal run of consecutive live K/V tiles [start, end), in
// visiting order (ascending, or -- "diagonal first" -- the tiles from the diagonal one to the last, then those before
// the diagonal; a row then has at most floor(Tk/2) + 1 runs).  Lane l looks at bit l of each 64-tile word: a live
// tile whose predecessor is not live starts a run, one whose successor is not live ends it; the k-th start and the
// k-th end of a row belong to the same run, so the two 16-bit halves are written independently at the position
// given by a ballot + prefix popcount.  `extra` (may be null, W words, any address space the caller's lambda reads):
// bits to be OR-ed into the mask row first.  Returns the number of runs in ns and of live tiles in n (same in every
// lane).
template <class ExtraBits>
__device__ __forceinline__ void compact_row(const uint64_t* __restrict__ mrow, ExtraBits extra, int i, int Tk, int W,
                                            int diagonal_first, uint32_t* __restrict__ row_runs, uint32_t& ns,
                                            uint32_t& n) {
  const int lane = threadIdx.x & 63;
  uint16_t* out = reinterpret_cast<uint16_t*>(row_runs);
  uint32_t ne = 0;
  ns = 0;
  n = 0;
  // runs of the live tiles inside [lo, hi), ascending, appended to the list
  auto emit = [&](int lo, int hi) {
    auto live_word = [&](int w) -> uint64_t {  // bit l set = tile 64w+l lies in [lo, hi) and is not skipped
      if (w < 0 || w >= W || 64 * w >= hi || 64 * w + 64 <= lo) return 0ull;
      uint64_t m = ~(mrow[w] | extra(w));
      if (hi - 64 * w < 64) m &= (1ull << (hi - 64 * w)) - 1ull;
      if (lo > 64 * w) m &= ~((1ull << (lo - 64 * w)) - 1ull);
      return m;
    };
    if (hi <= lo) return;
    uint64_t prev = 0ull, cur = live_word(lo >> 6);
    for (int w = lo >> 6; 64 * w < hi; ++w) {
      const uint64_t next = live_word(w + 1);
      const uint64_t starts = cur & ~((cur << 1) | (prev >> 63));
      const uint64_t ends = cur & ~((cur >> 1) | (next << 63));
      const uint64_t below = (1ull << lane) - 1ull;
      const int j = 64 * w + lane;
      if ((starts >> lane) & 1ull) out[2 * (ns + __popcll(starts & below))] = (uint16_t)j;
      if ((ends >> lane) & 1ull) out[2 * (ne + __popcll(ends & below)) + 1] = (uint16_t)(j + 1);
      ns += __popcll(starts);
      ne += __popcll(ends);
      n += __popcll(cur);
      prev = cur;
      cur = next;
    }
  };
  if (diagonal_first) {  // visiting order i, i+1, ..., Tk-1, 0, ..., i-1: the diagonal tile comes first
    const int d = min(i, Tk);
    emit(d, Tk);
    emit(0, d);
  } else {
    emit(0, Tk);
  }
}

// Skip-List compaction as a kernel of its own (the first call of a trajectory, and after the mask was imported;
// otherwise the fused kernel's epilogue has already built the lists of the next call): a wave takes kRowsPerWave
// consecutive rows (Implementation, "Producer and Skip-List Optimization").
__global__ __launch_bounds__(256) void compact_skiplist(const uint64_t* __restrict__ bits, int rows, int Tq, int Tk,
                                                         int W, int diagonal_first, int run_stride,
                                                         uint32_t* __restrict__ runs, uint32_t* __restrict__ nruns,
                                                         uint32_t* __restrict__ live_cnt) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  for (int row = wave * kRowsPerWave; row < min(rows, (wave + 1) * kRowsPerWave); ++row) {
    uint32_t ns, n;
    compact_row(bits + (size_t)row * W, [](int) { return 0ull; }, row % Tq, Tk, W, diagonal_first,
                runs + (size_t)row * run_stride, ns, n);
    if (lane == 0) {
      nruns[row] = ns;
      live_cnt[row] = n;
    }
  }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return *reinterpret_cast<uint32_t*>(&h);
}

__device__ __forceinline__ float other_half_max(float x) {
  // lanes l and l^32 exchange x; returns max(x, partner's x) in every lane
  const uint32_t u = __float_as_uint(x);
  const u32x2 sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

__device__ __forceinline__ float other_half_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  const u32x2 sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

// Row schedule, first half.  For every head, ranks its Q-tile rows by the length of their Skip-List, longest first
// (counting sort: one workgroup per head, histogram in LDS), and cuts the ranking into chunks of kChunkRows rows
// ("rank c" = rows ranked [c*kChunkRows, (c+1)*kChunkRows)).  The chunks of all heads are numbered rank-major,
// u = c * BH + (h + c) % BH; chunk_work[u] = the chunk's live tiles plus kRowOverhead per row (what a row costs
// besides its tiles, in tile times).
constexpr int kRowOverhead = 2;
__global__ __launch_bounds__(256) void order_rows_kernel(const uint32_t* __restrict__ live_cnt, int Tq, int Tk, int BH,
                                                          uint32_t* __restrict__ order,
                                                          uint32_t* __restrict__ chunk_work) {
  extern __shared__ uint32_t hist[];  // Tk + 1 bins; bin b counts rows with Tk - b live tiles; then one sum per chunk
  uint32_t* csum = hist + (Tk + 1);
  const int ranks = (Tq + kChunkRows - 1) / kChunkRows;
  const int bh = blockIdx.x, tid = threadIdx.x;
  const uint32_t* cnt = live_cnt + (size_t)bh * Tq;
  for (int b = tid; b <= Tk + ranks; b += 256) hist[b] = 0;
  __syncthreads();
  for (int i = tid; i < Tq; i += 256) atomicAdd(&hist[Tk - min((int)cnt[i], Tk)], 1u);
  __syncthreads();
  if (tid == 0) {  // exclusive prefix sum over at most 16384 bins
    uint32_t run = 0;
    for (int b = 0; b <= Tk; ++b) {
      const uint32_t c = hist[b];
      hist[b] = run;
      run += c;
    }
  }
  __syncthreads();
  for (int i = tid; i < Tq; i += 256) {
    const uint32_t live = (uint32_t)min((int)cnt[i], Tk);
    const uint32_t pos = atomicAdd(&hist[Tk - live], 1u);
    order[(size_t)bh * Tq + pos] = (uint32_t)i;
    atomicAdd(&csum[pos / kChunkRows], live + kRowOverhead);
  }
  __syncthreads();
  for (int c = tid; c < ranks; c += 256) chunk_work[(size_t)c * BH + (bh + c) % BH] = csum[c];
}

// Row schedule, second half: deals the chunks to the eight XCDs (workgroup id % 8) and writes the table the fused
// kernel reads its row from: slots[x * per_xcd + s] = row of the s-th workgroup of XCD x (0xffffffff: none; a chunk
// always occupies kChunkRows slots, so the chunks of a head's last rank leave some empty); xcd_rows[x] = slots in use.
// Chunks are taken in the order of u (longest ranks first; consecutive u of a rank belong to different heads), each
// going to the XCD with the least work so far among those holding fewer than per_xcd / kChunkRows chunks (the
// lowest-numbered one on a tie): every XCD ends up with the same work to within about one chunk, whatever the
// number of heads and however the sparsity differs between heads and ranks, and an XCD walks its chunks from long rows
// to short ones.  The workgroups sharing one L2 stream the K/V of the same head (a chunk stays together).
// The greedy pass is serial in the chunks (about 0.1 us each): wave 0 runs it with the state of XCD y in lane y --
// key = work << 3 | y, minimum over the eight lanes by three DPP steps -- for up to kDealMax chunks; with more chunks
// than that (64 per XCD) dealing them round-robin is balanced to within a percent or two and needs no pass at all.
// Every workgroup of this kernel repeats the pass (same inputs, same integers) and then fills its own share of the
// table.
constexpr int kDealMax = 512;
__device__ __forceinline__ uint32_t min_over_8_lanes(uint32_t key) {
  // lanes 8k..8k+7 all end up with the minimum of their eight keys
  key = min(key, (uint32_t)__builtin_amdgcn_update_dpp((int)key, (int)key, 0xB1, 0xf, 0xf, false));   // quad_perm 1,0,3,2
  key = min(key, (uint32_t)__builtin_amdgcn_update_dpp((int)key, (int)key, 0x4E, 0xf, 0xf, false));   // quad_perm 2,3,0,1
  key = min(key, (uint32_t)__builtin_amdgcn_update_dpp((int)key, (int)key, 0x141, 0xf, 0xf, false));  // row_half_mirror
  return key;
}

__global__ __launch_bounds__(256) void deal_rows_kernel(const uint32_t* __restrict__ chunk_work,
                                                         const uint32_t* __restrict__ order, int BH, int Tq,
                                                         int chunks, int per_xcd, uint32_t* __restrict__ slots,
                                                         uint32_t* __restrict__ xcd_rows) {
  __shared__ uint32_t work[kDealMax];  // work of chunk u
  __shared__ uint32_t dest[kDealMax];  // xcd << 29 | first slot of chunk u
  const int tid = threadIdx.x, lane = tid & 63;
  const int ranks = (Tq + kChunkRows - 1) / kChunkRows;
  const uint32_t cap = (uint32_t)(per_xcd / kChunkRows);
  const bool greedy = chunks <= kDealMax;
  if (greedy) {
    for (int u = tid; u < chunks; u += 256) work[u] = chunk_work[u];
    __syncthreads();
    if (tid < 64) {
      // a chunk's work is below 2^21 (64 rows of at most 16383 + kRowOverhead tiles), an XCD's below 2^27
      uint32_t load = 0, nch = 0, w = work[0];
      for (int u = 0; u < chunks; ++u) {
        const uint32_t w_next = work[min(u + 1, chunks - 1)];  // read ahead: keeps the LDS latency out of the chain
        const uint32_t key = (lane < 8 && nch < cap) ? (load << 3 | (uint32_t)lane) : 0xffffffffu;
        const int best = (int)(__builtin_amdgcn_readfirstlane(min_over_8_lanes(key)) & 7u);
        if (lane == best) {
          dest[u] = ((uint32_t)best << 29) | (nch * kChunkRows);
          load += w;
          nch += 1;
        }
        w = w_next;
      }
      if (blockIdx.x == 0 && lane < 8) xcd_rows[lane] = nch * kChunkRows;
    }
    __syncthreads();
  } else if (blockIdx.x == 0 && tid < 8) {  // round-robin: XCD x holds chunks x, x + 8, ...
    xcd_rows[tid] = (uint32_t)((chunks - tid + 7) / 8) * kChunkRows;
  }
  // the table: one entry per (head, position in its ranking padded to whole chunks)
  const long long padded = (long long)ranks * kChunkRows, total = (long long)BH * padded;
  const long long per_wg = (total + gridDim.x - 1) / gridDim.x;
  const long long lo = min(total, (long long)blockIdx.x * per_wg), hi = min(total, lo + per_wg);
  for (long long idx = lo + tid; idx < hi; idx += 256) {
    const int bh = (int)(idx / padded), pos = (int)(idx % padded);
    const int c = pos / kChunkRows, r = pos % kChunkRows;
    const int u = c * BH + (bh + c) % BH;
    const uint32_t d = greedy ? dest[u] : (((uint32_t)(u & 7) << 29) | (uint32_t)((u >> 3) * kChunkRows));
    const uint32_t s = (d & 0x1fffffffu) + (uint32_t)r;
    if (s < (uint32_t)per_xcd)
      slots[(size_t)(d >> 29) * per_xcd + s] = pos < Tq ? (uint32_t)bh * Tq + order[(size_t)bh * Tq + pos] : 0xffffffffu;
  }
}

// V -> V^T pre-pass.  The PV product contracts over the K/V index, so the matrix cores want, per lane, 8 V values
// of ONE feature d at 8 K/V positions: a 16-byte read from a [d][kv] layout, but a strided gather from V's [kv][d].
// (gfx950's transposing LDS read, ds_read_b64_tr_b16, delivers only 8 bytes per lane and measured at a third of the
// 16-byte read bandwidth, which made LDS the bound of the fused kernel.)  This kernel writes, once per call,
// vt[bh][d][n_pad] with n_pad = 128 * Tk, zero beyond the sequence, with the K/V index permuted inside every
// group of 16: position 8*h + t holds K/V offset 4*h + t + 4*(t >= 4) -- the order in which a lane of the fused
// kernel holds its P~ values.  One workgroup transposes one 128 x 128 tile through LDS.
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t* __restrict__ v, uint16_t* __restrict__ vt,
                                                           int64_t stride_b, int64_t stride_h, int64_t stride_n,
                                                           int H, int N, int Tk) {
  constexpr int kRow = 256 + 16;  // padded LDS row (bytes)
  __shared__ __attribute__((aligned(16))) char tile[128 * kRow];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = blockIdx.x % Tk, bh = blockIdx.x / Tk;
  const uint16_t* vb = v + (int64_t)(bh / H) * stride_b + (int64_t)(bh % H) * stride_h;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int r = (tid >> 4) + 16 * t, row = j * 128 + r;
    uint4 x = {0u, 0u, 0u, 0u};
    if (row < N) x = *reinterpret_cast<const uint4*>(vb + (int64_t)row * stride_n + 8 * (tid & 15));
    *reinterpret_cast<uint4*>(tile + r * kRow + 16 * (tid & 15)) = x;
  }
  __syncthreads();
  const int g = lane >> 4, i16 = lane & 15, r_src = i16 >> 2, c_src = lane & 3;
  uint16_t* out = vt + (int64_t)bh * 128 * (128 * (int64_t)Tk) + (int64_t)j * 128;
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    const int q = 8 * wave + x;                    // 32 (16-group, half, d-half) combinations per tile
    const int c16 = q >> 2, hh = (q >> 1) & 1, dhalf = q & 1;
    const char* src = tile + (16 * c16 + 4 * hh + r_src) * kRow + 2 * (64 * dhalf + 16 * g + 4 * c_src);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LA_LDS s16x4*)(src));
    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LA_LDS s16x4*)(src + 8 * kRow));
    const s16x8 o = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
    const int d = 64 * dhalf + 16 * g + i16;
    *reinterpret_cast<s16x8*>(out + (int64_t)d * (128 * (int64_t)Tk) + 16 * c16 + 8 * hh) = o;
  }
}

// Geometry of the fused kernel: a wave owns QB blocks of 32 Q rows, a workgroup (one Q tile of 128 rows) has 4/QB waves.
template <int QB>
struct Geo {
  static constexpr int kWaves = 4 / QB;
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kChunks = 16 / kWaves;  // 1 KB DMA pieces of a K (or V) stage per wave
};

// Per-lane constants of the fused kernel.
template <int QB>
struct Lane {
  u32x4 krsrc, vrsrc;  // buffer descriptors of this head's K (range-checked: rows past the end read as 0) and V^T
  uint32_t kdma[Geo<QB>::kChunks], vdma[Geo<QB>::kChunks];  // byte offsets (inside a stage) of this lane's DMA pieces
  uint32_t kread[8];  // LDS address of the K fragment for d-chunk kk in stage buffer 0 (stage and block: immediates)
  uint32_t vread[4];  // LDS address of the V^T fragment for column chunk cc in buffer 0 (d-block via immediates)
  uint32_t lds_wave;  // LDS address of this wave's first DMA piece inside stage buffer 0 (wave-uniform)
  uint32_t stride2;   // stride_n * 2 (bytes per token row)
  int hi;
  bool qvalid[QB];
  float c;            // scale * log2(e)
  float scale, thr;
  int N;
};

template <int QB, bool IMM>
struct State {
  bf16x8 qf[QB][8];
  f32x16 oacc[QB][4];
  f32x16 sA[QB][2], sB[QB][2];  // S^T of even / odd stages
  uint32_t pw[QB][16];          // P~^T of the previous stage, bf16 pairs; words 4cc..4cc+3 = B operand of chunk cc
                                // (IMM: of the previous odd stage)
  uint32_t pw0[QB][16];         // IMM only: P~^T of the previous even stage
  float m_run[QB], l_run[QB], mloc_tile[QB];
  // IMM only: row sum of the tile in flight (added to l_run once the tile is known not to have fired), and the
  // rescale factor of the previous stage, which O^T has not seen yet because its PV product runs a stage later
  float l_pend[QB], alpha_prev[QB];
  bool grew_prev;
};

// Buffer descriptor (V#) of a raw buffer of `bytes` bytes at `ptr`: loads at offsets >= bytes return zero.
__device__ __forceinline__ u32x4 make_rsrc(const void* ptr, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(ptr);
  u32x4 r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
  return r;
}

// Descriptor of the same buffer seen from `off` bytes in (wave-uniform, scalar arithmetic): base += off, size -= off
// (0 if off is past the end, so that every load through it returns zeros).  Folding the moving part of a DMA address
// into the descriptor leaves the per-lane offsets loop-invariant: no vector add per load.
__device__ __forceinline__ u32x4 rebase(const u32x4 r, uint32_t off) {
  off = __builtin_amdgcn_readfirstlane(off);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(r[0]), hi = __builtin_amdgcn_readfirstlane(r[1]);
  const uint32_t size = __builtin_amdgcn_readfirstlane(r[2]);
  // base += off (the high word holds only address bits here: stride and swizzle fields are zero); size =
  // max(size - off, 0).  Four scalar instructions; the compiler's own 64-bit add and saturating subtract take ten.
  uint32_t nlo, nhi, left;
  asm("s_add_u32 %0, %3, %5\n\ts_addc_u32 %1, %4, 0\n\ts_sub_u32 %2, %6, %5\n\ts_cselect_b32 %2, 0, %2"
      : "=&s"(nlo), "=&s"(nhi), "=&s"(left)
      : "s"(lo), "s"(hi), "s"(off), "s"(size)
      : "scc");
  u32x4 o = {nlo, nhi, left, (uint32_t)__builtin_amdgcn_readfirstlane(r[3])};
  return o;
}

// One 1 KB piece global -> LDS without registers: lane l's 16 bytes land at lds_addr + 16*l.  Written as inline
// assembly so that the compiler does not order later LDS reads of OTHER buffers behind this load (it would wait
// for vmcnt(0) before every LDS read); completion is enforced by the s_waitcnt vmcnt(0) + barrier ending a stage.
// (Issuing a stage's four pieces of K or V back to back with one M0 update -- their LDS offsets riding in the
// instruction offset -- was measured 3-6 % slower on the dense step: a burst of memory instructions holds up the
// MFMA behind it.)
// LDS address = lds_base (a wave-uniform register) + kLdsOff (a compile-time constant added on the scalar unit, so
// that the sixteen destinations of a stage pair do not each occupy a scalar register across the main loop).
template <int kLdsOff>
__device__ __forceinline__ void dma16(const u32x4 rsrc, uint32_t lds_base, uint32_t voffset) {
  asm volatile("s_add_u32 m0, %2, %3\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
               :
               : "v"(voffset), "s"(rsrc), "s"(lds_base), "n"(kLdsOff)
               : "memory", "m0", "scc");
}

template <int QB, int kBufOff, int X = 0>
__device__ __forceinline__ void dma_stage(const u32x4 rsrc, const uint32_t* off, uint32_t stage_byte_base,
                                          uint32_t lds_wave_addr) {
  if constexpr (X < Geo<QB>::kChunks) {
    dma16<kBufOff + 1024 * X>(rsrc, lds_wave_addr, off[X] + stage_byte_base);
    dma_stage<QB, kBufOff, X + 1>(rsrc, off, stage_byte_base, lds_wave_addr);
  }
}

// Piece x (compile-time after unrolling) of a stage: dispatch to the instance with that LDS offset.
template <int QB, int kBufOff>
__device__ __forceinline__ void dma_piece(int x, const u32x4 rsrc, const uint32_t* off, uint32_t stage_byte_base,
                                          uint32_t lds_wave_addr) {
  switch (x) {
    case 0: dma16<kBufOff + 0 * 1024>(rsrc, lds_wave_addr, off[0] + stage_byte_base); break;
    case 1: dma16<kBufOff + 1 * 1024>(rsrc, lds_wave_addr, off[1] + stage_byte_base); break;
    case 2: dma16<kBufOff + 2 * 1024>(rsrc, lds_wave_addr, off[2] + stage_byte_base); break;
    case 3: dma16<kBufOff + 3 * 1024>(rsrc, lds_wave_addr, off[3] + stage_byte_base); break;
    case 4: dma16<kBufOff + 4 * 1024>(rsrc, lds_wave_addr, off[4 % Geo<QB>::kChunks] + stage_byte_base); break;
    case 5: dma16<kBufOff + 5 * 1024>(rsrc, lds_wave_addr, off[5 % Geo<QB>::kChunks] + stage_byte_base); break;
    case 6: dma16<kBufOff + 6 * 1024>(rsrc, lds_wave_addr, off[6 % Geo<QB>::kChunks] + stage_byte_base); break;
    default: dma16<kBufOff + 7 * 1024>(rsrc, lds_wave_addr, off[7 % Geo<QB>::kChunks] + stage_byte_base); break;
  }
}

__device__ __forceinline__ bf16x8 p_operand(const uint32_t* w) {
  const u32x4 v = {w[0], w[1], w[2], w[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// S^T(next) = K Q^T for one 64-column stage held in LDS at byte offset sK (kread: absolute addresses in buffer 0).
template <int QB>
__device__ __forceinline__ void mma_qk(f32x16 (&nxt)[QB][2], const bf16x8 (&qf)[QB][8], int sK,
                                       const uint32_t (&kread)[8]) {
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) nxt[qb][blk][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const bf16x8 a = *reinterpret_cast<LA_LDS const bf16x8*>(kread[kk] + (uint32_t)(sK + 8192 * blk));
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        nxt[qb][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][kk], nxt[qb][blk], 0, 0, 0);
    }
  }
}

// O^T += V^T P~^T for one 64-column stage held in LDS at byte offset sV ([d][64 kv], 128-byte rows).
template <int QB>
__device__ __forceinline__ void mma_pv(f32x16 (&oacc)[QB][4], const uint32_t (&pw)[QB][16], int sV,
                                       const uint32_t (&vread)[4]) {
#pragma unroll
  for (int cc = 0; cc < 4; ++cc)
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const bf16x8 a = *reinterpret_cast<LA_LDS const bf16x8*>(vread[cc] + (uint32_t)(sV + 4096 * db));
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p_operand(&pw[qb][4 * cc]), oacc[qb][db], 0, 0, 0);
    }
}

// LDS -> register fragment k of a stage's matrix work: k < 16 is the V^T fragment (column chunk k/4, d-block k%4)
// of O^T += V^T P~^T, k >= 16 the K fragment (block (k-16)/8, d-chunk (k-16)%8) of S^T(s+1) = K Q^T.  Block 1 starts
// only at step 24, after the softmax has consumed block 1 of the current stage: its accumulators reuse those
// registers (alternating the two blocks was measured: no faster, six registers more).
// kread / vread hold absolute LDS addresses (of stage buffer 0), kK / kV are the byte offsets of the stage buffers
// read: every fragment address is one loop-invariant register plus an immediate.
// step k >= 16 of a stage multiplies d-chunk qk_kk(k) of K block qk_blk(k): block 0 first, then block 1
// (alternating the blocks, so that consecutive MFMAs share their Q fragment, measured 0.3 % faster for 4 more registers)
__device__ __forceinline__ constexpr int qk_blk(int k) { return (k - 16) >> 3; }
__device__ __forceinline__ constexpr int qk_kk(int k) { return k & 7; }

template <int kK, int kV>
__device__ __forceinline__ bf16x8 load_frag(int k, const uint32_t (&kread)[8], const uint32_t (&vread)[4]) {
  if (k >= 16) return *reinterpret_cast<LA_LDS const bf16x8*>(kread[qk_kk(k)] + (uint32_t)(kK + 8192 * qk_blk(k)));
  const int cc = k >> 2, db = k & 3;
  return *reinterpret_cast<LA_LDS const bf16x8*>(vread[cc] + (uint32_t)(kV + 4096 * db));
}

constexpr int kPrefetch = 3;  // LDS fragments in flight ahead of the MFMA that consumes them
constexpr int kDmaGap = 2;    // steps between two DMA issues of a stage

// One pipeline stage (64 K/V columns).  H = stage parity (half of the mask tile); j_tail = index of the ragged last
// tile of the sequence, whose columns past the end must be masked (-1 if the sequence ends on a tile boundary).
//
// The stage is written as 32 steps.  Step k issues the MFMA(s) of fragment k -- first the 16 of
// O^T += V^T(s-1) P~^T(s-1), then the 16 of S^T(s+1) -- and one slice of the online softmax of stage s (vector
// ALU), with scheduling fences between steps so that the compiler keeps this interleaving: the matrix cores and
// the vector ALU of the SIMD then work at the same time inside one wave.  P~ of stage s is written over P~ of
// stage s-1 word by word, each word after the last MFMA that reads it has been issued.
//
// IMM: the PV product of this stage is that of stage s-2 (same parity: its P~ and V^T buffers are those of parity
// H), issued only if pv_on (wave-uniform: the tile it belongs to did not fire); the V^T stage loaded here is that of
// stage s-1 (tile j_v, the other half), into the buffer of the other parity.
struct NoOp {
  __device__ __forceinline__ void operator()() const {}
};

// verdict_load / verdict_commit (first stage of a tile, deferred marking only): the combine of the PREVIOUS tile's four
// per-wave predicate results, spread over this stage -- its LDS read is issued at step 0 and used at step 12, so that
// the wave that does it never waits for it.
template <int QB, int H, bool IMM, class VLoad = NoOp, class VCommit = NoOp>
__device__ __forceinline__ void stage(State<QB, IMM>& st, const Lane<QB>& ln, char* smem, int j_cur, int j_nxt,
                                      int* flag_slot, int j_tail, int j_v = 0, bool pv_on = true,
                                      VLoad verdict_load = VLoad(), VCommit verdict_commit = VCommit()) {
  f32x16(&cur)[QB][2] = H ? st.sB : st.sA;
  f32x16(&nxt)[QB][2] = H ? st.sA : st.sB;
  uint32_t(&pwc)[QB][16] = (IMM && !H) ? st.pw0 : st.pw;

  // ---- DMA: K of stage s+2 (next tile, same half) and V of this stage go into the buffers of parity H; the
  // loads are issued one at a time between the steps below (kDmaGap steps apart) so that a full memory
  // instruction queue does not hold up the MFMAs behind it ----
  const u32x4 krs = rebase(ln.krsrc, (uint32_t)(j_nxt * kTile + H * kSub) * ln.stride2);
  const u32x4 vrs =
      rebase(ln.vrsrc, IMM ? (uint32_t)(j_v * kTile + (H ^ 1) * kSub) * 2u : (uint32_t)(j_cur * kTile + H * kSub) * 2u);
  constexpr int kVDst = kVOff + (IMM ? (H ^ 1) : H) * kStageBytes;  // V^T buffer the DMA of this stage fills
  constexpr int kC = Geo<QB>::kChunks;

  constexpr int kKSrc = kKOff + (H ^ 1) * kStageBytes;                // K stage read by S^T(s+1)
  constexpr int kVSrc = kVOff + (IMM ? H : (H ^ 1)) * kStageBytes;    // V^T stage read by the PV product
  bf16x8 frag[kPrefetch];
#pragma unroll
  for (int k = 0; k < kPrefetch; ++k)
    if (!IMM || pv_on) frag[k] = load_frag<kKSrc, kVSrc>(k, ln.kread, ln.vread);

  float pm[QB][4], mx[QB], m_new[QB], mc[QB], alpha[QB], lsum[QB], ta0[QB], ta1[QB], tb0[QB];
  bool ok = true, grew = false;
  // The ragged last tile of the sequence: its columns past the end leave the row maxima and sums (one scalar compare
  // and branch per stage, taken for one tile per row at most).  This lane's element r of block blk is column
  // 32*blk + 8*(r>>2) + (r&3) + 4*hi of the stage: the lane-independent part is compared with one per-lane limit.
  if (j_cur == j_tail) {
    int lim = ln.N - (j_cur * kTile + H * kSub) - 4 * ln.hi;
    asm volatile("" : "+v"(lim));  // keeps the compares inside this branch (else their lane masks are formed ahead of
                                   // time, for every stage, and held in scalar registers)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (32 * blk + 8 * (r >> 2) + (r & 3) >= lim) cur[qb][blk][r] = -INFINITY;
          asm volatile("" : "+v"(cur[qb][blk][r]));  // one lane mask alive at a time
        }
  }
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  auto mfma_part = [&](auto kc, auto qbc) __attribute__((always_inline)) {
    constexpr int k = decltype(kc)::value;  // the step index is a compile-time constant: every register index is static
    constexpr int qb = decltype(qbc)::value;
    // ---- matrix cores ----
    const bf16x8 a = frag[k % kPrefetch];
    if (k >= 16) {
      const int blk = qk_blk(k), kk = qk_kk(k);
      {
        if (kk == 0) {
          const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          nxt[qb][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.qf[qb][kk], zero, 0, 0, 0);
        } else {
          nxt[qb][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.qf[qb][kk], nxt[qb][blk], 0, 0, 0);
        }
      }
    } else {
      const int cc = k >> 2, db = k & 3;
      if (!IMM || pv_on)
        st.oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p_operand(&pwc[qb][4 * cc]), st.oacc[qb][db],
                                                                  0, 0, 0);
    }
  };
  auto mem_part = [&](auto kc) __attribute__((always_inline)) {
    constexpr int k = decltype(kc)::value;
    if (k + kPrefetch < 32) {
      if (!IMM || pv_on || k + kPrefetch >= 16)
        frag[k % kPrefetch] = load_frag<kKSrc, kVSrc>(k + kPrefetch, ln.kread, ln.vread);
    }
    if (k % kDmaGap == 0 && k / kDmaGap < 2 * kC) {
      const int x = k / kDmaGap;
      if (x < kC)
        dma_piece<QB, kVDst>(x, vrs, ln.vdma, 0u, ln.lds_wave);
      else
        dma_piece<QB, kKOff + H * kStageBytes>(x - kC, krs, ln.kdma, 0u, ln.lds_wave);
    }
    if (k == 0) verdict_load();
  };
  auto vector_part = [&](auto kc, auto qbc) __attribute__((always_inline)) {
    constexpr int k = decltype(kc)::value;
    constexpr int qb = decltype(qbc)::value;
    // ---- vector ALU: slice k of the online softmax of stage s (raw dot products; 1/sqrt(d) folded into c) ----
    {
      if (k < 4) {  // m_local: partial row maxima over 8 of this lane's 32 scores
        const int blk = k >> 1, r0 = 8 * (k & 1);
        float v = cur[qb][blk][r0];
#pragma unroll
        for (int r = r0 + 1; r < r0 + 8; ++r) v = fmaxf(v, cur[qb][blk][r]);
        pm[qb][k] = v;
      } else if (k == 4) {
        mx[qb] = other_half_max(fmaxf(fmaxf(pm[qb][0], pm[qb][1]), fmaxf(pm[qb][2], pm[qb][3])));
      } else if (k == 5) {  // m_ij = max(m_{i,j-1}, m_local) and the rescale factor of the earlier stages
        st.mloc_tile[qb] = H ? fmaxf(st.mloc_tile[qb], mx[qb]) : mx[qb];
        m_new[qb] = fmaxf(st.m_run[qb], mx[qb]);
        alpha[qb] = __builtin_amdgcn_exp2f((st.m_run[qb] - m_new[qb]) * ln.c);
        grew = grew || (m_new[qb] > st.m_run[qb]);
        st.m_run[qb] = m_new[qb];
        mc[qb] = m_new[qb] * ln.c;
        lsum[qb] = 0.f;
      } else if (k < 30) {
        // P~ = exp(S - m_ij), packed to bf16: 16 pairs of scores over 24 steps, four vector instructions per step
        // (a cycle of three steps does two pairs: exp exp | pack+sum, exp | exp, pack+sum)
        const int t = k - 6, c = t / 3, ph = t % 3;
        const int eA = 2 * c, eB = 2 * c + 1;
        if (ph == 0) {
          ta0[qb] = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[qb][eA >> 3][2 * (eA & 7)], ln.c, -mc[qb]));
          ta1[qb] = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[qb][eA >> 3][2 * (eA & 7) + 1], ln.c, -mc[qb]));
          // empty volatile asms pin every slice to its step: without them the compiler sinks all the exponentials
          // behind the last MFMA, where nothing overlaps them
          asm volatile("" : "+v"(ta0[qb]), "+v"(ta1[qb]));
        } else if (ph == 1) {
          uint32_t w = pack_bf16x2(ta0[qb], ta1[qb]);
          // the row sum adds the bf16-rounded weights, the same values the PV product uses
          lsum[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones, lsum[qb], false);
          tb0[qb] = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[qb][eB >> 3][2 * (eB & 7)], ln.c, -mc[qb]));
          asm volatile("" : "+v"(w), "+v"(lsum[qb]), "+v"(tb0[qb]));
          pwc[qb][eA] = w;  // word e belongs to chunk e/4, whose last reader was the MFMA of step 4*(e/4)+3 < k
        } else {
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[qb][eB >> 3][2 * (eB & 7) + 1], ln.c, -mc[qb]));
          uint32_t w = pack_bf16x2(tb0[qb], p1);
          lsum[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones, lsum[qb], false);
          asm volatile("" : "+v"(w), "+v"(lsum[qb]));
          pwc[qb][eB] = w;
        }
      } else if (k == 30) {
        if (IMM) {
          st.l_run[qb] *= alpha[qb];
          st.l_pend[qb] = H ? st.l_pend[qb] * alpha[qb] + lsum[qb] : lsum[qb];
        } else {
          st.l_run[qb] = st.l_run[qb] * alpha[qb] + lsum[qb];
        }
        if (H) {  // skip predicate of the whole 128-column tile, once its second half is in (eq. sparge_cond)
          const float g = (st.mloc_tile[qb] - m_new[qb]) * ln.scale;  // this row; max over rows = ballot below
          ok = ok && (!ln.qvalid[qb] || (g <= ln.thr));
        }
      }
    }
    if (H && k == 31 && qb == QB - 1)
      *flag_slot = __all(ok) ? 1 : 0;  // lane 0: the wave's slot; other lanes: a dummy word each
    if (k == 12 && qb == QB - 1) verdict_commit();
  };
  static_for(std::make_integer_sequence<int, 32>{}, [&](auto kc) __attribute__((always_inline)) {
    // matrix instruction and the memory instructions of the step first, then (fenced) the vector slice: measured
    // 1-1.5 % faster than leaving the order inside a step to the compiler (the memory instructions behind the vector
    // slice was the slowest order tried).  Issuing the MFMAs of 2, 4 or 8 steps back to back before their slices
    // (a coarser ping-pong between the two waves of a SIMD) was measured 0 / 2.5 / 6 % slower.
    static_for(std::make_integer_sequence<int, QB>{}, [&](auto qbc) __attribute__((always_inline)) {
      mfma_part(kc, qbc);
      if (decltype(qbc)::value == 0) mem_part(kc);
      __builtin_amdgcn_sched_barrier(0);
      vector_part(kc, qbc);
      __builtin_amdgcn_sched_barrier(0);
    });
  });
  // O^T of the earlier stages is rescaled after this stage's PV MFMAs (rare once the running max has settled).
  // IMM: O^T now holds the products up to stage s-2 and moves to the reference maximum of stage s-1, whose product
  // the next stage adds; this stage's own factor waits one stage.
  if (IMM ? st.grew_prev : (bool)__any(grew)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.oacc[qb][db][r] *= IMM ? st.alpha_prev[qb] : alpha[qb];
  }
  if (IMM) {
    st.grew_prev = __any(grew);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) st.alpha_prev[qb] = alpha[qb];
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

template <int QB, bool IMM>
__global__ __launch_bounds__(Geo<QB>::kThreads, 2 / QB) void lite_attn_fwd_kernel(const FwdParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int kWaves = Geo<QB>::kWaves, kThreads = Geo<QB>::kThreads, kChunks = Geo<QB>::kChunks;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31;

  // Consecutive workgroup ids land on different XCDs (id % 8): workgroup `slot` of an XCD computes the row that the
  // schedule table names for it (deal_rows_kernel: chunks of kChunkRows rows of one head side by side, so that the
  // workgroups sharing one L2 stream the same K/V; equal work per XCD; long rows first).
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  if (slot >= (int)p.xcd_rows[xcd]) return;
  const int row = (int)p.slots[(size_t)xcd * p.per_xcd + slot];
  if (row < 0) return;  // an empty slot behind a chunk shorter than kChunkRows
  const int i = row % p.Tq;
  const int bh = row / p.Tq;
  const int64_t base = (int64_t)(bh / p.H) * p.stride_b + (int64_t)(bh % p.H) * p.stride_h;
  const uint16_t* qb_ptr = p.q + base;
  uint16_t* ob = p.out + base;
  const int N = p.N;
  const int cnt = (int)p.live_cnt[row];
  // the Skip-List is read-only here: constant address space makes these wave-uniform reads scalar loads
  typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;
  const_u32_ptr runs = (const_u32_ptr)(p.runs + (size_t)row * p.run_stride);
  const int nruns = (int)p.nruns[row];
  int* flags = reinterpret_cast<int*>(smem + kFlagsOff);
  // mask bits set by this workgroup during the call (thread 0 writes them, wave 0 reads them in the epilogue)
  uint64_t* fired_bits = reinterpret_cast<uint64_t*>(smem + kFiredOff);
  if (p.build_next)
    for (int w = tid; w < p.W; w += kThreads) fired_bits[w] = 0;
  if (tid == 0) {  // statistics of the step: tiles skipped on entry, Skip-List entries read
    atomicAdd(p.stat_skipped_in, (unsigned long long)(p.Tk - cnt));
    atomicAdd(p.stat_runs, (unsigned long long)nruns);
  }

  Lane<QB> ln;
  ln.hi = lane >> 5;
  ln.N = N;
  ln.scale = p.scale;
  ln.thr = p.thr;
  ln.c = p.scale * 1.4426950408889634f;
  ln.stride2 = (uint32_t)(p.stride_n * 2);
  const uint32_t head_bytes = (uint32_t)(((int64_t)(N - 1) * p.stride_n + 128) * 2);
  ln.krsrc = make_rsrc(p.k + base, head_bytes);
  const uint32_t vt_row_bytes = (uint32_t)p.Tk * kTile * 2;  // one feature row of V^T: n_pad bf16
  ln.vrsrc = make_rsrc(p.vt + (size_t)bh * 128 * ((size_t)p.Tk * kTile), 128u * vt_row_bytes);
  ln.lds_wave = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(LA_LDS char*)smem + 1024 * kChunks * wave);
#pragma unroll
  for (int x = 0; x < kChunks; ++x) {
    const int r = 4 * (kChunks * wave + x) + (lane >> 4);  // row inside the stage that this lane's piece belongs to
    const int pc = lane & 15;                              // physical 16-byte chunk inside the 256-byte LDS row
    ln.kdma[x] = (uint32_t)r * ln.stride2 + 16 * (pc ^ (r & 15));
    // V^T stage: 128 feature rows x 128 bytes; this lane's piece is row rv, physical 16-byte slot pv
    const int rv = 8 * (kChunks * wave + x) + (lane >> 3), pv = lane & 7;
    ln.vdma[x] = (uint32_t)rv * vt_row_bytes + 16 * (pv ^ ((rv >> 1) & 7));
  }
  const uint32_t lds0 = (uint32_t)(size_t)(LA_LDS char*)smem;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) ln.kread[kk] = lds0 + lq * 256 + ((32 * kk) ^ (16 * (ln.hi ^ (lq & 15))));
#pragma unroll
  for (int cc = 0; cc < 4; ++cc) ln.vread[cc] = lds0 + lq * 128 + ((32 * cc + 16 * ln.hi) ^ (16 * ((lq >> 1) & 7)));
  const bool q_pinned = p.protect_len > 0 && i * kTile < p.protect_start + p.protect_len &&
                        p.protect_start < min(N, (i + 1) * kTile);

  State<QB, IMM> st;
  st.grew_prev = false;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    st.l_pend[qb] = 0.f;
    st.alpha_prev[qb] = 1.f;
    const int qrow = i * kTile + 32 * (QB * wave + qb) + lq;
    ln.qvalid[qb] = qrow < N;
    // Q^T fragments: B operand of S^T = K Q^T, kept for the whole row.
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      uint4 raw = {0u, 0u, 0u, 0u};
      if (ln.qvalid[qb])
        raw = *reinterpret_cast<const uint4*>(qb_ptr + (int64_t)qrow * p.stride_n + 16 * kk + 8 * ln.hi);
      st.qf[qb][kk] = *reinterpret_cast<bf16x8*>(&raw);
    }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.oacc[qb][db][r] = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) st.pw[qb][e] = 0u;
    st.m_run[qb] = -INFINITY;  // running row max of the raw dot products (m_{i,j-1} * sqrt(d))
    st.l_run[qb] = 0.f;        // this lane's half of the row sum
    st.mloc_tile[qb] = -INFINITY;
  }
  unsigned newly = 0;

  // lane 0 writes the wave's predicate flag, every other lane a private dummy word (keeps the stage branch-free)
  int* flag_slot0 = lane == 0 ? flags + wave : flags + 8 + lane;
  int* flag_slot1 = lane == 0 ? flags + 4 + wave : flags + 8 + lane;

  if (cnt > 0) {
    // Walk the run-length Skip-List with a cursor kept two tiles ahead of the tile being computed, so that the
    // scalar load of the next run entry is off the critical path.  At the end of the list the cursor stays put.
    int c_run = 0, c_j, c_end;
    {
      const uint32_t e = runs[0];
      c_j = (int)(e & 0xffffu);
      c_end = (int)(e >> 16);
    }
    auto advance = [&]() {
      if (c_j + 1 < c_end) {
        ++c_j;
      } else if (c_run + 1 < nruns) {
        ++c_run;
        const uint32_t e = runs[c_run];
        c_j = (int)(e & 0xffffu);
        c_end = (int)(e >> 16);
      }
    };
    int j_cur = c_j;
    advance();
    int j_nxt = c_j;
    // the last tile of a sequence that ends inside it needs its columns masked; the stages compare their tile index
    // with this one on the scalar unit (a bool would travel between their blocks as a lane mask)
    const int j_tail = (N & (kTile - 1)) != 0 ? p.Tk - 1 : -1;

    // prologue: the odd V^T buffer is read (times P~ = 0) before it is first filled: make it finite; K of
    // stages 0 and 1; then S^T(0)
    if (!IMM)
      for (int x = tid; x < kStageBytes / 16; x += kThreads)
        *reinterpret_cast<uint4*>(smem + kVOff + kStageBytes + 16 * x) = uint4{0u, 0u, 0u, 0u};
    dma_stage<QB, kKOff>(ln.krsrc, ln.kdma, (uint32_t)(j_cur * kTile) * ln.stride2, ln.lds_wave);
    dma_stage<QB, kKOff + kStageBytes>(ln.krsrc, ln.kdma, (uint32_t)(j_cur * kTile + kSub) * ln.stride2, ln.lds_wave);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    mma_qk<QB>(st.sA, st.qf, kKOff, ln.kread);
    __syncthreads();

    // IMM: every wave reads the four per-wave results and the pinned-range rule itself (it needs the verdict to
    // gate the tile's PV products); returns whether the tile fired (wave-uniform)
    auto finish_tile_imm = [&](int t, int j) -> bool {
      const int4 f = *reinterpret_cast<const int4*>(flags + (t & 1) * 4);
      static_assert(!IMM || kWaves == 4, "four per-wave flags per tile");
      const int all = __builtin_amdgcn_readfirstlane(f.x & f.y & f.z & f.w);
      const bool k_pinned = p.protect_len > 0 && j * kTile < p.protect_start + p.protect_len &&
                            p.protect_start < min(N, (j + 1) * kTile);
      const bool fired = all && !q_pinned && !k_pinned;
      if (tid == 0 && fired) {
        atomicOr(reinterpret_cast<unsigned long long*>(p.bits + (size_t)row * p.W + (j >> 6)), 1ull << (j & 63));
        fired_bits[j >> 6] |= 1ull << (j & 63);
        ++newly;
      }
      return fired;
    };
    // Deferred marking: the per-wave results of a finished tile meet in LDS; wave 0 combines them and updates the
    // mask, not at the barrier that ends the tile (it would be late for the next stage by the latency of an LDS read,
    // and the other three waves would wait for it at the next barrier) but during the first stage of the next tile.
    const bool wave0 = __builtin_amdgcn_readfirstlane(wave) == 0;
    int4 vflags = {0, 0, 0, 0};
    const int* v_slot = flags;  // LDS slot of the tile whose verdict is pending
    int v_j = -1;               // its K/V tile index (-1: none pending)
    auto mark_if_fired = [&](int all, int j) {
      if (tid == 0 && all) {
        const bool k_pinned = p.protect_len > 0 && j * kTile < p.protect_start + p.protect_len &&
                              p.protect_start < min(N, (j + 1) * kTile);
        if (!q_pinned && !k_pinned) {
          atomicOr(reinterpret_cast<unsigned long long*>(p.bits + (size_t)row * p.W + (j >> 6)), 1ull << (j & 63));
          fired_bits[j >> 6] |= 1ull << (j & 63);
          ++newly;
        }
      }
    };
    auto verdict_load = [&]() {
      static_assert(IMM || kWaves == 4, "four per-wave flags per tile");
      if (wave0) vflags = *reinterpret_cast<const int4*>(v_slot);
    };
    auto verdict_commit = [&]() {
      if (wave0 && v_j >= 0) mark_if_fired(vflags.x & vflags.y & vflags.z & vflags.w, v_j);
    };
    bool pv_on = false;  // IMM: the previous tile did not fire, its PV products are due
    int j_prev = j_cur;
    for (int t = 0; t < cnt; ++t) {
      advance();
      const int j_nn = c_j;  // needed one tile from now
      int* fs = (t & 1) ? flag_slot1 : flag_slot0;
      if constexpr (IMM) {
        stage<QB, 0, true>(st, ln, smem, j_cur, j_nxt, fs, j_tail, j_prev, pv_on);
        stage<QB, 1, true>(st, ln, smem, j_cur, j_nxt, fs, j_tail, j_cur, pv_on);
        pv_on = !finish_tile_imm(t, j_cur);
        if (pv_on) {
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) st.l_run[qb] += st.l_pend[qb];
        }
        j_prev = j_cur;
      } else {
        stage<QB, 0, false>(st, ln, smem, j_cur, j_nxt, fs, j_tail, 0, true, verdict_load, verdict_commit);
        stage<QB, 1, false>(st, ln, smem, j_cur, j_nxt, fs, j_tail);
        v_slot = flags + (t & 1) * 4;
        v_j = j_cur;
      }
      j_cur = j_nxt;
      j_nxt = j_nn;
    }
    if constexpr (IMM) {
      // drain: the second V^T stage of the last tile is still to be loaded; then both of its PV products, the
      // rescale factor of its second stage in between
      dma_stage<QB, kVOff + kStageBytes>(ln.vrsrc, ln.vdma, (uint32_t)(j_prev * kTile + kSub) * 2u, ln.lds_wave);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (pv_on) mma_pv<QB>(st.oacc, st.pw0, kVOff, ln.vread);
      if (st.grew_prev) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.oacc[qb][db][r] *= st.alpha_prev[qb];
      }
      if (pv_on) mma_pv<QB>(st.oacc, st.pw, kVOff + kStageBytes, ln.vread);
    } else {
      // drain: O^T += V^T P~^T of the last stage (odd parity buffer), and the verdict on the last tile
      mma_pv<QB>(st.oacc, st.pw, kVOff + kStageBytes, ln.vread);
      verdict_load();
      verdict_commit();
    }
    __syncthreads();
  }
  if (tid == 0 && newly) atomicAdd(p.stat_newly, (unsigned long long)newly);

  // ---- epilogue: O = acc / l, transposed through LDS so that global stores are 16 B and row-contiguous ----
  char* sO = smem;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l = other_half_sum(st.l_run[qb]);
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        uint2 w;
        w.x = pack_bf16x2(st.oacc[qb][db][4 * rg + 0] * inv, st.oacc[qb][db][4 * rg + 1] * inv);
        w.y = pack_bf16x2(st.oacc[qb][db][4 * rg + 2] * inv, st.oacc[qb][db][4 * rg + 3] * inv);
        *reinterpret_cast<uint2*>(sO + (32 * (QB * wave + qb) + lq) * kORow + 2 * (32 * db + 8 * rg + 4 * ln.hi)) = w;
      }
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 2048 / kThreads; ++t) {
    const int r = (tid >> 4) + (kThreads / 16) * t;
    const int grow = i * kTile + r;
    if (grow < N)
      *reinterpret_cast<uint4*>(ob + (int64_t)grow * p.stride_n + 8 * (tid & 15)) =
          *reinterpret_cast<const uint4*>(sO + r * kORow + 16 * (tid & 15));
  }

  // ---- second epilogue: the Skip-List this row will walk in the NEXT call, compacted from the mask row as this call
  // leaves it: the row as it was on entry (nobody else writes it) OR the bits this workgroup set, which it kept in
  // LDS, so that nothing depends on when its own atomics become visible to its loads.  The row's list is private to
  // this workgroup: it is overwritten in place, after its last read.  (The kernel arguments used here are read
  // again from the argument segment instead of being kept in scalar registers across the main loop.) ----
  typedef const __attribute__((address_space(4))) FwdParams* const_params_ptr;
  const_params_ptr e = (const_params_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(e));
  if (e->build_next && wave == 0) {
    uint32_t ns, n;
    compact_row(e->bits + (size_t)row * e->W, [&](int w) { return fired_bits[w]; }, i, e->Tk, e->W, e->diagonal_first,
                e->runs + (size_t)row * e->run_stride, ns, n);
    if (lane == 0) {
      e->nruns[row] = ns;
      e->live_cnt[row] = n;
    }
  }
}

int fwd_lds_bytes() { return kLdsBytes; }

hipError_t launch_clear(uint64_t* bits, size_t words, unsigned long long* stats, size_t nstats, hipStream_t st) {
  size_t n = words > nstats ? words : nstats;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(clear_state_kernel, dim3(blocks), dim3(256), 0, st, bits, words, stats, nstats);
  return hipGetLastError();
}

hipError_t launch_compact(const uint64_t* bits, int rows, int Tq, int Tk, int W, int diagonal_first, int run_stride,
                          uint32_t* runs, uint32_t* nruns, uint32_t* live_cnt, hipStream_t st) {
  hipLaunchKernelGGL(compact_skiplist, dim3((rows + 4 * kRowsPerWave - 1) / (4 * kRowsPerWave)), dim3(256), 0, st, bits,
                     rows, Tq, Tk, W, diagonal_first, run_stride, runs, nruns, live_cnt);
  return hipGetLastError();
}

hipError_t launch_transpose_v(const uint16_t* v, uint16_t* vt, int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              int BH, int H, int N, int Tk, hipStream_t st) {
  hipLaunchKernelGGL(transpose_v_kernel, dim3((unsigned)(BH * Tk)), dim3(256), 0, st, v, vt, stride_b, stride_h,
                     stride_n, H, N, Tk);
  return hipGetLastError();
}

constexpr int kQB = 1;  // 32 Q rows per wave, 4 waves per workgroup, 2 workgroups per CU

// LDS of order_rows_kernel: Tk + 1 bins and one sum per chunk of a head (more than 64 KB for the longest sequences)
static size_t order_lds_bytes(int Tq, int Tk) {
  return sizeof(uint32_t) * ((size_t)(Tk + 1) + (size_t)((Tq + kChunkRows - 1) / kChunkRows));
}

hipError_t prepare_fwd() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(lite_attn_fwd_kernel<kQB, false>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, fwd_lds_bytes());
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(lite_attn_fwd_kernel<1, true>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, fwd_lds_bytes());
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(order_rows_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)order_lds_bytes(16383, 16383));
}

hipError_t launch_order_rows(const uint32_t* live_cnt, int BH, int Tq, int Tk, uint32_t* order, uint32_t* chunk_work,
                             hipStream_t st) {
  hipLaunchKernelGGL(order_rows_kernel, dim3(BH), dim3(256), order_lds_bytes(Tq, Tk), st, live_cnt, Tq, Tk, BH, order,
                     chunk_work);
  return hipGetLastError();
}

hipError_t launch_deal_rows(const uint32_t* chunk_work, const uint32_t* order, int BH, int Tq, int chunks, int per_xcd,
                            uint32_t* slots, uint32_t* xcd_rows, hipStream_t st) {
  // every workgroup repeats the dealing and fills its share of the table: enough of them to keep the filling short
  const long long rows = (long long)BH * Tq;
  const int grid = (int)std::min<long long>(32, std::max<long long>(1, rows / 1024));
  hipLaunchKernelGGL(deal_rows_kernel, dim3(grid), dim3(256), 0, st, chunk_work, order, BH, Tq, chunks, per_xcd, slots,
                     xcd_rows);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdParams& p, bool immediate, hipStream_t st) {
  // one workgroup per slot of the schedule table; those past an XCD's last row return at once
  if (immediate)
    hipLaunchKernelGGL((lite_attn_fwd_kernel<1, true>), dim3(8 * p.per_xcd), dim3(Geo<1>::kThreads), fwd_lds_bytes(),
                       st, p);
  else
    hipLaunchKernelGGL((lite_attn_fwd_kernel<kQB, false>), dim3(8 * p.per_xcd), dim3(Geo<kQB>::kThreads),
                       fwd_lds_bytes(), st, p);
  return hipGetLastError();
}

}  // namespace la
