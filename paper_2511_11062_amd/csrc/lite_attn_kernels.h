// Internal interface between the C-ABI host code and the gfx950 kernels (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace la {

struct FwdParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* vt;                    // V^T scratch: [B*H][128][128*Tk], written by launch_transpose_v
  uint16_t* out;
  int64_t stride_b, stride_h, stride_n;  // elements
  int H, N, Tq, Tk, W;                   // W = uint64 words per mask row
  const uint32_t* runs;                  // [rows][run_stride] Skip-List: start | end << 16 per run of live tiles
  int run_stride;
  const uint32_t* nruns;                 // [rows] runs per row
  const uint32_t* live_cnt;              // [rows] live tiles per row
  uint64_t* bits;                        // [rows][W]
  unsigned long long* stat_newly;        // counter of the current step
  float thr;                             // signed threshold, natural-log units of S
  float scale;                           // 1/sqrt(d)
  int protect_start, protect_len;
  int rows_total;                        // B*H*Tq
  const uint32_t* order;                 // [B*H][Tq]: Q tiles of each head ranked by Skip-List length, longest first
};

int fwd_lds_bytes();
hipError_t prepare_fwd();
hipError_t launch_clear(uint64_t* bits, size_t words, unsigned long long* stats, size_t nstats, hipStream_t st);
hipError_t launch_compact(const uint64_t* bits, int rows, int Tq, int Tk, int W, int diagonal_first, int run_stride,
                          uint32_t* runs, uint32_t* nruns, uint32_t* live_cnt, unsigned long long* stat_skipped_in,
                          unsigned long long* stat_runs, hipStream_t st);
hipError_t launch_transpose_v(const uint16_t* v, uint16_t* vt, int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              int BH, int H, int N, int Tk, hipStream_t st);
hipError_t launch_mfma_peak(const void* data, float* sink, int iters, int blocks, hipStream_t st);
hipError_t launch_order_rows(const uint32_t* live_cnt, int BH, int Tq, int Tk, uint32_t* order, hipStream_t st);
hipError_t launch_fwd(const FwdParams& p, bool immediate, hipStream_t st);

}  // namespace la
