// Internal interface between the C-ABI host code and the gfx950 kernels (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lite_attn.h"

namespace la {

// Rows of one head that an XCD runs side by side (2 workgroups x 32 CUs): the unit of the row schedule ("chunk").
constexpr int kChunkRows = 64;

struct FwdParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* vt;                    // V^T scratch: [B*H][128][128*Tk], written by launch_transpose_v
  uint16_t* out;
  int64_t stride_b, stride_h, stride_n;  // elements
  int H, N, Tq, Tk, W;                   // W = uint64 words per mask row
  uint32_t* runs;                        // [rows][run_stride] Skip-List: start | end << 16 per run of live tiles
  int run_stride;
  uint32_t* nruns;                       // [rows] runs per row
  uint32_t* live_cnt;                    // [rows] live tiles per row
  uint64_t* bits;                        // [rows][W]
  unsigned long long* stat_skipped_in;   // counters of the current step
  unsigned long long* stat_newly;
  unsigned long long* stat_runs;
  float thr;                             // signed threshold, natural-log units of S
  float scale;                           // 1/sqrt(d)
  int protect_start, protect_len;
  int rows_total;                        // B*H*Tq
  const uint32_t* slots;                 // [8][per_xcd]: the row (index into [B*H][Tq]) that workgroup `slot` of an
  int per_xcd;                           //   XCD computes, written by launch_deal_rows; entries >= xcd_rows[xcd] unused
  const uint32_t* xcd_rows;              // [8] rows dealt to each XCD
  // build_next != 0: the epilogue rewrites runs / nruns / live_cnt for the NEXT call from the mask this call leaves;
  // diagonal_first: visiting order of the lists
  int build_next, diagonal_first;
};

// Tile geometry of a layer, derived from its descriptor.
struct Geometry {
  int Tq, Tk, W;   // Q tiles, K/V tiles, uint64 words per Skip-Mask row
  int run_stride;  // capacity of one row's run-length Skip-List: floor(Tk/2) + 1 runs (ascending order needs at most
                   // ceil(Tk/2); diagonal first can split one more run at the wrap-around)
  int BH;          // batch * heads
  int64_t rows;    // BH * Tq
  int chunks;      // BH * ceil(Tq / kChunkRows): units of the row schedule
  int per_xcd;     // row slots per XCD in the schedule table: (ceil(chunks / 8) + 1) chunks
};

// Byte offsets of the Skip-List buffers inside one allocation (256-byte aligned pieces).  Handles keep them between
// calls (a call's epilogue leaves the next call's lists there); the handle-free entry point rebuilds them per call.
struct ListLayout {
  size_t stats;     // 3 uint64 counters for callers without a handle (handles keep per-step counters of their own)
  size_t nruns;     // [rows] uint32 runs per row
  size_t live_cnt;  // [rows] uint32 live tiles per row
  size_t order;     // [BH][Tq] uint32 row ranking
  size_t chunk_work;  // [chunks] uint32 work of each chunk (live tiles + a per-row constant)
  size_t slots;     // [8][per_xcd] uint32 schedule table
  size_t xcd_rows;  // [8] uint32
  size_t runs;      // [rows][run_stride] uint32 Skip-List
  size_t total;
};

// lite_attn_host.cpp (no HIP calls): argument checks shared by the entry points, geometry, scratch layout
int check_desc(const lite_attn_desc_t* d);  // LITE_ATTN_OK or the error the header documents
int check_call(const void* q, const void* k, const void* v, const void* out, float threshold);
Geometry geometry(const lite_attn_desc_t& d);
ListLayout list_layout(const Geometry& g);
size_t vt_bytes(const Geometry& g);  // V^T scratch of one call: [BH][128][128*Tk] bf16, rounded up to 256 bytes

// lite_attn.cpp: the launches of one attention call on `stream`.  lists_ready: the Skip-Lists in `lists` already
// describe the mask (left by the previous call's epilogue); otherwise the compaction kernel builds them first.  Then
// the row schedule, the V^T pre-pass into `vt` and the fused attention kernel, whose epilogue builds the next call's
// lists if build_next.  `mid` (may be null) is recorded just before the attention kernel.
// Allocates nothing.
hipError_t launch_call(const lite_attn_desc_t& d, const Geometry& g, const ListLayout& ll, char* lists, uint16_t* vt,
                       const void* q, const void* k, const void* v, void* out, uint64_t* bits,
                       unsigned long long* stats3, float threshold, bool lists_ready, bool build_next,
                       hipStream_t stream, hipEvent_t mid);
int hip_fail(hipError_t e);  // remembers e for lite_attn_last_hip_error() and maps it to a lite_attn_error

int fwd_lds_bytes();
hipError_t prepare_fwd();
hipError_t launch_clear(uint64_t* bits, size_t words, unsigned long long* stats, size_t nstats, hipStream_t st);
hipError_t launch_compact(const uint64_t* bits, int rows, int Tq, int Tk, int W, int diagonal_first, int run_stride,
                          uint32_t* runs, uint32_t* nruns, uint32_t* live_cnt, hipStream_t st);
hipError_t launch_transpose_v(const uint16_t* v, uint16_t* vt, int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              int BH, int H, int N, int Tk, hipStream_t st);
hipError_t launch_order_rows(const uint32_t* live_cnt, int BH, int Tq, int Tk, uint32_t* order, uint32_t* chunk_work,
                             hipStream_t st);
hipError_t launch_deal_rows(const uint32_t* chunk_work, const uint32_t* order, int BH, int Tq, int chunks, int per_xcd,
                            uint32_t* slots, uint32_t* xcd_rows, hipStream_t st);
hipError_t launch_fwd(const FwdParams& p, bool immediate, hipStream_t st);

}  // namespace la
