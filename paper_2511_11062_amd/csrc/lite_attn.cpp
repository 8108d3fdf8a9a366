// Host side of the C ABI declared in include/lite_attn.h: handle, argument checks, launches.
#include "lite_attn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <new>

#include "lite_attn_kernels.h"

struct lite_attn_mask {
  lite_attn_desc_t desc;
  int Tq, Tk, W;
  int run_stride;   // capacity of one row's run-length Skip-List: Tk/2 + 1 runs (ascending order: at most
                    // ceil(Tk/2); diagonal first: the wrap at the last tile can split one more, floor(Tk/2) + 1)
  int64_t rows;
  uint64_t* d_bits;
  uint32_t* d_runs;   // [rows][run_stride] start | end << 16
  uint32_t* d_nruns;  // [rows]
  uint32_t* d_live_cnt;
  uint32_t* d_order;  // [B*H][Tq] rows of each head ranked by Skip-List length
  uint16_t* d_vt;  // V^T scratch of the current call: [B*H][128][128*Tk] bf16
  unsigned long long* d_stats;  // [max_steps][3]: skipped on entry, newly marked, Skip-List runs
  hipStream_t stream;
  int next_step;
  bool profile;
  hipEvent_t* events;  // [max_steps][3] once profiling was enabled: before the pre-passes, between, after attention
  bool* timed;         // [max_steps]
};

namespace {

thread_local int g_last_hip = 0;

int hip_fail(hipError_t e) {
  g_last_hip = (int)e;
  return e == hipErrorOutOfMemory ? LITE_ATTN_ENOMEM : LITE_ATTN_EHIP;
}

#define LA_HIP(expr)                        \
  do {                                      \
    hipError_t e_ = (expr);                 \
    if (e_ != hipSuccess) return hip_fail(e_); \
  } while (0)

int check_desc(const lite_attn_desc_t* d) {
  if (!d) return LITE_ATTN_EINVAL;
  if (d->batch < 1 || d->heads < 1 || d->seqlen < 1 || d->head_dim < 1 || d->tile_q < 1 || d->tile_k < 1)
    return LITE_ATTN_EINVAL;
  if (d->max_steps < 1) return LITE_ATTN_EINVAL;
  if ((d->flags & ~(LITE_ATTN_ORDER_DIAGONAL_FIRST | LITE_ATTN_PV_SKIP_IMMEDIATE)) != 0) return LITE_ATTN_EINVAL;
  if (d->protect_len < 0 || d->protect_start < 0 ||
      (d->protect_len > 0 && (int64_t)d->protect_start + d->protect_len > d->seqlen))
    return LITE_ATTN_EINVAL;
  // 16-byte vector accesses: every stride must be a multiple of 8 bf16 elements
  if (d->stride_n < d->head_dim || d->stride_b < 0 || d->stride_h < 0) return LITE_ATTN_EINVAL;
  if ((d->stride_n % 8) || (d->stride_b % 8) || (d->stride_h % 8)) return LITE_ATTN_EINVAL;
  if (d->batch > 1 && d->stride_b == 0) return LITE_ATTN_EINVAL;
  if (d->heads > 1 && d->stride_h == 0) return LITE_ATTN_EINVAL;
  if (d->head_dim != 128 || d->tile_q != 128 || d->tile_k != 128) return LITE_ATTN_EUNSUPPORTED;
  const int64_t Tk = ((int64_t)d->seqlen + 127) / 128;
  if (Tk > 16383) return LITE_ATTN_EUNSUPPORTED;  // row-schedule histogram (Tk + 1 bins) lives in 64 KB of LDS
  // K/V stages are addressed with 32-bit byte offsets from the head's base pointer
  if (((int64_t)d->seqlen + 128) * d->stride_n * 2 >= ((int64_t)1 << 32)) return LITE_ATTN_EUNSUPPORTED;
  const int64_t rows = (int64_t)d->batch * d->heads * Tk;
  if (rows > (int64_t)1 << 30) return LITE_ATTN_EUNSUPPORTED;
  return LITE_ATTN_OK;
}

}  // namespace

extern "C" {

int lite_attn_init_mask(const lite_attn_desc_t* desc, lite_attn_mask_t** out) {
  if (!out) return LITE_ATTN_EINVAL;
  int rc = check_desc(desc);
  if (rc != LITE_ATTN_OK) return rc;
  lite_attn_mask* m = new (std::nothrow) lite_attn_mask();
  if (!m) return LITE_ATTN_ENOMEM;
  m->desc = *desc;
  m->Tq = (desc->seqlen + desc->tile_q - 1) / desc->tile_q;
  m->Tk = (desc->seqlen + desc->tile_k - 1) / desc->tile_k;
  m->W = (m->Tk + 63) / 64;
  m->run_stride = m->Tk / 2 + 1;
  m->rows = (int64_t)desc->batch * desc->heads * m->Tq;
  m->stream = nullptr;
  m->next_step = 0;
  m->profile = false;
  m->events = nullptr;
  m->timed = nullptr;
  m->d_bits = nullptr; m->d_runs = nullptr; m->d_nruns = nullptr; m->d_live_cnt = nullptr;
  m->d_stats = nullptr; m->d_vt = nullptr; m->d_order = nullptr;
  hipError_t e = hipMalloc(&m->d_bits, sizeof(uint64_t) * (size_t)m->rows * m->W);
  if (e == hipSuccess) e = hipMalloc(&m->d_runs, sizeof(uint32_t) * (size_t)m->rows * m->run_stride);
  if (e == hipSuccess) e = hipMalloc(&m->d_nruns, sizeof(uint32_t) * (size_t)m->rows);
  if (e == hipSuccess) e = hipMalloc(&m->d_live_cnt, sizeof(uint32_t) * (size_t)m->rows);
  if (e == hipSuccess) e = hipMalloc(&m->d_order, sizeof(uint32_t) * (size_t)m->rows);
  if (e == hipSuccess)
    e = hipMalloc(&m->d_vt, sizeof(uint16_t) * (size_t)desc->batch * desc->heads * 128 * ((size_t)m->Tk * 128));
  if (e == hipSuccess) e = hipMalloc(&m->d_stats, sizeof(unsigned long long) * 3 * (size_t)desc->max_steps);
  if (e == hipSuccess) e = la::prepare_fwd();
  if (e == hipSuccess)
    e = la::launch_clear(m->d_bits, (size_t)m->rows * m->W, m->d_stats, 3 * (size_t)desc->max_steps, m->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
  if (e != hipSuccess) {
    lite_attn_free_mask(m);
    return hip_fail(e);
  }
  *out = m;
  return LITE_ATTN_OK;
}

int lite_attn_set_stream(lite_attn_mask_t* m, void* hip_stream) {
  if (!m) return LITE_ATTN_EINVAL;
  LA_HIP(hipStreamSynchronize(m->stream));  // work already queued keeps its order with what follows
  m->stream = reinterpret_cast<hipStream_t>(hip_stream);
  return LITE_ATTN_OK;
}

int lite_attn_fwd(const void* q, const void* k, const void* v, void* out, lite_attn_mask_t* m, float threshold,
                  int step) {
  if (!q || !k || !v || !out || !m) return LITE_ATTN_EINVAL;
  if (std::isnan(threshold) || threshold >= 0.f) return LITE_ATTN_EINVAL;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) return LITE_ATTN_EINVAL;
  if (step < 0 || step >= m->desc.max_steps) return LITE_ATTN_ESTEP;
  if (step != 0 && step != m->next_step) return LITE_ATTN_ESTEP;
  const lite_attn_desc_t& d = m->desc;
  if (step == 0)
    LA_HIP(la::launch_clear(m->d_bits, (size_t)m->rows * m->W, m->d_stats, 3 * (size_t)d.max_steps, m->stream));
  unsigned long long* st = m->d_stats + 3 * (size_t)step;
  hipEvent_t* ev = (m->profile && m->events) ? m->events + 3 * (size_t)step : nullptr;
  if (m->timed) m->timed[step] = ev != nullptr;
  if (ev) LA_HIP(hipEventRecord(ev[0], m->stream));
  LA_HIP(la::launch_compact(m->d_bits, (int)m->rows, m->Tq, m->Tk, m->W, d.flags & LITE_ATTN_ORDER_DIAGONAL_FIRST,
                            m->run_stride, m->d_runs, m->d_nruns, m->d_live_cnt, st, st + 2, m->stream));
  LA_HIP(la::launch_order_rows(m->d_live_cnt, d.batch * d.heads, m->Tq, m->Tk, m->d_order, m->stream));
  LA_HIP(la::launch_transpose_v(static_cast<const uint16_t*>(v), m->d_vt, d.stride_b, d.stride_h, d.stride_n,
                                d.batch * d.heads, d.heads, d.seqlen, m->Tk, m->stream));
  la::FwdParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.vt = m->d_vt;
  p.out = static_cast<uint16_t*>(out);
  p.stride_b = d.stride_b; p.stride_h = d.stride_h; p.stride_n = d.stride_n;
  p.H = d.heads; p.N = d.seqlen; p.Tq = m->Tq; p.Tk = m->Tk; p.W = m->W;
  p.runs = m->d_runs; p.run_stride = m->run_stride; p.nruns = m->d_nruns; p.live_cnt = m->d_live_cnt;
  p.bits = m->d_bits;
  p.stat_newly = st + 1;
  p.thr = threshold;
  p.scale = 1.0f / std::sqrt((float)d.head_dim);
  p.protect_start = d.protect_start; p.protect_len = d.protect_len;
  p.rows_total = (int)m->rows;
  p.order = m->d_order;
  if (ev) LA_HIP(hipEventRecord(ev[1], m->stream));
  LA_HIP(la::launch_fwd(p, (d.flags & LITE_ATTN_PV_SKIP_IMMEDIATE) != 0, m->stream));
  if (ev) LA_HIP(hipEventRecord(ev[2], m->stream));
  m->next_step = step + 1;
  return LITE_ATTN_OK;
}

int lite_attn_skip_stats(lite_attn_mask_t* m, int step, lite_attn_stats_t* host_out) {
  if (!m || !host_out) return LITE_ATTN_EINVAL;
  if (step < 0 || step >= m->next_step || step >= m->desc.max_steps) return LITE_ATTN_ESTEP;
  unsigned long long raw[3];
  LA_HIP(hipMemcpyAsync(raw, m->d_stats + 3 * (size_t)step, sizeof raw, hipMemcpyDeviceToHost, m->stream));
  LA_HIP(hipStreamSynchronize(m->stream));
  host_out->step = step;
  host_out->tiles_total = (uint64_t)m->rows * (uint64_t)m->Tk;
  host_out->tiles_skipped_in = raw[0];
  host_out->tiles_newly_marked = raw[1];
  host_out->live_list_bytes = raw[2] * sizeof(uint32_t);
  return LITE_ATTN_OK;
}

int lite_attn_profile(lite_attn_mask_t* m, int enable) {
  if (!m) return LITE_ATTN_EINVAL;
  if (enable && !m->events) {
    const size_t n = 3 * (size_t)m->desc.max_steps;
    hipEvent_t* ev = new (std::nothrow) hipEvent_t[n];
    bool* timed = new (std::nothrow) bool[m->desc.max_steps]();
    if (!ev || !timed) {
      delete[] ev;
      delete[] timed;
      return LITE_ATTN_ENOMEM;
    }
    for (size_t x = 0; x < n; ++x) {
      hipError_t e = hipEventCreate(&ev[x]);
      if (e != hipSuccess) {
        for (size_t y = 0; y < x; ++y) (void)hipEventDestroy(ev[y]);
        delete[] ev;
        delete[] timed;
        return hip_fail(e);
      }
    }
    m->events = ev;
    m->timed = timed;
  }
  m->profile = enable != 0;
  return LITE_ATTN_OK;
}

int lite_attn_kernel_times(lite_attn_mask_t* m, int step, float* host_prep_ms, float* host_fwd_ms) {
  if (!m || !host_prep_ms || !host_fwd_ms) return LITE_ATTN_EINVAL;
  if (step < 0 || step >= m->desc.max_steps || !m->events || !m->timed[step]) return LITE_ATTN_ESTEP;
  hipEvent_t* ev = m->events + 3 * (size_t)step;
  LA_HIP(hipEventSynchronize(ev[2]));
  LA_HIP(hipEventElapsedTime(host_prep_ms, ev[0], ev[1]));
  LA_HIP(hipEventElapsedTime(host_fwd_ms, ev[1], ev[2]));
  return LITE_ATTN_OK;
}

int lite_attn_mfma_peak(void* hip_stream, const void* dev_operands, int iters, float* host_ms, double* host_flops) {
  if (!dev_operands || !host_ms || !host_flops || iters < 1 || iters > (1 << 20)) return LITE_ATTN_EINVAL;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  int dev = 0, cus = 0;
  LA_HIP(hipGetDevice(&dev));
  LA_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int blocks = 2 * cus;  // 2 workgroups of 4 waves per CU: 2 waves per SIMD
  float* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipMalloc(&sink, sizeof(float));
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) e = la::launch_mfma_peak(dev_operands, sink, 64, blocks, st);  // warm-up
  if (e == hipSuccess) e = hipEventRecord(e0, st);
  if (e == hipSuccess) e = la::launch_mfma_peak(dev_operands, sink, iters, blocks, st);
  if (e == hipSuccess) e = hipEventRecord(e1, st);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(host_ms, e0, e1);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  if (e != hipSuccess) return hip_fail(e);
  *host_flops = (double)blocks * 4.0 * (double)iters * 32.0 * (2.0 * 32 * 32 * 16);
  return LITE_ATTN_OK;
}

size_t lite_attn_mask_words(const lite_attn_mask_t* m) { return m ? (size_t)m->rows * m->W : 0; }

int lite_attn_mask_export(lite_attn_mask_t* m, uint64_t* host_bits, size_t words) {
  if (!m || !host_bits || words != lite_attn_mask_words(m)) return LITE_ATTN_EINVAL;
  LA_HIP(hipMemcpyAsync(host_bits, m->d_bits, words * sizeof(uint64_t), hipMemcpyDeviceToHost, m->stream));
  LA_HIP(hipStreamSynchronize(m->stream));
  return LITE_ATTN_OK;
}

int lite_attn_mask_import(lite_attn_mask_t* m, const uint64_t* host_bits, size_t words, int next_step) {
  if (!m || !host_bits || words != lite_attn_mask_words(m)) return LITE_ATTN_EINVAL;
  if (next_step < 0 || next_step >= m->desc.max_steps) return LITE_ATTN_ESTEP;
  LA_HIP(hipMemcpyAsync(m->d_bits, host_bits, words * sizeof(uint64_t), hipMemcpyHostToDevice, m->stream));
  LA_HIP(hipStreamSynchronize(m->stream));
  m->next_step = next_step;
  return LITE_ATTN_OK;
}

int lite_attn_skipruns_export(lite_attn_mask_t* m, uint32_t* host_runs, uint32_t* host_nruns) {
  if (!m || !host_runs || !host_nruns) return LITE_ATTN_EINVAL;
  LA_HIP(la::launch_compact(m->d_bits, (int)m->rows, m->Tq, m->Tk, m->W,
                            m->desc.flags & LITE_ATTN_ORDER_DIAGONAL_FIRST, m->run_stride, m->d_runs, m->d_nruns,
                            m->d_live_cnt, nullptr, nullptr, m->stream));
  LA_HIP(hipMemcpyAsync(host_runs, m->d_runs, sizeof(uint32_t) * (size_t)m->rows * m->run_stride,
                        hipMemcpyDeviceToHost, m->stream));
  LA_HIP(hipMemcpyAsync(host_nruns, m->d_nruns, sizeof(uint32_t) * (size_t)m->rows, hipMemcpyDeviceToHost, m->stream));
  LA_HIP(hipStreamSynchronize(m->stream));
  return LITE_ATTN_OK;
}

size_t lite_attn_skipruns_stride(const lite_attn_mask_t* m) { return m ? (size_t)m->run_stride : 0; }

int lite_attn_skiplist_export(lite_attn_mask_t* m, uint16_t* host_live_idx, uint32_t* host_live_cnt) {
  if (!m || !host_live_idx || !host_live_cnt) return LITE_ATTN_EINVAL;
  uint32_t* runs = new (std::nothrow) uint32_t[(size_t)m->rows * m->run_stride];
  uint32_t* nruns = new (std::nothrow) uint32_t[(size_t)m->rows];
  int rc = (runs && nruns) ? lite_attn_skipruns_export(m, runs, nruns) : LITE_ATTN_ENOMEM;
  if (rc == LITE_ATTN_OK) {
    for (int64_t row = 0; row < m->rows; ++row) {  // expand the runs into the packed index list
      uint32_t n = 0;
      for (uint32_t x = 0; x < nruns[row]; ++x) {
        const uint32_t e = runs[row * m->run_stride + x];
        for (uint32_t j = e & 0xffffu; j < (e >> 16); ++j) host_live_idx[row * m->Tk + n++] = (uint16_t)j;
      }
      host_live_cnt[row] = n;
    }
  }
  delete[] runs;
  delete[] nruns;
  return rc;
}

void lite_attn_free_mask(lite_attn_mask_t* m) {
  if (!m) return;
  if (m->d_bits) (void)hipFree(m->d_bits);
  if (m->d_runs) (void)hipFree(m->d_runs);
  if (m->d_nruns) (void)hipFree(m->d_nruns);
  if (m->d_live_cnt) (void)hipFree(m->d_live_cnt);
  if (m->d_stats) (void)hipFree(m->d_stats);
  if (m->d_vt) (void)hipFree(m->d_vt);
  if (m->d_order) (void)hipFree(m->d_order);
  if (m->events) {
    for (size_t x = 0; x < 3 * (size_t)m->desc.max_steps; ++x) (void)hipEventDestroy(m->events[x]);
    delete[] m->events;
  }
  delete[] m->timed;
  delete m;
}

const char* lite_attn_strerror(int code) {
  switch (code) {
    case LITE_ATTN_OK: return "ok";
    case LITE_ATTN_EINVAL: return "invalid argument";
    case LITE_ATTN_ESTEP: return "step out of sequence";
    case LITE_ATTN_EUNSUPPORTED: return "unsupported shape (head_dim and tiles must be 128)";
    case LITE_ATTN_ENOMEM: return "out of memory";
    case LITE_ATTN_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

int lite_attn_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
