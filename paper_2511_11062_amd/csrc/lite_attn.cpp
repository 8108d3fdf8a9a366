// Host side of the C ABI declared in include/lite_attn.h: handles, contexts, launches (argument checks and buffer
// layouts are in lite_attn_host.cpp).
#include "lite_attn.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <new>

#include "lite_attn_kernels.h"

// Device memory that every call rewrites before reading it (nothing in it outlives a call): V^T.  A handle either
// owns one or borrows its context's.
struct la_scratch {
  void* base = nullptr;
  size_t bytes = 0;
};

struct lite_attn_ctx {
  la_scratch scratch;
  hipStream_t stream = nullptr;
  int device = 0;
  int handles = 0;  // live handles attached to this context
};

struct lite_attn_mask {
  lite_attn_desc_t desc;
  la::Geometry geo;
  la::ListLayout ll;
  uint64_t* d_bits;
  char* d_lists;      // Skip-Lists and row ranking (layout ll); kept between calls
  bool lists_valid;   // the lists describe the mask as it stands (left by the previous call's epilogue)
  unsigned long long* d_stats;  // [max_steps][3]: skipped on entry, newly marked, Skip-List runs
  la_scratch own;               // used when ctx == nullptr
  lite_attn_ctx* ctx;           // shared scratch + stream, or nullptr
  hipStream_t stream;           // used when ctx == nullptr
  int next_step;
  bool profile;
  hipEvent_t* events;  // [max_steps][3] once profiling was enabled: before the pre-passes, between, after attention
  bool* timed;         // [max_steps]
};

namespace {
thread_local int g_last_hip = 0;
}

namespace la {

int hip_fail(hipError_t e) {
  g_last_hip = (int)e;
  return e == hipErrorOutOfMemory ? LITE_ATTN_ENOMEM : LITE_ATTN_EHIP;
}

hipError_t launch_call(const lite_attn_desc_t& d, const Geometry& g, const ListLayout& ll, char* lists, uint16_t* vt,
                       const void* q, const void* k, const void* v, void* out, uint64_t* bits,
                       unsigned long long* stats3, float threshold, bool lists_ready, bool build_next,
                       hipStream_t stream, hipEvent_t mid) {
  uint32_t* runs = reinterpret_cast<uint32_t*>(lists + ll.runs);
  uint32_t* nruns = reinterpret_cast<uint32_t*>(lists + ll.nruns);
  uint32_t* live_cnt = reinterpret_cast<uint32_t*>(lists + ll.live_cnt);
  uint32_t* order = reinterpret_cast<uint32_t*>(lists + ll.order);
  uint32_t* chunk_work = reinterpret_cast<uint32_t*>(lists + ll.chunk_work);
  uint32_t* slots = reinterpret_cast<uint32_t*>(lists + ll.slots);
  uint32_t* xcd_rows = reinterpret_cast<uint32_t*>(lists + ll.xcd_rows);
  const int diagonal_first = (d.flags & LITE_ATTN_ORDER_DIAGONAL_FIRST) ? 1 : 0;
  hipError_t e = hipSuccess;
  if (!lists_ready) {
    e = launch_compact(bits, (int)g.rows, g.Tq, g.Tk, g.W, diagonal_first, g.run_stride, runs, nruns, live_cnt, stream);
    if (e != hipSuccess) return e;
  }
  // ranking a head's rows needs the counts of all of them, dealing the ranked chunks to the XCDs those of all heads:
  // two small kernels of their own
  e = launch_order_rows(live_cnt, g.BH, g.Tq, g.Tk, order, chunk_work, stream);
  if (e != hipSuccess) return e;
  e = launch_deal_rows(chunk_work, order, g.BH, g.Tq, g.chunks, g.per_xcd, slots, xcd_rows, stream);
  if (e != hipSuccess) return e;
  e = launch_transpose_v(static_cast<const uint16_t*>(v), vt, d.stride_b, d.stride_h, d.stride_n, g.BH, d.heads,
                         d.seqlen, g.Tk, stream);
  if (e != hipSuccess) return e;
  FwdParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.vt = vt;
  p.out = static_cast<uint16_t*>(out);
  p.stride_b = d.stride_b; p.stride_h = d.stride_h; p.stride_n = d.stride_n;
  p.H = d.heads; p.N = d.seqlen; p.Tq = g.Tq; p.Tk = g.Tk; p.W = g.W;
  p.runs = runs; p.run_stride = g.run_stride; p.nruns = nruns; p.live_cnt = live_cnt;
  p.bits = bits;
  p.stat_skipped_in = stats3; p.stat_newly = stats3 + 1; p.stat_runs = stats3 + 2;
  p.thr = threshold;
  p.scale = 1.0f / std::sqrt((float)d.head_dim);
  p.protect_start = d.protect_start; p.protect_len = d.protect_len;
  p.rows_total = (int)g.rows;
  p.slots = slots; p.per_xcd = g.per_xcd; p.xcd_rows = xcd_rows;
  p.build_next = build_next ? 1 : 0;
  p.diagonal_first = diagonal_first;
  if (mid) {
    e = hipEventRecord(mid, stream);
    if (e != hipSuccess) return e;
  }
  return launch_fwd(p, (d.flags & LITE_ATTN_PV_SKIP_IMMEDIATE) != 0, stream);
}

}  // namespace la

namespace {

using la::hip_fail;

#define LA_HIP(expr)                           \
  do {                                         \
    hipError_t e_ = (expr);                    \
    if (e_ != hipSuccess) return hip_fail(e_); \
  } while (0)

hipStream_t stream_of(const lite_attn_mask* m) { return m->ctx ? m->ctx->stream : m->stream; }
uint16_t* vt_of(const lite_attn_mask* m) { return static_cast<uint16_t*>(m->ctx ? m->ctx->scratch.base : m->own.base); }

int grow(la_scratch* s, size_t bytes) {
  if (bytes <= s->bytes) return LITE_ATTN_OK;
  if (s->base) LA_HIP(hipFree(s->base));
  s->base = nullptr;
  s->bytes = 0;
  LA_HIP(hipMalloc(&s->base, bytes));
  s->bytes = bytes;
  return LITE_ATTN_OK;
}

int init_common(const lite_attn_desc_t* desc, lite_attn_ctx* ctx, lite_attn_mask_t** out) {
  if (!out) return LITE_ATTN_EINVAL;
  int rc = la::check_desc(desc);
  if (rc != LITE_ATTN_OK) return rc;
  lite_attn_mask* m = new (std::nothrow) lite_attn_mask();
  if (!m) return LITE_ATTN_ENOMEM;
  m->desc = *desc;
  m->geo = la::geometry(*desc);
  m->ll = la::list_layout(m->geo);
  m->d_lists = nullptr;
  m->lists_valid = false;
  m->ctx = nullptr;
  m->stream = nullptr;
  m->next_step = 0;
  m->profile = false;
  m->events = nullptr;
  m->timed = nullptr;
  m->d_bits = nullptr;
  m->d_stats = nullptr;
  const size_t words = (size_t)m->geo.rows * m->geo.W, nstats = 3 * (size_t)desc->max_steps;
  const size_t vt = la::vt_bytes(m->geo);
  hipStream_t st = ctx ? ctx->stream : nullptr;
  rc = LITE_ATTN_OK;
  if (ctx) {
    // every call made so far through this context has to finish before its scratch may move
    hipError_t e = vt > ctx->scratch.bytes ? hipStreamSynchronize(ctx->stream) : hipSuccess;
    rc = e != hipSuccess ? hip_fail(e) : grow(&ctx->scratch, vt);
  } else {
    rc = grow(&m->own, vt);
  }
  if (rc == LITE_ATTN_OK) {
    hipError_t e = hipMalloc(&m->d_bits, sizeof(uint64_t) * words);
    if (e == hipSuccess) e = hipMalloc(&m->d_stats, sizeof(unsigned long long) * nstats);
    if (e == hipSuccess) e = hipMalloc(&m->d_lists, m->ll.total);
    if (e == hipSuccess) e = la::prepare_fwd();
    if (e == hipSuccess) e = la::launch_clear(m->d_bits, words, m->d_stats, nstats, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) rc = hip_fail(e);
  }
  if (rc != LITE_ATTN_OK) {
    lite_attn_free_mask(m);
    return rc;
  }
  if (ctx) {
    m->ctx = ctx;
    ++ctx->handles;
  }
  *out = m;
  return LITE_ATTN_OK;
}

}  // namespace

extern "C" {

int lite_attn_init_mask(const lite_attn_desc_t* desc, lite_attn_mask_t** out) { return init_common(desc, nullptr, out); }

int lite_attn_ctx_create(lite_attn_ctx_t** out) {
  if (!out) return LITE_ATTN_EINVAL;
  lite_attn_ctx* c = new (std::nothrow) lite_attn_ctx();
  if (!c) return LITE_ATTN_ENOMEM;
  hipError_t e = hipGetDevice(&c->device);
  if (e != hipSuccess) {
    delete c;
    return hip_fail(e);
  }
  *out = c;
  return LITE_ATTN_OK;
}

int lite_attn_ctx_set_stream(lite_attn_ctx_t* ctx, void* hip_stream) {
  if (!ctx) return LITE_ATTN_EINVAL;
  LA_HIP(hipStreamSynchronize(ctx->stream));  // work already queued keeps its order with what follows
  ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
  return LITE_ATTN_OK;
}

int lite_attn_init_mask_shared(const lite_attn_desc_t* desc, lite_attn_ctx_t* ctx, lite_attn_mask_t** out) {
  if (!ctx) return LITE_ATTN_EINVAL;
  return init_common(desc, ctx, out);
}

int lite_attn_ctx_free(lite_attn_ctx_t* ctx) {
  if (!ctx) return LITE_ATTN_OK;
  if (ctx->handles != 0) return LITE_ATTN_ESHARED;
  if (ctx->scratch.base) (void)hipFree(ctx->scratch.base);
  delete ctx;
  return LITE_ATTN_OK;
}

int lite_attn_set_stream(lite_attn_mask_t* m, void* hip_stream) {
  if (!m) return LITE_ATTN_EINVAL;
  if (m->ctx)  // the scratch is only safe while every handle of the context runs on the context's one stream
    return reinterpret_cast<hipStream_t>(hip_stream) == m->ctx->stream ? LITE_ATTN_OK : LITE_ATTN_ESHARED;
  LA_HIP(hipStreamSynchronize(m->stream));  // work already queued keeps its order with what follows
  m->stream = reinterpret_cast<hipStream_t>(hip_stream);
  return LITE_ATTN_OK;
}

int lite_attn_fwd(const void* q, const void* k, const void* v, void* out, lite_attn_mask_t* m, float threshold,
                  int step) {
  if (!m) return LITE_ATTN_EINVAL;
  int rc = la::check_call(q, k, v, out, threshold);
  if (rc != LITE_ATTN_OK) return rc;
  if (step < 0 || step >= m->desc.max_steps) return LITE_ATTN_ESTEP;
  if (step != 0 && step != m->next_step) return LITE_ATTN_ESTEP;
  const lite_attn_desc_t& d = m->desc;
  hipStream_t stream = stream_of(m);
  if (step == 0)
    LA_HIP(la::launch_clear(m->d_bits, (size_t)m->geo.rows * m->geo.W, m->d_stats, 3 * (size_t)d.max_steps, stream));
  unsigned long long* st = m->d_stats + 3 * (size_t)step;
  hipEvent_t* ev = (m->profile && m->events) ? m->events + 3 * (size_t)step : nullptr;
  if (m->timed) m->timed[step] = ev != nullptr;
  if (ev) LA_HIP(hipEventRecord(ev[0], stream));
  // Lists left by the previous call's epilogue are used when they still describe the mask: not at step 0 (the mask
  // was just cleared) and not after an import.  This call's epilogue then leaves the lists of the next call.
  const bool ready = m->lists_valid && step != 0;
  m->lists_valid = false;
  LA_HIP(la::launch_call(d, m->geo, m->ll, m->d_lists, vt_of(m), q, k, v, out, m->d_bits, st, threshold, ready, true,
                         stream, ev ? ev[1] : nullptr));
  m->lists_valid = true;
  if (ev) LA_HIP(hipEventRecord(ev[2], stream));
  m->next_step = step + 1;
  return LITE_ATTN_OK;
}

int lite_attn_skip_stats(lite_attn_mask_t* m, int step, lite_attn_stats_t* host_out) {
  if (!m || !host_out) return LITE_ATTN_EINVAL;
  if (step < 0 || step >= m->next_step || step >= m->desc.max_steps) return LITE_ATTN_ESTEP;
  unsigned long long raw[3];
  LA_HIP(hipMemcpyAsync(raw, m->d_stats + 3 * (size_t)step, sizeof raw, hipMemcpyDeviceToHost, stream_of(m)));
  LA_HIP(hipStreamSynchronize(stream_of(m)));
  host_out->step = step;
  host_out->tiles_total = (uint64_t)m->geo.rows * (uint64_t)m->geo.Tk;
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

size_t lite_attn_mask_words(const lite_attn_mask_t* m) { return m ? (size_t)m->geo.rows * m->geo.W : 0; }

int lite_attn_mask_export(lite_attn_mask_t* m, uint64_t* host_bits, size_t words) {
  if (!m || !host_bits || words != lite_attn_mask_words(m)) return LITE_ATTN_EINVAL;
  LA_HIP(hipMemcpyAsync(host_bits, m->d_bits, words * sizeof(uint64_t), hipMemcpyDeviceToHost, stream_of(m)));
  LA_HIP(hipStreamSynchronize(stream_of(m)));
  return LITE_ATTN_OK;
}

int lite_attn_mask_import(lite_attn_mask_t* m, const uint64_t* host_bits, size_t words, int next_step) {
  if (!m || !host_bits || words != lite_attn_mask_words(m)) return LITE_ATTN_EINVAL;
  if (next_step < 0 || next_step >= m->desc.max_steps) return LITE_ATTN_ESTEP;
  LA_HIP(hipMemcpyAsync(m->d_bits, host_bits, words * sizeof(uint64_t), hipMemcpyHostToDevice, stream_of(m)));
  LA_HIP(hipStreamSynchronize(stream_of(m)));
  m->next_step = next_step;
  m->lists_valid = false;  // the next call rebuilds its Skip-Lists from the imported mask
  return LITE_ATTN_OK;
}

int lite_attn_skipruns_export(lite_attn_mask_t* m, uint32_t* host_runs, uint32_t* host_nruns) {
  if (!m || !host_runs || !host_nruns) return LITE_ATTN_EINVAL;
  const la::Geometry& g = m->geo;
  uint32_t* runs = reinterpret_cast<uint32_t*>(m->d_lists + m->ll.runs);
  uint32_t* nruns = reinterpret_cast<uint32_t*>(m->d_lists + m->ll.nruns);
  hipStream_t stream = stream_of(m);
  // (if the lists were already in place -- left by the last call's epilogue -- this writes the same values again)
  LA_HIP(la::launch_compact(m->d_bits, (int)g.rows, g.Tq, g.Tk, g.W, m->desc.flags & LITE_ATTN_ORDER_DIAGONAL_FIRST,
                            g.run_stride, runs, nruns, reinterpret_cast<uint32_t*>(m->d_lists + m->ll.live_cnt),
                            stream));
  LA_HIP(hipMemcpyAsync(host_runs, runs, sizeof(uint32_t) * (size_t)g.rows * g.run_stride, hipMemcpyDeviceToHost,
                        stream));
  LA_HIP(hipMemcpyAsync(host_nruns, nruns, sizeof(uint32_t) * (size_t)g.rows, hipMemcpyDeviceToHost, stream));
  LA_HIP(hipStreamSynchronize(stream));
  return LITE_ATTN_OK;
}

size_t lite_attn_skipruns_stride(const lite_attn_mask_t* m) { return m ? (size_t)m->geo.run_stride : 0; }

int lite_attn_skiplist_export(lite_attn_mask_t* m, uint16_t* host_live_idx, uint32_t* host_live_cnt) {
  if (!m || !host_live_idx || !host_live_cnt) return LITE_ATTN_EINVAL;
  const la::Geometry& g = m->geo;
  uint32_t* runs = new (std::nothrow) uint32_t[(size_t)g.rows * g.run_stride];
  uint32_t* nruns = new (std::nothrow) uint32_t[(size_t)g.rows];
  int rc = (runs && nruns) ? lite_attn_skipruns_export(m, runs, nruns) : LITE_ATTN_ENOMEM;
  if (rc == LITE_ATTN_OK) {
    for (int64_t row = 0; row < g.rows; ++row) {  // expand the runs into the packed index list
      uint32_t n = 0;
      for (uint32_t x = 0; x < nruns[row]; ++x) {
        const uint32_t e = runs[row * g.run_stride + x];
        for (uint32_t j = e & 0xffffu; j < (e >> 16); ++j) host_live_idx[row * g.Tk + n++] = (uint16_t)j;
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
  if (m->ctx) {
    // the shared scratch stays with the context; calls of this handle still in flight only touch the scratch and
    // the buffers freed below, and hipFree waits for the device
    --m->ctx->handles;
  }
  if (m->d_bits) (void)hipFree(m->d_bits);
  if (m->d_stats) (void)hipFree(m->d_stats);
  if (m->d_lists) (void)hipFree(m->d_lists);
  if (m->own.base) (void)hipFree(m->own.base);
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
    case LITE_ATTN_ESHARED:
      return "not allowed while scratch is shared (a handle of a context runs on the context's stream; a context "
             "with live handles cannot be freed)";
    case LITE_ATTN_ESCRATCH: return "the shape needs more scratch than the static device array holds";
    default: return "unknown error";
  }
}

int lite_attn_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
