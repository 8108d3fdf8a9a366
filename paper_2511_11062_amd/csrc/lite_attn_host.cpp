// Pure host logic of the C ABI (no HIP call, no device code): descriptor and call checks, tile geometry, layout of
// the per-call scratch.  Kept apart so that it also builds with a plain C++ compiler under the CPU sanitizers.
#include <cmath>

#include "lite_attn_kernels.h"

namespace la {

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
  // LDS budgets: the row schedule's histogram (Tk + 1 bins) and the fused kernel's bitmap of newly set mask bits
  if (Tk > 16383) return LITE_ATTN_EUNSUPPORTED;
  // K/V stages are addressed with 32-bit byte offsets from the head's base pointer
  if (((int64_t)d->seqlen + 128) * d->stride_n * 2 >= ((int64_t)1 << 32)) return LITE_ATTN_EUNSUPPORTED;
  const int64_t rows = (int64_t)d->batch * d->heads * Tk;
  if (rows > (int64_t)1 << 30) return LITE_ATTN_EUNSUPPORTED;
  return LITE_ATTN_OK;
}

int check_call(const void* q, const void* k, const void* v, const void* out, float threshold) {
  if (!q || !k || !v || !out) return LITE_ATTN_EINVAL;
  if (std::isnan(threshold) || threshold >= 0.f) return LITE_ATTN_EINVAL;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) return LITE_ATTN_EINVAL;
  return LITE_ATTN_OK;
}

Geometry geometry(const lite_attn_desc_t& d) {
  Geometry g;
  g.Tq = (d.seqlen + d.tile_q - 1) / d.tile_q;
  g.Tk = (d.seqlen + d.tile_k - 1) / d.tile_k;
  g.W = (g.Tk + 63) / 64;
  g.run_stride = g.Tk / 2 + 1;
  g.BH = d.batch * d.heads;
  g.rows = (int64_t)g.BH * g.Tq;
  g.chunks = g.BH * ((g.Tq + kChunkRows - 1) / kChunkRows);
  g.per_xcd = ((g.chunks + 7) / 8 + 1) * kChunkRows;
  return g;
}

namespace {
size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
}  // namespace

ListLayout list_layout(const Geometry& g) {
  ListLayout l;
  size_t at = 0;
  l.stats = at;
  at += up256(3 * sizeof(unsigned long long));
  l.nruns = at;
  at += up256(sizeof(uint32_t) * (size_t)g.rows);
  l.live_cnt = at;
  at += up256(sizeof(uint32_t) * (size_t)g.rows);
  l.order = at;
  at += up256(sizeof(uint32_t) * (size_t)g.rows);
  l.chunk_work = at;
  at += up256(sizeof(uint32_t) * (size_t)g.chunks);
  l.slots = at;
  at += up256(sizeof(uint32_t) * 8 * (size_t)g.per_xcd);
  l.xcd_rows = at;
  at += up256(sizeof(uint32_t) * 8);
  l.runs = at;
  at += up256(sizeof(uint32_t) * (size_t)g.rows * g.run_stride);
  l.total = at;
  return l;
}

size_t vt_bytes(const Geometry& g) { return up256(sizeof(uint16_t) * (size_t)g.BH * 128 * ((size_t)g.Tk * 128)); }

}  // namespace la
