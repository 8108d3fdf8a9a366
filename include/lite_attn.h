/*
 * lite_attn.h -- C ABI of the MI355X (gfx950) LiteAttention forward path.
 *
 * One call of lite_attn_fwd is one self-attention call of one transformer
 * layer at one denoising timestep: a tiled FlashAttention-style forward
 * (S = Q K^T / sqrt(d), online softmax, O = P V; paper Preliminaries,
 * eqs. 1-3 and the tile recurrences after them) that
 *   - visits, for every Q tile, only the K/V tiles whose Skip-Mask bit is
 *     clear (Method, Algorithm 2 "QK-Skip"; Implementation, "Producer and
 *     Skip-List Optimization"),
 *   - evaluates the local skip predicate max(m_local - m_ij) <= -eps on every
 *     visited tile during the online softmax (Preliminaries, eq. sparge_cond;
 *     Implementation, "Skip-Mask Evaluation Mechanism"),
 *   - and sets the Skip-Mask bit of every tile the predicate marks; bits are
 *     only ever set, and a bit set in this call takes effect from the next
 *     call on (the marked tile is still accumulated in the call that marks
 *     it, as the Implementation section describes).
 * The Skip-Mask persists in the handle across calls (timesteps).
 *
 * All pointers named q, k, v, out are DEVICE pointers to bf16; everything
 * named host_* is a HOST pointer.  No function throws or aborts; every
 * function returning int returns 0 on success or a negative lite_attn_error.
 * The library never synchronises the device inside lite_attn_fwd.
 */
#ifndef LITE_ATTN_H
#define LITE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LITE_ATTN_OK = 0,
  LITE_ATTN_EINVAL = -1,       /* null pointer, non-positive size, threshold >= 0 or NaN, bad stride */
  LITE_ATTN_ESTEP = -2,        /* step is neither 0 nor last step + 1, or >= max_steps */
  LITE_ATTN_EUNSUPPORTED = -3, /* head_dim != 128, tile_q/tile_k != 128, more than 16383 K/V tiles (seqlen >
                                  2097024), or one head's K/V spanning 4 GiB or more ((seqlen+128)*stride_n*2 bytes) */
  LITE_ATTN_ENOMEM = -4,       /* host or device allocation failed */
  LITE_ATTN_EHIP = -5,         /* a HIP runtime call failed; lite_attn_last_hip_error() has its code */
  LITE_ATTN_ESHARED = -6,      /* refused because scratch is shared: lite_attn_set_stream on a handle of a context with
                                  any stream but the context's; lite_attn_ctx_free while handles are attached */
  LITE_ATTN_ESCRATCH = -7      /* lite_attn_fwd_static: the shape needs more than LITE_ATTN_STATIC_SCRATCH_BYTES */
} lite_attn_error;

/* desc.flags.  The skip predicate compares a tile with the running row maximum over the tiles visited BEFORE it, so
   the visiting order of the j loop decides how soon tiles can be judged against the true maximum (paper: Method,
   "Skipping Condition": other orderings reach the global maximum faster; its experiments use the linear order).
   Default: ascending j.  LITE_ATTN_ORDER_DIAGONAL_FIRST: Q tile i visits K/V tiles i, i+1, ..., Tk-1, 0, ..., i-1. */
#define LITE_ATTN_ORDER_DIAGONAL_FIRST 2
/* LITE_ATTN_PV_SKIP_IMMEDIATE: the paper's Algorithm 2 taken literally -- a tile whose predicate fires is dropped in
   the very call that marks it (its exp(S) V product and row sums are not accumulated), instead of contributing once
   more and being skipped from the next call on (the default, which is what the paper's Implementation section
   describes for its kernel).  The Skip-Mask after the call is the same in both modes: a fired tile cannot raise the
   running maximum.  The output of the marking call equals attention over the tiles live AFTER the call. */
#define LITE_ATTN_PV_SKIP_IMMEDIATE 1

/* Shape of one attention layer; fixed for the life of a handle. */
typedef struct {
  int32_t batch, heads, seqlen, head_dim; /* head_dim must be 128 */
  int32_t tile_q, tile_k;                 /* Skip-Mask granularity (rows x columns of S per bit); must be 128, 128 */
  int64_t stride_b, stride_h, stride_n;   /* element strides shared by q, k, v and out; head_dim is contiguous.
                                             [B,H,N,d]: (H*N*d, N*d, d);  [B,N,H,d]: (N*H*d, d, H*d) */
  int32_t protect_start, protect_len;     /* token range [start, start+len) never skipped: a tile whose Q rows or
                                             K/V columns intersect it is evaluated but never marked; len 0 = none */
  int32_t flags;                          /* 0, or an OR of the LITE_ATTN_* flags above */
  int32_t max_steps;                      /* capacity of the per-step statistics, >= 1 */
} lite_attn_desc_t;

/* Opaque handle: owns the device Skip-Mask ([B,H,Tq,ceil(Tk/64)] uint64, bit j%64 of word j/64 set = tile (i,j)
   skipped) and the statistics, and owns or borrows (lite_attn_init_mask_shared) the per-call scratch: Skip-List
   buffers and a copy of V^T (same size as V).
   Tq = ceil(N/tile_q), Tk = ceil(N/tile_k). */
typedef struct lite_attn_mask lite_attn_mask_t;

typedef struct {
  int32_t step;
  uint64_t tiles_total;        /* B*H*Tq*Tk */
  uint64_t tiles_skipped_in;   /* tiles already marked when the step started (not visited) */
  uint64_t tiles_newly_marked; /* tiles the predicate marked during the step */
  uint64_t live_list_bytes;    /* bytes of Skip-List entries (4 per run of live tiles) the attention kernel read */
} lite_attn_stats_t;

/* Allocates the handle and its device buffers on the current HIP device and clears the mask.
   Paper: the Skip-Mask is a persistent per-layer, per-head structure (Implementation, "LiteAttention").
   *out is written only on success.  Uses the null stream until lite_attn_set_stream.  The handle belongs to the
   device that is current here: every later call on it must be made with the same device current.  Calls on one
   handle are not thread-safe; different handles are independent. */
int lite_attn_init_mask(const lite_attn_desc_t* desc, lite_attn_mask_t** out);

/* All later work of this handle is enqueued on `hip_stream` (a hipStream_t, e.g. PyTorch's current stream).
   For a handle created with lite_attn_init_mask_shared this is refused (LITE_ATTN_ESHARED) unless `hip_stream`
   is its context's stream: set the stream on the context. */
int lite_attn_set_stream(lite_attn_mask_t* mask, void* hip_stream);

/* Scratch shared by the layers of a model (this library's own arrangement, nothing of the paper's).
   A call needs device scratch that nothing reads after the call has finished: the Skip-List, the row schedule and
   a transposed copy of V, together about the size of V.  A handle made by lite_attn_init_mask owns its own; a model
   with one handle per layer would hold that once per layer.  Handles made by lite_attn_init_mask_shared borrow the
   scratch of a context instead: one buffer on the context's device, grown to the largest layer attached so far.
   Sharing is safe because all handles of a context run on the context's ONE stream, where calls are serial:
     lite_attn_ctx_create       context on the current HIP device, null stream, no scratch yet
     lite_attn_ctx_set_stream   waits for the work queued on the old stream, then every handle of the context
                                (present and future) enqueues on `hip_stream`
     lite_attn_init_mask_shared like lite_attn_init_mask, the handle attached to `ctx`; may reallocate the shared
                                scratch (after waiting for the context's stream).  The handle's Skip-Mask and
                                statistics stay its own.
     lite_attn_ctx_free         LITE_ATTN_ESHARED while handles are attached (free them first); null is a no-op
   Calls on one context and its handles are not thread-safe. */
typedef struct lite_attn_ctx lite_attn_ctx_t;
int lite_attn_ctx_create(lite_attn_ctx_t** out);
int lite_attn_ctx_set_stream(lite_attn_ctx_t* ctx, void* hip_stream);
int lite_attn_init_mask_shared(const lite_attn_desc_t* desc, lite_attn_ctx_t* ctx, lite_attn_mask_t** out);
int lite_attn_ctx_free(lite_attn_ctx_t* ctx);

/* One attention call (Algorithm 2 with the deferred mask update, see top of file; desc.flags selects the
   immediate variant and the visiting order).
     q, k, v   device bf16, layout given by the handle's strides; borrowed, not modified; values must be finite
               (the kernels are built with the assumption that no NaN occurs)
     out       device bf16, same layout; every valid row is written
     skip_mask handle; its mask is read (via the Skip-List built from it at the start of the call) and updated
     threshold signed -eps of eq. (sparge_cond) in natural-log units of S = QK^T/sqrt(d), must be < 0;
               -INFINITY never marks anything (with an empty mask the result is dense attention)
     step      0 clears the mask and the statistics first (new denoising trajectory); otherwise must be the
               previous call's step + 1
   Asynchronous on the handle's stream; allocates nothing.  With profiling off (lite_attn_profile) the call only
   launches kernels -- no memset, memcpy or event nodes -- so a sequence of calls may be captured in a HIP graph; a
   replay repeats the captured steps (same step numbers, thresholds and pointers); the statistics counters of a
   replayed step keep adding up unless the replay includes step 0, which clears them. */
int lite_attn_fwd(const void* q, const void* k, const void* v, void* out, lite_attn_mask_t* skip_mask,
                  float threshold, int step);

/* The same attention call for callers that cannot allocate device memory at all -- code running under HIP graph
   capture, serving loops and harnesses that forbid hipMalloc -- and therefore cannot create a handle.  It allocates
   nothing and frees nothing: no hipMalloc, no hipFree, no allocating library routine.  Everything the other entry
   points keep in allocated device memory besides the Skip-Mask (Skip-List, row schedule, V^T, the call's counters)
   lives in ONE static device array of LITE_ATTN_STATIC_SCRATCH_BYTES that the library's code object brings along on
   every GPU it is loaded on and holds until the process ends.
     q, k, v, out, threshold   as for lite_attn_fwd
     desc            shape, strides, protected range and flags of the layer, as for lite_attn_init_mask (max_steps
                     must be >= 1 and is otherwise unused)
     dev_skip_mask   DEVICE pointer, 8-byte aligned, to the layer's Skip-Mask: B*H*Tq*ceil(Tk/64) uint64 words in the
                     handle's layout (bit j%64 of word j/64 of row (b*H+h)*Tq+i set = tile (i,j) skipped).  Input and
                     output: the caller owns it, keeps it between timesteps, and zeroes it to start a new trajectory
     hip_stream      hipStream_t on which the call's kernels are enqueued (asynchronous)
   A shape whose scratch (about the size of V plus 2*Tk+12 bytes per Q-tile row) exceeds the array is refused with
   LITE_ATTN_ESCRATCH before anything is launched: B*H*ceil(N/128) up to about 4000, e.g. the 12-head N=32760
   layer; the larger benchmark shapes need a handle.  The first call on a GPU looks up the array's address there and
   sets the attention kernel's function attributes (no allocation, but not work to record into a graph: make the first
   call on a GPU outside stream capture).
   Every call on a GPU uses that GPU's one array, which keeps the previous call's contents (what has to start at
   zero is cleared by the call itself): calls that overlap in time on one GPU -- two streams, two threads -- race;
   calls on one stream are safe. */
#define LITE_ATTN_STATIC_SCRATCH_BYTES (128u << 20)
int lite_attn_fwd_static(const void* q, const void* k, const void* v, void* out, const lite_attn_desc_t* desc,
                         uint64_t* dev_skip_mask, float threshold, void* hip_stream);

/* Statistics of one completed step (paper's sparsity = skipped fraction of tiles, Experiments "Metrics").
   Synchronises the handle's stream. */
int lite_attn_skip_stats(lite_attn_mask_t* mask, int step, lite_attn_stats_t* host_out);

/* Per-phase timing for benchmarks.  enable != 0 makes every later lite_attn_fwd record HIP events on the handle's
   stream around its two phases (events are created on the first enabled call; a few microseconds per call).
   lite_attn_kernel_times returns the durations of a completed step in milliseconds -- host_prep_ms: Skip-List
   compaction plus the V transposition pre-pass; host_fwd_ms: the fused attention kernel -- it synchronises the
   stream and fails with LITE_ATTN_ESTEP if that step was not run with profiling enabled. */
int lite_attn_profile(lite_attn_mask_t* mask, int enable);
int lite_attn_kernel_times(lite_attn_mask_t* mask, int step, float* host_prep_ms, float* host_fwd_ms);

/* Number of uint64 words of the whole mask: B*H*Tq*ceil(Tk/64). */
size_t lite_attn_mask_words(const lite_attn_mask_t* mask);

/* Copy the Skip-Mask to / from host memory (`words` must equal lite_attn_mask_words).  Both synchronise the
   stream.  Import overwrites the mask (it is the only way bits can be cleared besides step 0) and sets
   the expected next step to `next_step` (>= 0). */
int lite_attn_mask_export(lite_attn_mask_t* mask, uint64_t* host_bits, size_t words);
int lite_attn_mask_import(lite_attn_mask_t* mask, const uint64_t* host_bits, size_t words, int next_step);

/* Runs the Skip-List compaction on the current mask and copies the result to the host.
   Paper: the Skip-List is the run-length form of the mask that the loader walks -- consecutive non-skipped tiles are
   one (start, end) pair (Implementation, "Producer and Skip-List Optimization").
     host_runs  [B*H*Tq][lite_attn_skipruns_stride()] uint32: for each Q-tile row its maximal runs of live K/V tiles
                in visiting order, entry = start | end << 16 (end exclusive), in the first host_nruns[row] slots
     host_nruns [B*H*Tq] uint32
   Synchronises. */
int lite_attn_skipruns_export(lite_attn_mask_t* mask, uint32_t* host_runs, uint32_t* host_nruns);
size_t lite_attn_skipruns_stride(const lite_attn_mask_t* mask); /* entries per row = floor(Tk/2) + 1 */

/* Same list expanded on the host into packed tile indices:
     host_live_idx [B*H*Tq][Tk] uint16: indices of the row's live K/V tiles, in visiting order, in the first
                                        host_live_cnt[row] slots (the rest is unspecified)
     host_live_cnt [B*H*Tq]     uint32
   Synchronises. */
int lite_attn_skiplist_export(lite_attn_mask_t* mask, uint16_t* host_live_idx, uint32_t* host_live_cnt);

void lite_attn_free_mask(lite_attn_mask_t* mask);

const char* lite_attn_strerror(int code);
int lite_attn_last_hip_error(void); /* hipError_t of the last failed HIP call on this thread, 0 if none */

#ifdef __cplusplus
}
#endif
#endif /* LITE_ATTN_H */
