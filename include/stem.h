/*
 * libstem — the STEM token-indexed FFN layer on one MI355X (gfx950), C ABI.
 *
 * The layer (paper: Method, "STEM", the layer equation) replaces the up-projection
 * of a SwiGLU FFN by a row of a per-layer table indexed by the token id:
 *
 *     y_i = W_down ( SiLU(W_gate x_i) * E[ids_i] )          for every token i
 *
 * with W_gate [F,d], W_down [d,F] (the paper's shapes, Background) and the table
 * E [V,F] ("U_l in R^{V x d_ff}").  Token ids are 0-based here (the paper counts
 * from 1).  No bias, norm or residual is part of the layer.
 *
 * Conventions for every call
 *   - All matrices are row-major and dense (leading dimension = number of columns).
 *   - Unless a parameter says "host", every pointer is DEVICE memory owned by the
 *     caller, 16-byte aligned, valid until the work enqueued on `stream` has run.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work and return; they do not synchronise unless stated.
 *   - Element type of activations, weights and the table is the context's dtype
 *     (STEM_BF16: bfloat16 storage, fp32 accumulation and epilogue math;
 *      STEM_F32: fp32 throughout).  Weight gradients, table-row gradients and
 *     optimiser state are always fp32.
 *   - d_model and d_ff must be multiples of 64 for STEM_BF16 and of 4 for STEM_F32;
 *     T may be any value in [0, max_tokens].  T == 0 is a no-op that returns STEM_OK.
 *   - Errors: argument and shape errors are detected on the host before anything
 *     is launched and returned as a status; stem_last_error() gives the text.
 *     Token ids outside [0, E_rows) never cause an out-of-bounds access: kernels
 *     clamp them to a valid row (a negative id to row 0, any other to the last row)
 *     and raise a sticky flag that the next libstem call on the context (or
 *     stem_sync_status) reports as STEM_ERR_ID_RANGE; the results of the tokens with
 *     valid ids are unaffected.
 *   - The context owns only scratch memory (sort buffers, partial sums, the
 *     internal H and dG buffers, pinned staging, one side stream and its events),
 *     all sized from max_tokens.  Memory is allocated by the set-up calls only:
 *     stem_create, stem_reserve, stem_set_prefetch_mode, stem_cache_init,
 *     stem_profile_enable.  No call that enqueues work allocates or frees.
 *     Calls on one context must not overlap in time (they share that scratch).
 */
#ifndef STEM_H
#define STEM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct stem_ctx stem_ctx; /* opaque */

typedef enum {
  STEM_OK = 0,
  STEM_ERR_INVALID_ARG = 1, /* null pointer, bad enum, misaligned pointer            */
  STEM_ERR_SHAPE = 2,       /* negative size, T > max_tokens, E_rows < 1, ...        */
  STEM_ERR_ID_RANGE = 3,    /* a token id outside [0, E_rows) was seen by a kernel   */
  STEM_ERR_WORKSPACE = 4,   /* a caller-provided capacity is too small               */
  STEM_ERR_UNSUPPORTED = 5, /* d_model / d_ff not a supported multiple               */
  STEM_ERR_HIP = 6          /* a HIP runtime call failed; see stem_last_error        */
} stem_status;

typedef enum { STEM_F32 = 0, STEM_BF16 = 1 } stem_dtype;

typedef struct {
  int32_t d_model; /* d   */
  int32_t d_ff;    /* F   */
  int32_t vocab;   /* V: number of rows of a device-resident table (upper bound on ids) */
  int32_t dtype;   /* stem_dtype */
} stem_layer_desc;

/* AdamW hyper-parameters (paper, Experiments: weight decay 0.1, beta1 0.9, beta2 0.95;
 * eps is not given there, 1e-8 is the customary value).  step >= 1 is the global step. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  int64_t step;
} stem_adamw_hparams;

/* ---- context ------------------------------------------------------------------- */

/* Creates a context on HIP device `device` with scratch for calls of up to max_tokens
 * tokens.  *out is NULL on failure.  host pointers: out, desc. */
stem_status stem_create(stem_ctx** out, const stem_layer_desc* desc, int64_t max_tokens, int device);
/* Scratch that only some entry points need, allocated on request (a set-up call: it allocates,
 * enqueues nothing).  what: a sum of
 *   STEM_RESERVE_UP    one more [max_tokens, d_ff] activation and one more [d_ff, d_model] weight buffer,
 *                      for stem_ffn_up_forward / stem_ffn_up_backward (bf16 contexts);
 *   STEM_RESERVE_EDIT  index lists and 64 replacement rows for stem_edit_rows.
 * Those entry points return STEM_ERR_WORKSPACE until their scratch has been reserved. */
#define STEM_RESERVE_UP 1u
#define STEM_RESERVE_EDIT 2u
stem_status stem_reserve(stem_ctx* ctx, uint32_t what);
/* Synchronises the device and frees the context's scratch.  NULL is allowed. */
void stem_destroy(stem_ctx* ctx);
/* Text of the last error on this context (or of the last failed stem_create when
 * ctx is NULL).  Never NULL; valid until the next call on the context. */
const char* stem_last_error(const stem_ctx* ctx);
const char* stem_status_string(stem_status s);
/* Waits for `stream`, then reports and clears the sticky id-range flag. */
stem_status stem_sync_status(stem_ctx* ctx, void* stream);

/* ---- the layer (Method, STEM layer equation) ---------------------------------- */

/* Forward.  x [T,d], ids [T] int32, W_gate [F,d], W_down [d,F], E [E_rows,F], y [T,d].
 * G = x W_gate^T;  H = SiLU(G) * E[ids];  y = H W_down^T.
 * save_G, save_H: [T,F] in the context dtype, or NULL (inference) — what backward needs.
 * wait_event: NULL, or a hipEvent_t (as returned by stem_prefetch_rows) that marks E's
 * rows as ready.  When given, the gate GEMM is enqueued first, `stream` then waits on
 * the event, and the SiLU*gather runs as a separate kernel before the down GEMM, so
 * the row copy overlaps the gate GEMM.  When the event is the one the context's last
 * stem_prefetch_rows returned for the same T (bf16 contexts), the wait is finer: the
 * rows were copied in order of first use with an event per chunk of tokens, and the
 * gather and the down GEMM of each chunk start as soon as that chunk's rows are there.
 * When NULL the gather is fused into the gate GEMM's epilogue.  Calls of at most 512
 * tokens (a decode step) use 128x64 tiles so that both products fill the chip. */
stem_status stem_ffn_forward(stem_ctx* ctx, const void* x, const int32_t* ids, const void* W_gate,
                             const void* W_down, const void* E, int64_t E_rows, int64_t T, void* y,
                             void* save_G, void* save_H, void* wait_event, void* stream);

/* y = residual + layer(x): the forward pass with the layer's output added to a residual stream in the
 * down product's own epilogue (sum in fp32, rounded once), as stacked layers are joined (the paper's
 * model adds the FFN output to the residual stream; a decode step through many layers saves one
 * element-wise kernel per layer this way).  residual [T,d], context dtype; y may be the same buffer as
 * residual and as x (x is read completely before y is first written).  Inference form: no
 * activations are saved, the table is device-resident.  Everything else as in stem_ffn_forward. */
stem_status stem_ffn_forward_residual(stem_ctx* ctx, const void* x, const int32_t* ids, const void* W_gate,
                                      const void* W_down, const void* E, int64_t E_rows, int64_t T,
                                      const void* residual, void* y, void* stream);

/* Backward of L = sum_i <y_i, dy_i> (chain rule of the layer equation; the paper
 * prints none).  dy [T,d]; saved_G [T,F] as written by forward (required); saved_H
 * [T,F] or NULL (then H is recomputed from saved_G and E).
 *   dH = dy W_down ;  dU = dH * SiLU(G) ;  dG = dH * E[ids] * SiLU'(G)
 *   dx = dG W_gate ;  dW_down = dy^T H ;  dW_gate = dG^T x
 * Outputs: dx [T,d] (context dtype), dW_gate [F,d] fp32, dW_down [d,F] fp32 (overwritten
 * when accumulate == 0, added to otherwise), dU [T,F] (context dtype) = gradient with
 * respect to each token's gathered row, the input of stem_embed_grad.  dx may be NULL
 * (then the dx GEMM is skipped). */
stem_status stem_ffn_backward(stem_ctx* ctx, const void* dy, const void* x, const int32_t* ids,
                              const void* W_gate, const void* W_down, const void* E, int64_t E_rows,
                              const void* saved_G, const void* saved_H, int64_t T, void* dx,
                              float* dW_gate, float* dW_down, void* dU, int accumulate, void* stream);

/* ---- table gradient: only the touched rows (System Implementation: token
 *      de-duplication; gradients of the table rows go to the optimiser) ---------- */

/* Stable sort of (ids[i], i) by id, distinct ids with their run offsets, and the
 * per-row sums  dE_rows[j,:] = sum_{k in [seg_offsets[j], seg_offsets[j+1])} dU[perm[k],:]
 * added in a fixed order (bit-identical on every run; no floating-point atomics).
 * Outputs (device): sorted_ids [T], perm [T], uniq_ids [min(T,V)] ascending,
 * seg_offsets [min(T,V)+1] (seg_offsets[n_uniq] = T), n_uniq [1], dE_rows
 * [min(T,V), F] fp32 of which rows [0, n_uniq) are written.  dU is [T,F] in the context
 * dtype.  dE_rows and dU may both be NULL to run only the integer part. */
stem_status stem_embed_grad(stem_ctx* ctx, const int32_t* ids, const void* dU, int64_t T,
                            int32_t* sorted_ids, int32_t* perm, int32_t* uniq_ids,
                            int32_t* seg_offsets, int32_t* n_uniq, float* dE_rows, void* stream);

/* The floating-point half of stem_embed_grad alone, for a batch whose integer half is there
 * already: a call of stem_embed_grad with dU == NULL and the same T on this context, which also
 * leaves the run index of every sorted position in the context (until the next stem_embed_grad call).
 * The integer half depends on the token ids only, so a caller can enqueue it early, on another
 * stream, while the layer's products run, and call this one when dU exists; ordering the two calls
 * (an event the second stream waits on) is the caller's business.  perm, seg_offsets: as written by
 * that call.  dE_rows, dU: as in stem_embed_grad.  STEM_ERR_INVALID_ARG if T differs from that call's. */
stem_status stem_embed_grad_presorted(stem_ctx* ctx, const void* dU, int64_t T, const int32_t* perm,
                                      const int32_t* seg_offsets, float* dE_rows, void* stream);

/* stem_embed_grad for callers that cannot allocate device memory: code under HIP graph capture,
 * serving loops and harnesses that forbid hipMalloc.  It needs no context: the scratch that
 * stem_embed_grad takes from its context (run indices, sort buffers, partial sums of runs that
 * cross chunk borders) lives in one static device array of about 33 MiB that every GPU the library
 * runs on holds from the moment the library is loaded until the process ends.  The call allocates
 * and frees nothing.  It works on the CURRENT device (hipSetDevice is the caller's business); its
 * first call on a device looks the array's address up (make that call outside a stream capture).
 * dtype, vocab, d_ff: as in stem_layer_desc (d_ff a multiple of 8 for STEM_BF16, of 4 for STEM_F32).
 * All other arguments and all results are those of stem_embed_grad.  id_flag (device int32, may be
 * NULL) is set to 1 when an id outside [0, vocab) is seen (such ids are clamped as everywhere); it is
 * never cleared by the library, and with NULL the report is lost.
 * Limits: T <= STEM_NOALLOC_MAX_TOKENS and, when dE_rows is wanted, ceil(T/32) * 8 * d_ff bytes of
 * partial sums <= STEM_NOALLOC_PART_BYTES (T * d_ff <= 2^27: the 1B-shaped layer at 16384 tokens just
 * fits); larger calls return STEM_ERR_SHAPE with the limit in stem_last_error(NULL).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race; calls on one stream, or ordered by events, are safe.  Nothing in the array has
 * to be cleared between calls: every word a call reads it has written itself. */
#define STEM_NOALLOC_MAX_TOKENS 65536
#define STEM_NOALLOC_PART_BYTES (32u << 20)
stem_status stem_embed_grad_noalloc(int32_t dtype, int32_t vocab, int32_t d_ff, const int32_t* ids,
                                    const void* dU, int64_t T, int32_t* sorted_ids, int32_t* perm,
                                    int32_t* uniq_ids, int32_t* seg_offsets, int32_t* n_uniq, float* dE_rows,
                                    int32_t* id_flag, void* stream);

/* ---- optimiser: AdamW on the touched rows only --------------------------------- */

/* For each j < *n_uniq, row r = uniq_ids[j], element-wise with g = dE_rows[j]:
 *   m <- b1 m + (1-b1) g ;  v <- b2 v + (1-b2) g^2
 *   p <- p - lr*wd*p - lr * (m/(1-b1^step)) / (sqrt(v/(1-b2^step)) + eps)
 * p is master[r] (fp32).  For STEM_BF16, E[r] receives p rounded to nearest-even
 * bfloat16; for STEM_F32 `master` may be NULL and E itself is p.  m, v [V,F] fp32.
 * Rows not listed are not read or written.  uniq_ids, n_uniq: device, as produced by
 * stem_embed_grad; max_rows = capacity of uniq_ids / dE_rows (rows).  hp: host.
 * E, master, m, v may also live in pinned host memory (hipHostMalloc; training with a
 * host-resident table, System Implementation): the kernel then reads the touched rows of
 * master, m, v over the host link and writes them and the bf16 row back in the same pass,
 * so nothing but the touched rows ever moves.  Rows of E that a device-side copy or cache
 * holds (E_compact, the LFU cache) are not refreshed by this call. */
stem_status stem_embed_sparse_adamw(stem_ctx* ctx, const int32_t* uniq_ids, const int32_t* n_uniq,
                                    int64_t max_rows, const float* dE_rows, void* E, float* master,
                                    float* m, float* v, const stem_adamw_hparams* hp, void* stream);

/* ---- the layers STEM is compared with, through the same kernels (Background, SwiGLU FFN
 *      equation; appendix, the additive variant) ------------------------------------ */

/* y = (SiLU(x W_gate^T) * (x W_up^T + E[ids])) W_down^T;  with E == NULL (ids unused) the
 * dense SwiGLU FFN y = (SiLU(x W_gate^T) * (x W_up^T)) W_down^T.  W_up [F,d]; everything else
 * as in stem_ffn_forward.  save_G, save_Up, save_H: [T,F] bf16 or NULL; backward needs all
 * three.  STEM_BF16 contexts only (STEM_ERR_UNSUPPORTED otherwise); needs
 * stem_reserve(ctx, STEM_RESERVE_UP). */
stem_status stem_ffn_up_forward(stem_ctx* ctx, const void* x, const int32_t* ids, const void* W_gate,
                                const void* W_up, const void* W_down, const void* E, int64_t E_rows,
                                int64_t T, void* y, void* save_G, void* save_Up, void* save_H, void* stream);

/* Gradients of the above for upstream dy [T,d].  With v = x W_up^T (+ E[ids]):
 *   dH = dy W_down;  dV = dH * SiLU(G);  dG = dH * v * SiLU'(G);
 *   dx = dG W_gate + dV W_up;  dW_gate = dG^T x;  dW_up = dV^T x;  dW_down = dy^T H.
 * dV [T,F] bf16 is the gradient of the up projection's output and, when E is given, of
 * each token's gathered row: stem_embed_grad(ids, dV) then yields the table's gradient.
 * dx may be NULL.  dW_* fp32, overwritten unless accumulate != 0. */
stem_status stem_ffn_up_backward(stem_ctx* ctx, const void* dy, const void* x, const int32_t* ids,
                                 const void* W_gate, const void* W_up, const void* W_down, const void* E,
                                 int64_t E_rows, const void* saved_G, const void* saved_Up,
                                 const void* saved_H, int64_t T, void* dx, float* dW_gate, float* dW_up,
                                 float* dW_down, void* dV, int accumulate, void* stream);

/* ---- host-resident table (System Implementation: CPU offloading, asynchronous
 *      prefetch, token de-duplication) ------------------------------------------- */

/* E_host [V,F] lives in pinned host memory (hipHostMalloc); ids_host [T] is host memory.
 * De-duplicates ids on the host (distinct ids ascending), copies row uniq[j] of E_host to
 * E_compact[j] (device, capacity `cap` rows) on the context's side stream (rows travel in
 * the order in which the tokens first use them), and writes
 * remap[i] = j with uniq[j] == ids[i] (device [T]) there too, so that
 *   stem_ffn_forward(E = E_compact, ids = remap, E_rows = *n_uniq_host, wait_event = *ready_event)
 * is the same layer.  *n_uniq_host (host) is valid on return; uniq_ids_host (host, may be
 * NULL, capacity cap) receives the distinct ids.  *ready_event is a hipEvent_t owned by
 * the context, recorded after the copies, valid until the next stem_prefetch_rows call.
 * Returns STEM_ERR_WORKSPACE if there are more than cap distinct ids, STEM_ERR_ID_RANGE if
 * an id is outside [0, V).  Blocks only for the host-side de-duplication. */
stem_status stem_prefetch_rows(stem_ctx* ctx, const void* E_host, const int32_t* ids_host, int64_t T,
                               void* E_compact, int64_t cap, int32_t* remap, int64_t* n_uniq_host,
                               int32_t* uniq_ids_host, void** ready_event);

/* How stem_prefetch_rows moves the rows (a set-up call; the default is STEM_PREFETCH_KERNEL).
 *   STEM_PREFETCH_KERNEL  a copy kernel on the side stream reads the pinned table directly, row by row in
 *                         order of first use; the call blocks only for the host-side de-duplication.
 *   STEM_PREFETCH_MEMCPY  the form the paper's system section describes: the distinct rows are packed into
 *                         pinned staging by host threads and sent with hipMemcpyAsync, 32 MiB at a time,
 *                         packing one piece while the previous one is on the link.  The call then blocks
 *                         until the last piece has been packed (it waits on the copies of earlier pieces),
 *                         and the forward call waits for the whole copy, not chunk by chunk.  Switching to
 *                         it allocates the 64 MiB of staging. */
typedef enum { STEM_PREFETCH_KERNEL = 0, STEM_PREFETCH_MEMCPY = 1 } stem_prefetch_mode;
stem_status stem_set_prefetch_mode(stem_ctx* ctx, int mode);

/* Host-resident table with a cache of the most frequently used rows on the device (System
 * Implementation: LFU cache of hot rows, only misses are prefetched).
 *
 * stem_cache_init gives the context an empty cache of n_slots rows (0 removes it) and zero
 * frequency counts; the bookkeeping is on the host, the rows live in the caller's buffer
 * E_dev [n_slots + cap, F]: rows [0, n_slots) are cache slots, the rest is the staging area
 * of one batch.  E_dev must stay the same buffer from call to call, and a batch's forward
 * must have finished before the next stem_prefetch_rows_cached call overwrites the staging.
 *
 * stem_prefetch_rows_cached: counts every token of ids_host, maps each distinct id to its
 * cache slot (hit) or to staging row n_slots + k, k numbering the misses in order of first
 * use, copies the missed rows from E_host there on the side stream, writes remap (device
 * [T]) so that stem_ffn_forward(E = E_dev, ids = remap, E_rows = n_slots + cap,
 * wait_event = *ready_event) is the same layer, and then updates the cache for later
 * batches: the missed rows are offered in order (frequency descending, id ascending); each
 * takes a free slot (lowest first) or replaces the least frequent cached row this batch
 * did not use (frequency ascending, id ascending) if it is strictly more frequent; the
 * first candidate that fails ends the update; promoted rows are copied from their staging
 * rows on the device.  *n_uniq_host, *n_miss_host (host) are valid on return.
 * STEM_ERR_WORKSPACE if more than cap rows miss; STEM_ERR_ID_RANGE for an id outside [0, V).
 * stem_cache_state copies the table row held by each slot (-1 = free) to host memory. */
stem_status stem_cache_init(stem_ctx* ctx, int64_t n_slots);
stem_status stem_prefetch_rows_cached(stem_ctx* ctx, const void* E_host, const int32_t* ids_host, int64_t T,
                                      void* E_dev, int64_t cap, int32_t* remap, int64_t* n_uniq_host,
                                      int64_t* n_miss_host, void** ready_event);
stem_status stem_cache_state(stem_ctx* ctx, int32_t* id_in_slot_host, int64_t n_slots);

/* ---- knowledge editing (the paper's editing of STEM embeddings: the rows of a source
 *      entity's tokens are replaced by rows of a target entity's tokens) ------------ */

typedef enum {
  STEM_EDIT_REPLACE = 0,  /* n_s == n_t: source token j receives target token j's row */
  STEM_EDIT_PAD_LEFT = 1, /* n_s >= n_t: the target sequence padded on the left with pad_id */
  STEM_EDIT_COPY = 2,     /* n_s >= n_t: each target token floor(n_s/n_t) times, the last repeated to fill */
  STEM_EDIT_AVERAGE = 3   /* any lengths: every source token receives the mean of the target rows */
} stem_edit_mode;

/* Overwrites rows E[src_ids[j]], j < n_s, of one layer's table (device, [V,F], context dtype).
 * All replacement rows are read from the table as it was before the call, so sources and
 * targets may overlap (a swap is two one-to-one calls' worth in one).  backup (device,
 * [n_s,F], may be NULL) receives the old source rows; writing them back undoes the edit.
 * src_ids, tgt_ids: host memory, at most 64 tokens each.  The mean is taken in fp32 and
 * rounded to the table's dtype.  Needs stem_reserve(ctx, STEM_RESERVE_EDIT).  When n_s < n_t the caller chooses which target tokens to
 * keep (the paper selects them by hand) and passes that subset.  Waits for `stream` once
 * (the index upload is synchronous); the row kernels run on `stream`.  Applies to one
 * table: call it for every STEM layer's table to edit a model. */
stem_status stem_edit_rows(stem_ctx* ctx, void* E, const int32_t* src_ids, int64_t n_s, const int32_t* tgt_ids,
                           int64_t n_t, int mode, int32_t pad_id, void* backup, void* stream);

/* ---- measurement aid ------------------------------------------------------------ */

/* With profiling on, every kernel launch of the context is bracketed by HIP events on
 * the launch stream (the first stem_profile_enable(ctx, 1) creates the events: a set-up call).  stem_profile_read synchronises the device, adds the elapsed time
 * of every recorded launch to per-kernel totals, and returns kernel `k`'s name, total
 * milliseconds and launch count (k in [0, stem_profile_kernels())).  Reset clears totals. */
stem_status stem_profile_enable(stem_ctx* ctx, int on);
int stem_profile_kernels(void);
stem_status stem_profile_read(stem_ctx* ctx, int k, const char** name, double* total_ms, int64_t* launches);
stem_status stem_profile_reset(stem_ctx* ctx);

/* What this GPU sustains on the two resources the layer's kernels are priced against (the roofline
 * denominators stay the published peaks; these say how much of them is reachable on the box at hand).
 *   STEM_PEAK_MFMA_BF16: a loop of independent 32x32x16 bf16 MFMAs on register operands; *result in TFLOP/s.
 *                        buf_a: device memory (practically never written).
 *   STEM_PEAK_MFMA_BF16_DATA: the same number of MFMAs per wavefront, arranged as the 4 x 4 outer product of
 *                        fragments of a GEMM wave tile, on operands read from buf_a (its first 64 KiB, taken as
 *                        bf16 values: fill it with the data of interest, e.g. unit normals); buf_b: 4 bytes or
 *                        more (practically never written).  The rate depends on the data: the more operand bits
 *                        toggle, the more power the matrix cores draw and the lower the clock the chip sustains.
 *   STEM_PEAK_HBM_READ:  streaming read of buf_a [bytes]; *result in GB/s of bytes read.
 *   STEM_PEAK_HBM_COPY:  streaming copy buf_a -> buf_b [bytes each]; *result in GB/s of bytes read plus written.
 * Runs the kernel once untimed and `repeats` times between HIP events on `stream`, waits for each, and
 * reports the best run.  Works on the current device; needs no context; bytes (the size of buf_a, and of buf_b for
 * the copy) is a multiple of 16 and at least 65536.  result: host. */
typedef enum { STEM_PEAK_MFMA_BF16 = 0, STEM_PEAK_HBM_READ = 1, STEM_PEAK_HBM_COPY = 2, STEM_PEAK_MFMA_BF16_DATA = 3 } stem_peak_kind;
stem_status stem_measure_peak(int what, void* buf_a, void* buf_b, int64_t bytes, int repeats, void* stream,
                              double* result);

#ifdef __cplusplus
}
#endif
#endif /* STEM_H */
