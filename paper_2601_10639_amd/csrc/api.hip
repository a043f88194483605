// libstem C ABI: argument checks, the context's scratch, and the launch sequences of
// the STEM layer's forward, backward, table-gradient, optimiser and prefetch calls.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <thread>
#include <vector>

#include "stem_internal.h"

namespace {

char g_create_err[512] = "";

const char* const kKernelNames[K_COUNT_] = {
    "gemm_gate_fused", "gemm_gate_plain", "gemm_down",    "gemm_dh_fused", "gemm_dx",      "gemm_dw_down",
    "gemm_dw_gate",    "silu_gather",     "dh_epilogue",  "sort_count",    "sort_scan",    "sort_scatter",
    "sort_fused",      "unique",          "seg_reduce",   "seg_combine",   "sparse_adamw", "row_copy",
    "splitk_reduce",   "gemm_up",      "gemm_dw_up"};

#define fail stem_fail

#define HIP_TRY(c, expr)                                                                     \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return fail((c), STEM_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),  \
                  __FILE__, __LINE__);                                                       \
  } while (0)

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline size_t esize(const stem_ctx* c) { return c->desc.dtype == STEM_BF16 ? 2 : 4; }

// Common entry checks; returns STEM_OK to proceed.
stem_status enter(stem_ctx* c, int64_t T) {
  if (!c) return STEM_ERR_INVALID_ARG;
  if (T < 0) return fail(c, STEM_ERR_SHAPE, "T = %lld is negative", (long long)T);
  if (T > c->max_tokens)
    return fail(c, STEM_ERR_SHAPE, "T = %lld exceeds the context's max_tokens = %lld", (long long)T,
                (long long)c->max_tokens);
  hipError_t e = hipSetDevice(c->device);
  if (e != hipSuccess) return fail(c, STEM_ERR_HIP, "hipSetDevice(%d): %s", c->device, hipGetErrorString(e));
  if (*reinterpret_cast<volatile int32_t*>(c->flag)) {
    *reinterpret_cast<volatile int32_t*>(c->flag) = 0;
    return fail(c, STEM_ERR_ID_RANGE, "an earlier call saw a token id outside [0, E_rows)");
  }
  return STEM_OK;
}

template <typename T>
hipError_t dmalloc(T** p, size_t n) {
  *p = nullptr;
  if (n == 0) n = 1;
  return hipMalloc(reinterpret_cast<void**>(p), n * sizeof(T));
}

void release(stem_ctx* c) {
  if (!c) return;
  (void)hipSetDevice(c->device);
  (void)hipDeviceSynchronize();
  (void)hipFree(c->H_ws); (void)hipFree(c->dG_ws); (void)hipFree(c->dH_ws);
  (void)hipFree(c->splitk_ws); (void)hipFree(c->dw_ws);
  (void)hipFree(c->Up_ws);
  for (int i = 0; i < 2; ++i) { (void)hipFree(c->sort_keys[i]); (void)hipFree(c->sort_vals[i]); }
  (void)hipFree(c->sort_counts); (void)hipFree(c->seg_of); (void)hipFree(c->seg_part);
  (void)hipFree(c->uniq_dev);
  (void)hipFree(c->order_dev);
  if (c->order_pinned) (void)hipHostFree(c->order_pinned);
  for (int i = 0; i < STEM_PF_MAX_CHUNKS; ++i)
    if (c->pf_ev[i]) (void)hipEventDestroy(c->pf_ev[i]);
  if (c->flag) (void)hipHostFree(c->flag);
  if (c->uniq_pinned) (void)hipHostFree(c->uniq_pinned);
  if (c->remap_pinned) (void)hipHostFree(c->remap_pinned);
  if (c->pack_pinned) (void)hipHostFree(c->pack_pinned);
  free(c->slot);
  free(c->cache_id_in_slot); free(c->cache_slot_of); free(c->cache_freq);
  (void)hipFree(c->edit_idx_dev); (void)hipFree(c->edit_rep_dev);
  if (c->inst_pinned) (void)hipHostFree(c->inst_pinned);
  (void)hipFree(c->inst_dev);
  if (c->side) (void)hipStreamDestroy(c->side);
  if (c->ready) (void)hipEventDestroy(c->ready);
  for (int i = 0; i < 2; ++i) if (c->pack_done[i]) (void)hipEventDestroy(c->pack_done[i]);
  if (c->prof_ev) {
    for (int i = 0; i < 2 * STEM_MAX_PROF_EVENTS; ++i) if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
    free(c->prof_ev);
  }
  free(c);
}

EmbedScratch embed_scratch(const stem_ctx* c) {
  EmbedScratch w;
  w.sort_keys[0] = c->sort_keys[0]; w.sort_keys[1] = c->sort_keys[1];
  w.sort_vals[0] = c->sort_vals[0]; w.sort_vals[1] = c->sort_vals[1];
  w.sort_counts = c->sort_counts; w.seg_of = c->seg_of; w.seg_part = c->seg_part; w.flag = c->flag;
  return w;
}

}  // namespace

stem_status stem_fail(stem_ctx* c, stem_status st, const char* fmt, ...) {
  char* buf = c ? c->err : g_create_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, 512, fmt, ap);
  va_end(ap);
  return st;
}

extern "C" {

const char* stem_status_string(stem_status s) {
  switch (s) {
    case STEM_OK: return "STEM_OK";
    case STEM_ERR_INVALID_ARG: return "STEM_ERR_INVALID_ARG";
    case STEM_ERR_SHAPE: return "STEM_ERR_SHAPE";
    case STEM_ERR_ID_RANGE: return "STEM_ERR_ID_RANGE";
    case STEM_ERR_WORKSPACE: return "STEM_ERR_WORKSPACE";
    case STEM_ERR_UNSUPPORTED: return "STEM_ERR_UNSUPPORTED";
    case STEM_ERR_HIP: return "STEM_ERR_HIP";
  }
  return "STEM_ERR_?";
}

const char* stem_last_error(const stem_ctx* ctx) { return ctx ? ctx->err : g_create_err; }

stem_status stem_create(stem_ctx** out, const stem_layer_desc* desc, int64_t max_tokens, int device) {
  if (out) *out = nullptr;
  if (!out || !desc) return fail(nullptr, STEM_ERR_INVALID_ARG, "stem_create: null argument");
  if (desc->dtype != STEM_F32 && desc->dtype != STEM_BF16)
    return fail(nullptr, STEM_ERR_INVALID_ARG, "stem_create: dtype %d is not a stem_dtype", desc->dtype);
  if (desc->d_model <= 0 || desc->d_ff <= 0 || desc->vocab <= 0 || max_tokens < 0 || max_tokens > (1ll << 30))
    return fail(nullptr, STEM_ERR_SHAPE, "stem_create: d_model=%d d_ff=%d vocab=%d max_tokens=%lld", desc->d_model,
                desc->d_ff, desc->vocab, (long long)max_tokens);
  const int mult = desc->dtype == STEM_BF16 ? 64 : 4;
  if (desc->d_model % mult || desc->d_ff % mult)
    return fail(nullptr, STEM_ERR_UNSUPPORTED, "stem_create: d_model=%d and d_ff=%d must be multiples of %d",
                desc->d_model, desc->d_ff, mult);
  // The bf16 kernels address every operand and output of a product through 32-bit buffer offsets:
  // activations [max_tokens, d_ff], weights and fp32 weight gradients [d_ff, d_model] must each stay
  // below 2 GiB.  (The table is addressed with 64-bit pointers and has no such limit.)
  const int64_t lim = 0x7fffffff;
  if (desc->dtype == STEM_BF16 &&
      ((int64_t)max_tokens * std::max(desc->d_ff, desc->d_model) * 2 > lim || (int64_t)desc->d_ff * desc->d_model * 4 > lim))
    return fail(nullptr, STEM_ERR_SHAPE,
                "stem_create: max_tokens * max(d_ff, d_model) * 2 bytes = %lld and d_ff * d_model * 4 bytes = %lld must each "
                "stay below 2^31 (32-bit buffer offsets); split the batch",
                (long long)max_tokens * std::max(desc->d_ff, desc->d_model) * 2, (long long)desc->d_ff * desc->d_model * 4);
  if ((int64_t)max_tokens * desc->d_ff >= (1ll << 40))
    return fail(nullptr, STEM_ERR_SHAPE, "stem_create: max_tokens * d_ff too large");
  HIP_TRY(nullptr, hipSetDevice(device));

  stem_ctx* c = static_cast<stem_ctx*>(calloc(1, sizeof(stem_ctx)));
  if (!c) return fail(nullptr, STEM_ERR_HIP, "stem_create: out of host memory");
  c->desc = *desc;
  c->max_tokens = max_tokens;
  c->device = device;
  const size_t es = esize(c);
  const size_t TF = (size_t)max_tokens * desc->d_ff;
  hipError_t e = hipSuccess;
  auto ok = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  ok(hipMalloc(&c->H_ws, std::max<size_t>(TF * es, 16)));
  ok(hipMalloc(&c->dG_ws, std::max<size_t>(TF * es, 16)));
  if (desc->dtype == STEM_F32) ok(hipMalloc(&c->dH_ws, std::max<size_t>(TF * 4, 16)));
  if (desc->dtype == STEM_BF16) {
    ok(hipMalloc(reinterpret_cast<void**>(&c->splitk_ws), STEM_SPLITK_WS_BYTES));
    // Weight gradients are [d,F] outputs with K = T: a narrow layer has fewer 256x256 tiles than the
    // chip has compute units, so its K range is cut into slices (at most 8, at most ~256 workgroups).
    const int dw_tiles = ((desc->d_model + 255) / 256) * ((desc->d_ff + 255) / 256);
    c->dw_ksplit = 1;
    while (c->dw_ksplit < 8 && dw_tiles * c->dw_ksplit * 2 <= 256) c->dw_ksplit *= 2;
    if (c->dw_ksplit > 1)
      ok(hipMalloc(reinterpret_cast<void**>(&c->dw_ws), (size_t)c->dw_ksplit * desc->d_model * desc->d_ff * 4));
  }
  for (int i = 0; i < 2; ++i) {
    ok(dmalloc(&c->sort_keys[i], (size_t)max_tokens));
    ok(dmalloc(&c->sort_vals[i], (size_t)max_tokens));
  }
  ok(dmalloc(&c->sort_counts, (size_t)stem_sort_count_entries(std::max<int64_t>(max_tokens, 1))));
  ok(dmalloc(&c->seg_of, (size_t)max_tokens));
  ok(dmalloc(&c->seg_part, (size_t)stem_seg_chunks(std::max<int64_t>(max_tokens, 1)) * 2 * desc->d_ff));
  ok(dmalloc(&c->uniq_dev, (size_t)max_tokens));
  ok(dmalloc(&c->order_dev, 2 * (size_t)max_tokens));
  ok(hipHostMalloc(reinterpret_cast<void**>(&c->order_pinned), std::max<size_t>(max_tokens, 1) * 8, hipHostMallocDefault));
  for (int i = 0; i < STEM_PF_MAX_CHUNKS; ++i) ok(hipEventCreateWithFlags(&c->pf_ev[i], hipEventDisableTiming));
  ok(hipHostMalloc(reinterpret_cast<void**>(&c->flag), 64, hipHostMallocDefault));
  ok(hipHostMalloc(reinterpret_cast<void**>(&c->uniq_pinned), std::max<size_t>(max_tokens, 1) * 4, hipHostMallocDefault));
  ok(hipHostMalloc(reinterpret_cast<void**>(&c->remap_pinned), std::max<size_t>(max_tokens, 1) * 4, hipHostMallocDefault));
  ok(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
  ok(hipEventCreateWithFlags(&c->ready, hipEventDisableTiming));
  for (int i = 0; i < 2; ++i) ok(hipEventCreateWithFlags(&c->pack_done[i], hipEventDisableTiming));
  c->slot = static_cast<int32_t*>(malloc((size_t)desc->vocab * 4));
  if (e != hipSuccess || !c->slot) {
    snprintf(g_create_err, sizeof g_create_err, "stem_create: allocation failed: %s",
             e != hipSuccess ? hipGetErrorString(e) : "host malloc");
    release(c);
    return STEM_ERR_HIP;
  }
  memset(c->slot, 0xff, (size_t)desc->vocab * 4);
  c->seg_T = -1;
  *c->flag = 0;
  c->err[0] = 0;
  *out = c;
  return STEM_OK;
}

void stem_destroy(stem_ctx* ctx) { release(ctx); }

stem_status stem_reserve(stem_ctx* c, uint32_t what) {
  if (!c) return STEM_ERR_INVALID_ARG;
  if (what & ~(uint32_t)(STEM_RESERVE_UP | STEM_RESERVE_EDIT))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_reserve: unknown bits in 0x%x", what);
  HIP_TRY(c, hipSetDevice(c->device));
  if ((what & STEM_RESERVE_UP) && !c->Up_ws) {
    if (c->desc.dtype != STEM_BF16) return fail(c, STEM_ERR_UNSUPPORTED, "stem_reserve: STEM_RESERVE_UP needs a bf16 context");
    HIP_TRY(c, hipMalloc(&c->Up_ws, std::max<size_t>((size_t)c->max_tokens * c->desc.d_ff * 2, 16)));
  }
  if ((what & STEM_RESERVE_EDIT) && !c->edit_idx_dev) {
    HIP_TRY(c, hipMalloc(reinterpret_cast<void**>(&c->edit_idx_dev), 3 * STEM_EDIT_MAX_TOKENS * sizeof(int32_t)));
    HIP_TRY(c, hipMalloc(&c->edit_rep_dev, (size_t)STEM_EDIT_MAX_TOKENS * c->desc.d_ff * esize(c)));
  }
  return STEM_OK;
}

stem_status stem_set_prefetch_mode(stem_ctx* c, int mode) {
  if (!c) return STEM_ERR_INVALID_ARG;
  if (mode != STEM_PREFETCH_KERNEL && mode != STEM_PREFETCH_MEMCPY)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_set_prefetch_mode: unknown mode %d", mode);
  if (mode == STEM_PREFETCH_MEMCPY && !c->pack_pinned) {
    const size_t row_bytes = (size_t)c->desc.d_ff * esize(c);
    HIP_TRY(c, hipSetDevice(c->device));
    c->pack_bytes = std::max<size_t>((size_t)64 << 20, 2 * row_bytes);
    HIP_TRY(c, hipHostMalloc(reinterpret_cast<void**>(&c->pack_pinned), c->pack_bytes, hipHostMallocDefault));
  }
  c->prefetch_mode = mode;
  return STEM_OK;
}

stem_status stem_sync_status(stem_ctx* c, void* stream) {
  if (!c) return STEM_ERR_INVALID_ARG;
  HIP_TRY(c, hipSetDevice(c->device));
  HIP_TRY(c, hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  if (*reinterpret_cast<volatile int32_t*>(c->flag)) {
    *reinterpret_cast<volatile int32_t*>(c->flag) = 0;
    return fail(c, STEM_ERR_ID_RANGE, "a kernel saw a token id outside [0, E_rows)");
  }
  return STEM_OK;
}

static stem_status forward_impl(stem_ctx* c, const void* x, const int32_t* ids, const void* W_gate,
                                const void* W_down, const void* E, int64_t E_rows, int64_t T, void* y,
                                void* save_G, void* save_H, void* wait_event, const void* residual, void* stream) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (T == 0) return STEM_OK;
  if (!x || !ids || !W_gate || !W_down || !E || !y)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_forward: null pointer argument");
  if (misaligned(x) || misaligned(W_gate) || misaligned(W_down) || misaligned(E) || misaligned(y) ||
      misaligned(save_G) || misaligned(save_H) || misaligned(residual) || (reinterpret_cast<uintptr_t>(ids) & 3u))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_forward: pointers must be 16-byte aligned");
  if (E_rows < 1 || E_rows > INT32_MAX) return fail(c, STEM_ERR_SHAPE, "stem_ffn_forward: E_rows = %lld", (long long)E_rows);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int d = c->desc.d_model, F = c->desc.d_ff;
  void* H = save_H ? save_H : c->H_ws;

  if (c->desc.dtype == STEM_BF16) {
    GemmArgs a = {};
    a.A = static_cast<const bf16_t*>(x); a.lda = d;
    a.B = static_cast<const bf16_t*>(W_gate); a.ldb = d;
    a.M = (int)T; a.N = F; a.K = d;
    a.ids = ids; a.E = static_cast<const bf16_t*>(E); a.E_rows = (int)E_rows; a.flag = c->flag;
    // A decode-sized call (a few hundred tokens) takes the few-row kernel: 128x64 tiles, the down
    // product split along K so that both launches fill the chip.
    const bool few = T <= STEM_SKINNY_MAX_M;
    GemmArgs b = {};
    b.A = static_cast<const bf16_t*>(H); b.lda = F;
    b.B = static_cast<const bf16_t*>(W_down); b.ldb = F;
    b.M = (int)T; b.N = d; b.K = F; b.C = y; b.flag = c->flag;
    b.residual = static_cast<const bf16_t*>(residual);
    const int down_epi = residual ? EPI_BF16_RES : EPI_BF16;
    if (!wait_event) {
      a.outG = static_cast<bf16_t*>(save_G); a.outH = static_cast<bf16_t*>(H);
      if (few) HIP_TRY(c, stem_gemm_skinny_bf16(c, K_GEMM_GATE, EPI_GATE, a, s));
      else HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_GATE, OP_KC, OP_KC, EPI_GATE, a, s));
    } else {
      void* G = save_G ? save_G : c->dG_ws;
      a.C = G;
      if (few) HIP_TRY(c, stem_gemm_skinny_bf16(c, K_GEMM_GATE_PLAIN, EPI_BF16, a, s));
      else HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_GATE_PLAIN, OP_KC, OP_KC, EPI_BF16, a, s));
      if (wait_event == c->ready && c->pf_chunks > 1 && c->pf_T == T) {
        // Rows arrive in order of first use: run the gather and the down product chunk by chunk,
        // each as soon as the rows its tokens need are there, the later rows still on the link.
        for (int k = 0; k < c->pf_chunks; ++k) {
          const int64_t t0 = k * c->pf_chunk_tokens, tn = std::min(c->pf_chunk_tokens, T - t0);
          HIP_TRY(c, hipStreamWaitEvent(s, c->pf_ev[k], 0));
          HIP_TRY(c, stem_silu_gather(c, 1, static_cast<const bf16_t*>(G) + t0 * F, ids + t0, E, (int)E_rows,
                                      static_cast<bf16_t*>(H) + t0 * F, tn, F, s));
          GemmArgs bk = b;
          bk.A = static_cast<const bf16_t*>(H) + t0 * F;
          bk.C = static_cast<bf16_t*>(y) + t0 * d;
          if (residual) bk.residual = static_cast<const bf16_t*>(residual) + t0 * d;
          bk.M = (int)tn;
          HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DOWN, OP_KC, OP_KC, down_epi, bk, s));
        }
        return STEM_OK;
      }
      HIP_TRY(c, hipStreamWaitEvent(s, static_cast<hipEvent_t>(wait_event), 0));
      HIP_TRY(c, stem_silu_gather(c, 1, G, ids, E, (int)E_rows, H, T, F, s));
    }
    if (few) {
      b.ksplit = stem_gemm_skinny_ksplit(b.M, b.N, b.K);
      b.ws = c->splitk_ws;
      if ((size_t)b.ksplit * b.M * b.N * 4 > STEM_SPLITK_WS_BYTES) b.ksplit = 1;
      HIP_TRY(c, stem_gemm_skinny_bf16(c, K_GEMM_DOWN, b.ksplit > 1 ? EPI_SPLITK : EPI_BF16, b, s));
    } else {
      HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DOWN, OP_KC, OP_KC, down_epi, b, s));
    }
  } else {
    float* G = static_cast<float*>(save_G ? save_G : c->dG_ws);
    HIP_TRY(c, stem_sgemm(c, wait_event ? K_GEMM_GATE_PLAIN : K_GEMM_GATE, static_cast<const float*>(x), d, 1,
                          static_cast<const float*>(W_gate), d, 1, G, (int)T, F, d, 0, s));
    if (wait_event) HIP_TRY(c, hipStreamWaitEvent(s, static_cast<hipEvent_t>(wait_event), 0));
    HIP_TRY(c, stem_silu_gather(c, 0, G, ids, E, (int)E_rows, H, T, F, s));
    // with a residual the product is added to it: y starts as a copy of the residual unless it is the same buffer
    if (residual && residual != y)
      HIP_TRY(c, hipMemcpyAsync(y, residual, (size_t)T * d * 4, hipMemcpyDeviceToDevice, s));
    HIP_TRY(c, stem_sgemm(c, K_GEMM_DOWN, static_cast<const float*>(H), F, 1, static_cast<const float*>(W_down), F,
                          1, static_cast<float*>(y), (int)T, d, F, residual ? 1 : 0, s));
  }
  return STEM_OK;
}

stem_status stem_ffn_forward(stem_ctx* c, const void* x, const int32_t* ids, const void* W_gate,
                             const void* W_down, const void* E, int64_t E_rows, int64_t T, void* y,
                             void* save_G, void* save_H, void* wait_event, void* stream) {
  return forward_impl(c, x, ids, W_gate, W_down, E, E_rows, T, y, save_G, save_H, wait_event, nullptr, stream);
}

stem_status stem_ffn_forward_residual(stem_ctx* c, const void* x, const int32_t* ids, const void* W_gate,
                                      const void* W_down, const void* E, int64_t E_rows, int64_t T,
                                      const void* residual, void* y, void* stream) {
  if (c && !residual) return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_forward_residual: null residual");
  return forward_impl(c, x, ids, W_gate, W_down, E, E_rows, T, y, nullptr, nullptr, nullptr, residual, stream);
}

stem_status stem_ffn_backward(stem_ctx* c, const void* dy, const void* x, const int32_t* ids,
                              const void* W_gate, const void* W_down, const void* E, int64_t E_rows,
                              const void* saved_G, const void* saved_H, int64_t T, void* dx, float* dW_gate,
                              float* dW_down, void* dU, int accumulate, void* stream) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (!dW_gate || !dW_down) return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_backward: null weight-gradient pointer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int d = c->desc.d_model, F = c->desc.d_ff;
  if (T == 0) {
    if (!accumulate) {
      HIP_TRY(c, stem_fill_zero(dW_gate, (size_t)F * d * 4, s));
      HIP_TRY(c, stem_fill_zero(dW_down, (size_t)F * d * 4, s));
    }
    return STEM_OK;
  }
  if (!dy || !x || !ids || !W_gate || !W_down || !E || !saved_G || !dU)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_backward: null pointer argument");
  if (misaligned(dy) || misaligned(x) || misaligned(W_gate) || misaligned(W_down) || misaligned(E) ||
      misaligned(saved_G) || misaligned(saved_H) || misaligned(dx) || misaligned(dW_gate) ||
      misaligned(dW_down) || misaligned(dU) || (reinterpret_cast<uintptr_t>(ids) & 3u))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_backward: pointers must be 16-byte aligned");
  if (E_rows < 1 || E_rows > INT32_MAX) return fail(c, STEM_ERR_SHAPE, "stem_ffn_backward: E_rows = %lld", (long long)E_rows);

  const void* H = saved_H;
  if (!H) {
    HIP_TRY(c, stem_silu_gather(c, c->desc.dtype == STEM_BF16, saved_G, ids, E, (int)E_rows, c->H_ws, T, F, s));
    H = c->H_ws;
  }
  if (c->desc.dtype == STEM_BF16) {
    const bf16_t* dyb = static_cast<const bf16_t*>(dy);
    const bf16_t* Hb = static_cast<const bf16_t*>(H);
    bf16_t* dGb = static_cast<bf16_t*>(c->dG_ws);
    int dw_split = c->dw_ksplit;   // K slices of the weight-gradient GEMMs: at least 8 K tiles each
    while (dw_split > 1 && (T + 63) / 64 / dw_split < 8) dw_split /= 2;
    // Every operand is read as it is stored.  The weights of the two activation-gradient products
    // ([K, N] with N contiguous) and both operands of the weight-gradient products ([T, rows]) are
    // rows-contiguous: their tiles go to LDS unchanged and the fragment reads transpose them.
    {  // dH = dy W_down, fused into dU and dG
      GemmArgs a = {};
      a.A = dyb; a.lda = d; a.B = static_cast<const bf16_t*>(W_down); a.ldb = F;
      a.M = (int)T; a.N = F; a.K = d;
      a.ids = ids; a.E = static_cast<const bf16_t*>(E); a.E_rows = (int)E_rows; a.flag = c->flag;
      a.inG = static_cast<const bf16_t*>(saved_G); a.outdU = static_cast<bf16_t*>(dU); a.outdG = dGb;
      HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DH, OP_KC, OP_MC, EPI_DH, a, s));
    }
    {  // dW_down[d,F] = dy^T H
      GemmArgs a = {};
      a.A = dyb; a.lda = d; a.B = Hb; a.ldb = F;
      a.M = d; a.N = F; a.K = (int)T; a.C = dW_down; a.accumulate = accumulate; a.flag = c->flag;
      a.ksplit = dw_split; a.ws = c->dw_ws;
      HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DWDOWN, OP_MC, OP_MC, EPI_F32, a, s));
    }
    if (dx) {  // dx = dG W_gate
      GemmArgs a = {};
      a.A = dGb; a.lda = F; a.B = static_cast<const bf16_t*>(W_gate); a.ldb = d;
      a.M = (int)T; a.N = d; a.K = F; a.C = dx; a.flag = c->flag;
      HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DX, OP_KC, OP_MC, EPI_BF16, a, s));
    }
    {  // dW_gate[F,d] = dG^T x
      GemmArgs a = {};
      a.A = dGb; a.lda = F; a.B = static_cast<const bf16_t*>(x); a.ldb = d;
      a.M = F; a.N = d; a.K = (int)T; a.C = dW_gate; a.accumulate = accumulate; a.flag = c->flag;
      a.ksplit = dw_split; a.ws = c->dw_ws;
      HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DWGATE, OP_MC, OP_MC, EPI_F32, a, s));
    }
  } else {
    const float* dyf = static_cast<const float*>(dy);
    const float* Hf = static_cast<const float*>(H);
    const float* Wg = static_cast<const float*>(W_gate);
    const float* Wd = static_cast<const float*>(W_down);
    float* dH = static_cast<float*>(c->dH_ws);
    float* dG = static_cast<float*>(c->dG_ws);
    HIP_TRY(c, stem_sgemm(c, K_GEMM_DH, dyf, d, 1, Wd, 1, F, dH, (int)T, F, d, 0, s));
    HIP_TRY(c, stem_dh_epilogue_f32(c, dH, static_cast<const float*>(saved_G), ids, static_cast<const float*>(E),
                                    (int)E_rows, static_cast<float*>(dU), dG, T, F, s));
    HIP_TRY(c, stem_sgemm(c, K_GEMM_DWDOWN, dyf, 1, d, Hf, 1, F, dW_down, d, F, (int)T, accumulate, s));
    if (dx) HIP_TRY(c, stem_sgemm(c, K_GEMM_DX, dG, F, 1, Wg, 1, d, static_cast<float*>(dx), (int)T, d, F, 0, s));
    HIP_TRY(c, stem_sgemm(c, K_GEMM_DWGATE, dG, 1, F, static_cast<const float*>(x), 1, d, dW_gate, F, d, (int)T,
                          accumulate, s));
  }
  return STEM_OK;
}

// ---- dense SwiGLU FFN and the additive variant through the same kernels ---------------------------

static stem_status up_scratch(stem_ctx* c) {
  // these two entry points need one more [max_tokens, F] activation, which
  // stem_reserve(ctx, STEM_RESERVE_UP) allocates
  if (!c->Up_ws)
    return fail(c, STEM_ERR_WORKSPACE, "the dense and additive variants need stem_reserve(ctx, STEM_RESERVE_UP) first");
  return STEM_OK;
}

stem_status stem_ffn_up_forward(stem_ctx* c, const void* x, const int32_t* ids, const void* W_gate, const void* W_up,
                                const void* W_down, const void* E, int64_t E_rows, int64_t T, void* y, void* save_G,
                                void* save_Up, void* save_H, void* stream) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (c->desc.dtype != STEM_BF16) return fail(c, STEM_ERR_UNSUPPORTED, "stem_ffn_up_forward: bf16 contexts only");
  if (T == 0) return STEM_OK;
  if (!x || !W_gate || !W_up || !W_down || !y || (E && !ids))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_up_forward: null pointer argument");
  if (misaligned(x) || misaligned(W_gate) || misaligned(W_up) || misaligned(W_down) || misaligned(E) || misaligned(y) ||
      misaligned(save_G) || misaligned(save_Up) || misaligned(save_H) || (reinterpret_cast<uintptr_t>(ids) & 3u))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_up_forward: pointers must be 16-byte aligned");
  if (E && (E_rows < 1 || E_rows > INT32_MAX))
    return fail(c, STEM_ERR_SHAPE, "stem_ffn_up_forward: E_rows = %lld", (long long)E_rows);
  st = up_scratch(c);
  if (st != STEM_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int d = c->desc.d_model, F = c->desc.d_ff;
  void* H = save_H ? save_H : c->H_ws;
  void* Up = save_Up ? save_Up : c->Up_ws;
  GemmArgs u = {};   // Up = x W_up^T
  u.A = static_cast<const bf16_t*>(x); u.lda = d;
  u.B = static_cast<const bf16_t*>(W_up); u.ldb = d;
  u.M = (int)T; u.N = F; u.K = d; u.C = Up; u.flag = c->flag;
  HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_UP, OP_KC, OP_KC, EPI_BF16, u, s));
  GemmArgs a = u;    // G = x W_gate^T;  H = SiLU(G) * (Up [+ E[ids]])
  a.B = static_cast<const bf16_t*>(W_gate); a.C = nullptr;
  a.ids = ids; a.E = static_cast<const bf16_t*>(E); a.E_rows = (int)E_rows;
  a.inUp = static_cast<const bf16_t*>(Up);
  a.outG = static_cast<bf16_t*>(save_G); a.outH = static_cast<bf16_t*>(H);
  HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_GATE, OP_KC, OP_KC, E ? EPI_GATE_UPE : EPI_GATE_UP, a, s));
  GemmArgs b = {};   // y = H W_down^T
  b.A = static_cast<const bf16_t*>(H); b.lda = F;
  b.B = static_cast<const bf16_t*>(W_down); b.ldb = F;
  b.M = (int)T; b.N = d; b.K = F; b.C = y; b.flag = c->flag;
  HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DOWN, OP_KC, OP_KC, EPI_BF16, b, s));
  return STEM_OK;
}

stem_status stem_ffn_up_backward(stem_ctx* c, const void* dy, const void* x, const int32_t* ids, const void* W_gate,
                                 const void* W_up, const void* W_down, const void* E, int64_t E_rows,
                                 const void* saved_G, const void* saved_Up, const void* saved_H, int64_t T, void* dx,
                                 float* dW_gate, float* dW_up, float* dW_down, void* dV, int accumulate,
                                 void* stream) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (c->desc.dtype != STEM_BF16) return fail(c, STEM_ERR_UNSUPPORTED, "stem_ffn_up_backward: bf16 contexts only");
  if (!dW_gate || !dW_up || !dW_down)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_up_backward: null weight-gradient pointer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int d = c->desc.d_model, F = c->desc.d_ff;
  if (T == 0) {
    if (!accumulate) {
      HIP_TRY(c, stem_fill_zero(dW_gate, (size_t)F * d * 4, s));
      HIP_TRY(c, stem_fill_zero(dW_up, (size_t)F * d * 4, s));
      HIP_TRY(c, stem_fill_zero(dW_down, (size_t)F * d * 4, s));
    }
    return STEM_OK;
  }
  if (!dy || !x || !W_gate || !W_up || !W_down || !saved_G || !saved_Up || !saved_H || !dV || (E && !ids))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_up_backward: null pointer argument");
  if (misaligned(dy) || misaligned(x) || misaligned(W_gate) || misaligned(W_up) || misaligned(W_down) ||
      misaligned(E) || misaligned(saved_G) || misaligned(saved_Up) || misaligned(saved_H) || misaligned(dx) ||
      misaligned(dW_gate) || misaligned(dW_up) || misaligned(dW_down) || misaligned(dV) ||
      (reinterpret_cast<uintptr_t>(ids) & 3u))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_ffn_up_backward: pointers must be 16-byte aligned");
  if (E && (E_rows < 1 || E_rows > INT32_MAX))
    return fail(c, STEM_ERR_SHAPE, "stem_ffn_up_backward: E_rows = %lld", (long long)E_rows);
  st = up_scratch(c);
  if (st != STEM_OK) return st;

  const bf16_t* dyb = static_cast<const bf16_t*>(dy);
  bf16_t* dGb = static_cast<bf16_t*>(c->dG_ws);
  bf16_t* dVb = static_cast<bf16_t*>(dV);
  int dw_split = c->dw_ksplit;
  while (dw_split > 1 && (T + 63) / 64 / dw_split < 8) dw_split /= 2;
  {  // dH = dy W_down, fused into dV = dH * SiLU(G) and dG = dH * (Up [+ E[ids]]) * SiLU'(G)
    GemmArgs a = {};
    a.A = dyb; a.lda = d; a.B = static_cast<const bf16_t*>(W_down); a.ldb = F;
    a.M = (int)T; a.N = F; a.K = d;
    a.ids = ids; a.E = static_cast<const bf16_t*>(E); a.E_rows = (int)E_rows; a.flag = c->flag;
    a.inG = static_cast<const bf16_t*>(saved_G); a.inUp = static_cast<const bf16_t*>(saved_Up);
    a.outdU = dVb; a.outdG = dGb;
    HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DH, OP_KC, OP_MC, E ? EPI_DH_UPE : EPI_DH_UP, a, s));
  }
  {  // dW_down[d,F] = dy^T H
    GemmArgs a = {};
    a.A = dyb; a.lda = d; a.B = static_cast<const bf16_t*>(saved_H); a.ldb = F;
    a.M = d; a.N = F; a.K = (int)T; a.C = dW_down; a.accumulate = accumulate; a.flag = c->flag;
    a.ksplit = dw_split; a.ws = c->dw_ws;
    HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DWDOWN, OP_MC, OP_MC, EPI_F32, a, s));
  }
  if (dx) {  // dx = dG W_gate + dV W_up: one product over the concatenated K range
    GemmArgs a = {};
    a.A = dGb; a.lda = F; a.B = static_cast<const bf16_t*>(W_gate); a.ldb = d;
    a.A2 = dVb; a.B2 = static_cast<const bf16_t*>(W_up); a.K2 = F;
    a.M = (int)T; a.N = d; a.K = F; a.C = dx; a.flag = c->flag;
    HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DX, OP_KC, OP_MC, EPI_BF16, a, s));
  }
  {  // dW_gate[F,d] = dG^T x and dW_up[F,d] = dV^T x
    GemmArgs a = {};
    a.A = dGb; a.lda = F; a.B = static_cast<const bf16_t*>(x); a.ldb = d;
    a.M = F; a.N = d; a.K = (int)T; a.C = dW_gate; a.accumulate = accumulate; a.flag = c->flag;
    a.ksplit = dw_split; a.ws = c->dw_ws;
    HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DWGATE, OP_MC, OP_MC, EPI_F32, a, s));
    a.A = dVb; a.C = dW_up;
    HIP_TRY(c, stem_gemm_bf16(c, K_GEMM_DWUP, OP_MC, OP_MC, EPI_F32, a, s));
  }
  return STEM_OK;
}

stem_status stem_embed_grad(stem_ctx* c, const int32_t* ids, const void* dU, int64_t T, int32_t* sorted_ids,
                            int32_t* perm, int32_t* uniq_ids, int32_t* seg_offsets, int32_t* n_uniq,
                            float* dE_rows, void* stream) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (!seg_offsets || !n_uniq) return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_grad: null seg_offsets / n_uniq");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (T == 0) {
    HIP_TRY(c, stem_fill_zero(n_uniq, 4, s));
    HIP_TRY(c, stem_fill_zero(seg_offsets, 4, s));
    return STEM_OK;
  }
  if (!ids || !sorted_ids || !perm || !uniq_ids)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_grad: null pointer argument");
  if ((dU == nullptr) != (dE_rows == nullptr))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_grad: dU and dE_rows must both be given or both be NULL");
  if (misaligned(dU) || misaligned(dE_rows))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_grad: dU and dE_rows must be 16-byte aligned");
  const EmbedScratch ws = embed_scratch(c);
  HIP_TRY(c, stem_sort_unique(c, ws, ids, T, c->desc.vocab, sorted_ids, perm, uniq_ids, seg_offsets, n_uniq, s));
  c->seg_T = T;
  if (dU)
    HIP_TRY(c, stem_seg_reduce(c, ws, c->desc.dtype == STEM_BF16, dU, perm, seg_offsets, T, c->desc.d_ff, dE_rows, s));
  return STEM_OK;
}

stem_status stem_embed_grad_presorted(stem_ctx* c, const void* dU, int64_t T, const int32_t* perm,
                                      const int32_t* seg_offsets, float* dE_rows, void* stream) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (T == 0) return STEM_OK;
  if (!dU || !perm || !seg_offsets || !dE_rows)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_grad_presorted: null pointer argument");
  if (misaligned(dU) || misaligned(dE_rows))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_grad_presorted: dU and dE_rows must be 16-byte aligned");
  if (T != c->seg_T)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_grad_presorted: T = %lld, but the context's run index is that of a "
                "stem_embed_grad call with T = %lld", (long long)T, (long long)c->seg_T);
  HIP_TRY(c, stem_seg_reduce(c, embed_scratch(c), c->desc.dtype == STEM_BF16, dU, perm, seg_offsets, T, c->desc.d_ff,
                             dE_rows, static_cast<hipStream_t>(stream)));
  return STEM_OK;
}

stem_status stem_embed_sparse_adamw(stem_ctx* c, const int32_t* uniq_ids, const int32_t* n_uniq,
                                    int64_t max_rows, const float* dE_rows, void* E, float* master, float* m,
                                    float* v, const stem_adamw_hparams* hp, void* stream) {
  stem_status st = enter(c, 0);
  if (st != STEM_OK) return st;
  if (!uniq_ids || !n_uniq || !dE_rows || !E || !m || !v || !hp)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_sparse_adamw: null pointer argument");
  if (c->desc.dtype == STEM_BF16 && !master)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_sparse_adamw: the bf16 table needs an fp32 master copy");
  if (misaligned(dE_rows) || misaligned(E) || misaligned(master) || misaligned(m) || misaligned(v))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_sparse_adamw: pointers must be 16-byte aligned");
  if (max_rows < 0 || max_rows > INT32_MAX) return fail(c, STEM_ERR_SHAPE, "stem_embed_sparse_adamw: max_rows = %lld", (long long)max_rows);
  if (hp->step < 1) return fail(c, STEM_ERR_SHAPE, "stem_embed_sparse_adamw: step = %lld must be >= 1", (long long)hp->step);
  if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f && hp->beta2 >= 0.f && hp->beta2 < 1.f))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_embed_sparse_adamw: betas must lie in [0, 1)");
  HIP_TRY(c, stem_adamw(c, c->desc.dtype == STEM_BF16, uniq_ids, n_uniq, max_rows, dE_rows, E, master, m, v,
                        c->desc.d_ff, *hp, static_cast<hipStream_t>(stream)));
  return STEM_OK;
}

stem_status stem_prefetch_rows(stem_ctx* c, const void* E_host, const int32_t* ids_host, int64_t T,
                               void* E_compact, int64_t cap, int32_t* remap, int64_t* n_uniq_host,
                               int32_t* uniq_ids_host, void** ready_event) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (!E_host || (!ids_host && T > 0) || !E_compact || (!remap && T > 0) || !n_uniq_host || !ready_event)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_prefetch_rows: null pointer argument");
  if (misaligned(E_host) || misaligned(E_compact))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_prefetch_rows: tables must be 16-byte aligned");
  if (cap < 0) return fail(c, STEM_ERR_SHAPE, "stem_prefetch_rows: cap = %lld", (long long)cap);
  const int V = c->desc.vocab;
  const size_t row_bytes = (size_t)c->desc.d_ff * esize(c);

  // The pinned staging arrays are reused: wait until the previous prefetch's copies are done.
  HIP_TRY(c, hipStreamSynchronize(c->side));

  // De-duplicate: mark, then walk the marked ids in ascending order.
  for (int64_t i = 0; i < T; ++i) {
    const int32_t t = ids_host[i];
    if ((uint32_t)t >= (uint32_t)V) {
      for (int64_t k = 0; k < i; ++k) c->slot[ids_host[k]] = -1;
      return fail(c, STEM_ERR_ID_RANGE, "stem_prefetch_rows: ids[%lld] = %d is outside [0, %d)", (long long)i, t, V);
    }
    c->slot[t] = 0;
  }
  int64_t U = 0;
  if (T > 0) {
    // scanning all V slots costs O(V); sorting the marked ids costs O(U log U).  Take the cheaper.
    if ((int64_t)V <= 16 * T) {
      for (int32_t t = 0; t < V; ++t)
        if (c->slot[t] == 0) { c->slot[t] = (int32_t)U; c->uniq_pinned[U++] = t; }
    } else {
      for (int64_t i = 0; i < T; ++i) {
        const int32_t t = ids_host[i];
        if (c->slot[t] == 0) { c->slot[t] = 1; c->uniq_pinned[U++] = t; }
      }
      std::sort(c->uniq_pinned, c->uniq_pinned + U);
      for (int64_t j = 0; j < U; ++j) c->slot[c->uniq_pinned[j]] = (int32_t)j;
    }
  }
  // One pass over the tokens: the compact slot of every token, and the distinct rows in order of
  // first use, so that the rows the first tokens need cross the link first.  Long batches are cut
  // into chunks; an event after each chunk's rows lets the forward
  // call run the gather and the down product of a chunk while later rows are still on the link.
  // Chunk size: the down product of one chunk is about one round of 256x256 tiles
  // (STEM_PF_CHUNK_TILES); whole multiples of that if the batch is very long.
  const int64_t tile_cols = (c->desc.d_model + 255) / 256;
  int64_t chunk_tokens = std::max<int64_t>(1, STEM_PF_CHUNK_TILES / tile_cols) * 256;
  chunk_tokens *= std::max<int64_t>(1, ((T + chunk_tokens - 1) / chunk_tokens + STEM_PF_MAX_CHUNKS - 1) / STEM_PF_MAX_CHUNKS);
  int nchunks = (int)((T + chunk_tokens - 1) / chunk_tokens);
  if (nchunks < 2) { nchunks = 1; chunk_tokens = std::max<int64_t>(T, 1); }
  int64_t chunk_end[STEM_PF_MAX_CHUNKS] = {0};
  int32_t* src_row = c->order_pinned;
  int32_t* dst_slot = c->order_pinned + c->max_tokens;
  {
    int64_t k = 0;
    for (int64_t i = 0; i < T; ++i) {
      const int32_t t = ids_host[i];
      int32_t v = c->slot[t];
      if (v >= 0) {            // first use of this row
        src_row[k] = t;
        dst_slot[k] = v;
        ++k;
        c->slot[t] = -2 - v;   // seen; the slot stays recoverable
      } else {
        v = -2 - v;
      }
      c->remap_pinned[i] = v;
      if ((i + 1) % chunk_tokens == 0 || i + 1 == T) chunk_end[std::min<int64_t>(i / chunk_tokens, nchunks - 1)] = k;
    }
  }
  for (int64_t j = 0; j < U; ++j) c->slot[c->uniq_pinned[j]] = -1;
  *n_uniq_host = U;
  if (uniq_ids_host) memcpy(uniq_ids_host, c->uniq_pinned, (size_t)std::min<int64_t>(U, cap) * 4);
  c->pf_chunks = 0;
  if (U > cap)
    return fail(c, STEM_ERR_WORKSPACE, "stem_prefetch_rows: %lld distinct ids but E_compact holds %lld rows",
                (long long)U, (long long)cap);

  if (T > 0) HIP_TRY(c, hipMemcpyAsync(remap, c->remap_pinned, (size_t)T * 4, hipMemcpyHostToDevice, c->side));
  if (c->prefetch_mode == STEM_PREFETCH_MEMCPY) {
    // Pack the rows into pinned staging with a few host threads and copy chunk by chunk,
    // packing chunk i+1 while chunk i is on the link (staging allocated by stem_set_prefetch_mode).
    const size_t half = c->pack_bytes / 2;
    const int64_t rows_per = (int64_t)(half / row_bytes);
    const unsigned hw = std::thread::hardware_concurrency();
    const int nthr = (int)std::max(1u, std::min(8u, hw ? hw : 1u));
    int chunk = 0;
    for (int64_t j0 = 0; j0 < U; j0 += rows_per, ++chunk) {
      const int64_t nrows = std::min(rows_per, U - j0);
      char* stage = c->pack_pinned + (size_t)(chunk & 1) * half;
      if (chunk >= 2) HIP_TRY(c, hipEventSynchronize(c->pack_done[chunk & 1]));
      std::vector<std::thread> pool;
      for (int t = 0; t < nthr; ++t)
        pool.emplace_back([=]() {
          for (int64_t r = t; r < nrows; r += nthr)
            memcpy(stage + (size_t)r * row_bytes,
                   static_cast<const char*>(E_host) + (size_t)c->uniq_pinned[j0 + r] * row_bytes, row_bytes);
        });
      for (auto& th : pool) th.join();
      HIP_TRY(c, hipMemcpyAsync(static_cast<char*>(E_compact) + (size_t)j0 * row_bytes, stage,
                                (size_t)nrows * row_bytes, hipMemcpyHostToDevice, c->side));
      HIP_TRY(c, hipEventRecord(c->pack_done[chunk & 1], c->side));
    }
  } else if (U > 0) {
    HIP_TRY(c, hipMemcpyAsync(c->order_dev, src_row, (size_t)U * 4, hipMemcpyHostToDevice, c->side));
    HIP_TRY(c, hipMemcpyAsync(c->order_dev + c->max_tokens, dst_slot, (size_t)U * 4, hipMemcpyHostToDevice, c->side));
    int64_t k0 = 0;
    for (int k = 0; k < nchunks; ++k) {
      HIP_TRY(c, stem_copy_rows_kernel(c, E_host, c->order_dev + k0, c->order_dev + c->max_tokens + k0,
                                       chunk_end[k] - k0, (int64_t)row_bytes, E_compact, c->side));
      k0 = chunk_end[k];
      if (nchunks > 1) HIP_TRY(c, hipEventRecord(c->pf_ev[k], c->side));
    }
    if (nchunks > 1) { c->pf_chunks = nchunks; c->pf_T = T; c->pf_chunk_tokens = chunk_tokens; }
  }
  HIP_TRY(c, hipEventRecord(c->ready, c->side));
  *ready_event = c->ready;
  return STEM_OK;
}

// ---- host-resident table with a device-resident cache of the most frequently used rows ----------

stem_status stem_cache_init(stem_ctx* c, int64_t n_slots) {
  if (!c) return STEM_ERR_INVALID_ARG;
  if (n_slots < 0 || n_slots > INT32_MAX / 2)
    return fail(c, STEM_ERR_SHAPE, "stem_cache_init: n_slots = %lld", (long long)n_slots);
  const int V = c->desc.vocab;
  HIP_TRY(c, hipSetDevice(c->device));
  HIP_TRY(c, hipStreamSynchronize(c->side));
  free(c->cache_id_in_slot); free(c->cache_slot_of); free(c->cache_freq);
  c->cache_id_in_slot = nullptr; c->cache_slot_of = nullptr; c->cache_freq = nullptr;
  c->cache_slots = 0;
  if (n_slots == 0) return STEM_OK;
  if (!c->inst_pinned) {   // lists of promoted rows: staging row, cache slot
    HIP_TRY(c, hipHostMalloc(reinterpret_cast<void**>(&c->inst_pinned), std::max<size_t>(c->max_tokens, 1) * 8,
                             hipHostMallocDefault));
    HIP_TRY(c, hipMalloc(reinterpret_cast<void**>(&c->inst_dev), std::max<size_t>(c->max_tokens, 1) * 8));
  }
  c->cache_id_in_slot = static_cast<int32_t*>(malloc((size_t)n_slots * 4));
  c->cache_slot_of = static_cast<int32_t*>(malloc((size_t)V * 4));
  c->cache_freq = static_cast<uint32_t*>(calloc((size_t)V, 4));
  if (!c->cache_id_in_slot || !c->cache_slot_of || !c->cache_freq)
    return fail(c, STEM_ERR_HIP, "stem_cache_init: out of host memory");
  memset(c->cache_id_in_slot, 0xff, (size_t)n_slots * 4);
  memset(c->cache_slot_of, 0xff, (size_t)V * 4);
  c->cache_slots = n_slots;
  return STEM_OK;
}

stem_status stem_cache_state(stem_ctx* c, int32_t* id_in_slot_host, int64_t n) {
  if (!c || !id_in_slot_host) return STEM_ERR_INVALID_ARG;
  if (n != c->cache_slots) return fail(c, STEM_ERR_SHAPE, "stem_cache_state: n = %lld, cache has %lld slots",
                                       (long long)n, (long long)c->cache_slots);
  memcpy(id_in_slot_host, c->cache_id_in_slot, (size_t)n * 4);
  return STEM_OK;
}

stem_status stem_prefetch_rows_cached(stem_ctx* c, const void* E_host, const int32_t* ids_host, int64_t T,
                                      void* E_dev, int64_t cap, int32_t* remap, int64_t* n_uniq_host,
                                      int64_t* n_miss_host, void** ready_event) {
  stem_status st = enter(c, T);
  if (st != STEM_OK) return st;
  if (c->cache_slots <= 0) return fail(c, STEM_ERR_INVALID_ARG, "stem_prefetch_rows_cached: call stem_cache_init first");
  if (!E_host || (!ids_host && T > 0) || !E_dev || (!remap && T > 0) || !n_uniq_host || !n_miss_host || !ready_event)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_prefetch_rows_cached: null pointer argument");
  if (misaligned(E_host) || misaligned(E_dev))
    return fail(c, STEM_ERR_INVALID_ARG, "stem_prefetch_rows_cached: tables must be 16-byte aligned");
  if (cap < 0) return fail(c, STEM_ERR_SHAPE, "stem_prefetch_rows_cached: cap = %lld", (long long)cap);
  const int V = c->desc.vocab;
  const int64_t NS = c->cache_slots;
  const size_t row_bytes = (size_t)c->desc.d_ff * esize(c);
  HIP_TRY(c, hipStreamSynchronize(c->side));   // pinned staging arrays are reused

  for (int64_t i = 0; i < T; ++i)
    if ((uint32_t)ids_host[i] >= (uint32_t)V)
      return fail(c, STEM_ERR_ID_RANGE, "stem_prefetch_rows_cached: ids[%lld] = %d is outside [0, %d)", (long long)i,
                  ids_host[i], V);

  // One pass over the tokens.  c->slot marks the ids of this batch (-1 = not seen yet) and holds the
  // row each one reads: its cache slot, or a staging row behind the cache, numbered in order of
  // first use so that the rows the first tokens need cross the link first.
  const int64_t tile_cols = (c->desc.d_model + 255) / 256;
  int64_t chunk_tokens = std::max<int64_t>(1, STEM_PF_CHUNK_TILES / tile_cols) * 256;
  chunk_tokens *= std::max<int64_t>(1, ((T + chunk_tokens - 1) / chunk_tokens + STEM_PF_MAX_CHUNKS - 1) / STEM_PF_MAX_CHUNKS);
  int nchunks = (int)((T + chunk_tokens - 1) / chunk_tokens);
  if (nchunks < 2) { nchunks = 1; chunk_tokens = std::max<int64_t>(T, 1); }
  int64_t chunk_end[STEM_PF_MAX_CHUNKS] = {0};
  int32_t* src_row = c->order_pinned;
  int32_t* dst_row = c->order_pinned + c->max_tokens;
  int64_t U = 0, n_miss = 0;
  for (int64_t i = 0; i < T; ++i) {
    const int32_t t = ids_host[i];
    c->cache_freq[t] += 1;
    int32_t v = c->slot[t];
    if (v < 0) {   // first use in this batch
      c->uniq_pinned[U++] = t;
      v = c->cache_slot_of[t];
      if (v < 0) {
        v = (int32_t)(NS + n_miss);
        if (n_miss < c->max_tokens) { src_row[n_miss] = t; dst_row[n_miss] = v; }
        ++n_miss;
      }
      c->slot[t] = v;
    }
    c->remap_pinned[i] = v;
    if ((i + 1) % chunk_tokens == 0 || i + 1 == T) chunk_end[std::min<int64_t>(i / chunk_tokens, nchunks - 1)] = n_miss;
  }
  *n_uniq_host = U;
  *n_miss_host = n_miss;
  c->pf_chunks = 0;
  if (n_miss > cap) {
    for (int64_t j = 0; j < U; ++j) c->slot[c->uniq_pinned[j]] = -1;
    return fail(c, STEM_ERR_WORKSPACE, "stem_prefetch_rows_cached: %lld rows missed the cache but the staging area holds %lld",
                (long long)n_miss, (long long)cap);
  }

  if (T > 0) HIP_TRY(c, hipMemcpyAsync(remap, c->remap_pinned, (size_t)T * 4, hipMemcpyHostToDevice, c->side));
  if (n_miss > 0) {
    HIP_TRY(c, hipMemcpyAsync(c->order_dev, src_row, (size_t)n_miss * 4, hipMemcpyHostToDevice, c->side));
    HIP_TRY(c, hipMemcpyAsync(c->order_dev + c->max_tokens, dst_row, (size_t)n_miss * 4, hipMemcpyHostToDevice, c->side));
  }
  {
    int64_t k0 = 0;
    for (int k = 0; k < nchunks; ++k) {
      HIP_TRY(c, stem_copy_rows_kernel(c, E_host, c->order_dev + k0, c->order_dev + c->max_tokens + k0,
                                       chunk_end[k] - k0, (int64_t)row_bytes, E_dev, c->side));
      k0 = chunk_end[k];
      if (nchunks > 1) HIP_TRY(c, hipEventRecord(c->pf_ev[k], c->side));
    }
    if (nchunks > 1) { c->pf_chunks = nchunks; c->pf_T = T; c->pf_chunk_tokens = chunk_tokens; }
  }
  HIP_TRY(c, hipEventRecord(c->ready, c->side));
  *ready_event = c->ready;

  // Cache update for the batches to come (least frequently used): the rows missed now are offered
  // in order (frequency descending, id ascending); each takes a free slot (lowest first) or replaces
  // the coldest cached row this batch did not use (frequency ascending, id ascending) if it is
  // strictly more frequent; the first candidate that fails ends the update.  A promoted row is
  // copied device-to-device from its staging row, behind this batch's copies on the side stream.
  struct Ent { uint32_t f; int32_t id; int32_t aux; };
  std::vector<int32_t> free_slots;
  std::vector<Ent> cold, cand;
  uint32_t fmax = 0;
  for (int64_t k = 0; k < n_miss; ++k) fmax = std::max(fmax, c->cache_freq[src_row[k]]);
  uint32_t cold_min = UINT32_MAX;
  for (int64_t sidx = 0; sidx < NS; ++sidx) {
    const int32_t t = c->cache_id_in_slot[sidx];
    if (t < 0) { free_slots.push_back((int32_t)sidx); continue; }
    if (c->slot[t] >= 0) continue;                 // used by this batch: stays
    const uint32_t f = c->cache_freq[t];
    cold_min = std::min(cold_min, f);
    if (f < fmax) cold.push_back({f, t, (int32_t)sidx});   // only these can lose to a candidate
  }
  for (int64_t k = 0; k < n_miss; ++k) {
    const uint32_t f = c->cache_freq[src_row[k]];
    if (!free_slots.empty() || f > cold_min) cand.push_back({f, src_row[k], (int32_t)k});
  }
  std::sort(cand.begin(), cand.end(), [](const Ent& a, const Ent& b) { return a.f != b.f ? a.f > b.f : a.id < b.id; });
  {  // only the coldest |cand| rows can be replaced: select them, then order them
    auto colder = [](const Ent& a, const Ent& b) { return a.f != b.f ? a.f < b.f : a.id < b.id; };
    if (cold.size() > cand.size()) {
      std::nth_element(cold.begin(), cold.begin() + cand.size(), cold.end(), colder);
      cold.resize(cand.size());
    }
    std::sort(cold.begin(), cold.end(), colder);
  }
  int64_t n_inst = 0;
  size_t nf = 0, nc = 0;
  for (const Ent& e : cand) {
    int32_t sidx;
    if (nf < free_slots.size()) {
      sidx = free_slots[nf++];
    } else if (nc < cold.size() && e.f > cold[nc].f) {
      sidx = cold[nc].aux;
      c->cache_slot_of[cold[nc].id] = -1;
      ++nc;
    } else {
      break;
    }
    c->cache_id_in_slot[sidx] = e.id;
    c->cache_slot_of[e.id] = sidx;
    c->inst_pinned[n_inst] = (int32_t)(NS + e.aux);        // staging row that holds it
    c->inst_pinned[c->max_tokens + n_inst] = sidx;         // cache slot it moves to
    ++n_inst;
  }
  for (int64_t j = 0; j < U; ++j) c->slot[c->uniq_pinned[j]] = -1;
  if (n_inst > 0) {
    HIP_TRY(c, hipMemcpyAsync(c->inst_dev, c->inst_pinned, (size_t)n_inst * 4, hipMemcpyHostToDevice, c->side));
    HIP_TRY(c, hipMemcpyAsync(c->inst_dev + c->max_tokens, c->inst_pinned + c->max_tokens, (size_t)n_inst * 4,
                              hipMemcpyHostToDevice, c->side));
    HIP_TRY(c, stem_copy_rows_kernel(c, E_dev, c->inst_dev, c->inst_dev + c->max_tokens, n_inst, (int64_t)row_bytes,
                                     E_dev, c->side));
  }
  return STEM_OK;
}

// ---- knowledge editing: rows of a source entity's tokens replaced by a target entity's -----------

stem_status stem_edit_rows(stem_ctx* c, void* E, const int32_t* src_ids_host, int64_t n_s,
                           const int32_t* tgt_ids_host, int64_t n_t, int mode, int32_t pad_id, void* backup,
                           void* stream) {
  if (!c) return STEM_ERR_INVALID_ARG;
  if (!E || !src_ids_host || !tgt_ids_host)
    return fail(c, STEM_ERR_INVALID_ARG, "stem_edit_rows: null pointer argument");
  if (n_s < 1 || n_t < 1 || n_s > STEM_EDIT_MAX_TOKENS || n_t > STEM_EDIT_MAX_TOKENS)
    return fail(c, STEM_ERR_SHAPE, "stem_edit_rows: n_s = %lld, n_t = %lld must lie in [1, %d]", (long long)n_s,
                (long long)n_t, STEM_EDIT_MAX_TOKENS);
  const int V = c->desc.vocab;
  int32_t idx[3 * STEM_EDIT_MAX_TOKENS];
  int32_t* src = idx;
  int32_t* pick = idx + STEM_EDIT_MAX_TOKENS;
  int32_t* tgt = idx + 2 * STEM_EDIT_MAX_TOKENS;
  for (int64_t j = 0; j < n_s; ++j) {
    if ((uint32_t)src_ids_host[j] >= (uint32_t)V)
      return fail(c, STEM_ERR_ID_RANGE, "stem_edit_rows: source id %d is outside [0, %d)", src_ids_host[j], V);
    src[j] = src_ids_host[j];
  }
  for (int64_t k = 0; k < n_t; ++k) {
    if ((uint32_t)tgt_ids_host[k] >= (uint32_t)V)
      return fail(c, STEM_ERR_ID_RANGE, "stem_edit_rows: target id %d is outside [0, %d)", tgt_ids_host[k], V);
    tgt[k] = tgt_ids_host[k];
  }
  // which target token's row each source position receives (-1 = the mean of all target rows)
  if (mode == STEM_EDIT_REPLACE) {
    if (n_s != n_t) return fail(c, STEM_ERR_SHAPE, "stem_edit_rows: one-to-one replacement needs n_s == n_t");
    for (int64_t j = 0; j < n_s; ++j) pick[j] = tgt[j];
  } else if (mode == STEM_EDIT_PAD_LEFT || mode == STEM_EDIT_COPY) {
    if (n_s < n_t) return fail(c, STEM_ERR_SHAPE, "stem_edit_rows: padding and copying need n_s >= n_t");
    if (mode == STEM_EDIT_PAD_LEFT) {
      if ((uint32_t)pad_id >= (uint32_t)V)
        return fail(c, STEM_ERR_ID_RANGE, "stem_edit_rows: pad id %d is outside [0, %d)", pad_id, V);
      for (int64_t j = 0; j < n_s; ++j) pick[j] = j < n_s - n_t ? pad_id : tgt[j - (n_s - n_t)];
    } else {   // every target token floor(n_s / n_t) times, the last one as often as it takes
      const int64_t r = n_s / n_t;
      for (int64_t j = 0; j < n_s; ++j) pick[j] = tgt[std::min<int64_t>(j / r, n_t - 1)];
    }
  } else if (mode == STEM_EDIT_AVERAGE) {
    for (int64_t j = 0; j < n_s; ++j) pick[j] = -1;
  } else {
    return fail(c, STEM_ERR_INVALID_ARG, "stem_edit_rows: unknown mode %d", mode);
  }
  HIP_TRY(c, hipSetDevice(c->device));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!c->edit_idx_dev)
    return fail(c, STEM_ERR_WORKSPACE, "stem_edit_rows needs stem_reserve(ctx, STEM_RESERVE_EDIT) first");
  // the index lists are small and this call is rare: a synchronous upload keeps the host array on the stack
  HIP_TRY(c, hipStreamSynchronize(s));
  HIP_TRY(c, hipMemcpy(c->edit_idx_dev, idx, sizeof(idx), hipMemcpyHostToDevice));
  HIP_TRY(c, stem_edit_launch(c, c->desc.dtype == STEM_BF16, E, c->edit_idx_dev, c->edit_idx_dev + STEM_EDIT_MAX_TOKENS,
                              c->edit_idx_dev + 2 * STEM_EDIT_MAX_TOKENS, (int)n_s, (int)n_t, c->desc.d_ff,
                              c->edit_rep_dev, backup, s));
  return STEM_OK;
}

stem_status stem_profile_enable(stem_ctx* c, int on) {
  if (!c) return STEM_ERR_INVALID_ARG;
  if (on && !c->prof_ev) {
    HIP_TRY(c, hipSetDevice(c->device));
    c->prof_ev = static_cast<hipEvent_t*>(calloc(2 * STEM_MAX_PROF_EVENTS, sizeof(hipEvent_t)));
    if (!c->prof_ev) return fail(c, STEM_ERR_HIP, "stem_profile_enable: out of host memory");
    for (int i = 0; i < 2 * STEM_MAX_PROF_EVENTS; ++i) HIP_TRY(c, hipEventCreate(&c->prof_ev[i]));
  }
  c->prof_on = on ? 1 : 0;
  return STEM_OK;
}

int stem_profile_kernels(void) { return K_COUNT_; }

static stem_status prof_collect(stem_ctx* c) {
  if (c->prof_n == 0) return STEM_OK;
  HIP_TRY(c, hipSetDevice(c->device));
  HIP_TRY(c, hipDeviceSynchronize());
  for (int i = 0; i < c->prof_n; ++i) {
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
    c->prof_ms[c->prof_kid[i]] += ms;
    c->prof_launches[c->prof_kid[i]] += 1;
  }
  c->prof_n = 0;
  return STEM_OK;
}

stem_status stem_profile_read(stem_ctx* c, int k, const char** name, double* total_ms, int64_t* launches) {
  if (!c || k < 0 || k >= K_COUNT_) return STEM_ERR_INVALID_ARG;
  stem_status st = prof_collect(c);
  if (st != STEM_OK) return st;
  if (name) *name = kKernelNames[k];
  if (total_ms) *total_ms = c->prof_ms[k];
  if (launches) *launches = c->prof_launches[k];
  return STEM_OK;
}

stem_status stem_profile_reset(stem_ctx* c) {
  if (!c) return STEM_ERR_INVALID_ARG;
  stem_status st = prof_collect(c);
  for (int k = 0; k < K_COUNT_; ++k) { c->prof_ms[k] = 0; c->prof_launches[k] = 0; }
  return st;
}

}  // extern "C"
