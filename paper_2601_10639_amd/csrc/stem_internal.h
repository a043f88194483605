// Internal declarations shared by libstem's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/stem.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits

// ---- kernel ids for the profiling table -----------------------------------------
enum StemKernelId {
  K_GEMM_GATE = 0,   // G = X Wg^T with fused SiLU*gather epilogue
  K_GEMM_GATE_PLAIN, // G = X Wg^T, plain store (host-resident table mode)
  K_GEMM_DOWN,       // Y = H Wd^T
  K_GEMM_DH,         // dH = dY Wd with fused dU/dG epilogue
  K_GEMM_DX,         // dX = dG Wg
  K_GEMM_DWDOWN,     // dWd = dY^T H
  K_GEMM_DWGATE,     // dWg = dG^T X
  K_SILU_GATHER,     // H = SiLU(G) * E[ids] (stand-alone)
  K_DH_EPILOGUE,     // fp32 path: dU, dG from dH
  K_SORT_COUNT,
  K_SORT_SCAN,
  K_SORT_SCATTER,
  K_SORT_FUSED,
  K_UNIQUE,
  K_SEG_REDUCE,
  K_SEG_COMBINE,
  K_ADAMW,
  K_ROW_COPY,        // host-resident rows -> compact device table
  K_SPLITK_REDUCE,   // sum of split-K partial products
  K_GEMM_UP,         // Up = X Wu^T (dense SwiGLU and the additive variant)
  K_GEMM_DWUP,       // dWu = dV^T X
  K_COUNT_
};

#define STEM_MAX_PROF_EVENTS 8192
#define STEM_PF_MAX_CHUNKS 16
#define STEM_EDIT_MAX_TOKENS 64
#define STEM_PF_CHUNK_TILES 256     // one round of 256x256 down-product tiles per chunk (measured better than 224 and 512)

struct stem_ctx {
  stem_layer_desc desc;
  int64_t max_tokens;
  int device;
  char err[512];

  // scratch, all device memory unless noted
  void* H_ws;            // [max_tokens, F] context dtype
  void* dG_ws;           // [max_tokens, F] context dtype
  void* dH_ws;           // [max_tokens, F] fp32, STEM_F32 only
  void* Up_ws;           // [max_tokens, F] bf16, allocated by the first stem_ffn_up_* call
  float* splitk_ws;      // STEM_SPLITK_WS_BYTES: fp32 partial products of the few-row GEMMs
  float* dw_ws;          // [dw_ksplit][d*F] fp32 partial weight gradients, when the layer is narrow
  int dw_ksplit;         // K slices of the weight-gradient GEMMs (1 = no split)
  int32_t* sort_keys[2]; // [max_tokens]
  int32_t* sort_vals[2]; // [max_tokens]
  int32_t* sort_counts;  // [64 * waves]
  int32_t* seg_of;       // [max_tokens] index of the segment each sorted position is in
  int64_t seg_T;         // T of the call that last wrote seg_of (-1 = none)
  float* seg_part;       // [chunks][2][F] partial sums of segments that cross chunk borders
  int32_t* flag;         // pinned host int, device-visible: sticky id-range flag

  // host-resident table mode
  hipStream_t side;
  hipEvent_t ready;
  int32_t* slot;         // host [V], -1 = absent
  int32_t* uniq_pinned;  // pinned host [max_tokens]
  int32_t* remap_pinned; // pinned host [max_tokens]
  int32_t* uniq_dev;     // device [max_tokens]
  int32_t* order_pinned; // pinned host [2 * max_tokens]: table row, then compact slot, in order of first use
  int32_t* order_dev;    // device [2 * max_tokens]
  // chunks of the last prefetch: tokens [k * pf_chunk_tokens, ...) need only rows copied before pf_ev[k]
  int pf_chunks;         // 0 = the last prefetch recorded no per-chunk events
  int64_t pf_T, pf_chunk_tokens;
  hipEvent_t pf_ev[STEM_PF_MAX_CHUNKS];
  int prefetch_mode;     // STEM_PREFETCH_KERNEL or STEM_PREFETCH_MEMCPY
  char* pack_pinned;     // pinned host staging for the memcpy mode
  size_t pack_bytes;
  hipEvent_t pack_done[2];

  // device-resident cache of hot rows in host-resident mode (host-side bookkeeping; the rows
  // themselves live in the caller's buffer)
  int64_t cache_slots;       // 0 = no cache
  int32_t* cache_id_in_slot; // host [cache_slots], -1 = free
  int32_t* cache_slot_of;    // host [V], -1 = not cached
  uint32_t* cache_freq;      // host [V]: token occurrences seen so far
  int32_t* inst_pinned;      // pinned host [2 * max_tokens]: promoted rows (staging row, then cache slot)
  int32_t* inst_dev;         // device [2 * max_tokens]

  // knowledge editing: device scratch for up to STEM_EDIT_MAX_TOKENS source / target tokens
  int32_t* edit_idx_dev;     // [3 * STEM_EDIT_MAX_TOKENS]: source rows, picked rows, target rows
  void* edit_rep_dev;        // [STEM_EDIT_MAX_TOKENS, F] replacement rows

  // profiling
  int prof_on;
  hipEvent_t* prof_ev;   // 2 * STEM_MAX_PROF_EVENTS
  int prof_kid[STEM_MAX_PROF_EVENTS];
  int prof_n;
  double prof_ms[K_COUNT_];
  int64_t prof_launches[K_COUNT_];
};

// Brackets a launch with events when profiling is on.
struct ProfScope {
  stem_ctx* c;
  hipStream_t s;
  int idx;
  ProfScope(stem_ctx* ctx, int kid, hipStream_t st) : c(ctx), s(st), idx(-1) {
    if (c && c->prof_on && c->prof_n < STEM_MAX_PROF_EVENTS) {
      idx = c->prof_n++;
      c->prof_kid[idx] = kid;
      (void)hipEventRecord(c->prof_ev[2 * idx], s);
    }
  }
  ~ProfScope() {
    if (idx >= 0) (void)hipEventRecord(c->prof_ev[2 * idx + 1], s);
  }
};

// ---- bf16 MFMA GEMM family (gemm_bf16.hip) ---------------------------------------
// C[m,n] = sum_k Aop[m,k] * Bop[n,k].  An operand is "KC" when stored [rows, K] with K
// contiguous, "MC" when stored [K, rows] with rows contiguous.
enum { OP_KC = 0, OP_MC = 1 };
enum GemmEpilogue {
  EPI_BF16 = 0, // C -> bf16 [M,N]
  EPI_F32,      // C -> fp32 [M,N], optional +=
  EPI_GATE,     // G (optional) and H = SiLU(C) * E[ids[m], n], both bf16
  EPI_DH,       // dU = C * SiLU(G), dG = C * E[ids[m], n] * SiLU'(G), both bf16
  EPI_SPLITK,   // few-row kernel only: fp32 partial products per k slice, summed into bf16 C
  // dense SwiGLU (UP) and the additive variant (UPE): SiLU(C) is multiplied by Up or Up + E[ids]
  EPI_GATE_UP, EPI_GATE_UPE,
  EPI_DH_UP, EPI_DH_UPE,
  EPI_BF16_RES  // C + residual -> bf16 [M,N] (decode chains: the layer's output joins the residual stream)
};

struct GemmArgs {
  const bf16_t* A; // M-side operand
  const bf16_t* B; // N-side operand
  int M, N, K;
  int lda, ldb;    // leading dimensions of the stored operands
  void* C;         // EPI_BF16 / EPI_F32 output, ld = N
  const bf16_t* residual;  // EPI_BF16_RES (and the few-row kernel when not null): [M,N] bf16 added in fp32 before rounding
  int accumulate;  // EPI_F32: add to C
  const int32_t* ids;
  const bf16_t* E;
  int E_rows;
  bf16_t* outG;    // EPI_GATE: may be null
  bf16_t* outH;    // EPI_GATE
  const bf16_t* inUp; // *_UP, *_UPE: the up projection x W_up^T, [M,N] bf16
  const bf16_t* A2;  // optional second operand pair of a (KC,KC) product: C = A B^T + A2 B2^T
  const bf16_t* B2;
  int K2;
  const bf16_t* inG; // EPI_DH
  bf16_t* outdU;   // EPI_DH
  bf16_t* outdG;   // EPI_DH
  int32_t* flag;
  float* ws;       // split-K launches: [ksplit][M][N] fp32 partial products
  int ksplit;      // number of k slices (few-row kernel: EPI_SPLITK; large kernel: EPI_F32 with ksplit > 1)
  int kc_skip;     // set by the large kernel itself: elements a K slice starts after the operand's start
  int mt, nt;      // few-row kernel: tile counts and exact float reciprocals, filled in by the launcher
  float inv_mt, inv_per_z;
};

hipError_t stem_gemm_bf16(stem_ctx* ctx, int kid, int la, int lb, int epi, const GemmArgs& a, hipStream_t s);

// ---- few-row bf16 GEMM (gemm_skinny_bf16.hip): both operands K-contiguous, K % 64 == 0 --------
// 128x64 tiles; used when M is small enough that 256x256 tiles would leave most of the chip idle.
#define STEM_SKINNY_MAX_M 512
#define STEM_SPLITK_WS_BYTES ((size_t)8 << 20)   // >= ksplit * M * N * 4 whenever ksplit > 1
// k slices that bring the launch to about one workgroup per compute unit (1 = no split)
int stem_gemm_skinny_ksplit(int M, int N, int K);
// epi: EPI_BF16, EPI_GATE, or EPI_SPLITK (a.ksplit slices through a.ws, then summed into a.C)
hipError_t stem_gemm_skinny_bf16(stem_ctx* ctx, int kid, int epi, const GemmArgs& a, hipStream_t s);

// ---- fp32 path and element-wise kernels (kernels_f32.hip) -------------------------
// C[m,n] (+)= sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk]
hipError_t stem_sgemm(stem_ctx* ctx, int kid, const float* A, int64_t sam, int64_t sak, const float* B,
                      int64_t sbn, int64_t sbk, float* C, int M, int N, int K, int accumulate, hipStream_t s);
// out[c,r] = in[r,c] (bf16), leading dimension ldo, zero padding beyond R
hipError_t stem_fill_zero(void* p, size_t bytes, hipStream_t s);   // a kernel, not a memset node
// H = SiLU(G) * E[ids]; is_bf16 selects the element type of G, E, H
hipError_t stem_silu_gather(stem_ctx* ctx, int is_bf16, const void* G, const int32_t* ids, const void* E,
                            int E_rows, void* H, int64_t T, int F, hipStream_t s);
// fp32: dU = dH * SiLU(G); dG = dH * E[ids] * SiLU'(G)
hipError_t stem_dh_epilogue_f32(stem_ctx* ctx, const float* dH, const float* G, const int32_t* ids,
                                const float* E, int E_rows, float* dU, float* dG, int64_t T, int F,
                                hipStream_t s);

// ---- table gradient (embed_grad.hip) ----------------------------------------------
// Device scratch of the sort and the segmented sum: a context's own buffers, or pieces of the
// library's static scratch array (the entry point that allocates nothing).
struct EmbedScratch {
  int32_t* sort_keys[2]; // [T] each (multi-kernel sort only)
  int32_t* sort_vals[2]; // [T] each
  int32_t* sort_counts;  // [stem_sort_count_entries(T)]
  int32_t* seg_of;       // [T] index of the run each sorted position is in
  float* seg_part;       // [stem_seg_chunks(T)][2][F] partial sums of runs that cross chunk borders
  int32_t* flag;         // sticky id-range flag (host-pinned or device)
};
hipError_t stem_sort_unique(stem_ctx* prof, const EmbedScratch& ws, const int32_t* ids, int64_t T, int V,
                            int32_t* sorted_ids, int32_t* perm, int32_t* uniq_ids, int32_t* seg_offsets,
                            int32_t* n_uniq, hipStream_t s);
hipError_t stem_seg_reduce(stem_ctx* prof, const EmbedScratch& ws, int is_bf16, const void* dU, const int32_t* perm,
                           const int32_t* seg_offsets, int64_t T, int F, float* dE_rows, hipStream_t s);
int64_t stem_seg_chunks(int64_t max_tokens);
int64_t stem_sort_count_entries(int64_t max_tokens);
// error text for calls that have no context (stem_last_error(NULL) returns it)
stem_status stem_fail(stem_ctx* c, stem_status st, const char* fmt, ...);

// ---- optimiser (adamw.hip) ----------------------------------------------------------
hipError_t stem_adamw(stem_ctx* ctx, int is_bf16, const int32_t* uniq_ids, const int32_t* n_uniq,
                      int64_t max_rows, const float* g, void* E, float* master, float* m, float* v, int F,
                      const stem_adamw_hparams& hp, hipStream_t s);

// ---- host-resident rows (prefetch.hip) ----------------------------------------------
// E_compact[dst_slot[k]] = E_host[src_row[k]] for k in [0, n)
hipError_t stem_copy_rows_kernel(stem_ctx* ctx, const void* E_host, const int32_t* src_row, const int32_t* dst_slot,
                                 int64_t n, int64_t row_bytes, void* E_compact, hipStream_t s);

// ---- knowledge editing (edit.hip) ----------------------------------------------------------
// rows E[src[j]] <- (pick[j] >= 0 ? old E[pick[j]] : mean of the old rows E[tgt[0..n_t)]); the old
// source rows go to backup (may be null).  rep: [n_s, F] scratch in the table's dtype.
hipError_t stem_edit_launch(stem_ctx* ctx, int is_bf16, void* E, const int32_t* src_dev, const int32_t* pick_dev,
                            const int32_t* tgt_dev, int n_s, int n_t, int F, void* rep, void* backup, hipStream_t s);
