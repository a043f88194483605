// AdamW with decoupled weight decay on the table rows a batch touched, one pass over
// gradient row, master row and both moments; optionally refreshes the bf16 working copy.
#include "stem_internal.h"

namespace {

struct AdamConsts {
  float lr, b1, b2, eps, wd, inv_c1, inv_c2;  // inv_c = 1 / (1 - beta^step)
};

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// Workgroups stride over the touched rows; threads stride over the row in float4 steps.
template <bool BF16>
__global__ __launch_bounds__(256) void adamw_kernel(const int32_t* __restrict__ uniq_ids,
                                                    const int32_t* __restrict__ n_uniq, int max_rows, int V,
                                                    const float* __restrict__ g, void* __restrict__ E,
                                                    float* __restrict__ master, float* __restrict__ m,
                                                    float* __restrict__ v, int F, AdamConsts k, int32_t* flag) {
  int n = *n_uniq;
  if (n > max_rows) n = max_rows;
  for (int j = blockIdx.x; j < n; j += gridDim.x) {
    int r = uniq_ids[j];
    if ((unsigned)r >= (unsigned)V) {  // never write outside the table
      if (threadIdx.x == 0) *flag = 1;
      continue;
    }
    const size_t ro = (size_t)r * F;
    const float* gr = g + (size_t)j * F;
    float* pr = master ? master + ro : reinterpret_cast<float*>(E) + ro;
#pragma unroll 2
    for (int c = threadIdx.x * 4; c < F; c += 256 * 4) {
      const f32x4_t g4 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(gr + c));
      const f32x4_t p4 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(pr + c));
      const f32x4_t m4 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(m + ro + c));
      const f32x4_t v4 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(v + ro + c));
      const float gg[4] = {g4[0], g4[1], g4[2], g4[3]};
      float pp[4] = {p4[0], p4[1], p4[2], p4[3]};
      float mm[4] = {m4[0], m4[1], m4[2], m4[3]};
      float vv[4] = {v4[0], v4[1], v4[2], v4[3]};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        mm[q] = k.b1 * mm[q] + (1.0f - k.b1) * gg[q];
        vv[q] = k.b2 * vv[q] + (1.0f - k.b2) * gg[q] * gg[q];
        const float mhat = mm[q] * k.inv_c1;
        const float vhat = vv[q] * k.inv_c2;
        pp[q] = pp[q] - k.lr * k.wd * pp[q] - k.lr * mhat / (sqrtf(vhat) + k.eps);
      }
      const f32x4_t po = {pp[0], pp[1], pp[2], pp[3]}, mo = {mm[0], mm[1], mm[2], mm[3]}, vo = {vv[0], vv[1], vv[2], vv[3]};
      __builtin_nontemporal_store(po, reinterpret_cast<f32x4_t*>(pr + c));
      __builtin_nontemporal_store(mo, reinterpret_cast<f32x4_t*>(m + ro + c));
      __builtin_nontemporal_store(vo, reinterpret_cast<f32x4_t*>(v + ro + c));
      if (BF16) {
        bf16x4_t o;
        o[0] = (__bf16)pp[0]; o[1] = (__bf16)pp[1]; o[2] = (__bf16)pp[2]; o[3] = (__bf16)pp[3];
        *reinterpret_cast<bf16x4_t*>(reinterpret_cast<bf16_t*>(E) + ro + c) = o;
      } else if (master) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(E) + ro + c) = make_float4(pp[0], pp[1], pp[2], pp[3]);
      }
    }
  }
}

}  // namespace

hipError_t stem_adamw(stem_ctx* ctx, int is_bf16, const int32_t* uniq_ids, const int32_t* n_uniq,
                      int64_t max_rows, const float* g, void* E, float* master, float* m, float* v, int F,
                      const stem_adamw_hparams& hp, hipStream_t s) {
  if (max_rows <= 0) return hipSuccess;
  AdamConsts k;
  k.lr = hp.lr; k.b1 = hp.beta1; k.b2 = hp.beta2; k.eps = hp.eps; k.wd = hp.weight_decay;
  k.inv_c1 = (float)(1.0 / (1.0 - pow((double)hp.beta1, (double)hp.step)));
  k.inv_c2 = (float)(1.0 / (1.0 - pow((double)hp.beta2, (double)hp.step)));
  const int grid = (int)(max_rows < 4096 ? max_rows : 4096);
  ProfScope ps(ctx, K_ADAMW, s);
  if (is_bf16)
    hipLaunchKernelGGL(adamw_kernel<true>, dim3(grid), dim3(256), 0, s, uniq_ids, n_uniq, (int)max_rows,
                       ctx->desc.vocab, g, E, master, m, v, F, k, ctx->flag);
  else
    hipLaunchKernelGGL(adamw_kernel<false>, dim3(grid), dim3(256), 0, s, uniq_ids, n_uniq, (int)max_rows,
                       ctx->desc.vocab, g, E, master, m, v, F, k, ctx->flag);
  return hipGetLastError();
}
