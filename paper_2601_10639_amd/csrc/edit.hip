// Knowledge editing on the table: the rows of a source entity's tokens are replaced by rows
// derived from a target entity's tokens (one to one, left-padded, copied, or their mean).
// Two small kernels: gather the replacement rows (as the table was before the edit) and save
// the source rows; then write the replacements.  Sources and targets may overlap.
#include "stem_internal.h"

namespace {

// rep[j] = (pick[j] >= 0) ? E[pick[j]] : mean over the n_t target rows;  backup[j] = E[src[j]]
template <bool BF16>
__global__ __launch_bounds__(256) void edit_gather_kernel(const void* __restrict__ E, const int32_t* __restrict__ src,
                                                          const int32_t* __restrict__ pick,
                                                          const int32_t* __restrict__ tgt, int n_t, int F,
                                                          void* __restrict__ rep, void* __restrict__ backup) {
  const int j = blockIdx.x;
  const int64_t so = (int64_t)src[j] * F, ro = (int64_t)j * F;
  const int pk = pick[j];
  for (int c = threadIdx.x; c < F; c += 256) {
    if (BF16) {
      const bf16_t* e = static_cast<const bf16_t*>(E);
      if (backup) static_cast<bf16_t*>(backup)[ro + c] = e[so + c];
      if (pk >= 0) {
        static_cast<bf16_t*>(rep)[ro + c] = e[(int64_t)pk * F + c];
      } else {
        float s = 0.f;
        for (int k = 0; k < n_t; ++k) s += __uint_as_float((uint32_t)e[(int64_t)tgt[k] * F + c] << 16);
        const __bf16 r = (__bf16)(s / (float)n_t);
        static_cast<bf16_t*>(rep)[ro + c] = __builtin_bit_cast(bf16_t, r);
      }
    } else {
      const float* e = static_cast<const float*>(E);
      if (backup) static_cast<float*>(backup)[ro + c] = e[so + c];
      if (pk >= 0) {
        static_cast<float*>(rep)[ro + c] = e[(int64_t)pk * F + c];
      } else {
        float s = 0.f;
        for (int k = 0; k < n_t; ++k) s += e[(int64_t)tgt[k] * F + c];
        static_cast<float*>(rep)[ro + c] = s / (float)n_t;
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void edit_scatter_kernel(T* __restrict__ E, const int32_t* __restrict__ src, int F,
                                                           const T* __restrict__ rep) {
  const int j = blockIdx.x;
  for (int c = threadIdx.x; c < F; c += 256) E[(int64_t)src[j] * F + c] = rep[(int64_t)j * F + c];
}

}  // namespace

hipError_t stem_edit_launch(stem_ctx* ctx, int is_bf16, void* E, const int32_t* src_dev, const int32_t* pick_dev,
                            const int32_t* tgt_dev, int n_s, int n_t, int F, void* rep, void* backup, hipStream_t s) {
  if (n_s <= 0) return hipSuccess;
  (void)ctx;
  if (is_bf16) {
    hipLaunchKernelGGL(edit_gather_kernel<true>, dim3(n_s), dim3(256), 0, s, E, src_dev, pick_dev, tgt_dev, n_t, F, rep,
                       backup);
    hipLaunchKernelGGL(edit_scatter_kernel<bf16_t>, dim3(n_s), dim3(256), 0, s, static_cast<bf16_t*>(E), src_dev, F,
                       static_cast<const bf16_t*>(rep));
  } else {
    hipLaunchKernelGGL(edit_gather_kernel<false>, dim3(n_s), dim3(256), 0, s, E, src_dev, pick_dev, tgt_dev, n_t, F,
                       rep, backup);
    hipLaunchKernelGGL(edit_scatter_kernel<float>, dim3(n_s), dim3(256), 0, s, static_cast<float*>(E), src_dev, F,
                       static_cast<const float*>(rep));
  }
  return hipGetLastError();
}
