// Host-resident table: device-side copy of the distinct rows a batch needs, read
// straight from pinned host memory (each lane pulls 16 bytes over the host link).
#include "stem_internal.h"

namespace {

__global__ __launch_bounds__(256) void copy_rows_kernel(const uint4* __restrict__ src,
                                                        const int32_t* __restrict__ uniq, int64_t n,
                                                        int64_t row_vecs, uint4* __restrict__ dst) {
  for (int64_t j = blockIdx.x; j < n; j += gridDim.x) {
    const uint4* s = src + (int64_t)uniq[j] * row_vecs;
    uint4* d = dst + j * row_vecs;
    for (int64_t o = threadIdx.x; o < row_vecs; o += 256) d[o] = s[o];
  }
}

}  // namespace

hipError_t stem_copy_rows_kernel(stem_ctx* ctx, const void* E_host, const int32_t* uniq_dev, int64_t n,
                                 int64_t row_bytes, void* E_compact, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  ProfScope ps(ctx, K_ROW_COPY, s);
  const int grid = (int)(n < 128 ? n : 128);
  hipLaunchKernelGGL(copy_rows_kernel, dim3(grid), dim3(256), 0, s, (const uint4*)E_host, uniq_dev, n,
                     row_bytes / 16, (uint4*)E_compact);
  return hipGetLastError();
}
