// Host-resident table: device-side copy of the distinct rows a batch needs, read
// straight from pinned host memory (each lane pulls 16 bytes over the host link).
#include "stem_internal.h"

namespace {

// The host link, not the GPU, bounds this kernel (about 57 GB/s measured).  With one 16 KB row
// in flight per workgroup, 4 / 8 / 16 / 32 workgroups reach 12 / 22 / 40 / 56 GB/s and more add
// nothing, so 32 it is: the rest of the chip stays free for the gate product running beside it
// (with 128 workgroups that product was measured 30 % slower).
constexpr int COPY_WGS = 32;

__global__ __launch_bounds__(256) void copy_rows_kernel(const uint4* __restrict__ src,
                                                        const int32_t* __restrict__ src_row,
                                                        const int32_t* __restrict__ dst_slot, int64_t n,
                                                        int64_t row_vecs, uint4* __restrict__ dst) {
  for (int64_t j = blockIdx.x; j < n; j += gridDim.x) {
    const uint4* s = src + (int64_t)src_row[j] * row_vecs;
    uint4* d = dst + (int64_t)dst_slot[j] * row_vecs;
    for (int64_t o = threadIdx.x; o < row_vecs; o += 256) d[o] = s[o];
  }
}

}  // namespace

hipError_t stem_copy_rows_kernel(stem_ctx* ctx, const void* E_host, const int32_t* src_row, const int32_t* dst_slot,
                                 int64_t n, int64_t row_bytes, void* E_compact, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  ProfScope ps(ctx, K_ROW_COPY, s);
  const int grid = (int)(n < COPY_WGS ? n : COPY_WGS);
  hipLaunchKernelGGL(copy_rows_kernel, dim3(grid), dim3(256), 0, s, (const uint4*)E_host, src_row, dst_slot, n,
                     row_bytes / 16, (uint4*)E_compact);
  return hipGetLastError();
}
