// fp32 path of the STEM layer (small exactness-oriented runs) and the stand-alone
// element-wise kernels: H = SiLU(G) * E[ids] and the dU / dG products of backward.
#include "stem_internal.h"

namespace {

// C[m,n] (+)= sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk]; 64x64 tile, 16-wide K step,
// 256 threads each owning a 4x4 block.  Arbitrary strides cover all six products.
__global__ __launch_bounds__(256) void sgemm_kernel(const float* __restrict__ A, int64_t sam, int64_t sak,
                                                    const float* __restrict__ B, int64_t sbn, int64_t sbk,
                                                    float* __restrict__ C, int M, int N, int K, int accumulate) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int e = tid; e < 64 * 16; e += 256) {
      // index so that the contiguous direction of each operand is the fast one
      int r, k;
      if (sak == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
      float a = 0.f;
      if (m0 + r < M && k0 + k < K) a = A[(int64_t)(m0 + r) * sam + (int64_t)(k0 + k) * sak];
      As[k][r] = a;
      if (sbk == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
      float b = 0.f;
      if (n0 + r < N && k0 + k < K) b = B[(int64_t)(n0 + r) * sbn + (int64_t)(k0 + k) * sbk];
      Bs[k][r] = b;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float* c = C + (int64_t)m * N + n;
      *c = accumulate ? (*c + acc[i][j]) : acc[i][j];
    }
  }
}

__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + expf(-z)); }
__device__ __forceinline__ int checked_id(const int32_t* ids, int64_t t, int E_rows, int32_t* flag) {
  int id = ids[t];
  if ((unsigned)id >= (unsigned)E_rows) {
    *flag = 1;
    id = id < 0 ? 0 : E_rows - 1;
  }
  return id;
}

// fp32: one thread per 4 features of one token.
__global__ void silu_gather_f32_kernel(const float* __restrict__ G, const int32_t* __restrict__ ids,
                                       const float* __restrict__ E, int E_rows, float* __restrict__ H,
                                       int64_t T, int F, int32_t* flag) {
  const int F4 = F >> 2;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * F4) return;
  const int64_t t = i / F4;
  const int c = (int)(i - t * F4) * 4;
  const int id = checked_id(ids, t, E_rows, flag);
  const float4 g = *reinterpret_cast<const float4*>(G + t * F + c);
  const float4 e = *reinterpret_cast<const float4*>(E + (int64_t)id * F + c);
  float4 h;
  h.x = g.x * sigmoid_f(g.x) * e.x; h.y = g.y * sigmoid_f(g.y) * e.y;
  h.z = g.z * sigmoid_f(g.z) * e.z; h.w = g.w * sigmoid_f(g.w) * e.w;
  *reinterpret_cast<float4*>(H + t * F + c) = h;
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;

// bf16: one workgroup per token, 16 bytes (8 features) per thread per sweep; the
// gathered row and the activation row are both read as full contiguous rows.
__global__ __launch_bounds__(256) void silu_gather_bf16_kernel(const bf16_t* __restrict__ G,
                                                               const int32_t* __restrict__ ids,
                                                               const bf16_t* __restrict__ E, int E_rows,
                                                               bf16_t* __restrict__ H, int64_t T, int F,
                                                               int32_t* flag) {
  for (int64_t t = blockIdx.x; t < T; t += gridDim.x) {
    const int id = checked_id(ids, t, E_rows, flag);
    const bf16_t* g = G + t * F;
    const bf16_t* e = E + (int64_t)id * F;
    bf16_t* h = H + t * F;
    for (int c = threadIdx.x * 8; c < F; c += blockDim.x * 8) {
      const uint4 gv = *reinterpret_cast<const uint4*>(g + c);
      const uint4 ev = *reinterpret_cast<const uint4*>(e + c);
      const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w};
      const uint32_t ew[4] = {ev.x, ev.y, ev.z, ev.w};
      bf16x8_t out;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float g0 = __uint_as_float(gw[q] << 16), g1 = __uint_as_float(gw[q] & 0xffff0000u);
        const float e0 = __uint_as_float(ew[q] << 16), e1 = __uint_as_float(ew[q] & 0xffff0000u);
        out[2 * q] = (__bf16)(g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * e0);
        out[2 * q + 1] = (__bf16)(g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * e1);
      }
      *reinterpret_cast<bf16x8_t*>(h + c) = out;
    }
  }
}

__global__ void dh_epilogue_f32_kernel(const float* __restrict__ dH, const float* __restrict__ G,
                                       const int32_t* __restrict__ ids, const float* __restrict__ E,
                                       int E_rows, float* __restrict__ dU, float* __restrict__ dG, int64_t T,
                                       int F, int32_t* flag) {
  const int F4 = F >> 2;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * F4) return;
  const int64_t t = i / F4;
  const int c = (int)(i - t * F4) * 4;
  const int id = checked_id(ids, t, E_rows, flag);
  const float4 dh4 = *reinterpret_cast<const float4*>(dH + t * F + c);
  const float4 g4 = *reinterpret_cast<const float4*>(G + t * F + c);
  const float4 e4 = *reinterpret_cast<const float4*>(E + (int64_t)id * F + c);
  const float dh[4] = {dh4.x, dh4.y, dh4.z, dh4.w}, g[4] = {g4.x, g4.y, g4.z, g4.w};
  const float e[4] = {e4.x, e4.y, e4.z, e4.w};
  float du[4], dg[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float s = sigmoid_f(g[q]);
    du[q] = dh[q] * (g[q] * s);
    dg[q] = dh[q] * e[q] * (s * (1.0f + g[q] * (1.0f - s)));
  }
  *reinterpret_cast<float4*>(dU + t * F + c) = make_float4(du[0], du[1], du[2], du[3]);
  *reinterpret_cast<float4*>(dG + t * F + c) = make_float4(dg[0], dg[1], dg[2], dg[3]);
}

}  // namespace

// Zero fill by a kernel rather than hipMemsetAsync, so that every call of the library can be recorded
// into a HIP graph (memset nodes have replayed wrongly on this platform).
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, size_t words) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) p[i] = 0u;
}
hipError_t stem_fill_zero(void* p, size_t bytes, hipStream_t s) {   // bytes is a multiple of 4
  if (bytes == 0) return hipSuccess;
  const size_t words = bytes / 4;
  const unsigned grid = (unsigned)std::min<size_t>((words + 255) / 256, 2048);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, s, static_cast<uint32_t*>(p), words);
  return hipGetLastError();
}

hipError_t stem_sgemm(stem_ctx* ctx, int kid, const float* A, int64_t sam, int64_t sak, const float* B,
                      int64_t sbn, int64_t sbk, float* C, int M, int N, int K, int accumulate, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  ProfScope ps(ctx, kid, s);
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  hipLaunchKernelGGL(sgemm_kernel, grid, dim3(256), 0, s, A, sam, sak, B, sbn, sbk, C, M, N, K, accumulate);
  return hipGetLastError();
}

hipError_t stem_silu_gather(stem_ctx* ctx, int is_bf16, const void* G, const int32_t* ids, const void* E,
                            int E_rows, void* H, int64_t T, int F, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  ProfScope ps(ctx, K_SILU_GATHER, s);
  if (is_bf16) {
    const int grid = (int)(T < 65536 ? T : 65536);
    hipLaunchKernelGGL(silu_gather_bf16_kernel, dim3(grid), dim3(256), 0, s, (const bf16_t*)G, ids,
                       (const bf16_t*)E, E_rows, (bf16_t*)H, T, F, ctx->flag);
  } else {
    const int64_t n = T * (F / 4);
    hipLaunchKernelGGL(silu_gather_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       (const float*)G, ids, (const float*)E, E_rows, (float*)H, T, F, ctx->flag);
  }
  return hipGetLastError();
}

hipError_t stem_dh_epilogue_f32(stem_ctx* ctx, const float* dH, const float* G, const int32_t* ids,
                                const float* E, int E_rows, float* dU, float* dG, int64_t T, int F,
                                hipStream_t s) {
  if (T <= 0) return hipSuccess;
  ProfScope ps(ctx, K_DH_EPILOGUE, s);
  const int64_t n = T * (F / 4);
  hipLaunchKernelGGL(dh_epilogue_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dH, G, ids,
                     E, E_rows, dU, dG, T, F, ctx->flag);
  return hipGetLastError();
}
