// On-box peak calibration: what this GPU sustains on the two resources the layer's kernels are
// priced against, measured with the smallest kernels that use nothing else.
//   - MFMA: a loop of independent v_mfma_f32_32x32x16_bf16 on register operands (no LDS, no memory);
//   - HBM: a streaming read of a large buffer, and a streaming copy.
// The published peaks (2.5 PFLOP/s dense bf16, 8 TB/s) stay the denominators of the roofline
// fractions; these figures say how much of them any kernel can reach on the box at hand.
#include "stem_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

namespace {

constexpr int MFMA_CHAINS = 8;       // independent accumulators per wavefront
constexpr int MFMA_PER_ITER = 16;    // MFMAs per loop iteration (two per chain)

// Every wavefront issues iters * MFMA_PER_ITER MFMAs of 32*32*16*2 FLOP each.
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* __restrict__ sink) {
  f32x16_t acc[MFMA_CHAINS];
  bf16x8_t a, b;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    a[q] = (__bf16)(0.001f * (float)((threadIdx.x + q) & 15));
    b[q] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + q) & 7));
  }
#pragma unroll
  for (int c = 0; c < MFMA_CHAINS; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < MFMA_PER_ITER; ++u)
      acc[u % MFMA_CHAINS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[u % MFMA_CHAINS], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < MFMA_CHAINS; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[c][e];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive; practically never true
}

// The same rate with operands that carry data: every lane loads eight A and eight B fragments from
// `data` (caller-provided bf16 values, e.g. unit normals) and the loop forms the 4 x 4 outer product
// of fragments a GEMM wave tile forms, alternating between two fragment sets.  The MFMA count per
// wavefront equals mfma_loop_kernel's; what differs is how many operand and accumulator bits toggle
// per instruction, and with them the power drawn and the clock the chip sustains.
__global__ __launch_bounds__(256) void mfma_data_loop_kernel(int iters, const bf16x8_t* __restrict__ data,
                                                             float* __restrict__ sink) {
  f32x16_t acc[4][4];
  bf16x8_t a[2][4], b[2][4];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[s][i] = data[((s * 4 + i) * 2 + 0) * 256 + threadIdx.x];
      b[s][i] = data[((s * 4 + i) * 2 + 1) * 256 + threadIdx.x];
    }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  for (int it = 0; it < iters; it += 2) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s][i], b[s][j], acc[i][j], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) t += acc[i][j][e];
  if (t == 12345.678f) sink[0] = t;
}

// Streaming read: a workgroup takes contiguous 16 KB pieces (4 x 16 bytes per lane, whole lines), piece
// after piece with the grid as stride; one word per thread is (practically never) written at the end.
constexpr size_t PIECE16 = 256 * 4;   // 16-byte items per workgroup and step
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4_t* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
  u32x4_t s = {0, 0, 0, 0};
  for (size_t base = (size_t)blockIdx.x * PIECE16; base < n16; base += (size_t)gridDim.x * PIECE16) {
    u32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t i = base + u * 256 + threadIdx.x;
      v[u] = i < n16 ? __builtin_nontemporal_load(src + i) : s;
    }
    s ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  const uint32_t w = s[0] ^ s[1] ^ s[2] ^ s[3];
  if (w == 0x9e3779b9u) sink[0] = w;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst,
                                                          size_t n16) {
  for (size_t base = (size_t)blockIdx.x * PIECE16; base < n16; base += (size_t)gridDim.x * PIECE16) {
    u32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t i = base + u * 256 + threadIdx.x;
      if (i < n16) v[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t i = base + u * 256 + threadIdx.x;
      if (i < n16) __builtin_nontemporal_store(v[u], dst + i);
    }
  }
}

}  // namespace

extern "C" stem_status stem_measure_peak(int what, void* buf_a, void* buf_b, int64_t bytes, int repeats, void* stream,
                                         double* result) {
  if (!result || repeats < 1 || repeats > 1000)
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_measure_peak: result is NULL or repeats = %d is outside [1, 1000]", repeats);
  if (what < STEM_PEAK_MFMA_BF16 || what > STEM_PEAK_MFMA_BF16_DATA)
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_measure_peak: unknown measurement %d", what);
  if (!buf_a || ((what == STEM_PEAK_HBM_COPY || what == STEM_PEAK_MFMA_BF16_DATA) && !buf_b) || bytes < 65536 || (bytes & 15) ||
      (reinterpret_cast<uintptr_t>(buf_a) & 15u) || (reinterpret_cast<uintptr_t>(buf_b) & 15u))
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_measure_peak: buffers must be 16-byte aligned, bytes a multiple of 16 and >= 65536");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  const int mfma_iters = 4096, mfma_wgs = 256 * 8;   // 4 wavefronts per workgroup: 32 per compute unit over the launch
  const size_t n16 = (size_t)bytes / 16;
  auto launch = [&]() {
    if (what == STEM_PEAK_MFMA_BF16)
      hipLaunchKernelGGL(mfma_loop_kernel, dim3(mfma_wgs), dim3(256), 0, s, mfma_iters, static_cast<float*>(buf_a));
    else if (what == STEM_PEAK_MFMA_BF16_DATA)
      hipLaunchKernelGGL(mfma_data_loop_kernel, dim3(mfma_wgs), dim3(256), 0, s, mfma_iters,
                         static_cast<const bf16x8_t*>(buf_a), static_cast<float*>(buf_b));
    else if (what == STEM_PEAK_HBM_READ)
      hipLaunchKernelGGL(stream_read_kernel, dim3(256 * 16), dim3(256), 0, s, static_cast<const u32x4_t*>(buf_a), n16,
                         static_cast<uint32_t*>(buf_b ? buf_b : buf_a));
    else
      hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 16), dim3(256), 0, s, static_cast<const u32x4_t*>(buf_a),
                         static_cast<u32x4_t*>(buf_b), n16);
  };
  float best_ms = 0.f;
  if (e == hipSuccess) {
    launch();   // warm-up: code object, clocks
    for (int r = 0; r < repeats && e == hipSuccess; ++r) {
      (void)hipEventRecord(e0, s);
      launch();
      (void)hipEventRecord(e1, s);
      e = hipEventSynchronize(e1);
      float ms = 0.f;
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
      if (e == hipSuccess && (best_ms == 0.f || ms < best_ms)) best_ms = ms;
    }
    if (e == hipSuccess) e = hipGetLastError();
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (e != hipSuccess || best_ms <= 0.f)
    return stem_fail(nullptr, STEM_ERR_HIP, "stem_measure_peak: %s", hipGetErrorString(e));
  const double sec = (double)best_ms * 1e-3;
  if (what == STEM_PEAK_MFMA_BF16 || what == STEM_PEAK_MFMA_BF16_DATA)
    *result = (double)mfma_wgs * 4 * mfma_iters * MFMA_PER_ITER * (32.0 * 32 * 16 * 2) / sec / 1e12;   // TFLOP/s
  else
    *result = (double)bytes * (what == STEM_PEAK_HBM_COPY ? 2.0 : 1.0) / sec / 1e9;                      // GB/s
  return STEM_OK;
}
