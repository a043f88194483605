// bf16 MFMA GEMM for few rows (a decode step: a few hundred tokens against the layer's
// full weight matrices), gfx950.
//
// With M of a few hundred the 256x256-tile kernel leaves most compute units idle, and the
// product is bound by streaming the weights once from HBM and the activations many times
// from L2.  This kernel computes  C[m,n] = sum_k A[m,k] * B[n,k]  (both operands K-contiguous)
// on 128x64 output tiles, optionally split along K, so that a 256-row product against an
// 8192- or 2048-row weight matrix yields 256 workgroups.  A launch lasts about ten
// microseconds, so everything that is executed once per workgroup is kept short: instruction
// fetch of straight-line code is a visible part of such a kernel.
//
// Workgroup = 8 wavefronts = 2 (m) x 4 (the four 16-wide k-steps of each 64-wide K tile); a
// wavefront holds a 64x64 piece as 2x2 accumulators of v_mfma_f32_32x32x16_bf16 and does one
// k-step of every tile: 4 fragment reads for 4 independent MFMAs.  Operand tiles travel
// global -> registers -> LDS: each wavefront keeps the loads of four K tiles in flight in
// registers (whole 128-byte lines, 16 bytes per lane) and writes the oldest to one of two LDS
// stages (XOR-swizzled rows of 128 bytes, conflict-free for the fragment reads).  The
// direct-to-LDS load path was measured at about 32 bytes per clock and compute unit in this
// kernel, half of what register loads reach.  One barrier per K tile; the fragments of the
// next tile are read while the MFMAs of the current one run.
//
// At the end every wavefront writes its accumulators to LDS and all 512 threads run one
// short loop over the 128x64 tile: add the four k quarters in a fixed order, then the
// epilogue on 4 consecutive n per thread (16 threads cover one output row, so stores and the
// gathered table row are whole 128-byte lines): plain bf16 store, the fused
// SiLU * gathered-row of the gate product, or an fp32 partial tile for a split-K launch,
// which a second kernel sums in split order.
#include "stem_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __amdgpu_buffer_rsrc_t rsrc_t;

namespace {

constexpr int SBM = 128, SBN = 64, SBK = 64;
constexpr int DEPTH = 4;                      // K tiles in flight in registers (even)
constexpr int A_BYTES = SBM * SBK * 2;        // 16 KB
constexpr int B_BYTES = SBN * SBK * 2;        // 8 KB
constexpr int STAGE = A_BYTES + B_BYTES;      // 24 KB, two stages
constexpr int RED_PITCH = SBN * 4 + 16;       // fp32 row of the reduction buffer, padded
constexpr int RED_BYTES = 4 * SBM * RED_PITCH;  // four k quarters: 139264 bytes
constexpr uint32_t OOB = 0x80000000u;         // a buffer offset beyond any operand: reads as zero

__device__ __forceinline__ float sigmoidf_fast(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

__device__ __forceinline__ uint2 pack4(const float (&f)[4]) {
  bf16x4_t v;
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = (__bf16)f[q];
  return __builtin_bit_cast(uint2, v);
}

template <int EPI>
__global__ __launch_bounds__(512) void gemm_skinny_kernel(GemmArgs p) {
  __shared__ __attribute__((aligned(16))) char smem[RED_BYTES];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, kq = wave >> 1;

  // Workgroup -> (m tile, n tile, k slice).  Consecutive workgroup ids go round-robin over the
  // 8 XCDs; each XCD gets one contiguous run of the linear order, in which the m tiles of one
  // n tile are neighbours, so the weight rows they share are fetched from HBM once.
  // (mt <= 4 and the quotients are small: the float reciprocal is exact here.)
  int tm, tn, z;
  {
    const int nb = gridDim.x, b = blockIdx.x;
    const int q = nb >> 3, r = nb & 7;
    const int xcd = b & 7, idx = b >> 3;
    const int L = xcd * q + (xcd < r ? xcd : r) + idx;
    const int per_z = p.mt * p.nt;
    z = (int)(((float)L + 0.5f) * p.inv_per_z);
    const int in = L - z * per_z;
    tn = (int)(((float)in + 0.5f) * p.inv_mt);
    tm = in - tn * p.mt;
  }
  const int m0 = tm * SBM, n0 = tn * SBN;
  const int nk_all = p.K / SBK;
  const int per = (nk_all + p.ksplit - 1) / p.ksplit;
  const int kt0 = z * per;
  const int nk = (nk_all - kt0) < per ? (nk_all - kt0) : per;   // may be <= 0: an all-zero partial

  // ---- gate epilogue inputs, requested up front -------------------------------------------------
  // The epilogue multiplies by one gathered table row per output row.  Token ids are requested
  // first of all and the table rows right after the first operand tiles, so both latencies pass
  // under the main loop instead of standing, one after the other, at the end of a 20 us kernel.
  // thread -> rows it * 32 + (tid >> 4), it = 0..3, columns (tid & 15) * 4 .. +3 of the tile
  const int c4 = tid & 15;
  const int n = n0 + c4 * 4;
  int ids4[4] = {0, 0, 0, 0};
  uint2 ev[4];
  if (EPI == EPI_GATE) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int m = m0 + it * 32 + (tid >> 4);
      ids4[it] = p.ids[m < p.M ? m : p.M - 1];
    }
  }

  // ---- operand loads: wavefront w brings A row blocks 2w, 2w+1 and B row block w of a tile ------
  // lane -> row (lane >> 3) of the 8-row block, 16-byte chunk (lane & 7) of the 128-byte row
  const rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(p.A), 0, p.M * p.lda * 2, 0x00020000);
  const rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(p.B), 0, p.N * p.ldb * 2, 0x00020000);
  uint32_t goff[3], loff[3];
  {
    const int sub = lane >> 3, c = lane & 7;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int row = i < 2 ? (wave * 2 + i) * 8 + sub : wave * 8 + sub;
      const int grow = (i < 2 ? m0 : n0) + row;
      const int lim = i < 2 ? p.M : p.N, ld = i < 2 ? p.lda : p.ldb;
      goff[i] = grow < lim ? (uint32_t)((grow * ld + c * 8) * 2) : OOB;
      loff[i] = (uint32_t)((i < 2 ? 0 : A_BYTES) + row * 128 + ((c ^ ((row >> 1) & 7)) << 4));
    }
  }
  u32x4_t ring[DEPTH][3];
  // The K tiles of the slice are walked from a start that differs from one n tile to the next and
  // wraps around: at any moment the workgroups then read different stretches of their weight rows
  // (rows 4 or 16 KB apart, whose lines at one k sit in the same few memory channels).
  // (16-layer decode step 0.684-0.692 ms against 0.695-0.703 with every workgroup starting at the slice's first tile)
  int kpos = nk > 1 ? (int)(((long)tn * nk) / p.nt) % nk : 0;
  auto request = [&](u32x4_t(&r)[3]) {
    const int so = (kt0 + kpos) * (SBK * 2);
    r[0] = __builtin_amdgcn_raw_buffer_load_b128(ra, goff[0], so, 0);
    r[1] = __builtin_amdgcn_raw_buffer_load_b128(ra, goff[1], so, 0);
    r[2] = __builtin_amdgcn_raw_buffer_load_b128(rb, goff[2], so, 0);
    if (++kpos >= nk) kpos = 0;
  };
  auto commit = [&](const u32x4_t(&r)[3], int stage) {
    char* st = smem + stage * STAGE;
#pragma unroll
    for (int i = 0; i < 3; ++i) *reinterpret_cast<u32x4_t*>(st + loff[i]) = r[i];
  };

  // ---- fragment addresses (bytes within a stage): k-step kq of every tile --------------------
  const int frow = lane & 31, fk = lane >> 5;
  const uint32_t sw = (uint32_t)((((kq * 2 + fk) ^ (frow >> 1)) & 7) << 4);
  const uint32_t fa = (uint32_t)((wm * 64 + frow) * 128) + sw;
  const uint32_t fb = (uint32_t)(A_BYTES + frow * 128) + sw;
  auto read_frags = [&](int stage, bf16x8_t(&a)[2], bf16x8_t(&b)[2]) {
    const char* st = smem + stage * STAGE;
    a[0] = *reinterpret_cast<const bf16x8_t*>(st + fa);
    b[0] = *reinterpret_cast<const bf16x8_t*>(st + fb);
    a[1] = *reinterpret_cast<const bf16x8_t*>(st + fa + 32 * 128);
    b[1] = *reinterpret_cast<const bf16x8_t*>(st + fb + 32 * 128);
  };

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // ---- main loop -----------------------------------------------------------------------------
  // iteration t: tile t+1 goes from registers to its LDS stage, tile t+DEPTH is requested into
  // the registers just freed, barrier, the fragments of tile t+1 are read while the MFMAs of
  // tile t run.  Requests past the last tile wrap around to tiles already used; what they bring is never used.
#pragma unroll
  for (int s = 0; s < DEPTH; ++s) request(ring[s]);
  if (EPI == EPI_GATE) {
    const int n_ld = n < p.N ? n : 0;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      int id = ids4[it];
      if ((unsigned)id >= (unsigned)p.E_rows) {   // reported to the host, clamped so no access leaves the table
        *p.flag = 1;
        id = id < 0 ? 0 : p.E_rows - 1;
      }
      ev[it] = *reinterpret_cast<const uint2*>(p.E + (size_t)id * p.N + n_ld);
    }
  }
  commit(ring[0], 0);
  request(ring[0]);
  __syncthreads();
  bf16x8_t fra[2][2], frb[2][2];   // fragment double buffer, indexed by tile parity
  read_frags(0, fra[0], frb[0]);
  // slot: position in the ring that holds tile t+1; par: parity of t (stage of tile t)
  auto iteration = [&](u32x4_t(&r)[3], const int par) __attribute__((always_inline)) {
    commit(r, par ^ 1);
    request(r);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();   // tile t+1 visible to all; everybody has read the fragments of tile t
    __builtin_amdgcn_sched_barrier(0);
    read_frags(par ^ 1, fra[par ^ 1], frb[par ^ 1]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frb[par][j], fra[par][i], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  };
  int t = 0;
  for (; t + DEPTH <= nk; t += DEPTH) {
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) iteration(ring[(u + 1) % DEPTH], u & 1);
  }
#pragma unroll
  for (int u = 0; u < DEPTH - 1; ++u)
    if (t + u < nk) iteration(ring[(u + 1) % DEPTH], u & 1);
  __syncthreads();   // nobody reads a stage any more

  // ---- accumulators -> LDS: quarter kq, row, 64 fp32 columns ------------------------------------
  // lane holds row frow of each accumulator, columns j*32 + g*8 + fk*4 .. +3
  {
    char* red = smem + kq * (SBM * RED_PITCH) + (wm * 64 + frow) * RED_PITCH + fk * 16;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4_t w = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          *reinterpret_cast<f32x4_t*>(red + i * 32 * RED_PITCH + (j * 32 + g * 8) * 4) = w;
        }
  }
  __syncthreads();

  // ---- sum of the quarters and epilogue: thread -> row (idx >> 4), columns (idx & 15) * 4 .. +3 ----
  if (n >= p.N) return;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = it * 32 + (tid >> 4);
    const int m = m0 + row;
    const char* src = smem + row * RED_PITCH + c4 * 16;
    f32x4_t s = *reinterpret_cast<const f32x4_t*>(src);
#pragma unroll
    for (int qq = 1; qq < 4; ++qq) s += *reinterpret_cast<const f32x4_t*>(src + qq * (SBM * RED_PITCH));
    if (m >= p.M) continue;
    const float c[4] = {s[0], s[1], s[2], s[3]};
    const size_t o = (size_t)m * p.N + n;
    if (EPI == EPI_BF16) {
      float cr[4] = {c[0], c[1], c[2], c[3]};
      if (p.residual) {   // the layer's output joins the residual stream: added in fp32, rounded once
        const uint2 rv = *reinterpret_cast<const uint2*>(p.residual + o);
        cr[0] += __uint_as_float(rv.x << 16); cr[1] += __uint_as_float(rv.x & 0xffff0000u);
        cr[2] += __uint_as_float(rv.y << 16); cr[3] += __uint_as_float(rv.y & 0xffff0000u);
      }
      *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(p.C) + o) = pack4(cr);
    } else if (EPI == EPI_SPLITK) {
      *reinterpret_cast<f32x4_t*>(p.ws + ((size_t)z * p.M + m) * p.N + n) = s;
    } else {  // EPI_GATE
      const float e[4] = {__uint_as_float(ev[it].x << 16), __uint_as_float(ev[it].x & 0xffff0000u),
                          __uint_as_float(ev[it].y << 16), __uint_as_float(ev[it].y & 0xffff0000u)};
      float h[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) h[q] = c[q] * sigmoidf_fast(c[q]) * e[q];
      if (p.outG) *reinterpret_cast<uint2*>(p.outG + o) = pack4(c);
      *reinterpret_cast<uint2*>(p.outH + o) = pack4(h);
    }
  }
}

// out[i] = bf16(sum over the k slices, in slice order, of ws[z][i] (+ residual[i])); 4 elements per thread
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ ws, int ksplit, int64_t total,
                                                            const bf16_t* residual, bf16_t* out) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= total) return;
  f32x4_t s = *reinterpret_cast<const f32x4_t*>(ws + i);
  for (int z = 1; z < ksplit; ++z) {
    const f32x4_t w = *reinterpret_cast<const f32x4_t*>(ws + (size_t)z * total + i);
    s += w;
  }
  float c[4] = {s[0], s[1], s[2], s[3]};
  if (residual) {   // may be the same buffer as out: every thread reads its four elements before it writes them
    const uint2 rv = *reinterpret_cast<const uint2*>(residual + i);
    c[0] += __uint_as_float(rv.x << 16); c[1] += __uint_as_float(rv.x & 0xffff0000u);
    c[2] += __uint_as_float(rv.y << 16); c[3] += __uint_as_float(rv.y & 0xffff0000u);
  }
  *reinterpret_cast<uint2*>(out + i) = pack4(c);
}

}  // namespace

int stem_gemm_skinny_ksplit(int M, int N, int K) {
  const int tiles = ((M + SBM - 1) / SBM) * ((N + SBN - 1) / SBN);
  const int nk = (K + SBK - 1) / SBK;
  int ks = 1;
  while (ks < 8 && tiles * ks * 2 <= 256 && nk / (ks * 2) >= 8) ks *= 2;
  return ks;
}

hipError_t stem_gemm_skinny_bf16(stem_ctx* ctx, int kid, int epi, const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipSuccess;
  const int64_t lim = 0x7fffffff;
  if ((int64_t)a.M * a.lda * 2 > lim || (int64_t)a.N * a.ldb * 2 > lim) return hipErrorInvalidValue;
  if (a.K % SBK != 0 || a.N % 4 != 0) return hipErrorInvalidValue;
  GemmArgs p = a;
  p.mt = (a.M + SBM - 1) / SBM;
  p.nt = (a.N + SBN - 1) / SBN;
  p.inv_mt = 1.0f / (float)p.mt;
  p.inv_per_z = 1.0f / (float)(p.mt * p.nt);
  const int tiles = p.mt * p.nt;
  if (epi == EPI_SPLITK) {
    // C (bf16) = sum of ksplit fp32 partial products kept in the context's workspace
    if (p.ksplit < 1 || !p.ws || !p.C) return hipErrorInvalidValue;
    {
      ProfScope ps(ctx, kid, s);
      hipLaunchKernelGGL((gemm_skinny_kernel<EPI_SPLITK>), dim3(tiles * p.ksplit), dim3(512), 0, s, p);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t total = (int64_t)a.M * a.N;
    ProfScope ps(ctx, K_SPLITK_REDUCE, s);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, s, p.ws,
                       p.ksplit, total, p.residual, static_cast<bf16_t*>(p.C));
    return hipGetLastError();
  }
  p.ksplit = 1;
  ProfScope ps(ctx, kid, s);
  if (epi == EPI_BF16) hipLaunchKernelGGL((gemm_skinny_kernel<EPI_BF16>), dim3(tiles), dim3(512), 0, s, p);
  else if (epi == EPI_GATE) hipLaunchKernelGGL((gemm_skinny_kernel<EPI_GATE>), dim3(tiles), dim3(512), 0, s, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
