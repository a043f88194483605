// bf16 MFMA GEMMs of the STEM layer (gate, down, and the four backward products)
// for gfx950, with the layer's element-wise work fused into the epilogues.
//
// One kernel template computes  C[m,n] = sum_k Aop[m,k] * Bop[n,k]  on a 256x256
// output tile per workgroup (4 wavefronts, each a 128x128 quadrant held as 4x4
// accumulators of v_mfma_f32_32x32x16_bf16), stepping K by 64 through two LDS stages.
// Either operand may be stored K-contiguous ([rows,K]) or rows-contiguous ([K,rows]);
// the second kind is transposed 8x8 in registers on its way into LDS, so the MFMA
// loop always reads 16-byte K-contiguous fragments from one LDS layout.
//
// LDS tile layout: row r (an m or n index within the tile) owns 128 bytes = 8 chunks
// of 8 bf16; chunk c of row r sits at chunk slot c ^ ((r >> 1) & 7).  With that XOR a
// ds_read_b128 of one chunk column over 16 consecutive rows touches all 64 banks once.
//
// The MFMA is issued with the N-side fragment as its row operand and the M-side
// fragment as its column operand, so a lane ends up holding, for one m (token), groups
// of 4 consecutive n (features): row-major outputs, the gathered table row and the
// saved activations are then accessed 8 or 16 bytes at a time per lane.
#include "stem_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = 256 * BK * 2;  // one operand tile in LDS
constexpr int STAGE_BYTES = 2 * TILE_BYTES;

__device__ __forceinline__ uint32_t lds_off(int row, int chunk) {
  return (uint32_t)(row * 128 + (((chunk ^ (row >> 1)) & 7) << 4));
}

// ---- global -> registers ----------------------------------------------------------
// K-contiguous operand: thread t takes 16-byte chunk (t & 7) of rows (t >> 3) + 32 i.
__device__ __forceinline__ void load_kc(const bf16_t* __restrict__ base, int ld, int row0, int rows,
                                        int k0, int K, int tid, uint4 (&st)[8]) {
  const int kc = tid & 7;
  const int r = tid >> 3;
  const bool kok = (k0 + kc * 8) < K;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = row0 + r + 32 * i;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (kok && row < rows) v = *reinterpret_cast<const uint4*>(base + (size_t)row * ld + k0 + kc * 8);
    st[i] = v;
  }
}
__device__ __forceinline__ void store_kc(char* tile, int tid, const uint4 (&st)[8]) {
  const int kc = tid & 7;
  const int r = tid >> 3;
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<uint4*>(tile + lds_off(r + 32 * i, kc)) = st[i];
}

// rows-contiguous operand: thread t owns the 8(k) x 8(rows) block kb = t & 7, rb = t >> 3.
__device__ __forceinline__ void load_mc(const bf16_t* __restrict__ base, int ld, int row0, int rows,
                                        int k0, int K, int tid, uint4 (&st)[8]) {
  const int kb = tid & 7;
  const int rb = tid >> 3;
  const bool rok = (row0 + rb * 8) < rows;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    const int k = k0 + kb * 8 + kk;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (rok && k < K) v = *reinterpret_cast<const uint4*>(base + (size_t)k * ld + row0 + rb * 8);
    st[kk] = v;
  }
}
__device__ __forceinline__ uint32_t pick(const uint4& v, int q) {
  return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w;
}
__device__ __forceinline__ void store_mc(char* tile, int tid, const uint4 (&st)[8]) {
  const int kb = tid & 7;
  const int rb = tid >> 3;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int q = r >> 1;
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t lo = pick(st[2 * j], q), hi = pick(st[2 * j + 1], q);
      w[j] = (r & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
    }
    *reinterpret_cast<uint4*>(tile + lds_off(rb * 8 + r, kb)) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

template <int L>
__device__ __forceinline__ void load_op(const bf16_t* base, int ld, int row0, int rows, int k0, int K,
                                        int tid, uint4 (&st)[8]) {
  if (L == OP_KC) load_kc(base, ld, row0, rows, k0, K, tid, st);
  else load_mc(base, ld, row0, rows, k0, K, tid, st);
}
template <int L>
__device__ __forceinline__ void store_op(char* tile, int tid, const uint4 (&st)[8]) {
  if (L == OP_KC) store_kc(tile, tid, st);
  else store_mc(tile, tid, st);
}

// ---- epilogue math ------------------------------------------------------------------
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float sigmoidf_fast(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __expf(-z));
}
__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
  bf16x4_t v;
  v[0] = (__bf16)a; v[1] = (__bf16)b; v[2] = (__bf16)c; v[3] = (__bf16)d;
  return *reinterpret_cast<uint2*>(&v);
}
__device__ __forceinline__ void unpack4(uint2 u, float (&f)[4]) {
  f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
  f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
}

// Workgroup -> output tile.  Consecutive workgroup ids go round-robin over the 8 XCDs,
// each with its own L2; giving every XCD one contiguous run of tiles, walked in bands of
// 8 tile-rows, keeps the operand panels an XCD's workgroups share in that XCD's L2.
__device__ __forceinline__ void tile_of_block(int b, int nb, int ntm, int ntn, int& tm, int& tn) {
  const int q = nb >> 3, r = nb & 7;
  const int xcd = b & 7, idx = b >> 3;
  const int L = xcd * q + (xcd < r ? xcd : r) + idx;
  const int GM = 8;
  const int per_group = GM * ntn;
  const int group = L / per_group;
  const int first = group * GM;
  const int gsize = (ntm - first) < GM ? (ntm - first) : GM;
  const int in = L - group * per_group;
  tm = first + in % gsize;
  tn = in / gsize;
}

template <int LA, int LB, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs p) {
  __shared__ __attribute__((aligned(16))) char smem[2 * STAGE_BYTES];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int ntm = (p.M + BM - 1) / BM, ntn = (p.N + BN - 1) / BN;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, ntm, ntn, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 sa[8], sb[8];
  const int nk = (p.K + BK - 1) / BK;
  load_op<LA>(p.A, p.lda, m0, p.M, 0, p.K, tid, sa);
  load_op<LB>(p.B, p.ldb, n0, p.N, 0, p.K, tid, sb);
  store_op<LA>(smem, tid, sa);
  store_op<LB>(smem + TILE_BYTES, tid, sb);
  __syncthreads();

  const int frow = lane & 31;
  const int fk = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = (kt + 1) < nk;
    if (more) {
      load_op<LA>(p.A, p.lda, m0, p.M, (kt + 1) * BK, p.K, tid, sa);
      load_op<LB>(p.B, p.ldb, n0, p.N, (kt + 1) * BK, p.K, tid, sb);
    }
    const char* tA = smem + cur * STAGE_BYTES;
    const char* tB = tA + TILE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8_t fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[i] = *reinterpret_cast<const bf16x8_t*>(tA + lds_off(wm * 128 + i * 32 + frow, ks * 2 + fk));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        fb[j] = *reinterpret_cast<const bf16x8_t*>(tB + lds_off(wn * 128 + j * 32 + frow, ks * 2 + fk));
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (more) {
      char* nA = smem + (cur ^ 1) * STAGE_BYTES;
      store_op<LA>(nA, tid, sa);
      store_op<LB>(nA + TILE_BYTES, tid, sb);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds token m = .. + (lane & 31); for accumulator (i,j), register
  // group g (4 registers) covers features  j*32 + g*8 + (lane >> 5)*4 + {0,1,2,3}.
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + wm * 128 + i * 32 + frow;
    if (m >= p.M) continue;
    int id = 0;
    if (EPI == EPI_GATE || EPI == EPI_DH) {
      id = p.ids[m];
      if ((unsigned)id >= (unsigned)p.E_rows) {
        *p.flag = 1;
        id = id < 0 ? 0 : p.E_rows - 1;
      }
    }
    const size_t orow = (size_t)m * p.N;
    const size_t erow = (size_t)id * p.N;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * 128 + j * 32 + g * 8 + fk * 4;
        if (n >= p.N) continue;
        const float c0 = acc[i][j][4 * g + 0], c1 = acc[i][j][4 * g + 1];
        const float c2 = acc[i][j][4 * g + 2], c3 = acc[i][j][4 * g + 3];
        if (EPI == EPI_BF16) {
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(p.C) + orow + n) = pack4(c0, c1, c2, c3);
        } else if (EPI == EPI_F32) {
          float4* dst = reinterpret_cast<float4*>(reinterpret_cast<float*>(p.C) + orow + n);
          float4 v = make_float4(c0, c1, c2, c3);
          if (p.accumulate) {
            const float4 o = *dst;
            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
          }
          *dst = v;
        } else if (EPI == EPI_GATE) {
          float e[4];
          unpack4(*reinterpret_cast<const uint2*>(p.E + erow + n), e);
          const float c[4] = {c0, c1, c2, c3};
          float h[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) h[q] = c[q] * sigmoidf_fast(c[q]) * e[q];
          if (p.outG) *reinterpret_cast<uint2*>(p.outG + orow + n) = pack4(c0, c1, c2, c3);
          *reinterpret_cast<uint2*>(p.outH + orow + n) = pack4(h[0], h[1], h[2], h[3]);
        } else {  // EPI_DH
          float e[4], gz[4];
          unpack4(*reinterpret_cast<const uint2*>(p.E + erow + n), e);
          unpack4(*reinterpret_cast<const uint2*>(p.inG + orow + n), gz);
          const float c[4] = {c0, c1, c2, c3};
          float du[4], dg[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float sg = sigmoidf_fast(gz[q]);
            du[q] = c[q] * gz[q] * sg;
            dg[q] = c[q] * e[q] * sg * (1.0f + gz[q] * (1.0f - sg));
          }
          *reinterpret_cast<uint2*>(p.outdU + orow + n) = pack4(du[0], du[1], du[2], du[3]);
          *reinterpret_cast<uint2*>(p.outdG + orow + n) = pack4(dg[0], dg[1], dg[2], dg[3]);
        }
      }
    }
  }
}

template <int LA, int LB, int EPI>
hipError_t launch(stem_ctx* ctx, int kid, const GemmArgs& a, hipStream_t s) {
  const int ntm = (a.M + BM - 1) / BM, ntn = (a.N + BN - 1) / BN;
  ProfScope ps(ctx, kid, s);
  hipLaunchKernelGGL((gemm_bf16_kernel<LA, LB, EPI>), dim3(ntm * ntn), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t stem_gemm_bf16(stem_ctx* ctx, int kid, int la, int lb, int epi, const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipSuccess;
  if (la == OP_KC && lb == OP_KC) {
    if (epi == EPI_BF16) return launch<OP_KC, OP_KC, EPI_BF16>(ctx, kid, a, s);
    if (epi == EPI_GATE) return launch<OP_KC, OP_KC, EPI_GATE>(ctx, kid, a, s);
  } else if (la == OP_KC && lb == OP_MC) {
    if (epi == EPI_BF16) return launch<OP_KC, OP_MC, EPI_BF16>(ctx, kid, a, s);
    if (epi == EPI_DH) return launch<OP_KC, OP_MC, EPI_DH>(ctx, kid, a, s);
  } else if (la == OP_MC && lb == OP_MC) {
    if (epi == EPI_F32) return launch<OP_MC, OP_MC, EPI_F32>(ctx, kid, a, s);
  }
  return hipErrorInvalidValue;
}
