// bf16 MFMA GEMMs of the STEM layer (gate, down, and the four backward products)
// for gfx950, with the layer's element-wise work fused into the epilogues.
//
// One kernel template computes  C[m,n] = sum_k Aop[m,k] * Bop[n,k]  on a 256x256
// output tile per workgroup: 4 wavefronts, each a 128x128 quadrant held as 4x4
// accumulators of v_mfma_f32_32x32x16_bf16, K stepped by 64 through five 32 KB LDS
// slots (one operand tile each), so that every global request is made more than a
// whole K tile before its data is needed.
//
// Operands.  "KC" = stored [rows,K] with K contiguous: tiles go global -> LDS directly
// (buffer_load ... lds, 16 bytes per lane, whole 128-byte lines per row; half lines were
// measured to halve the L1 rate).  "MC" = stored [K,rows] with rows contiguous: tiles go
// through registers, are transposed 8x8 there and written to LDS, so the MFMA loop always
// reads 16-byte K-contiguous fragments from one LDS layout.  All loads are buffer loads:
// out-of-range rows / k read as zero, so ragged edges need no branches.
//
// LDS tile layout: row r (an m or n index within the tile) owns 128 bytes = 8 chunks of
// 8 bf16; chunk c of row r sits at chunk slot (c ^ (r >> 1) ^ (((r >> 3) & 3) << 1)) & 7.  With
// the first term a ds_read_b128 of one chunk column over 16 consecutive rows touches all 64
// banks once; the second term spreads rows 8 and 16 apart, which the transposing stores of a
// register-staged operand write together.  Measured per instruction with four wavefronts
// issuing: fragment reads 16 clocks (conflict-free) with or without the second term, those stores
// 64 clocks with it and 128 without; XORing the same two row bits into slot bits 0 and 1 instead
// makes the stores as cheap but the reads conflict 2-way.
//
// Schedule.  One iteration = one K tile = 4 k-steps of 16 MFMAs.  Fragments are double
// buffered in registers: while the MFMAs of k-step s run, the 8 fragment reads of step
// s+1 are issued between them.  The loads of later tiles are spread over the k-steps
// (a vector-memory instruction blocks the issuing wavefront for tens of cycles, during
// which its MFMA queue drains, so they are never issued back to back).  The single
// barrier per iteration sits before the last k-step, so that step overlaps the first
// fragment reads of the next tile, and the wait before it leaves the youngest requests
// in flight.  The loop is unrolled over the slot rotation (5 or 6 K tiles) so that every
// LDS address is a loop-invariant register plus an immediate.
//
// Epilogue.  The MFMA is issued with the N-side fragment as its row operand, so a lane
// holds, for one m, groups of 4 consecutive n.  Each wavefront stages its accumulators
// through LDS (fp32, 32 rows at a time) and reads them back row-contiguous: 16 lanes
// cover 128 consecutive n of one row, so the outputs, the gathered table row and the
// saved activations are all accessed as 16-byte pieces of whole 128-byte lines.
#include "stem_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __amdgpu_buffer_rsrc_t rsrc_t;

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = 256 * BK * 2;  // one operand tile in LDS
constexpr uint32_t OOB = 0x80000000u;  // a buffer offset beyond any operand: reads as zero

__device__ __forceinline__ uint32_t lds_addr(const char* p) {   // p points into LDS
  return (uint32_t)(uintptr_t)(lds_ptr_t)const_cast<char*>(p);
}
// chunk slot swizzle of a tile row (only bits 1..4 of the row: the same for rows 32 apart, so the
// fragments of a wavefront's four 32-row blocks sit at one address plus immediates)
__device__ __forceinline__ int lds_swz(int row) { return ((row >> 1) ^ (((row >> 3) & 3) << 1)) & 7; }
__device__ __forceinline__ uint32_t lds_off(int row, int chunk) {
  return (uint32_t)(row * 128 + (((chunk ^ lds_swz(row)) & 7) << 4));
}

// A buffer resource that moves along the operand: base advances, the record count shrinks.
// The descriptor is rebuilt once per K tile (a handful of scalar instructions), not per load.
struct Window {
  const char* base;
  int left;  // bytes from base to the end of the operand (operands stay below 2 GiB; may go negative)
  rsrc_t r;
  __device__ __forceinline__ void set(const void* p, int64_t bytes) {
    base = reinterpret_cast<const char*>(p);
    left = (int)bytes;
    rebuild();
  }
  __device__ __forceinline__ void rebuild() {
    r = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, left < 0 ? 0 : left, 0x00020000);
  }
  __device__ __forceinline__ rsrc_t rsrc() const { return r; }
  __device__ __forceinline__ void advance(int bytes) { base += bytes; left -= bytes; rebuild(); }
};

// ---- KC operand: global -> LDS direct -----------------------------------------------
// Wavefront w loads row groups g = w*8 + i (8 rows each); lane -> row g*8 + (lane >> 3),
// chunk slot lane & 7; the lane fetches the chunk that belongs in its slot.
struct LoaderKC {
  uint32_t off[8];
  Window win;
  // `skip`: elements by which p already points past the operand's first element (a K slice)
  __device__ __forceinline__ void init(const bf16_t* p, int ld, int rows, int row0, int wave, int lane, int skip) {
    win.set(p, ((int64_t)rows * ld - skip) * 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = (wave * 8 + i) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ lds_swz(row);
      off[i] = (row0 + row) < rows ? (uint32_t)(((int64_t)(row0 + row) * ld + c * 8) * 2) : OOB;
    }
  }
  // load i (0..7) of the tile the window points at, into `tile` (LDS, wave-uniform)
  __device__ __forceinline__ void issue(int i, char* tile, int wave) const {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(win.rsrc(), (lds_ptr_t)(tile + (wave * 8 + i) * 1024), 16, off[i], 0, 0,
                                             0);
  }
  __device__ __forceinline__ void next_tile() { win.advance(BK * 2); }
};

// ---- MC operand: global -> registers -> 8x8 transpose -> LDS ---------------------------
// Thread t owns the 8(k) x 8(rows) block kb = (t >> 3) & 7, rb = (t & 7) + 8 * (t >> 6) of the
// 64 x 256 tile: eight consecutive lanes read the eight 16-byte pieces of one 128-byte line (with
// consecutive lanes on different k rows instead, the same loads cost the products 5 % more time).
// The price is a 4-way bank conflict on the transposed LDS stores, which LDS has room for.
struct LoaderMC {
  uint32_t off0;
  uint32_t ld2;
  Window win;
  uint32_t wbase[4];   // offset within a tile of this thread's rows rb*8 + 2j; row 2j+1 is 128 bytes on
  uint4 st[2][8];   // two tiles' worth of loads may be in flight (the ring schedule); else only set 0
  __device__ __forceinline__ void init(const bf16_t* p, int ld, int rows, int K, int row0, int tid) {
    win.set(p, (int64_t)K * ld * 2);
    ld2 = (uint32_t)ld * 2;
    const int kb = (tid >> 3) & 7, rb = (tid & 7) + 8 * (tid >> 6);
    off0 = (row0 + rb * 8) < rows ? (uint32_t)(((int64_t)kb * 8 * ld + row0 + rb * 8) * 2) : OOB;
#pragma unroll
    for (int j = 0; j < 4; ++j) wbase[j] = lds_off(rb * 8 + 2 * j, kb);
  }
  __device__ __forceinline__ void issue(int kk, int set = 0) {
    const uint32_t o = off0 == OOB ? OOB : off0 + kk * ld2;
    st[set][kk] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(win.rsrc(), o, 0, 0));
  }
  __device__ __forceinline__ void next_tile() { win.advance((int)(BK * ld2)); }
  static __device__ __forceinline__ uint32_t pick(const uint4& v, int q) {
    return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w;
  }
  // rows r of this thread's block, transposed so that k runs along the 16-byte chunk, to the
  // tile at LDS address `tile`.  The store is written as assembly on purpose: for a compiler-made
  // LDS store the compiler first waits for every outstanding direct-to-LDS load (it cannot tell
  // that those go to other slots), which would drain the other operand's requests in the middle
  // of the K tile.  The callers order these stores themselves (lgkmcnt(0) and a barrier before
  // any wavefront reads the tile).
  __device__ __forceinline__ void commit(int r, uint32_t tile, int set = 0) const {
    const int q = r >> 1;
    u32x4_t w;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t lo = pick(st[set][2 * j], q), hi = pick(st[set][2 * j + 1], q);
      // one byte permute: the two high (odd r) or the two low (even r) halves of hi:lo
      w[j] = __builtin_amdgcn_perm(hi, lo, (r & 1) ? 0x07060302u : 0x05040100u);
    }
    const uint32_t a = tile + wbase[q];
    if (r & 1) asm volatile("ds_write_b128 %0, %1 offset:128" ::"v"(a), "v"(w) : "memory");
    else asm volatile("ds_write_b128 %0, %1" ::"v"(a), "v"(w) : "memory");
  }
};

// ---- epilogue math ------------------------------------------------------------------
__device__ __forceinline__ float sigmoidf_fast(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  bf16x8_t v;
#pragma unroll
  for (int q = 0; q < 8; ++q) v[q] = (__bf16)f[q];
  return __builtin_bit_cast(uint4, v);
}
__device__ __forceinline__ void unpack8(uint4 u, float (&f)[8]) {
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    f[2 * q] = __uint_as_float(w[q] << 16);
    f[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
  }
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
  // (KC,KC) products keep their operand tiles in a ring of five 32 KB slots (A and B tiles of
  // successive K tiles in turn) instead of two 64 KB stages: see the main loop.
  constexpr bool RING = (LA == OP_KC && LB == OP_KC);
  // products with exactly one register-staged operand use the same five slots: see their main loop
  constexpr bool RING_MC = ((LA == OP_KC) != (LB == OP_KC));
  static_assert(RING || RING_MC, "at least one operand takes the direct path");
  __shared__ __attribute__((aligned(16))) char smem[5 * TILE_BYTES];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int ntm = (p.M + BM - 1) / BM, ntn = (p.N + BN - 1) / BN;
  int tm, tn;
  if (EPI == EPI_F32 && p.ksplit > 1) {
    // Split along K (weight gradients of narrow layers: few output tiles, long K): slice z of the
    // K tiles, its product stored plainly to slice z of the partial buffer; a second kernel sums
    // the slices in order.  The slice is expressed by moving the operands and shrinking K.
    const int ntiles = ntm * ntn;
    const int z = blockIdx.x / ntiles;
    tile_of_block(blockIdx.x - z * ntiles, ntiles, ntm, ntn, tm, tn);
    const int nk_all = (p.K + BK - 1) / BK;
    const int per = (nk_all + p.ksplit - 1) / p.ksplit;
    const int k0 = z * per * BK;
    const int kmc = (p.K_mc > 0 ? p.K_mc : p.K) - k0;        // rows of a rows-contiguous operand left
    int klen = p.K - k0;
    if (klen > per * BK) klen = per * BK;
    if (klen < 0) klen = 0;
    p.A += LA == OP_KC ? (size_t)k0 : (size_t)k0 * p.lda;
    p.B += LB == OP_KC ? (size_t)k0 : (size_t)k0 * p.ldb;
    p.K = klen;
    p.K_mc = kmc < 0 ? 0 : (kmc < klen ? kmc : klen);
    p.kc_skip = k0;                                          // K-contiguous windows end k0 elements earlier
    p.C = p.ws + (size_t)z * p.M * p.N;
    p.accumulate = 0;
  } else {
    tile_of_block(blockIdx.x, gridDim.x, ntm, ntn, tm, tn);
  }
  const int m0 = tm * BM, n0 = tn * BN;
  // K rotation.  Workgroups on XCD x start their K loop x eighths of the way in and wrap around, so
  // the eight XCDs stream eight different stretches of the operands' rows at any moment instead of
  // the same one (measured: the down product, whose two operands have the same 16 KB row pitch, ran
  // 8 % slower without it; the other products with two direct operands are unchanged, and the
  // weight-gradient products gained nothing from the same rotation, so they do not rotate).  The sum over k is the same set of products in
  // a rotated order.  `rot` is the first K element of this workgroup's loop; 0 = no rotation.
  int rot = 0;
  if (RING && !p.A2) {
    const int nk_all = (p.K + BK - 1) / BK;
    if (nk_all >= 16) rot = (int)((long)(blockIdx.x & 7) * nk_all / 8) * BK;
  }
  if (RING && rot > 0) {   // expressed as two operand pairs: [rot, K) of A, B and then [0, rot)
    p.A2 = p.A; p.B2 = p.B; p.K2 = rot;
    p.A += rot; p.B += rot; p.K -= rot; p.kc_skip += rot;
  }

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  LoaderKC ka, kb_;
  LoaderMC ma, mb;
  if (LA == OP_KC) ka.init(p.A, p.lda, p.M, m0, wave, lane, p.kc_skip); else ma.init(p.A, p.lda, p.M, p.K_mc > 0 ? p.K_mc : p.K, m0, tid);
  if (LB == OP_KC) kb_.init(p.B, p.ldb, p.N, n0, wave, lane, p.kc_skip); else mb.init(p.B, p.ldb, p.N, p.K_mc > 0 ? p.K_mc : p.K, n0, tid);

  // fragments: lane -> row (lane & 31) of a 32-row block, k half (lane >> 5) of a k-step; within a k-step
  // they are read in the order a0,b0,b1,a1,b2,b3,a2,a3
  const int frow = lane & 31, fk = lane >> 5;
  // MFMA pair q (0..7), in an order that consumes fragments in the order they were read
  auto mma2 = [&](int q, bf16x8_t(&fa)[4], bf16x8_t(&fb)[4]) {
    constexpr int ii[16] = {0, 0, 1, 1, 0, 1, 0, 1, 2, 2, 2, 2, 3, 3, 3, 3};
    constexpr int jj[16] = {0, 1, 0, 1, 2, 2, 3, 3, 0, 1, 2, 3, 0, 1, 2, 3};
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int i = ii[2 * q + u], j = jj[2 * q + u];
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
  };

  // A second operand pair (A2, B2, K2; both K-contiguous, same leading dimensions) continues the
  // sum: after the K tiles of the first pair the windows move to the second.
  const int nk1 = (p.K + BK - 1) / BK;
  const int nk = nk1 + ((LA == OP_KC && LB == OP_KC && p.A2) ? (p.K2 + BK - 1) / BK : 0);
  // The gate epilogue reads one gathered table row per output row.  A few K tiles before the end
  // of the main loop each lane touches the 128-byte lines its wavefront will need, so that they
  // travel from HBM to L2 under the MFMA work instead of in a burst when all workgroups reach
  // their epilogues together.  (Measured: 0.05 ms off the gate product at d=2048, F=8192; the dH
  // product gains nothing from the same trick - its lines are evicted again before the epilogue,
  // FETCH_SIZE grows by 30 % - so it does not touch.)
  // The touching loads return asynchronously into their destination registers, so these stay
  // reserved (never reused by the compiler) until the wait that follows the main loop.
  constexpr bool TOUCH = (EPI == EPI_GATE);
  // Token ids of this wavefront's 128 output rows, lane l holding rows l and 64 + l, fetched here so
  // that their latency passes under the main loop.  The epilogue takes each row's id from these
  // registers by a lane permute: loading ids there would put a wait for the newest loads in front of
  // every block of table-row requests, and with it a wait for all the stores issued before them
  // (loads and stores return through one in-order counter), 3 to 4 us per block.
  constexpr bool NEED_IDS = (EPI == EPI_GATE || EPI == EPI_DH || EPI == EPI_GATE_UPE || EPI == EPI_DH_UPE);
  int row_id[2] = {0, 0};
  if (NEED_IDS) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int m = m0 + wm * 128 + h * 64 + lane;
      int id = p.ids[m < p.M ? m : p.M - 1];
      if ((unsigned)id >= (unsigned)p.E_rows) {   // reported to the host, clamped so no access leaves the table
        *p.flag = 1;
        id = id < 0 ? 0 : p.E_rows - 1;
      }
      row_id[h] = id;
    }
  }
  uint32_t touched[4] = {0, 0, 0, 0};
  auto touch_epilogue_inputs = [&]() {
    if (!TOUCH) return;
    const int ncol = n0 + wn * 128;
    const int col = ncol < p.N ? ncol : 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int id = row_id[h];
      const bf16_t* e = p.E + (size_t)id * p.N + col;
      // the second line of the row's 128 columns exists only if the matrix is that wide (d_ff may be
      // 64 modulo 128): otherwise touch the first line twice rather than the next row's memory
      const bf16_t* e2 = col + 64 < p.N ? e + 64 : e;
      asm volatile("global_load_dword %0, %2, off\n\tglobal_load_dword %1, %3, off"
                   : "=&v"(touched[2 * h]), "=&v"(touched[2 * h + 1]) : "v"(e), "v"(e2) : "memory");
    }
  };
  const int touch_at = nk > 8 ? ((nk - 6) & ~1) : -1;   // an even K tile index a few tiles before the end
  bf16x8_t xa[4], xb[4], ya[4], yb[4];
  if constexpr (RING_MC) {
  // ---- one direct and one register-staged operand: five 32 KB slots ---------------------------
  // The register-staged operand's K tile t lives in slot t & 1, the direct operand's in slot
  // 2 + t % 3.  While K tile t is multiplied: the staged loads of tile t+2 are requested during
  // its first k-step (into the register set that tile t's own data left), the direct loads of
  // tile t+2 during the next two k-steps (into the slot tile t-1 left), and in the last k-step
  // before the barrier the registers holding tile t+1 are transposed into LDS.  Every request has
  // more than a whole K tile's time before it is waited for, and two tiles' requests stay in
  // flight across the barrier.
  constexpr bool A_DIRECT = (LA == OP_KC);
  LoaderKC& kd = *(A_DIRECT ? &ka : &kb_);
  LoaderMC& mr = *(A_DIRECT ? &mb : &ma);
  const int wr = A_DIRECT ? wn : wm, wd = A_DIRECT ? wm : wn;
  uint32_t rr_addr[4], rd_addr[2][4];   // staged: slot 1 is an immediate away; direct: [slot pair][k-step]
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const uint32_t sw = (uint32_t)((((ks * 2 + fk) ^ lds_swz(frow)) & 7) << 4);
    rr_addr[ks] = (uint32_t)((wr * 128 + frow) * 128) + sw;
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) rd_addr[pr][ks] = (uint32_t)((2 + 2 * pr) * TILE_BYTES + (wd * 128 + frow) * 128) + sw;
  }
  // fragment q of k-step ks of a K tile with index t6 modulo 6
  auto rfrag_mc = [&](int t6, int ks, int q, bf16x8_t(&fa)[4], bf16x8_t(&fb)[4]) {
    constexpr int isA[8] = {1, 0, 0, 1, 0, 0, 1, 1};
    constexpr int idx[8] = {0, 0, 1, 1, 2, 3, 2, 3};
    const int sr = t6 & 1, sd = t6 % 3;
    const bool direct = (isA[q] != 0) == A_DIRECT;
    const char* src = direct ? smem + rd_addr[sd >> 1][ks] + (sd & 1) * TILE_BYTES + idx[q] * 4096
                             : smem + rr_addr[ks] + sr * TILE_BYTES + idx[q] * 4096;
    if (isA[q]) fa[idx[q]] = *reinterpret_cast<const bf16x8_t*>(src);
    else fb[idx[q]] = *reinterpret_cast<const bf16x8_t*>(src);
  };
  // prologue: staged 0, direct 0, staged 1, direct 1 requested; tile 0 made ready; staged 2 requested
#pragma unroll
  for (int h = 0; h < 2; ++h) {
#pragma unroll
    for (int q = 0; q < 8; ++q) mr.issue(q, h);
    mr.next_tile();
#pragma unroll
    for (int q = 0; q < 8; ++q) kd.issue(q, smem + (2 + h) * TILE_BYTES, wave);
    kd.next_tile();
  }
  asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
#pragma unroll
  for (int q = 0; q < 8; ++q) mr.commit(q, lds_addr(smem), 0);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    rfrag_mc(0, 0, q, xa, xb);
    mr.issue(q, 0);
  }
  mr.next_tile();
  auto mc_iteration = [&](const int t6) __attribute__((always_inline)) {
    const int nsr = (t6 & 1) ^ 1;                    // slot and register set of the staged tile t+1
    char* d2 = smem + (2 + (t6 + 2) % 3) * TILE_BYTES;   // receives the direct tile t+2
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_mc(t6, 1, q, ya, yb);
      if (q < 4) kd.issue(q, d2, wave);
      mma2(q, xa, xb);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_mc(t6, 2, q, xa, xb);
      if (q < 4) kd.issue(4 + q, d2, wave);
      mma2(q, ya, yb);
      __builtin_amdgcn_sched_barrier(0);
    }
    kd.next_tile();
    // pending, oldest first: staged t+1, direct t+1, staged t+2, direct t+2 (8 loads each)
    asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_mc(t6, 3, q, ya, yb);
      mr.commit(q, lds_addr(smem + nsr * TILE_BYTES), nsr);
      mma2(q, xa, xb);
      __builtin_amdgcn_sched_barrier(0);
    }
    // tile t+1 complete in LDS for every wavefront, and nobody reads tile t's slots any more
    asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_mc((t6 + 1) % 6, 0, q, xa, xb);
      mr.issue(q, nsr);
      mma2(q, ya, yb);
      __builtin_amdgcn_sched_barrier(0);
    }
    mr.next_tile();
  };
  int kt = 0;
  for (; kt + 6 <= nk; kt += 6) {
    mc_iteration(0);
    mc_iteration(1);
    mc_iteration(2);
    mc_iteration(3);
    mc_iteration(4);
    mc_iteration(5);
  }
  if (kt < nk) mc_iteration(0);
  if (kt + 1 < nk) mc_iteration(1);
  if (kt + 2 < nk) mc_iteration(2);
  if (kt + 3 < nk) mc_iteration(3);
  if (kt + 4 < nk) mc_iteration(4);
  } else {
  // ---- (KC,KC): ring of five 32 KB slots ------------------------------------------------------
  // Operand tiles alternate through the slots: A of K tile t in slot 2t mod 5, B in slot 2t+1 mod 5.
  // While K tile t is multiplied, A(t+1), B(t+1) are landing or landed and A(t+2) is requested
  // during the first two k-steps into the slot B(t-1) left; after the barrier that ends the reads
  // of K tile t, B(t+2) is requested into A(t)'s slot.  Every request thus has a whole K tile's
  // time (B) or more (A) before it is waited for, a request is always in flight across the
  // barrier, and the wait before the barrier leaves the youngest 8 loads pending.  With two 64 KB
  // stages the loads of a K tile were requested and drained within that tile's own time, and the
  // direct-load stream alone (no MFMA, no fragment reads) took as long as the whole kernel.
  uint32_t ra_addr[3][4], rb_addr[3][4];   // [slot pair][k-step]; the odd slot of a pair is an immediate away
#pragma unroll
  for (int pr = 0; pr < 3; ++pr)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const uint32_t sw = (uint32_t)((((ks * 2 + fk) ^ lds_swz(frow)) & 7) << 4);
      ra_addr[pr][ks] = (uint32_t)(pr * 2 * TILE_BYTES + (wm * 128 + frow) * 128) + sw;
      rb_addr[pr][ks] = (uint32_t)(pr * 2 * TILE_BYTES + (wn * 128 + frow) * 128) + sw;
    }
  auto rfrag_ring = [&](int sa, int sb, int ks, int q, bf16x8_t(&fa)[4], bf16x8_t(&fb)[4]) {
    constexpr int isA[8] = {1, 0, 0, 1, 0, 0, 1, 1};
    constexpr int idx[8] = {0, 0, 1, 1, 2, 3, 2, 3};
    if (isA[q])
      fa[idx[q]] = *reinterpret_cast<const bf16x8_t*>(smem + ra_addr[sa >> 1][ks] + (sa & 1) * TILE_BYTES + idx[q] * 4096);
    else
      fb[idx[q]] = *reinterpret_cast<const bf16x8_t*>(smem + rb_addr[sb >> 1][ks] + (sb & 1) * TILE_BYTES + idx[q] * 4096);
  };
  int a_to_switch = p.A2 ? nk1 : -1, b_to_switch = a_to_switch;
  auto next_A = [&]() {
    if (--a_to_switch == 0) ka.win.set(p.A2, ((int64_t)p.M * p.lda - (p.kc_skip - rot)) * 2); else ka.next_tile();
  };
  auto next_B = [&]() {
    if (--b_to_switch == 0) kb_.win.set(p.B2, ((int64_t)p.N * p.ldb - (p.kc_skip - rot)) * 2); else kb_.next_tile();
  };
  // prologue: A0, B0, A1, B1 into slots 0..3
#pragma unroll
  for (int h = 0; h < 4; ++h) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (h & 1) kb_.issue(q, smem + h * TILE_BYTES, wave); else ka.issue(q, smem + h * TILE_BYTES, wave);
    }
    if (h & 1) next_B(); else next_A();
  }
  asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 8; ++q) rfrag_ring(0, 1, 0, q, xa, xb);
  // K tile t with t mod 5 == tmod (all slot numbers are compile-time constants)
  auto ring_iteration = [&](const int tmod) __attribute__((always_inline)) {
    const int sa = (2 * tmod) % 5, sb = (2 * tmod + 1) % 5;        // this tile
    const int na = (2 * tmod + 2) % 5, nb = (2 * tmod + 3) % 5;    // the next tile
    const int ia = (2 * tmod + 4) % 5;                             // receives A(t+2); B(t+2) goes to sa
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_ring(sa, sb, 1, q, ya, yb);
      if (q < 4) ka.issue(q, smem + ia * TILE_BYTES, wave);
      mma2(q, xa, xb);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_ring(sa, sb, 2, q, xa, xb);
      if (q < 4) ka.issue(4 + q, smem + ia * TILE_BYTES, wave);
      mma2(q, ya, yb);
      __builtin_amdgcn_sched_barrier(0);
    }
    next_A();
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_ring(sa, sb, 3, q, ya, yb);
      mma2(q, xa, xb);
      __builtin_amdgcn_sched_barrier(0);
    }
    // A(t+1) and B(t+1) have landed (only the 8 loads of A(t+2) may be pending) and nobody reads
    // this tile's slots any more
    asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_ring(na, nb, 0, q, xa, xb);
      kb_.issue(q, smem + sa * TILE_BYTES, wave);
      mma2(q, ya, yb);
      __builtin_amdgcn_sched_barrier(0);
    }
    next_B();
  };
  int kt = 0;
  for (; kt + 5 <= nk; kt += 5) {
    if (TOUCH && kt <= touch_at && touch_at < kt + 5) touch_epilogue_inputs();
    ring_iteration(0);
    ring_iteration(1);
    ring_iteration(2);
    ring_iteration(3);
    ring_iteration(4);
  }
  if (TOUCH && kt <= touch_at) touch_epilogue_inputs();
  if (kt < nk) ring_iteration(0);
  if (kt + 1 < nk) ring_iteration(1);
  if (kt + 2 < nk) ring_iteration(2);
  if (kt + 3 < nk) ring_iteration(3);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (TOUCH)   // end of the touched registers' reservation
    asm volatile("" ::"v"(touched[0]), "v"(touched[1]), "v"(touched[2]), "v"(touched[3]));
  __syncthreads();

  // ---- epilogue: per wavefront, 32 rows at a time through LDS ----------------------------
  constexpr int SROW = 528;                   // staged row: 128 fp32 + 16 bytes of padding
  char* stg = smem + wave * 32768;            // 32 x 528 = 16896 bytes used
  const int srow = lane >> 4;                 // row within a group of 4
  const int scol = (lane & 15) * 8;           // first of this lane's 8 consecutive columns
  const int n = n0 + wn * 128 + scol;
  const bool n_ok = n < p.N;
  const int n_ld = n_ok ? n : 0;              // in-bounds column for the prefetching loads
  constexpr bool GATE_LIKE = (EPI == EPI_GATE || EPI == EPI_GATE_UP || EPI == EPI_GATE_UPE);
  constexpr bool DH_LIKE = (EPI == EPI_DH || EPI == EPI_DH_UP || EPI == EPI_DH_UPE);
  constexpr bool USE_E = (EPI == EPI_GATE || EPI == EPI_DH || EPI == EPI_GATE_UPE || EPI == EPI_DH_UPE);
  constexpr bool USE_UP = (EPI == EPI_GATE_UP || EPI == EPI_GATE_UPE || EPI == EPI_DH_UP || EPI == EPI_DH_UPE);
  constexpr bool FUSED = GATE_LIKE || DH_LIKE;

  // Everything the element-wise part needs from memory is requested one 32-row block ahead
  // (8 rows per lane and block), so the gathered table rows arrive while the previous block
  // is being staged and stored.
  // ev: gathered table row, uv: up-projection row (dense and additive variants), gv: saved G row
  uint4 ev[2][8], gv[2][8], uv[2][8];
  auto prefetch = [&](int i, int buf) __attribute__((always_inline)) {
    if (!FUSED) return;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int m = m0 + wm * 128 + i * 32 + pass * 4 + srow;
      const int mc = m < p.M ? m : p.M - 1;
      if (USE_E) {
        const int r = i * 32 + pass * 4 + srow;   // row within the wavefront's 128: held by lane r & 63
        const int id = __builtin_amdgcn_ds_bpermute((r & 63) * 4, row_id[i >> 1]);
        ev[buf][pass] = *reinterpret_cast<const uint4*>(p.E + (size_t)id * p.N + n_ld);
      }
      if (USE_UP) uv[buf][pass] = *reinterpret_cast<const uint4*>(p.inUp + (size_t)mc * p.N + n_ld);
      if (DH_LIKE) gv[buf][pass] = *reinterpret_cast<const uint4*>(p.inG + (size_t)mc * p.N + n_ld);
    }
  };
  // Outputs leave through buffer stores: a lane outside the matrix (ragged last tile) is given an
  // offset beyond the buffer and the hardware drops its store, so the element-wise part below is
  // straight-line code that the compiler schedules as a whole (the staged values of all eight
  // passes are read from LDS up front and the arithmetic of one pass covers the latency of the
  // next; with a branch around every store each pass waited for its own LDS reads: stamps inside
  // the kernel, 5.7 K clocks per 32-row block against 3.6 K of arithmetic).
  auto out_rsrc = [&](void* ptr, int esize) {
    return __builtin_amdgcn_make_buffer_rsrc(ptr, 0, ptr ? (int)((int64_t)p.M * p.N * esize) : 0, 0x00020000);
  };
  rsrc_t r0, r1;   // EPI_BF16 / EPI_F32: C;  gate-like: G (may be absent), H;  dH-like: dU, dG
  if (EPI == EPI_BF16) r0 = r1 = out_rsrc(p.C, 2);
  else if (EPI == EPI_BF16_RES) { r0 = out_rsrc(p.C, 2); r1 = out_rsrc(const_cast<bf16_t*>(p.residual), 2); }
  else if (EPI == EPI_F32) r0 = r1 = out_rsrc(p.C, 4);
  else if (GATE_LIKE) { r0 = out_rsrc(p.outG, 2); r1 = out_rsrc(p.outH, 2); }
  else { r0 = out_rsrc(p.outdU, 2); r1 = out_rsrc(p.outdG, 2); }
  auto store16 = [&](rsrc_t r, uint32_t off, uint4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), r, off, 0, 0);
  };
  prefetch(0, 0);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i + 1 < 4) prefetch(i + 1, (i + 1) & 1);
    // accumulators -> LDS: lane holds row frow, columns j*32 + g*8 + fk*4 .. +3
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x16_t v = acc[i][j];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4_t w = {v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
        *reinterpret_cast<f32x4_t*>(stg + frow * SROW + (j * 32 + g * 8 + fk * 4) * 4) = w;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    f32x4_t cv[8][2];
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int r = pass * 4 + srow;
      cv[pass][0] = *reinterpret_cast<const f32x4_t*>(stg + r * SROW + scol * 4);
      cv[pass][1] = *reinterpret_cast<const f32x4_t*>(stg + r * SROW + scol * 4 + 16);
    }
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int r = pass * 4 + srow;
      const int m = m0 + wm * 128 + i * 32 + r;
      const f32x4_t c0 = cv[pass][0], c1 = cv[pass][1];
      const float c[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
      const bool ok = n_ok && m < p.M;
      const uint32_t o = ok ? (uint32_t)m * (uint32_t)p.N + (uint32_t)n : 0u;   // element index, < 2^30
      const uint32_t o2 = ok ? o * 2u : OOB, o4 = ok ? o * 4u : OOB;
      if (EPI == EPI_BF16) {
        store16(r0, o2, pack8(c));
      } else if (EPI == EPI_BF16_RES) {
        float rz[8], sum[8];
        unpack8(__builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r1, o2, 0, 0)), rz);
#pragma unroll
        for (int q = 0; q < 8; ++q) sum[q] = c[q] + rz[q];
        store16(r0, o2, pack8(sum));
      } else if (EPI == EPI_F32) {
        // the previous value is fetched only when it is to be added to: otherwise the load is out of range and reads zero
        const uint32_t ol = p.accumulate ? o4 : OOB;
        const u32x4_t q0 = __builtin_amdgcn_raw_buffer_load_b128(r0, ol, 0, 0);
        const u32x4_t q1 = __builtin_amdgcn_raw_buffer_load_b128(r0, ol, 16, 0);
        const f32x4_t a0 = __builtin_bit_cast(f32x4_t, q0), a1 = __builtin_bit_cast(f32x4_t, q1);
        const f32x4_t v0 = {c[0] + a0[0], c[1] + a0[1], c[2] + a0[2], c[3] + a0[3]};
        const f32x4_t v1 = {c[4] + a1[0], c[5] + a1[1], c[6] + a1[2], c[7] + a1[3]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v0), r0, o4, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v1), r0, o4, 16, 0);
      } else {
        // e: what SiLU(G) is multiplied by: the gathered row, the up projection, or their sum
        float e[8];
        if (USE_E) unpack8(ev[i & 1][pass], e);
        if (USE_UP) {
          float u[8];
          unpack8(uv[i & 1][pass], u);
#pragma unroll
          for (int q = 0; q < 8; ++q) e[q] = USE_E ? e[q] + u[q] : u[q];
        }
        if (GATE_LIKE) {
          float h[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) h[q] = c[q] * sigmoidf_fast(c[q]) * e[q];
          store16(r0, o2, pack8(c));      // dropped by the hardware when G is not wanted (zero-sized buffer)
          store16(r1, o2, pack8(h));
        } else {  // dH product
          float gz[8], du[8], dg[8];
          unpack8(gv[i & 1][pass], gz);
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            // dU = C SiLU(G) = C g s;  dG = C e SiLU'(G) = C e s (1 + g (1 - s)) = e (dU (1 - s) + C s)
            const float sg = sigmoidf_fast(gz[q]);
            const float cs = c[q] * sg;
            du[q] = cs * gz[q];
            dg[q] = e[q] * fmaf(du[q], 1.0f - sg, cs);
          }
          store16(r0, o2, pack8(du));
          store16(r1, o2, pack8(dg));
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// C[i] = (accumulate ? C[i] : 0) + (sum over the K slices, in slice order, of ws[z][i]); 4 elements per thread
__global__ __launch_bounds__(256) void splitk_sum_f32_kernel(const float* __restrict__ ws, int ksplit, int64_t total,
                                                             float* __restrict__ C, int accumulate) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= total) return;
  f32x4_t s = *reinterpret_cast<const f32x4_t*>(ws + i);
  for (int z = 1; z < ksplit; ++z) s += *reinterpret_cast<const f32x4_t*>(ws + (size_t)z * total + i);
  if (accumulate) s += *reinterpret_cast<const f32x4_t*>(C + i);
  *reinterpret_cast<f32x4_t*>(C + i) = s;
}

template <int LA, int LB, int EPI>
hipError_t launch(stem_ctx* ctx, int kid, const GemmArgs& a, hipStream_t s) {
  const int ntm = (a.M + BM - 1) / BM, ntn = (a.N + BN - 1) / BN;
  if (EPI == EPI_F32 && a.ksplit > 1) {
    if (!a.ws || (a.M * (int64_t)a.N) % 4 != 0) return hipErrorInvalidValue;
    {
      ProfScope ps(ctx, kid, s);
      hipLaunchKernelGGL((gemm_bf16_kernel<LA, LB, EPI>), dim3(ntm * ntn * a.ksplit), dim3(256), 0, s, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t total = (int64_t)a.M * a.N;
    ProfScope ps(ctx, K_SPLITK_REDUCE, s);
    hipLaunchKernelGGL(splitk_sum_f32_kernel, dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, s, a.ws, a.ksplit,
                       total, static_cast<float*>(a.C), a.accumulate);
    return hipGetLastError();
  }
  ProfScope ps(ctx, kid, s);
  hipLaunchKernelGGL((gemm_bf16_kernel<LA, LB, EPI>), dim3(ntm * ntn), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t stem_gemm_bf16(stem_ctx* ctx, int kid, int la, int lb, int epi, const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipSuccess;
  // buffer offsets are 32-bit: every operand must stay below 2 GiB
  const int64_t lim = 0x7fffffff;
  const int64_t kmc = a.K_mc > 0 ? a.K_mc : a.K;
  const int64_t abytes = (la == OP_KC ? (int64_t)a.M : kmc) * a.lda * 2;
  const int64_t bbytes = (lb == OP_KC ? (int64_t)a.N : kmc) * a.ldb * 2;
  if (abytes > lim || bbytes > lim) return hipErrorInvalidValue;
  // so are the outputs' (buffer stores)
  if ((int64_t)a.M * a.N * (epi == EPI_F32 ? 4 : 2) > lim) return hipErrorInvalidValue;
  if (la == OP_KC && lb == OP_KC) {
    if (epi == EPI_BF16) return launch<OP_KC, OP_KC, EPI_BF16>(ctx, kid, a, s);
    if (epi == EPI_BF16_RES) return launch<OP_KC, OP_KC, EPI_BF16_RES>(ctx, kid, a, s);
    if (epi == EPI_GATE) return launch<OP_KC, OP_KC, EPI_GATE>(ctx, kid, a, s);
    if (epi == EPI_DH) return launch<OP_KC, OP_KC, EPI_DH>(ctx, kid, a, s);
    if (epi == EPI_GATE_UP) return launch<OP_KC, OP_KC, EPI_GATE_UP>(ctx, kid, a, s);
    if (epi == EPI_GATE_UPE) return launch<OP_KC, OP_KC, EPI_GATE_UPE>(ctx, kid, a, s);
    if (epi == EPI_DH_UP) return launch<OP_KC, OP_KC, EPI_DH_UP>(ctx, kid, a, s);
    if (epi == EPI_DH_UPE) return launch<OP_KC, OP_KC, EPI_DH_UPE>(ctx, kid, a, s);
  } else if (la == OP_KC && lb == OP_MC) {   // weight gradients: one operand rows-contiguous
    if (epi == EPI_F32) return launch<OP_KC, OP_MC, EPI_F32>(ctx, kid, a, s);
  } else if (la == OP_MC && lb == OP_KC) {
    if (epi == EPI_F32) return launch<OP_MC, OP_KC, EPI_F32>(ctx, kid, a, s);
  }
  return hipErrorInvalidValue;
}
