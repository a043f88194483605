// bf16 MFMA GEMMs of the STEM layer (gate, down, and the four backward products)
// for gfx950, with the layer's element-wise work fused into the epilogues.
//
// One kernel template computes  C[m,n] = sum_k Aop[m,k] * Bop[n,k]  on a 256x256
// output tile per workgroup: 4 wavefronts, each a 128x128 quadrant held as 4x4
// accumulators of v_mfma_f32_32x32x16_bf16, K stepped by 64 through a ring of five 32 KB
// LDS slots (one operand tile each), so that every global request is made more than a
// whole K tile before its data is needed.
//
// Operands.  "KC" = stored [rows,K] with K contiguous, "MC" = stored [K,rows] with rows
// contiguous.  Tiles of both kinds go global -> LDS directly (buffer_load ... lds, 16 bytes per
// lane, whole 128-byte lines; half lines were measured to halve the L1 rate) and keep the
// orientation they have in memory; what differs is the fragment read.  A KC tile gives an MFMA
// fragment (8 consecutive k of one row) as one 16-byte LDS read; an MC tile gives it as two
// ds_read_b64_tr_b16, the LDS read of gfx950 that transposes 16-bit values across 16 lanes.  So
// no operand is ever transposed in memory or in registers: the backward products read the
// weights, the activations and their gradients exactly as the forward pass left them.  (An
// earlier version staged MC tiles through registers with byte permutes and needed the other
// operand K-contiguous, i.e. four transposing kernels per backward pass; its weight-gradient
// loops ran at 2800-3060 clocks per K tile against 2050-2300 for this one.)  All loads are
// buffer loads: out-of-range rows / k read as zero, so ragged edges need no branches.
//
// LDS layout of a KC tile: row r (an m or n index within the tile) owns 128 bytes = 8 chunks of
// 8 bf16; chunk c of row r sits at chunk slot (c ^ (r >> 1) ^ (((r >> 3) & 3) << 1)) & 7.  With
// the first term a ds_read_b128 of one chunk column over 16 consecutive rows touches all 64
// banks once (measured per instruction with four wavefronts issuing: 16 clocks, conflict-free).
// The layout of an MC tile is described at its loader.
//
// Schedule.  One iteration = one K tile = 4 k-steps of 16 MFMAs.  Fragments are double
// buffered in registers: while the MFMAs of k-step s run, the 8 fragment reads of step
// s+1 are issued between them.  The loads of later tiles are spread over the k-steps
// (a vector-memory instruction blocks the issuing wavefront for tens of cycles, during
// which its MFMA queue drains, so they are never issued back to back).  The single
// barrier per iteration sits before the last k-step, so that step overlaps the first
// fragment reads of the next tile, and the wait before it leaves the youngest requests
// in flight.  The loop is unrolled over the slot rotation (5 K tiles) so that every
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
// chunk slot swizzle of a row of a K-contiguous tile (only bits 1..4 of the row: the same for rows 32
// apart, so the fragments of a wavefront's four 32-row blocks sit at one address plus immediates)
__device__ __forceinline__ int lds_swz(int row) { return ((row >> 1) ^ (((row >> 3) & 3) << 1)) & 7; }

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
  // the same descriptor as four words (base, stride 0, byte count, raw-buffer flags), for loads issued as assembly
  __device__ __forceinline__ u32x4_t words() const {
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    return u32x4_t{(uint32_t)b, (uint32_t)(b >> 32) & 0xffffu, (uint32_t)(left < 0 ? 0 : left), 0x00020000u};
  }
  __device__ __forceinline__ void advance(int bytes) { base += bytes; left -= bytes; rebuild(); }
};

// One direct-to-LDS load of 16 bytes per lane, written as assembly.  The compiler orders every
// transposing LDS read (ds_read_b64_tr_b16) after ALL outstanding direct-to-LDS loads it knows of
// (a wait for vmcnt(0) in front of each), which would drain the ring in every k-step; products
// with a rows-contiguous operand therefore issue their loads where the compiler does not see
// them.  Nothing returns to a register, and the kernel's own waits (vmcnt before each barrier) are
// what orders these loads against the reads, as they do for the compiler-made ones.  M0 (the LDS
// destination) is written inside the statement; the compiler never keeps a value of its own in M0
// across other code (it sets it directly in front of each instruction that reads it).
__device__ __forceinline__ void lds_dma_16(u32x4_t rs, uint32_t lds_dst, uint32_t off) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_dst), "v"(off), "s"(rs) : "memory");
}

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
  __device__ __forceinline__ void issue_opaque(int i, char* tile, int wave) const {
    lds_dma_16(win.words(), lds_addr(tile + (wave * 8 + i) * 1024), off[i]);
  }
  __device__ __forceinline__ void next_tile() { win.advance(BK * 2); }
};

// ---- MC operand: global -> LDS as stored, transposed by the fragment reads ----------------
// The 64 x 256 tile keeps the operand's own orientation in LDS: K row k owns 512 bytes = 32 chunks
// of 8 rows-of-the-product (m or n), chunk c at chunk slot c ^ ((k & 3) << 2).  A wavefront's load
// instruction fills 1 KB = two K rows; the lane fetches the chunk that belongs in its slot, so 32
// lanes read one 512-byte stretch of a global row.  ds_read_b64_tr_b16 then delivers MFMA fragments:
// within 16 lanes, lane 4a + b supplies the address of 4 consecutive 16-bit values of "row" a, piece
// b, and lane j receives the j-th value of rows 0..3 (checked on the device with an index pattern).
// With a = k and b = 4-column piece, lane j ends up with 4 consecutive k of column j: half a
// fragment.  The slot swizzle puts the four K rows that 16 lanes read in different 64-byte bank
// groups, so 32 lanes (one LDS pass of a 64-bit read) touch all 64 banks once.
struct LoaderMC {
  uint32_t off[8];
  uint32_t tile_bytes;   // one K tile further along the operand
  Window win;
  __device__ __forceinline__ void init(const bf16_t* p, int ld, int rows, int K, int row0, int wave, int lane) {
    win.set(p, (int64_t)K * ld * 2);
    tile_bytes = (uint32_t)ld * (BK * 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = (wave * 8 + i) * 2 + (lane >> 5);
      const int c = (lane & 31) ^ ((k & 3) << 2);
      off[i] = (row0 + c * 8) < rows ? (uint32_t)(((int64_t)k * ld + row0 + c * 8) * 2) : OOB;
    }
  }
  __device__ __forceinline__ void issue(int i, char* tile, int wave) const {
    lds_dma_16(win.words(), lds_addr(tile + (wave * 8 + i) * 1024), off[i]);
  }
  __device__ __forceinline__ void next_tile() { win.advance((int)tile_bytes); }
  // Byte offset within a tile of this lane's address for the first half (k + 0..3) of fragment i
  // (rows w*128 + i*32 .. +31 of the product) of k-step 0; the second half is 2048 bytes on, k-step
  // s another s * 8192.  Lane = 16 g + 4 a + b: K row 8 (g >> 1) + a, rows 16 (g & 1) + 4 b .. + 3.
  static __device__ __forceinline__ uint32_t frag_off(int w, int i, int lane) {
    const int g = lane >> 4, a = (lane >> 2) & 3, b = lane & 3;
    const int c = w * 16 + i * 4 + 2 * (g & 1) + (b >> 1);
    return (uint32_t)((8 * (g >> 1) + a) * 512 + ((c ^ (a << 2)) << 4) + 8 * (b & 1));
  }
};
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
// one MFMA fragment (8 consecutive k of this lane's row) from a tile in the layout above
__device__ __forceinline__ bf16x8_t lds_read_frag_tr(const char* p) {
  typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_ptr_t) const_cast<char*>(p));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_ptr_t) const_cast<char*>(p + 2048));
  return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

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
// GM tile-rows (down the rows of a band first), keeps the operand panels an XCD's workgroups
// share in that XCD's L2.  GM = 4: the 32 workgroups an XCD runs at a time cover 4 tile-rows
// x 8 tile-columns, i.e. 4 panels of the M-side operand (activations or their gradients, rows
// no other XCD reads) and 8 of the N-side one (mostly weights, which all XCDs read and the
// memory-side cache therefore holds).  With GM = 8 (8 + 4 panels, the same count) every product
// was 1-3 % slower.  The dH product takes GM = 7, which divides neither the 32 tiles an XCD runs
// at a time nor its run: the XCDs then sit at different rows and columns of their bands, and
// their epilogues (each reads a G tile and writes two tiles) meet less often: 0.565 ms with
// 8, 0.545 with 4 or 6, 0.537 with 3 or 5, 0.532 with 7, 0.545-0.55 with 9, 11, 13
// (d_model 2048, d_ff 8192, 16384 tokens).
template <int GM>
__device__ __forceinline__ void tile_of_block(int b, int nb, int ntm, int ntn, int& tm, int& tn) {
  const int q = nb >> 3, r = nb & 7;
  const int xcd = b & 7, idx = b >> 3;
  const int L = xcd * q + (xcd < r ? xcd : r) + idx;
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
  __shared__ __attribute__((aligned(16))) char smem[5 * TILE_BYTES];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int ntm = (p.M + BM - 1) / BM, ntn = (p.N + BN - 1) / BN;
  constexpr int BAND = (EPI == EPI_DH || EPI == EPI_DH_UP || EPI == EPI_DH_UPE) ? 7 : 4;   // see tile_of_block
  int tm, tn;
  if (EPI == EPI_F32 && p.ksplit > 1) {
    // Split along K (weight gradients of narrow layers: few output tiles, long K): slice z of the
    // K tiles, its product stored plainly to slice z of the partial buffer; a second kernel sums
    // the slices in order.  The slice is expressed by moving the operands and shrinking K.
    const int ntiles = ntm * ntn;
    const int z = blockIdx.x / ntiles;
    tile_of_block<BAND>(blockIdx.x - z * ntiles, ntiles, ntm, ntn, tm, tn);
    const int nk_all = (p.K + BK - 1) / BK;
    const int per = (nk_all + p.ksplit - 1) / p.ksplit;
    const int k0 = z * per * BK;
    int klen = p.K - k0;
    if (klen > per * BK) klen = per * BK;
    if (klen < 0) klen = 0;
    p.A += LA == OP_KC ? (size_t)k0 : (size_t)k0 * p.lda;
    p.B += LB == OP_KC ? (size_t)k0 : (size_t)k0 * p.ldb;
    p.K = klen;
    p.kc_skip = k0;                                          // K-contiguous windows end k0 elements earlier
    p.C = p.ws + (size_t)z * p.M * p.N;
    p.accumulate = 0;
  } else {
    tile_of_block<BAND>(blockIdx.x, gridDim.x, ntm, ntn, tm, tn);
  }
  const int m0 = tm * BM, n0 = tn * BN;
  // K rotation.  Workgroups on XCD x start their K loop x eighths of the way in and wrap around, so
  // the eight XCDs stream eight different stretches of the operands' rows at any moment instead of
  // the same one (measured: the down product, whose two operands have the same 16 KB row pitch, ran
  // 8 % slower without it; the other products with two direct operands are unchanged, and the
  // weight-gradient products gained nothing from the same rotation, so they do not rotate).  The sum over k is the same set of products in
  // a rotated order.  `rot` is the first K element of this workgroup's loop; 0 = no rotation.
  int rot = 0;
  if (LA == OP_KC && LB == OP_KC && !p.A2) {
    const int nk_all = (p.K + BK - 1) / BK;
    if (nk_all >= 16) rot = (int)((long)(blockIdx.x & 7) * nk_all / 8) * BK;
  }
  if (LA == OP_KC && LB == OP_KC && rot > 0) {   // expressed as two operand pairs: [rot, K) of A, B and then [0, rot)
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
  LoaderMC da, db;
  if (LA == OP_KC) ka.init(p.A, p.lda, p.M, m0, wave, lane, p.kc_skip); else da.init(p.A, p.lda, p.M, p.K, m0, wave, lane);
  if (LB == OP_KC) kb_.init(p.B, p.ldb, p.N, n0, wave, lane, p.kc_skip); else db.init(p.B, p.ldb, p.N, p.K, n0, wave, lane);

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

  // A second operand pair (A2, B2, K2; same layouts and leading dimensions as the first; A
  // K-contiguous) continues the sum: after the K tiles of the first pair the windows move to the second.
  const int nk1 = (p.K + BK - 1) / BK;
  const int nk = nk1 + ((LA == OP_KC && p.A2) ? (p.K2 + BK - 1) / BK : 0);
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
  // ---- main loop: ring of five 32 KB slots -----------------------------------------------------
  // Operand tiles alternate through the slots: A of K tile t in slot 2t mod 5, B in slot 2t+1 mod 5.
  // While K tile t is multiplied, A(t+1), B(t+1) are landing or landed and A(t+2) is requested
  // during the first two k-steps into the slot B(t-1) left; after the barrier that ends the reads
  // of K tile t, B(t+2) is requested into A(t)'s slot.  Every request thus has a whole K tile's
  // time (B) or more (A) before it is waited for, a request is always in flight across the
  // barrier, and the wait before the barrier leaves the youngest 8 loads pending.  With two 64 KB
  // stages the loads of a K tile were requested and drained within that tile's own time, and the
  // direct-load stream alone (no MFMA, no fragment reads) took as long as the whole kernel.
  // [slot pair][x]; the odd slot of a pair is an immediate away.  x = k-step for a K-contiguous operand
  // (whose swizzle depends on it; the fragment index is an immediate), x = fragment for a
  // rows-contiguous one (the other way round).
  uint32_t ra_addr[3][4], rb_addr[3][4];
#pragma unroll
  for (int pr = 0; pr < 3; ++pr)
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const uint32_t sw = (uint32_t)((((x * 2 + fk) ^ lds_swz(frow)) & 7) << 4);
      ra_addr[pr][x] = (uint32_t)(pr * 2 * TILE_BYTES) +
                       (LA == OP_KC ? (uint32_t)((wm * 128 + frow) * 128) + sw : LoaderMC::frag_off(wm, x, lane));
      rb_addr[pr][x] = (uint32_t)(pr * 2 * TILE_BYTES) +
                       (LB == OP_KC ? (uint32_t)((wn * 128 + frow) * 128) + sw : LoaderMC::frag_off(wn, x, lane));
    }
  auto rfrag_ring = [&](int sa, int sb, int ks, int q, bf16x8_t(&fa)[4], bf16x8_t(&fb)[4]) {
    constexpr int isA[8] = {1, 0, 0, 1, 0, 0, 1, 1};
    constexpr int idx[8] = {0, 0, 1, 1, 2, 3, 2, 3};
    if (isA[q]) {
      if (LA == OP_KC)
        fa[idx[q]] = *reinterpret_cast<const bf16x8_t*>(smem + ra_addr[sa >> 1][ks] + (sa & 1) * TILE_BYTES + idx[q] * 4096);
      else
        fa[idx[q]] = lds_read_frag_tr(smem + ra_addr[sa >> 1][idx[q]] + (sa & 1) * TILE_BYTES + ks * 8192);
    } else {
      if (LB == OP_KC)
        fb[idx[q]] = *reinterpret_cast<const bf16x8_t*>(smem + rb_addr[sb >> 1][ks] + (sb & 1) * TILE_BYTES + idx[q] * 4096);
      else
        fb[idx[q]] = lds_read_frag_tr(smem + rb_addr[sb >> 1][idx[q]] + (sb & 1) * TILE_BYTES + ks * 8192);
    }
  };
  int a_to_switch = p.A2 ? nk1 : -1, b_to_switch = a_to_switch;
  auto next_A = [&]() {
    if constexpr (LA == OP_KC) {
      if (--a_to_switch == 0) ka.win.set(p.A2, ((int64_t)p.M * p.lda - (p.kc_skip - rot)) * 2); else ka.next_tile();
    } else {
      da.next_tile();
    }
  };
  auto next_B = [&]() {
    if constexpr (LB == OP_KC) {
      if (--b_to_switch == 0) kb_.win.set(p.B2, ((int64_t)p.N * p.ldb - (p.kc_skip - rot)) * 2); else kb_.next_tile();
    } else {
      if (--b_to_switch == 0) db.win.set(p.B2, (int64_t)p.K2 * p.ldb * 2); else db.next_tile();
    }
  };
  constexpr bool OPAQUE = (LA == OP_MC || LB == OP_MC);   // see lds_dma_16
  auto issue_A = [&](int q, char* tile) {
    if constexpr (LA != OP_KC) da.issue(q, tile, wave);
    else if constexpr (OPAQUE) ka.issue_opaque(q, tile, wave);
    else ka.issue(q, tile, wave);
  };
  auto issue_B = [&](int q, char* tile) {
    if constexpr (LB != OP_KC) db.issue(q, tile, wave);
    else if constexpr (OPAQUE) kb_.issue_opaque(q, tile, wave);
    else kb_.issue(q, tile, wave);
  };
  // prologue: A0, B0, A1, B1 into slots 0..3
#pragma unroll
  for (int h = 0; h < 4; ++h) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (h & 1) issue_B(q, smem + h * TILE_BYTES); else issue_A(q, smem + h * TILE_BYTES);
    }
    if (h & 1) next_B(); else next_A();
  }
  // A0 and B0 have landed; A1 and B1 stay in flight across the barrier.  (A plain __syncthreads() here
  // makes the compiler wait for every direct-to-LDS load it knows of, i.e. for all four tiles: stamps
  // inside the kernel, 8-9 K clocks to the first MFMA against 5-6 K.)
  asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
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
      if (q < 4) issue_A(q, smem + ia * TILE_BYTES);
      mma2(q, xa, xb);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      rfrag_ring(sa, sb, 2, q, xa, xb);
      if (q < 4) issue_A(4 + q, smem + ia * TILE_BYTES);
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
      issue_B(q, smem + sa * TILE_BYTES);
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
  const int64_t abytes = (la == OP_KC ? (int64_t)a.M : (int64_t)a.K) * a.lda * 2;
  const int64_t bbytes = (lb == OP_KC ? (int64_t)a.N : (int64_t)std::max(a.K, a.K2)) * a.ldb * 2;
  if (abytes > lim || bbytes > lim) return hipErrorInvalidValue;
  if (a.A2 && la != OP_KC) return hipErrorInvalidValue;   // a second operand pair needs a K-contiguous A
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
  } else if (la == OP_KC && lb == OP_MC) {  // activation gradients: the weight as stored, rows-contiguous
    if (epi == EPI_BF16) return launch<OP_KC, OP_MC, EPI_BF16>(ctx, kid, a, s);
    if (epi == EPI_DH) return launch<OP_KC, OP_MC, EPI_DH>(ctx, kid, a, s);
    if (epi == EPI_DH_UP) return launch<OP_KC, OP_MC, EPI_DH_UP>(ctx, kid, a, s);
    if (epi == EPI_DH_UPE) return launch<OP_KC, OP_MC, EPI_DH_UPE>(ctx, kid, a, s);
  } else if (la == OP_MC && lb == OP_MC) {  // weight gradients: both operands [K, rows], rows contiguous
    if (epi == EPI_F32) return launch<OP_MC, OP_MC, EPI_F32>(ctx, kid, a, s);
  }
  return hipErrorInvalidValue;
}
