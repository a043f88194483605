// Gradient of the per-layer table, restricted to the rows a batch touches:
// stable LSD radix sort of (token id, position), distinct ids with run offsets, and a
// fixed-order segmented sum of the per-token row gradients.  Integer results are unique,
// floating sums use one fixed association, so every run gives the same bits.
#include "stem_internal.h"

namespace {

constexpr int RADIX_BITS = 6;          // one digit value per lane of a wavefront
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_WAVES = 16;         // wavefronts per workgroup
constexpr int KEYS_PER_WAVE = 256;     // 4 rounds of 64
constexpr int SORT_TILE = SORT_WAVES * KEYS_PER_WAVE;

__device__ __forceinline__ int load_key(const int32_t* __restrict__ keys, int64_t i, int V, int first_pass,
                                        int32_t* flag) {
  int k = keys[i];
  if (first_pass && (unsigned)k >= (unsigned)V) {
    *flag = 1;
    k = k < 0 ? 0 : V - 1;
  }
  return k;
}

// counts[d * nW + gw] = number of keys with digit d among wavefront gw's 256 keys
__global__ __launch_bounds__(1024) void sort_count_kernel(const int32_t* __restrict__ keys, int64_t T, int V,
                                                          int shift, int first_pass, int nW,
                                                          int32_t* __restrict__ counts, int32_t* flag) {
  __shared__ int hist[SORT_WAVES][RADIX];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int gw = blockIdx.x * SORT_WAVES + wave;
  hist[wave][lane] = 0;
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int r = 0; r < KEYS_PER_WAVE / 64; ++r) {
    const int64_t i = (int64_t)gw * KEYS_PER_WAVE + r * 64 + lane;
    if (i < T) {
      const int d = (load_key(keys, i, V, first_pass, flag) >> shift) & (RADIX - 1);
      atomicAdd(&hist[wave][d], 1);
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (gw < nW) counts[lane * nW + gw] = hist[wave][lane];
}

// in-place exclusive scan of n ints by one workgroup of 1024 threads
__global__ __launch_bounds__(1024) void scan_kernel(int32_t* __restrict__ a, int n) {
  __shared__ int wsum[16];
  __shared__ int carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (n + 1023) / 1024;
  const int b = tid * per, e = min(n, b + per);
  int s = 0;
  for (int i = b; i < e; ++i) s += a[i];
  int inc = s;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  if (tid == 0) {
    int c = 0;
    for (int w = 0; w < 16; ++w) { const int t = wsum[w]; wsum[w] = c; c += t; }
    carry_s = c;
  }
  __syncthreads();
  int run = wsum[wave] + inc - s;
  for (int i = b; i < e; ++i) { const int t = a[i]; a[i] = run; run += t; }
}

// Stable scatter by digit.  Within a wavefront, a key's rank among equal digits of the
// same 64-key round comes from ballots; rounds and wavefronts are ordered by the scan.
__global__ __launch_bounds__(1024) void sort_scatter_kernel(const int32_t* __restrict__ keys,
                                                            const int32_t* __restrict__ vals, int64_t T, int V,
                                                            int shift, int first_pass, int nW,
                                                            const int32_t* __restrict__ counts,
                                                            int32_t* __restrict__ out_keys,
                                                            int32_t* __restrict__ out_vals, int32_t* flag) {
  __shared__ int base[SORT_WAVES][RADIX];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int gw = blockIdx.x * SORT_WAVES + wave;
  if (gw >= nW) return;
  base[wave][lane] = counts[lane * nW + gw];
  __builtin_amdgcn_wave_barrier();
  const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll 1
  for (int r = 0; r < KEYS_PER_WAVE / 64; ++r) {
    const int64_t i = (int64_t)gw * KEYS_PER_WAVE + r * 64 + lane;
    const bool valid = i < T;
    int key = 0, val = 0, d = 0;
    if (valid) {
      key = load_key(keys, i, V, first_pass, flag);
      val = first_pass ? (int)i : vals[i];
      d = (key >> shift) & (RADIX - 1);
    }
    uint64_t same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < RADIX_BITS; ++b) {
      const bool bit = (d >> b) & 1;
      const uint64_t bb = __ballot(valid && bit);
      same &= bit ? bb : ~bb;
    }
    int pos = 0;
    if (valid) {
      const int rank = __popcll(same & below);
      pos = base[wave][d] + rank;
    }
    __builtin_amdgcn_wave_barrier();
    if (valid && (same & below) == 0) base[wave][d] += __popcll(same);
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      out_keys[pos] = key;
      out_vals[pos] = val;
    }
  }
}

// Distinct ids, run offsets, and for every sorted position the index of its run.
constexpr int UNIQ_ITEMS = 8;
__global__ __launch_bounds__(1024) void unique_kernel(const int32_t* __restrict__ sorted, int64_t T,
                                                      int32_t* __restrict__ uniq_ids,
                                                      int32_t* __restrict__ seg_offsets,
                                                      int32_t* __restrict__ n_uniq, int32_t* __restrict__ seg_of) {
  __shared__ int wsum[16];
  __shared__ int total_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int carry = 0;  // runs started before this sweep
  for (int64_t sweep = 0; sweep < T; sweep += 1024 * UNIQ_ITEMS) {
    const int64_t b = sweep + (int64_t)tid * UNIQ_ITEMS;
    int key[UNIQ_ITEMS];
    int prev = (b > 0 && b <= T) ? sorted[b - 1] : -1;
    int heads = 0;
    unsigned headmask = 0;
#pragma unroll
    for (int u = 0; u < UNIQ_ITEMS; ++u) {
      const int64_t k = b + u;
      if (k < T) {
        key[u] = sorted[k];
        const bool h = (k == 0) || key[u] != prev;
        prev = key[u];
        if (h) { ++heads; headmask |= 1u << u; }
      }
    }
    int inc = heads;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o);
      if (lane >= o) inc += t;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    if (tid == 0) {
      int c = 0;
      for (int w = 0; w < 16; ++w) { const int t = wsum[w]; wsum[w] = c; c += t; }
      total_s = c;
    }
    __syncthreads();
    int run = carry + wsum[wave] + inc - heads;  // runs started before this thread's first item
#pragma unroll
    for (int u = 0; u < UNIQ_ITEMS; ++u) {
      const int64_t k = b + u;
      if (k < T) {
        if (headmask & (1u << u)) {
          uniq_ids[run] = key[u];
          seg_offsets[run] = (int)k;
          ++run;
        }
        seg_of[k] = run - 1;
      }
    }
    carry += total_s;
    __syncthreads();
  }
  if (tid == 0) {
    seg_offsets[carry] = (int)T;
    *n_uniq = carry;
  }
}


// ---- one-workgroup path: sort, unique and run index in a single launch ---------------
// When bits(V-1) + bits(T-1) <= 32 the pair (id, position) packs into one 32-bit key, so
// two 64 KB LDS buffers hold the whole problem (T <= 16384).  The passes run over the id
// bits only; the position bits ride along and make the order total.
constexpr int FUSED_MAX_T = 16384;

__global__ __launch_bounds__(1024) void sort_unique_fused_kernel(const int32_t* __restrict__ ids, int T, int V,
                                                                 int pos_bits, int passes,
                                                                 int32_t* __restrict__ sorted_ids,
                                                                 int32_t* __restrict__ perm,
                                                                 int32_t* __restrict__ uniq_ids,
                                                                 int32_t* __restrict__ seg_offsets,
                                                                 int32_t* __restrict__ n_uniq,
                                                                 int32_t* __restrict__ seg_of, int32_t* flag) {
  __shared__ uint32_t buf[2][FUSED_MAX_T];
  __shared__ int table[RADIX * SORT_WAVES];  // [digit][wave], scanned in place
  __shared__ __attribute__((aligned(16))) uint8_t cnt8[SORT_WAVES][RADIX][16];
  __shared__ int wsum[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per_wave = (T + SORT_WAVES - 1) / SORT_WAVES;      // contiguous keys per wavefront
  const int w0 = wave * per_wave, w1 = min(T, w0 + per_wave);
  const uint32_t pos_mask = (1u << pos_bits) - 1u;
  constexpr int ITEMS = FUSED_MAX_T / 1024;
  {
    int kv[ITEMS];
#pragma unroll
    for (int u = 0; u < ITEMS; ++u) kv[u] = (tid + 1024 * u) < T ? ids[tid + 1024 * u] : 0;
    bool bad = false;
#pragma unroll
    for (int u = 0; u < ITEMS; ++u) {
      const int i = tid + 1024 * u;
      int k = kv[u];
      if ((unsigned)k >= (unsigned)V) { bad = true; k = k < 0 ? 0 : V - 1; }
      if (i < T) buf[0][i] = ((uint32_t)k << pos_bits) | (uint32_t)i;
    }
    if (bad) *flag = 1;
  }
  __syncthreads();
  const uint64_t below = (1ull << lane) - 1ull;
  int cur = 0;
  // Per pass and wavefront: 16 rounds of 64 keys.  A key's rank among equal digits of its round
  // comes from ballots; the per-round digit counts go to cnt8[wave][digit][round] (bytes), lane d
  // then turns digit d's 16 counts into running offsets, so no round waits for the one before.
  for (int p = 0; p < passes; ++p) {
    const int shift = pos_bits + p * RADIX_BITS;
    uint32_t key[ITEMS];
    uint32_t dr[ITEMS];  // digit | rank << 8 | valid << 16
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      const int i = w0 + r * 64 + lane;
      key[r] = i < w1 ? buf[cur][i] : 0u;
    }
    *reinterpret_cast<uint4*>(&cnt8[wave][lane][0]) = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      const bool valid = (w0 + r * 64 + lane) < w1;
      const int d = (key[r] >> shift) & (RADIX - 1);
      uint64_t same = __ballot(valid);
#pragma unroll
      for (int b = 0; b < RADIX_BITS; ++b) {
        const bool bit = (d >> b) & 1;
        const uint64_t bb = __ballot(valid && bit);
        same &= bit ? bb : ~bb;
      }
      const int rank = __popcll(same & below);
      if (valid && rank == 0) cnt8[wave][d][r] = (uint8_t)__popcll(same);
      dr[r] = (uint32_t)d | ((uint32_t)rank << 8) | (valid ? 1u << 16 : 0u);
    }
    __builtin_amdgcn_wave_barrier();
    // lane = digit: running offsets over the rounds
    const uint4 cv = *reinterpret_cast<const uint4*>(&cnt8[wave][lane][0]);
    const uint32_t cw[4] = {cv.x, cv.y, cv.z, cv.w};
    int pre[ITEMS];
    int tot = 0;
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      pre[r] = tot;
      tot += (int)((cw[r >> 2] >> ((r & 3) * 8)) & 0xffu);
    }
    table[lane * SORT_WAVES + wave] = tot;
    __syncthreads();
    {  // exclusive scan of the 1024 table entries, one per thread
      const int v = table[tid];
      int inc = v;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
      }
      if (lane == 63) wsum[wave] = inc;
      __syncthreads();
      if (tid == 0) {
        int c = 0;
        for (int w = 0; w < 16; ++w) { const int t = wsum[w]; wsum[w] = c; c += t; }
      }
      __syncthreads();
      table[tid] = wsum[wave] + inc - v;
    }
    __syncthreads();
    const int base = table[lane * SORT_WAVES + wave];  // first output slot of (digit = lane, this wavefront)
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
      const int d = dr[r] & 0xff;
      const int start = __shfl(base + pre[r], d);
      if (dr[r] >> 16) buf[cur ^ 1][start + (int)((dr[r] >> 8) & 0xff)] = key[r];
    }
    __syncthreads();
    cur ^= 1;
  }
  // Unpack and number the runs, position k = u * 1024 + tid throughout (coalesced in global memory,
  // conflict-free in LDS; with 16 consecutive positions per thread instead, every LDS access of this
  // part was a 16-way bank conflict and the part took 14 of the kernel's 47 us).
  // A position's run index is the number of run heads at or before it, minus one: heads of earlier
  // (sweep, wavefront) pairs from a scanned table of ballot counts, heads of earlier lanes from the ballot.
  int* cnt = table;                     // [sweep * SORT_WAVES + wave], reused
  uint64_t headmask[ITEMS];
  int idv[ITEMS];
#pragma unroll
  for (int u = 0; u < ITEMS; ++u) {
    const int k = tid + 1024 * u;
    bool head = false;
    idv[u] = 0;
    if (k < T) {
      const uint32_t key = buf[cur][k];
      const int id = (int)(key >> pos_bits);
      idv[u] = id;
      sorted_ids[k] = id;
      perm[k] = (int)(key & pos_mask);
      head = (k == 0) || id != (int)(buf[cur][k - 1] >> pos_bits);
    }
    headmask[u] = __ballot(head);
    if (lane == 0) cnt[u * SORT_WAVES + wave] = __popcll(headmask[u]);
  }
  __syncthreads();
  {  // exclusive scan of the ITEMS * SORT_WAVES = 256 counts by the first four wavefronts
    int v = 0, inc = 0;
    if (tid < ITEMS * SORT_WAVES) {
      v = cnt[tid];
      inc = v;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
      }
      if (lane == 63) wsum[wave] = inc;
    }
    __syncthreads();
    if (tid < ITEMS * SORT_WAVES) {
      int before = 0;
      for (int w = 0; w < wave; ++w) before += wsum[w];
      cnt[tid] = before + inc - v;
      if (tid == ITEMS * SORT_WAVES - 1) {
        const int total = before + inc;
        seg_offsets[total] = T;
        *n_uniq = total;
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < ITEMS; ++u) {
    const int k = tid + 1024 * u;
    if (k < T) {
      const bool head = (headmask[u] >> lane) & 1ull;
      const int run = cnt[u * SORT_WAVES + wave] + __popcll(headmask[u] & below) + (head ? 0 : -1);
      if (head) { uniq_ids[run] = idv[u]; seg_offsets[run] = k; }
      seg_of[k] = run;
    }
  }
}

// ---- segmented sum -----------------------------------------------------------------
constexpr int SEG_ROWS = 32;  // sorted positions per chunk

template <bool BF16> struct RowVec;
template <> struct RowVec<true> {
  static constexpr int COLS = 8;
  typedef __attribute__((ext_vector_type(4))) uint32_t raw_t;
  static __device__ __forceinline__ raw_t load(const void* base, int64_t row, int F, int col) {
    return __builtin_nontemporal_load(reinterpret_cast<const raw_t*>(reinterpret_cast<const bf16_t*>(base) + row * F + col));
  }
  static __device__ __forceinline__ void add(const raw_t& v, float (&acc)[8]) {
    const uint32_t w[4] = {v[0], v[1], v[2], v[3]};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc[2 * q] += __uint_as_float(w[q] << 16);
      acc[2 * q + 1] += __uint_as_float(w[q] & 0xffff0000u);
    }
  }
};
template <> struct RowVec<false> {
  static constexpr int COLS = 4;
  typedef float4 raw_t;
  static __device__ __forceinline__ raw_t load(const void* base, int64_t row, int F, int col) {
    return *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + row * F + col);
  }
  static __device__ __forceinline__ void add(const raw_t& v, float (&acc)[4]) {
    acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
  }
};

template <int COLS>
__device__ __forceinline__ void store_cols(float* dst, const float (&a)[COLS]) {
#pragma unroll
  for (int q = 0; q < COLS; q += 4) *reinterpret_cast<float4*>(dst + q) = make_float4(a[q], a[q + 1], a[q + 2], a[q + 3]);
}

// One workgroup sums the rows of sorted positions [c*SEG_ROWS, (c+1)*SEG_ROWS) for a slab
// of 256*COLS columns, in ascending position.  A run that lies wholly inside the chunk
// is written to its output row; the (at most two) pieces of runs that cross the chunk's
// borders go to part[c][0] (piece holding the chunk's first position) or part[c][1].
// The chunk's row numbers and run indices are fetched once into LDS, so all row loads can
// be in flight together and run ends need no further global reads.
template <bool BF16>
__global__ __launch_bounds__(256) void seg_reduce_kernel(const void* __restrict__ dU,
                                                         const int32_t* __restrict__ perm,
                                                         const int32_t* __restrict__ seg_of, int64_t T, int F,
                                                         float* __restrict__ dE_rows,
                                                         float* __restrict__ part) {
  constexpr int COLS = RowVec<BF16>::COLS;
  __shared__ int s_perm[SEG_ROWS];
  __shared__ int s_seg[SEG_ROWS + 2];  // [0] = run of the position before the chunk, [n+1] = of the one after
  const int c = blockIdx.y;
  const int k0 = c * SEG_ROWS;
  const int k1 = (int)min((int64_t)k0 + SEG_ROWS, T);
  const int n = k1 - k0;
  const int tid = threadIdx.x;
  if (tid < n) s_perm[tid] = perm[k0 + tid];
  if (tid < n + 2) {
    const int64_t k = (int64_t)k0 - 1 + tid;
    s_seg[tid] = (k >= 0 && k < T) ? seg_of[k] : -1;
  }
  __syncthreads();
  const int col = (blockIdx.x * 256 + tid) * COLS;
  if (col >= F) return;
  const int first_seg = s_seg[1], last_seg = s_seg[n];
  const bool first_open = s_seg[0] == first_seg;      // the first run began before the chunk
  const bool last_open = s_seg[n + 1] == last_seg;    // the last run goes on after the chunk
  float acc[COLS];
#pragma unroll
  for (int q = 0; q < COLS; ++q) acc[q] = 0.f;
  int cur = first_seg;

  auto flush = [&](int j) {
    const bool open = (j == first_seg && first_open) || (j == last_seg && last_open);
    float* dst = open ? part + ((int64_t)c * 2 + (j == first_seg ? 0 : 1)) * F + col
                      : dE_rows + (int64_t)j * F + col;
    store_cols<COLS>(dst, acc);
  };

  // all of the chunk's row loads are requested before the first store: loads and stores return
  // through one in-order counter, so a load requested after a store is not seen before that store
  // has been acknowledged
  constexpr int UNR = SEG_ROWS;
#pragma unroll
  for (int kb = 0; kb < SEG_ROWS; kb += UNR) {
    typename RowVec<BF16>::raw_t data[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u)
      if (kb + u < n) data[u] = RowVec<BF16>::load(dU, s_perm[kb + u], F, col);
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      if (kb + u < n) {
        const int sg = s_seg[kb + u + 1];
        if (sg != cur) {
          flush(cur);
          cur = sg;
#pragma unroll
          for (int q = 0; q < COLS; ++q) acc[q] = 0.f;
        }
        RowVec<BF16>::add(data[u], acc);
      }
    }
  }
  flush(cur);
}

// The chunk in which a border-crossing run starts adds up that run's pieces: workgroup = that chunk
// and a slab of 64 * COLS columns; the run's pieces are cut into four consecutive stretches, one per
// wavefront, each summed in chunk order, and the four sums are added in order.  (One fixed
// association, so every run gives the same bits.  With one thread summing all of a run's pieces the
// most frequent id's 69 pieces were a chain of five dependent rounds of loads.)
template <int COLS>
__global__ __launch_bounds__(256) void seg_combine_kernel(const int32_t* __restrict__ seg_of,
                                                          const int32_t* __restrict__ seg_offsets, int64_t T,
                                                          int F, float* __restrict__ dE_rows,
                                                          const float* __restrict__ part) {
  __shared__ float red[3][64][COLS + 1];
  const int c = blockIdx.x;
  const int k0 = c * SEG_ROWS;
  const int64_t k1 = (int64_t)k0 + SEG_ROWS;
  if (k1 >= T) return;                                 // nothing after this chunk
  // the four run indices that decide whether this chunk has anything to do, requested together
  const int j = seg_of[k1 - 1], after = seg_of[k1], first = seg_of[k0], before = k0 > 0 ? seg_of[k0 - 1] : -1;
  if (after != j) return;                              // the last run ends with the chunk
  if (first == j && before == j) return;               // the run began in an earlier chunk
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = (blockIdx.y * 64 + lane) * COLS;
  const bool live = col < F;
  const int slot = (first == j) ? 0 : 1;
  const int hi = seg_offsets[j + 1];
  const int n = (hi - 1) / SEG_ROWS - c + 1;           // pieces: this chunk's, then slot 0 of the following chunks
  const int q = (n + 3) >> 2;
  const int p0 = wave * q, p1 = min(n, p0 + q);
  float acc[COLS];
#pragma unroll
  for (int x = 0; x < COLS; ++x) acc[x] = 0.f;
  if (live) {
    constexpr int UNR = 16;
    for (int pb = p0; pb < p1; pb += UNR) {
      float data[UNR][COLS];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        if (pb + u < p1) {
          const int pc = pb + u;
          const float* src = part + ((int64_t)(c + pc) * 2 + (pc == 0 ? slot : 0)) * F + col;
#pragma unroll
          for (int x = 0; x < COLS; x += 4) {
            const float4 v = *reinterpret_cast<const float4*>(src + x);
            data[u][x] = v.x; data[u][x + 1] = v.y; data[u][x + 2] = v.z; data[u][x + 3] = v.w;
          }
        }
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u)
        if (pb + u < p1)
#pragma unroll
          for (int x = 0; x < COLS; ++x) acc[x] += data[u][x];
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int x = 0; x < COLS; ++x) red[wave - 1][lane][x] = acc[x];
  }
  __syncthreads();
  if (wave == 0 && live) {
    for (int w = 1; w < 4; ++w)
      if (w * q < n)
#pragma unroll
        for (int x = 0; x < COLS; ++x) acc[x] += red[w - 1][lane][x];
    store_cols<COLS>(dE_rows + (int64_t)j * F + col, acc);
  }
}

int bits_for(int V) {
  int b = 1;
  while (b < 31 && (1ll << b) < (long long)V) ++b;
  return b;
}

}  // namespace

int64_t stem_seg_chunks(int64_t max_tokens) { return (max_tokens + SEG_ROWS - 1) / SEG_ROWS; }
int64_t stem_sort_count_entries(int64_t max_tokens) {
  const int64_t tiles = (max_tokens + SORT_TILE - 1) / SORT_TILE;
  return tiles * SORT_WAVES * RADIX;
}

hipError_t stem_sort_unique(stem_ctx* ctx, const EmbedScratch& ws, const int32_t* ids, int64_t T, int V,
                            int32_t* sorted_ids, int32_t* perm, int32_t* uniq_ids, int32_t* seg_offsets,
                            int32_t* n_uniq, hipStream_t s) {
  const int passes = (bits_for(V) + RADIX_BITS - 1) / RADIX_BITS;
  const int pos_bits = bits_for((int)T);
  if (T <= FUSED_MAX_T && bits_for(V) + pos_bits <= 32) {
    ProfScope ps(ctx, K_SORT_FUSED, s);
    hipLaunchKernelGGL(sort_unique_fused_kernel, dim3(1), dim3(1024), 0, s, ids, (int)T, V, pos_bits, passes,
                       sorted_ids, perm, uniq_ids, seg_offsets, n_uniq, ws.seg_of, ws.flag);
    return hipGetLastError();
  }
  const int tiles = (int)((T + SORT_TILE - 1) / SORT_TILE);
  const int nW = tiles * SORT_WAVES;
  const int32_t* src_k = ids;
  const int32_t* src_v = nullptr;
  for (int p = 0; p < passes; ++p) {
    int32_t* dst_k = (p == passes - 1) ? sorted_ids : ws.sort_keys[p & 1];
    int32_t* dst_v = (p == passes - 1) ? perm : ws.sort_vals[p & 1];
    const int shift = p * RADIX_BITS;
    {
      ProfScope ps(ctx, K_SORT_COUNT, s);
      hipLaunchKernelGGL(sort_count_kernel, dim3(tiles), dim3(1024), 0, s, src_k, T, V, shift, p == 0, nW,
                         ws.sort_counts, ws.flag);
    }
    {
      ProfScope ps(ctx, K_SORT_SCAN, s);
      hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, ws.sort_counts, nW * RADIX);
    }
    {
      ProfScope ps(ctx, K_SORT_SCATTER, s);
      hipLaunchKernelGGL(sort_scatter_kernel, dim3(tiles), dim3(1024), 0, s, src_k, src_v, T, V, shift, p == 0,
                         nW, ws.sort_counts, dst_k, dst_v, ws.flag);
    }
    src_k = dst_k;
    src_v = dst_v;
  }
  {
    ProfScope ps(ctx, K_UNIQUE, s);
    hipLaunchKernelGGL(unique_kernel, dim3(1), dim3(1024), 0, s, sorted_ids, T, uniq_ids, seg_offsets, n_uniq,
                       ws.seg_of);
  }
  return hipGetLastError();
}

hipError_t stem_seg_reduce(stem_ctx* ctx, const EmbedScratch& ws, int is_bf16, const void* dU, const int32_t* perm,
                           const int32_t* seg_offsets, int64_t T, int F, float* dE_rows, hipStream_t s) {
  const int chunks = (int)((T + SEG_ROWS - 1) / SEG_ROWS);
  const int cols = is_bf16 ? 8 : 4;
  const int slabs = (F + 256 * cols - 1) / (256 * cols);
  {
    ProfScope ps(ctx, K_SEG_REDUCE, s);
    if (is_bf16)
      hipLaunchKernelGGL(seg_reduce_kernel<true>, dim3(slabs, chunks), dim3(256), 0, s, dU, perm, ws.seg_of, T, F,
                         dE_rows, ws.seg_part);
    else
      hipLaunchKernelGGL(seg_reduce_kernel<false>, dim3(slabs, chunks), dim3(256), 0, s, dU, perm, ws.seg_of, T,
                         F, dE_rows, ws.seg_part);
  }
  {
    ProfScope ps(ctx, K_SEG_COMBINE, s);
    if (is_bf16)
      hipLaunchKernelGGL(seg_combine_kernel<8>, dim3(chunks, (F + 511) / 512), dim3(256), 0, s, ws.seg_of, seg_offsets, T,
                         F, dE_rows, ws.seg_part);
    else
      hipLaunchKernelGGL(seg_combine_kernel<4>, dim3(chunks, (F + 255) / 256), dim3(256), 0, s, ws.seg_of, seg_offsets, T,
                         F, dE_rows, ws.seg_part);
  }
  return hipGetLastError();
}
