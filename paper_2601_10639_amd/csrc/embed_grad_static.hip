// stem_embed_grad_noalloc: the table-gradient call for callers that cannot allocate.
//
// Same kernels as stem_embed_grad (embed_grad.hip); what differs is where their scratch lives.
// stem_embed_grad uses buffers that stem_create allocated; here the scratch is one file-scope
// device array that exists from the moment the library is loaded, so the call needs neither a
// context nor any allocation.  Each GPU has its own copy of the array at its own address: the
// address is looked up once per device (hipGetSymbolAddress, with that device current) and kept;
// host code never uses the array's name as a pointer.
#include <mutex>

#include "stem_internal.h"

namespace {

constexpr int64_t MAX_T = STEM_NOALLOC_MAX_TOKENS;
constexpr size_t FLAG_BYTES = 256;
constexpr size_t INT_ARRAY_BYTES = (size_t)MAX_T * 4;                   // one [MAX_T] int32 array
constexpr size_t COUNT_BYTES = (size_t)(MAX_T / 4096) * 16 * 64 * 4;    // sort digit counts
constexpr size_t PART_BYTES = STEM_NOALLOC_PART_BYTES;                  // partial sums of border-crossing runs
constexpr size_t OFF_FLAG = 0;
constexpr size_t OFF_SEG_OF = OFF_FLAG + FLAG_BYTES;
constexpr size_t OFF_KEYS0 = OFF_SEG_OF + INT_ARRAY_BYTES;
constexpr size_t OFF_KEYS1 = OFF_KEYS0 + INT_ARRAY_BYTES;
constexpr size_t OFF_VALS0 = OFF_KEYS1 + INT_ARRAY_BYTES;
constexpr size_t OFF_VALS1 = OFF_VALS0 + INT_ARRAY_BYTES;
constexpr size_t OFF_COUNTS = OFF_VALS1 + INT_ARRAY_BYTES;
constexpr size_t OFF_PART = OFF_COUNTS + COUNT_BYTES;
constexpr size_t SCRATCH_BYTES = OFF_PART + PART_BYTES;
static_assert(OFF_PART % 256 == 0, "every piece of the scratch array stays 256-byte aligned");

// The scratch itself.  In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
unsigned char* g_ptr[MAX_DEVICES];   // device address of `scratch` on each GPU, once looked up

// Address of this device's copy of the scratch array (the device must be current).
hipError_t scratch_of(int device, unsigned char** out) {
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_ptr[device] = static_cast<unsigned char*>(p);
  }
  *out = g_ptr[device];
  return hipSuccess;
}

}  // namespace

extern "C" stem_status stem_embed_grad_noalloc(int32_t dtype, int32_t vocab, int32_t d_ff, const int32_t* ids,
                                               const void* dU, int64_t T, int32_t* sorted_ids, int32_t* perm,
                                               int32_t* uniq_ids, int32_t* seg_offsets, int32_t* n_uniq,
                                               float* dE_rows, int32_t* id_flag, void* stream) {
  if (dtype != STEM_F32 && dtype != STEM_BF16)
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_embed_grad_noalloc: dtype %d is not a stem_dtype", dtype);
  const int mult = dtype == STEM_BF16 ? 8 : 4;   // elements per 16-byte access
  if (vocab <= 0 || d_ff <= 0 || d_ff % mult)
    return stem_fail(nullptr, STEM_ERR_SHAPE, "stem_embed_grad_noalloc: vocab = %d, d_ff = %d (d_ff must be a multiple of %d)",
                     vocab, d_ff, mult);
  if (T < 0 || T > MAX_T)
    return stem_fail(nullptr, STEM_ERR_SHAPE, "stem_embed_grad_noalloc: T = %lld is outside [0, %lld], the most the static scratch holds",
                     (long long)T, (long long)MAX_T);
  if (!seg_offsets || !n_uniq)
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_embed_grad_noalloc: null seg_offsets / n_uniq");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (T == 0) {
    if ((e = stem_fill_zero(n_uniq, 4, s)) != hipSuccess || (e = stem_fill_zero(seg_offsets, 4, s)) != hipSuccess)
      return stem_fail(nullptr, STEM_ERR_HIP, "stem_embed_grad_noalloc: %s", hipGetErrorString(e));
    return STEM_OK;
  }
  if (!ids || !sorted_ids || !perm || !uniq_ids)
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_embed_grad_noalloc: null pointer argument");
  if ((dU == nullptr) != (dE_rows == nullptr))
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_embed_grad_noalloc: dU and dE_rows must both be given or both be NULL");
  if ((reinterpret_cast<uintptr_t>(dU) & 15u) || (reinterpret_cast<uintptr_t>(dE_rows) & 15u))
    return stem_fail(nullptr, STEM_ERR_INVALID_ARG, "stem_embed_grad_noalloc: dU and dE_rows must be 16-byte aligned");
  const size_t part_bytes = (size_t)stem_seg_chunks(T) * 2 * (size_t)d_ff * 4;
  if (dU && part_bytes > PART_BYTES)
    return stem_fail(nullptr, STEM_ERR_SHAPE,
                     "stem_embed_grad_noalloc: T = %lld with d_ff = %d needs %zu bytes of partial sums, the static scratch holds %zu "
                     "(T * d_ff <= %lld)", (long long)T, d_ff, part_bytes, PART_BYTES, (long long)(PART_BYTES / 8 * 32));
  int device = -1;
  if ((e = hipGetDevice(&device)) != hipSuccess || device < 0 || device >= MAX_DEVICES)
    return stem_fail(nullptr, STEM_ERR_HIP, "stem_embed_grad_noalloc: hipGetDevice: %s (device %d)", hipGetErrorString(e), device);
  unsigned char* base = nullptr;
  if ((e = scratch_of(device, &base)) != hipSuccess)
    return stem_fail(nullptr, STEM_ERR_HIP, "stem_embed_grad_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));

  EmbedScratch ws;
  ws.seg_of = reinterpret_cast<int32_t*>(base + OFF_SEG_OF);
  ws.sort_keys[0] = reinterpret_cast<int32_t*>(base + OFF_KEYS0);
  ws.sort_keys[1] = reinterpret_cast<int32_t*>(base + OFF_KEYS1);
  ws.sort_vals[0] = reinterpret_cast<int32_t*>(base + OFF_VALS0);
  ws.sort_vals[1] = reinterpret_cast<int32_t*>(base + OFF_VALS1);
  ws.sort_counts = reinterpret_cast<int32_t*>(base + OFF_COUNTS);
  ws.seg_part = reinterpret_cast<float*>(base + OFF_PART);
  // Without a caller-provided flag word the kernels still need somewhere to report a bad id: a word of
  // the scratch, whose previous content does not matter (it is only ever set to 1 and never read here).
  ws.flag = id_flag ? id_flag : reinterpret_cast<int32_t*>(base + OFF_FLAG);
  // Nothing else of the scratch has to start at zero: every word the kernels read was written earlier
  // in the same call (digit counts by the counting pass, run indices by the sort, partial sums by the
  // chunk that owns them), so what the previous call left behind is never seen.
  if ((e = stem_sort_unique(nullptr, ws, ids, T, vocab, sorted_ids, perm, uniq_ids, seg_offsets, n_uniq, s)) != hipSuccess)
    return stem_fail(nullptr, STEM_ERR_HIP, "stem_embed_grad_noalloc: sort launch: %s", hipGetErrorString(e));
  if (dU && (e = stem_seg_reduce(nullptr, ws, dtype == STEM_BF16, dU, perm, seg_offsets, T, d_ff, dE_rows, s)) != hipSuccess)
    return stem_fail(nullptr, STEM_ERR_HIP, "stem_embed_grad_noalloc: reduce launch: %s", hipGetErrorString(e));
  return STEM_OK;
}
