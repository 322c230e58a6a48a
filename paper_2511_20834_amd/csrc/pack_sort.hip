// Coordinate packing (Section 5.3), the one-time sort (Section 5.2) and the
// packed-native downsampling of a stride level (Eq. 1 via mask, sort, unique).
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "spc_internal.h"

namespace spc {

// ---------------------------------------------------------------- sort wrappers
// The library sort used outside the size range of the library's own sort enqueues more than kernels
// (its single-pass form clears its digit counters and look-back states with hipMemsetAsync), and such
// nodes in a captured graph have given wrong results on replays: a stale look-back state sends keys
// to positions outside the arrays.  Under stream capture these sizes are refused.
static int refuse_if_capturing(hipStream_t s, int64_t n) {
  if (!stream_is_capturing(s)) return SPC_OK;
  return set_error(SPC_ERR_UNSUPPORTED,
                   "%lld keys are sorted by the library sort, which cannot be recorded into a graph; "
                   "capture is supported up to %lld keys",
                   static_cast<long long>(n), static_cast<long long>(BS_MAX_N));
}

template <typename KeyT>
static int sort_pairs_t(const void* ki, void* ko, const int32_t* vi, int32_t* vo, int64_t n, int end_bit, void* temp,
                        size_t& temp_bytes, hipStream_t s) {
  hipError_t e = rocprim::radix_sort_pairs(temp, temp_bytes, static_cast<const KeyT*>(ki), static_cast<KeyT*>(ko), vi, vo,
                                           static_cast<size_t>(n), 0u, static_cast<unsigned>(end_bit), s);
  if (e != hipSuccess) return set_error(SPC_ERR_HIP, "radix_sort_pairs: %s", hipGetErrorString(e));
  return SPC_OK;
}
template <typename KeyT>
static int sort_keys_t(const void* ki, void* ko, int64_t n, int end_bit, void* temp, size_t& temp_bytes, hipStream_t s) {
  hipError_t e = rocprim::radix_sort_keys(temp, temp_bytes, static_cast<const KeyT*>(ki), static_cast<KeyT*>(ko),
                                          static_cast<size_t>(n), 0u, static_cast<unsigned>(end_bit), s);
  if (e != hipSuccess) return set_error(SPC_ERR_HIP, "radix_sort_keys: %s", hipGetErrorString(e));
  return SPC_OK;
}

size_t sort_pairs_temp_bytes(int key_bits, int64_t n) {
  size_t b = 0;
  if (key_bits == 32) sort_pairs_t<uint32_t>(nullptr, nullptr, nullptr, nullptr, n, 32, nullptr, b, nullptr);
  else sort_pairs_t<uint64_t>(nullptr, nullptr, nullptr, nullptr, n, 64, nullptr, b, nullptr);
  return b;
}
int sort_pairs(int key_bits, const void* ki, void* ko, const int32_t* vi, int32_t* vo, int64_t n, int end_bit, void* temp,
               size_t temp_bytes, hipStream_t s) {
  return key_bits == 32 ? sort_pairs_t<uint32_t>(ki, ko, vi, vo, n, end_bit, temp, temp_bytes, s)
                        : sort_pairs_t<uint64_t>(ki, ko, vi, vo, n, end_bit, temp, temp_bytes, s);
}
size_t sort_keys_temp_bytes(int key_bits, int64_t n) {
  size_t b = 0;
  if (key_bits == 32) sort_keys_t<uint32_t>(nullptr, nullptr, n, 32, nullptr, b, nullptr);
  else sort_keys_t<uint64_t>(nullptr, nullptr, n, 64, nullptr, b, nullptr);
  return b;
}
int sort_keys(int key_bits, const void* ki, void* ko, int64_t n, int end_bit, void* temp, size_t temp_bytes, hipStream_t s) {
  return key_bits == 32 ? sort_keys_t<uint32_t>(ki, ko, n, end_bit, temp, temp_bytes, s)
                        : sort_keys_t<uint64_t>(ki, ko, n, end_bit, temp, temp_bytes, s);
}

// ---------------------------------------------------------------- kernels
// One thread per voxel: 16-byte coalesced load of (b,x,y,z), one key store.
template <typename KeyT>
__global__ __launch_bounds__(256) void pack_kernel(const int4* __restrict__ coords, int64_t n, PackParams p,
                                                   KeyT* __restrict__ keys, int32_t* __restrict__ iota,
                                                   int32_t* __restrict__ status) {
  const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (i >= n) return;
  keys[i] = pack_key<KeyT>(coords[i], p, status);
  if (iota) iota[i] = static_cast<int32_t>(i);
}

template <typename KeyT>
__global__ __launch_bounds__(256) void dup_check_kernel(const KeyT* __restrict__ keys, int64_t n, int32_t* __restrict__ status) {
  const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (i + 1 < n && keys[i] == keys[i + 1] && keys[i] != ~KeyT(0)) atomicOr(status, 2);
}

__global__ void set_int_kernel(int32_t* p, int32_t v) { *p = v; }

template <typename KeyT>
__global__ __launch_bounds__(256) void mask_kernel(const KeyT* __restrict__ in, int64_t n, KeyT mask, KeyT* __restrict__ out) {
  const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (i < n) out[i] = in[i] & mask;
}

// Order-preserving removal of repeated keys from a sorted array, in three launches:
// heads per block, exclusive scan of the block counts, compacting write.
constexpr int UQ_THREADS = 256;
constexpr int UQ_ITEMS = 8;
constexpr int UQ_BLOCK = UQ_THREADS * UQ_ITEMS;

template <typename KeyT>
__device__ inline bool is_head(const KeyT* keys, int64_t i) { return i == 0 || keys[i] != keys[i - 1]; }

__device__ inline int block_exclusive_scan(int v, int* total) {
  // 256 threads = 4 waves; wave scan by shuffles, then the 4 wave totals through LDS.
  __shared__ int wave_sum[UQ_THREADS / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int x = v;
  for (int d = 1; d < 64; d <<= 1) {
    int y = __shfl_up(x, d, 64);
    if (lane >= d) x += y;
  }
  if (lane == 63) wave_sum[wave] = x;
  __syncthreads();
  int base = 0, tot = 0;
  for (int w = 0; w < UQ_THREADS / 64; ++w) {
    int s = wave_sum[w];
    if (w < wave) base += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return base + x - v;
}

template <typename KeyT>
__global__ __launch_bounds__(UQ_THREADS) void unique_count_kernel(const KeyT* __restrict__ keys, int64_t n,
                                                                  int32_t* __restrict__ block_counts) {
  const int64_t base = int64_t(blockIdx.x) * UQ_BLOCK;
  int c = 0;
  for (int it = 0; it < UQ_ITEMS; ++it) {
    const int64_t i = base + it * UQ_THREADS + threadIdx.x;
    if (i < n && is_head(keys, i)) ++c;
  }
  int total;
  block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

// Single workgroup: exclusive scan of n_blocks counts in place; the grand total goes to *n_out.
__global__ __launch_bounds__(UQ_THREADS) void scan_counts_kernel(int32_t* __restrict__ counts, int n_blocks,
                                                                 int32_t* __restrict__ n_out) {
  int carry = 0;
  for (int b0 = 0; b0 < n_blocks; b0 += UQ_THREADS) {
    const int i = b0 + threadIdx.x;
    const int v = i < n_blocks ? counts[i] : 0;
    int total;
    const int ex = block_exclusive_scan(v, &total);
    if (i < n_blocks) counts[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) *n_out = carry;
}

template <typename KeyT>
__global__ __launch_bounds__(UQ_THREADS) void unique_write_kernel(const KeyT* __restrict__ keys, int64_t n,
                                                                  const int32_t* __restrict__ block_base,
                                                                  KeyT* __restrict__ out) {
  const int64_t base = int64_t(blockIdx.x) * UQ_BLOCK;
  int run = block_base[blockIdx.x];
  for (int it = 0; it < UQ_ITEMS; ++it) {  // items are visited in array order, so ranks stay ordered
    const int64_t i = base + it * UQ_THREADS + threadIdx.x;
    const bool head = i < n && is_head(keys, i);
    int total;
    const int ex = block_exclusive_scan(head ? 1 : 0, &total);
    if (head) out[run + ex] = keys[i];
    run += total;
  }
}

template <typename KeyT>
static int downsample_t(const void* src, int64_t n, const PackInfo& pi, int m, Level* lv, hipStream_t s) {
  if (use_bucket_sort(n)) {
    char* scratch = static_cast<char*>(pool_alloc(bucket_sort_ws_bytes(pi.key_bits, n), s));
    if (!scratch) return SPC_ERR_NOMEM;
    const int rc = bucket_mask_unique(pi.key_bits, src, n, level_mask(pi, m), pi.used_bits, lv->keys, lv->n_dev, scratch, s);
    pool_free(scratch, s);  // reuse is ordered behind these kernels on this stream
    return rc;
  }
  if (n > 0 && n < BS_MIN_N) return small_mask_unique(pi.key_bits, src, n, level_mask(pi, m), pi.used_bits, lv->keys, lv->n_dev, s);
  if (n > 0) SPC_RETURN_IF(refuse_if_capturing(s, n));
  const size_t ksz = sizeof(KeyT);
  const size_t tb = sort_keys_temp_bytes(pi.key_bits, n);
  const int n_blocks = static_cast<int>((n + UQ_BLOCK - 1) / UQ_BLOCK);
  // scratch: masked keys | sorted keys | block counts | sort temp
  const size_t off_sorted = (n * ksz + 255) / 256 * 256;
  const size_t off_counts = off_sorted * 2;
  const size_t off_temp = off_counts + (size_t(n_blocks) * 4 + 255) / 256 * 256;
  char* scratch = static_cast<char*>(pool_alloc(off_temp + tb + 256, s));
  if (!scratch) return SPC_ERR_NOMEM;
  KeyT* masked = reinterpret_cast<KeyT*>(scratch);
  KeyT* sorted = reinterpret_cast<KeyT*>(scratch + off_sorted);
  int32_t* counts = reinterpret_cast<int32_t*>(scratch + off_counts);
  const KeyT mask = static_cast<KeyT>(level_mask(pi, m));
  const int grid = static_cast<int>((n + 255) / 256);
  int rc = SPC_OK;
  if (n > 0) {
    hipLaunchKernelGGL(mask_kernel<KeyT>, dim3(grid), dim3(256), 0, s, static_cast<const KeyT*>(src), n, mask, masked);
    rc = sort_keys(pi.key_bits, masked, sorted, n, pi.used_bits, scratch + off_temp, tb, s);
    if (rc == SPC_OK) {
      hipLaunchKernelGGL(unique_count_kernel<KeyT>, dim3(n_blocks), dim3(UQ_THREADS), 0, s, sorted, n, counts);
      hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(UQ_THREADS), 0, s, counts, n_blocks, lv->n_dev);
      hipLaunchKernelGGL(unique_write_kernel<KeyT>, dim3(n_blocks), dim3(UQ_THREADS), 0, s, sorted, n, counts,
                         static_cast<KeyT*>(lv->keys));
    }
  } else {
    hipLaunchKernelGGL(set_int_kernel, dim3(1), dim3(1), 0, s, lv->n_dev, 0);
  }
  // The scratch block returns to the cache now; reuse is ordered behind these kernels
  // as long as later library calls are ordered after this stream's work.
  pool_free(scratch, s);
  if (rc == SPC_OK && hipGetLastError() != hipSuccess) rc = set_error(SPC_ERR_HIP, "downsample launch failed");
  return rc;
}

int downsample_level(const void* src_keys, int64_t n_src, const int* /*n_src_dev*/, const PackInfo& pi, int m, Level** out,
                     hipStream_t stream) {
  Level* lv = new Level;
  lv->cap = n_src;
  lv->stride = 1 << m;
  lv->owns_keys = true;
  lv->stream = stream;
  lv->captured = stream_is_capturing(stream);
  lv->keys = pool_alloc(std::max<size_t>(size_t(n_src) * (pi.key_bits / 8), 256), stream);
  lv->n_dev = static_cast<int*>(pool_alloc(256, stream));
  if (!lv->keys || !lv->n_dev) {
    level_unref(lv);
    return SPC_ERR_NOMEM;
  }
  int rc = pi.key_bits == 32 ? downsample_t<uint32_t>(src_keys, n_src, pi, m, lv, stream)
                             : downsample_t<uint64_t>(src_keys, n_src, pi, m, lv, stream);
  if (rc == SPC_OK) {
    if (hipEventCreateWithFlags(&lv->ready, hipEventDisableTiming) != hipSuccess ||
        hipEventRecord(lv->ready, stream) != hipSuccess)
      rc = set_error(SPC_ERR_HIP, "event record failed");
  }
  if (rc != SPC_OK) {
    level_unref(lv);
    return rc;
  }
  *out = lv;
  return SPC_OK;
}

}  // namespace spc

// ---------------------------------------------------------------- C ABI
// Device memory of spc_pack_coords_noalloc: the sort's scratch (partitioned keys and indices, bin
// tables, rank windows, status word) for up to SPC_NOALLOC_MAX_N voxels with 64-bit keys.  Part of the
// code object: every GPU the library runs on holds its own copy until the process ends.  Host code never
// passes the array's name to a kernel: it is a host-side stand-in; the device address comes from
// hipGetSymbolAddress, once per device.
constexpr size_t NOALLOC_SCRATCH_BYTES = size_t(13) << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace spc {
namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
int noalloc_scratch(void** out) {
  int dev = 0;
  SPC_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return set_error(SPC_ERR_UNSUPPORTED, "device index %d beyond %d", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return set_error(SPC_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SPC_OK;
}
}  // namespace
}  // namespace spc

extern "C" int spc_pack_coords_noalloc(const int32_t* coords, int64_t n, const spc_pack_desc* d, void* keys_out,
                                       int32_t* perm_out, int32_t flags, void* stream) {
  using namespace spc;
  PackInfo pi;
  SPC_RETURN_IF(check_desc(d, &pi));
  if (n < 1 || n > SPC_NOALLOC_MAX_N)
    return set_error(SPC_ERR_UNSUPPORTED, "spc_pack_coords_noalloc takes 1..%lld voxels, got %lld",
                     static_cast<long long>(SPC_NOALLOC_MAX_N), static_cast<long long>(n));
  size_t need = 0;
  SPC_RETURN_IF(spc_pack_coords(nullptr, n, d, nullptr, nullptr, nullptr, &need, flags, nullptr));
  if (need > NOALLOC_SCRATCH_BYTES)
    return set_error(SPC_ERR_UNSUPPORTED, "%lld voxels need %zu bytes of scratch, the static buffer holds %zu",
                     static_cast<long long>(n), need, NOALLOC_SCRATCH_BYTES);
  void* ws = nullptr;
  SPC_RETURN_IF(noalloc_scratch(&ws));
  size_t have = NOALLOC_SCRATCH_BYTES;
  // every part of the scratch that is read is written first by the kernels of the same call (the
  // status word by a one-thread kernel), so nothing of the previous call's contents matters
  return spc_pack_coords(coords, n, d, keys_out, perm_out, ws, &have, flags, stream);
}

extern "C" int spc_pack_coords(const int32_t* coords, int64_t n, const spc_pack_desc* d, void* keys_out, int32_t* perm_out,
                               void* workspace, size_t* workspace_bytes, int32_t flags, void* stream) {
  using namespace spc;
  PackInfo pi;
  SPC_RETURN_IF(check_desc(d, &pi));
  if (n < 0 || n > 0x7fffffff) return set_error(SPC_ERR_ARG, "n out of range");
  if (!workspace_bytes) return set_error(SPC_ERR_ARG, "workspace_bytes is NULL");
  const size_t ksz = pi.key_bits / 8;
  const size_t nn = static_cast<size_t>(std::max<int64_t>(n, 1));
  const size_t off_iota = (nn * ksz + 255) / 256 * 256;
  const size_t off_status = off_iota + (nn * 4 + 255) / 256 * 256;
  const size_t off_temp = off_status + 256;
  const bool bucket = use_bucket_sort(n);
  const size_t tb = bucket ? bucket_sort_ws_bytes(pi.key_bits, nn)
                           : std::max(sort_pairs_temp_bytes(pi.key_bits, nn), sort_keys_temp_bytes(pi.key_bits, nn));
  const size_t need = off_temp + tb + 256;
  if (!workspace) {
    *workspace_bytes = need;
    return SPC_OK;
  }
  if (*workspace_bytes < need) return set_error(SPC_ERR_ARG, "workspace too small: %zu < %zu", *workspace_bytes, need);
  if (!coords || !keys_out) return set_error(SPC_ERR_ARG, "NULL coords or keys_out");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool small = n > 0 && n < BS_MIN_N;
  if (!bucket && !small && n > 0) SPC_RETURN_IF(refuse_if_capturing(s, n));
  char* ws = static_cast<char*>(workspace);
  void* keys_tmp = ws;
  int32_t* iota = reinterpret_cast<int32_t*>(ws + off_iota);
  // the status word is only kept when somebody is going to read it
  int32_t* status = (flags & SPC_PACK_VALIDATE) ? reinterpret_cast<int32_t*>(ws + off_status) : nullptr;
  PackParams p{pi.sh_b, pi.sh_x, pi.sh_y, pi.bits_b, pi.bits_x, pi.bits_y, pi.bits_z, d->origin[0], d->origin[1], d->origin[2], d->pad};
  if (status) hipLaunchKernelGGL(set_int_kernel, dim3(1), dim3(1), 0, s, status, 0);
  if (bucket) {
    SPC_RETURN_IF(bucket_pack_sort(pi.key_bits, reinterpret_cast<const int4*>(coords), n, p, pi.used_bits, status, keys_out, perm_out,
                                   ws + off_temp, s));
    if (flags & SPC_PACK_VALIDATE) {
      const int grid = static_cast<int>((n + 255) / 256);
      if (pi.key_bits == 32)
        hipLaunchKernelGGL(dup_check_kernel<uint32_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint32_t*>(keys_out), n, status);
      else
        hipLaunchKernelGGL(dup_check_kernel<uint64_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint64_t*>(keys_out), n, status);
    }
  } else if (small) {
    SPC_RETURN_IF(small_pack_sort(pi.key_bits, reinterpret_cast<const int4*>(coords), n, p, pi.used_bits, status, keys_out, perm_out, s));
    if (flags & SPC_PACK_VALIDATE) {
      const int grid = static_cast<int>((n + 255) / 256);
      if (pi.key_bits == 32)
        hipLaunchKernelGGL(dup_check_kernel<uint32_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint32_t*>(keys_out), n, status);
      else
        hipLaunchKernelGGL(dup_check_kernel<uint64_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint64_t*>(keys_out), n, status);
    }
  } else if (n > 0) {
    const int grid = static_cast<int>((n + 255) / 256);
    if (pi.key_bits == 32)
      hipLaunchKernelGGL(pack_kernel<uint32_t>, dim3(grid), dim3(256), 0, s, reinterpret_cast<const int4*>(coords), n, p,
                         static_cast<uint32_t*>(keys_tmp), perm_out ? iota : nullptr, status);
    else
      hipLaunchKernelGGL(pack_kernel<uint64_t>, dim3(grid), dim3(256), 0, s, reinterpret_cast<const int4*>(coords), n, p,
                         static_cast<uint64_t*>(keys_tmp), perm_out ? iota : nullptr, status);
    // all-ones keys of rejected rows must keep their place at the end: sort every key bit then
    const int end_bit = (flags & SPC_PACK_VALIDATE) ? pi.key_bits : pi.used_bits;
    if (perm_out) SPC_RETURN_IF(sort_pairs(pi.key_bits, keys_tmp, keys_out, iota, perm_out, n, end_bit, ws + off_temp, tb, s));
    else SPC_RETURN_IF(sort_keys(pi.key_bits, keys_tmp, keys_out, n, end_bit, ws + off_temp, tb, s));
    if (flags & SPC_PACK_VALIDATE) {
      if (pi.key_bits == 32)
        hipLaunchKernelGGL(dup_check_kernel<uint32_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint32_t*>(keys_out), n, status);
      else
        hipLaunchKernelGGL(dup_check_kernel<uint64_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint64_t*>(keys_out), n, status);
    }
  }
  SPC_HIP_CHECK(hipGetLastError());
  if (flags & SPC_PACK_VALIDATE) {
    int32_t st = 0;
    SPC_HIP_CHECK(hipMemcpyAsync(&st, status, sizeof(st), hipMemcpyDeviceToHost, s));
    SPC_HIP_CHECK(hipStreamSynchronize(s));
    if (st & 1) return set_error(SPC_ERR_RANGE, "a coordinate does not fit its packed field (guard band included)");
    if (st & 2) return set_error(SPC_ERR_DUP, "duplicate voxel coordinates");
  }
  return SPC_OK;
}
