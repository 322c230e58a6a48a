// Internal declarations shared by the translation units of libspc (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>
#include <vector>

#include "spc.h"

namespace spc {

// ---------------------------------------------------------------- errors
int set_error(int code, const char* fmt, ...);
#define SPC_HIP_CHECK(expr)                                                                       \
  do {                                                                                            \
    hipError_t e__ = (expr);                                                                      \
    if (e__ != hipSuccess)                                                                        \
      return ::spc::set_error(SPC_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), \
                              __FILE__, __LINE__);                                                \
  } while (0)
#define SPC_RETURN_IF(expr)     \
  do {                          \
    int rc__ = (expr);          \
    if (rc__ != SPC_OK) return rc__; \
  } while (0)

// ---------------------------------------------------------------- device block cache
// hipMalloc costs tens of microseconds and synchronises; kernel maps are built per
// frame, so freed blocks are kept and handed out again — only to work on the stream
// that last used them, which makes stream order the only synchronisation needed.
void* pool_alloc(size_t bytes, hipStream_t stream);  // nullptr on failure (error set)
void pool_free(void* p, hipStream_t stream);
int pool_release_all();
// Makes everything enqueued on `waiter` from now on run after what `producer` holds at this moment
// (an event recorded on `producer`; nothing happens when the two are the same stream).  Used before a
// block goes back to the cache of a stream other than the one whose kernels last read it.
void order_stream_after(hipStream_t waiter, hipStream_t producer);

// ---------------------------------------------------------------- packing
struct PackInfo {
  int key_bits;
  int sh_b, sh_x, sh_y;  // left shifts of the batch/x/y fields (z has shift 0)
  int bits_b, bits_x, bits_y, bits_z;
  int used_bits;
};
int check_desc(const spc_pack_desc* d, PackInfo* pi);
// Mask that clears the low m bits of every spatial field (Section 5.3).
uint64_t level_mask(const PackInfo& pi, int m);

// ---------------------------------------------------------------- offset subsets
// Subset of the K^3 weight offsets (bit k of word k/32): all of them for a single dataflow, the dense or the
// sparse ones of the hybrid dual dataflow (Section 5.4).
constexpr int KMASK_WORDS = 11;  // 7^3 = 343 bits
struct KMask {
  uint32_t w[KMASK_WORDS];
#ifdef __HIPCC__
  __host__ __device__
#endif
  bool has(int k) const { return (w[k >> 5] >> (k & 31)) & 1u; }
};
// L1 norm of weight offset k in units of the input stride (Section 5.4: offsets below the threshold are the
// dense ones).  Even kernel sizes have offsets {0, 1} per axis.
inline int offset_l1(int K, int k) {
  const int iz = k % K, iy = (k / K) % K, ix = k / (K * K);
  if (K % 2 == 0) return ix + iy + iz;
  const int c = (K - 1) / 2;
  return (ix > c ? ix - c : c - ix) + (iy > c ? iy - c : c - iy) + (iz > c ? iz - c : c - iz);
}

// ---------------------------------------------------------------- coordinate levels
// One sorted packed-key array (a stride level).  n is known on the host for the
// caller's own array; for derived levels it lives on the device until the host asks.
struct Level {
  std::atomic<int> refs{1};
  void* keys = nullptr;   // device
  bool owns_keys = false;
  int64_t cap = 0;        // rows allocated / upper bound of n
  int64_t n_host = -1;    // -1: not yet fetched
  int64_t n_fetched = -1; // last value read back from n_dev (equals n_host unless the level was built under capture)
  bool captured = false;  // produced while its stream was being captured into a graph: every replay rewrites it
  int* n_dev = nullptr;   // device int (nullptr when n_host is authoritative from the start)
  int stride = 1;
  hipEvent_t ready = nullptr;  // recorded after the level's last kernel
  hipStream_t stream = nullptr;  // stream the level was produced on
  std::vector<hipStream_t> readers;  // other streams whose kernels read the keys (map searches)
  void add_reader(hipStream_t s) {
    if (s == stream) return;
    for (hipStream_t r : readers)
      if (r == s) return;
    readers.push_back(s);
  }
};
void level_unref(Level* l);
bool stream_is_capturing(hipStream_t s);

// Derive the level with stride 2^m of `src_keys` (mask, sort, unique).  Enqueues only.
int downsample_level(const void* src_keys, int64_t n_src, const int* n_src_dev, const PackInfo& pi, int m,
                     Level** out, hipStream_t stream);

// ---------------------------------------------------------------- packing (Section 5.3)
struct PackParams {
  int sh_b, sh_x, sh_y;
  int bits_b, bits_x, bits_y, bits_z;
  int ox, oy, oz, pad;
};

#ifdef __HIPCC__
// Key of one (b,x,y,z) row.  A field that does not fit (guard band on both sides included)
// gives the all-ones key and sets `bad`.
template <typename KeyT>
__device__ inline KeyT pack_key_flag(const int4 c, const PackParams& p, bool& bad) {
  const int64_t fx = int64_t(c.y) - p.ox, fy = int64_t(c.z) - p.oy, fz = int64_t(c.w) - p.oz;
  const bool ok = c.x >= 0 && (int64_t(c.x) < (int64_t(1) << p.bits_b)) && fx >= 0 && fy >= 0 && fz >= 0 &&
                  fx + 2 * int64_t(p.pad) < (int64_t(1) << p.bits_x) && fy + 2 * int64_t(p.pad) < (int64_t(1) << p.bits_y) &&
                  fz + 2 * int64_t(p.pad) < (int64_t(1) << p.bits_z);
  bad |= !ok;
  return ok ? (KeyT(c.x) << p.sh_b) | (KeyT(fx + p.pad) << p.sh_x) | (KeyT(fy + p.pad) << p.sh_y) | KeyT(fz + p.pad)
            : ~KeyT(0);
}
// Same, raising bit 0 of *status (when status is not NULL) for a rejected row.
template <typename KeyT>
__device__ inline KeyT pack_key(const int4 c, const PackParams& p, int32_t* status) {
  bool bad = false;
  const KeyT k = pack_key_flag<KeyT>(c, p, bad);
  if (bad && status) atomicOr(status, 1);
  return k;
}
// Pins a loaded value in a vector register at this point of the program (used after a whole
// batch of loads has been issued): the compiler can then neither sink the loads into later
// branches nor spread them between other memory operations.  Loads and stores share one completion counter on this target, so a load
// that is waited for between stores also waits for every store issued before it.
#define SPC_PIN_LOADED(x) asm volatile("" : "+v"(x))
#endif

// ---------------------------------------------------------------- bucket sort (own kernels)
constexpr int BS_MAX_WG = 128;      // workgroups of the count / scatter passes
constexpr int BS_MAX_BIN_BITS = 14;
constexpr int BS_MAX_BIN = 1 << BS_MAX_BIN_BITS;  // fine bins (top used key bits)
// Sizes of the partitioning sort; below: one workgroup in LDS; above: rocPRIM (with 16384 bins at most, the windows of
// the rank pass outgrow its LDS beyond that).  3 * 10^6 keys: pack + sort 150 us against 177 us with rocPRIM,
// 5 * 10^6: 234 against 286.
constexpr int64_t BS_MIN_N = 4096, BS_MAX_N = 8192 * 1024;
inline bool use_bucket_sort(int64_t n) { return n >= BS_MIN_N && n <= BS_MAX_N; }
constexpr int BS_PART = 64;         // keys per rank workgroup
constexpr int BS_PAD_KEYS = 32;     // all-ones keys kept behind the scattered keys
struct BucketPlan {
  int n_wg, per, shift, n_bin;
};
BucketPlan bucket_plan(int64_t n, int used_bits);
size_t bucket_sort_ws_bytes(int key_bits, int64_t n);
// coords -> sorted keys (+ permutation); enqueues four kernels (count, colscan, scatter, rank)
int bucket_pack_sort(int key_bits, const int4* coords, int64_t n, const PackParams& pp, int used_bits, int32_t* status,
                     void* keys_out, int32_t* perm_out, void* ws, hipStream_t s);
// sorted distinct values of keys_in & mask, count to *n_out [device]; enqueues five kernels
int bucket_mask_unique(int key_bits, const void* keys_in, int64_t n, uint64_t mask, int used_bits, void* keys_out,
                       int32_t* n_out, void* ws, hipStream_t s);

// fewer than BS_MIN_N keys: one workgroup sorts them in LDS, one launch (n_out [device] receives the distinct count)
int small_pack_sort(int key_bits, const int4* coords, int64_t n, const PackParams& pp, int used_bits, int32_t* status, void* keys_out,
                    int32_t* perm_out, hipStream_t s);
int small_mask_unique(int key_bits, const void* keys_in, int64_t n, uint64_t mask, int used_bits, void* keys_out, int32_t* n_out,
                      hipStream_t s);

// ---------------------------------------------------------------- sort (rocPRIM radix sort)
size_t sort_pairs_temp_bytes(int key_bits, int64_t n);
int sort_pairs(int key_bits, const void* keys_in, void* keys_out, const int32_t* vals_in, int32_t* vals_out,
               int64_t n, int end_bit, void* temp, size_t temp_bytes, hipStream_t s);
size_t sort_keys_temp_bytes(int key_bits, int64_t n);
int sort_keys(int key_bits, const void* keys_in, void* keys_out, int64_t n, int end_bit, void* temp,
              size_t temp_bytes, hipStream_t s);

}  // namespace spc

// ---------------------------------------------------------------- kernel map object
struct spc_kmap {
  std::atomic<int> refs{1};
  spc::PackInfo pi{};
  spc_layer_desc desc{};
  int K3 = 0;
  bool sym = false;                 // WS lists hold offsets k < (K^3-1)/2 only (symmetric half-map)
  int k_lim = 0;                    // offsets that have a WS list of their own
  int hybrid_t = 0;                 // > 0: built for the hybrid dual dataflow with this threshold
  spc::KMask os_k{}, ws_k{};        // offsets whose matrix column / whose list the build wrote
  spc::Level* in_level = nullptr;   // the layer's input voxels
  spc::Level* out_level = nullptr;  // the layer's output voxels
  const int32_t* in_perm = nullptr; // caller's row number of every input voxel (borrowed), or NULL
  int64_t out_cap = 0;              // rows allocated in os_map / ws lists
  int64_t n_out_hint = -1;          // caller's estimate of n_out for kernel selection while n_host is unknown
  bool captured = false;            // built while its stream was being captured into a graph
  int64_t n_blocks_cap = 0;         // 32-row blocks allocated
  int mask_words = 0;               // ceil(K3/32)
  int32_t* os_map = nullptr;        // blocked OS layout [n_blocks][K3][32]: entry (i,k) at ((i/32)*K3+k)*32 + i%32
  uint32_t* block_masks = nullptr;  // [n_blocks][mask_words]: bit k set iff some row of the block has offset k
  int32_t* ws_in = nullptr;         // [K3][out_cap]
  int32_t* ws_out = nullptr;        // [K3][out_cap]
  int32_t* nnz_dev = nullptr;       // [K3]
  int32_t* tile_counts = nullptr;   // [K3][n_tiles] scratch of the two-pass compaction
  int2* tile_pairs = nullptr;       // per search tile a slab of compacted (in, out) pairs (scratch of the list build)
  int64_t ws_stride = 0;            // entries between consecutive lists in ws_in / ws_out
  int32_t* inv_parent = nullptr;    // strided maps, on request: for every INPUT voxel p its pair (out q, offset k) as q*K^3+k
  spc_kmap* twin = nullptr;         // transposed map derived from its strided twin (a reference is held): WS lists alias the twin's
  int tile = 0, n_tiles = 0;
  std::vector<int64_t> nnz_host;    // filled lazily
  hipEvent_t ready = nullptr;       // recorded after the last build kernel
  bool wait_on_use = false;         // nobody has joined the build stream: consumers on other streams wait for `ready`
  hipStream_t last_waiter = nullptr;  // the consumer stream that has waited for `ready` most recently
  std::vector<hipStream_t> consumers;  // streams other than `stream` whose feature kernels have read the map
  std::vector<hipEvent_t> aux_events;  // fork/join events of the network build that made this map
  hipStream_t stream = nullptr;     // stream the map was built on
  int device = 0;
};
