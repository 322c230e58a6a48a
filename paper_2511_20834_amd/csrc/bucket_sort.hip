// Sort of packed voxel keys for the cloud sizes of this workload (thousands to about half a
// million keys): one most-significant-digit split into fine bins, then ranking (pack + sort) or a
// per-bucket network sort (downsampling).  Short launches, no look-back spinning, no global atomics:
//
//   count    each workgroup produces its share of the keys (packing coordinates, Section 5.3,
//            or masking the keys of a finer level, Section 5.5), histograms the top `fb` used
//            key bits ("fine bins") in LDS and writes one row of the table [workgroup][bin];
//   colscan  exclusive prefixes down the table's columns: where a workgroup's keys of a bin go
//            inside the bin, and the bin totals;
//   scatter  each workgroup scans the bin totals (where every bin starts) and moves its keys,
//            with their source index, to their bin's range.  Pack + sort: the workgroups also
//            write, for every 64 scattered positions, the window of whole bins that covers them.
//            Downsampling: workgroup 0 cuts the bin sequence into buckets of about BS_TARGET
//            keys (the buckets adapt to the key distribution: a LiDAR sweep is many times denser
//            near the sensor);
//   rank     (pack + sort) 64 keys per workgroup; a key's final position is the start of its
//            window plus the number of window keys that sort before it, counted by comparing
//            against every window key (see bs_rank_kernel).  Quadratic in the bin size, but
//            spread evenly over the chip whatever the key distribution;
//   unique   (downsampling) one workgroup per bucket: bitonic network over the keys in LDS
//            (min/max steps, three compare distances per pass: a thread holds the 8 keys those
//            distances connect; distances below 512 run inside the waves without barriers);
//            the bucket's distinct keys are counted and left at the start of the bucket's range;
//   gather   (downsampling) compacts the buckets' distinct keys.
//
// x is the most significant spatial field, so a bin is a slab of the scene.  In the downsampling
// path a single bin that outgrows the LDS tile (a dense slab) is sorted straight in global memory
// by the all-ascending form of the network (first step of every merge compares mirrored
// positions), which sorts any length when the missing tail is taken as +infinity: comparators
// that touch the tail are skipped.  Correct for any input, slow only for degenerate ones.
// The rank kernel orders (key, scattered position) pairs, so equal keys (not a valid cloud, but
// not rejected unless validation was asked for) still get distinct positions and the permutation
// is complete whatever the input.
#include <algorithm>

#include "spc_internal.h"

namespace spc {

constexpr int BS_THREADS = 256;   // sort / gather workgroups
constexpr int BS_WIDE = 1024;     // count / scan / scatter workgroups
constexpr int BS_CAP = 4096;      // keys per LDS tile

__device__ inline int bs_bin(uint64_t key, int shift, int n_bin) {
  const uint64_t b = key >> shift;
  return b < uint64_t(n_bin) ? static_cast<int>(b) : n_bin - 1;  // all-ones keys of rejected rows go last
}

// ---------------------------------------------------------------- key sources
// A source splits "fetch" from "make the key": the kernels below fetch a batch of rows first and
// only then compute, so that the batch's loads are in flight together.
template <typename KeyT>
struct SrcPack {
  const int4* coords;
  PackParams p;
  int32_t* status;
  struct Raw {
    int4 c;
  };
  __device__ Raw load(int64_t i) const { return Raw{coords[i]}; }
  __device__ static void pin(Raw& r) { SPC_PIN_LOADED(r.c.x); }
  __device__ KeyT key(const Raw& r, bool& bad) const { return pack_key_flag<KeyT>(r.c, p, bad); }
  __device__ bool skip(const Raw&, KeyT) const { return false; }
  __device__ void report(bool bad) const {
    if (bad && status) atomicOr(status, 1);
  }
};
template <typename KeyT>
struct SrcMask {
  const KeyT* keys;
  KeyT mask;
  struct Raw {
    KeyT cur, prev;
    bool has_prev;
  };
  __device__ Raw load(int64_t i) const { return Raw{keys[i], keys[i > 0 ? i - 1 : 0], i > 0}; }
  __device__ static void pin(Raw& r) {
    SPC_PIN_LOADED(r.cur);
    SPC_PIN_LOADED(r.prev);
  }
  __device__ KeyT key(const Raw& r, bool&) const { return r.cur & mask; }
  // The finer level is sorted, so runs along z collapse to runs of equal masked keys: only the
  // first key of a run takes part (the result is the set of distinct keys either way).
  __device__ bool skip(const Raw& r, KeyT key) const { return r.has_prev && (r.prev & mask) == key; }
  __device__ void report(bool) const {}
};

// ---------------------------------------------------------------- count
template <typename KeyT, typename Src>
__global__ __launch_bounds__(BS_WIDE) void bs_count_kernel(Src src, int64_t n, int per, int shift, int n_bin,
                                                           KeyT* __restrict__ keys0, int32_t* __restrict__ table) {
  __shared__ int hist[BS_MAX_BIN];
  for (int b = threadIdx.x; b < n_bin; b += BS_WIDE) hist[b] = 0;
  __syncthreads();
  const int64_t lo = int64_t(blockIdx.x) * per, hi = min<int64_t>(n, lo + per);
  bool bad = false;
  // four rows per thread and pass, fetched before any of them is turned into a key
  for (int64_t i0 = lo + threadIdx.x; i0 < hi; i0 += 4 * BS_WIDE) {
    typename Src::Raw raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) raw[u] = src.load(min<int64_t>(i0 + u * BS_WIDE, hi - 1));
#pragma unroll
    for (int u = 0; u < 4; ++u) Src::pin(raw[u]);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      bool bad_u = false;
      const KeyT key = src.key(raw[u], bad_u);
      if (i0 + u * BS_WIDE < hi) {
        bad |= bad_u;
        keys0[i0 + u * BS_WIDE] = key;
        if (!src.skip(raw[u], key)) atomicAdd(&hist[bs_bin(key, shift, n_bin)], 1);
      }
    }
  }
  src.report(bad);
  __syncthreads();
  for (int b = threadIdx.x; b < n_bin; b += BS_WIDE) table[int64_t(blockIdx.x) * n_bin + b] = hist[b];
}

// ---------------------------------------------------------------- column scan
// One thread per four bins: before[w][f] receives the number of keys of bin f held by workgroups
// < w, tot[f] the bin's total.  The loads of 16 table rows are in flight together.
constexpr int BS_COL_THREADS = 64;
__global__ __launch_bounds__(BS_COL_THREADS) void bs_colscan_kernel(const int32_t* __restrict__ table,
                                                                    int32_t* __restrict__ before, int n_wg, int n_bin,
                                                                    int32_t* __restrict__ tot) {
  constexpr int ROWS = 16;
  const int f0 = (blockIdx.x * BS_COL_THREADS + threadIdx.x) * 4;
  if (f0 >= n_bin) return;  // n_bin is a multiple of 4
  int4 run = make_int4(0, 0, 0, 0);
  for (int w0 = 0; w0 < n_wg; w0 += ROWS) {
    int4 c[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) c[r] = *reinterpret_cast<const int4*>(table + int64_t(min(w0 + r, n_wg - 1)) * n_bin + f0);
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
      if (w0 + r < n_wg) {
        *reinterpret_cast<int4*>(before + int64_t(w0 + r) * n_bin + f0) = run;
        run.x += c[r].x;
        run.y += c[r].y;
        run.z += c[r].z;
        run.w += c[r].w;
      }
  }
  *reinterpret_cast<int4*>(tot + f0) = run;
}

// ---------------------------------------------------------------- scatter
// Every workgroup scans the bin totals on its own (16 KB; cheaper than one more launch): start
// of bin f, then the workgroup's first position in the bin.  Workgroup 0 also cuts the bin
// sequence into buckets: bucket j starts at the first bin whose start is >= j * target
// (bstart[n_bucket] = n).
template <typename KeyT, bool DEDUP>
__global__ __launch_bounds__(BS_WIDE) void bs_scatter_kernel(const KeyT* __restrict__ keys0, int64_t n, int per, int shift,
                                                             int n_bin, const int32_t* __restrict__ before,
                                                             const int32_t* __restrict__ tot, int target, int n_bucket,
                                                             KeyT* __restrict__ keys1, int32_t* __restrict__ vals1,
                                                             int32_t* __restrict__ bstart, int2* __restrict__ win) {
  __shared__ int pos[BS_MAX_BIN + 1];  // bin starts, then this workgroup's running position in every bin
  __shared__ int bin_start[DEDUP ? 1 : BS_MAX_BIN + 1];
  __shared__ int wave_tot[BS_WIDE / 64];
  static_assert(BS_MAX_BIN == 4 * BS_WIDE, "one int4 of bins per thread");
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int f0 = t * 4;
  int4 c = make_int4(0, 0, 0, 0), bef = c;
  if (f0 < n_bin) {
    c = *reinterpret_cast<const int4*>(tot + f0);
    bef = *reinterpret_cast<const int4*>(before + int64_t(blockIdx.x) * n_bin + f0);
  }
  const int sum = c.x + c.y + c.z + c.w;
  int x = sum;
  for (int d = 1; d < 64; d <<= 1) {
    const int y = __shfl_up(x, d, 64);
    if (lane >= d) x += y;
  }
  if (lane == 63) wave_tot[wave] = x;
  __syncthreads();
  int base = x - sum, total = 0;  // total: keys that take part (all of them unless DEDUP)
  for (int w = 0; w < BS_WIDE / 64; ++w) {
    if (w < wave) base += wave_tot[w];
    total += wave_tot[w];
  }
  const int4 st = make_int4(base, base + c.x, base + c.x + c.y, base + c.x + c.y + c.z);
  if (DEDUP && blockIdx.x == 0) {
    if (f0 < n_bin) *reinterpret_cast<int4*>(pos + f0) = st;
    if (t == 0) pos[n_bin] = total;
    __syncthreads();
    // bin f opens every bucket j with start(f-1) < j * target <= start(f); bucket 0 opens at bin 0
    for (int f = t; f < n_bin; f += BS_WIDE) {
      const int s1 = pos[f];
      const int j0 = f == 0 ? 0 : pos[f - 1] / target + 1;
      for (int j = j0; j <= s1 / target && j < n_bucket; ++j) bstart[j] = s1;
    }
    // buckets whose threshold lies beyond the last bin's start are empty
    for (int j = pos[n_bin - 1] / target + 1 + t; j < n_bucket; j += BS_WIDE) bstart[j] = total;
    if (t == 0) bstart[n_bucket] = total;
    __syncthreads();
  }
  if (f0 < n_bin) *reinterpret_cast<int4*>(pos + f0) = make_int4(st.x + bef.x, st.y + bef.y, st.z + bef.z, st.w + bef.w);
  if (!DEDUP) {  // the bin starts themselves, for the rank windows at the end
    if (f0 < n_bin) *reinterpret_cast<int4*>(bin_start + f0) = st;
    if (t == 0) bin_start[n_bin] = total;
  }
  __syncthreads();
  const int64_t lo = int64_t(blockIdx.x) * per, hi = min<int64_t>(n, lo + per);
  for (int64_t i0 = lo + threadIdx.x; i0 < hi; i0 += 4 * BS_WIDE) {
    // all keys of the pass are fetched, then all positions drawn, then everything stored
    KeyT key[4], prev[4];
    bool use[4];
    int p[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = min<int64_t>(i0 + u * BS_WIDE, hi - 1);
      key[u] = keys0[i];
      prev[u] = DEDUP ? keys0[i > 0 ? i - 1 : 0] : KeyT(0);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      SPC_PIN_LOADED(key[u]);
      if (DEDUP) SPC_PIN_LOADED(prev[u]);
      const int64_t i = min<int64_t>(i0 + u * BS_WIDE, hi - 1);
      use[u] = i0 + u * BS_WIDE < hi && !(DEDUP && i > 0 && prev[u] == key[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) p[u] = use[u] ? atomicAdd(&pos[bs_bin(key[u], shift, n_bin)], 1) : 0;
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (use[u]) {
        keys1[p[u]] = key[u];
        vals1[p[u]] = static_cast<int32_t>(i0 + u * BS_WIDE);
      }
  }
  if (!DEDUP) {
    // Rank windows (see bs_rank_kernel): part p = scattered positions [p * BS_PART, ...) is ranked
    // inside the range of whole bins that covers it.  Parts are dealt round-robin to the workgroups,
    // one per thread: two binary searches over the bin starts in LDS, done last, while the scattered
    // stores drain.
    if (blockIdx.x == 0 && t < BS_PAD_KEYS) keys1[total + t] = ~KeyT(0);  // the rank kernel reads whole steps
    const int part = blockIdx.x + t * gridDim.x;
    if (int64_t(part) * BS_PART < total) {
      const int x0 = part * BS_PART, x1 = min(x0 + BS_PART, total) - 1;
      // last bin whose start is <= x: the (non-empty) bin that holds position x; both searches in step
      int fa = 0, fb = 0;
      for (int step = n_bin >> 1; step > 0; step >>= 1) {
        const int sa = bin_start[fa + step], sb = bin_start[fb + step];
        if (sa <= x0) fa += step;
        if (sb <= x1) fb += step;
      }
      win[part] = make_int2(bin_start[fa], bin_start[fb + 1]);
    }
  }
}

// ---------------------------------------------------------------- sort
// Element = (key, source index).  32-bit keys travel as one 64-bit word.
template <typename KeyT>
struct Elem;
template <>
struct Elem<uint32_t> {
  uint64_t kv;
  __device__ static Elem make(uint32_t k, int32_t v) { return Elem{(uint64_t(k) << 32) | uint32_t(v)}; }
  __device__ uint32_t key() const { return static_cast<uint32_t>(kv >> 32); }
  __device__ int32_t val() const { return static_cast<int32_t>(uint32_t(kv)); }
  __device__ bool operator<(const Elem& o) const { return kv < o.kv; }
};
template <>
struct Elem<uint64_t> {
  uint64_t k;
  int32_t v;
  __device__ static Elem make(uint64_t k, int32_t v) { return Elem{k, v}; }
  __device__ uint64_t key() const { return k; }
  __device__ int32_t val() const { return v; }
  __device__ bool operator<(const Elem& o) const { return k < o.k || (k == o.k && v < o.v); }
};

// Accessor of the global-memory fallback: the bucket's range of (key, index) pairs.
template <typename KeyT>
struct GlobalRange {
  KeyT* k;
  int32_t* v;
  __device__ Elem<KeyT> get(int i) const { return Elem<KeyT>::make(k[i], v[i]); }
  __device__ void put(int i, const Elem<KeyT>& x) const {
    k[i] = x.key();
    v[i] = x.val();
  }
};

template <typename Acc>
__device__ inline void bs_cmpxchg(const Acc& a, int i, int j) {
  const auto x = a.get(i), y = a.get(j);
  if (y < x) {
    a.put(i, y);
    a.put(j, x);
  }
}

// LDS position of tile element i: one element of padding per 32, so that the strided accesses
// of the short compare distances (a thread's 8 elements are then neighbours, and lanes are 8
// elements apart) spread over the banks instead of hitting the same few.
__device__ inline int bs_at(int i) { return i + (i >> 5); }

// Standard bitonic network on a power-of-two tile of keys in LDS, NB consecutive compare distances
// per barrier: the thread's 2^NB keys are those whose indices differ in bits ltop .. ltop-NB+1.
// The merge of blocks of 2^lk sorts ascending where bit lk of the index is clear; a descending
// block runs the same min/max steps on complemented keys.
template <int NB, typename KeyT>
__device__ inline void bs_lds_round(KeyT* tile, int P, int lk, int ltop) {
  constexpr int R = 1 << NB;
  const int lbot = ltop - NB + 1;
  for (int t = threadIdx.x; t < (P >> NB); t += BS_THREADS) {
    const int base = ((t >> lbot) << (ltop + 1)) | (t & ((1 << lbot) - 1));
    const KeyT flip = (base & (1 << lk)) ? ~KeyT(0) : KeyT(0);
    KeyT e[R];
#pragma unroll
    for (int q = 0; q < R; ++q) e[q] = tile[bs_at(base | (q << lbot))] ^ flip;
#pragma unroll
    for (int sb = NB - 1; sb >= 0; --sb)
#pragma unroll
      for (int q = 0; q < R; ++q)
        if (!(q & (1 << sb))) {
          const int q2 = q | (1 << sb);
          const KeyT lo = min(e[q], e[q2]), hi = max(e[q], e[q2]);
          e[q] = lo;
          e[q2] = hi;
        }
#pragma unroll
    for (int q = 0; q < R; ++q) tile[bs_at(base | (q << lbot))] = e[q] ^ flip;
  }
  __syncthreads();
}

// The same step for compare distances below 512, without a barrier: a wave owns whole chunks of
// 512 keys (64 lanes x 8 keys), the steps of such distances never leave a chunk, and the LDS
// executes one wave's accesses in program order.
constexpr int BS_CHUNK_BITS = 9;
template <int NB, typename KeyT>
__device__ inline void bs_wave_round(KeyT* tile, int P, int lk, int ltop) {
  constexpr int R = 1 << NB;
  const int lbot = ltop - NB + 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int csize = min(P, 1 << BS_CHUNK_BITS);
  for (int c0 = wave << BS_CHUNK_BITS; c0 < P; c0 += (BS_THREADS / 64) << BS_CHUNK_BITS)
    for (int u = lane; u < (csize >> NB); u += 64) {
      const int base = c0 | ((u >> lbot) << (ltop + 1)) | (u & ((1 << lbot) - 1));
      const KeyT flip = (base & (1 << lk)) ? ~KeyT(0) : KeyT(0);
      KeyT e[R];
#pragma unroll
      for (int q = 0; q < R; ++q) e[q] = tile[bs_at(base | (q << lbot))] ^ flip;
#pragma unroll
      for (int sb = NB - 1; sb >= 0; --sb)
#pragma unroll
        for (int q = 0; q < R; ++q)
          if (!(q & (1 << sb))) {
            const int q2 = q | (1 << sb);
            const KeyT lo = min(e[q], e[q2]), hi = max(e[q], e[q2]);
            e[q] = lo;
            e[q2] = hi;
          }
#pragma unroll
      for (int q = 0; q < R; ++q) tile[bs_at(base | (q << lbot))] = e[q] ^ flip;
    }
  __builtin_amdgcn_wave_barrier();
}

// compare distances 2^ltop .. 1 of merge lk, all inside the waves' chunks
template <typename KeyT>
__device__ inline void bs_wave_rounds(KeyT* tile, int P, int lk, int ltop) {
  const int first = (ltop + 1) % 3;
  if (first == 1) {
    bs_wave_round<1>(tile, P, lk, ltop);
    ltop -= 1;
  } else if (first == 2) {
    bs_wave_round<2>(tile, P, lk, ltop);
    ltop -= 2;
  }
  for (; ltop >= 2; ltop -= 3) bs_wave_round<3>(tile, P, lk, ltop);
}

// Sorts tile[0, P), P = 2^lp <= 4096; every thread of the workgroup calls it (after a barrier that
// made the tile complete; it ends with one).  Merges of blocks up to 512 run inside the waves;
// a longer merge starts with one workgroup-wide step over its distances of 512 and more.
template <typename KeyT>
__device__ inline void bs_lds_bitonic(KeyT* tile, int lp) {
  const int P = 1 << lp;
  for (int lk = 1; lk <= min(lp, BS_CHUNK_BITS); ++lk) bs_wave_rounds(tile, P, lk, lk - 1);
  __syncthreads();
  for (int lk = BS_CHUNK_BITS + 1; lk <= lp; ++lk) {
    const int nb = lk - BS_CHUNK_BITS;  // 1..3 distances reach across chunks
    if (nb == 1) bs_lds_round<1>(tile, P, lk, lk - 1);
    else if (nb == 2) bs_lds_round<2>(tile, P, lk, lk - 1);
    else bs_lds_round<3>(tile, P, lk, lk - 1);
    bs_wave_rounds(tile, P, lk, BS_CHUNK_BITS - 1);
    __syncthreads();
  }
}

// Sorts positions [0, m) ascending; every thread of the workgroup calls it.
template <typename Acc>
__device__ inline void bs_bitonic(const Acc& a, int m) {
  int lp = 0;
  while ((1 << lp) < m) ++lp;
  const int half = (1 << lp) >> 1;
  for (int lk = 1; lk <= lp; ++lk) {  // merges of blocks of k = 2^lk
    const int k = 1 << lk, lh = lk - 1;
    for (int t = threadIdx.x; t < half; t += BS_THREADS) {  // mirrored step
      const int blk = t >> lh, off = t & ((1 << lh) - 1);
      const int i = (blk << lk) + off, j = (blk << lk) + k - 1 - off;
      if (j < m) bs_cmpxchg(a, i, j);
    }
    __syncthreads();
    for (int ld = lk - 2; ld >= 0; --ld) {  // half-cleaners of distance d = 2^ld
      for (int t = threadIdx.x; t < half; t += BS_THREADS) {
        const int i = ((t >> ld) << (ld + 1)) + (t & ((1 << ld) - 1)), j = i + (1 << ld);
        if (j < m) bs_cmpxchg(a, i, j);
      }
      __syncthreads();
    }
  }
}

// ---------------------------------------------------------------- rank (pack + sort path)
// After the scatter the keys are ordered by bin, unordered inside a bin.  Workgroup p takes the
// BS_PART = 64 keys at scattered positions [p * BS_PART, ...), one per lane, each of its four waves
// a quarter of the comparisons, and ranks each of them inside the window of whole bins that covers those positions (widened to multiples of 32
// positions): every key before the window is smaller and every key behind it larger, so
// window start + (number of window keys that sort before mine) is the key's final position.
// "Sorts before" is (key, scattered position) order, which makes the positions of equal keys
// distinct without any atomics; below and above the workgroup's own 64 positions that is a plain
// <= resp. < on the key.  Every lane of a wave compares its key with the same window key at the same
// time, so the window is read with scalar loads (128 bytes per step, the next step's load in
// flight while the current one is compared) and a comparison is two vector instructions with a
// scalar operand; LDS only carries the four partial counts of a key to the wave that stores.  (Reading the window back from LDS at a wave-uniform address
// was measured four times slower: 16-byte LDS reads of one address by all lanes are not broadcast.)
// Work per key grows with the window, i.e. with the size of the bins involved, but a big bin is
// shared by as many workgroups as it has parts: no workgroup sorts a dense region of the scene
// alone, which is what bounded the compare-exchange network this replaces on the pack + sort path.
// The scatter leaves BS_RANK_STEP all-ones keys behind the last key, so that whole steps can be
// read at the end of the array.
constexpr int BS_RANK_STEP = BS_PAD_KEYS;  // positions; a window is a whole number of steps
// 128 bytes of keys at a wave-uniform address in scalar registers.  The load is issued by hand and
// its arrival awaited by hand, one compare step later: left to the compiler, the load of a step
// ends up right in front of its first use and every step pays the scalar-memory latency.
typedef uint32_t bs_u32x16 __attribute__((ext_vector_type(16)));
struct BsChunk {
  bs_u32x16 lo, hi;
  __device__ void issue(const void* p) {
    asm volatile("s_load_dwordx16 %0, %2, 0x0\n\ts_load_dwordx16 %1, %2, 0x40" : "=&s"(lo), "=&s"(hi) : "s"(p) : "memory");
  }
  // the counters are operands only to keep the compare step that runs under the load in front of the wait
  __device__ void arrive(int (&c)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(lo), "+s"(hi), "+v"(c[0]), "+v"(c[1]), "+v"(c[2]), "+v"(c[3]));
  }
  template <typename KeyT>
  __device__ KeyT key(int q) const {  // q-th key of the chunk, q a compile-time constant after unrolling
    if constexpr (sizeof(KeyT) == 4) return q < 16 ? lo[q] : hi[q - 16];
    else return q < 8 ? (uint64_t(lo[2 * q + 1]) << 32) | lo[2 * q] : (uint64_t(hi[2 * q - 15]) << 32) | hi[2 * q - 16];
  }
};

// keys k[a, b) that sort before (key, x): MODE 0 for positions below the workgroup's own 64 (equal
// keys count), 2 for positions above (they do not), 1 for the own positions (full comparison).
// a and b are multiples of BS_RANK_STEP.
template <int MODE, typename KeyT>
__device__ inline int bs_count_before(const KeyT* __restrict__ k, int a, int b, KeyT key, int x) {
  constexpr int C = 128 / sizeof(KeyT);  // keys per chunk
  static_assert(BS_RANK_STEP % C == 0, "a step of positions is a whole number of chunks");
  int c[4] = {0, 0, 0, 0};
  if (a >= b) return 0;
  auto compare = [&](const BsChunk& ch, int j) {
#pragma unroll
    for (int q = 0; q < C; ++q) {
      const KeyT e = ch.template key<KeyT>(q);
      bool before;
      if (MODE == 0) before = e <= key;
      else if (MODE == 2) before = e < key;
      else before = e < key || (e == key && j + q < x);
      c[q & 3] += before ? 1 : 0;
    }
  };
  BsChunk A, B;
  A.issue(k + a);
  A.arrive(c);
  for (int j = a; j < b; j += 2 * C) {  // the last chunk is fetched once more instead of running past b
    B.issue(k + min(j + C, b - C));
    compare(A, j);
    B.arrive(c);
    if (j + C < b) {
      A.issue(k + min(j + 2 * C, b - C));
      compare(B, j + C);
      A.arrive(c);
    }
  }
  return (c[0] + c[1]) + (c[2] + c[3]);
}

template <typename KeyT>
__global__ __launch_bounds__(BS_THREADS) void bs_rank_kernel(const KeyT* __restrict__ keys1, const int32_t* __restrict__ vals1,
                                                             const int2* __restrict__ win, int n, KeyT* __restrict__ out_k,
                                                             int32_t* __restrict__ out_v) {
  constexpr int WAVES = BS_THREADS / 64;
  static_assert(BS_PART == 64, "one key per lane");
  __shared__ int partial[WAVES][BS_PART];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int own0 = blockIdx.x * BS_PART;
  const int x = own0 + lane;
  const bool act = x < n;
  const int2 w = win[blockIdx.x];
  const KeyT key = act ? keys1[x] : ~KeyT(0);
  const int32_t val = (act && out_v && wave == 0) ? vals1[x] : 0;
  const int n_pad = (n + BS_RANK_STEP - 1) & ~(BS_RANK_STEP - 1);  // positions n .. n_pad - 1 hold all-ones keys
  const int g0 = w.x & ~(BS_RANK_STEP - 1);
  const int g1 = min(max((w.y + BS_RANK_STEP - 1) & ~(BS_RANK_STEP - 1), own0 + BS_PART), n_pad);
  // the window is cut into the part below the own positions, the own positions and the part above;
  // each is shared out among the waves in contiguous quarters (rounded to whole steps)
  const int own1 = min(own0 + BS_PART, g1);
  auto quarter = [&](int a, int b, int& qa, int& qb) {
    const int steps = (b - a) / BS_RANK_STEP, per = (steps + WAVES - 1) / WAVES;
    qa = min(a + wave * per * BS_RANK_STEP, b);
    qb = min(qa + per * BS_RANK_STEP, b);
  };
  int qa, qb;
  quarter(g0, own0, qa, qb);
  int c = bs_count_before<0>(keys1, qa, qb, key, x);
  quarter(own0, own1, qa, qb);
  c += bs_count_before<1>(keys1, qa, qb, key, x);
  quarter(own1, g1, qa, qb);
  c += bs_count_before<2>(keys1, qa, qb, key, x);
  partial[wave][lane] = c;
  __syncthreads();
  if (wave == 0 && act) {
    int r = g0;
#pragma unroll
    for (int v = 0; v < WAVES; ++v) r += partial[v][lane];
    out_k[r] = key;
    if (out_v) out_v[r] = val;
  }
}

// Downsampling path: one workgroup per bucket sorts the bucket's keys with the network above and
// leaves its distinct keys at the start of the bucket's range of out_k, their number in
// ucount[bucket].  A bucket that outgrows the LDS tile is sorted in global memory (vals1 travels
// along as the network's second field and is otherwise unused).
template <typename KeyT>
__global__ __launch_bounds__(BS_THREADS) void bs_unique_kernel(KeyT* __restrict__ keys1, int32_t* __restrict__ vals1,
                                                               const int32_t* __restrict__ bstart, KeyT* __restrict__ out_k,
                                                               int32_t* __restrict__ ucount) {
  constexpr int CAP = BS_CAP;
  constexpr int EPT = CAP / BS_THREADS;
  __shared__ KeyT tile[CAP + CAP / 32];
  __shared__ int wave_tot[BS_THREADS / 64];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int s = bstart[blockIdx.x], m = bstart[blockIdx.x + 1] - s;
  if (m <= 0) {
    if (t == 0) ucount[blockIdx.x] = 0;
    return;
  }
  const bool in_lds = m <= CAP;
  if (in_lds) {
    int lp = 0;
    while ((1 << lp) < m) ++lp;
    const int P = 1 << lp;
    KeyT key[EPT];  // all loads of the thread in flight together
#pragma unroll
    for (int r = 0; r < EPT; ++r) {
      const int i = r * BS_THREADS + t;
      key[r] = i < m ? keys1[s + i] : ~KeyT(0);
    }
#pragma unroll
    for (int r = 0; r < EPT; ++r) {
      const int i = r * BS_THREADS + t;
      if (i < P) tile[bs_at(i)] = key[r];
    }
    __syncthreads();
    bs_lds_bitonic(tile, lp);
  } else {
    bs_bitonic(GlobalRange<KeyT>{keys1 + s, vals1 + s}, m);
  }
  auto key_at = [&](int i) -> KeyT { return in_lds ? tile[bs_at(i)] : keys1[s + i]; };
  // heads of runs of equal keys, compacted in order (positions are visited in array order)
  int run = 0;
  for (int i0 = 0; i0 < m; i0 += BS_THREADS) {
    const int i = i0 + t;
    const bool head = i < m && (i == 0 || key_at(i) != key_at(i - 1));
    const KeyT kv = i < m ? key_at(i) : KeyT(0);
    const unsigned long long bal = __ballot(head);
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int base = run, tot = 0;
    for (int w = 0; w < BS_THREADS / 64; ++w) {
      if (w < wave) base += wave_tot[w];
      tot += wave_tot[w];
    }
    // out_k is a different buffer from keys1, so positions still to be read are not overwritten
    if (head) out_k[s + base + __popcll(bal & ((1ull << lane) - 1ull))] = kv;
    run += tot;
    __syncthreads();
  }
  if (t == 0) ucount[blockIdx.x] = run;
}

// Compacts the buckets' unique keys: out[prefix(ucount)[b] + i] = in[bstart[b] + i]; total to *n_out.
template <typename KeyT>
__global__ __launch_bounds__(BS_THREADS) void bs_gather_kernel(const KeyT* __restrict__ in, const int32_t* __restrict__ bstart,
                                                               const int32_t* __restrict__ ucount, int n_bucket,
                                                               KeyT* __restrict__ out, int32_t* __restrict__ n_out) {
  __shared__ int pre[BS_MAX_BUCKET];
  __shared__ int wave_tot[BS_THREADS / 64];
  constexpr int PER = BS_MAX_BUCKET / BS_THREADS;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int loc[PER], sum = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int b = t * PER + j;
    loc[j] = b < n_bucket ? ucount[b] : 0;
    sum += loc[j];
  }
  int x = sum;
  for (int d = 1; d < 64; d <<= 1) {
    const int y = __shfl_up(x, d, 64);
    if (lane >= d) x += y;
  }
  if (lane == 63) wave_tot[wave] = x;
  __syncthreads();
  int base = x - sum, total = 0;
  for (int w = 0; w < BS_THREADS / 64; ++w) {
    if (w < wave) base += wave_tot[w];
    total += wave_tot[w];
  }
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int b = t * PER + j;
    if (b < n_bucket) pre[b] = base;
    base += loc[j];
  }
  __syncthreads();
  if (blockIdx.x == 0 && t == 0) *n_out = total;
  for (int b = blockIdx.x; b < n_bucket; b += gridDim.x) {
    const int c = ucount[b], src = bstart[b], dst = pre[b];
    for (int i = t; i < c; i += BS_THREADS) out[dst + i] = in[src + i];
  }
}

// ---------------------------------------------------------------- host
BucketPlan bucket_plan(int64_t n, int used_bits) {
  BucketPlan p{};
  int n_wg = static_cast<int>(std::min<int64_t>(std::max<int64_t>((n + 4095) / 4096, 1), BS_MAX_WG));
  p.per = static_cast<int>(((n + n_wg - 1) / n_wg + BS_WIDE - 1) / BS_WIDE * BS_WIDE);
  p.n_wg = static_cast<int>(std::max<int64_t>((n + p.per - 1) / p.per, 1));
  // About 16 keys per bin of the key space: packing descriptors round every field up to whole
  // bits and scenes are far from cubic, so typically a quarter of the bins is populated.
  int fb = 8;
  while (fb < BS_MAX_BIN_BITS && (int64_t(16) << fb) < n) ++fb;
  fb = std::max(2, std::min(fb, used_bits));
  p.shift = used_bits - fb;
  p.n_bin = 1 << fb;
  p.target = BS_TARGET;
  p.n_bucket = static_cast<int>(std::max<int64_t>((n + p.target - 1) / p.target, 1));
  return p;
}

size_t bucket_sort_ws_bytes(int key_bits, int64_t n) {
  const size_t nn = static_cast<size_t>(std::max<int64_t>(n, 1));
  const size_t k = ((nn + BS_PAD_KEYS) * (key_bits / 8) + 255) / 256 * 256, v = (nn * 4 + 255) / 256 * 256;
  return 2 * k + v + (2 * size_t(BS_MAX_WG) * BS_MAX_BIN + BS_MAX_BIN + 64 + 2 * (size_t(BS_MAX_BUCKET) + 64) + 2 * BS_MAX_PART) * 4;
}

namespace {
template <typename KeyT>
struct Ws {
  KeyT* keys0;
  KeyT* keys1;
  int32_t* vals1;
  int32_t* table;
  int32_t* before;
  int32_t* fstart;
  int32_t* bstart;
  int32_t* ucount;
  int2* win;
};
template <typename KeyT>
Ws<KeyT> carve(void* ws, int64_t n) {
  const size_t nn = static_cast<size_t>(std::max<int64_t>(n, 1));
  const size_t k = ((nn + BS_PAD_KEYS) * sizeof(KeyT) + 255) / 256 * 256, v = (nn * 4 + 255) / 256 * 256;
  char* c = static_cast<char*>(ws);
  Ws<KeyT> w;
  w.keys0 = reinterpret_cast<KeyT*>(c);
  w.keys1 = reinterpret_cast<KeyT*>(c + k);
  w.vals1 = reinterpret_cast<int32_t*>(c + 2 * k);
  w.table = reinterpret_cast<int32_t*>(c + 2 * k + v);
  w.before = w.table + size_t(BS_MAX_WG) * BS_MAX_BIN;
  w.fstart = w.before + size_t(BS_MAX_WG) * BS_MAX_BIN;
  w.bstart = w.fstart + BS_MAX_BIN + 64;
  w.ucount = w.bstart + BS_MAX_BUCKET + 64;
  w.win = reinterpret_cast<int2*>(w.ucount + BS_MAX_BUCKET + 64);  // 8-byte aligned: every part above is a multiple of 256 bytes
  return w;
}

// count, scan, scatter: keys1/vals1 partitioned by fine bin, bstart = bucket boundaries
template <typename KeyT, bool DEDUP, typename Src>
void partition(const Src& src, int64_t n, const BucketPlan& p, const Ws<KeyT>& w, hipStream_t s) {
  const size_t lds = 0;
  hipLaunchKernelGGL((bs_count_kernel<KeyT, Src>), dim3(p.n_wg), dim3(BS_WIDE), lds, s, src, n, p.per, p.shift, p.n_bin, w.keys0,
                     w.table);
  const int col_wg = (p.n_bin / 4 + BS_COL_THREADS - 1) / BS_COL_THREADS;
  hipLaunchKernelGGL(bs_colscan_kernel, dim3(col_wg), dim3(BS_COL_THREADS), 0, s, w.table, w.before, p.n_wg, p.n_bin, w.fstart);
  hipLaunchKernelGGL((bs_scatter_kernel<KeyT, DEDUP>), dim3(p.n_wg), dim3(BS_WIDE), 0, s, w.keys0, n, p.per, p.shift, p.n_bin, w.before,
                     w.fstart, p.target, p.n_bucket, w.keys1, w.vals1, w.bstart, w.win);
}
}  // namespace

template <typename KeyT>
static int pack_sort_t(const int4* coords, int64_t n, const PackParams& pp, int used_bits, int32_t* status, void* keys_out,
                       int32_t* perm_out, void* ws, hipStream_t s) {
  const BucketPlan p = bucket_plan(n, used_bits);
  const Ws<KeyT> w = carve<KeyT>(ws, n);
  partition<KeyT, false>(SrcPack<KeyT>{coords, pp, status}, n, p, w, s);
  const int n_part = static_cast<int>((n + BS_PART - 1) / BS_PART);
  hipLaunchKernelGGL(bs_rank_kernel<KeyT>, dim3(n_part), dim3(BS_THREADS), 0, s, w.keys1, w.vals1, w.win, static_cast<int>(n),
                     static_cast<KeyT*>(keys_out), perm_out);
  if (hipGetLastError() != hipSuccess) return set_error(SPC_ERR_HIP, "sort launch failed");
  return SPC_OK;
}

int bucket_pack_sort(int key_bits, const int4* coords, int64_t n, const PackParams& pp, int used_bits, int32_t* status,
                     void* keys_out, int32_t* perm_out, void* ws, hipStream_t s) {
  return key_bits == 32 ? pack_sort_t<uint32_t>(coords, n, pp, used_bits, status, keys_out, perm_out, ws, s)
                        : pack_sort_t<uint64_t>(coords, n, pp, used_bits, status, keys_out, perm_out, ws, s);
}

template <typename KeyT>
static int mask_unique_t(const void* keys_in, int64_t n, uint64_t mask, int used_bits, void* keys_out, int32_t* n_out, void* ws,
                         hipStream_t s) {
  const BucketPlan p = bucket_plan(n, used_bits);
  const Ws<KeyT> w = carve<KeyT>(ws, n);
  partition<KeyT, true>(SrcMask<KeyT>{static_cast<const KeyT*>(keys_in), static_cast<KeyT>(mask)}, n, p, w, s);
  // distinct keys of every bucket land at the start of its range in keys0 (free again by now)
  hipLaunchKernelGGL(bs_unique_kernel<KeyT>, dim3(p.n_bucket), dim3(BS_THREADS), 0, s, w.keys1, w.vals1, w.bstart, w.keys0, w.ucount);
  hipLaunchKernelGGL(bs_gather_kernel<KeyT>, dim3(std::min(p.n_bucket, 256)), dim3(BS_THREADS), 0, s, w.keys0, w.bstart, w.ucount,
                     p.n_bucket, static_cast<KeyT*>(keys_out), n_out);
  if (hipGetLastError() != hipSuccess) return set_error(SPC_ERR_HIP, "downsample launch failed");
  return SPC_OK;
}

int bucket_mask_unique(int key_bits, const void* keys_in, int64_t n, uint64_t mask, int used_bits, void* keys_out,
                       int32_t* n_out, void* ws, hipStream_t s) {
  return key_bits == 32 ? mask_unique_t<uint32_t>(keys_in, n, mask, used_bits, keys_out, n_out, ws, s)
                        : mask_unique_t<uint64_t>(keys_in, n, mask, used_bits, keys_out, n_out, ws, s);
}

}  // namespace spc
