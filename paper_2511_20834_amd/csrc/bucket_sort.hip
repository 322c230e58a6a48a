// Sort of packed voxel keys for the cloud sizes of this workload (thousands to a few million
// keys): one most-significant-digit split into fine bins, then every key is ranked by
// counting inside the window of bins around it (from 600 k keys on after a second split of the
// window in LDS, see bs_rank_lds_kernel).  Short launches, no look-back spinning:
//
//   count    each workgroup produces its share of the keys (packing coordinates, Section 5.3,
//            or masking the keys of a finer level, Section 5.5), histograms the top `fb` used
//            key bits ("fine bins") in LDS and writes one row of the table [workgroup][bin];
//   colscan  exclusive prefixes down the table's columns: where a workgroup's keys of a bin go
//            inside the bin, and the bin totals;
//   scatter  each workgroup scans the bin totals (where every bin starts) and moves its keys,
//            with their source index, to their bin's range; the workgroups also write, for every
//            64 scattered positions, the window of whole bins that covers them;
//   rank     64 keys per workgroup; a key's final position is the start of its window plus the
//            number of window keys that sort before it, counted by comparing against every
//            window key (see bs_rank_kernel).  Quadratic in the bin size, but spread evenly over
//            the chip whatever the key distribution (a LiDAR sweep is many times denser near the
//            sensor, and x, the most significant spatial field, makes a bin a slab of the scene).
//
// Pack + sort ranks (key, scattered position) pairs, so equal keys (not a valid cloud, but not
// rejected unless validation was asked for) still get distinct positions and the permutation is
// complete whatever the input.  Downsampling ranks the masked keys alone: equal keys fall on one
// position, first arrivals are marked in a bitmap and counted per chunk with global atomics,
// and a fifth kernel, compact, closes the gaps.
#include <algorithm>

#include "spc_internal.h"

namespace spc {

constexpr int BS_THREADS = 256;   // sort / gather workgroups
constexpr int BS_WIDE = 1024;     // count / scan / scatter workgroups

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
  extern __shared__ int hist[];  // [n_bin]
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
// of bin f, then the workgroup's first position in the bin, and moves its keys, with their source
// index, to their bin's range.  It also prepares the rank pass: for every BS_PART scattered
// positions the window of whole bins that covers them, BS_PAD_KEYS all-ones keys behind the last
// key, the number of keys that take part and, for the downsampling variant (DEDUP: of a run of
// equal adjacent keys only the first takes part), the cleared position bitmap and chunk counters.
template <typename KeyT, bool DEDUP>
__global__ __launch_bounds__(BS_WIDE) void bs_scatter_kernel(const KeyT* __restrict__ keys0, int64_t n, int per, int shift,
                                                             int n_bin, const int32_t* __restrict__ before,
                                                             const int32_t* __restrict__ tot, KeyT* __restrict__ keys1,
                                                             int32_t* __restrict__ vals1, int2* __restrict__ win,
                                                             int32_t* __restrict__ n_part_keys, uint32_t* __restrict__ bits,
                                                             int n_words, int32_t* __restrict__ ccnt, int n_chunks,
                                                             int32_t* __restrict__ rest_count) {
  extern __shared__ int lds_bins[];
  int* pos = lds_bins;                    // [n_bin + 1] this workgroup's running position in every bin
  int* bin_start = lds_bins + n_bin + 1;  // [n_bin + 1] where every bin starts
  __shared__ int wave_tot[BS_WIDE / 64];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  if (DEDUP) {  // the rank pass marks positions and counts them per chunk: both start from zero
    for (int i = blockIdx.x * BS_WIDE + t; i < n_words; i += gridDim.x * BS_WIDE) bits[i] = 0u;
    for (int i = blockIdx.x * BS_WIDE + t; i < n_chunks; i += gridDim.x * BS_WIDE) ccnt[i] = 0;
  }
  // exclusive scan of the bin totals, four bins per thread and round (one round up to 4096 bins)
  int total = 0;  // keys that take part (all of them unless DEDUP)
  for (int r0 = 0; r0 < n_bin; r0 += 4 * BS_WIDE) {
    const int f0 = r0 + t * 4;
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
    if (r0 > 0) __syncthreads();  // the wave totals of the round before have been read
    if (lane == 63) wave_tot[wave] = x;
    __syncthreads();
    int base = total + x - sum;
    for (int w = 0; w < BS_WIDE / 64; ++w) {
      if (w < wave) base += wave_tot[w];
      total += wave_tot[w];
    }
    if (f0 < n_bin) {
      const int s0 = base, s1 = base + c.x, s2 = s1 + c.y, s3 = s2 + c.z;
      pos[f0] = s0 + bef.x;
      pos[f0 + 1] = s1 + bef.y;
      pos[f0 + 2] = s2 + bef.z;
      pos[f0 + 3] = s3 + bef.w;
      bin_start[f0] = s0;
      bin_start[f0 + 1] = s1;
      bin_start[f0 + 2] = s2;
      bin_start[f0 + 3] = s3;
    }
  }
  if (t == 0) bin_start[n_bin] = total;
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
        if (!DEDUP) vals1[p[u]] = static_cast<int32_t>(i0 + u * BS_WIDE);
      }
  }
  // Rank windows (see bs_rank_kernel): part p = scattered positions [p * BS_PART, ...) is ranked
  // inside the range of whole bins that covers it.  Parts are dealt round-robin to the workgroups,
  // one per thread: two binary searches over the bin starts in LDS, done last, while the scattered
  // stores drain.
  if (blockIdx.x == 0) {
    if (t < BS_PAD_KEYS) keys1[total + t] = ~KeyT(0);  // the rank kernels read whole steps
    if (t == 0 && n_part_keys) *n_part_keys = total;
    if (t == 0) *rest_count = 0;  // windows left over by bs_rank_lds_kernel
  }
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
#ifndef BS_RANK_SOLO_N
#define BS_RANK_SOLO_N 400000
#endif
#ifndef BS_RANK_LDS_N
#define BS_RANK_LDS_N 600000  // keys from which the ranking splits its windows once more in LDS (bs_rank_lds_kernel)
#endif
constexpr int BS_RANK_STEP = BS_PAD_KEYS;  // positions; a window is a whole number of steps
// 128 bytes of keys at a wave-uniform address in scalar registers.  The load is issued by hand and
// its arrival awaited by hand, one compare step later: left to the compiler, the load of a step
// ends up right in front of its first use and every step pays the scalar-memory latency.
typedef uint32_t bs_u32x16 __attribute__((ext_vector_type(16)));
struct BsChunk {
  bs_u32x16 lo, hi;
  // SCALAR: the caller's address is in scalar registers already (derived from blockIdx and kernel arguments);
  // otherwise it is the same in every lane but arrives in vector registers (a part number read from a list)
  template <bool SCALAR>
  __device__ void issue(const void* p) {
    const void* q = p;
    if constexpr (!SCALAR) {
      const uint64_t a = reinterpret_cast<uint64_t>(p);
      const uint32_t a_lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
      const uint32_t a_hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
      q = reinterpret_cast<const void*>((static_cast<uint64_t>(a_hi) << 32) | a_lo);
    }
    asm volatile("s_load_dwordx16 %0, %2, 0x0\n\ts_load_dwordx16 %1, %2, 0x40" : "=&s"(lo), "=&s"(hi) : "s"(q) : "memory");
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
template <int MODE, bool SCALAR = true, typename KeyT>
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
  A.template issue<SCALAR>(k + a);
  A.arrive(c);
  for (int j = a; j < b; j += 2 * C) {  // the last chunk is fetched once more instead of running past b
    B.template issue<SCALAR>(k + min(j + C, b - C));
    compare(A, j);
    B.arrive(c);
    if (j + C < b) {
      A.template issue<SCALAR>(k + min(j + 2 * C, b - C));
      compare(B, j + C);
      A.arrive(c);
    }
  }
  return (c[0] + c[1]) + (c[2] + c[3]);
}

// (a device function of the part number: the kernel below ranks part blockIdx.x, bs_rank_rest_kernel the parts
// of the windows that bs_rank_lds_kernel has left over)
template <typename KeyT, int WAVES, bool LISTED = false>
__device__ inline void bs_rank_part(int part, const KeyT* __restrict__ keys1, const int32_t* __restrict__ vals1,
                                    const int2* __restrict__ win, int n, KeyT* __restrict__ out_k, int32_t* __restrict__ out_v) {
  static_assert(BS_PART == 64, "one key per lane");
  __shared__ int partial[WAVES][BS_PART];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int own0 = part * BS_PART;
  const int x = own0 + lane;
  const bool act = x < n;
  const int2 w = win[part];
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
  int c = bs_count_before<0, !LISTED>(keys1, qa, qb, key, x);
  quarter(own0, own1, qa, qb);
  c += bs_count_before<1, !LISTED>(keys1, qa, qb, key, x);
  quarter(own1, g1, qa, qb);
  c += bs_count_before<2, !LISTED>(keys1, qa, qb, key, x);
  int r = g0 + c;
  if constexpr (WAVES > 1) {
    partial[wave][lane] = c;
    __syncthreads();
    r = g0;
#pragma unroll
    for (int v = 0; v < WAVES; ++v) r += partial[v][lane];
  }
  if (wave == 0 && act) {
    out_k[r] = key;
    if (out_v) out_v[r] = val;
  }
}

template <typename KeyT, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void bs_rank_kernel(const KeyT* __restrict__ keys1, const int32_t* __restrict__ vals1,
                                                             const int2* __restrict__ win, int n, KeyT* __restrict__ out_k,
                                                             int32_t* __restrict__ out_v) {
  bs_rank_part<KeyT, WAVES>(blockIdx.x, keys1, vals1, win, n, out_k, out_v);
}

// ---------------------------------------------------------------- rank + compact (downsampling path)
// The distinct masked keys in ascending order.  Ranking as above, on the key alone: equal keys get
// equal positions, so position = window start + (number of window keys smaller than mine) leaves the
// sorted sequence with gaps where a key occurs more than once (the count pass has dropped equal
// neighbours, but the children of one coarse voxel sit in up to four separate runs of the finer
// level).  A position is marked in a bitmap by whoever gets there first, and counted once in its
// chunk of BS_CHUNK positions; bs_compact_kernel then closes the gaps.
constexpr int BS_CHUNK = 1024;
template <typename KeyT, bool LISTED = false>
__device__ inline void bs_rank_unique_part(int part, const KeyT* __restrict__ keys1, const int2* __restrict__ win, int n,
                                           KeyT* __restrict__ sorted, uint32_t* __restrict__ bits, int32_t* __restrict__ ccnt) {
  constexpr int WAVES = BS_THREADS / 64;
  __shared__ int partial[WAVES][BS_PART];
  __shared__ uint32_t lbits[64];
  const int own0 = part * BS_PART;
  if (own0 >= n) return;  // (the whole workgroup)
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int x = own0 + lane;
  const bool act = x < n;
  const int2 w = win[part];
  const KeyT key = act ? keys1[x] : ~KeyT(0);
  const int n_pad = (n + BS_RANK_STEP - 1) & ~(BS_RANK_STEP - 1);  // positions n .. n_pad - 1 hold all-ones keys
  const int g0 = w.x & ~(BS_RANK_STEP - 1);
  const int g1 = min((w.y + BS_RANK_STEP - 1) & ~(BS_RANK_STEP - 1), n_pad);
  const int steps = (g1 - g0) / BS_RANK_STEP, per = (steps + WAVES - 1) / WAVES;
  const int qa = min(g0 + wave * per * BS_RANK_STEP, g1), qb = min(qa + per * BS_RANK_STEP, g1);
  partial[wave][lane] = bs_count_before<2, !LISTED>(keys1, qa, qb, key, x);
  __syncthreads();
  if (wave == 0) {
    int r = g0;
#pragma unroll
    for (int v = 0; v < WAVES; ++v) r += partial[v][lane];
    if (act) sorted[r] = key;  // equal keys write the same value
    // The 64 positions lie in the window, typically within a few hundred positions of its start:
    // their bits are collected in LDS first (64 words from the window start on), so that the global
    // bitmap sees one atomic per word instead of one per key; what a word's atomic finds newly set
    // is counted for the word's chunk (a chunk is 32 words), one counter update per chunk.
    lbits[lane] = 0u;
    __builtin_amdgcn_wave_barrier();
    const int rel = r - g0;
    const bool far = act && rel >= 64 * 32;
    if (act && !far) atomicOr(&lbits[rel >> 5], 1u << (rel & 31));
    __builtin_amdgcn_wave_barrier();
    // lane i then owns word i of the 64; a position beyond them (a very large window) goes to the
    // global bitmap on its own, in a second round
#pragma unroll
    for (int round = 0; round < 2; ++round) {
      const int word_i = round == 0 ? (g0 >> 5) + lane : r >> 5;
      const uint32_t word = round == 0 ? lbits[lane] : (far ? 1u << (r & 31) : 0u);
      if (round == 1 && !__ballot(far)) break;  // uniform
      int fresh = 0;
      if (word) fresh = __popc(word & ~atomicOr(&bits[word_i], word));
      const int chunk = word_i / (BS_CHUNK / 32);
      unsigned long long todo = __ballot(fresh > 0);
      while (todo) {
        const int leader = __builtin_ctzll(todo);
        const int c = __shfl(chunk, leader, 64);
        const bool mine = fresh > 0 && chunk == c;
        int sum = mine ? fresh : 0;
        for (int d = 32; d > 0; d >>= 1) sum += __shfl_xor(sum, d, 64);
        if (lane == leader) atomicAdd(&ccnt[c], sum);
        todo &= ~__ballot(mine);
      }
    }
  }
}

template <typename KeyT>
__global__ __launch_bounds__(BS_THREADS) void bs_rank_unique_kernel(const KeyT* __restrict__ keys1, const int2* __restrict__ win,
                                                                    const int32_t* __restrict__ n_kept,
                                                                    KeyT* __restrict__ sorted, uint32_t* __restrict__ bits,
                                                                    int32_t* __restrict__ ccnt) {
  // (the grid is sized for the level before the equal neighbours were dropped)
  bs_rank_unique_part<KeyT>(blockIdx.x, keys1, win, *n_kept, sorted, bits, ccnt);
}

// out = the marked positions of `sorted`, in order; their number to *n_out.  One workgroup per chunk
// of BS_CHUNK positions: the keys before the chunk are the sum of the earlier chunks' counters.
template <typename KeyT>
__global__ __launch_bounds__(BS_THREADS) void bs_compact_kernel(const KeyT* __restrict__ sorted, const uint32_t* __restrict__ bits,
                                                                const int32_t* __restrict__ ccnt,
                                                                const int32_t* __restrict__ n_kept, KeyT* __restrict__ out,
                                                                int32_t* __restrict__ n_out) {
  static_assert(BS_CHUNK == 4 * BS_THREADS, "four positions per thread");
  __shared__ int red[2][BS_THREADS / 64];
  __shared__ int wsum[BS_CHUNK / 32];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int n = *n_kept, n_chunks = (n + BS_CHUNK - 1) / BS_CHUNK, b = blockIdx.x;
  int before = 0, all = 0;
  for (int i = t; i < n_chunks; i += BS_THREADS) {
    const int c = ccnt[i];
    all += c;
    before += i < b ? c : 0;
  }
  for (int d = 32; d > 0; d >>= 1) {
    before += __shfl_xor(before, d, 64);
    all += __shfl_xor(all, d, 64);
  }
  if (lane == 0) {
    red[0][wave] = before;
    red[1][wave] = all;
  }
  const int wi = t >> 3, sub = t & 7;  // eight threads per bitmap word, four positions each
  const uint32_t word = b < n_chunks ? bits[b * (BS_CHUNK / 32) + wi] : 0u;
  if (sub == 0) wsum[wi] = __popc(word);
  __syncthreads();
  before = 0;
  all = 0;
  for (int w = 0; w < BS_THREADS / 64; ++w) {
    before += red[0][w];
    all += red[1][w];
  }
  if (b == 0 && t == 0) *n_out = all;
  int rank = before + __popc(word & ((1u << (4 * sub)) - 1u));
  for (int w = 0; w < wi; ++w) rank += wsum[w];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int bit = 4 * sub + j;
    if ((word >> bit) & 1u) out[rank++] = sorted[b * BS_CHUNK + wi * 32 + bit];
  }
}

// ---------------------------------------------------------------- rank in LDS (large inputs)
// The ranking above compares every key with its whole window, which is quadratic in the bin size, and the bin
// count is capped (an LDS histogram per workgroup in the count pass): from about half a million keys on that pass
// sets the time of the sort.  Here a workgroup takes BS_LP scattered positions and the window of whole bins around
// them (through the 64-position windows the scatter pass has written), and splits the window once more in LDS:
//   * a thread owns eight consecutive window keys; a key's bin rank inside the window is a prefix sum of "the bin
//     changes here" flags (the scattered array is ordered by bin), so the empty bins of a sparse key space cost
//     nothing;
//   * sub-bin = (bin rank, the next sb key bits below the bin bits), sb chosen per window so that all sub-bins fit
//     the LDS histogram; histogram, exclusive scan, and the keys move, with their window index, to their sub-bin's
//     slots (LDS atomics for the slot: the order inside a sub-bin does not matter);
//   * a key's final position is window start + start of its sub-bin + the number of keys of the sub-bin that sort
//     before it, in (key, window index) order for pack + sort and on the key alone for downsampling (equal keys
//     then share a position; the one with the smallest window index marks the position and is counted for its chunk,
//     which is the same on every workgroup that sees the bin, because all of a bin's keys lie in every window that
//     touches it).
// A window that does not fit (bins of thousands of keys: the floors and walls of dense indoor scenes) is left to
// bs_rank_rest_kernel: the workgroup appends its number to a list, and the 64-position parts of the listed
// workgroups are ranked by comparing against their own windows as above, spread over a fixed grid.
constexpr int BS_LP = 2048;    // own positions per workgroup (a multiple of BS_PART)
constexpr int BS_LW = 4096;    // window keys a workgroup holds
constexpr int BS_LSUB = 4096;  // sub-bins
constexpr int BS_LT = 512;     // threads: eight window keys each
constexpr int BS_LK = BS_LW / BS_LT;
static_assert(BS_LP % BS_PART == 0 && BS_LW >= BS_LP && BS_LK == 8, "window layout");

template <typename KeyT, bool UNIQUE>
__global__ __launch_bounds__(BS_LT) void bs_rank_lds_kernel(const KeyT* __restrict__ keys1, const int32_t* __restrict__ vals1,
                                                            const int2* __restrict__ win, int n_h,
                                                            const int32_t* __restrict__ n_d, int shift, int n_bin,
                                                            KeyT* __restrict__ out_k, int32_t* __restrict__ out_v,
                                                            uint32_t* __restrict__ bits, int32_t* __restrict__ ccnt,
                                                            int32_t* __restrict__ rest_count, int32_t* __restrict__ rest) {
  constexpr int WAVES = BS_LT / 64;
  __shared__ KeyT skey[BS_LW];
  __shared__ uint16_t sidx[BS_LW];
  __shared__ int hist[BS_LSUB];
  __shared__ KeyT s_last[BS_LT];
  __shared__ int wave_tot[WAVES];
  __shared__ uint32_t s_bits[BS_LW / 32 + 2];
  __shared__ int s_cc[BS_LW / BS_CHUNK + 2];
  const int n = n_d ? *n_d : n_h;
  const int own0 = blockIdx.x * BS_LP;
  if (own0 >= n) return;
  const int own1 = min(own0 + BS_LP, n);
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int g0 = win[own0 / BS_PART].x, g1 = win[(own1 - 1) / BS_PART].y;
  const int W = g1 - g0;
  if (W > BS_LW) {  // the window does not fit: bs_rank_rest_kernel ranks these positions
    if (t == 0) rest[atomicAdd(rest_count, 1)] = blockIdx.x;
    return;
  }
  // ---- window keys, eight consecutive ones per thread
  KeyT k[BS_LK];
  const int j0 = t * BS_LK;
#pragma unroll
  for (int u = 0; u < BS_LK; ++u) k[u] = keys1[g0 + min(j0 + u, W - 1)];
  for (int i = t; i < BS_LSUB; i += BS_LT) hist[i] = 0;
  if (UNIQUE) {
    for (int i = t; i < BS_LW / 32 + 2; i += BS_LT) s_bits[i] = 0u;
    if (t < BS_LW / BS_CHUNK + 2) s_cc[t] = 0;
  }
  s_last[t] = k[BS_LK - 1];
  __syncthreads();
  // bin rank inside the window: inclusive prefix of the "bin changes" flags, minus one
  int d[BS_LK], flags = 0;
  {
    int prev_bin = t > 0 ? bs_bin(s_last[t - 1], shift, n_bin) : -1;
#pragma unroll
    for (int u = 0; u < BS_LK; ++u) {
      const int bin = bs_bin(k[u], shift, n_bin);
      flags += (j0 + u < W && bin != prev_bin) ? 1 : 0;
      d[u] = flags;
      prev_bin = bin;
    }
  }
  int x = flags;
  for (int s = 1; s < 64; s <<= 1) {
    const int y = __shfl_up(x, s, 64);
    if (lane >= s) x += y;
  }
  if (lane == 63) wave_tot[wave] = x;
  __syncthreads();
  int base = x - flags, n_bins_here = 0;
  for (int w = 0; w < WAVES; ++w) {
    if (w < wave) base += wave_tot[w];
    n_bins_here += wave_tot[w];
  }
  // sub-bin bits: as many as keep (bins in the window) << sb within the histogram, at most the key bits below the bins
  int sb = 0;
  while (sb < shift && sb < 12 && ((n_bins_here << (sb + 1)) <= BS_LSUB)) ++sb;
  const KeyT sub_mask = (KeyT(1) << sb) - 1;
  int id[BS_LK];
#pragma unroll
  for (int u = 0; u < BS_LK; ++u) {
    id[u] = ((base + d[u] - 1) << sb) | static_cast<int>((k[u] >> (shift - sb)) & sub_mask);
    if (j0 + u < W) atomicAdd(&hist[id[u]], 1);
  }
  __syncthreads();
  // exclusive scan of the sub-bin counts, eight per thread (BS_LSUB = 8 * BS_LT)
  static_assert(BS_LSUB == BS_LK * BS_LT, "eight sub-bins per thread");
  {
    int c[BS_LK], sum = 0;
#pragma unroll
    for (int u = 0; u < BS_LK; ++u) {
      c[u] = hist[j0 + u];
      sum += c[u];
    }
    int y = sum;
    for (int s = 1; s < 64; s <<= 1) {
      const int z = __shfl_up(y, s, 64);
      if (lane >= s) y += z;
    }
    __syncthreads();  // everybody has read the counts and the wave totals of the flags
    if (lane == 63) wave_tot[wave] = y;
    __syncthreads();
    int run = y - sum;
    for (int w = 0; w < wave; ++w) run += wave_tot[w];
#pragma unroll
    for (int u = 0; u < BS_LK; ++u) {
      hist[j0 + u] = run;  // becomes the sub-bin's cursor
      run += c[u];
    }
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < BS_LK; ++u)
    if (j0 + u < W) {
      const int slot = atomicAdd(&hist[id[u]], 1);
      skey[slot] = k[u];
      sidx[slot] = static_cast<uint16_t>(j0 + u);
    }
  __syncthreads();
  // after the moves hist[i] is the end of sub-bin i, i.e. the start of sub-bin i + 1
  const int o0 = own0 - g0, o1 = own1 - g0;  // the own positions, as window indices
#pragma unroll
  for (int u = 0; u < BS_LK; ++u) {
    const int j = j0 + u;
    if (j < o0 || j >= o1) continue;
    const int lo = id[u] > 0 ? hist[id[u] - 1] : 0, hi = hist[id[u]];
    int c = lo;
    bool first = true;  // UNIQUE: no equal key at a smaller window index
    for (int s = lo; s < hi; ++s) {
      const KeyT e = skey[s];
      const int ej = sidx[s];
      if constexpr (UNIQUE) {
        c += e < k[u] ? 1 : 0;
        first = first && !(e == k[u] && ej < j);
      } else {
        c += (e < k[u] || (e == k[u] && ej < j)) ? 1 : 0;
      }
    }
    const int r = g0 + c;
    out_k[r] = k[u];
    if constexpr (!UNIQUE) {
      if (out_v) out_v[r] = vals1[g0 + j];
    } else if (first) {
      const int rel = r - (g0 & ~31);
      atomicOr(&s_bits[rel >> 5], 1u << (rel & 31));
    }
  }
  if constexpr (UNIQUE) {
    __syncthreads();
    const int word0 = g0 >> 5, chunk0 = word0 / (BS_CHUNK / 32);
    if (t < BS_LW / 32 + 2) {
      const uint32_t word = s_bits[t];
      if (word) {  // the marks of different workgroups in one word are different bits
        atomicOr(&bits[word0 + t], word);
        atomicAdd(&s_cc[(word0 + t) / (BS_CHUNK / 32) - chunk0], __popc(word));
      }
    }
    __syncthreads();
    if (t < BS_LW / BS_CHUNK + 2 && s_cc[t]) atomicAdd(&ccnt[chunk0 + t], s_cc[t]);
  }
}

// The parts bs_rank_lds_kernel has listed (none for most clouds: the workgroups then read the count and leave).
constexpr int BS_REST_WG = 2048;
template <typename KeyT, bool UNIQUE>
__global__ __launch_bounds__(BS_THREADS) void bs_rank_rest_kernel(const int32_t* __restrict__ rest_count,
                                                                  const int32_t* __restrict__ rest,
                                                                  const KeyT* __restrict__ keys1, const int32_t* __restrict__ vals1,
                                                                  const int2* __restrict__ win, int n_h,
                                                                  const int32_t* __restrict__ n_d, KeyT* __restrict__ out_k,
                                                                  int32_t* __restrict__ out_v, uint32_t* __restrict__ bits,
                                                                  int32_t* __restrict__ ccnt) {
  constexpr int PER = BS_LP / BS_PART;  // 64-position parts per listed workgroup
  const int n = n_d ? *n_d : n_h;
  const int todo = *rest_count * PER;
  for (int i = blockIdx.x; i < todo; i += gridDim.x) {
    const int part = rest[i / PER] * PER + i % PER;
    if (part * BS_PART >= n) continue;  // (uniform)
    if constexpr (UNIQUE) bs_rank_unique_part<KeyT, true>(part, keys1, win, n, out_k, bits, ccnt);
    else bs_rank_part<KeyT, BS_THREADS / 64, true>(part, keys1, vals1, win, n, out_k, out_v);
    __syncthreads();  // the part functions' LDS is reused by the next part
  }
}

// ---------------------------------------------------------------- small levels: one workgroup, one launch
// Fewer than BS_MIN_N keys (the tiny cloud of a unit test, the coarsest levels of a network): the partitioning
// scheme of the large path inside one workgroup and LDS.  The keys are produced (packed or masked) straight into
// LDS and counted into 1024 bins of their top used bits; a scan gives the bin starts; the keys move, with their source
// index, to their bin's range; and every key's final place is its bin's start plus the number of (key, index)
// pairs of the bin that sort before it (the index breaks ties, so equal keys of an invalid cloud still get distinct
// places).  The downsampling form writes the sorted keys back to LDS and keeps the first key of every run of equal
// keys (a scan over the head flags).  One launch of a few microseconds where the large path has four (five) and a
// library sort more; nothing but kernels is enqueued, so it can be recorded into a graph.  Work is quadratic in the
// bin sizes: a cloud whose keys all share their top 10 used bits costs n^2 = 16 M comparisons at most.
constexpr int BS_SMALL_THREADS = 1024;
constexpr int BS_SMALL_BIN_BITS = 10;
constexpr int BS_SMALL_BINS = 1 << BS_SMALL_BIN_BITS;
static_assert(BS_SMALL_BINS <= BS_SMALL_THREADS && BS_SMALL_BINS % 64 == 0, "one thread clears a bin; wave 0 scans whole groups");
constexpr int BS_SMALL_MAX = 4096;  // >= BS_MIN_N - 1
template <typename KeyT, typename Src, bool DEDUP>
__global__ __launch_bounds__(BS_SMALL_THREADS) void bs_small_sort_kernel(Src src, int n, int shift, KeyT* __restrict__ out_k,
                                                                        int32_t* __restrict__ out_v, int32_t* __restrict__ n_out) {
  __shared__ KeyT sk0[BS_SMALL_MAX], sk1[BS_SMALL_MAX];
  __shared__ int16_t sv1[BS_SMALL_MAX];
  __shared__ int s_start[BS_SMALL_BINS + 1], s_cur[BS_SMALL_BINS];
  __shared__ int wave_tot[BS_SMALL_THREADS / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < BS_SMALL_BINS) s_cur[tid] = 0;
  __syncthreads();
  bool bad = false;
  for (int i = tid; i < n; i += BS_SMALL_THREADS) {
    bool bad_i = false;
    const KeyT key = src.key(src.load(i), bad_i);
    bad |= bad_i;
    sk0[i] = key;
    atomicAdd(&s_cur[bs_bin(key, shift, BS_SMALL_BINS)], 1);
  }
  src.report(bad);
  __syncthreads();
  if (wave == 0) {  // exclusive scan of the bin counts, PL consecutive bins per lane
    constexpr int PL = BS_SMALL_BINS / 64;
    int c[PL], sum = 0;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      c[u] = s_cur[lane * PL + u];
      sum += c[u];
    }
    int x = sum;
    for (int d = 1; d < 64; d <<= 1) {
      const int y = __shfl_up(x, d, 64);
      if (lane >= d) x += y;
    }
    int run = x - sum;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      s_start[lane * PL + u] = run;
      s_cur[lane * PL + u] = run;
      run += c[u];
    }
    if (lane == 63) s_start[BS_SMALL_BINS] = run;
  }
  __syncthreads();
  for (int i = tid; i < n; i += BS_SMALL_THREADS) {
    const KeyT key = sk0[i];
    const int p = atomicAdd(&s_cur[bs_bin(key, shift, BS_SMALL_BINS)], 1);
    sk1[p] = key;
    sv1[p] = static_cast<int16_t>(i);
  }
  __syncthreads();
  for (int x = tid; x < n; x += BS_SMALL_THREADS) {
    const KeyT key = sk1[x];
    const int vi = sv1[x];
    const int b = bs_bin(key, shift, BS_SMALL_BINS);
    const int a = s_start[b], e = s_start[b + 1];
    int r = a;
    int y = a;
    // eight candidates per trip, read before any is compared: one LDS round trip per trip instead of one per key
    // (a bin of the tiny test cloud holds a few hundred keys, and the loop was nine tenths of the kernel)
    for (; y + 8 <= e; y += 8) {
      KeyT ky[8];
      int16_t vy[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        ky[u] = sk1[y + u];
        vy[u] = sv1[y + u];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) r += (ky[u] < key || (ky[u] == key && vy[u] < vi)) ? 1 : 0;
    }
    for (; y < e; ++y) {
      const KeyT ky = sk1[y];
      r += (ky < key || (ky == key && sv1[y] < vi)) ? 1 : 0;
    }
    if (DEDUP) {
      sk0[r] = key;  // sorted sequence, kept in LDS for the pass below
    } else {
      out_k[r] = key;
      if (out_v) out_v[r] = vi;
    }
  }
  if (!DEDUP) return;
  __syncthreads();
  // distinct keys: thread t owns the run of positions [t * per, (t + 1) * per)
  const int per = (n + BS_SMALL_THREADS - 1) / BS_SMALL_THREADS;
  int cnt = 0;
  for (int u = 0; u < per; ++u) {
    const int i = tid * per + u;
    cnt += (i < n && (i == 0 || sk0[i] != sk0[i - 1])) ? 1 : 0;
  }
  int x = cnt;
  for (int d = 1; d < 64; d <<= 1) {
    const int y = __shfl_up(x, d, 64);
    if (lane >= d) x += y;
  }
  if (lane == 63) wave_tot[wave] = x;
  __syncthreads();
  int base = x - cnt, total = 0;
  for (int w = 0; w < BS_SMALL_THREADS / 64; ++w) {
    if (w < wave) base += wave_tot[w];
    total += wave_tot[w];
  }
  for (int u = 0; u < per; ++u) {
    const int i = tid * per + u;
    if (i < n && (i == 0 || sk0[i] != sk0[i - 1])) out_k[base++] = sk0[i];
  }
  if (tid == 0) *n_out = total;
}

template <typename KeyT, typename Src, bool DEDUP>
static void launch_small_sort(const Src& src, int64_t n, int used_bits, void* out_k, int32_t* out_v, int32_t* n_out, hipStream_t s) {
  static_assert(BS_SMALL_MAX >= BS_MIN_N - 1, "the small path covers every size below the partitioning sort's");
  const int shift = std::max(0, used_bits - BS_SMALL_BIN_BITS);  // bins = the top used key bits
  hipLaunchKernelGGL((bs_small_sort_kernel<KeyT, Src, DEDUP>), dim3(1), dim3(BS_SMALL_THREADS), 0, s, src, static_cast<int>(n), shift,
                     static_cast<KeyT*>(out_k), out_v, n_out);
}

int small_pack_sort(int key_bits, const int4* coords, int64_t n, const PackParams& pp, int used_bits, int32_t* status, void* keys_out,
                    int32_t* perm_out, hipStream_t s) {
  if (key_bits == 32)
    launch_small_sort<uint32_t, SrcPack<uint32_t>, false>(SrcPack<uint32_t>{coords, pp, status}, n, used_bits, keys_out, perm_out, nullptr, s);
  else
    launch_small_sort<uint64_t, SrcPack<uint64_t>, false>(SrcPack<uint64_t>{coords, pp, status}, n, used_bits, keys_out, perm_out, nullptr, s);
  if (hipGetLastError() != hipSuccess) return set_error(SPC_ERR_HIP, "sort launch failed");
  return SPC_OK;
}

int small_mask_unique(int key_bits, const void* keys_in, int64_t n, uint64_t mask, int used_bits, void* keys_out, int32_t* n_out,
                      hipStream_t s) {
  if (key_bits == 32)
    launch_small_sort<uint32_t, SrcMask<uint32_t>, true>(SrcMask<uint32_t>{static_cast<const uint32_t*>(keys_in), static_cast<uint32_t>(mask)}, n,
                                                         used_bits, keys_out, nullptr, n_out, s);
  else
    launch_small_sort<uint64_t, SrcMask<uint64_t>, true>(SrcMask<uint64_t>{static_cast<const uint64_t*>(keys_in), mask}, n, used_bits,
                                                         keys_out, nullptr, n_out, s);
  if (hipGetLastError() != hipSuccess) return set_error(SPC_ERR_HIP, "downsample launch failed");
  return SPC_OK;
}

// ---------------------------------------------------------------- host
BucketPlan bucket_plan(int64_t n, int used_bits) {
  BucketPlan p{};
  int n_wg = static_cast<int>(std::min<int64_t>(std::max<int64_t>((n + 4095) / 4096, 1), BS_MAX_WG));
  p.per = static_cast<int>(((n + n_wg - 1) / n_wg + BS_WIDE - 1) / BS_WIDE * BS_WIDE);
  p.n_wg = static_cast<int>(std::max<int64_t>((n + p.per - 1) / p.per, 1));
  // About 16 keys per bin of the key space up to 4096 bins: packing descriptors round every field up
  // to whole bits and scenes are far from cubic, so typically a quarter of the bins is populated.
  // Beyond that, more bins only pay once the rank pass is bound by its comparisons and not by its
  // launch: 8192 bins from 200 k keys, 16384 from 512 k (10^6 keys: rank 51 -> 32 us; 300 k keys
  // with 16384 bins: slower by 2 us for the longer scans).
  int fb = 8;
  while (fb < 12 && (int64_t(16) << fb) < n) ++fb;
  if (n > 200000) fb = 13;
  if (n > 524288) fb = 14;
  static_assert(BS_MAX_BIN_BITS >= 14, "bin table sizes");
  fb = std::max(2, std::min(fb, used_bits));
  p.shift = used_bits - fb;
  p.n_bin = 1 << fb;
  return p;
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
  int2* win;
  int32_t* n_kept;
  int32_t* ccnt;
  uint32_t* bits;
  int32_t* rest_count;  // workgroups of bs_rank_lds_kernel whose window did not fit, and their numbers
  int32_t* rest;
  int n_words, n_chunks;
};
size_t words_for(int64_t n) { return static_cast<size_t>(n / 32 + 64); }    // bitmap words the downsampling path clears and reads
size_t chunks_for(int64_t n) { return static_cast<size_t>(n / BS_CHUNK + 2); }
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
  const BucketPlan cap = bucket_plan(n, 64);  // as many workgroups and at least as many bins as any plan for n keys
  const size_t tbl = (size_t(cap.n_wg) * cap.n_bin + 63) / 64 * 64;
  w.before = w.table + tbl;
  w.fstart = w.before + tbl;
  w.win = reinterpret_cast<int2*>(w.fstart + cap.n_bin + 64);  // 8-byte aligned: every part above is a multiple of 256 bytes
  w.n_kept = reinterpret_cast<int32_t*>(w.win + (nn / BS_PART + 2));
  w.ccnt = w.n_kept + 2;
  w.n_chunks = static_cast<int>(chunks_for(n));
  w.bits = reinterpret_cast<uint32_t*>(w.ccnt + w.n_chunks);
  w.n_words = static_cast<int>(words_for(n));
  w.rest_count = w.n_kept + 1;
  w.rest = reinterpret_cast<int32_t*>(w.bits + w.n_words);
  return w;
}

// count, column scan, scatter: keys1 (vals1) partitioned by fine bin, rank windows
template <typename KeyT, bool DEDUP, typename Src>
void partition(const Src& src, int64_t n, const BucketPlan& p, const Ws<KeyT>& w, hipStream_t s) {
  hipLaunchKernelGGL((bs_count_kernel<KeyT, Src>), dim3(p.n_wg), dim3(BS_WIDE), size_t(p.n_bin) * 4, s, src, n, p.per, p.shift,
                     p.n_bin, w.keys0, w.table);
  const int col_wg = (p.n_bin / 4 + BS_COL_THREADS - 1) / BS_COL_THREADS;
  hipLaunchKernelGGL(bs_colscan_kernel, dim3(col_wg), dim3(BS_COL_THREADS), 0, s, w.table, w.before, p.n_wg, p.n_bin, w.fstart);
  // (the scatter pass holds two ints per bin: beyond 8191 bins that is more than the default LDS limit)
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bs_scatter_kernel<KeyT, DEDUP>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (2 * BS_MAX_BIN + 2) * 4);
  (void)attr;
  hipLaunchKernelGGL((bs_scatter_kernel<KeyT, DEDUP>), dim3(p.n_wg), dim3(BS_WIDE), size_t(2 * p.n_bin + 2) * 4, s, w.keys0, n, p.per,
                     p.shift, p.n_bin, w.before,
                     w.fstart, w.keys1, w.vals1, w.win, DEDUP ? w.n_kept : static_cast<int32_t*>(nullptr), w.bits, w.n_words, w.ccnt,
                     w.n_chunks, w.rest_count);
}
}  // namespace

size_t bucket_sort_ws_bytes(int key_bits, int64_t n) {
  const size_t nn = static_cast<size_t>(std::max<int64_t>(n, 1));
  const size_t k = ((nn + BS_PAD_KEYS) * (key_bits / 8) + 255) / 256 * 256, v = (nn * 4 + 255) / 256 * 256;
  const BucketPlan cap = bucket_plan(n, 64);
  const size_t tbl = (size_t(cap.n_wg) * cap.n_bin + 63) / 64 * 64;
  return 2 * k + v + (2 * tbl + cap.n_bin + 64 + 2 * (nn / BS_PART + 2) + 2 + chunks_for(n) + words_for(n) + (nn / BS_LP + 2)) * 4;
}

template <typename KeyT>
static int pack_sort_t(const int4* coords, int64_t n, const PackParams& pp, int used_bits, int32_t* status, void* keys_out,
                       int32_t* perm_out, void* ws, hipStream_t s) {
  const BucketPlan p = bucket_plan(n, used_bits);
  const Ws<KeyT> w = carve<KeyT>(ws, n);
  partition<KeyT, false>(SrcPack<KeyT>{coords, pp, status}, n, p, w, s);
  const int n_part = static_cast<int>((n + BS_PART - 1) / BS_PART);
  // Four waves share a part's window while the launch is latency-bound (its time is that of the part with
  // the largest window); from BS_RANK_SOLO_N keys on (25 parts per CU) the pass is bound by how many parts
  // a CU has in flight, and one wave per part (no LDS, no barrier, four times the parts per CU) is
  // faster: 10^6 keys 32 -> 26 us, 2 * 10^6 keys 145 -> 129 us for the whole sort; at 240 k keys of
  // dense indoor scenes it was slower (37 -> 47 us).
  if (n >= BS_RANK_LDS_N) {
    hipLaunchKernelGGL((bs_rank_lds_kernel<KeyT, false>), dim3(static_cast<int>((n + BS_LP - 1) / BS_LP)), dim3(BS_LT), 0, s, w.keys1,
                       w.vals1, w.win, static_cast<int>(n), static_cast<const int32_t*>(nullptr), p.shift, p.n_bin,
                       static_cast<KeyT*>(keys_out), perm_out, static_cast<uint32_t*>(nullptr), static_cast<int32_t*>(nullptr),
                       w.rest_count, w.rest);
    hipLaunchKernelGGL((bs_rank_rest_kernel<KeyT, false>), dim3(BS_REST_WG), dim3(BS_THREADS), 0, s, w.rest_count, w.rest, w.keys1,
                       w.vals1, w.win, static_cast<int>(n), static_cast<const int32_t*>(nullptr), static_cast<KeyT*>(keys_out),
                       perm_out, static_cast<uint32_t*>(nullptr), static_cast<int32_t*>(nullptr));
  } else if (n >= BS_RANK_SOLO_N)
    hipLaunchKernelGGL((bs_rank_kernel<KeyT, 1>), dim3(n_part), dim3(64), 0, s, w.keys1, w.vals1, w.win, static_cast<int>(n),
                       static_cast<KeyT*>(keys_out), perm_out);
  else
    hipLaunchKernelGGL((bs_rank_kernel<KeyT, BS_THREADS / 64>), dim3(n_part), dim3(BS_THREADS), 0, s, w.keys1, w.vals1, w.win,
                       static_cast<int>(n), static_cast<KeyT*>(keys_out), perm_out);
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
  // the sorted keys (with gaps) go to keys0, which is free again by now
  const int n_part = static_cast<int>((n + BS_PART - 1) / BS_PART), n_chunk = static_cast<int>((n + BS_CHUNK - 1) / BS_CHUNK);
  if (n >= BS_RANK_LDS_N) {
    hipLaunchKernelGGL((bs_rank_lds_kernel<KeyT, true>), dim3(static_cast<int>((n + BS_LP - 1) / BS_LP)), dim3(BS_LT), 0, s, w.keys1,
                       static_cast<const int32_t*>(nullptr), w.win, static_cast<int>(n), w.n_kept, p.shift, p.n_bin, w.keys0,
                       static_cast<int32_t*>(nullptr), w.bits, w.ccnt, w.rest_count, w.rest);
    hipLaunchKernelGGL((bs_rank_rest_kernel<KeyT, true>), dim3(BS_REST_WG), dim3(BS_THREADS), 0, s, w.rest_count, w.rest, w.keys1,
                       static_cast<const int32_t*>(nullptr), w.win, static_cast<int>(n), w.n_kept, w.keys0,
                       static_cast<int32_t*>(nullptr), w.bits, w.ccnt);
  } else
    hipLaunchKernelGGL(bs_rank_unique_kernel<KeyT>, dim3(n_part), dim3(BS_THREADS), 0, s, w.keys1, w.win, w.n_kept, w.keys0, w.bits,
                       w.ccnt);
  hipLaunchKernelGGL(bs_compact_kernel<KeyT>, dim3(n_chunk), dim3(BS_THREADS), 0, s, w.keys0, w.bits, w.ccnt, w.n_kept,
                     static_cast<KeyT*>(keys_out), n_out);
  if (hipGetLastError() != hipSuccess) return set_error(SPC_ERR_HIP, "downsample launch failed");
  return SPC_OK;
}

int bucket_mask_unique(int key_bits, const void* keys_in, int64_t n, uint64_t mask, int used_bits, void* keys_out,
                       int32_t* n_out, void* ws, hipStream_t s) {
  return key_bits == 32 ? mask_unique_t<uint32_t>(keys_in, n, mask, used_bits, keys_out, n_out, ws, s)
                        : mask_unique_t<uint64_t>(keys_in, n, mask, used_bits, keys_out, n_out, ws, s);
}

}  // namespace spc
