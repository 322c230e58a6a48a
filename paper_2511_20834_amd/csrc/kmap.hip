// Kernel-map construction: the one-shot search over sorted packed keys
// (Sections 5.2-5.3), the output-stationary |V_q| x K^3 layout, the filtered
// weight-stationary lists (Section 5.4, cases I and II) and the network-wide
// builder (Section 5.5).
//
// What is kept from the paper: no query structure is built; offsets are split into
// K^2 groups that share (dx,dy); only the smallest-z query of a group is searched and
// the other K-1 are resolved on consecutive positions; queries are formed by adding a
// packed offset to a packed key.
// What is different (CDNA4): a workgroup owns a contiguous tile of sorted output
// voxels.  Because adding a constant keeps the order, all queries of a tile and group
// fall into one contiguous window of the input array.  The 2 K^2 window bounds are found
// by groups of lanes, 16-ary (4-ary for K >= 5), the first rounds on 256 probes shared by all
// searches in LDS (one or two dependent loads for 2^18 keys instead of 18), the
// windows are copied into LDS with coalesced loads, and every lane then searches in LDS
// with the window state in scalar registers (the kernel is bound by instruction issue).
// Windows that do not fit the LDS budget are searched in global memory, restricted to
// the window, with the same code.
#include <algorithm>
#include <map>
#include <set>
#include <tuple>

#include "spc_internal.h"

namespace spc {

constexpr int SEARCH_THREADS = 256;       // 128 and 512 measured slower at every level size (10^5 .. 3 * 10^6 voxels)
constexpr int WIN_CAP_BYTES = 20 * 1024;  // LDS budget for staged windows per workgroup (several workgroups share a CU)
constexpr int N_PROBES = 256;             // first-round probes of the window-bound searches (a power of 4 and of 16)
constexpr int MAX_K = 7;
constexpr int WS_MAX_K3_SEARCH = MAX_K * MAX_K * MAX_K;

template <typename KeyT>
struct SearchParams {
  KeyT X0, dX;    // packed x offset of ix = 0 and its step per ix (wrapping arithmetic: the offsets of an axis are
  KeyT Y0, dY;    // an arithmetic sequence); the same for y
  KeyT zmin;      // packed smallest z offset
  KeyT zstep;     // distance between consecutive z offsets (= input stride)
  int zrev;       // 1: z offsets descend with iz (transposed maps)
  unsigned long long need;  // bit g: group g = ix * K + iy has an offset in one of the two subsets
};

__device__ inline int lanemask_lt_popc(unsigned long long m) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(m >> 32), __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(m), 0));
}

// Window-bound searches over keys[0,n): groups of P lanes run one search each (64/P searches per wave
// instruction), U passes of them interleaved so that the loads of all passes are in flight together.
// upper=false: first index with key >= q; true: first index with key > q.  q and upper are the same
// in all lanes of a group, and odd groups search upper bounds.  The first rounds need no memory
// access: every search starts from the same N_PROBES probes (the last key of every 1/N_PROBES slice, loaded
// once per workgroup into LDS), searched P-ary by the group's lanes with a ballot per round.  From then on
// lane p of a group probes the last key of the p-th of P sub-slices, and the group's bits of the ballot
// give the sub-slice.  The searches stop once every answer is known to within `slack` positions and return
// the outer ends (slack 0: exact bounds): a window that is a few keys too wide costs less than
// another round of dependent loads.  P = 16 reads 16 cache lines per search and round where a search
// by the whole wave read 64, for the same number of dependent rounds at these sizes (2^18 keys:
// 4096 -> 256 -> 16); with 25 groups of offsets the wave-wide form spent most of the kernel
// fetching probe lines.
template <typename KeyT>
__device__ inline KeyT lane_value(KeyT v, int src_lane) {
  if constexpr (sizeof(KeyT) == 4) {
    return static_cast<KeyT>(__builtin_amdgcn_readlane(static_cast<int>(v), src_lane));
  } else {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v)), src_lane);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v >> 32)), src_lane);
    return (static_cast<KeyT>(hi) << 32) | lo;
  }
}

template <typename KeyT, int P, int U>
__device__ inline void group_bounds(const KeyT* __restrict__ keys, int n, const KeyT* s_probe, const KeyT (&q)[U], int (&res)[U],
                                    int slack) {
  constexpr int Q = 64 / P;
  static_assert(Q % 2 == 0, "odd groups search upper bounds");
  const int lane = threadIdx.x & 63, grp = lane / P, p = lane % P;
  const bool upper = (grp & 1) != 0;
  const int chunk0 = (n + N_PROBES - 1) / N_PROBES;
  int lo[U], hi[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    // number of probes before the answer, P-ary in LDS (probe j is the last key of slice j; slices past the
    // end of the array hold no probe and count as "not before")
    int base = 0;
    bool all = false;
#pragma unroll
    for (int sub = N_PROBES / P; sub >= 1; sub /= P) {
      const int j = base + (p + 1) * sub - 1;
      const KeyT pv = s_probe[j];
      const bool pr = (long long)j * chunk0 < n && (upper ? (pv <= q[u]) : (pv < q[u]));
      const int c = __popcll((__ballot(pr) >> (grp * P)) & ((1ull << P) - 1));
      if (sub == N_PROBES / P && c == P) all = true;  // only the first round can find every probe before the answer
      base += (c == P ? P - 1 : c) * sub;  // (when all are before, the value of base no longer matters)
    }
    const int c = all ? N_PROBES : base;
    if ((long long)c * chunk0 >= n) {  // every slice lies before the answer (or there are no keys)
      lo[u] = n;
      hi[u] = n;
    } else {
      lo[u] = c * chunk0;
      hi[u] = min(lo[u] + chunk0 - 1, n - 1);
    }
  }
  auto unfinished = [&]() {
    int maxlen = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) maxlen = max(maxlen, hi[u] - lo[u]);
    return __ballot(maxlen > slack) != 0;
  };
  while (unfinished()) {  // every round shortens every unfinished search
    bool pred[U];
    int chunk[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int len = hi[u] - lo[u];
      chunk[u] = (len + P - 1) / P;
      const long long first = (long long)lo[u] + (long long)p * chunk[u];
      // clamped, unconditional load: the loads of all passes are issued back to back
      const long long idx = max(0ll, min(min(first + chunk[u] - 1, (long long)hi[u] - 1), (long long)n - 1));
      const KeyT v = keys[idx];
      pred[u] = len > 0 && first < hi[u] && (upper ? (v <= q[u]) : (v < q[u]));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int len = hi[u] - lo[u];
      const unsigned long long bal = __ballot(pred[u]);
      if (len > 0) {
        const int c = __popcll((bal >> (grp * P)) & ((1ull << P) - 1));
        const int nlo = lo[u] + c * chunk[u];
        if (c * chunk[u] >= len) {  // every sub-slice lies before the answer
          lo[u] = hi[u];
        } else {
          hi[u] = min(nlo + chunk[u] - 1, hi[u] - 1);
          lo[u] = nlo;
        }
      }
    }
  }
  // the answer lies in [lo, hi]: the low end for a window start, the high end for a window end
#pragma unroll
  for (int u = 0; u < U; ++u) res[u] = upper ? hi[u] : lo[u];
}

// Per-lane lower bound in a window of wsz keys (used for windows that stay in global memory).
template <typename KeyT, typename Ptr>
__device__ inline int lane_lower_bound(Ptr win, int wsz, KeyT q) {
  int lo = 0, len = wsz;
  while (len > 0) {
    const int half = len >> 1;
    const bool less = win[lo + half] < q;
    lo = less ? lo + half + 1 : lo;
    len = less ? len - half - 1 : half;
  }
  return lo;
}

// Groups whose LDS searches one lane keeps in flight together.  K <= 3: five (one lane's share of the nine groups
// in one go; 44 registers with 32-bit keys, 64 with 64-bit keys).  Larger kernels: four (three and five measured
// within 5 % on 240 k voxels, 5x5x5).
constexpr int SEARCH_GB_SMALL = 5, SEARCH_GB_LARGE = 4;
// Whether some part p < parts has `rem` groups left after whole batches of gb (its groups are p, p + parts, ... < G).
__host__ __device__ constexpr bool remainder_occurs(int G, int parts, int gb, int rem) {
  for (int p = 0; p < parts && p < G; ++p)
    if (((G - p + parts - 1) / parts) % gb == rem) return true;
  return false;
}
// Output voxels per search workgroup (a multiple of the wave size that divides SEARCH_THREADS).  Every tile pays for
// its window bounds, their placement and the staging, so longer tiles do less work per voxel, and shorter ones
// spread a small level over more compute units: 3x3x3, 128 -> 256 rows: 3 * 10^6 voxels 162 -> 140 us,
// 10^6 60 -> 56 us, 120 k 16.8 -> 21 us; 5x5x5, 64 -> 128 rows: 240 k voxels 65 -> 62 us.
constexpr int64_t SEARCH_LONG_TILE_FROM = 750000;  // output voxels from which K <= 3 takes 256-row tiles
inline int search_tile(int K, int64_t n_out) { return K <= 3 ? (n_out >= SEARCH_LONG_TILE_FROM ? 256 : 128) : K <= 5 ? 128 : 64; }

// Two outputs, each for its own subset of the K^3 offsets (Section 5.4: all offsets in one of them for a single
// dataflow; the dense offsets in the matrix and the sparse ones in the lists for the hybrid dual dataflow):
//   os_k: columns of the blocked |V_q| x K^3 matrix M and bits of the per-block offset masks (M = NULL: none);
//   ws_k: (PAIRS = true) weight-stationary lists.  They never pass through a matrix: a tile keeps, per (group,
//         row), the position of its lower bound and the hit bits of the group's K queries in LDS (5 bytes where
//         the matrix has 4 K), and once all groups are searched it writes the hits of the ws_k offsets as
//         compacted (in, out) pairs, offset-major and row-ascending, into its own slab of `tile_pairs` (slab =
//         tile * K^3 pairs, of which only the first sum-of-hits are touched); tile_counts gets the hits per
//         (offset, tile).
// Groups none of whose offsets is wanted are not searched (the second half of a symmetric map, for example).
template <typename KeyT, int K, int TILE, bool PAIRS>
__global__ __launch_bounds__(SEARCH_THREADS) void kmap_search_kernel(
    const KeyT* __restrict__ in_keys, int n_in_h, const int* __restrict__ n_in_d, const KeyT* __restrict__ out_keys,
    int n_out_h, const int* __restrict__ n_out_d, SearchParams<KeyT> sp, int32_t* __restrict__ M,
    uint32_t* __restrict__ block_masks, int32_t* __restrict__ tile_counts, int n_tiles_cap,
    const int32_t* __restrict__ in_perm, KMask os_k, KMask ws_k, int2* __restrict__ tile_pairs,
    int32_t* __restrict__ inv_parent) {
  constexpr int G = K * K, K3 = K * K * K;
  constexpr int tile = TILE;
  constexpr int SEARCH_GB = K <= 3 ? SEARCH_GB_SMALL : SEARCH_GB_LARGE;
  constexpr int MW = (K3 + 31) / 32;   // mask words per 32-row block
  constexpr int MAX_BLOCKS = TILE / 32;
  constexpr int WIN_CAP = WIN_CAP_BYTES / sizeof(KeyT);
  constexpr int NW = SEARCH_THREADS / 64;
  // lanes per window-bound search: with many groups of offsets the probe lines fetched count for more than the
  // number of dependent rounds (240 k voxels, 5x5x5: 16 lanes 98.6 us, 8 lanes 94.6, 4 lanes 92.2)
  constexpr int BOUND_P = G <= 9 ? 16 : 4;
  constexpr int BOUND_SLACK = G <= 9 ? 32 : 16;  // extra keys per window end: 2 * G * slack must stay small next to WIN_CAP
  extern __shared__ __align__(16) unsigned char smem[];
  KeyT* okeys = reinterpret_cast<KeyT*>(smem);   // [tile]
  KeyT* win = okeys + tile;                      // [WIN_CAP + MAX_K]: staged windows, and room for reads behind the last one
  int32_t* s_pos = reinterpret_cast<int32_t*>(win + WIN_CAP + MAX_K);       // PAIRS: [G][tile] input position of the group's lower bound
  uint8_t* s_hit = reinterpret_cast<uint8_t*>(s_pos + G * tile);      // PAIRS: [G][tile] bit t: the group's t-th query (ascending z) hit
  __shared__ int s_off[PAIRS ? K3 + 1 : 1];                           // PAIRS: where every offset's pairs start in the tile's slab
  __shared__ KeyT s_probe[N_PROBES];
  __shared__ int4 s_grp[G];  // window of group g: x = first input position, y = keys, z = place in `win` (-1: not staged)
  __shared__ int s_bound[2 * G];
  __shared__ int s_cnt[K3];
  __shared__ unsigned s_mask[MAX_BLOCKS * MW];
  __shared__ KeyT s_gd[G];  // packed (dx,dy,zmin) offset of every group

  const int n_in = n_in_d ? *n_in_d : n_in_h;
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  const int i0 = blockIdx.x * tile;
  if (i0 >= n_out) return;  // whole workgroup leaves together
  const int rows = min(tile, n_out - i0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // first-round probes of the window-bound searches (the same N_PROBES keys for everybody: L2-resident)
  {
    const int chunk0 = (n_in + N_PROBES - 1) / N_PROBES;
    for (int j = tid; j < N_PROBES; j += SEARCH_THREADS)
      s_probe[j] = (n_in > 0 && (long long)j * chunk0 < n_in) ? in_keys[min((long long)(j + 1) * chunk0 - 1, (long long)n_in - 1)] : KeyT(0);
  }

  for (int v = tid; v < rows; v += SEARCH_THREADS) okeys[v] = out_keys[i0 + v];
  for (int k = tid; k < K3; k += SEARCH_THREADS) s_cnt[k] = 0;
  for (int k = tid; k < MAX_BLOCKS * MW; k += SEARCH_THREADS) s_mask[k] = 0u;
  for (int k = tid; k < 2 * G; k += SEARCH_THREADS) s_bound[k] = 0;
  if (tid < G) s_gd[tid] = sp.X0 + KeyT(tid / K) * sp.dX + sp.Y0 + KeyT(tid % K) * sp.dY + sp.zmin;
  __syncthreads();
  const KeyT kfirst = okeys[0], klast = okeys[rows - 1];
  const KeyT zspan = KeyT(K - 1) * sp.zstep;

  // ---- window bounds: search s = 2*g + side; pass u of wave w runs searches (u*NW + w)*Q .. +Q-1, one per group
  // of BOUND_P lanes (searches past the last one repeat it and are not recorded)
  {
    constexpr int Q = 64 / BOUND_P;
    constexpr int U = (2 * G + NW * Q - 1) / (NW * Q);
    const int grp = lane / BOUND_P;
    auto run_bounds = [&](auto U_) {
      constexpr int UU = decltype(U_)::value;
      KeyT q[UU];
      int res[UU];
#pragma unroll
      for (int u = 0; u < UU; ++u) {
        const int sc = min((u * NW + wave) * Q + grp, 2 * G - 1);
        const KeyT d = s_gd[sc >> 1];
        q[u] = (grp & 1) ? KeyT(klast + d + zspan) : KeyT(kfirst + d);
      }
      group_bounds<KeyT, BOUND_P, UU>(in_keys, n_in, s_probe, q, res, BOUND_SLACK);
#pragma unroll
      for (int u = 0; u < UU; ++u) {
        const int sc = (u * NW + wave) * Q + grp;
        // only groups with a wanted offset are searched: the others keep empty windows
        if (lane % BOUND_P == 0 && sc < 2 * G && ((sp.need >> (sc >> 1)) & 1ull)) s_bound[sc] = res[u];
      }
    };
    // the last pass is short of searches: only the waves that have one there run it
    if (U == 1 || ((U - 1) * NW + wave) * Q < 2 * G) run_bounds(std::integral_constant<int, U>{});
    else run_bounds(std::integral_constant<int, (U > 1 ? U - 1 : 1)>{});
  }
  __syncthreads();

  // ---- window placement in LDS: a prefix sum over the groups by wave 0; groups whose window
  // ends beyond the LDS budget stay in global memory
  if (wave == 0) {
    const int lo = lane < G ? s_bound[2 * lane] : 0;
    const int sz = lane < G ? max(0, s_bound[2 * lane + 1] - lo) : 0;
    int incl = sz;
    for (int d = 1; d < 64; d <<= 1) {
      const int y = __shfl_up(incl, d, 64);
      if (lane >= d) incl += y;
    }
    if (lane < G) s_grp[lane] = make_int4(lo, sz, incl <= WIN_CAP ? incl - sz : -1, 0);
  }
  __syncthreads();

  // ---- staging, window after window.  A team of lanes copies a window, lane e its keys e, e + team size, ...:
  // the whole workgroup for the long windows of 128-row tiles, a wave for the short ones of 64-row tiles (with
  // 25 or 49 groups a workgroup-wide copy would leave three lanes in four idle), the waves then taking different
  // groups.  Window positions and sizes are read into scalar registers, so a copy costs a compare and two
  // address additions per lane, and the loads of all of a team's windows are in flight together.
  {
    constexpr int TEAM = tile >= 128 ? SEARCH_THREADS : 64;  // lanes per window
    const __amdgpu_buffer_rsrc_t keys_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<KeyT*>(in_keys), 0, sizeof(KeyT) == 4 ? n_in * 4 : 0, 0x00020000);
    constexpr int N_TEAMS = SEARCH_THREADS / TEAM;
    constexpr int STAGE_U = (G + N_TEAMS - 1) / N_TEAMS;       // windows per team
    const int team = __builtin_amdgcn_readfirstlane(tid / TEAM), lt = tid % TEAM;
    KeyT tmp[STAGE_U];
    int woff[STAGE_U], wsz[STAGE_U], wlo[STAGE_U];
    int longest = 0;
#pragma unroll
    for (int i = 0; i < STAGE_U; ++i) {
      const int g = team + i * N_TEAMS;
      const int4 gw = s_grp[min(g, G - 1)];
      wlo[i] = __builtin_amdgcn_readfirstlane(gw.x);
      woff[i] = __builtin_amdgcn_readfirstlane(gw.z);
      wsz[i] = g < G && woff[i] >= 0 ? __builtin_amdgcn_readfirstlane(gw.y) : 0;
      longest = max(longest, wsz[i]);
      // (through a descriptor of the n_in keys: lanes past the window read a neighbouring key or, past the
      // array, zero; nothing of that is stored)
      if constexpr (sizeof(KeyT) == 4) {
        tmp[i] = __builtin_amdgcn_raw_buffer_load_b32(keys_rsrc, lt * 4, wlo[i] * 4, 0);
      } else {
        tmp[i] = 0;
        if (lt < wsz[i]) tmp[i] = (in_keys + wlo[i])[lt];
      }
    }
#pragma unroll
    for (int i = 0; i < STAGE_U; ++i)
      if (lt < wsz[i]) (win + woff[i])[lt] = tmp[i];
    if (longest > TEAM) {  // rare
#pragma unroll
      for (int i = 0; i < STAGE_U; ++i)
        for (int e = lt + TEAM; e < wsz[i]; e += TEAM) (win + woff[i])[e] = (in_keys + wlo[i])[e];
    }
  }
  __syncthreads();

  // ---- per-lane searches.  A wave holds 64 consecutive output voxels and takes NJ groups of offsets at a time,
  // their searches interleaved (independent LDS chains hide each other's latency).  The phase is bound by the
  // number of vector instructions, so everything that is the same for the 64 lanes lives in scalar registers:
  // a group's window (LDS position, size, position in the input array) and the remaining length n of its search.
  // A search keeps the LDS byte address `ab` of the key before its lower bound's current base; a round probes the
  // key half = ceil(n/2) further on and moves the base behind it when that key is smaller than the query, which
  // leaves floor(n/2) keys: one addition, one compare and one select per round, no bounds to check (a probe never
  // leaves the window; finished searches probe the key at `ab` again, which changes nothing).
  const int64_t b0 = int64_t(i0) >> 5;
  const int rows32 = (rows + 31) & ~31;
  constexpr int parts = SEARCH_THREADS / tile;     // threads per output voxel
  const int v = tid % tile;
  const int part = __builtin_amdgcn_readfirstlane(tid / tile);  // uniform in a wave (tile is a multiple of 64)
  const bool act = v < rows;
  const bool stored = v < rows32;                  // rows past the end of the last block hold -1
  const KeyT okey = okeys[min(v, rows - 1)];       // lanes past the end repeat the last row; their results are dropped
  const int v0 = __builtin_amdgcn_readfirstlane(v & ~63);
  const int bl0 = v0 >> 5;                         // the wave's two 32-row blocks: bl0, bl0 + 1
  int32_t* Mw = M + (b0 + bl0) * int64_t(K3) * 32;  // uniform; lane l writes at l%32 of block bl0 + l/32
  const unsigned lane_off = (unsigned(lane >> 5) * unsigned(K3 * 32) + unsigned(lane & 31)) * 4u;  // bytes
  // (pointers typed as LDS addresses: 32 bits wide, and every access through them is an LDS instruction)
  using LdsBytes = const __attribute__((address_space(3))) unsigned char*;
  using LdsKey = const __attribute__((address_space(3))) KeyT*;
  const LdsBytes lbase = (LdsBytes)smem;
  constexpr unsigned KB = sizeof(KeyT);
  unsigned hbits[MW];  // offsets this lane's row has hit, among those of the matrix (the block masks are their OR over 32 lanes)
#pragma unroll
  for (int w = 0; w < MW; ++w) hbits[w] = 0u;
  // subset tests on the kernel arguments: the word is picked with scalar selects (static indices keep the masks in
  // scalar registers), so a test costs no LDS access
  auto subset_word = [&](const KMask& m, int wd) {
    unsigned x = m.w[0];
#pragma unroll
    for (int i = 1; i < MW; ++i) x = wd == i ? m.w[i] : x;
    return x;
  };
  // the K bits of group g (offsets g*K .. g*K + K - 1) in a subset
  auto subset_field = [&](const KMask& m, int g) {
    const int wd = (g * K) >> 5, sh = (g * K) & 31;
    const unsigned long long two = (static_cast<unsigned long long>(wd + 1 < MW ? subset_word(m, wd + 1) : 0u) << 32) | subset_word(m, wd);
    return static_cast<unsigned>(two >> sh) & ((1u << K) - 1u);
  };
  // row numbers are fetched through a buffer descriptor of in_perm's n_in entries: the hardware returns 0 for
  // positions past the end (candidates behind the last key of the array), so no lane needs a bounds check
  const __amdgpu_buffer_rsrc_t perm_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(in_perm), 0, in_perm ? n_in * 4 : 0, 0x00020000);
  const int col0 = sp.zrev ? K - 1 : 0, cstep = sp.zrev ? -1 : 1;  // column of a group's query t: col0 + t * cstep
  auto search_groups = [&](auto NJ_, int gb) {
    constexpr int NJ = decltype(NJ_)::value;
    int g[NJ], wsz[NJ], wlo[NJ], n[NJ];
    bool glob[NJ];
    LdsBytes ab0[NJ], ab[NJ];
    KeyT q0[NJ];
    int nmax = 0;
    bool any_glob = false;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      g[j] = gb + j * parts;  // < G (the caller counts the groups)
      const int4 gw = s_grp[g[j]];  // (groups without a wanted offset have empty windows)
      wlo[j] = __builtin_amdgcn_readfirstlane(gw.x);
      wsz[j] = __builtin_amdgcn_readfirstlane(gw.y);
      const int woff = __builtin_amdgcn_readfirstlane(gw.z);
      glob[j] = woff < 0 && wsz[j] > 0;  // window kept in global memory
      any_glob |= glob[j];
      n[j] = woff >= 0 ? wsz[j] : 0;
      // LDS address of the key before the window: the output keys lie before the windows, so this is a valid
      // address for the first window too
      ab0[j] = lbase + (unsigned(tile) + unsigned(max(woff, 0))) * KB - KB;
      ab[j] = ab0[j];
      q0[j] = okey + s_gd[g[j]];
      nmax = max(nmax, n[j]);
    }
    for (int rounds = nmax > 0 ? 32 - __builtin_clz(nmax) : 0; rounds > 0; --rounds) {
      LdsBytes cand[NJ];
      KeyT kv[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int rest = n[j] >> 1, half = n[j] - rest;  // half = ceil(n / 2)
        n[j] = rest;
        cand[j] = ab[j] + unsigned(half) * KB;
        kv[j] = *(LdsKey)cand[j];
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j) ab[j] = kv[j] < q0[j] ? cand[j] : ab[j];
    }
    // the K keys from each lower bound on: the K z-consecutive queries of a group hit consecutive
    // positions (keys are sorted integers whose z components are multiples of the input stride,
    // Section 5.2).  Reads may run up to K - 1 keys past the window, into the next window or the padding
    // behind the last one; `rem` below says how many of them belong to the window.
    KeyT w[NJ][K];
    int pos[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
#pragma unroll
      for (int i = 0; i < K; ++i) w[j][i] = *(LdsKey)(ab[j] + (i + 1) * KB);
      pos[j] = static_cast<int>((ab[j] - ab0[j]) / KB);
    }
    if (any_glob) {  // windows that stayed in global memory (rare): per-lane lower bound, same K keys
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        if (glob[j]) {
          pos[j] = lane_lower_bound<KeyT>(in_keys + wlo[j], wsz[j], q0[j]);
#pragma unroll
          for (int i = 0; i < K; ++i) w[j][i] = in_keys[wlo[j] + min(pos[j] + i, wsz[j] - 1)];
        }
    }
    // what the map stores for position rpos + i: the position, or the caller's row number of that voxel.  The
    // row numbers of all NJ groups are requested before the first of them is used.
    int rpos[NJ];
    int32_t val[NJ][K];
    bool valid[NJ][K];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int rem = wsz[j] - pos[j];  // window keys from the lower bound on
      rpos[j] = wlo[j] + pos[j];        // the lower bound's position in the input array
#pragma unroll
      for (int i = 0; i < K; ++i) {
        valid[j][i] = act && i < rem;
        val[j][i] = rpos[j] + i;
      }
      if (in_perm) {
#pragma unroll
        for (int i = 0; i < K; ++i) val[j][i] = __builtin_amdgcn_raw_buffer_load_b32(perm_rsrc, rpos[j] * 4 + i * 4, 0, 0);
      }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      // query t (ascending z) sits i <= t positions behind the lower bound, i = number of earlier queries that hit
      KeyT d[K];
#pragma unroll
      for (int i = 0; i < K; ++i) d[i] = w[j][i] - q0[j];
      int32_t r[K];
      bool hit[K];
      unsigned hm = 0u;  // bit t: query t hit
#pragma unroll
      for (int t = 0; t < K; ++t) {
        r[t] = -1;
        hit[t] = false;
        const KeyT dt = KeyT(t) * sp.zstep;
#pragma unroll
        for (int i = 0; i <= t; ++i) {
          const bool m = valid[j][i] && d[i] == dt;
          r[t] = m ? val[j][i] : r[t];
          hit[t] = hit[t] || m;
        }
        if constexpr (PAIRS) hm |= hit[t] ? 1u << t : 0u;
      }
      const int gj = g[j];
      // column of query t: offsets of a group ascend with z, queries too unless the z offsets descend with iz
      auto col = [&](int t) { return col0 + t * cstep; };
      // inverse of a strided map whose offsets partition the inputs (K = layer stride): every input voxel is hit by
      // exactly one (output, offset), which is all its transposed twin needs (such maps are built without a
      // row permutation, so r holds positions)
      if (inv_parent) {
#pragma unroll
        for (int t = 0; t < K; ++t)
          if (hit[t]) inv_parent[r[t]] = (i0 + v) * K3 + gj * K + col(t);
      }
      if constexpr (PAIRS) {
        // the tile's records stay in LDS; hits are counted per offset (a wave speaks for its 64 rows)
        const unsigned wsf = subset_field(ws_k, gj);
        s_pos[gj * tile + v] = rpos[j];
        s_hit[gj * tile + v] = static_cast<uint8_t>(hm);
#pragma unroll
        for (int t = 0; t < K; ++t) {
          if (!((wsf >> col(t)) & 1u)) continue;
          const unsigned long long bal = __ballot(hit[t]);
          if (bal && lane == 0) atomicAdd(&s_cnt[gj * K + col(t)], __popcll(bal));
        }
      }
      if (!M) continue;  // no offset goes to the matrix (uniform over the launch)
      const unsigned osf = subset_field(os_k, gj);
      // Every store into the blocked map M[block][k][32] is two full 128-byte segments.
      if (stored) {
        char* Mb = reinterpret_cast<char*>(Mw);  // + a 32-bit offset: column k starts k * 128 bytes into the block
        if (osf == (1u << K) - 1u) {  // all of the group's offsets (the usual case)
#pragma unroll
          for (int t = 0; t < K; ++t) *reinterpret_cast<int32_t*>(Mb + (lane_off + unsigned(gj * K + col(t)) * 128u)) = r[t];
        } else {
#pragma unroll
          for (int t = 0; t < K; ++t)
            if ((osf >> col(t)) & 1u) *reinterpret_cast<int32_t*>(Mb + (lane_off + unsigned(gj * K + col(t)) * 128u)) = r[t];
        }
      }
      // the row's hits among the matrix offsets, as bits gj*K .. gj*K + K - 1 of the lane's mask words
      unsigned hc = 0u;
#pragma unroll
      for (int t = 0; t < K; ++t) hc |= hit[t] ? 1u << col(t) : 0u;
      const int wd = (gj * K) >> 5, sh = (gj * K) & 31;
      const unsigned long long f = static_cast<unsigned long long>(hc & osf) << sh;
#pragma unroll
      for (int w = 0; w < MW; ++w) hbits[w] |= (wd == w ? static_cast<unsigned>(f) : 0u) | (wd + 1 == w ? static_cast<unsigned>(f >> 32) : 0u);
    }
  };
  // the wave's groups: part, part + parts, ...; SEARCH_GB at a time, then the remainder
  {
    const int mine = part < G ? (G - part + parts - 1) / parts : 0;
    int done = 0;
    for (; done + SEARCH_GB <= mine; done += SEARCH_GB) search_groups(std::integral_constant<int, SEARCH_GB>{}, part + done * parts);
    const int left = mine - done;
    const int gb = part + done * parts;
    // (only the remainders that some part of this kernel size can have are compiled)
    if constexpr (remainder_occurs(G, parts, SEARCH_GB, 1)) if (left == 1) search_groups(std::integral_constant<int, 1>{}, gb);
    if constexpr (remainder_occurs(G, parts, SEARCH_GB, 2)) if (left == 2) search_groups(std::integral_constant<int, 2>{}, gb);
    if constexpr (remainder_occurs(G, parts, SEARCH_GB, 3)) if (left == 3) search_groups(std::integral_constant<int, 3>{}, gb);
    if constexpr (remainder_occurs(G, parts, SEARCH_GB, 4)) if (left == 4) search_groups(std::integral_constant<int, 4>{}, gb);
    static_assert(SEARCH_GB <= 5, "remainders above four groups are not dispatched");
  }
  if (M) {
#pragma unroll
    for (int w = 0; w < MW; ++w)
      if (hbits[w]) atomicOr(&s_mask[(bl0 + (lane >> 5)) * MW + w], hbits[w]);
  }
  __syncthreads();
  if constexpr (PAIRS) {
    // where every offset's pairs start in the slab: exclusive prefix of the counts, by wave 0
    if (wave == 0) {
      int carry = 0;
      for (int k0 = 0; k0 < K3; k0 += 64) {
        const int k = k0 + lane;
        const int c = k < K3 ? s_cnt[k] : 0;
        int x = c;
        for (int d = 1; d < 64; d <<= 1) {
          const int y = __shfl_up(x, d, 64);
          if (lane >= d) x += y;
        }
        if (k < K3) s_off[k] = carry + x - c;
        carry += __shfl(x, 63, 64);
      }
      if (lane == 0) s_off[K3] = carry;
    }
    for (int k = tid; k < K3; k += SEARCH_THREADS) tile_counts[int64_t(k) * n_tiles_cap + blockIdx.x] = s_cnt[k];
    __syncthreads();
    // compaction: a wave takes an offset at a time and walks the tile's rows in steps of 64; the hit's input
    // position is the group's lower bound plus the number of the group's earlier queries that hit
    int2* slab = tile_pairs + int64_t(blockIdx.x) * tile * K3;
    for (int k = wave; k < K3; k += NW) {
      if (s_cnt[k] == 0) continue;  // uniform (offsets outside ws_k are never counted)
      const int g = k / K, tk = k - g * K, tq = sp.zrev ? K - 1 - tk : tk;
      int at = s_off[k];
      for (int v0 = 0; v0 < rows; v0 += 64) {
        const int vv = v0 + lane;
        const unsigned msk = vv < tile ? s_hit[g * tile + vv] : 0u;
        const bool hit = vv < rows && ((msk >> tq) & 1u);
        const unsigned long long bal = __ballot(hit);
        if (hit) {
          const int jpos = s_pos[g * tile + vv] + __popc(msk & ((1u << tq) - 1u));
          slab[at + lanemask_lt_popc(bal)] = make_int2(in_perm ? in_perm[jpos] : jpos, i0 + vv);
        }
        at += __popcll(bal);
      }
    }
  }
  if (M) {
    const int n_bl = rows32 >> 5;
    for (int e = tid; e < n_bl * MW; e += SEARCH_THREADS) block_masks[b0 * MW + e] = s_mask[e];
  }
}

// Weight-stationary lists from the tiles' slabs of compacted pairs (the search kernel in its PAIRS form): one
// workgroup per tile copies its hits, offset by offset, to where the scan of the per-tile counts puts them.  List k
// comes out ordered by output index, without atomics and without a |V_q| x K^3 matrix having existed.
__global__ __launch_bounds__(256) void ws_fill_pairs_kernel(const int2* __restrict__ tile_pairs, int n_out_h,
                                                            const int* __restrict__ n_out_d, int K3, int tile,
                                                            const int32_t* __restrict__ tile_base, int n_tiles_cap,
                                                            const int32_t* __restrict__ nnz, int32_t* __restrict__ ws_in,
                                                            int32_t* __restrict__ ws_out, int64_t ws_stride, int k_lim) {
  __shared__ int s_off[WS_MAX_K3_SEARCH + 1], s_dst[WS_MAX_K3_SEARCH];
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  const int i0 = blockIdx.x * tile;
  if (i0 >= n_out) return;
  const int n_tiles = (n_out + tile - 1) / tile;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // counts of this tile (difference of consecutive scanned bases) and their exclusive prefix
  if (wave == 0) {
    int carry = 0;
    for (int k0 = 0; k0 < K3; k0 += 64) {
      const int k = k0 + lane;
      int c = 0;
      if (k < k_lim) {
        const int32_t* col = tile_base + int64_t(k) * n_tiles_cap;
        const int b = col[blockIdx.x];
        c = (int(blockIdx.x) + 1 < n_tiles ? col[blockIdx.x + 1] : nnz[k]) - b;
        s_dst[k] = b;
      }
      int x = c;
      for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
      }
      if (k < K3) s_off[k] = carry + x - c;
      carry += __shfl(x, 63, 64);
    }
    if (lane == 0) s_off[K3] = carry;
  }
  __syncthreads();
  const int total = s_off[K3];
  const int2* slab = tile_pairs + int64_t(blockIdx.x) * tile * K3;
  for (int e = tid; e < total; e += 256) {
    int k = 0;  // last offset whose pairs start at or before e (offsets without pairs share their successor's start)
    for (int bit = 256; bit > 0; bit >>= 1)
      if (k + bit < K3 && s_off[k + bit] <= e) k += bit;
    const int2 pr = slab[e];
    const int64_t dst = int64_t(k) * ws_stride + s_dst[k] + (e - s_off[k]);
    ws_in[dst] = pr.x;
    ws_out[dst] = pr.y;
  }
}

// One workgroup per offset k: exclusive scan of that offset's per-tile counts in place, total into nnz[k].
// A thread owns a run of consecutive tiles; the runs are fetched in batches of WS_SCAN_U loads per thread that are
// all in flight together (a loop of load, scan, store rounds over 256 tiles at a time took 7.6 us for 3750 tiles:
// fifteen dependent round trips).
constexpr int WS_SCAN_U = 8;
__global__ __launch_bounds__(256) void ws_scan_kernel(int32_t* __restrict__ tile_counts, int n_tiles_cap, int tile,
                                                      int n_out_h, const int* __restrict__ n_out_d,
                                                      int32_t* __restrict__ nnz, int k_lim) {
  __shared__ int wave_sum[4];
  if (int(blockIdx.x) >= k_lim) {  // offsets without a list of their own (second half of a symmetric map)
    if (threadIdx.x == 0) nnz[blockIdx.x] = 0;
    return;
  }
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  const int n_tiles = (n_out + tile - 1) / tile;
  int32_t* c = tile_counts + int64_t(blockIdx.x) * n_tiles_cap;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int carry = 0;
  for (int b0 = 0; b0 < n_tiles; b0 += 256 * WS_SCAN_U) {
    const int first = b0 + threadIdx.x * WS_SCAN_U;  // this thread's run: tiles first .. first + WS_SCAN_U - 1
    int v[WS_SCAN_U];
#pragma unroll
    for (int u = 0; u < WS_SCAN_U; ++u) v[u] = first + u < n_tiles ? c[first + u] : 0;
    int sum = 0;
#pragma unroll
    for (int u = 0; u < WS_SCAN_U; ++u) sum += v[u];
    int x = sum;
    for (int d = 1; d < 64; d <<= 1) {
      const int y = __shfl_up(x, d, 64);
      if (lane >= d) x += y;
    }
    if (b0 > 0) __syncthreads();  // the wave sums of the round before have been read
    if (lane == 63) wave_sum[wave] = x;
    __syncthreads();
    int base = 0, tot = 0;
    for (int w = 0; w < 4; ++w) {
      const int s = wave_sum[w];
      if (w < wave) base += s;
      tot += s;
    }
    int run = carry + base + x - sum;
#pragma unroll
    for (int u = 0; u < WS_SCAN_U; ++u) {
      if (first + u < n_tiles) c[first + u] = run;
      run += v[u];
    }
    carry += tot;
  }
  if (threadIdx.x == 0) nnz[blockIdx.x] = carry;
}

// Output-stationary layout of a transposed layer from the inverse its strided twin's search left behind (pairs
// of a transposed layer are the twin's pairs with the roles swapped, Section 5.5: maps shared between layers).
// Where the twin's offsets partition its inputs (K = layer stride, e.g. 2x2x2 at stride 2), every output voxel p of
// the transposed layer has exactly one pair, (input parent[p] / K^3, offset parent[p] % K^3): a thread per voxel
// writes its row of the blocked matrix (full lines per offset) and the block masks fall out of ballots.
__global__ __launch_bounds__(256) void transposed_from_parent_kernel(const int32_t* __restrict__ parent, int n_h,
                                                                     const int* __restrict__ n_d, int K3,
                                                                     int32_t* __restrict__ Mt, uint32_t* __restrict__ block_masks) {
  const int n = n_d ? *n_d : n_h;
  const int64_t p = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int64_t blk = p >> 5;
  if (blk * 32 >= n) return;  // whole 32-row blocks leave together (the ballots below stay among one wave's lanes)
  const int pr = p < n ? parent[p] : -1;
  const int q = pr < 0 ? -1 : pr / K3, kp = pr < 0 ? -1 : pr - q * K3;
  const int half = (threadIdx.x >> 5) & 1;
  uint32_t mask = 0;  // K3 <= 32 here
  for (int k = 0; k < K3; ++k) {
    Mt[(blk * K3 + k) * 32 + (p & 31)] = k == kp ? q : -1;
    const unsigned long long b = __ballot(k == kp);
    if ((half ? unsigned(b >> 32) : unsigned(b)) != 0u) mask |= 1u << k;
  }
  if ((p & 31) == 0) block_masks[blk] = mask;
}

__global__ void copy_int_kernel(const int* src, int* dst) { *dst = *src; }

// ---------------------------------------------------------------- host side
static int axis_offset(int K, int s, int i) { return (K % 2 == 1) ? (i - (K - 1) / 2) * s : i * s; }


static std::atomic<int64_t> g_search_launches{0};  // searches enqueued by this process (see spc_search_count)

template <typename KeyT, int K, int TILE>
static int launch_search(spc_kmap* m, hipStream_t s) {
  const PackInfo& pi = m->pi;
  const int sp_stride = m->desc.in_stride;
  const int sign = m->desc.transposed ? -1 : 1;
  SearchParams<KeyT> sp{};
  auto packed = [&](int i, int shift) {  // offset of index i along an axis, shifted into its field (wrapping)
    return static_cast<KeyT>(static_cast<uint64_t>(int64_t(sign) * axis_offset(K, sp_stride, i)) << shift);
  };
  sp.X0 = packed(0, pi.sh_x);
  sp.dX = K > 1 ? static_cast<KeyT>(packed(1, pi.sh_x) - sp.X0) : KeyT(0);
  sp.Y0 = packed(0, pi.sh_y);
  sp.dY = K > 1 ? static_cast<KeyT>(packed(1, pi.sh_y) - sp.Y0) : KeyT(0);
  const int64_t z_a = int64_t(sign) * axis_offset(K, sp_stride, 0), z_b = int64_t(sign) * axis_offset(K, sp_stride, K - 1);
  sp.zmin = static_cast<KeyT>(static_cast<uint64_t>(std::min(z_a, z_b)));
  sp.zstep = static_cast<KeyT>(sp_stride);
  sp.zrev = (K > 1 && z_a > z_b) ? 1 : 0;
  for (int g = 0; g < K * K; ++g)
    for (int t = 0; t < K; ++t)
      if ((m->os_map && m->os_k.has(g * K + t)) || m->ws_k.has(g * K + t)) sp.need |= 1ull << g;
  const Level* in = m->in_level;
  const Level* out = m->out_level;
  const bool pairs = (m->desc.layout & SPC_LAYOUT_WS) != 0;
  const size_t lds = size_t(m->tile) * sizeof(KeyT) + WIN_CAP_BYTES + MAX_K * sizeof(KeyT) + (pairs ? size_t(K) * K * m->tile * 5 : 0);
  auto go = [&](auto PAIRS_) {
    constexpr bool PAIRS = decltype(PAIRS_)::value;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&kmap_search_kernel<KeyT, K, TILE, PAIRS>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    (void)attr;
    hipLaunchKernelGGL((kmap_search_kernel<KeyT, K, TILE, PAIRS>), dim3(m->n_tiles), dim3(SEARCH_THREADS), lds, s,
                       static_cast<const KeyT*>(in->keys), static_cast<int>(in->n_host < 0 ? 0 : in->n_host), in->n_dev,
                       static_cast<const KeyT*>(out->keys), static_cast<int>(out->n_host < 0 ? 0 : out->n_host), out->n_dev,
                       sp, m->os_map, m->block_masks, m->tile_counts, m->n_tiles, m->in_perm, m->os_k, m->ws_k,
                       m->tile_pairs, m->inv_parent);
  };
  if (m->n_tiles > 0) {
    if (pairs) go(std::true_type{});
    else go(std::false_type{});
  }
  g_search_launches.fetch_add(1, std::memory_order_relaxed);
  return SPC_OK;
}

template <typename KeyT>
static int launch_search_k(spc_kmap* m, hipStream_t s) {
  switch (m->desc.K) {
    case 1: return m->tile == 256 ? launch_search<KeyT, 1, 256>(m, s) : launch_search<KeyT, 1, 128>(m, s);
    case 2: return m->tile == 256 ? launch_search<KeyT, 2, 256>(m, s) : launch_search<KeyT, 2, 128>(m, s);
    case 3: return m->tile == 256 ? launch_search<KeyT, 3, 256>(m, s) : launch_search<KeyT, 3, 128>(m, s);
    case 5: return launch_search<KeyT, 5, 128>(m, s);
    case 7: return launch_search<KeyT, 7, 64>(m, s);
  }
  return set_error(SPC_ERR_UNSUPPORTED, "kernel size %d not built (1,2,3,5,7 are)", m->desc.K);
}

static void kmap_free(spc_kmap* m) {
  if (m->twin) {  // a transposed map derived from its strided twin: the lists (if any) are the twin's
    if (m->ws_in) {
      m->ws_in = m->ws_out = nullptr;
      m->nnz_dev = nullptr;
    }
    // whoever read this map may have read the twin's arrays: the twin's release waits for them as well
    for (hipStream_t c : m->consumers) m->twin->consumers.push_back(c);
    m->twin->consumers.push_back(m->stream);
    spc_kmap* t = m->twin;
    m->twin = nullptr;
    if (t->refs.fetch_sub(1) == 1) kmap_free(t);
  }
  // The arrays return to the build stream's cache, where the next build may take them at once: that
  // stream first waits for the feature kernels other streams have enqueued on this map.
  for (hipStream_t c : m->consumers) order_stream_after(m->stream, c);
  pool_free(m->os_map, m->stream);
  pool_free(m->block_masks, m->stream);
  pool_free(m->ws_in, m->stream);
  pool_free(m->ws_out, m->stream);
  pool_free(m->nnz_dev, m->stream);
  pool_free(m->tile_counts, m->stream);
  pool_free(m->tile_pairs, m->stream);
  pool_free(m->inv_parent, m->stream);
  level_unref(m->in_level);
  level_unref(m->out_level);
  if (m->ready) (void)hipEventDestroy(m->ready);
  for (hipEvent_t e : m->aux_events) (void)hipEventDestroy(e);
  delete m;
}

static int check_layer(const spc_layer_desc* l) {
  if (!l) return set_error(SPC_ERR_ARG, "layer descriptor is NULL");
  auto pow2 = [](int v) { return v >= 1 && (v & (v - 1)) == 0; };
  if (l->K != 1 && l->K != 2 && l->K != 3 && l->K != 5 && l->K != 7)
    return set_error(SPC_ERR_UNSUPPORTED, "kernel size %d not built (1,2,3,5,7 are)", l->K);
  if (!pow2(l->in_stride) || !pow2(l->layer_stride)) return set_error(SPC_ERR_ARG, "strides must be powers of two");
  if (l->transposed != 0 && l->transposed != 1) return set_error(SPC_ERR_ARG, "transposed must be 0 or 1");
  if (l->transposed && l->layer_stride == 1) return set_error(SPC_ERR_ARG, "a transposed layer needs layer_stride > 1");
  const int base = l->layout & SPC_LAYOUT_BOTH;
  const int thr = (l->layout >> 8) & 0xff;
  if (l->layout < 1 || (l->layout & ~0xff07) || base == 0)
    return set_error(SPC_ERR_ARG, "layout must be OS, WS or BOTH (| WS_SYM) (| HYBRID_T(t))");
  if (thr && base != SPC_LAYOUT_BOTH) return set_error(SPC_ERR_ARG, "a hybrid threshold needs both layouts");
  if (l->layout & SPC_LAYOUT_WS_SYM) {
    if (!(l->layout & SPC_LAYOUT_WS)) return set_error(SPC_ERR_ARG, "WS_SYM modifies the WS layout");
    if (l->layer_stride != 1 || l->K % 2 == 0 || l->K < 3)
      return set_error(SPC_ERR_ARG, "the symmetric half-map needs a submanifold layer with odd K >= 3");
  }
  return SPC_OK;
}

// The packing descriptor must suit the layer (Section 5.3): packed(q) + packed(delta) = packed(q + delta)
// holds only while no field borrows or carries, i.e. while the guard band covers the layer's largest
// offset component; and masking the low bits of a field equals floor() on the raw coordinate only if
// the field's bias, origin - pad, is a multiple of the layer's output stride.
static int check_desc_layer(const spc_pack_desc* d, const spc_layer_desc* l) {
  const int64_t reach = int64_t(l->K % 2 ? (l->K - 1) / 2 : l->K - 1) * l->in_stride;
  if (d->pad < reach)
    return set_error(SPC_ERR_ARG, "guard band pad = %d is smaller than the layer's reach %lld (K = %d, in_stride = %d)", d->pad,
                     static_cast<long long>(reach), l->K, l->in_stride);
  const int64_t so = int64_t(l->in_stride) * l->layer_stride;
  for (int a = 0; a < 3; ++a)
    if ((int64_t(d->origin[a]) - d->pad) % so != 0)
      return set_error(SPC_ERR_ARG, "origin[%d] - pad = %lld is not a multiple of the layer's output stride %lld", a,
                       static_cast<long long>(int64_t(d->origin[a]) - d->pad), static_cast<long long>(so));
  return SPC_OK;
}

static int ilog2(int v) {
  int b = 0;
  while ((1 << b) < v) ++b;
  return b;
}

// Builds the map object for given input/output levels (references are taken).
static int build_on_levels(Level* in, Level* out, const PackInfo& pi, const spc_layer_desc& l, hipStream_t s, spc_kmap** res,
                           const int32_t* in_perm = nullptr, bool want_inverse = false) {
  spc_kmap* m = new spc_kmap;
  m->in_perm = in_perm;
  m->pi = pi;
  m->desc = l;
  m->K3 = l.K * l.K * l.K;
  m->sym = (l.layout & SPC_LAYOUT_WS_SYM) != 0;
  m->k_lim = m->sym ? (m->K3 - 1) / 2 : m->K3;
  // Offsets of the matrix and of the lists.  With a threshold (hybrid dual dataflow, Section 5.4) the offsets
  // whose L1 norm is below it go to the matrix only and the others to the lists only; a symmetric map keeps
  // lists for the first half of its offsets.
  m->hybrid_t = (l.layout >> 8) & 0xff;
  for (int k = 0; k < m->K3; ++k) {
    const bool dense = m->hybrid_t == 0 || offset_l1(l.K, k) < m->hybrid_t;
    const bool sparse = m->hybrid_t == 0 || !dense;
    if ((l.layout & SPC_LAYOUT_OS) && dense) m->os_k.w[k >> 5] |= 1u << (k & 31);
    if ((l.layout & SPC_LAYOUT_WS) && sparse && k < m->k_lim) m->ws_k.w[k >> 5] |= 1u << (k & 31);
  }
  m->stream = s;
  m->captured = stream_is_capturing(s);
  m->in_level = in;
  in->refs++;
  in->add_reader(s);
  m->out_level = out;
  out->refs++;
  out->add_reader(s);
  (void)hipGetDevice(&m->device);
  m->out_cap = out->n_host >= 0 ? out->n_host : out->cap;
  m->tile = search_tile(l.K, m->out_cap);
  m->n_tiles = static_cast<int>((m->out_cap + m->tile - 1) / m->tile);
  m->n_blocks_cap = (m->out_cap + 31) / 32;
  m->mask_words = (m->K3 + 31) / 32;
  const size_t cells = std::max<size_t>(size_t(m->n_blocks_cap) * 32 * m->K3, 64);
  const bool with_os = (l.layout & SPC_LAYOUT_OS) != 0;
  // the |V_q| x K^3 matrix and its block masks exist only when the output-stationary layout is asked for
  if (with_os) {
    m->os_map = static_cast<int32_t*>(pool_alloc(cells * 4, s));
    m->block_masks = static_cast<uint32_t*>(pool_alloc(std::max<size_t>(size_t(m->n_blocks_cap) * m->mask_words * 4, 256), s));
  }
  m->nnz_dev = static_cast<int32_t*>(pool_alloc(std::max<size_t>(size_t(m->K3) * 4, 256), s));
  m->ws_stride = m->out_cap;
  if (want_inverse && !in_perm)
    m->inv_parent = static_cast<int32_t*>(pool_alloc(std::max<size_t>(size_t(in->n_host >= 0 ? in->n_host : in->cap) * 4, 256), s));
  bool ok = m->nnz_dev && (!with_os || (m->os_map && m->block_masks)) && (m->inv_parent || !(want_inverse && !in_perm));
  if (ok && (l.layout & SPC_LAYOUT_WS)) {
    m->ws_in = static_cast<int32_t*>(pool_alloc(cells * 4, s));
    m->ws_out = static_cast<int32_t*>(pool_alloc(cells * 4, s));
    m->tile_counts = static_cast<int32_t*>(pool_alloc(std::max<size_t>(size_t(m->n_tiles) * m->K3 * 4, 256), s));
    // slabs of compacted pairs, one per search tile (bounded by tile * K^3 pairs each; a tile writes its hits only)
    m->tile_pairs = static_cast<int2*>(pool_alloc(std::max<size_t>(size_t(m->n_tiles) * m->tile * m->K3 * 8, 256), s));
    ok = m->ws_in && m->ws_out && m->tile_counts && m->tile_pairs;
  }
  if (!ok) {
    kmap_free(m);
    return SPC_ERR_NOMEM;
  }
  int rc = pi.key_bits == 32 ? launch_search_k<uint32_t>(m, s) : launch_search_k<uint64_t>(m, s);
  if (rc == SPC_OK && (l.layout & SPC_LAYOUT_WS)) {
    const int n_out_h = static_cast<int>(out->n_host < 0 ? 0 : out->n_host);
    hipLaunchKernelGGL(ws_scan_kernel, dim3(m->K3), dim3(256), 0, s, m->tile_counts, m->n_tiles, m->tile, n_out_h,
                       out->n_dev, m->nnz_dev, m->k_lim);
    if (m->n_tiles > 0)
      hipLaunchKernelGGL(ws_fill_pairs_kernel, dim3(m->n_tiles), dim3(256), 0, s, m->tile_pairs, n_out_h, out->n_dev, m->K3,
                         m->tile, m->tile_counts, m->n_tiles, m->nnz_dev, m->ws_in, m->ws_out, m->out_cap, m->k_lim);
    // the slabs are dead once the lists are filled: back to the cache (reuse is ordered behind this stream's work)
    pool_free(m->tile_pairs, s);
    m->tile_pairs = nullptr;
  }
  if (rc == SPC_OK && hipGetLastError() != hipSuccess) rc = set_error(SPC_ERR_HIP, "kernel-map launch failed");
  if (rc == SPC_OK && (hipEventCreateWithFlags(&m->ready, hipEventDisableTiming) != hipSuccess ||
                       hipEventRecord(m->ready, s) != hipSuccess))
    rc = set_error(SPC_ERR_HIP, "event record failed");
  if (rc != SPC_OK) {
    kmap_free(m);
    return rc;
  }
  *res = m;
  return SPC_OK;
}

// A strided layer whose offsets partition its inputs (K = layer stride, even K: offsets {0..K-1} * in_stride) can
// hand its pairs to the transposed layer of the same geometry instead of a second search.
static bool twin_can_share(const spc_layer_desc& strided, const spc_layer_desc& transposed) {
  return !strided.transposed && transposed.transposed && strided.K == transposed.K && strided.in_stride == transposed.in_stride &&
         strided.layer_stride == transposed.layer_stride && strided.K == strided.layer_stride && strided.K % 2 == 0 &&
         strided.K * strided.K * strided.K <= 32;
}

// The transposed map from its strided twin (see transposed_from_parent_kernel): the matrix from the twin's inverse,
// the lists by taking the twin's with inputs and outputs swapped (for a fixed offset both index sequences ascend
// together, so the order by output index is kept).  Returns SPC_ERR_UNSUPPORTED when the twin lacks what is needed.
static int build_transposed_from_twin(spc_kmap* twin, Level* coarse, Level* fine, const PackInfo& pi, const spc_layer_desc& l,
                                      hipStream_t s, spc_kmap** res) {
  const bool with_os = (l.layout & SPC_LAYOUT_OS) != 0, with_ws = (l.layout & SPC_LAYOUT_WS) != 0;
  if (!twin_can_share(twin->desc, l) || (l.layout & ~SPC_LAYOUT_BOTH) || (with_os && !twin->inv_parent) ||
      (with_ws && (!(twin->desc.layout & SPC_LAYOUT_WS) || twin->hybrid_t || twin->sym)))
    return SPC_ERR_UNSUPPORTED;
  spc_kmap* m = new spc_kmap;
  m->pi = pi;
  m->desc = l;
  m->K3 = l.K * l.K * l.K;
  m->k_lim = m->K3;
  for (int k = 0; k < m->K3; ++k) {
    if (with_os) m->os_k.w[k >> 5] |= 1u << (k & 31);
    if (with_ws) m->ws_k.w[k >> 5] |= 1u << (k & 31);
  }
  m->stream = s;
  m->captured = stream_is_capturing(s);
  m->in_level = coarse;
  coarse->refs++;
  m->out_level = fine;
  fine->refs++;
  (void)hipGetDevice(&m->device);
  m->out_cap = fine->n_host >= 0 ? fine->n_host : fine->cap;
  m->tile = search_tile(l.K, m->out_cap);
  m->n_tiles = static_cast<int>((m->out_cap + m->tile - 1) / m->tile);
  m->n_blocks_cap = (m->out_cap + 31) / 32;
  m->mask_words = 1;
  m->twin = twin;
  twin->refs++;
  int rc = SPC_OK;
  if (s != twin->stream && twin->ready && hipStreamWaitEvent(s, twin->ready, 0) != hipSuccess)
    rc = set_error(SPC_ERR_HIP, "hipStreamWaitEvent failed");
  if (rc == SPC_OK && with_os) {
    m->os_map = static_cast<int32_t*>(pool_alloc(std::max<size_t>(size_t(m->n_blocks_cap) * 32 * m->K3 * 4, 256), s));
    m->block_masks = static_cast<uint32_t*>(pool_alloc(std::max<size_t>(size_t(m->n_blocks_cap) * 4, 256), s));
    if (!m->os_map || !m->block_masks) rc = SPC_ERR_NOMEM;
    else if (m->out_cap > 0)
      hipLaunchKernelGGL(transposed_from_parent_kernel, dim3(static_cast<unsigned>((m->out_cap + 255) / 256)), dim3(256), 0, s,
                         twin->inv_parent, static_cast<int>(fine->n_host < 0 ? 0 : fine->n_host), fine->n_host < 0 ? fine->n_dev : nullptr,
                         m->K3, m->os_map, m->block_masks);
  }
  if (rc == SPC_OK && with_ws) {
    m->ws_in = twin->ws_out;
    m->ws_out = twin->ws_in;
    m->nnz_dev = twin->nnz_dev;
    m->ws_stride = twin->ws_stride;
  }
  if (rc == SPC_OK && hipGetLastError() != hipSuccess) rc = set_error(SPC_ERR_HIP, "kernel-map launch failed");
  if (rc == SPC_OK && (hipEventCreateWithFlags(&m->ready, hipEventDisableTiming) != hipSuccess ||
                       hipEventRecord(m->ready, s) != hipSuccess))
    rc = set_error(SPC_ERR_HIP, "event record failed");
  if (rc != SPC_OK) {
    kmap_free(m);
    return rc;
  }
  *res = m;
  return SPC_OK;
}

static Level* borrowed_level(const void* keys, int64_t n, int stride) {
  Level* lv = new Level;
  lv->keys = const_cast<void*>(keys);
  lv->owns_keys = false;
  lv->cap = n;
  lv->n_host = n;
  lv->stride = stride;
  return lv;
}

// Host copy of a level's voxel count in lv->n_fetched.  A level built under stream capture is
// rewritten by every replay of the graph: its events cannot be waited for (they belong to the
// capture), so the whole device is drained instead, and the value is never cached.
static int fetch_level_n(Level* lv) {
  if (lv->n_host >= 0) {
    lv->n_fetched = lv->n_host;
    return SPC_OK;
  }
  if (lv->captured) SPC_HIP_CHECK(hipDeviceSynchronize());
  else if (lv->ready) SPC_HIP_CHECK(hipEventSynchronize(lv->ready));
  int v = 0;
  SPC_HIP_CHECK(hipMemcpy(&v, lv->n_dev, sizeof(int), hipMemcpyDeviceToHost));
  lv->n_fetched = v;
  if (!lv->captured) lv->n_host = v;
  return SPC_OK;
}

// Waits until the map's arrays are complete (see fetch_level_n for captured builds).
static int wait_map(const spc_kmap* m) {
  if (m->captured) SPC_HIP_CHECK(hipDeviceSynchronize());
  else if (m->ready) SPC_HIP_CHECK(hipEventSynchronize(m->ready));
  return SPC_OK;
}

// Layout every distinct map of a network is built with: the union of what its layers ask for; a map
// shared by layers that disagree about the half-map keeps the full lists.
using NetKey = std::tuple<int, int, int, int>;
static NetKey net_key(const spc_layer_desc& l) { return NetKey(l.K, l.in_stride, l.layer_stride, l.transposed); }
static std::map<NetKey, int> net_layouts(const spc_layer_desc* layers, int n_layers) {
  std::map<NetKey, int> want;
  for (int i = 0; i < n_layers; ++i) want[net_key(layers[i])] |= layers[i].layout & 0xff;
  // a hybrid threshold survives only if every layer that shares the map asks for that same threshold
  for (auto& kv : want) {
    int thr = -1;
    for (int i = 0; i < n_layers; ++i)
      if (net_key(layers[i]) == kv.first) {
        const int t = (layers[i].layout >> 8) & 0xff;
        thr = thr < 0 ? t : (thr == t ? t : 0);
      }
    if (thr > 0) kv.second |= thr << 8;
  }
  for (auto& kv : want) {
    bool all_sym = true;
    for (int i = 0; i < n_layers; ++i)
      if (net_key(layers[i]) == kv.first && (layers[i].layout & SPC_LAYOUT_WS) && !(layers[i].layout & SPC_LAYOUT_WS_SYM))
        all_sym = false;
    if (!all_sym) kv.second &= ~SPC_LAYOUT_WS_SYM;
  }
  return want;
}

// One map of a network build.  A transposed layer whose strided twin has been built on the same stream (no
// cross-stream edge is added) takes the twin's pairs; a strided layer with such a transposed twin among the
// wanted maps leaves its inverse behind for it.  Everything else is searched.
static int build_network_map(const NetKey& key, const spc_layer_desc& l, const std::map<NetKey, int>& want,
                             const std::map<NetKey, spc_kmap*>& maps, Level* fine, Level* coarse, const PackInfo& pi, hipStream_t s,
                             spc_kmap** m) {
  const NetKey other(std::get<0>(key), std::get<1>(key), std::get<2>(key), l.transposed ? 0 : 1);
  if (l.transposed) {
    auto it = maps.find(other);
    if (it != maps.end() && it->second->stream == s) {
      const int rc = build_transposed_from_twin(it->second, coarse, fine, pi, l, s, m);
      if (rc != SPC_ERR_UNSUPPORTED) return rc;
    }
    return build_on_levels(coarse, fine, pi, l, s, m);
  }
  spc_layer_desc t = l;
  t.transposed = 1;
  const bool inverse = want.count(other) != 0 && twin_can_share(l, t);
  return build_on_levels(fine, coarse, pi, l, s, m, nullptr, inverse);
}

// SPC_NET_PIPELINED: one build stream, work in the order of first use (a level right before the first
// map that reads it), no join: the maps are marked so that their consumers wait for them.
static int build_network_pipelined(const void* v0_keys, int64_t n0, const PackInfo& pi, const spc_layer_desc* layers,
                                   int n_layers, spc_kmap** out, hipStream_t sb, hipStream_t sl, hipEvent_t fork) {
  // sl: the stream of the coordinate levels (sb itself, or a stream of its own: every level comes straight from
  // V_0, so the levels then run ahead of the searches, which wait for the level they read)
  std::map<int, Level*> levels;
  levels[1] = borrowed_level(v0_keys, n0, 1);
  const std::map<NetKey, int> want = net_layouts(layers, n_layers);
  std::map<NetKey, spc_kmap*> maps;
  std::set<Level*> awaited;
  spc_kmap* first = nullptr;
  int rc = SPC_OK;
  if (sl != sb)  // all levels up front, in the order of first use
    for (int i = 0; i < n_layers && rc == SPC_OK; ++i) {
      const int need[2] = {layers[i].in_stride, layers[i].in_stride * layers[i].layer_stride};
      for (int j = 0; j < 2 && rc == SPC_OK; ++j) {
        if (levels.count(need[j])) continue;
        Level* lv = nullptr;
        rc = downsample_level(v0_keys, n0, nullptr, pi, ilog2(need[j]), &lv, sl);
        if (rc == SPC_OK) levels[need[j]] = lv;
      }
    }
  for (int i = 0; i < n_layers && rc == SPC_OK; ++i) {
    const NetKey key = net_key(layers[i]);
    if (maps.count(key)) continue;
    spc_layer_desc l = layers[i];
    l.layout = want.at(key);
    const int need[2] = {l.in_stride, l.in_stride * l.layer_stride};
    for (int j = 0; j < 2 && rc == SPC_OK; ++j) {
      if (!levels.count(need[j])) {  // one build stream: the level right before the first map that reads it
        Level* lv = nullptr;
        rc = downsample_level(v0_keys, n0, nullptr, pi, ilog2(need[j]), &lv, sb);
        if (rc == SPC_OK) levels[need[j]] = lv;
      } else if (sl != sb && levels[need[j]]->ready && awaited.insert(levels[need[j]]).second) {
        if (hipStreamWaitEvent(sb, levels[need[j]]->ready, 0) != hipSuccess) rc = set_error(SPC_ERR_HIP, "hipStreamWaitEvent failed");
      }
    }
    if (rc != SPC_OK) break;
    Level* fine = levels[l.in_stride];
    Level* coarse = levels[l.in_stride * l.layer_stride];
    spc_kmap* m = nullptr;
    rc = build_network_map(key, l, want, maps, fine, coarse, pi, sb, &m);
    if (rc == SPC_OK) {
      m->wait_on_use = true;
      maps[key] = m;
      if (!first) first = m;
    }
  }
  // the fork event lives as long as the maps (a capture of this call refers to it)
  if (rc == SPC_OK && first) first->aux_events.push_back(fork);
  else (void)hipEventDestroy(fork);
  if (rc == SPC_OK)
    for (int i = 0; i < n_layers; ++i) {
      spc_kmap* m = maps[net_key(layers[i])];
      m->refs++;
      out[i] = m;
    }
  for (auto& kv : maps)  // drop the builder's own reference
    if (kv.second->refs.fetch_sub(1) == 1) kmap_free(kv.second);
  for (auto& kv : levels) level_unref(kv.second);
  return rc;
}

}  // namespace spc

using namespace spc;

extern "C" {

int spc_build_kmap(const void* in_keys, int64_t n_in, const spc_pack_desc* d, const spc_layer_desc* l, spc_kmap** out,
                   void* stream) {
  return spc_build_kmap_perm(in_keys, n_in, nullptr, d, l, out, stream);
}

int spc_build_kmap_perm(const void* in_keys, int64_t n_in, const int32_t* in_perm, const spc_pack_desc* d,
                        const spc_layer_desc* l, spc_kmap** out, void* stream) {
  PackInfo pi;
  SPC_RETURN_IF(check_desc(d, &pi));
  SPC_RETURN_IF(check_layer(l));
  SPC_RETURN_IF(check_desc_layer(d, l));
  if (!out) return set_error(SPC_ERR_ARG, "out is NULL");
  if (n_in < 0 || n_in > 0x7fffffff || (!in_keys && n_in > 0)) return set_error(SPC_ERR_ARG, "bad in_keys / n_in");
  if (int64_t(n_in) * l->K * l->K * l->K > (int64_t(1) << 40)) return set_error(SPC_ERR_ARG, "map too large");
  hipStream_t s = static_cast<hipStream_t>(stream);
  Level* given = borrowed_level(in_keys, n_in, l->in_stride);
  Level* derived = nullptr;
  int rc = SPC_OK;
  if (l->layer_stride > 1) rc = downsample_level(in_keys, n_in, nullptr, pi, ilog2(l->in_stride * l->layer_stride), &derived, s);
  if (rc == SPC_OK) {
    if (in_perm && l->transposed) rc = set_error(SPC_ERR_ARG, "in_perm applies to the given level, which a transposed layer writes");
    else if (in_perm && (l->layout & SPC_LAYOUT_WS_SYM))
      rc = set_error(SPC_ERR_ARG, "a symmetric half-map swaps inputs and outputs: both must be numbered alike (no in_perm)");
    else if (l->layer_stride == 1) rc = build_on_levels(given, given, pi, *l, s, out, in_perm);
    else if (!l->transposed) rc = build_on_levels(given, derived, pi, *l, s, out, in_perm);
    else rc = build_on_levels(derived, given, pi, *l, s, out);
  }
  level_unref(given);
  level_unref(derived);
  return rc;
}

int spc_build_kmaps_network(const void* v0_keys, int64_t n0, const spc_pack_desc* d, const spc_layer_desc* layers,
                            int32_t n_layers, spc_kmap** out, void* const* streams, int32_t n_streams, int32_t flags) {
  PackInfo pi;
  SPC_RETURN_IF(check_desc(d, &pi));
  if (!layers || !out || n_layers < 1) return set_error(SPC_ERR_ARG, "layers/out NULL or n_layers < 1");
  if (!streams || n_streams < 1) return set_error(SPC_ERR_ARG, "at least one stream is required");
  if (n0 < 0 || n0 > 0x7fffffff || (!v0_keys && n0 > 0)) return set_error(SPC_ERR_ARG, "bad v0_keys / n0");
  for (int i = 0; i < n_layers; ++i) {
    SPC_RETURN_IF(check_layer(&layers[i]));
    SPC_RETURN_IF(check_desc_layer(d, &layers[i]));
  }
  const int ns = (flags & SPC_NET_SEQUENTIAL) ? 1 : n_streams;
  std::vector<hipStream_t> st(ns);
  for (int i = 0; i < ns; ++i) st[i] = static_cast<hipStream_t>(streams[i]);

  // fork: every other stream waits for what streams[0] has enqueued so far (the pack/sort)
  hipEvent_t fork = nullptr;
  const bool pipelined = (flags & SPC_NET_PIPELINED) && ns >= 2;
  if (ns > 1) {
    SPC_HIP_CHECK(hipEventCreateWithFlags(&fork, hipEventDisableTiming));
    SPC_HIP_CHECK(hipEventRecord(fork, st[0]));
    for (int i = 1; i < (pipelined ? std::min(ns, 3) : ns); ++i) SPC_HIP_CHECK(hipStreamWaitEvent(st[i], fork, 0));
  }
  if (pipelined) return build_network_pipelined(v0_keys, n0, pi, layers, n_layers, out, st[1], ns >= 3 ? st[2] : st[1], fork);

  // ---- phase 1: all coordinate levels, each straight from V_0 (closed form, Section 5.5)
  std::map<int, Level*> levels;          // stride -> level
  std::map<int, int> level_stream;       // stride -> index of the stream that produces it
  levels[1] = borrowed_level(v0_keys, n0, 1);
  level_stream[1] = 0;
  int rc = SPC_OK, next = 0;
  for (int i = 0; i < n_layers && rc == SPC_OK; ++i) {
    const int need[2] = {layers[i].in_stride, layers[i].in_stride * layers[i].layer_stride};
    for (int j = 0; j < 2 && rc == SPC_OK; ++j) {
      if (levels.count(need[j])) continue;
      const int si = (next++) % ns;
      Level* lv = nullptr;
      rc = downsample_level(v0_keys, n0, nullptr, pi, ilog2(need[j]), &lv, st[si]);
      if (rc == SPC_OK) {
        levels[need[j]] = lv;
        level_stream[need[j]] = si;
      }
    }
  }

  std::vector<hipEvent_t> aux;
  if (fork) aux.push_back(fork);
  // Under stream capture the two-phase shape is forced: recording the free-form dependency
  // pattern (streams waiting for each other's levels) has crashed the runtime's capture on
  // ROCm 7.2, while fork / join / fork / join through streams[0] records fine.
  const bool barrier = ns > 1 && ((flags & SPC_NET_PHASE_BARRIER) || stream_is_capturing(st[0]));
  if (barrier && rc == SPC_OK) {
    // all levels complete on streams[0], then every stream continues from there
    for (int i = 1; i < ns; ++i) {
      hipEvent_t j = nullptr;
      if (hipEventCreateWithFlags(&j, hipEventDisableTiming) != hipSuccess || hipEventRecord(j, st[i]) != hipSuccess ||
          hipStreamWaitEvent(st[0], j, 0) != hipSuccess)
        rc = set_error(SPC_ERR_HIP, "joining stream %d failed", i);
      if (j) aux.push_back(j);
    }
    hipEvent_t f2 = nullptr;
    if (hipEventCreateWithFlags(&f2, hipEventDisableTiming) != hipSuccess || hipEventRecord(f2, st[0]) != hipSuccess)
      rc = set_error(SPC_ERR_HIP, "fork failed");
    if (f2) aux.push_back(f2);
    for (int i = 1; i < ns && rc == SPC_OK; ++i)
      if (hipStreamWaitEvent(st[i], f2, 0) != hipSuccess) rc = set_error(SPC_ERR_HIP, "fork failed");
  }

  // ---- phase 2: one search per distinct (K, in_stride, layer_stride, transposed)
  using Key = NetKey;
  std::map<Key, spc_kmap*> maps;
  std::map<Key, int> want = net_layouts(layers, n_layers);
  // A stream waits for each foreign event at most once (stream order covers everything it
  // enqueues later), and the other streams join streams[0] once, at the end: few, distinct
  // cross-stream edges, which is also what a graph capture of this call records.
  std::vector<std::set<hipEvent_t>> waited(ns);
  std::map<Key, int> map_stream;
  next = 0;
  for (auto& kv : want) {
    if (rc != SPC_OK) break;
    spc_layer_desc l{std::get<0>(kv.first), std::get<1>(kv.first), std::get<2>(kv.first), std::get<3>(kv.first), kv.second};
    Level* fine = levels[l.in_stride];
    Level* coarse = levels[l.in_stride * l.layer_stride];
    Level* in = l.transposed ? coarse : fine;
    Level* outl = l.transposed ? fine : coarse;
    // a transposed map goes to the stream of its strided twin (built just before it: the keys are ordered that way),
    // so that it can take the twin's pairs without a cross-stream wait
    const Key twin_key(std::get<0>(kv.first), std::get<1>(kv.first), std::get<2>(kv.first), 0);
    const int si = (l.transposed && map_stream.count(twin_key)) ? map_stream[twin_key] : (next++) % ns;
    map_stream[kv.first] = si;
    for (Level* dep : {in, outl})  // the map's stream waits for the levels it reads
      if (!barrier && dep->ready && level_stream[dep->stride] != si && waited[si].insert(dep->ready).second) {
        hipError_t e = hipStreamWaitEvent(st[si], dep->ready, 0);
        if (e != hipSuccess) rc = set_error(SPC_ERR_HIP, "hipStreamWaitEvent: %s", hipGetErrorString(e));
      }
    spc_kmap* m = nullptr;
    if (rc == SPC_OK) rc = build_network_map(kv.first, l, want, maps, fine, coarse, pi, st[si], &m);
    if (rc == SPC_OK) maps[kv.first] = m;
  }
  // join: streams[0] continues only after everything the other streams were given
  for (int i = 1; i < ns; ++i) {
    hipEvent_t j = nullptr;
    if (hipEventCreateWithFlags(&j, hipEventDisableTiming) != hipSuccess || hipEventRecord(j, st[i]) != hipSuccess ||
        hipStreamWaitEvent(st[0], j, 0) != hipSuccess)
      rc = set_error(SPC_ERR_HIP, "joining stream %d failed", i);
    if (j) aux.push_back(j);
  }
  // these events live as long as the maps (a capture of this call refers to them): the first map owns them
  if (rc == SPC_OK && !maps.empty()) maps.begin()->second->aux_events = aux;
  else
    for (hipEvent_t e : aux) (void)hipEventDestroy(e);

  if (rc == SPC_OK) {
    for (int i = 0; i < n_layers; ++i) {
      spc_kmap* m = maps[Key(layers[i].K, layers[i].in_stride, layers[i].layer_stride, layers[i].transposed)];
      m->refs++;
      out[i] = m;
    }
  }
  for (auto& kv : maps)  // drop the builder's own reference
    if (kv.second->refs.fetch_sub(1) == 1) kmap_free(kv.second);
  for (auto& kv : levels) level_unref(kv.second);
  return rc;
}

int spc_kmap_set_size_hint(spc_kmap* m, int64_t n_out_hint) {
  if (!m || n_out_hint < 0) return set_error(SPC_ERR_ARG, "map is NULL or hint < 0");
  m->n_out_hint = n_out_hint;
  return SPC_OK;
}

void spc_kmap_destroy(spc_kmap* m) {
  if (m && m->refs.fetch_sub(1) == 1) kmap_free(m);
}

int64_t spc_kmap_n_in(spc_kmap* m) {
  if (!m) return set_error(SPC_ERR_ARG, "map is NULL");
  int rc = fetch_level_n(m->in_level);
  return rc != SPC_OK ? rc : m->in_level->n_fetched;
}
int64_t spc_kmap_n_out(spc_kmap* m) {
  if (!m) return set_error(SPC_ERR_ARG, "map is NULL");
  int rc = fetch_level_n(m->out_level);
  return rc != SPC_OK ? rc : m->out_level->n_fetched;
}
int32_t spc_kmap_kvol(const spc_kmap* m) { return m ? m->K3 : SPC_ERR_ARG; }
const void* spc_kmap_out_keys(const spc_kmap* m) { return m ? m->out_level->keys : nullptr; }
const void* spc_kmap_in_keys(const spc_kmap* m) { return m ? m->in_level->keys : nullptr; }
const int32_t* spc_kmap_os_map(const spc_kmap* m) { return (m && (m->desc.layout & SPC_LAYOUT_OS)) ? m->os_map : nullptr; }

int spc_kmap_copy_out_keys(spc_kmap* m, void* keys_host, int64_t cap) {
  if (!m || !keys_host) return set_error(SPC_ERR_ARG, "NULL argument");
  SPC_RETURN_IF(wait_map(m));
  SPC_RETURN_IF(fetch_level_n(m->out_level));
  const int64_t n = m->out_level->n_fetched;
  if (cap < n) return set_error(SPC_ERR_ARG, "room for %lld keys, map has %lld", (long long)cap, (long long)n);
  if (n > 0) SPC_HIP_CHECK(hipMemcpy(keys_host, m->out_level->keys, size_t(n) * (m->pi.key_bits / 8), hipMemcpyDeviceToHost));
  return SPC_OK;
}

int spc_kmap_ws_lists(const spc_kmap* m, const int32_t** in_idx, const int32_t** out_idx, const int32_t** nnz_dev,
                      int64_t* ws_stride) {
  if (!m) return set_error(SPC_ERR_ARG, "map is NULL");
  if (!(m->desc.layout & SPC_LAYOUT_WS)) return set_error(SPC_ERR_ARG, "map was built without the WS layout");
  if (in_idx) *in_idx = m->ws_in;
  if (out_idx) *out_idx = m->ws_out;
  if (nnz_dev) *nnz_dev = m->nnz_dev;
  if (ws_stride) *ws_stride = m->ws_stride;
  return SPC_OK;
}

int spc_kmap_export_triples(spc_kmap* m, int32_t which, int32_t* triples, int64_t cap, int64_t* nnz_out) {
  if (!m || !nnz_out) return set_error(SPC_ERR_ARG, "NULL argument");
  if (which != SPC_LAYOUT_OS && which != SPC_LAYOUT_WS) return set_error(SPC_ERR_ARG, "which must be OS or WS");
  if (which == SPC_LAYOUT_WS && !(m->desc.layout & SPC_LAYOUT_WS)) return set_error(SPC_ERR_ARG, "WS layout was not built");
  if (which == SPC_LAYOUT_OS && !(m->desc.layout & SPC_LAYOUT_OS)) return set_error(SPC_ERR_ARG, "OS layout was not built");
  SPC_RETURN_IF(wait_map(m));
  SPC_RETURN_IF(fetch_level_n(m->out_level));
  const int64_t n_out = m->out_level->n_fetched;
  const int K3 = m->K3;
  int64_t nnz = 0;
  if (which == SPC_LAYOUT_OS) {
    std::vector<int32_t> M(size_t((n_out + 31) / 32) * 32 * K3);
    if (!M.empty()) SPC_HIP_CHECK(hipMemcpy(M.data(), m->os_map, M.size() * 4, hipMemcpyDeviceToHost));
    for (int k = 0; k < K3; ++k)
      for (int64_t i = 0; i < n_out && m->os_k.has(k); ++i) {  // (a hybrid map holds the dense offsets only)
        const int32_t j = M[((i >> 5) * K3 + k) * 32 + (i & 31)];
        if (j < 0) continue;
        if (nnz < cap && triples) {
          triples[3 * nnz] = k;
          triples[3 * nnz + 1] = j;
          triples[3 * nnz + 2] = static_cast<int32_t>(i);
        }
        ++nnz;
      }
  } else {
    std::vector<int32_t> cnt(K3);
    SPC_HIP_CHECK(hipMemcpy(cnt.data(), m->nnz_dev, size_t(K3) * 4, hipMemcpyDeviceToHost));
    std::vector<int32_t> a, b;
    const int kc = (K3 - 1) / 2;
    auto emit = [&](int k, int32_t in, int32_t out) {
      if (nnz < cap && triples) {
        triples[3 * nnz] = k;
        triples[3 * nnz + 1] = in;
        triples[3 * nnz + 2] = out;
      }
      ++nnz;
    };
    for (int k = 0; k < K3; ++k) {
      if (m->hybrid_t && m->os_k.has(k)) continue;  // a hybrid map keeps lists for the sparse offsets only
      // symmetric half-map: offset k > centre is the list of K^3-1-k with the roles swapped (both
      // index sequences of a list ascend, so the order by output index is kept); the centre pairs
      // every voxel with itself
      if (m->sym && k == kc) {
        for (int64_t i = 0; i < n_out; ++i) emit(k, static_cast<int32_t>(i), static_cast<int32_t>(i));
        continue;
      }
      const bool mirror = m->sym && k > kc;
      const int ks = mirror ? K3 - 1 - k : k;
      const int c = cnt[ks];
      if (c < 0 || c > m->ws_stride) return set_error(SPC_ERR_HIP, "corrupt WS count %d at offset %d", c, ks);
      a.resize(c);
      b.resize(c);
      if (c) {
        SPC_HIP_CHECK(hipMemcpy(a.data(), m->ws_in + int64_t(ks) * m->ws_stride, size_t(c) * 4, hipMemcpyDeviceToHost));
        SPC_HIP_CHECK(hipMemcpy(b.data(), m->ws_out + int64_t(ks) * m->ws_stride, size_t(c) * 4, hipMemcpyDeviceToHost));
      }
      for (int e = 0; e < c; ++e) emit(k, mirror ? b[e] : a[e], mirror ? a[e] : b[e]);
    }
  }
  *nnz_out = nnz;
  return SPC_OK;
}

int64_t spc_search_count(void) { return g_search_launches.load(std::memory_order_relaxed); }

int spc_kmap_search_info(const spc_kmap* m, int32_t* tile_rows, int32_t* window_keys) {
  if (!m) return set_error(SPC_ERR_ARG, "map is NULL");
  if (tile_rows) *tile_rows = m->tile;
  if (window_keys) *window_keys = WIN_CAP_BYTES / (m->pi.key_bits / 8);
  return SPC_OK;
}

int spc_kmap_nnz(spc_kmap* m, int64_t* nnz_host) {
  if (!m || !nnz_host) return set_error(SPC_ERR_ARG, "NULL argument");
  if (m->nnz_host.empty() || m->captured) {
    SPC_RETURN_IF(wait_map(m));
    SPC_RETURN_IF(fetch_level_n(m->out_level));
    std::vector<int64_t> cnt(m->K3, 0);
    if (m->hybrid_t) {  // dense offsets are counted in the matrix below, the others come from the lists' lengths
      std::vector<int32_t> c(m->K3);
      SPC_HIP_CHECK(hipMemcpy(c.data(), m->nnz_dev, size_t(m->K3) * 4, hipMemcpyDeviceToHost));
      const int kc = (m->K3 - 1) / 2;
      for (int k = 0; k < m->K3; ++k)
        if (!m->os_k.has(k)) cnt[k] = (m->sym && k == kc) ? m->out_level->n_fetched : c[(m->sym && k > kc) ? m->K3 - 1 - k : k];
    }
    if ((m->desc.layout & SPC_LAYOUT_WS) && !m->hybrid_t) {
      std::vector<int32_t> c(m->K3);
      SPC_HIP_CHECK(hipMemcpy(c.data(), m->nnz_dev, size_t(m->K3) * 4, hipMemcpyDeviceToHost));
      for (int k = 0; k < m->K3; ++k) cnt[k] = c[k];
      if (m->sym) {  // the second half mirrors the first, the centre pairs every voxel with itself
        const int kc = (m->K3 - 1) / 2;
        cnt[kc] = m->out_level->n_fetched;
        for (int k = kc + 1; k < m->K3; ++k) cnt[k] = cnt[m->K3 - 1 - k];
      }
    } else {
      const int64_t n_out = m->out_level->n_fetched;
      std::vector<int32_t> M(size_t((n_out + 31) / 32) * 32 * m->K3);
      if (!M.empty()) SPC_HIP_CHECK(hipMemcpy(M.data(), m->os_map, M.size() * 4, hipMemcpyDeviceToHost));
      for (int64_t i = 0; i < n_out; ++i)
        for (int k = 0; k < m->K3; ++k)
          if (m->os_k.has(k)) cnt[k] += M[((i >> 5) * m->K3 + k) * 32 + (i & 31)] >= 0;
    }
    m->nnz_host = cnt;
  }
  for (int k = 0; k < m->K3; ++k) nnz_host[k] = m->nnz_host[k];
  return SPC_OK;
}

}  // extern "C"
