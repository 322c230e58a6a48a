// Feature computation, Eq. (2): out[i,:] = sum_k F[M[i,k],:] W_k, in the
// output-stationary and the weight-stationary dataflow (Section 2.2, Section 5.4).
//
// fp16 / bf16: the per-offset contraction runs on 32x32x16 MFMA with fp32
// accumulators.  A wave owns 32-row blocks of output voxels (OS) or of (in,out)
// pairs (WS).  Gathered feature rows go straight from global memory (L2) into the
// MFMA A-operand registers: lane l needs 8 consecutive channels of row l%32, which is
// one 16-byte load, so no LDS round trip is needed for them.  The weight slice W_k is
// re-laid once per call into B-operand order and staged through LDS, where all waves
// of the workgroup read it with conflict-free 16-byte loads.
// OS skips an offset for a 32-row block when no row has a valid entry — outputs are
// spatially sorted, so emptiness is coherent (the map builder records it per block).
// fp32 (and channel counts the MFMA tiling does not cover) use plain FMA kernels.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "spc_internal.h"

namespace spc {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <typename T>
struct Mfma;
template <>
struct Mfma<_Float16> {
  using V8 = half8;
  __device__ static inline floatx16 mma(V8 a, V8 b, floatx16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
};
template <>
struct Mfma<__bf16> {
  using V8 = bf16x8;
  __device__ static inline floatx16 mma(V8 a, V8 b, floatx16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
};

template <typename T>
__device__ inline float to_f32(T v) { return static_cast<float>(v); }
template <typename T>
__device__ inline T from_f32(float v) { return static_cast<T>(v); }  // round to nearest even

// f(integral_constant<int,0>) ... f(integral_constant<int,N-1>): loops whose index must be a
// compile-time constant (register arrays that are never indexed dynamically)
template <int... S, typename Fn>
__device__ inline void static_for_impl(std::integer_sequence<int, S...>, Fn&& f) {
  (f(std::integral_constant<int, S>{}), ...);
}
template <int N, typename Fn>
__device__ inline void static_for(Fn&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

constexpr int CONV_THREADS = 256;
constexpr int CK = 64;  // input channels staged per step

// W [K3][cin][cout]  ->  Wp [K3][cin/16][cout/32][64 lanes][8]: lane l holds channels
// 16*kk + 8*(l/32) + 0..7 of output column 32*nb + l%32 (the B operand of one MFMA).
// Input channels cin_src..cin-1 (padding up to a multiple of 16) are written as zeros.
template <typename T>
__global__ __launch_bounds__(256) void prepack_weights_kernel(const T* __restrict__ W, T* __restrict__ Wp, int K3, int cin_src,
                                                              int cin, int cout) {
  const int KK = cin / 16, NB = cout / 32;
  const int64_t gid = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  const int64_t total = int64_t(K3) * KK * NB * 64;
  if (gid >= total) return;
  const int lane = gid & 63;
  int64_t t = gid >> 6;
  const int nb = t % NB;
  t /= NB;
  const int kk = t % KK;
  const int k = t / KK;
  const int c0 = kk * 16 + 8 * (lane >> 5);
  const T* src = W + (int64_t(k) * cin_src + c0) * cout + nb * 32 + (lane & 31);
  T* dst = Wp + gid * 8;
#pragma unroll
  for (int j = 0; j < 8; ++j) dst[j] = c0 + j < cin_src ? src[int64_t(j) * cout] : T(0);
}

// Feature rows padded with zeros to a multiple of 16 channels (layers such as a 4-channel stem).
template <typename T>
__global__ __launch_bounds__(256) void pad_rows_kernel(const T* __restrict__ F, int64_t ld_in, int n_h, const int* __restrict__ n_d,
                                                       int cin, int cin_pad, T* __restrict__ out) {
  const int n = n_d ? *n_d : n_h;
  const int64_t gid = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  const int64_t r = gid / cin_pad;
  const int c = static_cast<int>(gid - r * cin_pad);
  if (r < n) out[gid] = c < cin ? F[r * ld_in + c] : T(0);
}

// Shared inner step: stage nkk*NB B-fragments of offset k, channels [c0, c0+16*nkk), then
// multiply the wave's RB row blocks.  idx[rb] is the gathered input row (or -1) of lane%32.
template <typename T, int NB, int RB>
__device__ inline void contract_offset(const T* __restrict__ F, int64_t ld_in, const T* __restrict__ Wp_k, int cin,
                                       const int (&idx)[RB], bool wave_has, typename Mfma<T>::V8* sB,
                                       floatx16 (&acc)[RB][NB]) {
  using V8 = typename Mfma<T>::V8;
  const int tid = threadIdx.x, lane = tid & 63, lh = lane >> 5;
  for (int c0 = 0; c0 < cin; c0 += CK) {
    const int nkk = min(CK, cin - c0) / 16;
    if (c0 > 0) __syncthreads();  // previous chunk fully consumed
    const V8* src = reinterpret_cast<const V8*>(Wp_k) + int64_t(c0 / 16) * NB * 64;
    for (int e = tid; e < nkk * NB * 64; e += CONV_THREADS) sB[e] = src[e];
    __syncthreads();
    if (wave_has) {
      V8 a[RB][CK / 16];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int kk = 0; kk < CK / 16; ++kk) {
          V8 v = {};
          if (kk < nkk && idx[rb] >= 0) v = *reinterpret_cast<const V8*>(F + int64_t(idx[rb]) * ld_in + c0 + kk * 16 + 8 * lh);
          a[rb][kk] = v;
        }
#pragma unroll
      for (int kk = 0; kk < CK / 16; ++kk) {
        if (kk < nkk) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const V8 b = sB[(kk * NB + nb) * 64 + lane];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[rb][nb] = Mfma<T>::mma(a[rb][kk], b, acc[rb][nb]);
          }
        }
      }
    }
  }
}

// Output-stationary kernel: waves are autonomous, weights are staged through LDS in phases.
//
// A workgroup of WAVES waves walks the weight tensor once, in phases of up to HALF_BYTES.
// The phases alternate between two halves of the LDS buffer: while a phase is being
// consumed, every thread already holds its share of the next phase in registers (loaded
// before the compute started) and drops it into the other half afterwards — one barrier
// per phase, and the L2 latency of the weights is off the critical path.
// Each wave owns RB adjacent blocks of 32 consecutive output voxels and processes — on its
// own, without further synchronisation — those of its steps whose weights are resident.
// A step is one offset k with at least one valid row in the wave's blocks (the map
// builder's block masks say which) and one chunk of CKS input channels:
//   A operand: 32 gathered feature rows per block, straight from global memory into
//              registers (lane l reads 16 bytes: channels 8*(l/32)..+7 of row l%32 per
//              16-channel slab), kept in a ring of D buffers so that D-1 gathers are in
//              flight behind the one being multiplied; rows without an input voxel gather
//              from a zero row (selecting the address, not the data, keeps the loaded
//              registers untouched until use, so nothing waits on a prefetch);
//   B operand: 16-byte conflict-free LDS reads, each reused for the RB blocks;
//   MFMA 32x32x16 into fp32 accumulators that stay in registers for the whole kernel
//   (no atomics; the offset order is ascending, so results are bit-reproducible).
// Tiles (a wave's RB blocks) go to the XCDs in chunks of PHASE_XCD_CHUNK and, inside an XCD, to
// the workgroups round-robin: a workgroup's waves sit in different parts of the cloud (dense
// and sparse regions mix, which balances the CUs and the XCDs), while neighbouring blocks,
// which gather the same feature rows, run on the same XCD and share its L2.
constexpr int HALF_BYTES = 72 * 1024;  // 9 offsets of 64x64 fp16: one x-slab of a 3x3x3 kernel per phase
constexpr int KLIST_CAP = 352;  // >= 7^3
constexpr int WS_MAX_K3 = 343;  // 7^3: the largest kernel the library takes
__device__ __align__(16) uint32_t g_zero_row[64];  // zero-initialised, never written

constexpr int PHASE_XCD_CHUNK = 16;  // tiles (of two 32-row blocks) per chunk; 4 to 64 measured alike
__host__ __device__ inline int64_t phase_tiles_per_xcd(int64_t n_tiles) {
  const int64_t n_chunks = (n_tiles + PHASE_XCD_CHUNK - 1) / PHASE_XCD_CHUNK;
  return (n_chunks + 7) / 8 * PHASE_XCD_CHUNK;
}

// Workgroups per XCD: as few as hold the XCD's tiles with every wave busy, but not fewer than the XCD has
// CUs for this launch (32, shared by the slabs of output channels): one workgroup fills a CU's LDS, so a launch
// with fewer workgroups than CUs leaves CUs idle while the others gather at a fixed rate per CU; better that
// every CU runs a workgroup with some of its waves idle.
__host__ __device__ inline int phase_wgs_per_xcd(int64_t tiles_per_xcd, int waves, int n_slabs) {
  const int64_t full = (tiles_per_xcd + waves - 1) / waves;
  const int64_t spread = 32 / n_slabs > 1 ? 32 / n_slabs : 1;
  const int64_t s = spread < tiles_per_xcd ? spread : tiles_per_xcd;
  return static_cast<int>(full > s ? full : s);
}

template <typename T, int NB, int RB, int WAVES, int NKK, int D>
__global__ __launch_bounds__(64 * WAVES) void conv_os_phase_kernel(const int32_t* __restrict__ M,
                                                                   const uint32_t* __restrict__ block_masks,
                                                                   int mask_words, int n_out_h,
                                                                   const int* __restrict__ n_out_d, int K3,
                                                                   const T* __restrict__ F, int64_t ld_in,
                                                                   const T* __restrict__ Wp, T* __restrict__ out,
                                                                   int64_t ld_out, int cin, int relu, int chunks_per_phase,
                                                                   int n_wg_per_xcd, int nb_total, KMask kmask,
                                                                   const float* __restrict__ init) {
  using V8 = typename Mfma<T>::V8;
  constexpr int CKS = 16 * NKK;
  constexpr int THREADS = 64 * WAVES;
  constexpr int cout = NB * 32;
  constexpr int SV = (HALF_BYTES / 16 + THREADS - 1) / THREADS;  // staging vectors per thread per phase
  extern __shared__ __align__(16) unsigned char smem[];
  V8* sW = reinterpret_cast<V8*>(smem);
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int16_t* klist = reinterpret_cast<int16_t*>(smem + 2 * HALF_BYTES) + wave * KLIST_CAP;
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  const int64_t n_blocks = (int64_t(n_out) + 31) >> 5;
  // blockIdx.y selects a slab of NB*32 output channels; the staged weights and everything below
  // then look exactly like a layer with that many output channels
  const int slab = blockIdx.y;
  out += slab * (NB * 32);
  // tile = RB adjacent blocks; tile t -> (XCD, workgroup within the XCD, wave).  Workgroups go to the
  // XCDs round-robin, so blockIdx.x & 7 is the XCD.
  const int64_t n_tiles = (n_blocks + RB - 1) / RB;
  // The tile sequence is dealt to the XCDs in chunks of PHASE_XCD_CHUNK tiles: a chunk is long enough
  // for its gathers to stay in one XCD's L2 (neighbours in x and y are tens to hundreds of rows away
  // in the sorted order), and short enough that every XCD gets its share of the dense and of the
  // sparse regions of the scene (with one contiguous range per XCD, the XCD that held the region
  // around the sensor of a LiDAR sweep finished 7 us after the first one).
  const int64_t tiles_per_xcd = phase_tiles_per_xcd(n_tiles);
  const int xcd = blockIdx.x & 7, wg_in_xcd = blockIdx.x >> 3;
  // The grid was sized from the host's bound of the output count; the count itself may only be known
  // here.  Only as many workgroups as that count fills take part (all of their waves busy) and
  // the tiles of an XCD are dealt to them round-robin; the others leave at once.
  const int n_wg_used = phase_wgs_per_xcd(tiles_per_xcd, WAVES, gridDim.y);
  if (wg_in_xcd >= n_wg_used) return;
  const int64_t t_in_xcd = int64_t(wave) * n_wg_used + wg_in_xcd;
  const int64_t tile = ((t_in_xcd / PHASE_XCD_CHUNK) * 8 + xcd) * PHASE_XCD_CHUNK + t_in_xcd % PHASE_XCD_CHUNK;
  const bool active = t_in_xcd < tiles_per_xcd && tile < n_tiles;
  const int64_t blk0 = tile * RB;
  const int nch = cin / CKS;
  (void)n_wg_per_xcd;

  // phase 0 of the weights is requested first, so that its latency overlaps the set-up below
  const int n_chunks = K3 * nch;
  V8 st[SV];
  auto stage_load = [&](int c_lo) {
    const int hi = min(n_chunks, c_lo + chunks_per_phase);
    const int n_vec = static_cast<int>(int64_t(hi - c_lo) * CKS * cout / 8);
    // vector v of the phase, in slab view [chunk][kk][nb][lane], comes from [.][.][nb_total][lane] in memory
    const V8* src = reinterpret_cast<const V8*>(Wp);
#pragma unroll
    for (int i = 0; i < SV; ++i) {
      const int v = min(i * THREADS + tid, n_vec - 1);
      const int t = v >> 6, nbs = t % NB, kkg = t / NB;
      st[i] = src[((int64_t(c_lo) * NKK + kkg) * nb_total + slab * NB + nbs) * 64 + (v & 63)];
    }
  };
  auto stage_store = [&](int c_lo, V8* half) {
    const int hi = min(n_chunks, c_lo + chunks_per_phase);
    const int n_vec = static_cast<int>(int64_t(hi - c_lo) * CKS * cout / 8);
#pragma unroll
    for (int i = 0; i < SV; ++i)
      if (i * THREADS + tid < n_vec) half[i * THREADS + tid] = st[i];
  };
  stage_load(0);

  // offsets present in this wave's blocks: union of the blocks' masks, one word per 32 offsets,
  // parked in LDS; the positions below walk its set bits in ascending order with scalar ops
  unsigned* smask = reinterpret_cast<unsigned*>(klist);
  for (int wd = lane; wd < mask_words; wd += 64) {
    unsigned m = 0;
    if (active) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        if (blk0 + rb < n_blocks) m |= block_masks[(blk0 + rb) * mask_words + wd];
    }
    smask[wd] = m & kmask.w[wd];
  }
  __builtin_amdgcn_wave_barrier();

  floatx16 acc[RB][NB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[rb][nb][r] = 0.f;

  // A position is (mask word, remaining bits of that word, channel chunk, current offset k).
  // Positions past the end keep their last k, so that the pipeline issues the same loads every
  // step (the surplus ones are never consumed).
  struct Pos {
    int wd;
    unsigned rem;
    int ch, k;
    bool valid;
  };
  auto settle = [&](Pos& p) {
    while (p.rem == 0 && p.wd + 1 < mask_words) {
      ++p.wd;
      p.rem = __builtin_amdgcn_readfirstlane(smask[p.wd]);
    }
    if (p.rem != 0) p.k = p.wd * 32 + __builtin_ctz(p.rem);
    else p.valid = false;
  };
  auto advance = [&](Pos& p) {
    if (++p.ch == nch) {
      p.ch = 0;
      p.rem &= p.rem - 1;
      settle(p);
    }
  };
  Pos p0{0, static_cast<unsigned>(__builtin_amdgcn_readfirstlane(smask[0])), 0, 0, true};
  settle(p0);
  // a block past the end (odd tail) reads block 0's map rows; its results are never stored
  const int32_t* Mb[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) Mb[rb] = M + ((active && blk0 + rb < n_blocks) ? blk0 + rb : 0) * int64_t(K3) * 32 + lr;
  auto load_idx = [&](const Pos& p, int (&dst)[RB]) {
    const int k32 = p.k * 32;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) dst[rb] = Mb[rb][k32];
  };
  const T* zero_row = reinterpret_cast<const T*>(g_zero_row) + 8 * lh;
  auto gather = [&](const Pos& p, const int (&j)[RB], V8 (&dst)[RB][NKK]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const T* src = j[rb] < 0 ? zero_row : F + int64_t(j[rb]) * ld_in + p.ch * CKS + 8 * lh;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) dst[rb][kk] = *reinterpret_cast<const V8*>(src + kk * 16);
    }
  };

  // ring of D A-operand buffers: step u lives in buffer u % D and is refilled, once consumed,
  // with step u + D; jj[b] holds the map indices for that refill, themselves loaded D steps earlier
  V8 a[D][RB][NKK];
  int jj[D][RB];
  Pos pc = p0;  // current step
  Pos pg = p0;  // next step to gather
  Pos pi = p0;  // next step whose map indices are loaded
#pragma unroll
  for (int b = 0; b < D; ++b) {
    load_idx(pg, jj[b]);
    gather(pg, jj[b], a[b]);
    advance(pg);
  }
  pi = pg;
#pragma unroll
  for (int b = 0; b < D; ++b) {
    load_idx(pi, jj[b]);
    advance(pi);
  }

  int c_hi = 0;
  int64_t e_lo = 0;
  const V8* sWp = sW;  // LDS half of the current phase
  auto can_step = [&]() -> bool { return pc.valid && pc.k * nch + pc.ch < c_hi; };
  auto step = [&](auto B_) {
    constexpr int B = decltype(B_)::value;
    const V8* Bk = sWp + ((int64_t(pc.k) * cin + pc.ch * CKS) * cout - e_lo) / 8 + lane;
    V8 bw[NKK][NB];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) bw[kk][nb] = Bk[(kk * NB + nb) * 64];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[rb][nb] = Mfma<T>::mma(a[B][rb][kk], bw[kk][nb], acc[rb][nb]);
    gather(pg, jj[B], a[B]);
    advance(pg);
    load_idx(pi, jj[B]);
    advance(pi);
    advance(pc);
  };
  auto rotate_ring = [&]() {  // buffer 1 becomes buffer 0 (used when a phase ends off-phase; rare)
    V8 t[RB][NKK];
    int tj[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      tj[rb] = jj[0][rb];
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) t[rb][kk] = a[0][rb][kk];
    }
#pragma unroll
    for (int b = 0; b + 1 < D; ++b)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        jj[b][rb] = jj[b + 1][rb];
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) a[b][rb][kk] = a[b + 1][rb][kk];
      }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      jj[D - 1][rb] = tj[rb];
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) a[D - 1][rb][kk] = t[rb][kk];
    }
  };

  stage_store(0, sW);
  __syncthreads();
  int half = 0;
  for (int c_lo = 0; c_lo < n_chunks; c_lo += chunks_per_phase) {
    c_hi = min(n_chunks, c_lo + chunks_per_phase);
    e_lo = int64_t(c_lo) * CKS * cout;
    sWp = sW + half * (HALF_BYTES / 16);
    const bool more = c_hi < n_chunks;
    if (more) stage_load(c_hi);
    for (;;) {  // the current step always sits in buffer 0 here
      if (!can_step()) break;
      step(std::integral_constant<int, 0>{});
      if (!can_step()) { rotate_ring(); break; }
      step(std::integral_constant<int, 1>{});
      if constexpr (D == 3) {
        if (!can_step()) { rotate_ring(); rotate_ring(); break; }
        step(std::integral_constant<int, 2>{});
      }
    }
    half ^= 1;
    if (more) stage_store(c_hi, sW + half * (HALF_BYTES / 16));
    __syncthreads();  // next phase visible; everybody is done with the half it will overwrite next
  }
  // D layout of the 32x32 MFMA: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  // Row offsets are compile-time multiples of the (wave-uniform) row pitch on top of one pointer per
  // block, and full blocks skip the per-row bound check: the 64 two-byte stores of a wave then cost a
  // handful of instructions each instead of a 64-bit index computation.
  if (active) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int64_t i0 = (blk0 + rb) * 32;
      const int rows = static_cast<int>(max<int64_t>(0, min<int64_t>(32, n_out - i0)));
      if (rows == 0) continue;
      T* prow = out + (i0 + 4 * lh) * ld_out + lr;
      // hybrid dataflow: the weight-stationary part of the sum arrives in an fp32 buffer [n_out][cout]
      const int64_t ld_init = int64_t(nb_total) * 32;
      const float* irow = init + (i0 + 4 * lh) * ld_init + slab * (NB * 32) + lr;  // used only when init is given
      auto store_all = [&](auto FULL_) {
        constexpr bool FULL = decltype(FULL_)::value;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int rr = 8 * (r / 4) + (r % 4);  // row = rr + 4 * lh
            if (FULL || rr + 4 * lh < rows) {
              float v = acc[rb][nb][r];
              if (init) v += irow[rr * ld_init + nb * 32];
              if (relu) v = fmaxf(v, 0.f);
              prow[rr * ld_out + nb * 32] = from_f32<T>(v);
            }
          }
      };
      if (rows == 32) store_all(std::true_type{});
      else store_all(std::false_type{});
    }
  }
}

// Output-stationary kernel for layers whose weight traffic is small next to the chip's L2
// bandwidth (few output voxels, or few channels): one workgroup per block of 32 output voxels
// and slab of NB*32 output channels, and the offsets present in the block are dealt round-robin
// to the workgroup's four waves (a split of the reduction over k, Eq. (2)).  Nothing is staged
// through LDS and no barrier sits inside the loop: a wave reads the B fragments of its offsets
// straight from the prepacked weights (1 KB coalesced per fragment, L2-resident) next to the
// gathered A rows, D = 2 (offset, 16-channel slab) entries ahead of the MFMA that consumes them.
// The four partial accumulators meet in LDS and are summed in wave order, so results stay
// bit-reproducible; the sum leaves LDS transposed, each thread storing consecutive channels of
// one row.  Compared with the phase kernel this trades redundant weight reads (every block
// re-reads its offsets' weights) for many more, much shorter dependency chains, which is what
// the coarse levels of a network need: there a layer has fewer row blocks than the chip has
// compute units.
constexpr int SPLITK_WAVES = 4;
constexpr int SPLITK_KL_CAP = 96;  // >= ceil(7^3 / 4) + 1

// LOOP: the grid was sized from an estimate of the output count and tiles are walked with a grid
// stride; otherwise one tile per workgroup (the loop costs about 30 registers per lane).
template <typename T, int NB, int RB, int D, bool LOOP>
__global__ __launch_bounds__(64 * SPLITK_WAVES) void conv_os_splitk_kernel(const int32_t* __restrict__ M,
                                                                          const uint32_t* __restrict__ block_masks,
                                                                          int mask_words, int n_out_h,
                                                                          const int* __restrict__ n_out_d, int K3,
                                                                          const T* __restrict__ F, int64_t ld_in,
                                                                          const T* __restrict__ Wp, T* __restrict__ out,
                                                                          int64_t ld_out, int cin, int relu, int nb_total,
                                                                          int vec_store, KMask kmask,
                                                                          const float* __restrict__ init) {
  using V8 = typename Mfma<T>::V8;
  extern __shared__ __align__(16) unsigned char smem[];
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  const int64_t n_blocks = (int64_t(n_out) + 31) >> 5;
  const int slab = blockIdx.y;
  const int KK = cin / 16;
  // tiles of RB blocks; the trip count is uniform per workgroup, so the barriers below are
  // reached by all of its waves or by none
  for (int64_t blk0 = int64_t(blockIdx.x) * RB; blk0 < n_blocks; blk0 += LOOP ? int64_t(gridDim.x) * RB : n_blocks) {
  // Everything that depends on the thread index is derived anew in every trip from a value the
  // compiler cannot see through: hoisted out of the loop, the lane constants of the set-up and of the
  // epilogue would stay in registers across the whole body (26 registers, two waves per SIMD).
  int tid = threadIdx.x;
  if constexpr (LOOP) asm volatile("" : "+v"(tid));
  const int lane = tid & 63, lr = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int idx_rows = (K3 + SPLITK_WAVES - 1) / SPLITK_WAVES + 1;  // per wave, with the all-invalid row at the end
  int32_t* sIdx = reinterpret_cast<int32_t*>(smem) + wave * idx_rows * (RB * 32);
  int16_t* kl = reinterpret_cast<int16_t*>(smem + size_t(SPLITK_WAVES) * idx_rows * (RB * 128)) + wave * SPLITK_KL_CAP;

  // this wave's offsets: those present in the tile (union of the builder's block masks) whose
  // rank is wave mod 4
  int cnt = 0;
  for (int wd = 0; wd < mask_words; ++wd) {
    unsigned m = 0;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      if (blk0 + rb < n_blocks) m |= block_masks[(blk0 + rb) * mask_words + wd];
    m = __builtin_amdgcn_readfirstlane(m & kmask.w[wd]);
    if (lane < 32 && ((m >> lane) & 1u)) {
      const int rank = cnt + __builtin_popcount(m & ((1u << lane) - 1u));
      if ((rank & (SPLITK_WAVES - 1)) == wave) kl[rank / SPLITK_WAVES] = static_cast<int16_t>(wd * 32 + lane);
    }
    cnt += __builtin_popcount(m);
  }
  const int n_i = cnt > wave ? (cnt - wave + SPLITK_WAVES - 1) / SPLITK_WAVES : 0;
  if (lane == 0) kl[n_i] = 0;  // entries past the end read offset 0's weights (never multiplied)
  __builtin_amdgcn_wave_barrier();
  // their map rows (32 input indices per block), eight (offset, block) pairs per pass:
  // lane -> (pair, 4 rows); blocks past the end of the level count as all-invalid
  {
    const int part = lane & 7;
    for (int p = lane >> 3; p < n_i * RB; p += 8) {
      const int i = p / RB, rb = p % RB;
      int4 v = {-1, -1, -1, -1};
      if (blk0 + rb < n_blocks)
        v = *reinterpret_cast<const int4*>(M + ((blk0 + rb) * int64_t(K3) + kl[i]) * 32 + part * 4);
      *reinterpret_cast<int4*>(sIdx + p * 32 + part * 4) = v;
    }
    for (int q = lane; q < RB * 32; q += 64) sIdx[n_i * RB * 32 + q] = -1;
  }
  __builtin_amdgcn_wave_barrier();

  floatx16 acc[RB][NB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[rb][nb][r] = 0.f;

  // entry e = (i-th offset of this wave, 16-channel slab kk), kk fastest
  const int n_entries = n_i * KK;
  const T* zero_row = reinterpret_cast<const T*>(g_zero_row) + 8 * lh;
  const V8* Wv = reinterpret_cast<const V8*>(Wp) + int64_t(slab) * NB * 64 + lane;
  V8 a[D][RB];
  V8 b[D][NB];
  int i_n = 0, kk_n = 0;
  int idx_n[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) idx_n[rb] = sIdx[rb * 32 + lr];
  int k_n = __builtin_amdgcn_readfirstlane(static_cast<int>(kl[0]));
  auto issue = [&](auto S_) {
    constexpr int S = decltype(S_)::value;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const T* src = idx_n[rb] < 0 ? zero_row : F + int64_t(idx_n[rb]) * ld_in + kk_n * 16 + 8 * lh;
      a[S][rb] = *reinterpret_cast<const V8*>(src);
    }
    const V8* wsrc = Wv + (int64_t(k_n) * KK + kk_n) * nb_total * 64;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) b[S][nb] = wsrc[nb * 64];
    if (++kk_n == KK) {
      kk_n = 0;
      i_n = min(i_n + 1, n_i);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) idx_n[rb] = sIdx[(i_n * RB + rb) * 32 + lr];
      k_n = __builtin_amdgcn_readfirstlane(static_cast<int>(kl[i_n]));
    }
  };
  static_for<D>([&](auto S_) { issue(S_); });
  for (int e0 = 0; e0 < n_entries; e0 += D) {
    static_for<D>([&](auto S_) {
      constexpr int S = decltype(S_)::value;
      if (e0 + S < n_entries) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) acc[rb][nb] = Mfma<T>::mma(a[S][rb], b[S][nb], acc[rb][nb]);
      }
      issue(S_);
    });
  }

  // The four partial sums meet in one LDS tile (the index area is dead by now): the waves add
  // theirs in turn, last wave first.  Value (rb, nb, r, lane) sits at float
  // (((rb*NB + nb)*4 + r/4)*64 + lane)*4 + r%4, so a lane moves four registers per access.
  float4* red4 = reinterpret_cast<float4*>(smem);
  for (int w = SPLITK_WAVES - 1; w >= 0; --w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float4* p = red4 + ((rb * NB + nb) * 4 + q) * 64 + lane;
            float4 t = {acc[rb][nb][4 * q], acc[rb][nb][4 * q + 1], acc[rb][nb][4 * q + 2], acc[rb][nb][4 * q + 3]};
            if (w != SPLITK_WAVES - 1) {
              const float4 u = *p;
              t.x += u.x;
              t.y += u.y;
              t.z += u.z;
              t.w += u.w;
            }
            *p = t;
          }
    }
  }
  __syncthreads();
  // D layout of the 32x32 MFMA: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  // Thread t stores EPT consecutive channels of row t/8 of every block.
  constexpr int EPT = NB * 4;
  const float* red = reinterpret_cast<const float*>(smem);
  const int row = tid >> 3, c0 = (tid & 7) * EPT;
  const int nb = c0 >> 5, cc = c0 & 31;
  const int q = row >> 3, h = (row & 7) >> 2, rr = row & 3;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int64_t i = (blk0 + rb) * 32 + row;
    const float* p = red + ((((rb * NB + nb) * 4 + q) * 64) + h * 32 + cc) * 4 + rr;
    T o[EPT];
    // hybrid dataflow: the weight-stationary part of the sum arrives in an fp32 buffer [n_out][cout]
    const float* ip = (init && i < n_out) ? init + i * (nb_total * 32) + slab * (NB * 32) + c0 : nullptr;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      float v = p[4 * j];
      if (ip) v += ip[j];
      o[j] = from_f32<T>(relu ? fmaxf(v, 0.f) : v);
    }
    if (i < n_out) {
      T* dst = out + i * ld_out + slab * (NB * 32) + c0;
      if (vec_store) {
        if constexpr (EPT == 8) *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(o);
        else *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(o);
      } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j) dst[j] = o[j];
      }
    }
  }
  if constexpr (LOOP) __syncthreads();  // the LDS tile is reused as the next tile's index area
  }
}

// Weight-stationary: workgroup = one offset k and 4 x RB blocks of 32 (in,out) pairs;
// partial sums are merged into an fp32 buffer with hardware float atomics.  On a symmetric
// half-map every pair block is used twice: as stored with W_k, and with input and output
// swapped with the weights of the opposite offset (Section 5.4).
template <typename T, int NB, int RB>
__global__ __launch_bounds__(CONV_THREADS) void conv_ws_mfma_kernel(const int32_t* __restrict__ ws_in,
                                                                    const int32_t* __restrict__ ws_out,
                                                                    const int32_t* __restrict__ nnz, int64_t ws_stride,
                                                                    const T* __restrict__ F, int64_t ld_in,
                                                                    const T* __restrict__ Wp, float* __restrict__ accum,
                                                                    int cin, KMask kmask, int sym, int K3, int n_out_h,
                                                                    const int* __restrict__ n_out_d) {
  using V8 = typename Mfma<T>::V8;
  constexpr int WROWS = 32 * RB, TROWS = 4 * WROWS;
  extern __shared__ __align__(16) unsigned char smem[];
  V8* sB = reinterpret_cast<V8*>(smem);
  __shared__ int s_out[TROWS], s_in[TROWS];
  __shared__ int s_first[WS_MAX_K3 + 1];  // first work item of every offset; [n_k] = number of items
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, lh = lane >> 5;
  // The list lengths only exist on the device, so the grid cannot be cut to the work: a fixed number of
  // workgroups walks the items (offset k, chunk of TROWS pairs) with a grid stride.  Every workgroup
  // numbers the items itself: chunks per offset, scanned by wave 0.
  // symmetric half-map: lists exist for k < centre; the centre offset pairs every voxel with itself
  const int kc = (K3 - 1) / 2;
  const int n_k = sym ? kc + 1 : K3;
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  if (wave == 0) {
    int carry = 0;
    for (int k0 = 0; k0 < n_k; k0 += 64) {
      const int k = k0 + lane;
      int c = 0;
      if (k < n_k && kmask.has(k)) c = ((sym && k == kc ? n_out : nnz[k]) + TROWS - 1) / TROWS;
      int x = c;
      for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
      }
      if (k < n_k) s_first[k] = carry + x - c;
      carry += __shfl(x, 63, 64);
    }
    if (lane == 0) s_first[n_k] = carry;
  }
  __syncthreads();
  const int n_items = s_first[n_k];
  const int cout = NB * 32;
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
  // last offset whose first item is <= item (offsets without items share their successor's first item)
  int k = 0;
  for (int bit = 256; bit > 0; bit >>= 1)
    if (k + bit < n_k && s_first[k + bit] <= item) k += bit;
  const bool centre = sym && k == kc;
  const int cnt = centre ? n_out : nnz[k];
  const int p0 = (item - s_first[k]) * TROWS;
  const int rows = min(TROWS, cnt - p0);
  const int32_t* li = ws_in + int64_t(k) * ws_stride + p0;
  const int32_t* lo = ws_out + int64_t(k) * ws_stride + p0;
  __syncthreads();  // everybody is done with the item before (its index lists and its weights)
  for (int r = tid; r < TROWS; r += CONV_THREADS) {
    s_out[r] = r < rows ? (centre ? p0 + r : lo[r]) : -1;
    s_in[r] = r < rows ? (centre ? p0 + r : li[r]) : -1;
  }
  __syncthreads();
  // pass 0: F[in] W_k -> out.  pass 1 (symmetric maps, not the centre): F[out] W_{K^3-1-k} -> in
  const int passes = (sym && !centre) ? 2 : 1;
  for (int pass = 0; pass < passes; ++pass) {
    const int* gat = pass == 0 ? s_in : s_out;
    const int* sca = pass == 0 ? s_out : s_in;
    const int kw = pass == 0 ? k : K3 - 1 - k;
    floatx16 acc[RB][NB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][nb][r] = 0.f;
    int idx[RB];
    bool has = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      idx[rb] = gat[wave * WROWS + rb * 32 + lr];
      has |= idx[rb] >= 0;
    }
    const bool wave_has = __ballot(has) != 0ull;
    if (pass > 0) __syncthreads();  // everybody is done with the weights of the pass before
    contract_offset<T, NB, RB>(F, ld_in, Wp + int64_t(kw) * cin * cout, cin, idx, wave_has, sB, acc);
    if (!wave_has) continue;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = wave * WROWS + rb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
        const int o = sca[row];
        if (o >= 0) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) unsafeAtomicAdd(accum + int64_t(o) * cout + nb * 32 + lr, acc[rb][nb][r]);
        }
      }
  }
  }  // items
}

// ---------------------------------------------------------------- plain FMA kernels
template <typename T>
__global__ __launch_bounds__(256) void conv_os_simple_kernel(const int32_t* __restrict__ M, int n_out_h,
                                                             const int* __restrict__ n_out_d, int K3,
                                                             const T* __restrict__ F, int64_t ld_in,
                                                             const T* __restrict__ W, T* __restrict__ out,
                                                             int64_t ld_out, int cin, int cout, int relu, KMask kmask,
                                                             const float* __restrict__ init) {
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  const int64_t gid = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  const int64_t i = gid / cout;
  const int co = static_cast<int>(gid - i * cout);
  if (i >= n_out) return;
  float acc = init ? init[gid] : 0.f;
  // map entries are fetched eight offsets at a time, so that their loads (and then the feature
  // rows') are in flight together instead of one dependent chain per offset
  const int32_t* Mi = M + (i >> 5) * int64_t(K3) * 32 + (i & 31);
  for (int k0 = 0; k0 < K3; k0 += 8) {
    int j[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int k = k0 + u;
      j[u] = (k < K3 && kmask.has(k)) ? Mi[k * 32] : -1;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (j[u] < 0) continue;
      const T* f = F + int64_t(j[u]) * ld_in;
      const T* w = W + int64_t(k0 + u) * cin * cout + co;
#pragma unroll 8
      for (int ci = 0; ci < cin; ++ci) acc = fmaf(to_f32(f[ci]), to_f32(w[int64_t(ci) * cout]), acc);
    }
  }
  if (relu) acc = fmaxf(acc, 0.f);
  out[i * ld_out + co] = from_f32<T>(acc);
}

template <typename T>
__global__ __launch_bounds__(256) void conv_ws_simple_kernel(const int32_t* __restrict__ ws_in,
                                                             const int32_t* __restrict__ ws_out,
                                                             const int32_t* __restrict__ nnz, int64_t ws_stride,
                                                             const T* __restrict__ F, int64_t ld_in,
                                                             const T* __restrict__ W, float* __restrict__ accum,
                                                             int cin, int cout, KMask kmask, int sym, int K3, int n_out_h,
                                                             const int* __restrict__ n_out_d) {
  const int k = blockIdx.y;
  if (!kmask.has(k)) return;
  const int kc = (K3 - 1) / 2;
  const bool centre = sym && k == kc;
  const int64_t gid = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  const int64_t p = gid / cout;
  const int co = static_cast<int>(gid - p * cout);
  if (p >= (centre ? (n_out_d ? *n_out_d : n_out_h) : nnz[k])) return;
  const int j = centre ? static_cast<int>(p) : ws_in[int64_t(k) * ws_stride + p];
  const int o = centre ? static_cast<int>(p) : ws_out[int64_t(k) * ws_stride + p];
  const int passes = (sym && !centre) ? 2 : 1;  // second pass: the opposite offset, roles swapped
  for (int pass = 0; pass < passes; ++pass) {
    const T* f = F + int64_t(pass == 0 ? j : o) * ld_in;
    const T* w = W + int64_t(pass == 0 ? k : K3 - 1 - k) * cin * cout + co;
    float acc = 0.f;
    for (int ci = 0; ci < cin; ++ci) acc = fmaf(to_f32(f[ci]), to_f32(w[int64_t(ci) * cout]), acc);
    unsafeAtomicAdd(accum + int64_t(pass == 0 ? o : j) * cout + co, acc);
  }
}

__global__ __launch_bounds__(256) void zero_f32_kernel(float4* __restrict__ p, int64_t n4) {
  const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (i < n4) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

template <typename T>
__global__ __launch_bounds__(256) void finalize_kernel(const float* __restrict__ accum, int n_out_h,
                                                       const int* __restrict__ n_out_d, int cout, T* __restrict__ out,
                                                       int64_t ld_out, int relu) {
  const int n_out = n_out_d ? *n_out_d : n_out_h;
  const int64_t gid = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  const int64_t i = gid / cout;
  const int co = static_cast<int>(gid - i * cout);
  if (i >= n_out) return;
  float v = accum[gid];
  if (relu) v = fmaxf(v, 0.f);
  out[i * ld_out + co] = from_f32<T>(v);
}

// ---------------------------------------------------------------- dispatch
struct ConvArgs {
  int packed;
  spc_kmap* m;
  const void* F;
  int64_t ld_in;
  const void* W;
  void* out;
  int64_t ld_out;
  int cin, cout, relu, dataflow;
  int os_variant;  // 0: chosen from the layer's size, 1: phase kernel, 2: split-k kernel
  int splitk_rb;   // 0: chosen from the layer's size, else row blocks per workgroup (1, 2)
  int n_out_h;
  const int* n_out_d;
  int64_t rows_cap;  // upper bound of the output rows (exact when the host knows the count)
  int64_t rows_sel;  // best host-side estimate of the output rows: kernel selection and launch shape only
  KMask os_mask, ws_mask;  // offsets of the output-stationary / weight-stationary part
  bool any_os, any_ws;
  hipStream_t s;
};

// OS: one grid row of workgroups per slab of NB*32 output channels (NB = 2, or 1 when cout is an
// odd multiple of 32).  Small slabs keep the accumulators of two row blocks in registers and give
// the coarse, wide layers of a network enough workgroups to fill the chip.
template <typename T, int NB>
static void launch_os_mfma(const ConvArgs& a, const T* Wp, const float* init) {
  // 64-column slabs: sixteen waves with one row block each (twice the gathers in flight per CU; measured
  // 8-23 % faster than eight waves with two blocks on 120 k and 240 k voxels, 64..256 channels);
  // 32-column slabs: eight waves with two blocks (each weight fragment read from LDS serves both)
  constexpr int WAVES = NB == 2 ? 16 : 8;
  constexpr int RBK = NB == 2 ? 1 : 2;  // row blocks per wave
  constexpr int DEPTH = 2;
  const int nb_total = a.cout / 32, n_slabs = nb_total / NB;
  const int64_t n_blocks = (a.rows_cap + 31) / 32;
  const int64_t n_tiles = (n_blocks + RBK - 1) / RBK;
  const int64_t tiles_per_xcd = phase_tiles_per_xcd(n_tiles);
  const int per_xcd = phase_wgs_per_xcd(tiles_per_xcd, WAVES, n_slabs);
  const size_t lds = 2 * HALF_BYTES + size_t(WAVES) * KLIST_CAP * 2;
  auto go = [&](auto NKK_) {
    constexpr int NKK = decltype(NKK_)::value;
    const int cpp = std::max(1, HALF_BYTES / (16 * NKK * NB * 32 * int(sizeof(T))));
    // once per instantiation (initialisation of a local static is thread-safe); a failure shows up as a failed launch
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_os_phase_kernel<T, NB, RBK, WAVES, NKK, DEPTH>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    (void)attr;
    hipLaunchKernelGGL((conv_os_phase_kernel<T, NB, RBK, WAVES, NKK, DEPTH>), dim3(per_xcd * 8, n_slabs), dim3(64 * WAVES), lds,
                       a.s, a.m->os_map, a.m->block_masks, a.m->mask_words, a.n_out_h, a.n_out_d, a.m->K3,
                       static_cast<const T*>(a.F), a.ld_in, Wp, static_cast<T*>(a.out), a.ld_out, a.cin, a.relu, cpp, per_xcd,
                       nb_total, a.os_mask, init);
  };
  if (a.cin % 64 == 0) go(std::integral_constant<int, 4>{});
  else if (a.cin % 32 == 0) go(std::integral_constant<int, 2>{});
  else go(std::integral_constant<int, 1>{});
}

static size_t splitk_lds_bytes(int K3, int NB, int RB) {
  const int idx_rows = (K3 + SPLITK_WAVES - 1) / SPLITK_WAVES + 1;
  return std::max(size_t(SPLITK_WAVES) * idx_rows * RB * 128 + size_t(SPLITK_WAVES) * SPLITK_KL_CAP * 2,
                  size_t(RB) * NB * 16 * 64 * 4);
}

template <typename T, int NB, int RB>
static void launch_os_splitk(const ConvArgs& a, const T* Wp, const float* init) {
  // entries in flight per wave: two.  Deeper rings cost the registers that hold more waves per SIMD, and the
  // waves hide more latency than the ring does (25 layers of a UNet on 120 k voxels, all on this kernel: 403 us
  // summed with 6-12 entries, 352 us with two or three, 391 us with one)
  constexpr int D = 2;
  const int nb_total = a.cout / 32, n_slabs = nb_total / NB;
  // an estimated output count sizes the grid of the variant that walks tiles with a grid stride
  const bool loop = a.rows_sel != a.rows_cap;
  const int64_t n_blocks = std::max<int64_t>((a.rows_sel + 31) / 32, 1);
  const size_t lds = splitk_lds_bytes(a.m->K3, NB, RB);
  // once per instantiation: both variants may use all of a CU's LDS (large kernels need more than the default 64 KB)
  static const hipError_t attr = [] {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_os_splitk_kernel<T, NB, RB, D, false>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    const hipError_t f = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_os_splitk_kernel<T, NB, RB, D, true>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return e != hipSuccess ? e : f;
  }();
  (void)attr;
  constexpr int EPT = NB * 4;
  T* out = static_cast<T*>(a.out);
  const int vec = a.ld_out % EPT == 0 && reinterpret_cast<uintptr_t>(out) % (EPT * sizeof(T)) == 0;
  const dim3 grid(static_cast<unsigned>((n_blocks + RB - 1) / RB), n_slabs);
  if (loop)
    hipLaunchKernelGGL((conv_os_splitk_kernel<T, NB, RB, D, true>), grid, dim3(64 * SPLITK_WAVES), lds, a.s, a.m->os_map,
                       a.m->block_masks, a.m->mask_words, a.n_out_h, a.n_out_d, a.m->K3, static_cast<const T*>(a.F), a.ld_in, Wp,
                       out, a.ld_out, a.cin, a.relu, nb_total, vec, a.os_mask, init);
  else
    hipLaunchKernelGGL((conv_os_splitk_kernel<T, NB, RB, D, false>), grid, dim3(64 * SPLITK_WAVES), lds, a.s, a.m->os_map,
                       a.m->block_masks, a.m->mask_words, a.n_out_h, a.n_out_d, a.m->K3, static_cast<const T*>(a.F), a.ld_in, Wp,
                       out, a.ld_out, a.cin, a.relu, nb_total, vec, a.os_mask, init);
}

// Row blocks per workgroup of the split-k kernel: more blocks share each weight fragment read
// (less L2 traffic) but leave fewer workgroups and cost registers; one block measured faster than two
// at every size (120 k voxels 64->64: 37.4 vs 39.1 us; 240 k voxels 5x5x5 32->32: 37.7 vs 47.7), so two
// is only taken on request.
static int splitk_rb(const ConvArgs& a, int NB) {
  int rb = a.splitk_rb ? a.splitk_rb : 1;
  while (rb > 1 && splitk_lds_bytes(a.m->K3, NB, rb) > 80 * 1024) rb >>= 1;
  return rb;
}

template <typename T, int NB>
static void launch_os_splitk_any(const ConvArgs& a, const T* Wp, const float* init) {
  switch (splitk_rb(a, NB)) {
    case 2: launch_os_splitk<T, NB, 2>(a, Wp, init); break;
    default: launch_os_splitk<T, NB, 1>(a, Wp, init); break;
  }
}

// Measured crossover on MI355X (3x3x3 layers, 32..256 channels, 18 k / 49 k / 120 k voxels).  The phase
// kernel stages every weight once per sixteen row blocks and wins where that matters: enough tiles for
// 64 sixteen-wave workgroups (per slab of output channels; they are dealt to up to 256 workgroups, see
// phase_wgs_per_xcd) and enough input channels behind every tile.  Below that the split-k kernel's many
// short workgroups win in spite of their redundant weight reads: us, phase / split-k, 49 k voxels
// 32->64 15.2 / 11.6, 64->64 19.4 / 19.1, 64->128 25.5 / 30.6; 18 k voxels 64->64 17.5 / 10.7, 128->128
// 29.7 / 28.8, 128->256 38.8 / 46.5; 120 k voxels 32->64 20.6 / 22.9, 64->64 30.5 / 37.3.  With 32-column
// slabs the split-k kernel wins or ties at every size measured (32->32: 120 k voxels 18.8 / 15.6, 10^6
// voxels 118 / 80, 3 * 10^6 voxels 359 / 269; 64->32 at 120 k voxels 27.6 / 27.4).  Large kernels (5x5x5
// and up) favour the split-k kernel at every size measured.
static bool prefer_splitk(const ConvArgs& a) {
  const int64_t n_blocks = (a.rows_sel + 31) / 32;
  const int n_slabs = a.cout % 64 == 0 ? a.cout / 64 : a.cout / 32;
  const int64_t wgs = (n_blocks + 15) / 16 * n_slabs;
  if (a.m->K3 > 64 || wgs < 64 || a.cout % 64 != 0) return true;
  return wgs * a.cin < 7000;
}

template <typename T, int NB, int RB>
static void launch_ws_mfma(const ConvArgs& a, const T* Wp, float* accum) {
  constexpr int TROWS = 128 * RB;
  const size_t lds = size_t(CK / 16) * NB * 64 * 16;
  // at most this many items exist (every offset's list holds at most one pair per output row); the grid stops
  // at a few workgroups per CU and strides
  const int gy = a.m->sym ? (a.m->K3 - 1) / 2 + 1 : a.m->K3;  // a symmetric map is walked up to the centre offset
  const int64_t max_items = ((a.rows_cap + TROWS - 1) / TROWS) * gy;
  const int gx = static_cast<int>(std::min<int64_t>(max_items, 2048));
  hipLaunchKernelGGL((conv_ws_mfma_kernel<T, NB, RB>), dim3(gx), dim3(CONV_THREADS), lds, a.s, a.m->ws_in, a.m->ws_out,
                     a.m->nnz_dev, a.m->ws_stride, static_cast<const T*>(a.F), a.ld_in, Wp, accum, a.cin, a.ws_mask,
                     a.m->sym ? 1 : 0, a.m->K3, a.n_out_h, a.n_out_d);
}

// Shapes the MFMA kernels run (16-bit types): input channels a multiple of 16 (smaller or ragged
// counts are zero-padded by the caller below), output channels a multiple of 32 for the OS
// part and one of 32/64/128/256 for the WS part.
static bool mfma_shape(int cin, int cout, bool any_ws) {
  if (cin % 16 != 0 || cout % 32 != 0) return false;
  return !any_ws || cout == 32 || cout == 64 || cout == 128 || cout == 256;
}

// The weight-stationary part (if any) accumulates into an fp32 buffer first; the output-stationary
// part (if any) then starts from that buffer and writes the layer's output, otherwise a small
// kernel rounds the buffer.
template <typename T>
static int conv_typed(const ConvArgs& a0, bool allow_mfma) {
  ConvArgs a = a0;
  const int K3 = a.m->K3;
  const int64_t out_elems = a.rows_cap * a.cout;
  const bool aligned = a.ld_in % 8 == 0 && reinterpret_cast<uintptr_t>(a.F) % 16 == 0;
  const int cin_pad = (a.cin + 15) / 16 * 16;
  if (a.packed && !(allow_mfma && mfma_shape(cin_pad, a.cout, a.any_ws)))
    return set_error(SPC_ERR_ARG, "packed weights given for a shape the MFMA kernels do not run");
  if (a.rows_cap <= 0) return SPC_OK;
  // ragged input channel counts and unaligned rows go through a zero-padded copy of the features
  // (prepacked weights already hold zeros for the padding channels)
  const bool repack_rows = cin_pad != a.cin || !aligned;
  const bool use_mfma = allow_mfma && mfma_shape(cin_pad, a.cout, a.any_ws);
  float* accum = nullptr;
  if (a.any_ws) {
    accum = static_cast<float*>(pool_alloc(std::max<size_t>(size_t(out_elems) * 4 + 16, 256), a.s));
    if (!accum) return SPC_ERR_NOMEM;
    const int64_t n4 = (out_elems + 3) / 4;
    hipLaunchKernelGGL(zero_f32_kernel, dim3((n4 + 255) / 256), dim3(256), 0, a.s, reinterpret_cast<float4*>(accum), n4);
  }
  const float* init = a.any_os ? accum : nullptr;  // what the OS part starts from
  int rc = SPC_OK;
  if constexpr (!std::is_same<T, float>::value) {
    if (use_mfma) {
      T* Fpad = nullptr;
      if (repack_rows) {
        const Level* il = a.m->in_level;
        const int64_t rows_in = il->n_host < 0 ? il->cap : il->n_host;
        Fpad = static_cast<T*>(pool_alloc(std::max<size_t>(size_t(rows_in) * cin_pad * sizeof(T), 256), a.s));
        if (!Fpad) {
          pool_free(accum, a.s);
          return SPC_ERR_NOMEM;
        }
        const int64_t total = rows_in * cin_pad;
        if (total > 0)
          hipLaunchKernelGGL(pad_rows_kernel<T>, dim3((total + 255) / 256), dim3(256), 0, a.s, static_cast<const T*>(a.F), a.ld_in,
                             static_cast<int>(il->n_host < 0 ? 0 : il->n_host), il->n_host < 0 ? il->n_dev : nullptr, a.cin, cin_pad,
                             Fpad);
        a.F = Fpad;
        a.ld_in = cin_pad;
      }
      const T* Wp = static_cast<const T*>(a.W);
      T* Wtmp = nullptr;
      if (!a.packed) {
        Wtmp = static_cast<T*>(pool_alloc(size_t(K3) * cin_pad * a.cout * sizeof(T), a.s));
        if (!Wtmp) {
          pool_free(accum, a.s);
          pool_free(Fpad, a.s);
          return SPC_ERR_NOMEM;
        }
        const int64_t total = int64_t(K3) * (cin_pad / 16) * (a.cout / 32) * 64;
        hipLaunchKernelGGL(prepack_weights_kernel<T>, dim3((total + 255) / 256), dim3(256), 0, a.s, static_cast<const T*>(a.W),
                           Wtmp, K3, a.cin, cin_pad, a.cout);
        Wp = Wtmp;
      }
      a.cin = cin_pad;
      if (a.any_ws) {
        switch (a.cout) {
          case 32: launch_ws_mfma<T, 1, 2>(a, Wp, accum); break;
          case 64: launch_ws_mfma<T, 2, 2>(a, Wp, accum); break;
          case 128: launch_ws_mfma<T, 4, 1>(a, Wp, accum); break;
          case 256: launch_ws_mfma<T, 8, 1>(a, Wp, accum); break;
        }
      }
      if (a.any_os) {
        const bool splitk = a.os_variant == 2 || (a.os_variant == 0 && prefer_splitk(a));
        if (splitk) {
          if (a.cout % 64 == 0) launch_os_splitk_any<T, 2>(a, Wp, init);
          else launch_os_splitk_any<T, 1>(a, Wp, init);
        } else {
          if (a.cout % 64 == 0) launch_os_mfma<T, 2>(a, Wp, init);
          else launch_os_mfma<T, 1>(a, Wp, init);
        }
      }
      // reuse of these blocks is ordered behind this stream's work
      pool_free(Wtmp, a.s);
      pool_free(Fpad, a.s);
    }
  }
  if (!use_mfma) {
    // nnz[k] <= n_out for every offset
    if (a.any_ws)
      hipLaunchKernelGGL(conv_ws_simple_kernel<T>, dim3((out_elems + 255) / 256, a.m->sym ? (K3 - 1) / 2 + 1 : K3), dim3(256), 0,
                         a.s, a.m->ws_in, a.m->ws_out, a.m->nnz_dev, a.m->ws_stride, static_cast<const T*>(a.F), a.ld_in,
                         static_cast<const T*>(a.W), accum, a.cin, a.cout, a.ws_mask, a.m->sym ? 1 : 0, K3, a.n_out_h, a.n_out_d);
    if (a.any_os)
      hipLaunchKernelGGL(conv_os_simple_kernel<T>, dim3((out_elems + 255) / 256), dim3(256), 0, a.s, a.m->os_map, a.n_out_h,
                         a.n_out_d, K3, static_cast<const T*>(a.F), a.ld_in, static_cast<const T*>(a.W), static_cast<T*>(a.out),
                         a.ld_out, a.cin, a.cout, a.relu, a.os_mask, init);
  }
  if (!a.any_os)
    hipLaunchKernelGGL(finalize_kernel<T>, dim3((out_elems + 255) / 256), dim3(256), 0, a.s, accum, a.n_out_h, a.n_out_d, a.cout,
                       static_cast<T*>(a.out), a.ld_out, a.relu);
  pool_free(accum, a.s);
  if (hipGetLastError() != hipSuccess) rc = set_error(SPC_ERR_HIP, "feature kernel launch failed");
  return rc;
}

// Common part of the two entry points: offsets with L1 norm < t run output-stationary, the others
// weight-stationary.
static int conv_entry(spc_kmap* m, const void* feats_in, int64_t ld_in, const void* weights, void* feats_out, int64_t ld_out,
                      int32_t cin, int32_t cout, int32_t dtype, int32_t t, int32_t flags, void* stream) {
  if (!m || !feats_in || !weights || !feats_out) return set_error(SPC_ERR_ARG, "NULL argument");
  if (cin < 1 || cout < 1 || ld_in < cin || ld_out < cout) return set_error(SPC_ERR_ARG, "bad channel counts or row pitches");
  ConvArgs a{};
  a.m = m;
  for (int k = 0; k < m->K3; ++k) {
    const bool dense = offset_l1(m->desc.K, k) < t;
    (dense ? a.os_mask : a.ws_mask).w[k >> 5] |= 1u << (k & 31);
    (dense ? a.any_os : a.any_ws) = true;
  }
  if (a.any_os && !(m->desc.layout & SPC_LAYOUT_OS)) return set_error(SPC_ERR_ARG, "map has no OS layout");
  if (a.any_ws && !(m->desc.layout & SPC_LAYOUT_WS)) return set_error(SPC_ERR_ARG, "map has no WS layout");
  // a map built for one threshold of the hybrid dual dataflow holds every offset in one layout only
  for (int k = 0; k < m->K3 && m->hybrid_t; ++k) {
    const bool dense = a.os_mask.has(k);
    const int ks = (m->sym && k > (m->K3 - 1) / 2) ? m->K3 - 1 - k : k;  // a symmetric map derives the second half
    const bool have = dense ? m->os_k.has(k) : (m->ws_k.has(ks) || (m->sym && k == (m->K3 - 1) / 2));
    if (!have)
      return set_error(SPC_ERR_ARG, "map was built for the hybrid threshold %d: offset %d is not in the %s layout", m->hybrid_t, k,
                       dense ? "OS" : "WS");
  }
  a.F = feats_in;
  a.ld_in = ld_in;
  a.W = weights;
  a.out = feats_out;
  a.ld_out = ld_out;
  a.cin = cin;
  a.cout = cout;
  a.relu = (flags & SPC_CONV_RELU) ? 1 : 0;
  a.packed = (flags & SPC_CONV_PACKED_WEIGHTS) ? 1 : 0;
  if ((flags & SPC_CONV_OS_PHASE) && (flags & SPC_CONV_OS_SPLITK)) return set_error(SPC_ERR_ARG, "two OS kernel variants requested");
  a.os_variant = (flags & SPC_CONV_OS_PHASE) ? 1 : (flags & SPC_CONV_OS_SPLITK) ? 2 : 0;
  a.splitk_rb = (flags >> 8) & 7;  // tuning aid: SPC_CONV_OS_SPLITK | (rb << 8)
  if (a.splitk_rb != 0 && a.splitk_rb != 1 && a.splitk_rb != 2)
    return set_error(SPC_ERR_ARG, "row blocks per workgroup must be 1 or 2");
  const Level* ol = m->out_level;
  a.n_out_h = static_cast<int>(ol->n_host < 0 ? 0 : ol->n_host);
  a.n_out_d = ol->n_host < 0 ? ol->n_dev : nullptr;
  a.rows_cap = ol->n_host < 0 ? m->out_cap : ol->n_host;
  a.rows_sel = (ol->n_host < 0 && m->n_out_hint >= 0) ? std::min(m->n_out_hint, a.rows_cap) : a.rows_cap;
  a.s = static_cast<hipStream_t>(stream);
  // a map of a pipelined network build: nobody has joined its build stream, this stream waits for the map itself
  // (once per consumer stream: stream order covers the later layers that share the map)
  if (m->wait_on_use && m->ready && m->stream != a.s && m->last_waiter != a.s) {
    SPC_HIP_CHECK(hipStreamWaitEvent(a.s, m->ready, 0));
    m->last_waiter = a.s;
  }
  // remembered for spc_kmap_destroy: the build stream's cache must not hand the map's arrays out again
  // before this stream's kernels have read them
  if (a.s != m->stream && std::find(m->consumers.begin(), m->consumers.end(), a.s) == m->consumers.end())
    m->consumers.push_back(a.s);
  switch (dtype) {
    case SPC_DTYPE_F16: return conv_typed<_Float16>(a, true);
    case SPC_DTYPE_BF16: return conv_typed<__bf16>(a, true);
    case SPC_DTYPE_F32: return conv_typed<float>(a, false);
  }
  return set_error(SPC_ERR_ARG, "bad dtype");
}

}  // namespace spc

extern "C" int spc_conv_forward(spc_kmap* m, const void* feats_in, int64_t ld_in, const void* weights, void* feats_out,
                                int64_t ld_out, int32_t cin, int32_t cout, int32_t dtype, int32_t dataflow, int32_t flags,
                                void* stream) {
  if (dataflow != SPC_DATAFLOW_OS && dataflow != SPC_DATAFLOW_WS) return spc::set_error(SPC_ERR_ARG, "bad dataflow");
  // single dataflows are the two ends of the threshold range
  const int32_t t = dataflow == SPC_DATAFLOW_OS ? 0x7fffffff : 0;
  return spc::conv_entry(m, feats_in, ld_in, weights, feats_out, ld_out, cin, cout, dtype, t, flags, stream);
}

extern "C" int spc_conv_forward_hybrid(spc_kmap* m, const void* feats_in, int64_t ld_in, const void* weights, void* feats_out,
                                       int64_t ld_out, int32_t cin, int32_t cout, int32_t dtype, int32_t t, int32_t flags,
                                       void* stream) {
  if (t < 0) return spc::set_error(SPC_ERR_ARG, "threshold t must be >= 0");
  return spc::conv_entry(m, feats_in, ld_in, weights, feats_out, ld_out, cin, cout, dtype, t, flags, stream);
}

extern "C" int spc_conv_tune_threshold(spc_kmap* m, const void* feats_in, int64_t ld_in, const void* weights,
                                       const void* packed_weights, void* feats_out, int64_t ld_out, int32_t cin, int32_t cout,
                                       int32_t dtype, int32_t flags, int32_t reps, float ws_build_us, float* us_per_t,
                                       int32_t cap, int32_t* n_t, int32_t* best_t, void* stream) {
  using namespace spc;
  if (!m || !us_per_t || !n_t || !best_t || !weights) return set_error(SPC_ERR_ARG, "NULL argument");
  if (reps < 1 || reps > 1000) return set_error(SPC_ERR_ARG, "reps must be in 1..1000");
  if (flags & SPC_CONV_PACKED_WEIGHTS) return set_error(SPC_ERR_ARG, "pass prepacked weights as packed_weights, not by flag");
  if ((m->desc.layout & SPC_LAYOUT_BOTH) != SPC_LAYOUT_BOTH || m->hybrid_t)
    return set_error(SPC_ERR_ARG, "tuning needs a map that holds both layouts for every offset");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  SPC_HIP_CHECK(hipStreamIsCapturing(s, &cs));
  if (cs != hipStreamCaptureStatusNone) return set_error(SPC_ERR_UNSUPPORTED, "tuning waits for the device: not under stream capture");
  int l1_max = 0;
  for (int k = 0; k < m->K3; ++k) l1_max = std::max(l1_max, offset_l1(m->desc.K, k));
  const int count = l1_max + 2;  // t = 0 (all offsets weight-stationary) .. l1_max + 1 (all output-stationary)
  *n_t = count;
  if (cap < count) return set_error(SPC_ERR_ARG, "us_per_t holds %d entries, the layer has %d thresholds", cap, count);
  const bool mfma_shape = dtype != SPC_DTYPE_F32 && cout % 32 == 0;
  const bool ws_takes_packed = cout == 32 || cout == 64 || cout == 128 || cout == 256;
  auto run = [&](int t) {
    const bool ws_part = t <= l1_max;
    const bool packed = packed_weights && mfma_shape && (!ws_part || ws_takes_packed);
    return conv_entry(m, feats_in, ld_in, packed ? packed_weights : weights, feats_out, ld_out, cin, cout, dtype, t,
                      flags | (packed ? SPC_CONV_PACKED_WEIGHTS : 0), stream);
  };
  hipEvent_t e0 = nullptr, e1 = nullptr;
  SPC_HIP_CHECK(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return set_error(SPC_ERR_HIP, "hipEventCreate failed");
  }
  int rc = SPC_OK, best = 0;
  for (int t = 0; t < count && rc == SPC_OK; ++t) {
    rc = run(t);  // untimed: fills the block cache for this shape
    if (rc == SPC_OK && hipEventRecord(e0, s) != hipSuccess) rc = set_error(SPC_ERR_HIP, "hipEventRecord failed");
    for (int r = 0; r < reps && rc == SPC_OK; ++r) rc = run(t);
    if (rc != SPC_OK) break;
    float ms = 0.f;
    if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
      rc = set_error(SPC_ERR_HIP, "timing a threshold failed");
      break;
    }
    us_per_t[t] = ms * 1e3f / float(reps) + (t <= l1_max ? ws_build_us : 0.f);
    if (us_per_t[t] < us_per_t[best]) best = t;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != SPC_OK) return rc;
  *best_t = best;
  return run(best);  // feats_out holds the layer's output under the chosen threshold
}

extern "C" int spc_conv_prepare_weights(const void* weights, int32_t kvol, int32_t cin, int32_t cout, int32_t dtype,
                                        void* packed_out, void* stream) {
  using namespace spc;
  if (!weights || !packed_out || kvol < 1) return set_error(SPC_ERR_ARG, "NULL argument or kvol < 1");
  if ((dtype != SPC_DTYPE_F16 && dtype != SPC_DTYPE_BF16) || cin < 1 || cout < 32 || cout % 32 != 0)
    return set_error(SPC_ERR_UNSUPPORTED, "no MFMA kernel for dtype %d, cin %d, cout %d", dtype, cin, cout);
  const int cin_pad = (cin + 15) / 16 * 16;  // the padding channels are written as zeros
  const int64_t total = int64_t(kvol) * (cin_pad / 16) * (cout / 32) * 64;
  // both 16-bit types move as raw 2-byte elements
  hipLaunchKernelGGL(prepack_weights_kernel<_Float16>, dim3((total + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const _Float16*>(weights), static_cast<_Float16*>(packed_out), kvol, cin, cin_pad, cout);
  SPC_HIP_CHECK(hipGetLastError());
  return SPC_OK;
}

namespace spc {
// 16 bytes per thread: a 128-byte feature row is read and written by eight adjacent lanes.
__global__ __launch_bounds__(256) void permute_rows16_kernel(const uint4* __restrict__ src, int64_t src_pitch_v,
                                                             const int32_t* __restrict__ perm, int64_t n, int row_v,
                                                             uint4* __restrict__ dst, int64_t dst_pitch_v) {
  const int64_t gid = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  const int64_t r = gid / row_v;
  const int w = static_cast<int>(gid - r * row_v);
  if (r < n) dst[r * dst_pitch_v + w] = src[int64_t(perm[r]) * src_pitch_v + w];
}
__global__ __launch_bounds__(256) void permute_rows_kernel(const uint32_t* __restrict__ src, int64_t src_pitch_w,
                                                           const int32_t* __restrict__ perm, int64_t n, int row_w,
                                                           uint32_t* __restrict__ dst, int64_t dst_pitch_w) {
  const int64_t gid = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  const int64_t r = gid / row_w;
  const int w = static_cast<int>(gid - r * row_w);
  if (r < n) dst[r * dst_pitch_w + w] = src[int64_t(perm[r]) * src_pitch_w + w];
}
}  // namespace spc

extern "C" int spc_permute_rows(const void* src, int64_t src_pitch, const int32_t* perm, int64_t n, int64_t row_bytes, void* dst,
                                int64_t dst_pitch, void* stream) {
  using namespace spc;
  if (!src || !perm || !dst) return set_error(SPC_ERR_ARG, "NULL argument");
  if (n < 0 || row_bytes < 4 || row_bytes % 4 || src_pitch % 4 || dst_pitch % 4 || src_pitch < row_bytes || dst_pitch < row_bytes)
    return set_error(SPC_ERR_ARG, "rows and pitches must be multiples of 4 bytes, pitch >= row");
  const bool vec16 = row_bytes % 16 == 0 && src_pitch % 16 == 0 && dst_pitch % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(src) % 16 == 0 && reinterpret_cast<uintptr_t>(dst) % 16 == 0;
  const int64_t total = n * (row_bytes / (vec16 ? 16 : 4));
  if (total > 0 && vec16)
    hipLaunchKernelGGL(permute_rows16_kernel, dim3((total + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), src_pitch / 16, perm, n, static_cast<int>(row_bytes / 16),
                       static_cast<uint4*>(dst), dst_pitch / 16);
  else if (total > 0)
    hipLaunchKernelGGL(permute_rows_kernel, dim3((total + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint32_t*>(src), src_pitch / 4, perm, n, static_cast<int>(row_bytes / 4),
                       static_cast<uint32_t*>(dst), dst_pitch / 4);
  SPC_HIP_CHECK(hipGetLastError());
  return SPC_OK;
}
