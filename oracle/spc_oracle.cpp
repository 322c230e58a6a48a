// CPU oracle for the sparse-convolution (SpC) layer — TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, obviously-correct implementation of what the hot path computes,
// written from the paper's definitions.  It shares no code with the HIP library
// and is used only by the tests, the smoke check and the benchmark's CPU-baseline
// leg.  Voxels are handled as unpacked integer tuples with a std::unordered_map
// lookup; features are accumulated in fp64 in ascending offset order.
//
// Passages followed (section / equation of the paper):
//   * orc_sort_coords      — Section 5.2, "key observation": coordinates are kept
//                            lexicographically sorted; x is most significant
//                            because it occupies the top bits of a packed key
//                            (Section 5.3); the batch index ranks above x.
//   * orc_downsample       — Section 2.1, Eq. (1): V_q = floor(V_p / s_q) * s_q,
//                            unique values kept, result sorted (Section 5.2).
//   * orc_offsets          — Section 2.1: Delta(K, s_p), K^3 offsets that are
//                            multiples of s_p, e.g. Delta(5,2) = {-4,-2,0,2,4}^3;
//                            Section 5.2 fixes the order (z fastest: group 0 is
//                            (-1,-1,-1), (-1,-1,0), (-1,-1,1)).
//   * orc_kernel_map       — Section 2.2 step 1: M[i,k] = j iff p_j = q_i + delta_k,
//                            otherwise -1.
//   * orc_conv             — Section 2.1, Eq. (2).
//   * orc_pack_keys        — Section 5.3: one integer per voxel, b_x top bits for
//                            x, then b_y bits for y, then b_z bits for z.
//   * orc_kernel_map_transposed / even K — not defined in the paper; readings are
//                            stated at the functions.
//
// Every function is pinned by CPU tests against something other than itself
// (brute force, closed forms on full grids, dense convolution, hand-worked cases).
#include <algorithm>
#include <array>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

using Coord = std::array<int32_t, 4>;  // (b, x, y, z)

struct CoordHash {
  size_t operator()(const Coord& c) const noexcept {
    uint64_t h = 0xcbf29ce484222325ull;
    for (int32_t v : c) {
      h ^= static_cast<uint32_t>(v);
      h *= 0x100000001b3ull;
      h ^= h >> 29;
    }
    return static_cast<size_t>(h);
  }
};

inline int64_t floor_div(int64_t a, int64_t b) {  // b > 0, rounds toward -infinity
  int64_t q = a / b;
  if ((a % b != 0) && (a < 0)) --q;
  return q;
}

inline Coord load(const int32_t* p) { return Coord{p[0], p[1], p[2], p[3]}; }

// Offsets per axis for kernel size K and input stride s_p.
//   odd K : (i - (K-1)/2) * s_p, i = 0..K-1             (Section 2.1 example)
//   even K: i * s_p, i = 0..K-1  — reading for the 2x2x2 stride-2 layers of
//           UNet-style stacks, which the paper does not spell out: it is the
//           choice under which a stride-2 layer equals a dense stride-2,
//           zero-padding convolution.
inline int32_t axis_offset(int K, int s_p, int i) {
  return (K % 2 == 1) ? (i - (K - 1) / 2) * s_p : i * s_p;
}

}  // namespace

extern "C" {

int orc_num_threads() {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
  omp_set_num_threads(n);
#else
  (void)n;
#endif
}

// perm[r] = index (into the caller's rows) of the r-th smallest coordinate in
// lexicographic (b, x, y, z) order.  Returns 0, or 1 if two rows are equal.
int orc_sort_coords(const int32_t* coords, int64_t n, int64_t* perm) {
  std::vector<int64_t> idx(n);
  for (int64_t i = 0; i < n; ++i) idx[i] = i;
  std::sort(idx.begin(), idx.end(), [&](int64_t a, int64_t b) {
    return load(coords + 4 * a) < load(coords + 4 * b);
  });
  int dup = 0;
  for (int64_t i = 0; i < n; ++i) {
    perm[i] = idx[i];
    if (i && load(coords + 4 * idx[i]) == load(coords + 4 * idx[i - 1])) dup = 1;
  }
  return dup;
}

// Eq. (1): every spatial component is replaced by floor(v / s_q) * s_q, the
// batch index is untouched, duplicates are dropped and the result is sorted.
// `out` must hold n rows; returns the number of output voxels.
int64_t orc_downsample(const int32_t* coords, int64_t n, int32_t s_q, int32_t* out) {
  std::vector<Coord> v(n);
  for (int64_t i = 0; i < n; ++i) {
    Coord c = load(coords + 4 * i);
    for (int a = 1; a < 4; ++a) c[a] = static_cast<int32_t>(floor_div(c[a], s_q) * s_q);
    v[i] = c;
  }
  std::sort(v.begin(), v.end());
  v.erase(std::unique(v.begin(), v.end()), v.end());
  for (size_t i = 0; i < v.size(); ++i) std::memcpy(out + 4 * i, v[i].data(), 16);
  return static_cast<int64_t>(v.size());
}

// offsets[k] = (dx, dy, dz) with k = (ix*K + iy)*K + iz (z fastest).
void orc_offsets(int32_t K, int32_t s_p, int32_t* offsets) {
  for (int ix = 0; ix < K; ++ix)
    for (int iy = 0; iy < K; ++iy)
      for (int iz = 0; iz < K; ++iz) {
        int k = (ix * K + iy) * K + iz;
        offsets[3 * k + 0] = axis_offset(K, s_p, ix);
        offsets[3 * k + 1] = axis_offset(K, s_p, iy);
        offsets[3 * k + 2] = axis_offset(K, s_p, iz);
      }
}

// Kernel map: M[i*K^3 + k] = j iff in[j] == out[i] + delta_k (same batch), else -1.
// The index of a voxel is its row in the arrays passed in (callers pass sorted rows).
void orc_kernel_map(const int32_t* in_coords, int64_t n_in, const int32_t* out_coords, int64_t n_out,
                    int32_t K, int32_t s_p, int32_t* M) {
  const int K3 = K * K * K;
  std::vector<int32_t> off(3 * K3);
  orc_offsets(K, s_p, off.data());
  std::unordered_map<Coord, int32_t, CoordHash> table;
  table.reserve(static_cast<size_t>(n_in) * 2);
  for (int64_t j = 0; j < n_in; ++j) table.emplace(load(in_coords + 4 * j), static_cast<int32_t>(j));
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n_out; ++i) {
    const Coord q = load(out_coords + 4 * i);
    for (int k = 0; k < K3; ++k) {
      Coord p{q[0], q[1] + off[3 * k], q[2] + off[3 * k + 1], q[3] + off[3 * k + 2]};
      auto it = table.find(p);
      M[i * K3 + k] = (it == table.end()) ? -1 : it->second;
    }
  }
}

// Transposed layer (reading; the paper is silent): the output voxels are the
// finer level's voxels and the pairs are those of the matching strided layer
// with input and output swapped, offset index kept:
//   Mt[i*K^3 + k] = j  iff  fine[i] == coarse[j] + delta_k,  delta_k in Delta(K, s_fine).
void orc_kernel_map_transposed(const int32_t* coarse, int64_t n_coarse, const int32_t* fine, int64_t n_fine,
                               int32_t K, int32_t s_fine, int32_t* Mt) {
  const int K3 = K * K * K;
  std::vector<int32_t> off(3 * K3);
  orc_offsets(K, s_fine, off.data());
  std::unordered_map<Coord, int32_t, CoordHash> table;
  table.reserve(static_cast<size_t>(n_coarse) * 2);
  for (int64_t j = 0; j < n_coarse; ++j) table.emplace(load(coarse + 4 * j), static_cast<int32_t>(j));
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n_fine; ++i) {
    const Coord f = load(fine + 4 * i);
    for (int k = 0; k < K3; ++k) {
      Coord c{f[0], f[1] - off[3 * k], f[2] - off[3 * k + 1], f[3] - off[3 * k + 2]};
      auto it = table.find(c);
      Mt[i * K3 + k] = (it == table.end()) ? -1 : it->second;
    }
  }
}

// Canonical form of a map: all (k, j, i) with j = M[i,k] >= 0, sorted
// lexicographically.  `triples` must hold n_out*K3 rows of 3; returns nnz.
int64_t orc_triples(const int32_t* M, int64_t n_out, int32_t K3, int32_t* triples) {
  int64_t nnz = 0;
  for (int k = 0; k < K3; ++k)
    for (int64_t i = 0; i < n_out; ++i) {
      int32_t j = M[i * K3 + k];
      if (j >= 0) {
        triples[3 * nnz] = k;
        triples[3 * nnz + 1] = j;
        triples[3 * nnz + 2] = static_cast<int32_t>(i);
        ++nnz;
      }
    }
  std::vector<std::array<int32_t, 3>> t(nnz);
  std::memcpy(t.data(), triples, sizeof(int32_t) * 3 * nnz);
  std::sort(t.begin(), t.end());
  std::memcpy(triples, t.data(), sizeof(int32_t) * 3 * nnz);
  return nnz;
}

// Eq. (2): out[i, :] = sum over k ascending of F[M[i,k], :] * W[k] (W[k] is
// Cin x Cout, row-major), accumulated in fp64.
void orc_conv(const int32_t* M, int64_t n_out, int32_t K3, const double* F, const double* W,
              int32_t cin, int32_t cout, double* out) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t i = 0; i < n_out; ++i) {
    double* o = out + i * cout;
    for (int c = 0; c < cout; ++c) o[c] = 0.0;
    for (int k = 0; k < K3; ++k) {
      const int32_t j = M[i * K3 + k];
      if (j < 0) continue;
      const double* f = F + static_cast<int64_t>(j) * cin;
      const double* w = W + static_cast<int64_t>(k) * cin * cout;
      for (int ci = 0; ci < cin; ++ci) {
        const double fv = f[ci];
        const double* wr = w + static_cast<int64_t>(ci) * cout;
        for (int c = 0; c < cout; ++c) o[c] += fv * wr[c];
      }
    }
  }
}

// Packed key of a voxel (Section 5.3): fields from the top: batch, x, y, z.
// Reading for what the paper leaves open: each spatial value is stored as
// v - origin[a] + pad (a bias that keeps neighbour queries inside their field),
// the batch index sits above x.  A row is in range when 0 <= v - origin[a] and
// v - origin[a] + 2*pad < 2^bits on every axis (guard band on both sides) and the
// batch index fits its field.  Returns the number of rows out of range (their key
// is set to all ones).
int64_t orc_pack_keys(const int32_t* coords, int64_t n, int32_t bits_b, int32_t bits_x, int32_t bits_y,
                      int32_t bits_z, const int32_t* origin, int32_t pad, uint64_t* keys) {
  const int bits[4] = {bits_b, bits_x, bits_y, bits_z};
  int64_t bad = 0;
  for (int64_t i = 0; i < n; ++i) {
    uint64_t key = 0;
    bool ok = true;
    for (int a = 0; a < 4; ++a) {
      int64_t v = coords[4 * i + a];
      if (a > 0) {
        // the guard band must fit on both sides of the value: then v + delta stays inside
        // the field for every offset component |delta| <= pad (packed additivity, Section 5.3)
        const int64_t f = v - origin[a - 1];
        if (f < 0 || f + 2 * int64_t(pad) >= (int64_t(1) << bits[a])) ok = false;
        v = f + pad;
      } else if (v < 0 || v >= (int64_t(1) << bits[a])) {
        ok = false;
      }
      key = (key << bits[a]) | (static_cast<uint64_t>(v) & ((uint64_t(1) << bits[a]) - 1));
    }
    if (!ok) {
      key = ~uint64_t(0);
      ++bad;
    }
    keys[i] = key;
  }
  return bad;
}

}  // extern "C"
