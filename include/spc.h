/*
 * spc.h — C ABI of the MI355X (gfx950) sparse-convolution (SpC) layer library.
 *
 * The library implements the two halves of an SpC layer as defined in Section 2
 * of the Spira paper (arXiv 2511.20834):
 *   voxel indexing   — packing, sorting, downsampling (Eq. 1) and kernel-map
 *                      construction (Section 2.2, Sections 5.2, 5.3, 5.5);
 *   feature computation — Eq. (2), in an output-stationary or a weight-stationary
 *                      dataflow (Section 2.2, Section 5.4).
 *
 * Conventions
 *   - Every function returns SPC_OK (0) or a negative SPC_ERR_* code; a message for
 *     the calling thread's last error is available from spc_last_error().
 *   - Pointers marked [device] are device (HBM) addresses on the current HIP device,
 *     owned by the caller; [host] pointers are ordinary host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work on it and return without waiting unless stated otherwise.
 *   - Voxel indices are int32; a kernel map entry of -1 means "no input voxel".
 *   - The offset index of a K x K x K kernel is k = (ix*K + iy)*K + iz (z fastest,
 *     the group order of Section 5.2).  Per axis, index i stands for the offset
 *     (i - (K-1)/2) * in_stride for odd K and i * in_stride for even K.
 *   - No function may be called concurrently on the same spc_kmap from two threads.
 */
#ifndef SPC_H_
#define SPC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPC_OK 0
#define SPC_ERR_ARG (-1)         /* null pointer, bad size, bad enum, inconsistent descriptor */
#define SPC_ERR_RANGE (-2)       /* a coordinate does not fit its packed field incl. guard band */
#define SPC_ERR_DUP (-3)         /* duplicate voxel coordinates (only reported in validate mode) */
#define SPC_ERR_UNSUPPORTED (-4) /* valid request this build has no kernel for */
#define SPC_ERR_HIP (-5)         /* a HIP runtime call failed; message holds hipGetErrorString */
#define SPC_ERR_NOMEM (-6)       /* device allocation failed */

#define SPC_DTYPE_F16 0
#define SPC_DTYPE_BF16 1
#define SPC_DTYPE_F32 2

#define SPC_LAYOUT_OS 1   /* |V_q| x K^3 matrix of input indices (Section 5.4, case I) */
#define SPC_LAYOUT_WS 2   /* per-offset filtered (in,out) lists (Section 5.4, case II) */
#define SPC_LAYOUT_BOTH 3
/* Modifier of the WS layout for submanifold layers (layer_stride 1, odd K): lists are kept for the
 * offsets k < (K^3-1)/2 only.  Offset K^3-1-k is the same list with input and output swapped
 * (delta_n = -delta_l: M[i,l] = j  <=>  M[j,n] = i) and the centre offset pairs every voxel with
 * itself, so the feature kernel derives both from the stored half (Section 5.4).  Without the OS
 * layout the search itself visits only that half of the offsets. */
#define SPC_LAYOUT_WS_SYM 4
/* Modifier of SPC_LAYOUT_BOTH for the hybrid dual dataflow with threshold t (Section 5.4, 1 <= t <= 255): the
 * offsets whose L1 norm (in units of the input stride) is below t, the dense ones, are written into the OS
 * matrix only, the others into the WS lists only, so the map build moves |V_q| x K_dense matrix entries plus the
 * sparse offsets' pairs instead of both full layouts.  Such a map serves spc_conv_forward_hybrid with that same
 * t (other requests return SPC_ERR_ARG); accessors report each offset from the layout that holds it. */
#define SPC_LAYOUT_HYBRID_T(t) ((t) << 8)

#define SPC_DATAFLOW_OS 0 /* output-stationary: no atomics, bit-reproducible */
#define SPC_DATAFLOW_WS 1 /* weight-stationary: fp32 atomic accumulation */

#define SPC_PACK_VALIDATE 1 /* spc_pack_coords: check ranges and duplicates, wait, report */
#define SPC_CONV_RELU 1     /* spc_conv_forward: apply max(x,0) before the output is stored */
#define SPC_CONV_PACKED_WEIGHTS 2 /* spc_conv_forward: `weights` came from spc_conv_prepare_weights */
#define SPC_CONV_OS_PHASE 4  /* spc_conv_forward, OS, 16-bit types: force the LDS-staged phase kernel */
#define SPC_CONV_OS_SPLITK 8 /* spc_conv_forward, OS, 16-bit types: force the split-k kernel */
#define SPC_CONV_SPLITK_RB(rb) ((rb) << 8) /* with SPC_CONV_OS_SPLITK: 32-row blocks per workgroup (1, 2; 0 = by size) */
#define SPC_NET_SEQUENTIAL 1 /* spc_build_kmaps_network: one stream, level by level (for comparison) */
#define SPC_NET_PHASE_BARRIER 2 /* spc_build_kmaps_network: all levels join streams[0] before any map search starts */
#define SPC_NET_PIPELINED 4 /* spc_build_kmaps_network: maps on streams[1] (levels on streams[2]) in the order the layers need them; streams[0] is not held up */

/*
 * Packing descriptor (Section 5.3).  A key holds, from the most significant bit
 * down: bits_b bits of batch index, bits_x bits of x, bits_y of y, bits_z of z.
 * A spatial field stores v - origin[a] + pad.  The guard band `pad` keeps every
 * neighbour query q + delta inside its field, so that adding the packed offset to a
 * packed coordinate never borrows or carries between fields (the paper's
 * packed(q)+packed(delta)=packed(q+delta) holds only then).  For downsampling by
 * masking to agree with floor() on the raw coordinates, origin[a] - pad must be a
 * multiple of the largest output stride used.  key_bits is 32 or 64 and
 * bits_b+bits_x+bits_y+bits_z must not exceed it.  The builders check both rules
 * against every layer they are given and return SPC_ERR_ARG when pad is smaller
 * than the layer's largest offset component ((K-1)/2 * in_stride for odd K,
 * (K-1) * in_stride for even K) or when origin[a] - pad is not a multiple of
 * in_stride * layer_stride: maps built on such keys would hold false matches.
 */
typedef struct spc_pack_desc {
  int32_t key_bits;
  int32_t bits_b, bits_x, bits_y, bits_z;
  int32_t origin[3];
  int32_t pad;
} spc_pack_desc;

/*
 * Host helper: fills `out` for coordinates with lo[a] <= v <= hi[a] (inclusive, raw
 * units), batch indices in [0, n_batch), the largest output stride `max_stride`
 * (power of two) and the largest |offset component| `max_reach` of any layer.  Picks
 * the smallest fields; key_bits = 32 if they fit, else 64 (or forces `key_bits` when
 * it is 32 or 64).  Returns SPC_ERR_RANGE if even 64 bits do not suffice.
 */
int spc_pack_desc_fit(const int32_t lo[3], const int32_t hi[3], int32_t n_batch, int32_t max_stride,
                      int32_t max_reach, int32_t key_bits, spc_pack_desc* out);

/*
 * Pack and sort (Sections 5.2-5.3; done once per network on the initial coordinates).
 *   coords_bxyz [device] n rows of int32 (b, x, y, z), unique, any order.
 *   keys_out    [device] n keys (uint32 or uint64 per d->key_bits), ascending.
 *   perm_out    [device] n int32, may be NULL: keys_out[r] is the key of input row
 *               perm_out[r]; the caller gathers feature rows with it once.
 *   workspace   [device] scratch; call with workspace == NULL to get the size needed
 *               in *workspace_bytes (nothing is enqueued then).
 *   flags       SPC_PACK_VALIDATE: wait for the stream and return SPC_ERR_RANGE /
 *               SPC_ERR_DUP if a row does not fit its field or occurs twice.  Without
 *               it nothing is waited for: a row that does not fit gets the all-ones key
 *               (sorted last), repeated rows are sorted like any others and perm_out
 *               stays a complete permutation; kernel maps built on such keys are not
 *               meaningful.
 */
int spc_pack_coords(const int32_t* coords_bxyz, int64_t n, const spc_pack_desc* d, void* keys_out,
                    int32_t* perm_out, void* workspace, size_t* workspace_bytes, int32_t flags,
                    void* stream);

/*
 * spc_pack_coords for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, flags and
 * results as spc_pack_coords; the sort's scratch lives in a buffer that is part of the library image
 * (13 MiB per GPU, held until the process ends), so the call neither allocates nor frees anything.
 * Takes 1 <= n <= SPC_NOALLOC_MAX_N voxels (the sizes the library's own sort kernels cover within
 * that buffer); other sizes return SPC_ERR_UNSUPPORTED and enqueue nothing.  All calls on one GPU share
 * the buffer: calls whose work may overlap on that GPU (different streams without an ordering between
 * them, different host threads) race; order them, or use spc_pack_coords with workspaces of their own.
 */
#define SPC_NOALLOC_MAX_N 262144
int spc_pack_coords_noalloc(const int32_t* coords_bxyz, int64_t n, const spc_pack_desc* d, void* keys_out,
                            int32_t* perm_out, int32_t flags, void* stream);

/*
 * One layer's voxel-indexing request.
 *   K            kernel size per axis (1, 2, 3, 5 or 7).
 *   in_stride    s_p: stride of the layer's input coordinates (power of two).
 *   layer_stride s_l: 1 = submanifold (V_q = V_p); 2^m = strided, V_q from Eq. (1).
 *   transposed   0/1.  1: the layer upsamples.  Its OUTPUT voxels are the level with
 *                stride in_stride, its INPUT voxels that level downsampled by
 *                layer_stride, and pair (in j, out i, offset k) exists iff
 *                out_i = in_j + delta_k with delta_k from Delta(K, in_stride) — the
 *                pairs of the strided layer with roles swapped.  (The paper does not
 *                define transposed layers; this is the usual generalised-SpC reading.)
 *   layout       SPC_LAYOUT_OS, _WS or _BOTH: which representation(s) to build (| SPC_LAYOUT_WS_SYM,
 *                | SPC_LAYOUT_HYBRID_T(t)).  The WS lists are compacted tile by tile inside the search
 *                and never pass through a |V_q| x K^3 matrix; without SPC_LAYOUT_OS no matrix exists.
 */
typedef struct spc_layer_desc {
  int32_t K, in_stride, layer_stride, transposed, layout;
} spc_layer_desc;

typedef struct spc_kmap spc_kmap; /* opaque; owned by the library; release with spc_kmap_destroy */

/*
 * Build one kernel map with the one-shot search of Section 5.2 on packed keys
 * (Section 5.3).  in_keys [device]: n_in sorted unique keys of the level with stride
 * l->in_stride (all spatial components multiples of it).  For layer_stride > 1 the
 * coarser level is produced first (mask, sort, unique: Section 5.3).  Nothing is
 * waited for; the handle keeps device pointers into in_keys, which must stay alive
 * and unchanged while the map is in use.
 */
int spc_build_kmap(const void* in_keys, int64_t n_in, const spc_pack_desc* d, const spc_layer_desc* l,
                   spc_kmap** out, void* stream);

/*
 * Same, with the sort permutation folded into the map: in_perm [device] int32[n_in] is the
 * perm_out of spc_pack_coords (sorted position -> caller's row), and every input index the
 * map stores is in_perm[j] instead of j.  spc_conv_forward on such a map reads the caller's
 * feature matrix in its original row order, so the first layer of a network needs no
 * spc_permute_rows; its output rows are in sorted order like any other layer's.  in_perm
 * is read by the build only (a build captured into a graph reads it on every replay).
 * NULL in_perm = spc_build_kmap.  Not available for transposed layers and symmetric half-maps.
 */
int spc_build_kmap_perm(const void* in_keys, int64_t n_in, const int32_t* in_perm, const spc_pack_desc* d,
                        const spc_layer_desc* l, spc_kmap** out, void* stream);

/*
 * Network-wide voxel indexing (Section 5.5).  v0_keys [device]: the n0 sorted keys of
 * the stride-1 level.  Every coordinate level any layer needs is derived directly from
 * v0_keys (closed form of Section 5.5), all levels concurrently over `streams`; then
 * all distinct kernel maps are built concurrently.  Layers with equal (K, in_stride,
 * layer_stride, transposed) receive the same handle (reference counted; call
 * spc_kmap_destroy once per returned handle).  streams [host]: n_streams hipStream_t;
 * on return streams[0] has been made to wait for all the work, nothing else is waited
 * for.  out [host]: n_layers handles.
 * SPC_NET_PIPELINED (needs n_streams >= 2): all maps are built on streams[1], in the order in which
 * the layers first need them, the levels on streams[2] if there is one (else on streams[1], each
 * right before the first map that reads it), and streams[0] is not made to wait: every
 * spc_conv_forward waits for its own map on its own stream, so the first layers of a network run
 * while the maps of the later ones are still being built.  Under stream capture every returned
 * map must then be used by a spc_conv_forward on the capturing stream before the capture ends
 * (that is what joins streams[1] back).
 */
int spc_build_kmaps_network(const void* v0_keys, int64_t n0, const spc_pack_desc* d,
                            const spc_layer_desc* layers, int32_t n_layers, spc_kmap** out,
                            void* const* streams, int32_t n_streams, int32_t flags);

/* Sizes.  For strided / transposed maps the counts are produced on the device; these
 * calls wait for the build to finish the first time.  Return a negative SPC_ERR_* on failure. */
int64_t spc_kmap_n_in(spc_kmap* m);
int64_t spc_kmap_n_out(spc_kmap* m);
int32_t spc_kmap_kvol(const spc_kmap* m); /* K^3 */
/* [device] sorted keys of the layer's output (resp. input) voxels; valid while the map lives. */
const void* spc_kmap_out_keys(const spc_kmap* m);
const void* spc_kmap_in_keys(const spc_kmap* m);
/* Copies the n_out sorted output keys to keys_host [host] (uint32 or uint64 per key_bits; `cap`
 * keys of room).  Waits for the build. */
int spc_kmap_copy_out_keys(spc_kmap* m, void* keys_host, int64_t cap);
/* [device] OS layout, NULL if not built.  The |V_q| x K^3 matrix is stored in blocks of 32
 * consecutive output voxels, offset-major inside a block: entry (i, k) sits at
 * ((i/32)*K^3 + k)*32 + i%32, so the 32 entries an MFMA row block needs for one offset are one
 * 128-byte line.  Rows past n_out in the last block hold -1. */
const int32_t* spc_kmap_os_map(const spc_kmap* m);
/* [device] WS layout: list k occupies entries [k*ws_stride, k*ws_stride + nnz[k]) of both
 * arrays, ordered by ascending output index; *nnz_dev [device] int32[K^3].  NULL if not built. */
int spc_kmap_ws_lists(const spc_kmap* m, const int32_t** in_idx, const int32_t** out_idx,
                      const int32_t** nnz_dev, int64_t* ws_stride);
/* How the search of Section 5.2 was laid out for this map: *tile_rows = consecutive sorted output voxels
 * one workgroup owns, *window_keys = input keys of their neighbour windows it can stage in LDS (the
 * groups of offsets whose windows no longer fit are searched in global memory).  Host values, no wait.
 * Either pointer may be NULL. */
int spc_kmap_search_info(const spc_kmap* m, int32_t* tile_rows, int32_t* window_keys);
/* Number of kernel-map searches this process has enqueued so far (host counter, no wait).  A network build
 * searches once per distinct map, and not at all for a transposed map whose strided twin (same K, strides; K equal
 * to the layer stride, as the 2x2x2 stride-2 layers of a UNet) is part of the same build: that map is derived from
 * the twin's pairs (Section 5.5, maps shared between layers). */
int64_t spc_search_count(void);
/* nnz_host [host] int64[K^3]: valid entries per offset.  Waits for the build. */
int spc_kmap_nnz(spc_kmap* m, int64_t* nnz_host);
/*
 * Debug/test export: copies the map to the host as (k, in, out) int32 triples in the
 * order offsets ascending, then output index ascending (which is the lexicographic
 * order of the triples).  which = SPC_LAYOUT_OS or SPC_LAYOUT_WS selects the
 * representation read.  triples [host] holds `cap` rows; *nnz_out receives the total.
 * Waits for the build.
 */
int spc_kmap_export_triples(spc_kmap* m, int32_t which, int32_t* triples, int64_t cap, int64_t* nnz_out);
/*
 * A strided layer's output count exists only on the device until somebody waits for it.
 * spc_conv_forward picks its kernel from the output count; while the host does not know it
 * (nobody called spc_kmap_n_out, or the map was built under stream capture and is rewritten by
 * every replay) it assumes the upper bound n_in.  This sets a better estimate, e.g. the count a
 * previous cloud of the same scene produced.  The estimate steers kernel selection and launch
 * shape only: every kernel reads the true count on the device, so any value gives a correct
 * result.
 */
int spc_kmap_set_size_hint(spc_kmap* m, int64_t n_out_hint);
/*
 * Releases a handle (maps shared by several layers of a network are reference counted).  Does not
 * wait: the map's arrays go back to the block cache of the stream the map was built on, and that
 * stream is first made to wait (an event, no host wait) for every stream that has run
 * spc_conv_forward on the map, so a build that follows immediately cannot overwrite arrays a
 * feature kernel is still reading.  Those streams must still exist when the map is destroyed.
 * Kernels of the caller's own that read the accessor pointers (os_map, ws lists, keys) on other
 * streams are not known to the library: order them before the destroy yourself.
 */
void spc_kmap_destroy(spc_kmap* m);

/*
 * Feature computation, Eq. (2):  out[i,:] = sum_k feats_in[M[i,k],:] * W_k.
 *   feats_in  [device] n_in rows of cin elements, row pitch ld_in elements.
 *   weights   [device] [K^3][cin][cout] row-major, same dtype as the features.
 *   feats_out [device] n_out rows of cout elements, row pitch ld_out (lets a caller
 *             write straight into one half of a concatenated buffer).  Overwritten.
 *   dtype     SPC_DTYPE_F16 / BF16: MFMA contraction, fp32 accumulation, output rounded
 *             to nearest even.  SPC_DTYPE_F32: fp32 FMA arithmetic throughout.
 *   dataflow  SPC_DATAFLOW_OS needs the OS layout, SPC_DATAFLOW_WS the WS layout
 *             (Section 2.2).  OS results are bit-reproducible; WS uses fp32 atomics.
 *   flags     SPC_CONV_RELU; SPC_CONV_PACKED_WEIGHTS (see spc_conv_prepare_weights);
 *             SPC_CONV_OS_PHASE or SPC_CONV_OS_SPLITK pick one of the two OS MFMA kernels
 *             (default: chosen from the layer's size; both give the same result up to the
 *             fp32 summation order, and each one alone is bit-reproducible).
 * 16-bit layers with cout % 32 == 0 (OS) or cout in {32,64,128,256} (WS) run on MFMA; input
 * channel counts that are not a multiple of 16, and rows that are not 16-byte aligned, are
 * first copied into a zero-padded scratch buffer.  Everything else runs plain FMA kernels.
 * Nothing is waited for, and nothing is allocated with hipMalloc once the library's block
 * cache holds the scratch sizes of this call (i.e. after one call of the same shape on the same
 * stream), so a warmed-up call sequence can be captured into a HIP graph: spc_pack_coords
 * (without SPC_PACK_VALIDATE), spc_build_kmap(s_network), spc_conv_forward and
 * spc_permute_rows only enqueue kernels, event records and event waits — as long as every sort
 * is the library's own, i.e. the cloud (for strided layers: the level that is downsampled) has
 * at most 8 388 608 voxels.  Above that the sort is rocPRIM's, which also
 * enqueues memsets; under stream capture spc_pack_coords and the builders then return
 * SPC_ERR_UNSUPPORTED instead of recording them (replayed memset nodes are not reliable on the
 * target systems, and a radix sort that starts from stale counters writes out of bounds).  Maps built under
 * capture must stay alive as long as the graph; their accessors that wait (n_out, nnz,
 * export) drain the device and read the values of the latest replay.
 */
int spc_conv_forward(spc_kmap* m, const void* feats_in, int64_t ld_in, const void* weights, void* feats_out,
                     int64_t ld_out, int32_t cin, int32_t cout, int32_t dtype, int32_t dataflow,
                     int32_t flags, void* stream);

/*
 * Hybrid dual dataflow (Section 5.4): weight offsets whose L1 norm, in units of the layer's input
 * stride, is below the threshold t (the dense ones: the centre and its nearest neighbours) are
 * computed output-stationary, the others weight-stationary, and the two partial sums are merged
 * without an extra pass: the weight-stationary part accumulates in an fp32 buffer from which the
 * output-stationary kernel starts.  t = 0 is the pure weight-stationary dataflow, any t above the
 * largest norm (3 * (K-1)/2 for odd K) the pure output-stationary one.  The map must hold both
 * layouts unless one part is empty.  Everything else as spc_conv_forward.
 */
int spc_conv_forward_hybrid(spc_kmap* m, const void* feats_in, int64_t ld_in, const void* weights, void* feats_out,
                            int64_t ld_out, int32_t cin, int32_t cout, int32_t dtype, int32_t t, int32_t flags,
                            void* stream);

/*
 * One-time tuning of the hybrid threshold of one layer (Section 5.4: the threshold is chosen per layer by timing
 * it once on sample data).  Runs the layer's feature computation for every threshold t = 0 (all offsets
 * weight-stationary) .. L1max + 1 (all output-stationary), one untimed call and `reps` (1..1000) timed ones each,
 * between two events on `stream`, and waits for them: not capturable.
 *   m              map holding both full layouts (SPC_LAYOUT_BOTH without a hybrid threshold of its own).
 *   weights        [device] plain [K^3][cin][cout]; packed_weights [device] the same weights from
 *                  spc_conv_prepare_weights, or NULL: used for the thresholds and shapes that take them.
 *   flags          SPC_CONV_RELU and the OS kernel choice only.
 *   ws_build_us    what the weight-stationary lists add to the build of this map (measured by the caller, may be
 *                  0): added to every threshold that has a weight-stationary part.
 *   us_per_t       [host] `cap` floats; receives microseconds per call for t = 0 .. *n_t - 1.  *n_t is set even
 *                  when cap is too small (SPC_ERR_ARG), so a caller can size the array from a first call.
 *   best_t         [host] the fastest threshold.  On return feats_out holds the layer's output computed with it.
 * Feature and output arguments as spc_conv_forward.
 */
int spc_conv_tune_threshold(spc_kmap* m, const void* feats_in, int64_t ld_in, const void* weights,
                            const void* packed_weights, void* feats_out, int64_t ld_out, int32_t cin, int32_t cout,
                            int32_t dtype, int32_t flags, int32_t reps, float ws_build_us, float* us_per_t, int32_t cap,
                            int32_t* n_t, int32_t* best_t, void* stream);

/*
 * Weights are constant during inference, so their re-layout into MFMA operand order can
 * be hoisted out of the layer call.  Writes K^3 * cin16 * cout elements to packed_out [device]
 * (same dtype), cin16 = cin rounded up to a multiple of 16 (the padding channels are zeros; a
 * layer with such a cin still copies its feature rows into a padded scratch buffer at every call),
 * for use with SPC_CONV_PACKED_WEIGHTS.  Returns SPC_ERR_UNSUPPORTED for the shapes/dtypes
 * that do not take prepacked weights (fp32, cout % 32 != 0); those layers take the plain
 * [K^3][cin][cout] weights only.  The WS dataflow accepts prepacked weights for cout in
 * {32,64,128,256}.
 */
int spc_conv_prepare_weights(const void* weights, int32_t kvol, int32_t cin, int32_t cout, int32_t dtype,
                             void* packed_out, void* stream);

/*
 * Row gather used once per cloud after spc_pack_coords (Section 5.2: one initial sort):
 * dst[r, :] = src[perm[r], :] for r < n; rows of `row_bytes` bytes (a multiple of 4), row
 * pitches in bytes.  All pointers [device].
 */
int spc_permute_rows(const void* src, int64_t src_pitch, const int32_t* perm, int64_t n, int64_t row_bytes,
                     void* dst, int64_t dst_pitch, void* stream);

/*
 * Measurement aids (Section 6 reports rates; these give the machine's own denominators next to the data-sheet
 * ones).  spc_probe_copy: a plain copy kernel, dst[0..bytes) = src[0..bytes) ([device], bytes a multiple of 16):
 * its rate is what a streaming kernel can reach on this GPU, and its known size calibrates the profiler's byte
 * counters.  spc_probe_mfma: every wave of the chip issues `iters` x 4 independent 32x32x16 fp16 MFMAs from
 * registers; *flops [host] receives the floating-point operations of the launch, sink [device] one float.
 * Both only enqueue; time them with events on `stream`.
 */
int spc_probe_copy(const void* src, void* dst, int64_t bytes, void* stream);
int spc_probe_mfma(int32_t iters, float* sink, double* flops, void* stream);

/* Releases the library's cached device blocks (maps still alive keep theirs). Waits for the device. */
int spc_release_cache(void);

const char* spc_last_error(void);
const char* spc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPC_H_ */
