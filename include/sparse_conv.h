/*
 * sparse_conv.h -- C ABI of the MI355X (gfx950) direct sparse convolution library.
 *
 * The operation is the one defined in the paper's section "Convolution operation using a sparse
 * operation on GPGPU": a dense NCHW activation tensor is convolved (cross-correlation, zero
 * padding, no bias) with an unstructured-pruned weight tensor stored per output channel in CSR
 * form (rowptr RP, column index Lambda, values theta).  Every row is padded to the same stored
 * count N_nz (the paper's "standardised sparse level"), which makes the layout a fixed-width
 * ELL-like table, and the column indices are "pre-stretched" once into flat offsets into the
 * padded input so the kernel (the paper's Algorithm 3) only gathers, multiplies and accumulates:
 *
 *     Y[b,d,p,q] = sum_{j < N_nz} theta[d,j] * Xp[b, p*s_h*Wp + q*s_w + lambda[d,j]]
 *
 * with Xp the zero-padded input of one sample (C planes of Hp x Wp), Hp = H + 2*pad_h,
 * Wp = W + 2*pad_w, P = (Hp - R)/s_h + 1, Q = (Wp - S)/s_w + 1.
 *
 * Conventions
 *   - All functions return sc_status_t; SC_OK is 0.  No exception crosses this boundary.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory of the
 *     current device.  `stream` is a hipStream_t passed as an opaque pointer (NULL = the null stream).
 *   - Host arrays given to the create calls are borrowed for the duration of the call and copied.
 *   - The plan owns its device tables (weights, offsets, scales, codebook) until
 *     sparse_conv_plan_destroy.  x, y and workspace are borrowed and never retained or freed.
 *   - sparse_conv_forward is asynchronous on `stream`, never synchronises and never allocates.
 *     A plan is immutable between create / set_tuning / autotune calls, so forward may be issued
 *     concurrently on several streams as long as each uses its own workspace.
 *   - Inputs must be finite: the zero-valued filler entries of padded rows are multiplied like any
 *     other entry.
 *   - Argument validation happens on the host before the first HIP call, so every error below
 *     except SC_ERR_HIP / SC_ERR_OOM can be produced (and tested) without a GPU.
 */
#ifndef SPARSE_CONV_H
#define SPARSE_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sparse_conv_plan sparse_conv_plan_t; /* opaque, library-owned */

typedef enum {
    SC_OK = 0,
    SC_ERR_NULL = 1,        /* a required pointer is NULL */
    SC_ERR_SHAPE = 2,       /* non-positive dimension, empty output, N <= 0 */
    SC_ERR_CSR = 3,         /* rowptr not starting at 0 / not monotone, column outside [0, C*R*S),
                               codebook index > 15 */
    SC_ERR_UNSUPPORTED = 4, /* unknown dtype, missing scales/codebook for a quantised dtype,
                               tuning that does not fit this layer */
    SC_ERR_RANGE = 5,       /* one padded sample or one output sample has >= 2^31 elements */
    SC_ERR_OOM = 6,         /* device or host allocation failed */
    SC_ERR_WORKSPACE = 7,   /* workspace NULL or smaller than sparse_conv_workspace_size */
    SC_ERR_HIP = 8          /* a HIP runtime call or kernel launch failed */
} sc_status_t;

/* Storage / arithmetic variants (weights x activations -> accumulator -> output):
 *   SC_F32     f32 x f32 -> f32 -> f32
 *   SC_F16     f16 x f16 -> f32 -> f16 (one rounding at the store)
 *   SC_I8      i8  x i8  -> i32 -> i32 (exact; the per-channel scales are carried, not applied)
 *   SC_CB4_I8  4-bit index into a 16-entry i8 codebook x i8 -> i32 -> i32 (the paper's non-linear,
 *              cluster-based quantisation: each stored weight is a centroid index)
 *   SC_CB4_F16 4-bit index into a 16-entry f16 codebook x f16 -> f32 -> f16 (the paper's 4b/16b
 *              configuration: 16 centroids in sixteen-bit format, half-precision activations) */
typedef enum { SC_F32 = 0, SC_F16 = 1, SC_I8 = 2, SC_CB4_I8 = 3, SC_CB4_F16 = 4 } sc_dtype_t;

/* Layer geometry.  Weights are D rows (output channels) by K = C*R*S columns, a column being the
 * filter tap (c, r, s) flattened as (c*R + r)*S + s (PyTorch's weight.view(D, -1)). */
typedef struct {
    int32_t C, D, H, W, R, S, stride_h, stride_w, pad_h, pad_w;
} sc_layer_t;

/* Kernel families (sc_tuning_t.variant). */
enum {
    SC_VARIANT_AUTO = 0,   /* let the library pick by heuristic */
    SC_VARIANT_GATHER = 1, /* Algorithm-3 shape: one workgroup = one output channel x a tile of output
                              positions (flat over sample, row, column); (theta, lambda) row in LDS;
                              input gathered from global memory (a padded copy in the workspace
                              when pad > 0) */
    SC_VARIANT_SLAB = 2,   /* one workgroup = one sample x an output tile x all output channels;
                              the input tile (all C channels, halo and zero padding included) is
                              staged once in LDS and every row of (theta, lambda) is streamed over it */
    SC_VARIANT_DENSE = 3   /* the densified tile on the matrix cores, for layers that are not sparse
                              enough for the gather kernels to win (the per-layer choice of the
                              paper's "Main scheme", whose dense side is here a kernel of the
                              library): the stored entries are scattered once into a dense weight
                              array in MFMA operand order, the input tile is staged in LDS
                              channel-minor, and 16 x 16 blocks of (output channel, position) are
                              accumulated by v_mfma_f32_16x16x32_f16 / v_mfma_i32_16x16x64_i8.
                              SC_F16, SC_CB4_F16, SC_I8, SC_CB4_I8 only; not for tables that store a
                              column twice in one row.  Integer results are exact.  Fields: tile_p =
                              output rows per workgroup, sub_batch = samples per workgroup (whole
                              planes only, up to 16), chunk_c = input channels per LDS chunk (a
                              multiple of 32 for 16-bit, 64 for 8-bit activations), tile_d = output
                              channels per workgroup (16, 32, 64 or 128), waves_m, wg_per_cu; 0 = heuristic */
};

/* Launch shape of sparse_conv_forward; the analogue of the paper's per-layer choice of the
 * sub-batch size sb_S that fixes the number of thread blocks N_B = b_S * D / sb_S.
 * Fields that do not apply to a variant are ignored.  All-zero = SC_VARIANT_AUTO. */
typedef struct {
    int32_t variant;    /* SC_VARIANT_* */
    int32_t wg_threads; /* workgroup size: 64..1024, multiple of 64.  DENSE: 256 (0 = that) or 512 -- with 512 two
                           groups of four waves own the same outputs and take the even and the odd steps
                           of the contraction (filter tap x channel block), meeting through LDS at the end */
    int32_t sub_batch;  /* GATHER: output positions per thread that share each (theta, lambda) read
                           from LDS (the role of sb_S), 1, 2, 4 or 8.  SLAB with pipeline = 0 and
                           chunk_c > 0: samples per workgroup (0 / 1 = one; 2..4 for tiles of at most
                           64 positions, each scalar-loaded weight then feeds that many samples;
                           with pack >= 1, on pointwise layers and whole-plane tiles: 2..16 samples
                           whose planes lie end to end along the position axis of one packed tile,
                           within pack's limit of 8 positions per lane; with pack = 3: 2..8 groups of
                           interleaved samples per workgroup, the lanes numbered over (group, position) --
                           for planes so small that one group leaves most of a wave idle; the tile
                           positions of all groups must fit the 64 lanes) */
    int32_t tile_p;     /* SLAB: output rows per tile (pointwise layers: ignored) */
    int32_t tile_q;     /* SLAB: output columns per tile (pointwise layers: pixels per tile) */
    int32_t wg_per_cu;  /* SLAB: workgroups the LDS budget is sized for (1..8) */
    int32_t wsrc;       /* SLAB: how a wave gets (theta, lambda): 0 = staged in LDS, broadcast reads;
                           1 = scalar loads from global memory; 2 = wave-uniform vector loads from
                           global memory (vector L1), software-pipelined; 3 = one entry per lane by
                           coalesced vector loads, broadcast with v_readlane */
    int32_t split_n;    /* GATHER: lanes that share one output, each summing every split_n-th stored
                           entry, combined by a wavefront-level shuffle reduction: 1, 4, 16 or 64.
                           SLAB (given explicitly) with pipeline = 0 and chunk_c > 0, SC_F32 / SC_I8: 2..16 =
                           the channel chunks of a tile are dealt to that many workgroups, which add their
                           partial sums into y with atomic adds (y is cleared by a small kernel first) -- for
                           layers with fewer tiles than CUs; at most as many as there are chunks.  fp32
                           results of such a shape depend on the order in which the workgroups arrive
                           (last bits, within the tolerance of the type); int8 results do not.
                           DENSE, one-shot form with four waves and the whole contraction in one chunk: 2..16 =
                           a workgroup walks over that many blocks of tile_d output channels, one after the
                           other, with its tile staged once and resident in LDS (for layers with few input
                           and many output channels); same results as with 0 */
    int32_t pipeline;   /* SLAB, pointwise layers: 1 = persistent workgroups that stream tile i+1 into a
                           second LDS buffer (direct-to-LDS loads issued by dedicated waves) while
                           tile i is multiplied; needs wsrc != 0.  2 = the same double buffering with
                           no dedicated waves: every wave issues its share of the copy of tile i+1 and
                           then multiplies its rows of tile i (contiguous row ranges, one barrier per
                           tile); needs wsrc = 1 and at least one stored weight per row; with chunk_c > 0 at
                           most 4 positions per lane and 8 rows per wave.  0 = one tile per workgroup.
                           DENSE: 1 = the chunks of input channels are staged by `producers` waves of their
                           own into two LDS buffers, one chunk ahead of the multiplying waves (which run
                           over the steps of all chunks without draining their weights in flight);
                           chunk_c then defaults to two channel blocks.  Same results as with 0 for four
                           multiplying waves; with eight, the two groups split the steps of the whole
                           contraction instead of each chunk's (another fixed summation order) */
    int32_t producers;  /* SLAB with pipeline = 1: waves of the workgroup that only copy tiles (1, 2 or 4);
                           DENSE with pipeline = 1: staging waves behind the multiplying ones (1 .. 4, 0 = 2) */
    int32_t chunk_c;    /* SLAB: input channels per LDS buffer (0 = all of them); with pipeline = 0 for any
                           layer shape (wsrc = 1 or 3, at most 4 positions per lane and 8 rows per wave), with
                           pipeline = 1 or 2 for pointwise layers (wsrc = 1).  With
                           chunk_c < C a tile is multiplied chunk by chunk, each wave keeping the
                           accumulators of its output channels in registers across the chunks, so
                           wide tiles fit LDS even for layers with many input channels */
    int32_t tile_d;     /* SLAB with chunk_c > 0: output channels per workgroup (0 = all of them) */
    int32_t ragged;     /* SLAB with chunk_c > 0: 1 = walk every row over its own stored entries only (the
                           filler entries that unify the row lengths are left out of the per-chunk
                           segments), 0 = the unified table of the method.  For measuring what the
                           padding costs on tables whose rows differ in length */
    int32_t pack;       /* SLAB with chunk_c > 0 (pack = 2 also with chunk_c = 0 on pointwise layers, pipeline
                           0 or 1) and wsrc = 1, one sample per workgroup (pipeline = 0 on a pointwise
                           layer: or sub_batch samples end to end in one tile): packed positions.
                           1 (SC_F16 / SC_I8) = every lane owns the 2 / 4 adjacent positions of one 32-bit
                           word of the staged tile; 2 (SC_F32 / SC_F16) = the 4 / 8 adjacent positions of one
                           128-bit word.  One LDS read then feeds that many multiply-adds (at most 8
                           positions per lane), and 128-bit LDS reads move more bytes per clock than 32-bit
                           ones.  With pipeline = 0 on a layer whose offsets are not whole words (not
                           pointwise) LDS holds as many shifted images of each chunk as a word has
                           positions.  0 = one position per LDS read.  With pipeline = 1 or 2 a lane's results
                           leave as one store and y must be aligned to it (4 bytes for pack = 1 with f16,
                           16 bytes otherwise); pack = 2 there needs 16-byte aligned rows.
                           3 (SC_F32 / SC_F16 / SC_I8, pipeline = 0, chunk_c > 0) = samples
                           interleaved: a workgroup takes 4 (f32, i8) or 8 (f16) consecutive samples and an
                           LDS word (128 bits; 32 bits for i8) holds the same element of each, so every
                           offset is a whole word on any layer shape -- one LDS read per stored weight
                           feeds that many samples; at most 8 / word-size positions per lane */
    int32_t waves_m;    /* DENSE: how many of the workgroup's four waves lie along the output channels
                           (1, 2 or 4; the others along the positions).  A wave then owns tile_d / waves_m
                           output channels (16, 32 or 64) and up to 128 positions.  0 = heuristic */
    int32_t buffers;    /* SLAB with pipeline = 1 and chunk_c > 0: LDS chunk buffers.  0 (or 2) = two, the
                           producer waves share the copy of every chunk; 3 .. 5 = producers + 1 buffers
                           (producers is set to match when 0): every producer wave copies whole chunks by
                           itself, so that as many chunks as there are producers are in flight while one
                           is multiplied -- the memory latency of a chunk is spread over several phases */
    int32_t stage_rows; /* SLAB with pack = 3, SC_F32: 1 = the interleaved samples are staged by rows -- a thread
                           loads the same 16 (or 8) bytes of an input row of each of the 4 samples and
                           writes 4 (2) LDS words -- instead of one table look-up and 4 element loads per
                           word.  For unit strides (or strides of two) with tiles as wide as the plane
                           and rows that are whole 16- or 8-byte loads; a caller whose x is not 16-byte
                           aligned is served by the table form.  0 = by table.
                           DENSE, pointwise layers (1 x 1, unit stride, no padding): 1 = the tile
                           is copied to LDS in its natural layout ([channel][position], plain wide loads, no
                           transposition in registers) and the matrix operands are read with gfx950's
                           transposing LDS reads; same results as with 0.  With pipeline = 1 the staging waves
                           copy the chunks with direct-to-LDS loads: one sample per workgroup, runs and planes
                           of whole 16-byte words, x 16-byte aligned (SC_ERR_UNSUPPORTED at launch otherwise) */
} sc_tuning_t;

typedef struct {
    int32_t n;                     /* unified stored entries per output channel (N_nz) */
    int32_t P, Q;                  /* output height and width */
    int64_t X_size;                /* elements of one padded input sample, C*Hp*Wp */
    int64_t true_nnz;              /* stored entries before row padding (sum of CSR row lengths) */
    int64_t macs_per_sample;       /* D*P*Q*n: multiply-accumulates executed per sample */
    int64_t useful_macs_per_sample;/* P*Q*true_nnz: those that involve a caller-supplied entry */
    int64_t act_bytes_per_sample;  /* C*H*W*e_x + D*P*Q*e_y */
    int64_t weight_bytes;          /* D*n*(e_w + 4) (+ scales, codebook): read once per launch */
    int32_t lds_bytes;             /* LDS per workgroup of the current tuning */
    int32_t grid_size;             /* workgroups per launch for the N last used by set_tuning /
                                      autotune (0 if unknown) */
    sc_tuning_t tuning;            /* current tuning, heuristic defaults resolved */
    int32_t out_P, out_Q;          /* extents of y (P, Q unless the epilogue pools) */
    int32_t out_elem_bytes;        /* bytes per element of y (1 when the epilogue requantises) */
} sc_plan_info_t;

/* Build a plan from CSR weights (host arrays).
 *   rowptr  [D+1]  rowptr[0] = 0, non-decreasing; nnz = rowptr[D]
 *   colidx  [nnz]  each in [0, C*R*S); any order within a row; duplicates add up
 *   values  [nnz]  f32 (SC_F32), IEEE half bits (SC_F16), i8 (SC_I8), u8 index < 16 (SC_CB4_I8, SC_CB4_F16)
 *   scales  [D]    per-output-channel dequantisation scale, required for SC_I8 / SC_CB4_I8, else NULL
 *   codebook[16]   centroids, i8 (SC_CB4_I8) or IEEE half bits (SC_CB4_F16); required for those, else NULL
 * Rows are padded to n = max row length with zero-valued entries that repeat the row's last column
 * (column 0 for an empty row); then a device pass stretches every column to its input offset.
 * Errors: SC_ERR_NULL, SC_ERR_SHAPE, SC_ERR_CSR, SC_ERR_UNSUPPORTED, SC_ERR_RANGE, SC_ERR_OOM, SC_ERR_HIP.
 * On error *out is NULL. */
sc_status_t sparse_conv_plan_create_csr(const sc_layer_t* layer, sc_dtype_t dtype,
                                        const int32_t* rowptr, const int32_t* colidx,
                                        const void* values, const float* scales,
                                        const void* codebook, void* stream,
                                        sparse_conv_plan_t** out);

/* Same, from an already unified table: colidx / values are [D][n] row-major (n >= 0). */
sc_status_t sparse_conv_plan_create_ell(const sc_layer_t* layer, sc_dtype_t dtype, int32_t n,
                                        const int32_t* colidx, const void* values,
                                        const float* scales, const void* codebook, void* stream,
                                        sparse_conv_plan_t** out);

void sparse_conv_plan_destroy(sparse_conv_plan_t* plan); /* NULL is allowed */

/* Geometry, traffic model and current tuning of a plan: the unified stored count N_nz of the section
 * "Convolution operation using a sparse operation on GPGPU", the output extents that follow from
 * the padded input of eq. load_in_to_registers (t_in_p), and the multiply-accumulate count that the
 * GPU results section states is the dense count reduced by the sparsity ratio. */
sc_status_t sparse_conv_plan_info(const sparse_conv_plan_t* plan, sc_plan_info_t* info);

/* Test hook for the stretch pass (same section: the column-index array Lambda "is modified to store
 * these pre-computed indexes"; the formula itself is the one that makes Algorithm 3's address
 * t_in_p + lambda hit input element (c, p*s_h + r, q*s_w + s)): copies the device-built canonical offsets
 * lambda[d][j] = c*Hp*Wp + r*Wp + s (elements, relative to one padded sample) to host_out [D*n].
 * Synchronises the device. */
sc_status_t sparse_conv_plan_debug_offsets(const sparse_conv_plan_t* plan, int32_t* host_out);

/* Replace the launch shape -- the per-layer choice the paper makes through sb_S (eq. N_B and the
 * table "Impact of the number of thread blocks").  Fields left 0 are filled by heuristic.  SC_ERR_UNSUPPORTED if the
 * shape does not fit the layer (e.g. the slab does not fit in LDS); the previous tuning stays.
 * Rebuilds the variant-specific offset table on `stream` and waits for it. */
sc_status_t sparse_conv_plan_set_tuning(sparse_conv_plan_t* plan, const sc_tuning_t* tuning,
                                        void* stream);
sc_status_t sparse_conv_plan_get_tuning(const sparse_conv_plan_t* plan, sc_tuning_t* tuning);

/* Bytes of device workspace sparse_conv_forward needs for batch N with the current tuning
 * (0 unless the GATHER variant has to materialise a padded input, as the paper's own kernel is fed:
 * the GPU results section lists its inputs with the padding already in place, 226 x 226 for
 * 224 x 224). */
sc_status_t sparse_conv_workspace_size(const sparse_conv_plan_t* plan, int32_t N, size_t* bytes);

/* Upper bound of sparse_conv_workspace_size over every tuning autotune may try. */
sc_status_t sparse_conv_workspace_size_max(const sparse_conv_plan_t* plan, int32_t N, size_t* bytes);

/* The forward pass of Algorithm 3 ("Convolution operation using a sparse operation on GPGPU"):
 * every output value is the sum over the N_nz stored entries of its output channel of
 * theta * input[t_in_p + lambda] (eq. load_in_to_registers), one accumulator per output, one store.
 * Y = conv(X): x_dev [N,C,H,W] unpadded, y_dev [N,D,P,Q], both contiguous device memory in the
 * plan's storage types, aligned to their element size.  Asynchronous on `stream`; allocates nothing.
 * The pipelined launch shapes (tuning.pipeline = 1 or 2) copy rows with 16-byte (4-byte where the
 * rows allow no more) direct-to-LDS loads and need x_dev aligned to that; with tuning.pack they
 * also store 4 / 16 bytes at a time and need y_dev aligned to that: such a shape with other pointers
 * returns SC_ERR_UNSUPPORTED and launches nothing.  Every other shape takes any pointers.
 * Errors: SC_ERR_NULL, SC_ERR_SHAPE (N <= 0), SC_ERR_WORKSPACE, SC_ERR_UNSUPPORTED, SC_ERR_HIP. */
sc_status_t sparse_conv_forward(const sparse_conv_plan_t* plan, const void* x_dev, void* y_dev,
                                int32_t N, void* workspace_dev, size_t workspace_bytes,
                                void* stream);

/* For callers that cannot allocate or pass a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same result as sparse_conv_forward, but the scratch
 * memory of the launch shape (the padded copy of the input that SC_VARIANT_GATHER makes when the
 * layer has padding) is a static device array of SC_STATIC_WORKSPACE_BYTES inside the library, one
 * per GPU, held until the process ends.  Calls no hipMalloc / hipFree and no allocating library
 * routine; asynchronous on `stream`.  x_dev / y_dev as for sparse_conv_forward.
 * Every call on one GPU shares that GPU's array (each call rewrites all of the part it uses, so a
 * smaller call after a larger one is fine): calls that overlap in time on one GPU -- different
 * streams or threads -- race, serialise them.
 * Errors: SC_ERR_NULL, SC_ERR_SHAPE (N <= 0), SC_ERR_WORKSPACE (this N needs more than
 * SC_STATIC_WORKSPACE_BYTES: use sparse_conv_forward with a workspace), SC_ERR_UNSUPPORTED,
 * SC_ERR_HIP. */
#define SC_STATIC_WORKSPACE_BYTES (32u << 20)
sc_status_t sparse_conv_forward_static(const sparse_conv_plan_t* plan, const void* x_dev, void* y_dev,
                                       int32_t N, void* stream);

/* Per-layer launch-shape search: the gfx950 counterpart of the paper's empirical per-layer tuning
 * of the sub-batch size sb_S and with it of the number of thread blocks (eq. N_B = b_S * D / sb_S and
 * the table "Impact of the number of thread blocks" in the GPU results).  Times every candidate
 * tuning that fits the layer on the caller's buffers (y_dev is overwritten) with HIP events on
 * `stream`, times the fastest few (of every kernel family) again over a ring of scratch copies of x
 * and scratch outputs larger than twice the 256 MB last-level cache (so that the choice holds for a
 * caller that streams activations from HBM), keeps the fastest of those, and leaves it installed.
 * Synchronises.
 *   workspace_dev   must hold sparse_conv_workspace_size_max(plan, N) bytes.  When it holds
 *                   sparse_conv_autotune_workspace_size(plan, N) bytes the ring lies in it and the
 *                   call allocates no device memory besides the tables of the tunings it installs;
 *                   otherwise the ring (0.5-1 GB, aligned like x_dev / y_dev) is allocated for the
 *                   duration of the call and freed, and if that fails the second round runs on
 *                   the caller's buffers.
 * Candidates that these pointers rule out (see sparse_conv_forward) are skipped, so the installed
 * shape is valid for buffers aligned like x_dev and y_dev.
 * On any error the tuning the plan had on entry is installed again before the call returns.
 * On layers with fewer tiles than compute units the winner can be a shape that sums the partial
 * results of several workgroups with atomic adds (SLAB with split_n > 1, see sc_tuning_t): an SC_F32
 * result then depends on the arrival order of the workgroups in its last bits.  A caller that needs
 * run-to-run identical bits reads the tuning back (sparse_conv_plan_get_tuning) and, if split_n > 1
 * on a SLAB tuning, installs another one (any candidate of sparse_conv_plan_candidate without it).
 * Errors: SC_ERR_NULL, SC_ERR_SHAPE, SC_ERR_WORKSPACE, SC_ERR_UNSUPPORTED (no candidate runs),
 * SC_ERR_OOM, SC_ERR_HIP. */
sc_status_t sparse_conv_plan_autotune(sparse_conv_plan_t* plan, const void* x_dev, void* y_dev,
                                      int32_t N, void* workspace_dev, size_t workspace_bytes,
                                      void* stream);

/* Bytes of workspace with which sparse_conv_plan_autotune takes its ring of scratch buffers from the
 * caller instead of allocating it (an upper bound over the alignments x_dev / y_dev may have). */
sc_status_t sparse_conv_autotune_workspace_size(const sparse_conv_plan_t* plan, int32_t N, size_t* bytes);

/* Fused epilogue of a layer of a network that the paper's main scheme configures layer by layer (its
 * VGG-16 experiments: convolution, ReLU, 2 x 2 max-pooling between stages; its "Quantisation" section:
 * activations re-quantised from layer to layer with q = round(x / sigma)).  Applied to the accumulator
 * before the one store, in this order:
 *   relu     1: max(0, .)
 *   pool     2: 2 x 2 max-pooling with stride 2 (an odd last output row / column is dropped); 0: none
 *   requant  1 (SC_I8 / SC_CB4_I8 only): the output is int8,
 *               clamp(round_half_even(float32(acc) * requant_scale[d]), -127, 127),
 *            every step in single precision (requant_scale[d] = s_w[d] * s_x / sigma_next, host [D])
 * y_dev is then [N, D, P', Q'] with P' = P / 2, Q' = Q / 2 when pooling, in int8 when requantising
 * (sc_plan_info_t.out_P / out_Q / out_elem_bytes).  Available in SC_VARIANT_GATHER (with split_n = 1;
 * sub_batch is ignored) and SC_VARIANT_DENSE (with pooling: an even tile_p or whole planes); a plan
 * with an epilogue refuses SC_VARIANT_SLAB tunings and the dense-library path, and the autotuner /
 * dispatch only try what is left.  All-zero *ep removes the epilogue.
 * Errors: SC_ERR_NULL, SC_ERR_UNSUPPORTED (bad field, requant on a floating-point plan or without
 * scales, pooling a layer with P < 2 or Q < 2), SC_ERR_OOM, SC_ERR_HIP. */
typedef struct {
    int32_t relu, pool, requant;
} sc_epilogue_t;
sc_status_t sparse_conv_plan_set_epilogue(sparse_conv_plan_t* plan, const sc_epilogue_t* ep,
                                          const float* requant_scale, void* stream);

/* Which implementation sparse_conv_forward runs for a plan. */
enum {
    SC_PATH_SPARSE = 0,   /* the gather kernels (SC_VARIANT_GATHER / SC_VARIANT_SLAB) */
    SC_PATH_DENSE = 1,    /* the library's densified tile on the matrix cores (SC_VARIANT_DENSE) */
    SC_PATH_LIBRARY = 2   /* the dense library's convolution (MIOpen, looked up at run time) */
};

/* Record of sparse_conv_plan_dispatch: milliseconds per forward pass of each contender (-1: not
 * available for this layer or machine), the launch shapes of the two in-library contenders, and
 * the choice that was installed. */
typedef struct {
    int32_t choice;              /* SC_PATH_* */
    float sparse_ms;             /* gather kernels, tuned, cold ring */
    float dense_ms;              /* densified MFMA tile, tuned, cold ring */
    float library_ms;            /* dense library on the caller's buffer pair (cache-warm) */
    sc_tuning_t sparse_tuning;
    sc_tuning_t dense_tuning;
} sc_dispatch_t;

/* Per-layer dispatch: steps 3 and 4 of the paper's "Main scheme" -- compare the layer's time in the
 * sparse kernel with the dense convolution's, then configure the network layer by layer.  Tunes the
 * gather kernels and (16- / 8-bit activations) the densified MFMA tile like
 * sparse_conv_plan_autotune, each over the cold ring, sets up the dense library's convolution of
 * the same layer from the plan's weights (fp32 / fp16 layers, when a MIOpen is in the process or
 * can be loaded; NCHW buffers, whatever layout changes the library makes are inside its time) and
 * times it on the caller's buffers, records all three in *out and installs the fastest (the
 * library only when it wins by more than 10 %, its figure being cache-warm).  sparse_conv_forward
 * then runs that path; with SC_PATH_LIBRARY it must be called with the N given here and a workspace
 * of sparse_conv_workspace_size bytes.  A later sparse_conv_plan_set_tuning / _autotune goes back
 * to the library's own kernels.  y_dev is overwritten; synchronises; workspace as for
 * sparse_conv_plan_autotune (the library's own workspace is allocated for the measurement if the
 * caller's is too small).
 * Errors: as sparse_conv_plan_autotune. */
sc_status_t sparse_conv_plan_dispatch(sparse_conv_plan_t* plan, const void* x_dev, void* y_dev, int32_t N,
                                      void* workspace_dev, size_t workspace_bytes, void* stream,
                                      sc_dispatch_t* out);

/* After sparse_conv_plan_dispatch: run another of the contenders it measured (its recorded launch
 * shape, or the dense library with the algorithm it picked) -- the "configure the network" step of
 * the paper's main scheme done by hand.  SC_ERR_UNSUPPORTED if there was no dispatch yet or that
 * contender was not available. */
sc_status_t sparse_conv_plan_set_path(sparse_conv_plan_t* plan, int32_t path, void* stream);

/* Number of candidates sparse_conv_plan_autotune would time for this plan, and the i-th of them
 * (for tests that check that every candidate computes the same result). */
sc_status_t sparse_conv_plan_num_candidates(const sparse_conv_plan_t* plan, int32_t* count);
sc_status_t sparse_conv_plan_candidate(const sparse_conv_plan_t* plan, int32_t index,
                                       sc_tuning_t* tuning);

/* Plan-time helper, host only: the paper's linear fixed-point quantiser (section "Quantisation",
 * the mapping q = mu + sigma * round((x - mu) / sigma) with mu = 0 and a power-of-two step):
 *     m         = saturate_at * max |x|                  (saturate_at = 1: no saturation; the paper
 *                                                         saturates activations at 0.99)
 *     int_bits  = ceil(log2(m)),  frac_bits = total_bits - int_bits - 1,  sigma = 2^-frac_bits
 *     code      = round(clip(x, -m, m) / sigma)           nearest, ties to even
 * saturated to the two's-complement range [-2^(total_bits-1), 2^(total_bits-1) - 1]; the quantised
 * value is sigma * code.  One sigma for the whole array (per tensor), so the codes of a weight
 * tensor and of an activation tensor feed SC_I8 directly, with 2^-frac_bits as the scale.
 *   x      [count] host f32, finite          codes [count] host i8
 *   total_bits 2..8                          saturate_at in (0, 1]
 *   *frac_bits receives frac_bits (may be negative or exceed total_bits; all-zero input: total_bits - 1)
 * Errors: SC_ERR_NULL (x or codes NULL with count > 0, frac_bits NULL), SC_ERR_UNSUPPORTED
 * (total_bits or saturate_at out of range), SC_ERR_RANGE (a non-finite element). */
sc_status_t sparse_conv_quantize_pow2(const float* x, size_t count, int32_t total_bits,
                                      float saturate_at, int8_t* codes, int32_t* frac_bits);

const char* sparse_conv_status_string(sc_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_CONV_H */
