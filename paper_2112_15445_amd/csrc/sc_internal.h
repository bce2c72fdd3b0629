// Internal declarations shared by the translation units of libsparseconv (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

#include "sparse_conv.h"

namespace sc {

constexpr int kMaxLdsBytes = 160 * 1024;  // LDS per CU on gfx950 (one workgroup may take all of it)
constexpr int kNumCU = 256;
constexpr int kWave = 64;
constexpr int kMaxVpt = 8;                // output positions per lane in the slab kernel

// Geometry of the SLAB variant for one (plan, tuning) pair, all derived on the host.
//
// The output plane is cut into tiles of TP x TQ pixels.  For one tile the workgroup stages, per
// input channel, the input region the tile needs, split by stride phase into nsub = nsh*nsw
// sub-planes of SR rows x Qs columns (row pitch Qs), so that a tile-local output position
//     f = tp*Qs + tq
// reads, for filter tap (c, r, s), the LDS element
//     f + c*chan_pitch + ((r % nsh')*nsw + (s % nsw'))*sub_pitch + (r / s_h)*Qs + (s / s_w)
// i.e. "position + pre-stretched offset", exactly the addressing of Algorithm 3 but inside the tile.
// Positions with tq >= TQ are computed on halo data and discarded at the store.
// Pointwise layers (1x1, stride 1, no padding) are flattened to a single row of H*W pixels.
struct SlabGeom {
    int Hf, Wf, Pf, Qf;        // (possibly flattened) input and output extents
    int TP, TQ;                // output tile
    int tiles_p, tiles_q;      // tiles per sample along each axis
    int nsh, nsw;              // stride phases that are actually referenced: min(R, s_h), min(S, s_w)
    int SR, Qs;                // rows / row pitch of one sub-plane
    int sub_pitch, chan_pitch; // elements
    int F;                     // flat positions per tile = TP*Qs
    int vpt;                   // ceil(F / 64); packed positions: 32-bit words per lane, ceil(F / (64*pack))
    int pack;                  // positions per lane and LDS read: 1, or 2 (f16) / 4 (i8) with tuning.pack
    int copies, copy_bytes;    // packed one-shot form: images of a chunk in LDS, copy s shifted by s elements
    int slab_bytes;            // C*chan_pitch*e_x rounded up to 16
    int wcap;                  // (theta, lambda) entries per weight stage in LDS
    int DS, JC;                // rows per stage, entries per row per stage
    int lds_bytes;             // total dynamic LDS
    int vec;                   // 1: slab rows can be staged with 16-byte loads
    int dmab;                  // bytes per lane of the direct-to-LDS copy the rows allow: 16, 4 or 0
    int ns;                    // samples per workgroup (chunked one-shot form, tiles of <= 64 positions)
    int si;                    // 1: an LDS word holds the same position of `pack` consecutive samples (tuning.pack = 3)
    int sg;                    // ... and this many such sample groups per workgroup, laid along the lanes (tuning.sub_batch)
    int srow;                  // interleaved samples staged by rows (tuning.stage_rows)
    int ksplit;                // chunked one-shot form: workgroups that share the chunks of a tile (tuning.split_n; 1: off)
    int nbuf;                  // chunk buffers of the producer/consumer form with channel chunks (2, or producers + 1)
    int fs;                    // samples laid end to end along the tile's position axis (packed one-shot chunked form on pointwise layers); 1: off
    int nwaves;
    float inv_chan_pitch, inv_sub_pitch, inv_Qs;
    // channel-chunked pipelined form (tuning.chunk_c > 0)
    int CC, nchunks;           // channels per LDS buffer, buffers per tile
    int DTW, ndt;              // output channels per workgroup, workgroup columns
    int rpw;                   // output channels per consumer wave, ceil(DTW / consumers)
};

// Geometry of the DENSE (matrix-core) variant for one (plan, tuning) pair.
struct MfmaGeom {
    int TP, NS;            // output rows and samples per workgroup (NS > 1 only with whole planes)
    int tiles_p;           // row tiles per sample
    int Hs, Ws;            // staged input rows / columns of one sample (halo and padding included)
    int npos_s, npos;      // staged positions and output positions per workgroup
    int NCB;               // channel blocks of 32 (f16) / 64 (i8) input channels, ceil(C / block)
    int CC, nchunks;       // input channels per LDS chunk (a multiple of the block), chunks
    int pitch;             // bytes per staged position
    int DB, ndb;           // output channels per workgroup, blocks of them
    int WM, MW, NW;        // waves along the output channels; 16-row / 16-column blocks per wave
    int KG;                // groups of four waves that split the steps of the contraction (1 or 2)
    int PW;                // pipelined form: waves that stage the chunks (0 = the one-shot form)
    int bufsz;             // bytes of one chunk buffer
    int nat;               // 1 = pointwise layer staged in its natural layout ([channel][position])
    int DL;                // one-shot form: blocks of DB output channels a workgroup walks over (1 = one)
    int lds_bytes;
    int epi_pitch;         // elements per output-channel row of the LDS exchange of the fused epilogue
};

struct LibraryConv;   // dense_library.hip: the dense library's convolution of this layer (per-layer dispatch)

struct Plan {
    sc_layer_t L;
    sc_dtype_t dtype;
    int n = 0;
    int np = 0;                     // n rounded up to an even count (row pitch of d_wl32)
    int Hp = 0, Wp = 0, P = 0, Q = 0;
    int64_t X_size = 0;
    int64_t true_nnz = 0;
    int ex = 4, ey = 4;             // bytes per input / output element
    std::vector<int32_t> h_col;     // [D*n] unified table, columns ascending per row
    std::vector<int32_t> h_len;     // [D] stored entries of every row before unification
    int32_t* d_col = nullptr;       // [D*n]
    void* d_theta = nullptr;        // [D*n] f32 | f16 | i8, or ceil(D*n/2) bytes of packed 4-bit indices
    int32_t* d_lam = nullptr;       // [D*n] canonical offsets (elements into one padded sample)
    int32_t* d_lam_slab = nullptr;  // [D*n] byte offsets into the LDS slab of the current tuning
    int32_t* d_lam_slab_spare = nullptr;  // the buffer the next tuning's offsets are built in
    int2* d_wl32_spare = nullptr;   // likewise for d_wl32
    int2* d_wlc = nullptr;          // chunked form of that table: segments (row, chunk), even-padded
    int32_t* d_seg_off = nullptr;   // [D*nchunks + 1] start of every segment in d_wlc (entries)
    int32_t* d_first_j = nullptr;   // [D*nchunks] index within its row of a segment's first entry
    int2* d_wl32 = nullptr;         // [D*np] {theta widened to 32 bits, slab byte offset} for scalar loads
    float* d_scales = nullptr;      // [D]
    void* d_codebook = nullptr;     // [16] i8 or f16 centroids
    unsigned char* d_wfrag = nullptr;  // dense weights in MFMA operand order (DENSE variant), built on first use
    int32_t* d_len = nullptr;       // [D] stored entries of every row before unification (device copy of h_len)
    bool has_dup = false;           // some row stores a column twice (such a table cannot be densified exactly)
    sc_epilogue_t epi{};            // fused epilogue (all zero: none)
    float* d_requant = nullptr;     // [D] requantisation multipliers (epi.requant)
    int Po = 0, Qo = 0;             // extents of y: (P, Q), halved when the epilogue pools
    LibraryConv* libconv = nullptr; // set by sparse_conv_plan_dispatch when it measured the dense library
    int path = 0;                   // SC_PATH_*: which implementation sparse_conv_forward runs
    sc_dispatch_t dispatch{};       // the last record of sparse_conv_plan_dispatch (choice -1 before the first)
    sc_tuning_t tuning{};
    SlabGeom geom{};
    MfmaGeom mg{};
    int last_N = 0;
};

// plan.hip
sc_status_t resolve_tuning(const Plan& p, const sc_tuning_t& in, sc_tuning_t* out, SlabGeom* geom, MfmaGeom* mgeom);
sc_status_t launch_stretch(const Plan& p, int32_t* d_out, int nsh, int nsw, int s_h, int s_w,
                           int chan_pitch, int sub_pitch, int row_pitch, int scale, int chan_mod,
                           hipStream_t stream);
int elem_size_x(sc_dtype_t dt);
int elem_size_y(sc_dtype_t dt);

// gather.hip
size_t gather_workspace_bytes(const Plan& p, int N);
int gather_grid_size(const Plan& p, const sc_tuning_t& t, int N);
sc_status_t launch_gather(const Plan& p, const void* x, void* y, int N, void* ws, size_t ws_bytes,
                          hipStream_t stream);

// slab.hip
sc_status_t launch_slab(const Plan& p, const void* x, void* y, int N, hipStream_t stream);
int slab_grid_size(const Plan& p, const SlabGeom& g, int N);
bool slab_rows_stageable(const Plan& p, const SlabGeom& g);   // tuning.stage_rows applies to this layer and tile
sc_status_t expand_weights(const Plan& p, const int32_t* lam_slab, int2* wl32_out, hipStream_t stream);
sc_status_t expand_weights_chunked(const Plan& p, const SlabGeom& g, const int32_t* lam_slab, const int32_t* seg_off,
                                   const int32_t* first_j, int2* wlc_out, hipStream_t stream);
constexpr int kMaxRowsPerWave = 8;

// dense_library.hip
sc_status_t library_conv_create(const Plan& p, const void* x, void* y, int N, hipStream_t stream, LibraryConv** out);
sc_status_t library_conv_forward(LibraryConv* c, const void* x, void* y, int N, void* ws, size_t ws_bytes, hipStream_t stream);
size_t library_conv_workspace(const LibraryConv* c);
int library_conv_batch(const LibraryConv* c);
void library_conv_destroy(LibraryConv* c);

// dense_mfma.hip
int mfma_chan_block(sc_dtype_t dt);
size_t mfma_weight_bytes(const Plan& p);
sc_status_t mfma_densify(const Plan& p, unsigned char* out, hipStream_t stream);
bool mfma_geometry(const Plan& p, int TP, int NS, int CC, int DB, int WM, int lds_budget, MfmaGeom* out, int KG = 1, int PW = 0, int nat = 0, int DL = 1);
inline bool has_epilogue(const Plan& p) { return p.epi.relu || p.epi.pool || p.epi.requant; }
int mfma_grid_size(const Plan& p, const MfmaGeom& g, int N);
sc_status_t launch_mfma(const Plan& p, const void* x, void* y, int N, hipStream_t stream);

}  // namespace sc
