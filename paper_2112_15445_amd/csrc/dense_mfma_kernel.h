// Kernel of the DENSE variant (the densified tile on the matrix cores) and its typed launcher;
// included by dense_mfma.hip (host side) and by the two translation units that instantiate it for
// 16-bit and 8-bit activations.  See dense_mfma.hip for the formulation.
#pragma once

#include <mutex>
#include <type_traits>

#include "sc_device.h"
#include "sc_dma.h"
#include "sc_internal.h"

namespace sc {

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef int int4v_ __attribute__((ext_vector_type(4)));
typedef unsigned uint4w __attribute__((ext_vector_type(4)));

// (Measured on this chip: the 16 x 16 block instructions used here sustain 1.3 PFLOP/s in fp16
// with four waves per SIMD and 0.8 with one, the 32 x 32 ones 2.3 and 2.0.  The layers this
// variant serves are too small for the wave tiles of 64 x 128 outputs that the 32 x 32 form needs
// to be fed from LDS and L2 at that rate: built that way it was 10 - 40 % slower on every layer
// tried, so the blocks stay 16 x 16.)
template <sc_dtype_t DT> constexpr bool kIntActs = DT == SC_I8 || DT == SC_CB4_I8;
// input channels contracted by one MFMA, and held by one lane (16 bytes)
template <sc_dtype_t DT> constexpr int kChanBlock = kIntActs<DT> ? 64 : 32;
template <sc_dtype_t DT> constexpr int kChanVec = kIntActs<DT> ? 16 : 8;

struct MfmaArgs {
    int C, D, N, H, W, P, Q, S, RS, s_h, s_w, pad_h, pad_w;
    int TP, NS, tiles_p, Hs, Ws, npos_s, npos, CC, nchunks, NCB, pitch, DB, ndb, epv;
    // pipelined form: bytes of one of the two chunk buffers; channel blocks of the last chunk; reciprocals
    // of the steps per full chunk, of the channel blocks per chunk (full, last) and of S
    int bufsz, cbs_last;
    int TPQ;                 // natural layout: positions of one sample in the tile (TP * Q)
    int DL, ndbg;            // one-shot form: output-channel blocks per workgroup, groups of them (ndb / DL, rounded up)
    float inv_ndbg;
    float inv_spc, inv_ccb, inv_cbs_last, inv_S;
    float inv_ndb, inv_tiles_p, inv_HsWs, inv_Ws, inv_TPQ, inv_Q;
    // fused epilogue (epi = 0: none): ReLU, 2 x 2 max-pooling, requantisation multipliers (or NULL),
    // row pitch of the LDS exchange, extents of y
    int epi, epi_relu, epi_pool, epi_pitch, Po, Qo;
    const float* requant;
};

sc_status_t launch_mfma_f16(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_i8(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_pipe_f16(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_pipe_i8(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_nat_f16(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_nat_i8(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_pipe_nat_f16(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_pipe_nat_i8(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_dl_f16(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);
sc_status_t launch_mfma_dl_i8(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream);

// floor(e / d) for 0 <= e < 2^19 given inv = 1.0f / d (exact: the half-integer bias keeps the
// product at least 1/(2d) away from every integer, well above the two float roundings)
__device__ inline int fdiv19(int e, float inv) { return (int)(((float)e + 0.5f) * inv); }

// ------------------------------------------------------------------------------------------------
// Staging of one chunk of CC input channels of the tile, transposed on the way: global memory is
// channel-major (NCHW), the LDS tile channel-minor.  One block = CV consecutive channels x EPV
// consecutive columns of one input row: CV loads of EPV elements each (the widest load the row
// length and the pointer allow: 16, 8, 4, 2 or 1 bytes), transposed in registers, written as EPV
// 16-byte LDS words (one staged position each).  Blocks are dealt to the threads column-group
// fastest, so the loads of a wave run along input rows; VB blocks per round, all loads of a round
// issued before the first is used.  Channels past the layer's last are written as zeros; positions
// that show padding (or samples past the batch) are zeroed by a second, cheap loop.
// ------------------------------------------------------------------------------------------------
struct StageArgs {
    int nsv;               // samples of this workgroup inside the batch
    int ilo, nrows;        // staged rows that lie inside the input: [ilo, ilo + nrows)
    int rlo;               // input row of staged row ilo
    int wcols;             // input columns that are staged: [0, wcols)
};

// blocks a thread has in flight per round: the multiplying waves keep this small (their registers
// hold accumulators); waves that only stage (the pipelined kernel) take about 64 registers' worth
template <int EPV> constexpr int kStageVB = EPV >= 8 ? 1 : (EPV >= 2 ? 2 : 4);
template <typename X, int CV, int EPV>
constexpr int stage_vb_wide()
{
    const int words = EPV * (int)sizeof(X) >= 4 ? EPV * (int)sizeof(X) / 4 : 1;   // registers per load
    const int v = 64 / (CV * words);
    return v > 8 ? 8 : (v < 1 ? 1 : v);
}

// padding: staged positions outside the input or past the batch are zeros
__device__ __forceinline__ void stage_pad(unsigned char* lds, int tid, int NT, int cgroups, const StageArgs& sa, const MfmaArgs& a)
{
    for (int pos = tid; pos < a.npos_s; pos += NT) {
        const int sm = fdiv19(pos, a.inv_HsWs);
        const int rem = pos - sm * (a.Hs * a.Ws);
        const int i = fdiv19(rem, a.inv_Ws);
        const int w = rem - i * a.Ws;
        const bool inside = sm < sa.nsv && i >= sa.ilo && i < sa.ilo + sa.nrows && w >= a.pad_w && w < a.pad_w + sa.wcols;
        if (!inside)
            for (int cg = 0; cg < cgroups; ++cg) *reinterpret_cast<uint4w*>(lds + pos * a.pitch + cg * 16) = uint4w{0u, 0u, 0u, 0u};
    }
}

template <typename X, int CV, int EPV, int VB>
__device__ __forceinline__ void stage_chunk(const X* __restrict__ xc, unsigned char* lds, int tid, int NT, int cgroups, int cleft,
                                            const StageArgs& sa, const MfmaArgs& a, int plane)
{
    struct alignas(EPV * sizeof(X)) Vec { X e[EPV]; };
    const int G = (sa.wcols + EPV - 1) / EPV;
    const int rowsG = sa.nrows * G, per_cg = sa.nsv * rowsG;
    const int nblocks = cgroups * per_cg;
    const float inv_per_cg = 1.0f / (float)max(per_cg, 1), inv_rowsG = 1.0f / (float)max(rowsG, 1), inv_G = 1.0f / (float)max(G, 1);
    for (int v0 = tid; v0 < nblocks; v0 += NT * VB) {
        Vec val[VB][CV];
        int dst[VB], vcg[VB], col[VB];
#pragma unroll
        for (int u = 0; u < VB; ++u) {
            const int v = v0 + u * NT;
            const int vv = v < nblocks ? v : 0;            // (past the end: block 0 again, not written)
            const int cg = fdiv19(vv, inv_per_cg);
            const int rb = vv - cg * per_cg;
            const int sm = fdiv19(rb, inv_rowsG);
            const int r2 = rb - sm * rowsG;
            const int ii = fdiv19(r2, inv_G);
            const int g = r2 - ii * G;
            vcg[u] = v < nblocks ? cg : -1;
            col[u] = g * EPV;
            dst[u] = ((sm * a.Hs + sa.ilo + ii) * a.Ws + a.pad_w + g * EPV) * a.pitch + cg * 16;
            const X* src = xc + sm * a.C * plane + (sa.rlo + ii) * a.W + g * EPV;
#pragma unroll
            for (int j = 0; j < CV; ++j) {
                const int c = cg * CV + j;
                val[u][j] = *reinterpret_cast<const Vec*>(src + (c < cleft ? c : 0) * plane);
            }
        }
#pragma unroll
        for (int u = 0; u < VB; ++u) {
            if (vcg[u] < 0) continue;
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                X o[CV];
#pragma unroll
                for (int j = 0; j < CV; ++j) o[j] = (vcg[u] * CV + j < cleft) ? val[u][j].e[e] : X(0);
                uint4w pk;
                __builtin_memcpy(&pk, o, 16);
                if (col[u] + e < sa.wcols) *reinterpret_cast<uint4w*>(lds + dst[u] + e * a.pitch) = pk;
            }
        }
    }
}

// the same for the load width the launch found (elements per load: the widest power of two, up to
// 16 bytes, that divides the row length and the caller's pointer)
template <typename X, int CV, bool WIDE>
__device__ __forceinline__ void stage_chunk_epv(int epv, const X* __restrict__ xc, unsigned char* lds, int tid, int NT, int cgroups,
                                                int cleft, const StageArgs& sa, const MfmaArgs& a, int plane)
{
#define SC_STAGE(E) stage_chunk<X, CV, E, WIDE ? stage_vb_wide<X, CV, E>() : kStageVB<E>>(xc, lds, tid, NT, cgroups, cleft, sa, a, plane)
    switch (epv) {
        case 16: if constexpr (sizeof(X) == 1) { SC_STAGE(16); } break;
        case 8: SC_STAGE(8); break;
        case 4: SC_STAGE(4); break;
        case 2: SC_STAGE(2); break;
        default: SC_STAGE(1); break;
    }
#undef SC_STAGE
}

// One step of the contraction = one filter tap x one block of CB input channels of the resident
// chunk.  The step counter and everything derived from it are wave-uniform and advance by scalar
// arithmetic; past the last step the counter stays where it is (the operand prefetch then reloads
// the last step's operands instead of branching).
struct StepCursor {
    int cb, r, s, tap;
    template <int STEPS = 1>
    __device__ __forceinline__ void advance(int cbs, int S, bool more)
    {
        if (!more) return;
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            if (++cb == cbs) {
                cb = 0;
                ++tap;
                if (++s == S) { s = 0; ++r; }
            }
        }
    }
};

// ------------------------------------------------------------------------------------------------
// Pointwise layers (1 x 1, unit stride, no padding), tuning.stage_rows = 1: the tile is staged in
// its natural layout, [channel][position] -- the positions of a tile are one contiguous run per
// (sample, channel) in NCHW, so staging is a plain copy with the widest loads the run lengths and
// the pointer allow and no transposition in registers -- and the MFMA operands are read with
// gfx950's transposing LDS reads.  ds_read_b64_tr_b16: in every group of 16 lanes, lane i receives
// element i % 4 of the 8-byte words that lanes 4 j + i / 4 addressed, j = 0 .. 3; when lanes
// 4 j .. 4 j + 3 address 16 consecutive positions of channel row j, lane i holds 4 channels of
// position i -- half of a 16-bit operand (two reads).  ds_read_b64_tr_b8 is the same with 8 rows
// of 16 one-byte positions (lanes 2 j, 2 j + 1 address row j): 8 channels per read.  Row pitch:
// a multiple of 64 bytes plus 32, so that the rows of a group fall into different banks.
// Columns past the tile's positions hold whatever LDS held (their outputs are not stored, and a
// column only feeds its own output); channel rows past the layer's last are written as zeros.
// ------------------------------------------------------------------------------------------------
#define SC_LDS_AS __attribute__((address_space(3)))
template <typename X>
__device__ __forceinline__ uint4w read_operand_tr(const unsigned char* lds, int off, int pitch)
{
    uint4w r;
    if constexpr (sizeof(X) == 2) {
        typedef __attribute__((__vector_size__(4 * sizeof(__fp16)))) __fp16 h4;
        const h4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4f16((SC_LDS_AS h4*)((SC_LDS_AS unsigned char*)lds + off));
        const h4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4f16((SC_LDS_AS h4*)((SC_LDS_AS unsigned char*)lds + off + 4 * pitch));
        __builtin_memcpy(&r, &lo, 8);
        __builtin_memcpy(reinterpret_cast<unsigned char*>(&r) + 8, &hi, 8);
    } else {
        typedef __attribute__((__vector_size__(2 * sizeof(int)))) int i2;
        const i2 lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((SC_LDS_AS i2*)((SC_LDS_AS unsigned char*)lds + off));
        const i2 hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((SC_LDS_AS i2*)((SC_LDS_AS unsigned char*)lds + off + 8 * pitch));
        __builtin_memcpy(&r, &lo, 8);
        __builtin_memcpy(reinterpret_cast<unsigned char*>(&r) + 8, &hi, 8);
    }
    return r;
}
#undef SC_LDS_AS

// copy of one chunk: `rows` channel rows (the first min(rows, cleft) from memory, the rest zeros),
// each nsv runs of cnt elements (cnt a multiple of EPV), run (sm, c) to columns sm * a.TPQ ...
template <typename X, int EPV>
__device__ __forceinline__ void stage_rows_nat(const X* __restrict__ xc, unsigned char* lds, int tid, int NT, int rows, int cleft,
                                               int nsv, int cnt, const MfmaArgs& a, int plane)
{
    struct alignas(EPV * sizeof(X)) Vec { X e[EPV]; };
    constexpr int VB = 8;                                  // loads in flight per thread
    const int G = cnt / EPV, per_c = nsv * G;
    const int live = min(rows, cleft);
    const int nblocks = live * per_c;
    const float inv_per_c = 1.0f / (float)max(per_c, 1), inv_G = 1.0f / (float)max(G, 1);
    for (int v0 = tid; v0 < nblocks; v0 += NT * VB) {
        Vec val[VB];
        int dst[VB];
#pragma unroll
        for (int u = 0; u < VB; ++u) {
            const int v = v0 + u * NT;
            const int vv = v < nblocks ? v : 0;            // (past the end: block 0 again, not written)
            const int c = fdiv19(vv, inv_per_c);
            const int rem = vv - c * per_c;
            const int sm = fdiv19(rem, inv_G);
            const int g = rem - sm * G;
            dst[u] = v < nblocks ? c * a.pitch + (sm * a.TPQ + g * EPV) * (int)sizeof(X) : -1;
            val[u] = *reinterpret_cast<const Vec*>(xc + (int64_t)(sm * a.C + c) * plane + g * EPV);
        }
#pragma unroll
        for (int u = 0; u < VB; ++u)
            if (dst[u] >= 0) *reinterpret_cast<Vec*>(lds + dst[u]) = val[u];
    }
    const int w16 = a.pitch >> 4;                          // 16-byte words per row
    for (int i = tid; i < (rows - live) * w16; i += NT)
        *reinterpret_cast<uint4w*>(lds + live * a.pitch + i * 16) = uint4w{0u, 0u, 0u, 0u};
}

// ------------------------------------------------------------------------------------------------
// What follows the contraction, shared by the kernels below: the step groups add up their
// accumulators (KG = 2), then the outputs are stored, with the fused epilogue if the plan has one.
// Called by the 256 * KG multiplying threads of the workgroup (tid = 0 .. 256 * KG - 1), all of them.
// ------------------------------------------------------------------------------------------------
template <sc_dtype_t DT, int MW, int NW, int WM, int KG, typename Acc>
__device__ __forceinline__ void mfma_finish(Acc (&acc)[MW][NW], const MfmaArgs& a, unsigned char* lds,
                                            typename Types<DT>::Y* __restrict__ y, int tid, int kgrp, int wm, int wn, int kg,
                                            int n16, int mblk0, const int64_t (&yoff)[NW], int b0, int p0, int db, int PQ)
{
    constexpr int NT = 256 * KG;
    if constexpr (KG > 1) {
        // ------------------------------------------------------------ the two step groups meet: the
        // second puts its accumulator blocks into LDS (the tile has been consumed), the first adds them
        using A = typename Types<DT>::A;
        __syncthreads();
        A* ex = reinterpret_cast<A*>(lds);
        if (kgrp == 1) {
#pragma unroll
            for (int m = 0; m < MW; ++m)
#pragma unroll
                for (int i = 0; i < NW; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        ex[((wm * MW + m) * 16 + 4 * kg + j) * a.epi_pitch + (wn * NW + i) * 16 + n16] = acc[m][i][j];
        }
        __syncthreads();
        if (kgrp == 1) {
            if (!a.epi_pool) return;                       // (the pooling epilogue below needs every thread)
        } else {
#pragma unroll
            for (int m = 0; m < MW; ++m)
#pragma unroll
                for (int i = 0; i < NW; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[m][i][j] += ex[((wm * MW + m) * 16 + 4 * kg + j) * a.epi_pitch + (wn * NW + i) * 16 + n16];
        }
    }
    if (a.epi_pool) {
        // ------------------------------------------------------------ fused epilogue with pooling: the waves
        // put their accumulator blocks into LDS as [output channel][tile position] (the tile has
        // been consumed), then every thread finishes elements of y: the maximum over its 2 x 2
        // window, ReLU, and the store -- as the layer's type or, requantised, as an 8-bit code.
        // The stores run along the rows of y.  (Without pooling the epilogue is elementwise and is
        // applied where the accumulators are stored, below.)
        using A = typename Types<DT>::A;
        __syncthreads();
        A* ex = reinterpret_cast<A*>(lds);
        if (kgrp == 0) {
#pragma unroll
            for (int m = 0; m < MW; ++m)
#pragma unroll
                for (int i = 0; i < NW; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        ex[((wm * MW + m) * 16 + 4 * kg + j) * a.epi_pitch + (wn * NW + i) * 16 + n16] = acc[m][i][j];
        }
        __syncthreads();
        const int pl = a.epi_pool ? 2 : 1;
        const int TPo = a.TP / pl;                          // output rows of y per tile (TP is even, or the whole plane)
        const int per_s = TPo * a.Qo, per_d = a.NS * per_s; // elements of y per output channel of the tile
        const float inv_per_s = 1.0f / (float)max(per_s, 1), inv_Qo = 1.0f / (float)a.Qo;
        const int prow0 = p0 / pl;
        // a thread keeps to one element position of the tile (decoded once) and walks over the
        // output channels; the threads are laid out as (channel group, position) with the
        // positions a power of two wide, so that small tiles still use every thread and the
        // stores of a wave run along the rows of y
        int pw2 = 1;
        while (pw2 < per_d && pw2 < NT) pw2 <<= 1;
        const int dgroups = NT / pw2;
        const int o_first = tid & (pw2 - 1), dg = tid / pw2;
        for (int o = o_first; o < per_d; o += pw2) {
            const int sm = fdiv19(o, inv_per_s);
            const int r2 = o - sm * per_s;
            const int tpo = fdiv19(r2, inv_Qo);
            const int tqo = r2 - tpo * a.Qo;
            if (b0 + sm >= a.N || prow0 + tpo >= a.Po) continue;
            const A* src = ex + sm * (a.TP * a.Q) + (tpo * pl) * a.Q + tqo * pl;
            const int64_t off0 = (((int64_t)(b0 + sm) * a.D) * a.Po + prow0 + tpo) * a.Qo + tqo;
            const int64_t dstride = (int64_t)a.Po * a.Qo;
            for (int dl = dg; dl < a.DB; dl += dgroups) {
                const int d = db * a.DB + dl;
                if (d >= a.D) break;
                const A* sp = src + dl * a.epi_pitch;
                A v = sp[0];
                if (a.epi_pool) v = max(max(sp[0], sp[1]), max(sp[a.Q], sp[a.Q + 1]));
                if (a.epi_relu) v = max(v, A(0));
                const int64_t off = off0 + d * dstride;
                if constexpr (kIntActs<DT>) {
                    if (a.requant) {
                        const float q = rintf(__int2float_rn(v) * a.requant[d]);
                        reinterpret_cast<int8_t*>(y)[off] = (int8_t)(int)fminf(fmaxf(q, -127.0f), 127.0f);
                        continue;
                    }
                }
                store_out(y + off, narrow<DT>(v));
            }
        }
        return;
    }
    // ---------------------------------------------------------------- store: a lane holds, for its
    // position (column n16 of the block), the four output channels 4 * kg .. 4 * kg + 3 of each row block
    if (!a.epi) {
#pragma unroll
        for (int m = 0; m < MW; ++m) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int d = (mblk0 + m) * 16 + 4 * kg + j;
                if (d < a.D) {
#pragma unroll
                    for (int i = 0; i < NW; ++i)
                        if (yoff[i] >= 0) store_out(y + yoff[i] + (int64_t)d * PQ, narrow<DT>(acc[m][i][j]));
                }
            }
        }
        return;
    }
    // the same with an elementwise epilogue: ReLU and / or requantisation to 8-bit codes on the way
    // (a branch of its own, so that the plain store above keeps its registers and schedule)
#pragma unroll
    for (int m = 0; m < MW; ++m) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int d = (mblk0 + m) * 16 + 4 * kg + j;
            if (d < a.D) {
                float rq = 0.0f;
                if constexpr (kIntActs<DT>) {
                    if (a.requant) rq = a.requant[d];
                }
#pragma unroll
                for (int i = 0; i < NW; ++i) {
                    if (yoff[i] < 0) continue;
                    auto v = acc[m][i][j];
                    if (a.epi_relu) v = max(v, decltype(v)(0));
                    if constexpr (kIntActs<DT>) {
                        if (a.requant) {
                            const float q = rintf(__int2float_rn(v) * rq);
                            reinterpret_cast<int8_t*>(y)[yoff[i] + (int64_t)d * PQ] = (int8_t)(int)fminf(fmaxf(q, -127.0f), 127.0f);
                            continue;
                        }
                    }
                    store_out(y + yoff[i] + (int64_t)d * PQ, narrow<DT>(v));
                }
            }
        }
    }
}

// KG = 2: eight waves.  The two groups of four waves own the same outputs and take the even and the odd
// steps of the contraction; their accumulators meet through LDS at the end (a fixed order: the
// result does not depend on timing).  Two waves then share a SIMD, which is what the matrix
// instructions need to issue back to back, at no more traffic: every operand is still fetched once.
template <sc_dtype_t DT, int MW, int NW, int WM, int KG, bool NAT>
__global__ void __launch_bounds__(256 * KG)
mfma_conv_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                 const uint4w* __restrict__ wfrag, const MfmaArgs a)
{
#define SC_DL_DECODE const int bt = fdiv19(wg, a.inv_ndb); const int db = wg - bt * a.ndb;
#define SC_DL_MBLK0 const int mblk0 = db * (a.DB >> 4) + wm * MW;            /* first 16-row block of this wave */
#define SC_DL_BEGIN
#define SC_DL_IF_FIRST
#define SC_DL_END
#include "dense_mfma_conv_body.inc"
#undef SC_DL_DECODE
#undef SC_DL_MBLK0
#undef SC_DL_BEGIN
#undef SC_DL_IF_FIRST
#undef SC_DL_END
}

// The same with tuning.split_n blocks of tile_d output channels per workgroup, one after the other: the
// tile is staged once (a single chunk) and stays in LDS, and the stores of one block drain while the
// next is multiplied -- for layers with few input and many output channels, where a workgroup per
// block would spend its time starting, staging and draining.  Four waves, no exchange through LDS
// (no pooling).
template <sc_dtype_t DT, int MW, int NW, int WM, int KG, bool NAT>
__global__ void __launch_bounds__(256 * KG)
mfma_conv_dl_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                    const uint4w* __restrict__ wfrag, const MfmaArgs a)
{
#define SC_DL_DECODE const int bt = fdiv19(wg, a.inv_ndbg); const int db0 = (wg - bt * a.ndbg) * a.DL;
#define SC_DL_MBLK0
#define SC_DL_BEGIN                                                                           \
    for (int it = 0; it < a.DL; ++it) {                                                       \
        const int db = db0 + it;                                                              \
        if (db >= a.ndb) break;                                                               \
        const int mblk0 = db * (a.DB >> 4) + wm * MW;                                         \
        if (it > 0) {                                                                         \
            _Pragma("unroll") for (int m = 0; m < MW; ++m)                                    \
                _Pragma("unroll") for (int i = 0; i < NW; ++i) acc[m][i] = Acc{0, 0, 0, 0};   \
        }
#define SC_DL_IF_FIRST if (it == 0)
#define SC_DL_END }
#include "dense_mfma_conv_body.inc"
#undef SC_DL_DECODE
#undef SC_DL_MBLK0
#undef SC_DL_BEGIN
#undef SC_DL_IF_FIRST
#undef SC_DL_END
}

// ------------------------------------------------------------------------------------------------
// The pipelined form (tuning.pipeline = 1): the same tile, contraction and weight layout, but the
// chunks of input channels are staged by waves of their own (tuning.producers of them, behind the
// 4 * KG multiplying waves) into two LDS buffers, one chunk ahead of the multiplication.  The
// multiplying waves run over the steps of all chunks in one loop -- the ring of weights in flight
// never drains -- and meet the staging waves at one barrier per chunk: barrier k says "chunk k is
// staged" and, with it, "chunk k - 1 has been multiplied" (so its buffer may take chunk k + 1).
// The barriers wait for LDS traffic only (s_waitcnt lgkmcnt(0)): the weights a wave has in flight
// from L2 stay in flight across them.  With KG = 2 the two groups take the even and the odd steps
// of that one sequence.  Small chunks are the point: only the first is staged before any
// multiplication starts, and the two buffers of a small chunk leave LDS for more workgroups.
// The staging waves end when the last chunk is staged; the barriers of the epilogue are then met
// by the multiplying waves alone (a barrier waits only for the waves of a workgroup that have
// not ended).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// NAT (pointwise layers, tuning.stage_rows = 1): the chunk buffers hold the tile in its natural
// layout, [channel][position] with no padding between the rows -- the image the direct-to-LDS
// loads of gfx950 write, so the staging waves copy a chunk without touching a register -- and the
// operands are read with the transposing LDS reads (see above).  One sample per workgroup.
template <sc_dtype_t DT, int MW, int NW, int WM, int KG, bool NAT>
__global__ void __launch_bounds__(256 * KG + 256)
mfma_pipe_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                 const uint4w* __restrict__ wfrag, const MfmaArgs a)
{
    using X = typename Types<DT>::X;
    using Acc = typename std::conditional<kIntActs<DT>, int4v_, float4v>::type;
    constexpr int CB = kChanBlock<DT>, CV = kChanVec<DT>;
    constexpr int NTC = 256 * KG;                            // multiplying threads
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave8 >= 4 * KG;

    const int grid = gridDim.x;
    const int wg = (grid & 7) == 0 ? (int)(blockIdx.x & 7) * (grid >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int bt = fdiv19(wg, a.inv_ndb);
    const int db = wg - bt * a.ndb;
    const int bg = fdiv19(bt, a.inv_tiles_p);
    const int tpi = bt - bg * a.tiles_p;
    const int b0 = bg * a.NS, p0 = tpi * a.TP;
    const int row0 = p0 * a.s_h - a.pad_h;
    const int plane = a.H * a.W, PQ = a.P * a.Q;
    const int cgroups = a.CC / CV;                           // 16-byte channel groups per staged position
    const int CCB = a.CC / CB;                               // channel blocks per chunk (the last may have fewer)

    StageArgs sa;
    sa.nsv = min(a.NS, a.N - b0);
    sa.ilo = max(0, -row0);
    sa.nrows = max(0, min(a.Hs, a.H - row0) - sa.ilo);
    sa.rlo = row0 + sa.ilo;
    sa.wcols = min(a.W, a.Ws - a.pad_w);
    const X* xb = x + (int64_t)b0 * a.C * plane;

    if (producer) {
        const int ptid = tid - NTC, pn = (int)blockDim.x - NTC;
        for (int k = 0; k < a.nchunks; ++k) {
            const int c0 = k * a.CC;
            if constexpr (NAT) {
                // rows of this chunk (whole channel blocks), those of them that exist in the layer
                const int rows = min(CCB, a.NCB - k * CCB) * CB, live = min(rows, a.C - c0);
                unsigned char* buf = lds + (k & 1) * a.bufsz;
                dma_tile<X>(xb + (int64_t)c0 * plane + p0 * a.Q, buf, live, a.TPQ, plane, p0 * a.Q, ptid >> 6, pn >> 6, lane, a.inv_TPQ);
                for (int i = ptid; i < (rows - live) * a.pitch / 16; i += pn)
                    *reinterpret_cast<uint4w*>(buf + live * a.pitch + i * 16) = uint4w{0u, 0u, 0u, 0u};
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the copies of this wave have landed
            } else {
                stage_chunk_epv<X, CV, true>(a.epv, xb + (int64_t)c0 * plane, lds + (k & 1) * a.bufsz, ptid, pn, cgroups, a.C - c0, sa, a, plane);
            }
            lds_barrier();                                   // barrier k
        }
        return;
    }

    const int kgrp = KG > 1 ? wave8 >> 2 : 0;
    const int wave = wave8 & 3;
    const int wm = wave % WM, wn = wave / WM;
    const int n16 = lane & 15, kg = lane >> 4;

    int bbase[NW];                                           // (filled in below, once the first loads are out)
    int64_t yoff[NW];
    Acc acc[MW][NW];
    const int mblk0 = db * (a.DB >> 4) + wm * MW;
    const int wrow = a.RS * a.NCB * 64;

    // The steps of all chunks in one sequence: chunk, then filter tap, then channel block of the
    // chunk.  What a step needs -- the byte offset of its tile operands in LDS, of its weights in
    // the weight array, and its chunk -- is computed 64 steps at a time, one step per lane, and
    // read back with v_readlane: the loop itself carries no cursor arithmetic and no branches
    // but the barrier test.  Steps past the wave's last repeat the last (operands are prefetched
    // without a test).
    const int total = a.RS * a.NCB;
    const int nsteps = KG > 1 ? (total - kgrp + KG - 1) / KG : total;    // this wave's steps
    const int last = max(nsteps - 1, 0);
    const int SPC = a.RS * CCB;                              // steps of a full chunk
    auto table = [&](int base, int& vt, int& vw, int& vc) {
        const int g = kgrp + KG * min(base + lane, last);
        const int ch = fdiv19(g, a.inv_spc);
        const int rem = g - ch * SPC;
        const bool tail = ch == a.nchunks - 1;
        const int cbs = tail ? a.cbs_last : CCB;
        const int tap = fdiv19(rem, tail ? a.inv_cbs_last : a.inv_ccb);
        const int cb = rem - tap * cbs;
        const int r = fdiv19(tap, a.inv_S);
        const int sx = tap - r * a.S;
        vt = NAT ? (ch & 1) * a.bufsz + cb * CB * a.pitch
                 : (ch & 1) * a.bufsz + (r * a.Ws + sx) * a.pitch + cb * (CB * (int)sizeof(X));
        vw = (tap * a.NCB + ch * CCB + cb) * 1024;           // (64 lanes x 16 bytes per operand block)
        vc = ch;
    };
    constexpr int PF = MW >= 4 ? 4 : 6;                      // steps of weights in flight
    uint4w aq[PF][MW], bq[2][NW];
    int wtab, xtab, ctab, unused0, unused1;
    table(0, xtab, wtab, ctab);
    int wi = 0, wbase = 0, xi = 0, xbase = 0, nbar = 0;
    // the weights of this wave's row blocks: a wave-uniform base (per step) plus a per-lane offset
    const unsigned char* wrows = reinterpret_cast<const unsigned char*>(wfrag) + (int64_t)mblk0 * wrow * 16;
    unsigned woffm[MW];
#pragma unroll
    for (int m = 0; m < MW; ++m) woffm[m] = (unsigned)(m * wrow + lane) * 16u;
    const unsigned char* wstep = wrows;
    auto next_w = [&]() {                                    // the weight cursor moves on one step
        if (wi == 64) { wbase += 64; wi = 0; table(wbase, unused0, wtab, unused1); }
        wstep = wrows + __builtin_amdgcn_readlane(wtab, wi);
        ++wi;
    };
    auto fetch_w1 = [&](uint4w& av, int m) { av = *reinterpret_cast<const uint4w*>(wstep + woffm[m]); };
    auto fetch_x = [&](uint4w (&bv)[NW]) {
        if (xi == 64) { xbase += 64; xi = 0; table(xbase, xtab, unused0, ctab); }
        const int toff = __builtin_amdgcn_readlane(xtab, xi);
        const int ch = __builtin_amdgcn_readlane(ctab, xi);
        ++xi;
        while (nbar <= ch) { lds_barrier(); ++nbar; }        // the chunk of this step is staged
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            if constexpr (NAT) bv[i] = read_operand_tr<X>(lds, bbase[i] + toff, a.pitch);
            else bv[i] = *reinterpret_cast<const uint4w*>(lds + bbase[i] + toff);
        }
    };
    auto mfma1 = [&](Acc& c, const uint4w& av, const uint4w& bv) {
        if constexpr (kIntActs<DT>)
            c = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(int4v_, av), __builtin_bit_cast(int4v_, bv), c, 0, 0, 0);
        else
            c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, av), __builtin_bit_cast(half8v, bv), c, 0, 0, 0);
    };
    if (nsteps > 0) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            next_w();
#pragma unroll
            for (int m = 0; m < MW; ++m) fetch_w1(aq[u][m], m);
        }
    }
    // The padding of both buffers is written once, here, while the first chunk and the first
    // weights are on their way (the staging waves went straight to their loads): staging never
    // touches it, and the first barrier orders it before any read.
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (!NAT) {
        stage_pad(lds, tid, NTC, cgroups, sa, a);
        if (a.nchunks > 1) stage_pad(lds + a.bufsz, tid, NTC, cgroups, sa, a);
    }

    // positions of this lane's NW column blocks (as in the one-shot kernel), and the accumulators
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const int f = ((wn * NW + i) * 16 + n16);
        const int sm = fdiv19(f, a.inv_TPQ);
        const int rem = f - sm * (a.TP * a.Q);
        const int tp = fdiv19(rem, a.inv_Q);
        const int tq = rem - tp * a.Q;
        const bool ok = f < a.npos && b0 + sm < a.N && p0 + tp < a.P;
        if constexpr (NAT) {
            constexpr int LPR = sizeof(X) == 2 ? 4 : 2;        // lanes per row of a group of the transposing read
            bbase[i] = (kg * CV + n16 / LPR) * a.pitch + (wn * NW + i) * 16 * (int)sizeof(X) + (n16 % LPR) * 8;
        } else {
            bbase[i] = (ok ? ((sm * a.Hs + tp * a.s_h) * a.Ws + tq * a.s_w) * a.pitch : 0) + kg * 16;
        }
        yoff[i] = ok ? ((int64_t)(b0 + sm) * a.D) * PQ + (p0 + tp) * a.Q + tq : -1;
    }

#pragma unroll
    for (int m = 0; m < MW; ++m)
#pragma unroll
        for (int i = 0; i < NW; ++i) acc[m][i] = Acc{0, 0, 0, 0};

    if (nsteps > 0) {
        fetch_x(bq[0]);
        __builtin_amdgcn_sched_barrier(0);
        const int main_steps = nsteps / PF * PF;
        for (int ks = 0; ks < main_steps; ks += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                // Step ks + u.  The tile operands of the next step are requested first; a row of
                // weights is requested again (for step ks + u + PF) as soon as the matrix
                // instructions that read it have been issued, so that the address arithmetic and
                // the loads issue while the matrix pipe works.  The barrier at the end keeps the
                // compiler from moving loads from one step into another.
                fetch_x(bq[(u + 1) & 1]);
                next_w();
#pragma unroll
                for (int m = 0; m < MW; ++m) {
#pragma unroll
                    for (int i = 0; i < NW; ++i) mfma1(acc[m][i], aq[u][m], bq[u & 1][i]);
                    fetch_w1(aq[u][m], m);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int u = 0; u < PF - 1; ++u) {
            if (main_steps + u < nsteps) {
                fetch_x(bq[(u + 1) & 1]);
#pragma unroll
                for (int m = 0; m < MW; ++m)
#pragma unroll
                    for (int i = 0; i < NW; ++i) mfma1(acc[m][i], aq[u][m], bq[u & 1][i]);
            }
        }
    }
    while (nbar < a.nchunks) { lds_barrier(); ++nbar; }      // (a wave without steps in the last chunks)
    mfma_finish<DT, MW, NW, WM, KG>(acc, a, lds, y, tid, kgrp, wm, wn, kg, n16, mblk0, yoff, b0, p0, db, PQ);
}

template <sc_dtype_t DT, int MW, int NW, int WM, int KG, int MODE>
static sc_status_t launch_mfma_kg(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = [] {
        if constexpr (MODE == 1 || MODE == 3) return &mfma_pipe_kernel<DT, MW, NW, WM, KG, MODE == 3>;
        else if constexpr (MODE == 4 || MODE == 5) return &mfma_conv_dl_kernel<DT, MW, NW, WM, KG, MODE == 5>;
        else return &mfma_conv_kernel<DT, MW, NW, WM, KG, MODE == 2>;
    }();
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256 * KG + (MODE == 1 || MODE == 3 ? 64 * p.mg.PW : 0)), p.mg.lds_bytes, stream, static_cast<const X*>(x),
                       static_cast<Y*>(y), reinterpret_cast<const uint4w*>(p.d_wfrag), a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

template <sc_dtype_t DT, int MW, int NW, int WM, int MODE>
static sc_status_t launch_mfma_one(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    if constexpr (MODE == 4 || MODE == 5) {               // (several output-channel blocks per workgroup: four waves)
        return p.mg.KG == 1 ? launch_mfma_kg<DT, MW, NW, WM, 1, MODE>(p, a, x, y, grid, stream) : SC_ERR_UNSUPPORTED;
    } else {
        return p.mg.KG == 2 ? launch_mfma_kg<DT, MW, NW, WM, 2, MODE>(p, a, x, y, grid, stream)
                            : launch_mfma_kg<DT, MW, NW, WM, 1, MODE>(p, a, x, y, grid, stream);
    }
}

template <sc_dtype_t DT, int MW, int WM, int MODE>
static sc_status_t launch_mfma_nw(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    switch (p.mg.NW) {
        case 1: return launch_mfma_one<DT, MW, 1, WM, MODE>(p, a, x, y, grid, stream);
        case 2: return launch_mfma_one<DT, MW, 2, WM, MODE>(p, a, x, y, grid, stream);
        case 4: return launch_mfma_one<DT, MW, 4, WM, MODE>(p, a, x, y, grid, stream);
        case 8:
            if constexpr (MW <= 2) return launch_mfma_one<DT, MW, 8, WM, MODE>(p, a, x, y, grid, stream);
            break;
    }
    return SC_ERR_UNSUPPORTED;
}

template <sc_dtype_t DT, int MODE>
static sc_status_t launch_mfma_typed(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    const int key = p.mg.WM * 10 + p.mg.MW;
    switch (key) {
        case 11: return launch_mfma_nw<DT, 1, 1, MODE>(p, a, x, y, grid, stream);
        case 12: return launch_mfma_nw<DT, 2, 1, MODE>(p, a, x, y, grid, stream);
        case 14: return launch_mfma_nw<DT, 4, 1, MODE>(p, a, x, y, grid, stream);
        case 21: return launch_mfma_nw<DT, 1, 2, MODE>(p, a, x, y, grid, stream);
        case 22: return launch_mfma_nw<DT, 2, 2, MODE>(p, a, x, y, grid, stream);
        case 24: return launch_mfma_nw<DT, 4, 2, MODE>(p, a, x, y, grid, stream);
        case 41: return launch_mfma_nw<DT, 1, 4, MODE>(p, a, x, y, grid, stream);
        case 42: return launch_mfma_nw<DT, 2, 4, MODE>(p, a, x, y, grid, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

}  // namespace sc
