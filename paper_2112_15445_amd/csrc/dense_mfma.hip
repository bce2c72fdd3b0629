// DENSE variant: the densified tile on the matrix cores (MFMA), for 16- and 8-bit activations.
//
// The gather kernels execute one vector multiply-add instruction per stored weight and output
// position; on gfx950 the matrix cores multiply 16- and 8-bit operands 32 to 64 times faster than
// the vector ALU does, so below a (high) break-even sparsity it is faster to put the zeros back and
// multiply the layer as a dense tile -- the paper's own answer for layers that are not sparse enough
// (its main scheme compares each layer with the dense library and configures the network layer by
// layer), here as a kernel of the library that reads the same NCHW tensors, needs no layout change
// in HBM and gives the same result: the sum over the stored entries of a row of
// theta * input[base + lambda], the entries that are not stored contributing exact zeros.
//
// Formulation: Y[b, d, p, q] = sum_k Wd[d, k] * Xcol[k, (b, p, q)] with k = (r, s, c) -- filter tap
// major, input channel minor -- contracted 32 (f16) or 64 (i8) values at a time by
// v_mfma_f32_16x16x32_f16 / v_mfma_i32_16x16x64_i8: a 16 x 16 block of (output channel, position)
// per instruction, fp32 / int32 accumulation.  One workgroup (4 waves) = NS samples x TP output
// rows x all columns x DB output channels:
//   * the input region of the tile is staged in LDS TRANSPOSED, channel-minor
//     ([sample][row][column][channel], zero padding and channel padding written as zeros), because
//     an MFMA operand holds 8 (16) consecutive k of one position in each lane; a filter tap is then
//     a constant byte offset (r * Ws + s) * pitch added to the lane's position, exactly the
//     "position + pre-stretched offset" addressing of the sparse kernels;
//   * the weights are densified once per plan into MFMA-operand order, so a wave fetches an operand
//     with one coalesced 1 KB load from global memory (L2-resident, shared by all workgroups);
//   * every wave keeps MW x NW blocks of 16 x 16 accumulators in registers; several workgroups per
//     CU overlap the staging of one with the multiplication of another.
// Integer results are exact (bit-identical to the gather kernels); f16 results differ from them in
// summation order only.
#include <mutex>
#include <type_traits>

#include "sc_device.h"
#include "sc_internal.h"

namespace sc {

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef int int4v_ __attribute__((ext_vector_type(4)));
typedef unsigned uint4w __attribute__((ext_vector_type(4)));

template <sc_dtype_t DT> constexpr bool kIntActs = DT == SC_I8 || DT == SC_CB4_I8;
// input channels contracted by one MFMA, and held by one lane (16 bytes)
template <sc_dtype_t DT> constexpr int kChanBlock = kIntActs<DT> ? 64 : 32;
template <sc_dtype_t DT> constexpr int kChanVec = kIntActs<DT> ? 16 : 8;

int mfma_chan_block(sc_dtype_t dt) { return (dt == SC_I8 || dt == SC_CB4_I8) ? 64 : 32; }

// ------------------------------------------------------------------------------------------------
// Densify: scatter the stored entries of the unified table into the dense weight array in MFMA
// operand order.  Element (d, tap, c) lives at
//     ((((d / 16) * RS + tap) * NCB + c / CB) * 64 + (d % 16) + 16 * ((c % CB) / CV)) * 16 bytes
//     + ((c % CB) % CV) * e_w
// so that lane l of a wave reads the 16 bytes at index l of block (d / 16, tap, c / CB): row d % 16
// of the 16 x CB operand, k group l / 16.  Entries j >= len[d] are the fillers that unify the row
// lengths: they carry no value and are skipped (the array is zeroed beforehand).
// ------------------------------------------------------------------------------------------------
template <sc_dtype_t DT>
__global__ void __launch_bounds__(256)
densify_kernel(const void* __restrict__ theta, const int32_t* __restrict__ col, const int32_t* __restrict__ len,
               const void* __restrict__ codebook, unsigned char* __restrict__ out, int D, int n, int RS, int NCB)
{
    constexpr int CB = kChanBlock<DT>, CV = kChanVec<DT>;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)D * n) return;
    const int d = (int)(i / n), j = (int)(i - (int64_t)d * n);
    if (j >= len[d]) return;
    const int k = col[i] & 0x7fffffff;
    const int c = k / RS, tap = k - c * RS;
    const int cblk = c / CB, cin = c - cblk * CB;
    const int kg = cin / CV, jj = cin - kg * CV;
    const int64_t blk = ((int64_t)(d >> 4) * RS + tap) * NCB + cblk;
    unsigned char* dst = out + (blk * 64 + (d & 15) + 16 * kg) * 16;
    if constexpr (kIntActs<DT>) {
        int w;
        if constexpr (DT == SC_I8) w = static_cast<const int8_t*>(theta)[i];
        else w = static_cast<const int8_t*>(codebook)[(static_cast<const uint8_t*>(theta)[i >> 1] >> ((i & 1) * 4)) & 15];
        reinterpret_cast<int8_t*>(dst)[jj] = (int8_t)w;
    } else {
        __half w;
        if constexpr (DT == SC_F16) w = static_cast<const __half*>(theta)[i];
        else w = static_cast<const __half*>(codebook)[(static_cast<const uint8_t*>(theta)[i >> 1] >> ((i & 1) * 4)) & 15];
        reinterpret_cast<__half*>(dst)[jj] = w;
    }
}

size_t mfma_weight_bytes(const Plan& p)
{
    const int CB = mfma_chan_block(p.dtype);
    const int64_t NCB = (p.L.C + CB - 1) / CB;
    // rows padded to a whole 128-channel workgroup block so that every operand load is in bounds
    const int64_t rows16 = (int64_t)((p.L.D + 127) / 128) * 8;
    return (size_t)(rows16 * p.L.R * p.L.S * NCB * 64 * 16);
}

sc_status_t mfma_densify(const Plan& p, unsigned char* out, hipStream_t stream)
{
    const int64_t cnt = (int64_t)p.L.D * p.n;
    if (hipMemsetAsync(out, 0, mfma_weight_bytes(p), stream) != hipSuccess) return SC_ERR_HIP;
    if (cnt == 0) return SC_OK;
    const unsigned blocks = (unsigned)((cnt + 255) / 256);
    const int CB = mfma_chan_block(p.dtype);
    const int NCB = (p.L.C + CB - 1) / CB;
#define SC_DENSIFY(DT)                                                                              \
    hipLaunchKernelGGL(densify_kernel<DT>, dim3(blocks), dim3(256), 0, stream, p.d_theta, p.d_col,  \
                       p.d_len, p.d_codebook, out, p.L.D, p.n, p.L.R * p.L.S, NCB)
    switch (p.dtype) {
        case SC_F16: SC_DENSIFY(SC_F16); break;
        case SC_CB4_F16: SC_DENSIFY(SC_CB4_F16); break;
        case SC_I8: SC_DENSIFY(SC_I8); break;
        case SC_CB4_I8: SC_DENSIFY(SC_CB4_I8); break;
        default: return SC_ERR_UNSUPPORTED;
    }
#undef SC_DENSIFY
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

// ------------------------------------------------------------------------------------------------
// Geometry of one (plan, tuning) pair, derived on the host.
// ------------------------------------------------------------------------------------------------
bool mfma_geometry(const Plan& p, int TP, int NS, int CC, int DB, int lds_budget, MfmaGeom* out)
{
    const sc_layer_t& L = p.L;
    MfmaGeom g{};
    const int CB = mfma_chan_block(p.dtype);
    if (TP < 1 || NS < 1 || NS > 16 || CC < CB || CC % CB) return false;
    if (DB != 16 && DB != 32 && DB != 64 && DB != 128) return false;
    g.TP = std::min(TP, p.P);
    g.NS = g.TP < p.P ? 1 : NS;                   // several samples only with whole planes
    g.tiles_p = (p.P + g.TP - 1) / g.TP;
    g.Hs = (g.TP - 1) * L.stride_h + L.R;
    g.Ws = (p.Q - 1) * L.stride_w + L.S;
    g.npos_s = g.NS * g.Hs * g.Ws;
    g.npos = g.NS * g.TP * p.Q;
    g.NCB = (L.C + CB - 1) / CB;
    g.CC = std::min(CC, g.NCB * CB);
    g.nchunks = (g.NCB * CB + g.CC - 1) / g.CC;
    g.pitch = g.CC * p.ex + 16;                   // bytes per staged position: a multiple of 16, odd in units of 16
    g.DB = DB;
    g.ndb = (L.D + DB - 1) / DB;
    g.WM = DB == 128 ? 2 : 1;
    g.MW = DB / (16 * g.WM);
    const int WN = 4 / g.WM;
    const int NB = (g.npos + 15) / 16;
    const int nw = (NB + WN - 1) / WN;
    g.NW = nw <= 1 ? 1 : (nw <= 2 ? 2 : 4);
    if (nw > 4) return false;
    const int64_t lds = (int64_t)g.npos_s * g.pitch + (int64_t)g.npos_s * 4;      // the tile and its source-offset table
    if (lds > lds_budget || lds > kMaxLdsBytes) return false;
    g.lds_bytes = (int)((lds + 15) / 16 * 16);
    *out = g;
    return true;
}

struct MfmaArgs {
    int C, D, N, H, W, P, Q, S, RS, s_h, s_w, pad_h, pad_w;
    int TP, NS, tiles_p, Hs, Ws, npos_s, npos, CC, nchunks, NCB, pitch, DB, ndb, tile_bytes;
    float inv_ndb, inv_tiles_p, inv_HsWs, inv_Ws, inv_TPQ, inv_Q, inv_S;
};

// floor(e / d) for 0 <= e < 2^19 given inv = 1.0f / d (exact: the half-integer bias keeps the
// product at least 1/(2d) away from every integer, well above the two float roundings)
__device__ inline int fdiv19(int e, float inv) { return (int)(((float)e + 0.5f) * inv); }

template <sc_dtype_t DT, int MW, int NW, int WM>
__global__ void __launch_bounds__(256)
mfma_conv_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                 const uint4w* __restrict__ wfrag, const MfmaArgs a)
{
    using X = typename Types<DT>::X;
    using Acc = typename std::conditional<kIntActs<DT>, int4v_, float4v>::type;
    constexpr int CB = kChanBlock<DT>, CV = kChanVec<DT>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int n16 = lane & 15, kg = lane >> 4;

    // workgroup -> (sample group, row tile, output-channel block); the blocks of one tile are
    // neighbours so that they find the tile in the L2 their siblings loaded.  Workgroups are dealt
    // round-robin to the 8 XCDs: number them so that each XCD gets a contiguous run.
    const int grid = gridDim.x;
    const int wg = (grid & 7) == 0 ? (int)(blockIdx.x & 7) * (grid >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int bt = fdiv19(wg, a.inv_ndb);
    const int db = wg - bt * a.ndb;
    const int bg = fdiv19(bt, a.inv_tiles_p);
    const int tpi = bt - bg * a.tiles_p;
    const int b0 = bg * a.NS, p0 = tpi * a.TP;
    const int row0 = p0 * a.s_h - a.pad_h, col0 = -a.pad_w;
    const int plane = a.H * a.W, PQ = a.P * a.Q;

    // positions of this lane's NW column blocks: byte offset of the staged position in LDS (plus
    // the lane's k group) and element offset of the output inside y, or -1
    int bbase[NW];
    int64_t yoff[NW];
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const int f = ((wn * NW + i) * 16 + n16);
        const int sm = fdiv19(f, a.inv_TPQ);
        const int rem = f - sm * (a.TP * a.Q);
        const int tp = fdiv19(rem, a.inv_Q);
        const int tq = rem - tp * a.Q;
        const bool ok = f < a.npos && b0 + sm < a.N && p0 + tp < a.P;
        bbase[i] = (ok ? ((sm * a.Hs + tp * a.s_h) * a.Ws + tq * a.s_w) * a.pitch : 0) + kg * 16;
        yoff[i] = ok ? ((int64_t)(b0 + sm) * a.D) * PQ + (p0 + tp) * a.Q + tq : -1;
    }

    Acc acc[MW][NW];
#pragma unroll
    for (int m = 0; m < MW; ++m)
#pragma unroll
        for (int i = 0; i < NW; ++i) acc[m][i] = Acc{0, 0, 0, 0};

    const int mblk0 = db * (a.DB >> 4) + wm * MW;            // first 16-row block of this wave
    const int cgroups = a.CC / CV;                           // 16-byte channel groups per staged position

    // Where every staged position lies in the input (element offset inside channel 0 of sample b0),
    // or -1 where it shows padding or a sample past the batch: worked out once, kept in LDS behind
    // the tile, so that copying a chunk costs one table read, CV loads and one 16-byte LDS write
    // per channel group of a position
    int* srctab = reinterpret_cast<int*>(lds + a.tile_bytes);
    for (int pos = tid; pos < a.npos_s; pos += 256) {
        const int sm = fdiv19(pos, a.inv_HsWs);
        const int rem = pos - sm * (a.Hs * a.Ws);
        const int i = fdiv19(rem, a.inv_Ws);
        const int w = rem - i * a.Ws;
        const int row = row0 + i, col = col0 + w;
        const bool in = row >= 0 && row < a.H && col >= 0 && col < a.W && b0 + sm < a.N;
        srctab[pos] = in ? sm * a.C * plane + row * a.W + col : -1;
    }
    const X* xb = x + (int64_t)b0 * a.C * plane;
    const uint4w* wbase[MW];
#pragma unroll
    for (int m = 0; m < MW; ++m) wbase[m] = wfrag + (int64_t)(mblk0 + m) * a.RS * a.NCB * 64 + lane;
    // vectors (position, channel group) are dealt to the threads position-fastest: thread t takes
    // t, t + 256, ...; the step of 256 is q256 whole channel groups plus r256 positions
    const int q256 = 256 / a.npos_s, r256 = 256 - q256 * a.npos_s;
    const int cg_first = fdiv19(tid, 1.0f / (float)a.npos_s), pos_first = tid - cg_first * a.npos_s;

    for (int ch = 0; ch < a.nchunks; ++ch) {
        const int c0 = ch * a.CC;
        __syncthreads();                 // table written / the previous chunk has been multiplied
        // ------------------------------------------------------------ stage the chunk, transposed:
        // one 16-byte LDS write = CV consecutive channels of one staged position; consecutive
        // threads hold consecutive positions, so each of the CV loads of a wave covers contiguous
        // runs of a channel plane
        {
            const int cleft = a.C - c0;                      // channels of the layer from c0 on
            const X* xc = xb + (int64_t)c0 * plane;
            int cg = cg_first, pos = pos_first;
            while (cg < cgroups) {
                // (branch-free: a position that shows padding and a channel past the layer's last
                // load a valid element all the same and drop it, so that the CV loads are issued
                // back to back)
                const int so = srctab[pos];
                const int sofs = so >= 0 ? so : 0;
                X val[CV];
#pragma unroll
                for (int j = 0; j < CV; ++j) {
                    const int c = cg * CV + j;
                    const X v = xc[sofs + (c < cleft ? c : 0) * plane];
                    val[j] = (so >= 0 && c < cleft) ? v : X(0);
                }
                uint4w pk;
                __builtin_memcpy(&pk, val, 16);
                *reinterpret_cast<uint4w*>(lds + pos * a.pitch + cg * 16) = pk;
                cg += q256;
                pos += r256;
                if (pos >= a.npos_s) { pos -= a.npos_s; ++cg; }
            }
        }
        __syncthreads();
        // ------------------------------------------------------------ multiply: one step = one
        // filter tap x one block of CB channels.  The weights come from L2 (latency of several
        // hundred clocks, against 16 clocks per MFMA): the operands of the next PF steps are kept
        // in flight in a ring of registers; the tile operands, which come from LDS, one step ahead.
        const int cbs = min(a.CC, a.NCB * CB - c0) / CB;     // channel blocks in this chunk
        const int gcb0 = c0 / CB;
        const int ksteps = a.RS * cbs;
        const float inv_cbs = 1.0f / (float)cbs;
        auto decode = [&](int ks, int& toff, int& woff) {
            const int tap = fdiv19(ks, inv_cbs);
            const int cb = ks - tap * cbs;
            const int r = fdiv19(tap, a.inv_S), sx = tap - r * a.S;
            toff = (r * a.Ws + sx) * a.pitch + cb * (CB * (int)sizeof(X));
            woff = (tap * a.NCB + gcb0 + cb) * 64;
        };
        auto fetch_w = [&](int ks, uint4w (&av)[MW]) {
            int toff, woff;
            decode(ks, toff, woff);
#pragma unroll
            for (int m = 0; m < MW; ++m) av[m] = wbase[m][woff];
        };
        auto fetch_x = [&](int ks, uint4w (&bv)[NW]) {
            int toff, woff;
            decode(ks, toff, woff);
#pragma unroll
            for (int i = 0; i < NW; ++i) bv[i] = *reinterpret_cast<const uint4w*>(lds + bbase[i] + toff);
        };
        auto multiply = [&](const uint4w (&av)[MW], const uint4w (&bv)[NW]) {
#pragma unroll
            for (int m = 0; m < MW; ++m)
#pragma unroll
                for (int i = 0; i < NW; ++i) {
                    if constexpr (kIntActs<DT>)
                        acc[m][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(int4v_, av[m]),
                                                                          __builtin_bit_cast(int4v_, bv[i]), acc[m][i], 0, 0, 0);
                    else
                        acc[m][i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, av[m]),
                                                                           __builtin_bit_cast(half8v, bv[i]), acc[m][i], 0, 0, 0);
                }
        };
        constexpr int PF = MW >= 4 ? 4 : 6;                  // steps of weights in flight (even)
        uint4w aq[PF][MW], bq[2][NW];
        const int last = ksteps - 1;
#pragma unroll
        for (int u = 0; u < PF; ++u) fetch_w(min(u, last), aq[u]);
        fetch_x(0, bq[0]);
        __builtin_amdgcn_sched_barrier(0);
        const int main_steps = ksteps / PF * PF;
        for (int ks = 0; ks < main_steps; ks += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                // Step ks + u: request the tile operands of the next step, multiply, then refill
                // this step's slot of the weight ring with the weights of step ks + u + PF -- after
                // the MFMAs that read the slot, so that the slot keeps its registers from one
                // round of the ring to the next.  Indices past the end are clamped (a few redundant
                // loads instead of branches: the body stays straight-line code with static wait
                // counts); the scheduling barriers keep the compiler from sinking the loads of
                // later steps down to their first use, which would put the L2 latency back on the
                // critical path.
                fetch_x(min(ks + u + 1, last), bq[(u + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                multiply(aq[u], bq[u & 1]);
                __builtin_amdgcn_sched_barrier(0);
                fetch_w(min(ks + u + PF, last), aq[u]);
            }
        }
        uint4w (&bcur)[NW] = bq[0];
        for (int ks = main_steps; ks < ksteps; ++ks) {       // at most PF - 1 steps
            uint4w acur[MW];
            fetch_w(ks, acur);
            fetch_x(ks, bcur);
            multiply(acur, bcur);
        }
    }
    // ---------------------------------------------------------------- store: a lane holds, for its
    // position (column n16 of the block), the four output channels 4 * kg .. 4 * kg + 3 of each row block
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
}

int mfma_grid_size(const Plan& p, const MfmaGeom& g, int N)
{
    (void)p;
    return ((N + g.NS - 1) / g.NS) * g.tiles_p * g.ndb;
}

template <sc_dtype_t DT, int MW, int NW, int WM>
static sc_status_t launch_mfma_one(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = mfma_conv_kernel<DT, MW, NW, WM>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), p.mg.lds_bytes, stream, static_cast<const X*>(x),
                       static_cast<Y*>(y), reinterpret_cast<const uint4w*>(p.d_wfrag), a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

template <sc_dtype_t DT, int MW, int WM>
static sc_status_t launch_mfma_nw(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    switch (p.mg.NW) {
        case 1: return launch_mfma_one<DT, MW, 1, WM>(p, a, x, y, grid, stream);
        case 2: return launch_mfma_one<DT, MW, 2, WM>(p, a, x, y, grid, stream);
        case 4: return launch_mfma_one<DT, MW, 4, WM>(p, a, x, y, grid, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

template <sc_dtype_t DT>
static sc_status_t launch_mfma_dt(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    if (p.mg.WM == 2) return launch_mfma_nw<DT, 4, 2>(p, a, x, y, grid, stream);
    switch (p.mg.MW) {
        case 1: return launch_mfma_nw<DT, 1, 1>(p, a, x, y, grid, stream);
        case 2: return launch_mfma_nw<DT, 2, 1>(p, a, x, y, grid, stream);
        case 4: return launch_mfma_nw<DT, 4, 1>(p, a, x, y, grid, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

sc_status_t launch_mfma(const Plan& p, const void* x, void* y, int N, hipStream_t stream)
{
    const MfmaGeom& g = p.mg;
    if (!p.d_wfrag) return SC_ERR_UNSUPPORTED;
    const int64_t grid = (int64_t)((N + g.NS - 1) / g.NS) * g.tiles_p * g.ndb;
    if (grid >= (1 << 19)) return SC_ERR_UNSUPPORTED;                       // fdiv19() range
    if ((int64_t)g.NS * p.L.C * p.L.H * p.L.W >= (1ll << 31)) return SC_ERR_UNSUPPORTED;
    MfmaArgs a{};
    a.C = p.L.C; a.D = p.L.D; a.N = N; a.H = p.L.H; a.W = p.L.W; a.P = p.P; a.Q = p.Q;
    a.S = p.L.S; a.RS = p.L.R * p.L.S; a.s_h = p.L.stride_h; a.s_w = p.L.stride_w; a.pad_h = p.L.pad_h; a.pad_w = p.L.pad_w;
    a.TP = g.TP; a.NS = g.NS; a.tiles_p = g.tiles_p; a.Hs = g.Hs; a.Ws = g.Ws; a.npos_s = g.npos_s; a.npos = g.npos;
    a.CC = g.CC; a.nchunks = g.nchunks; a.NCB = g.NCB; a.pitch = g.pitch; a.DB = g.DB; a.ndb = g.ndb;
    a.tile_bytes = g.npos_s * g.pitch;
    a.inv_ndb = 1.0f / (float)g.ndb; a.inv_tiles_p = 1.0f / (float)g.tiles_p; a.inv_S = 1.0f / (float)p.L.S;
    a.inv_HsWs = 1.0f / (float)(g.Hs * g.Ws); a.inv_Ws = 1.0f / (float)g.Ws;
    a.inv_TPQ = 1.0f / (float)(g.TP * p.Q); a.inv_Q = 1.0f / (float)p.Q;
    if (g.npos_s >= (1 << 19)) return SC_ERR_UNSUPPORTED;
    switch (p.dtype) {
        case SC_F16: return launch_mfma_dt<SC_F16>(p, a, x, y, (int)grid, stream);
        // (the codebook variants were decoded when the weights were densified: same arithmetic)
        case SC_CB4_F16: return launch_mfma_dt<SC_F16>(p, a, x, y, (int)grid, stream);
        case SC_I8: return launch_mfma_dt<SC_I8>(p, a, x, y, (int)grid, stream);
        case SC_CB4_I8: return launch_mfma_dt<SC_I8>(p, a, x, y, (int)grid, stream);
        default: return SC_ERR_UNSUPPORTED;
    }
}

}  // namespace sc
