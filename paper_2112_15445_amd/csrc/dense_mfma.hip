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
//     CU overlap the staging of one with the multiplication of another;
//   * two kernels share this tile and the epilogue: the one-shot form (a chunk of input channels
//     is staged by all waves, then multiplied; four waves, or eight that split the steps) and the
//     pipelined form (waves of their own stage the chunks into two LDS buffers, one chunk ahead of
//     the multiplying waves).
// Integer results are exact (bit-identical to the gather kernels); f16 results differ from them in
// summation order only.
#include "dense_mfma_kernel.h"

namespace sc {

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
bool mfma_geometry(const Plan& p, int TP, int NS, int CC, int DB, int WM, int lds_budget, MfmaGeom* out, int KG, int PW, int nat, int DL)
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
    g.nat = nat;
    g.DB = DB;
    g.ndb = (L.D + DB - 1) / DB;
    // the four waves: WM along the output channels (MW 16-row blocks each), 4 / WM along the
    // positions (NW 16-column blocks each, at most 8)
    if (WM != 1 && WM != 2 && WM != 4) return false;
    g.WM = WM;
    if (DB % (16 * WM)) return false;
    g.MW = DB / (16 * WM);
    if (g.MW != 1 && g.MW != 2 && g.MW != 4) return false;
    const int WN = 4 / WM;
    const int NB = (g.npos + 15) / 16;
    const int nw = (NB + WN - 1) / WN;
    if (nw > 8) return false;
    g.NW = nw <= 1 ? 1 : (nw <= 2 ? 2 : (nw <= 4 ? 4 : 8));
    if (g.NW == 8 && g.MW == 4) return false;     // 32 accumulator blocks per wave: not instantiated
    if (KG != 1 && KG != 2) return false;
    g.KG = KG;
    if (PW < 0 || PW > 4) return false;
    g.PW = PW;
    if (nat) {
        // natural layout: pointwise layers only, the one-shot form; a row of LDS per channel, as many
        // columns as the waves' blocks cover, pitch a multiple of 64 bytes plus 32
        if (nat != 1 || L.R != 1 || L.S != 1 || L.stride_h != 1 || L.stride_w != 1 || L.pad_h || L.pad_w) return false;
        g.pitch = (WN * g.NW * 16 * p.ex + 63) / 64 * 64 + 32;
        if (PW) {
            // pipelined: the buffers are what the direct-to-LDS loads write -- rows back to back, one
            // sample per workgroup, runs and planes whole 16-byte words
            if (g.NS != 1 || (g.TP * p.Q * p.ex) % 16 || (L.H * L.W * p.ex) % 16) return false;
            g.pitch = g.TP * p.Q * p.ex;
        }
    }
    // the pipelined form keeps two chunk buffers (one if the layer is a single chunk)
    g.bufsz = nat ? g.CC * g.pitch : (int)(((int64_t)g.npos_s * g.pitch + 15) / 16 * 16);
    // (unpadded rows: the blocks of the waves may reach past the end of the last row)
    if (nat && PW) g.bufsz += (std::max(0, WN * g.NW * 16 * p.ex - g.pitch) + 15) / 16 * 16;
    int64_t lds = (int64_t)g.bufsz * (PW > 0 && g.nchunks > 1 ? 2 : 1);
    // pooling windows must not straddle tiles
    if (has_epilogue(p) && p.epi.pool && g.TP < p.P && (g.TP & 1)) return false;
    if ((has_epilogue(p) && p.epi.pool) || KG == 2) {
        // the accumulators are exchanged through LDS (between the two step groups, or for pooling)
        g.epi_pitch = (4 / g.WM) * g.NW * 16 + 1;
        lds = std::max<int64_t>(lds, (int64_t)g.DB * g.epi_pitch * 4);
    }
    // several output-channel blocks per workgroup: the tile stays in LDS, so one chunk, no exchange through LDS
    if (DL < 1 || DL > 16) return false;
    g.DL = std::min(DL, g.ndb);
    if (g.DL > 1 && (g.nchunks != 1 || KG != 1 || PW || (has_epilogue(p) && p.epi.pool))) return false;
    if (lds > lds_budget || lds > kMaxLdsBytes) return false;
    g.lds_bytes = (int)((lds + 15) / 16 * 16);
    *out = g;
    return true;
}

int mfma_grid_size(const Plan& p, const MfmaGeom& g, int N)
{
    (void)p;
    return ((N + g.NS - 1) / g.NS) * g.tiles_p * ((g.ndb + g.DL - 1) / g.DL);
}

sc_status_t launch_mfma(const Plan& p, const void* x, void* y, int N, hipStream_t stream)
{
    const MfmaGeom& g = p.mg;
    if (!p.d_wfrag) return SC_ERR_UNSUPPORTED;
    const int ndbg = (g.ndb + g.DL - 1) / g.DL;
    const int64_t grid = (int64_t)((N + g.NS - 1) / g.NS) * g.tiles_p * ndbg;
    if (grid >= (1 << 19)) return SC_ERR_UNSUPPORTED;                       // fdiv19() range
    if ((int64_t)g.NS * p.L.C * p.L.H * p.L.W >= (1ll << 31)) return SC_ERR_UNSUPPORTED;
    MfmaArgs a{};
    a.C = p.L.C; a.D = p.L.D; a.N = N; a.H = p.L.H; a.W = p.L.W; a.P = p.P; a.Q = p.Q;
    a.S = p.L.S; a.RS = p.L.R * p.L.S; a.s_h = p.L.stride_h; a.s_w = p.L.stride_w; a.pad_h = p.L.pad_h; a.pad_w = p.L.pad_w;
    a.TP = g.TP; a.NS = g.NS; a.tiles_p = g.tiles_p; a.Hs = g.Hs; a.Ws = g.Ws; a.npos_s = g.npos_s; a.npos = g.npos;
    a.bufsz = g.bufsz;
    a.DL = g.DL; a.ndbg = ndbg; a.inv_ndbg = 1.0f / (float)ndbg;
    {
        const int ccb = g.CC / mfma_chan_block(p.dtype);
        a.cbs_last = g.NCB - (g.nchunks - 1) * ccb;
        a.inv_spc = 1.0f / (float)(p.L.R * p.L.S * ccb); a.inv_ccb = 1.0f / (float)ccb;
        a.inv_cbs_last = 1.0f / (float)a.cbs_last; a.inv_S = 1.0f / (float)p.L.S;
        if (g.PW && (mfma_weight_bytes(p) >= (1ull << 31) || (int64_t)p.L.R * p.L.S * g.NCB >= (1 << 18))) return SC_ERR_UNSUPPORTED;
    }
    a.CC = g.CC; a.nchunks = g.nchunks; a.NCB = g.NCB; a.pitch = g.pitch; a.DB = g.DB; a.ndb = g.ndb;
    a.epi = has_epilogue(p) ? 1 : 0; a.epi_relu = p.epi.relu; a.epi_pool = p.epi.pool; a.epi_pitch = g.epi_pitch;
    a.Po = p.Po; a.Qo = p.Qo; a.requant = p.epi.requant ? p.d_requant : nullptr;
    if ((int64_t)g.DB * g.NS * g.TP * p.Q >= (1 << 19)) return SC_ERR_UNSUPPORTED;
    // elements per staging load: the widest power of two (up to 16 bytes) that divides the row length
    // and the caller's pointer
    a.epv = 1;
    a.TPQ = g.TP * p.Q;
    for (int e = 16 / p.ex; e > 1; e >>= 1) {
        // (natural layout: a run of the tile starts at a multiple of TP * Q inside its plane and is whole loads long)
        const bool fits = g.nat ? (p.L.H * p.L.W) % e == 0 && (g.TP * p.Q) % e == 0 : p.L.W % e == 0;
        if (fits && reinterpret_cast<uintptr_t>(x) % (uintptr_t)(e * p.ex) == 0) { a.epv = e; break; }
    }
    if (g.nat && (int64_t)g.CC * g.NS * g.TP * p.Q >= (1 << 19)) return SC_ERR_UNSUPPORTED;     // fdiv19() range of the copy
    // (the direct-to-LDS copies of the pipelined natural-layout form move 16-byte words)
    if (g.nat && g.PW && reinterpret_cast<uintptr_t>(x) % 16 != 0) return SC_ERR_UNSUPPORTED;
    a.inv_ndb = 1.0f / (float)g.ndb; a.inv_tiles_p = 1.0f / (float)g.tiles_p;
    a.inv_HsWs = 1.0f / (float)(g.Hs * g.Ws); a.inv_Ws = 1.0f / (float)g.Ws;
    a.inv_TPQ = 1.0f / (float)(g.TP * p.Q); a.inv_Q = 1.0f / (float)p.Q;
    if (g.npos_s >= (1 << 19)) return SC_ERR_UNSUPPORTED;
    switch (p.dtype) {
        // (the codebook variants were decoded when the weights were densified: same arithmetic)
        case SC_F16:
        case SC_CB4_F16:
            if (g.DL > 1) return launch_mfma_dl_f16(p, a, x, y, (int)grid, stream);
            return g.nat ? (g.PW ? launch_mfma_pipe_nat_f16(p, a, x, y, (int)grid, stream) : launch_mfma_nat_f16(p, a, x, y, (int)grid, stream))
                         : (g.PW ? launch_mfma_pipe_f16(p, a, x, y, (int)grid, stream) : launch_mfma_f16(p, a, x, y, (int)grid, stream));
        case SC_I8:
        case SC_CB4_I8:
            if (g.DL > 1) return launch_mfma_dl_i8(p, a, x, y, (int)grid, stream);
            return g.nat ? (g.PW ? launch_mfma_pipe_nat_i8(p, a, x, y, (int)grid, stream) : launch_mfma_nat_i8(p, a, x, y, (int)grid, stream))
                         : (g.PW ? launch_mfma_pipe_i8(p, a, x, y, (int)grid, stream) : launch_mfma_i8(p, a, x, y, (int)grid, stream));
        default: return SC_ERR_UNSUPPORTED;
    }
}

}  // namespace sc
