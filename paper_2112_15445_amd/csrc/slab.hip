// SLAB variant: the gfx950-first shape of the paper's Algorithm 3.
//
// One workgroup owns one sample and one tile of output pixels and computes ALL output channels for
// it.  It first stages the input region the tile needs -- every input channel, halo and zero
// padding included -- in LDS (up to 160 KB per CU), so the input is read from HBM once instead of
// once per output channel, and no padded copy of the input ever exists in HBM.  Then the rows of
// the (theta, lambda) table are streamed over the resident tile: the waves of the workgroup split
// the output channels, each lane owns VPT tile positions (lane, lane+64, ...), and for every
// stored entry the lane gathers   slab[position + lambda]   from LDS -- consecutive lanes read
// consecutive LDS words, so the gather is bank-conflict free for any lambda -- and accumulates in
// registers; one store per output value.  lambda here is the offset pre-stretched for the tile's
// LDS layout (see SlabGeom), already scaled to bytes.
//
// Kernels in this file (all follow the paper's "Convolution operation using a sparse operation on
// GPGPU": output = sum over the stored (theta, lambda) entries of a row of theta * input[base +
// lambda], with the unified number of entries per row):
//   slab_kernel        one tile, every input channel resident, one shot
//   slab_cc_kernel     one tile, input channels staged chunk by chunk, accumulators kept in
//                      registers across the chunks; output-channel blocks; several samples per tile
//   slab_async_kernel  pointwise layers: persistent workgroups, two tile buffers, producer waves
//                      copy tile i+1 with direct-to-LDS loads while consumer waves multiply tile i
//   slab_chunk_kernel  the same with channel chunks
//   slab_sym_kernel / slab_symc_kernel   the same without dedicated producer waves
//
// 16- and 8-bit activations can be multiplied as packed positions (tuning.pack; always in
// slab_async_kernel with scalar-load weights): a lane owns the 2 or 4 adjacent positions of one
// aligned 32-bit LDS word, so one LDS read feeds 2 or 4 multiply-adds.  Where filter taps would
// put the word off a word boundary (any layer that is not pointwise) slab_cc_kernel keeps 2 or 4
// images of the chunk in LDS, image s shifted by s elements, and the segment table points every
// entry at the image in which its word is aligned.
//
// (theta, lambda) reaches the lanes in one of four ways (tuning.wsrc):
//   0  rows are staged in LDS in groups (decoding 4-bit codebook indices on the way) and read back
//      with wave-uniform (broadcast) LDS reads, as Algorithm 3 does from shared memory;
//   1  rows are read with scalar loads from a pre-expanded {theta32, lambda} table in global
//      memory, which keeps the LDS pipe free for the gather itself;
//   2  the same table is read with wave-uniform 16-byte vector loads (all lanes the same address),
//      which are counted by vmcnt and can therefore be kept several groups ahead of their use
//      without ever waiting on the LDS counter;
//   3  lane j of the wave loads entry j of the row (one coalesced vector load per 64 entries, one
//      chunk ahead) and every entry is broadcast to the wave with two v_readlane: two more VALU
//      instructions per entry, but no scalar-cache or LDS latency in the inner loop.
#include <mutex>

#include "sc_device.h"
#include "sc_dma.h"
#include "sc_internal.h"

namespace sc {

struct SlabArgs {
    int C, D, n, N;
    int Hf, Wf, Pf, Qf;
    int s_h, s_w, pad_h, pad_w;
    int TP, TQ, tiles_p, tiles_q;
    int nsw, Qs, sub_pitch, chan_pitch, F;
    int slab_elems, slab_bytes, wcap, DS, JC, vec, np, nprod, dmab;
    int CC, nchunks, DTW, ndt;           // channel-chunked one-shot form
    int copies, copy_bytes;              // packed positions: shifted images of a chunk
    int SR;                              // rows of one channel image
    int FS;                              // samples laid end to end in one tile (1: off)
    int fs_vec;                          // ... and every sample's chunk is a 16-byte aligned block of whole 16-byte words
    int SG;                              // interleaved samples: sample groups per workgroup, laid along the lanes (1: off)
    int ksplit, cps;                     // chunks of a tile dealt to ksplit workgroups, cps chunks each (1: off)
    float inv_ksplit;
    float inv_chan_pitch, inv_sub_pitch, inv_Qs, inv_tiles, inv_tiles_q, inv_ndt;
    int64_t x_sample_stride, y_plane;
};


template <sc_dtype_t DT> __device__ inline int weight_bits(typename Types<DT>::WL w)
{
    if constexpr (DT == SC_F32 || kHalfActs<DT>) return __float_as_int(w);
    else return w;
}
template <sc_dtype_t DT> __device__ inline typename Types<DT>::WL weight_from_bits(int b)
{
    if constexpr (DT == SC_F32 || kHalfActs<DT>) return __int_as_float(b);
    else return b;
}

// Expand the compact weight table to {theta widened to 32 bits, LDS byte offset} pairs for the
// scalar-load path.  Rows are packed with an even pitch np = round_up(n, 2) (a zero weight at
// offset 0 fills an odd row), so the table of a small layer stays inside the 16 KB scalar cache.
template <sc_dtype_t DT>
__global__ void __launch_bounds__(256)
expand_weights_kernel(const void* __restrict__ theta, const int32_t* __restrict__ lam,
                      int2* __restrict__ out, int D, int n, int np)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)D * np) return;
    const int d = (int)(i / np), j = (int)(i - (int64_t)d * np);
    int2 e = make_int2(0, 0);
    if (j < n) {
        const int64_t g = (int64_t)d * n + j;
        const int l = lam[g];
        e = make_int2(weight_bits<DT>(load_weight<DT>(theta, g, l, nullptr)), l & 0x7fffffff);
    }
    out[i] = e;
}

typedef int int16v __attribute__((ext_vector_type(16)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

// One group = 8 {theta32, lambda} pairs = 64 bytes of the expanded weight table.
//   WSRC 1: one 16-dword scalar load (values arrive in SGPRs; latency of the scalar cache / L2)
//   WSRC 2: four 16-byte buffer loads at a wave-uniform address (values arrive in VGPRs, the same in
//           every lane; served by the vector L1, counted by vmcnt, so the compiler can keep several
//           groups in flight independently of the LDS traffic)
template <int WSRC>
__device__ inline void load_group(int (&o)[16], const int2* __restrict__ wl32,
                                  __amdgpu_buffer_rsrc_t rsrc, int64_t entry)
{
    if constexpr (WSRC == 3) {
        (void)o; (void)wl32; (void)rsrc; (void)entry;
    } else if constexpr (WSRC == 1) {
        const int16v t = *reinterpret_cast<const int16v*>(wl32 + entry);
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i] = t[i];
    } else {
        const int base = (int)(entry * 8);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4v t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, 0, base + q * 16, 0);
            o[4 * q + 0] = (int)t.x; o[4 * q + 1] = (int)t.y; o[4 * q + 2] = (int)t.z; o[4 * q + 3] = (int)t.w;
        }
    }
}

// Two {theta32, lambda} pairs (16 bytes).
template <int WSRC>
__device__ inline void load_pair(int* o, const int2* __restrict__ wl32, __amdgpu_buffer_rsrc_t rsrc,
                                 int64_t entry)
{
    typedef int int4v __attribute__((ext_vector_type(4)));
    if constexpr (WSRC == 1) {
        const int4v t = *reinterpret_cast<const int4v*>(wl32 + entry);
        o[0] = t.x; o[1] = t.y; o[2] = t.z; o[3] = t.w;
    } else if constexpr (WSRC == 2) {
        const uint4v t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, 0, (int)(entry * 8), 0);
        o[0] = (int)t.x; o[1] = (int)t.y; o[2] = (int)t.z; o[3] = (int)t.w;
    } else {
        (void)o; (void)wl32; (void)rsrc; (void)entry;
    }
}

// One (theta, lambda) entry applied to one slot of a lane.  E = 1: the slot is one position.
// E > 1: the slot is an aligned 32-bit word (2 halves or 4 bytes) or an aligned 128-bit word
// (4 floats or 8 halves) of E adjacent positions, so one LDS read feeds E multiply-adds; the
// 128-bit reads also move 1.6 times the bytes per clock of the 32-bit ones on this chip.
template <sc_dtype_t DT, int E>
__device__ __forceinline__ void mac_slot(typename Types<DT>::A (&acc)[E], typename Types<DT>::WL w,
                                         const unsigned char* p)
{
    using X = typename Types<DT>::X;
    constexpr int SB = E * (int)sizeof(X);      // bytes per slot
    static_assert(E == 1 || SB == 4 || (SB == 16 && sizeof(X) >= 2), "slot: one element, 32 or 128 bits");
    if constexpr (E == 1) {
        mac1<DT>(acc[0], w, *reinterpret_cast<const X*>(p));
    } else if constexpr (SB == 4) {
        const uint32_t xd = *reinterpret_cast<const uint32_t*>(p);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if constexpr (DT == SC_F16)
                acc[e] += w * __half2float(__ushort_as_half((unsigned short)(xd >> (16 * e))));
            else   // one 4-way int8 dot product with the weight in byte e and zeros elsewhere: no unpacking
                acc[e] = __builtin_amdgcn_sdot4((int)xd, (w & 0xff) << (8 * e), acc[e], false);
        }
    } else {
        const uint4v xq = *reinterpret_cast<const uint4v*>(p);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (DT == SC_F32) {
                acc[q] += w * __uint_as_float(xq[q]);
            } else {
                acc[2 * q] += w * __half2float(__ushort_as_half((unsigned short)(xq[q] & 0xffffu)));
                acc[2 * q + 1] += w * __half2float(__ushort_as_half((unsigned short)(xq[q] >> 16)));
            }
        }
    }
}

// The E results of a slot leave as one store: 2 halves as one 32-bit word; 4 int32, 4 floats or
// 8 halves as 16 bytes.
template <sc_dtype_t DT, int E>
__device__ __forceinline__ void store_slot(typename Types<DT>::Y* yp, const typename Types<DT>::A (&acc)[E])
{
    typedef int int4v __attribute__((ext_vector_type(4)));
    if constexpr (E == 1) {
        store_out(yp, narrow<DT>(acc[0]));
    } else if constexpr (DT == SC_F16 && E == 2) {
        const uint32_t lo = __half_as_ushort(__float2half(acc[0]));
        const uint32_t hi = __half_as_ushort(__float2half(acc[1]));
        store_out(reinterpret_cast<uint32_t*>(yp), lo | (hi << 16));
    } else if constexpr (DT == SC_F16 && E == 8) {
        int4v v;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            v[q] = (int)((uint32_t)__half_as_ushort(__float2half(acc[2 * q])) |
                         ((uint32_t)__half_as_ushort(__float2half(acc[2 * q + 1])) << 16));
        __builtin_nontemporal_store(v, reinterpret_cast<int4v*>(yp));
    } else if constexpr (DT == SC_F32) {
        int4v v = {__float_as_int(acc[0]), __float_as_int(acc[1]), __float_as_int(acc[2]), __float_as_int(acc[3])};
        __builtin_nontemporal_store(v, reinterpret_cast<int4v*>(yp));
    } else {
        store_out4(yp, acc[0], acc[1], acc[2], acc[3]);
    }
}

// Rows d = first, first + stride, ... of the layer over the tile resident at lane_base: for every
// stored entry gather slab[position + lambda] for the lane's VPT positions and accumulate; one
// store per output.  Groups are fetched one ahead of the group being multiplied.
template <sc_dtype_t DT, int VPT, int WSRC>
__device__ inline void stream_rows(const int2* __restrict__ wl32, __amdgpu_buffer_rsrc_t rsrc,
                                   const unsigned char* lane_base, typename Types<DT>::Y* yb,
                                   const int (&out_off)[VPT], int first, int stride, int D, int n, int np,
                                   int64_t y_plane)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    if constexpr (WSRC == 3) {
        // Lane-distributed rows: lane j of the wave loads entry j of the row chunk (one coalesced
        // 512-byte vector load per 64 entries, fetched one chunk ahead), and each entry is then
        // broadcast with two v_readlane.  No scalar-cache latency, no LDS traffic for the weights.
        const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        A acc3[VPT];
        int2 cur2 = make_int2(0, 0), nxt2;
        if (first < D && lane < n) cur2 = wl32[(int64_t)first * np + lane];
        for (int d = first; d < D; d += stride) {
#pragma unroll
            for (int k = 0; k < VPT; ++k) acc3[k] = A(0);
            for (int c0 = 0; c0 < n; c0 += 64) {
                const int cnt = min(64, n - c0);
                // next chunk: same row, or the first chunk of this wave's next row
                const bool more = c0 + 64 < n;
                const int dn = more ? d : d + stride;
                const int cn = more ? c0 + 64 : 0;
                nxt2 = make_int2(0, 0);
                if (dn < D && cn + lane < n) nxt2 = wl32[(int64_t)dn * np + cn + lane];
                auto mac = [&](int j) {
                    const WL w = weight_from_bits<DT>(__builtin_amdgcn_readlane(cur2.x, j));
                    const unsigned char* pj = lane_base + __builtin_amdgcn_readlane(cur2.y, j);
#pragma unroll
                    for (int k = 0; k < VPT; ++k)
                        mac1<DT>(acc3[k], w, *reinterpret_cast<const X*>(pj + k * 64 * (int)sizeof(X)));
                };
                int j = 0;
                for (; j + 8 <= cnt; j += 8) {
                    mac(j); mac(j + 1); mac(j + 2); mac(j + 3);
                    mac(j + 4); mac(j + 5); mac(j + 6); mac(j + 7);
                }
                for (; j < cnt; ++j) mac(j);
                cur2 = nxt2;
            }
            Y* yd = yb + (int64_t)d * y_plane;
#pragma unroll
            for (int k = 0; k < VPT; ++k)
                if (out_off[k] >= 0) store_out(yd + out_off[k], narrow<DT>(acc3[k]));
        }
        return;
    }
    // Rows are packed with an even pitch np: ng full groups of 8 pairs, then up to 3 pairs of 2.
    const int ng = np >> 3;
    const int tail = (np & 7) >> 1;
    A acc[VPT];
    auto mac = [&](int wbits, int lam) {
        const WL w = weight_from_bits<DT>(wbits);
        const unsigned char* pj = lane_base + lam;
#pragma unroll
        for (int k = 0; k < VPT; ++k)
            mac1<DT>(acc[k], w, *reinterpret_cast<const X*>(pj + k * 64 * (int)sizeof(X)));
    };
    if constexpr (WSRC == 1) {
        // Scalar loads, 8 entries at a time, through the constant address space and with no
        // software prefetch: with nothing else pending on the scalar/LDS counter the eight gathers
        // of a group can be waited for one by one, so the multiply-adds start when the first value
        // arrives, and the other waves of the workgroup hide the scalar load.  The tail load
        // reaches up to six entries past the row (the next row, or the slack behind the table).
        typedef const int16v __attribute__((address_space(4)))* c16_t;
        for (int d = first; d < D; d += stride) {
            const int2* prow = wl32 + (int64_t)d * np;
#pragma unroll
            for (int k = 0; k < VPT; ++k) acc[k] = A(0);
            for (int g = 0; g < ng; ++g) {
                const int16v c = *(c16_t)(prow + 8 * g);
#pragma unroll
                for (int i = 0; i < 8; ++i) mac(c[2 * i], c[2 * i + 1]);
            }
            if (tail > 0) {
                const int16v c = *(c16_t)(prow + 8 * ng);
                mac(c[0], c[1]); mac(c[2], c[3]);
                if (tail > 1) { mac(c[4], c[5]); mac(c[6], c[7]); }
                if (tail > 2) { mac(c[8], c[9]); mac(c[10], c[11]); }
            }
            Y* yd = yb + (int64_t)d * y_plane;
#pragma unroll
            for (int k = 0; k < VPT; ++k)
                if (out_off[k] >= 0) store_out(yd + out_off[k], narrow<DT>(acc[k]));
        }
        return;
    }
    // Wave-uniform vector loads: full groups ping-pong between two register sets (A, B) and are
    // fetched one ahead of their use, across row boundaries; the tail pairs of a row are fetched
    // when the row starts.
    int ga[16], gb[16], tl[12];
    auto mac8 = [&](const int (&c)[16]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) mac(c[2 * i], c[2 * i + 1]);
    };
    if (ng > 0 && first < D) load_group<WSRC>(ga, wl32, rsrc, (int64_t)first * np);
    for (int d = first; d < D; d += stride) {
        const int64_t rowb = (int64_t)d * np;
        const bool has_next_row = d + stride < D;
        const int64_t nextb = (int64_t)(d + stride) * np;
#pragma unroll
        for (int t = 0; t < 3; ++t)
            if (t < tail) load_pair<WSRC>(&tl[4 * t], wl32, rsrc, rowb + ng * 8 + 2 * t);
#pragma unroll
        for (int k = 0; k < VPT; ++k) acc[k] = A(0);
        int g = 0;
        while (g < ng) {
            // A holds group g of this row
            if (g + 1 < ng) load_group<WSRC>(gb, wl32, rsrc, rowb + (g + 1) * 8);
            else if (has_next_row) load_group<WSRC>(gb, wl32, rsrc, nextb);
            mac8(ga);
            ++g;
            if (g < ng) {
                // B holds group g of this row
                if (g + 1 < ng) load_group<WSRC>(ga, wl32, rsrc, rowb + (g + 1) * 8);
                else if (has_next_row) load_group<WSRC>(ga, wl32, rsrc, nextb);
                mac8(gb);
                ++g;
            } else {
                // odd group count: the next row's first group sits in B; hand it to A
#pragma unroll
                for (int i = 0; i < 16; ++i) ga[i] = gb[i];
            }
        }
#pragma unroll
        for (int t = 0; t < 3; ++t)
            if (t < tail) {
                mac(tl[4 * t + 0], tl[4 * t + 1]);
                mac(tl[4 * t + 2], tl[4 * t + 3]);
            }
        Y* yd = yb + (int64_t)d * y_plane;
#pragma unroll
        for (int k = 0; k < VPT; ++k)
            if (out_off[k] >= 0) store_out(yd + out_off[k], narrow<DT>(acc[k]));
    }
}

// Scalar-load row stream of pointwise layers with packed positions: lane l owns the E adjacent
// positions (k*64 + l)*E .. +E-1 of slot k -- one 32-bit word (E = 2 halves / 4 bytes) or one
// 128-bit word (E = 4 floats / 8 halves) -- so one LDS read feeds E multiply-adds and the outputs of
// a lane leave as one 4- or 16-byte store.  Needs channel rows that are whole words (tile width
// and plane size multiples of E), which the direct-to-LDS forms guarantee.  out_off[k] is the
// element offset of the lane's first position of slot k inside the output plane, or -1.  Same loop
// shape as the unpacked stream: 8 entries per scalar load, no software prefetch, tail pairs from
// one over-reaching load.
template <sc_dtype_t DT, int VW, int E>
__device__ inline void stream_rows_packed(const int2* __restrict__ wl32, const unsigned char* lane_base,
                                          typename Types<DT>::Y* yb, const int (&out_off)[VW], int first,
                                          int stride, int D, int np, int64_t y_plane)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    constexpr int SB = E * (int)sizeof(X);       // bytes per slot
    static_assert(SB == 4 || SB == 16, "packed positions: 32- or 128-bit words");
    typedef const int16v __attribute__((address_space(4)))* c16_t;
    const int ng = np >> 3;
    const int tail = (np & 7) >> 1;
    A acc[VW][E];
    auto mac = [&](int wbits, int lam) {
        const WL w = weight_from_bits<DT>(wbits);
        const unsigned char* pj = lane_base + lam;
#pragma unroll
        for (int k = 0; k < VW; ++k) mac_slot<DT, E>(acc[k], w, pj + k * 64 * SB);
    };
    for (int d = first; d < D; d += stride) {
        const int2* prow = wl32 + (int64_t)d * np;
#pragma unroll
        for (int k = 0; k < VW; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) acc[k][e] = A(0);
        for (int g = 0; g < ng; ++g) {
            const int16v c = *(c16_t)(prow + 8 * g);
#pragma unroll
            for (int i = 0; i < 8; ++i) mac(c[2 * i], c[2 * i + 1]);
        }
        if (tail > 0) {
            const int16v c = *(c16_t)(prow + 8 * ng);
            mac(c[0], c[1]); mac(c[2], c[3]);
            if (tail > 1) { mac(c[4], c[5]); mac(c[6], c[7]); }
            if (tail > 2) { mac(c[8], c[9]); mac(c[10], c[11]); }
        }
        Y* yd = yb + (int64_t)d * y_plane;
#pragma unroll
        for (int k = 0; k < VW; ++k)
            if (out_off[k] >= 0) store_slot<DT, E>(yd + out_off[k], acc[k]);
    }
}

template <sc_dtype_t DT, int VPT, int WSRC, int E>
__global__ void
slab_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
            const void* __restrict__ theta, const int32_t* __restrict__ lam,
            const int2* __restrict__ wl32, const void* __restrict__ codebook, const SlabArgs a)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    X* slab = reinterpret_cast<X*>(lds);
    int2* wst = reinterpret_cast<int2*>(lds + a.slab_bytes);
    unsigned char* cb_s = lds + a.slab_bytes + a.wcap * 8;

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = nthreads >> 6;

    // workgroup -> (sample, tile)
    const int tiles = a.tiles_p * a.tiles_q;
    const int b = fdiv(blockIdx.x, a.inv_tiles);
    const int t = blockIdx.x - b * tiles;
    const int tpi = fdiv(t, a.inv_tiles_q);
    const int tqi = t - tpi * a.tiles_q;
    const int p0 = tpi * a.TP, q0 = tqi * a.TQ;

    // ---------------------------------------------------------------- stage the input tile in LDS
    const X* xb = x + (int64_t)b * a.x_sample_stride;
    if (a.vec) {
        // pointwise layers: the tile is C rows of TQ consecutive pixels; 16-byte loads
        constexpr int EPV = 16 / (int)sizeof(X);
        const int vpr = a.Qs / EPV;
        const float inv_vpr = 1.0f / (float)vpr;
        const int total = a.C * vpr;
        for (int v = tid; v < total; v += nthreads) {
            const int c = fdiv(v, inv_vpr);
            const int col = q0 + (v - c * vpr) * EPV;
            uint4 val = make_uint4(0, 0, 0, 0);
            if (col < a.Wf) val = *reinterpret_cast<const uint4*>(xb + (int64_t)c * a.Wf + col);
            *reinterpret_cast<uint4*>(slab + c * a.chan_pitch + (v - c * vpr) * EPV) = val;
        }
    } else {
        // Offset of every element of one staged channel image inside the input plane, or -1 where
        // the image shows zero padding / lies outside the plane: computed once, so that staging
        // costs one division, one table read and one load per element; four elements per thread
        // and pass, loads first, so that four loads are in flight.
        const int row0 = p0 * a.s_h - a.pad_h, col0 = q0 * a.s_w - a.pad_w;
        const float inv_nsw = 1.0f / (float)a.nsw;
        int* tab = reinterpret_cast<int*>(lds + a.slab_bytes + a.wcap * 8 + 64);
        const int plane = a.Hf * a.Wf;
        for (int rem = tid; rem < a.chan_pitch; rem += nthreads) {
            const int sub = fdiv(rem, a.inv_sub_pitch);
            const int rem2 = rem - sub * a.sub_pitch;
            const int i = fdiv(rem2, a.inv_Qs);
            const int k = rem2 - i * a.Qs;
            const int ph = fdiv(sub, inv_nsw), pw = sub - ph * a.nsw;
            const int row = row0 + i * a.s_h + ph;
            const int col = col0 + k * a.s_w + pw;
            tab[rem] = (row >= 0 && row < a.Hf && col >= 0 && col < a.Wf) ? row * a.Wf + col : -1;
        }
        __syncthreads();
        for (int e0 = tid; e0 < a.slab_elems; e0 += 4 * nthreads) {
            X v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * nthreads;
                v[u] = X(0);
                if (e < a.slab_elems) {
                    const int c = fdiv(e, a.inv_chan_pitch);
                    const int o = tab[e - c * a.chan_pitch];
                    if (o >= 0) v[u] = load_in(xb + (int64_t)c * plane + o);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * nthreads;
                if (e < a.slab_elems) slab[e] = v[u];
            }
        }
    }
    if constexpr (kCodebook<DT>) {
        if (tid < kCodebookBytes<DT>) cb_s[tid] = static_cast<const unsigned char*>(codebook)[tid];
    }

    // ---------------------------------------------------------------- per-lane output bookkeeping
    // (E > 1, pointwise layers with scalar-load weights: slot k of a lane is the 128-bit word of
    // positions (k * 64 + lane) * E .. + E - 1; tile widths are whole words, so a word is valid or
    // not as one)
    static_assert(E == 1 || WSRC == 1, "packed positions: scalar-load weights");
    int out_off[VPT];
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const int f = (k * 64 + lane) * E;
        const int tp = fdiv(f, a.inv_Qs);
        const int tq = f - tp * a.Qs;
        const bool ok = f < a.F && tq < a.TQ && q0 + tq < a.Qf && p0 + tp < a.Pf;
        out_off[k] = ok ? (p0 + tp) * a.Qf + q0 + tq : -1;
    }
    Y* yb = y + (int64_t)b * a.D * a.y_plane;
    const unsigned char* lane_base = lds + lane * E * (int)sizeof(X);

    if constexpr (WSRC != 0) {
        // ------------------------------------------------------------ weights straight from global
        // memory (scalar loads or wave-uniform vector loads), no weight stage in LDS
        __syncthreads();  // slab complete
        if constexpr (E > 1) {
            stream_rows_packed<DT, VPT, E>(wl32, lane_base, yb, out_off, wave, nwaves, a.D, a.np, a.y_plane);
        } else {
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<int2*>(wl32), 0, (int)((int64_t)a.D * a.np * 8), 0x00020000);
            stream_rows<DT, VPT, WSRC>(wl32, rsrc, lane_base, yb, out_off, wave, nwaves, a.D, a.n, a.np, a.y_plane);
        }
        return;
    }

    // ---------------------------------------------------------------- stream the weight rows
    A acc[VPT];
    for (int ds0 = 0; ds0 < a.D; ds0 += a.DS) {
        const int rows = min(a.DS, a.D - ds0);
        int j0 = 0;
        do {
            const int jc = min(a.JC, a.n - j0);
            if constexpr (WSRC == 0) {
                __syncthreads();  // slab complete / previous stage consumed
                if (jc == a.n) {
                    const int cnt = rows * a.n;
                    const int64_t g0 = (int64_t)ds0 * a.n;
                    for (int e = tid; e < cnt; e += nthreads) {
                        const int l = lam[g0 + e];
                        wst[e] = make_int2(weight_bits<DT>(load_weight<DT>(theta, g0 + e, l, cb_s)),
                                           l & 0x7fffffff);
                    }
                } else {
                    const int cnt = rows * jc;
                    const float inv_jc = 1.0f / (float)jc;
                    for (int e = tid; e < cnt; e += nthreads) {
                        const int dd = fdiv(e, inv_jc);
                        const int64_t g = (int64_t)(ds0 + dd) * a.n + j0 + (e - dd * jc);
                        const int l = lam[g];
                        wst[e] = make_int2(weight_bits<DT>(load_weight<DT>(theta, g, l, cb_s)),
                                           l & 0x7fffffff);
                    }
                }
                __syncthreads();
            }
            for (int dd = wave; dd < rows; dd += nwaves) {
                if (j0 == 0) {
#pragma unroll
                    for (int k = 0; k < VPT; ++k) acc[k] = A(0);
                }
                if constexpr (WSRC == 0) {
                    const int2* wrow = wst + dd * jc;
#pragma unroll 8
                    for (int j = 0; j < jc; ++j) {
                        const int2 e = wrow[j];
                        const WL w = weight_from_bits<DT>(e.x);
                        const unsigned char* pj = lane_base + e.y;
#pragma unroll
                        for (int k = 0; k < VPT; ++k)
                            mac1<DT>(acc[k], w, *reinterpret_cast<const X*>(pj + k * 64 * (int)sizeof(X)));
                    }
                }
                if (j0 + jc >= a.n) {
                    Y* yd = yb + (int64_t)(ds0 + dd) * a.y_plane;
#pragma unroll
                    for (int k = 0; k < VPT; ++k)
                        if (out_off[k] >= 0) store_out(yd + out_off[k], narrow<DT>(acc[k]));
                }
            }
            j0 += a.JC;
        } while (j0 < a.n);
    }
}

// ------------------------------------------------------------------------------------------------
// Persistent, double-buffered form of the slab kernel for pointwise layers (tuning.pipeline = 1).
//
// One workgroup per CU walks over (sample, tile) pairs.  Its last tuning.producers waves are producers: they
// copy the next tile global -> LDS with the direct-to-LDS loads of gfx950 (16 bytes per lane, no
// VGPR staging, up to 63 in flight per wave) into the buffer that is not being read.  The other
// waves are consumers: they run the scalar-load gather-MAC of the one-shot kernel over the current
// buffer and store the outputs.  Keeping loads and stores in different waves keeps their vmcnt
// counters apart, so "my tile has landed" never has to wait for output stores, and the HBM stream
// of tile i+1 overlaps the arithmetic of tile i.  Two workgroup barriers per tile hand the buffers
// over.  Lanes whose pixels lie past the end of the plane load nothing; what they compute on stale
// LDS contents is never stored.
// ------------------------------------------------------------------------------------------------

template <sc_dtype_t DT, int VPT, int WSRC, int E>
__global__ void
slab_async_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                  const int2* __restrict__ wl32, const SlabArgs a)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = blockDim.x >> 6;
    const int nprod = a.nprod;
    const int ncons = nwaves - nprod;
    const int tiles = a.tiles_q;
    const int total = a.N * tiles;
    const float inv_TQ = a.inv_Qs;
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles per
    // round (its L2 then sees whole stretches of every channel row) when the grid is a multiple of 8
    const int step = gridDim.x;
    const int first = (step & 7) == 0 ? (int)(blockIdx.x & 7) * (step >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;

    if (wave >= ncons) {
        // ------------------------------------------------------------------ producer waves
        const int pw = wave - ncons;
        // Producers run at raised wave priority so that their short instruction streams are not
        // queued behind the consumers' long ones.
        __builtin_amdgcn_s_setprio(3);
        auto issue = [&](int t, int buf) {
            const int b = fdiv(t, a.inv_tiles);
            const int q0 = (t - b * tiles) * a.TQ;
            dma_tile<X>(x + (int64_t)b * a.x_sample_stride + q0, lds + buf * a.slab_bytes, a.C, a.TQ,
                        a.Wf, q0, pw, nprod, lane, inv_TQ);
        };
        if (first < total) issue(first, 0);
        int it = 0;
        for (int t = first; t < total; t += step, ++it) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // tile t has landed
            __syncthreads();                                   // A: consumers may read buffer it&1
            if (t + step < total) issue(t + step, (it + 1) & 1);
            __syncthreads();                                   // B: buffer it&1 is free again
        }
        return;
    }

    // ---------------------------------------------------------------------- consumer waves
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int2*>(wl32), 0, (int)((int64_t)a.D * a.np * 8), 0x00020000);
    int it = 0;
    for (int t = first; t < total; t += step, ++it) {
        const int b = fdiv(t, a.inv_tiles);
        const int q0 = (t - b * tiles) * a.TQ;
        // E > 1 (scalar-load weights): positions packed by the 32- or 128-bit word (VPT then
        // counts words per lane); otherwise lane l owns positions l, l + 64, ...
        constexpr bool kPacked = E > 1;
        static_assert(!kPacked || WSRC == 1, "packed positions: scalar-load weights");
        int out_off[VPT];
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int f = (k * 64 + lane) * E;
            out_off[k] = (f < a.TQ && q0 + f < a.Qf) ? q0 + f : -1;
        }
        Y* yb = y + (int64_t)b * a.D * a.y_plane;
        const unsigned char* lane_base = lds + (it & 1) * a.slab_bytes + lane * E * (int)sizeof(X);
        __syncthreads();  // A
        if constexpr (kPacked)
            stream_rows_packed<DT, VPT, E>(wl32, lane_base, yb, out_off, wave, ncons, a.D, a.np, a.y_plane);
        else
            stream_rows<DT, VPT, WSRC>(wl32, rsrc, lane_base, yb, out_off, wave, ncons, a.D, a.n, a.np, a.y_plane);
        __syncthreads();  // B
    }
}

// ------------------------------------------------------------------------------------------------
// Symmetric persistent form for pointwise layers (tuning.pipeline = 2): every wave of the
// workgroup both copies and multiplies.
//
// Right after the barrier that opens tile i each wave issues its share of the direct-to-LDS copy of
// tile i+1 into the other buffer, then multiplies its rows of tile i.  The D rows are dealt to the
// waves as contiguous ranges, so with D a multiple of the wave count every wave has the same work
// and no wave is set aside for copying; one barrier per tile both publishes tile i+1 and frees the
// buffer of tile i-1.  The copies are hand-issued (dma16<true>), so the wave waits on vmcnt itself:
// once per tile, just before the store of its last row -- by then its share of tile i+1 (issued a
// whole tile earlier) and its earlier stores have long completed, and the last store stays in
// flight across the barrier.
//
// Rows are packed with an even pitch np and fetched 8 entries at a time by scalar loads through
// the constant address space.
// ------------------------------------------------------------------------------------------------
template <sc_dtype_t DT, int VPT>
__global__ void
slab_sym_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                const int2* __restrict__ wl32, const SlabArgs a)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    typedef const int16v __attribute__((address_space(4)))* c16_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = blockDim.x >> 6;
    const int tiles = a.tiles_q;
    const int total = a.N * tiles;
    // (XCD-aware: contiguous runs of work items per XCD, see slab_async_kernel)
    const int step = gridDim.x;
    const int first = (step & 7) == 0 ? (int)(blockIdx.x & 7) * (step >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    if (first >= total) return;

    // contiguous row range of this wave
    const int base_rows = a.D / nwaves, extra = a.D - base_rows * nwaves;
    const int row0 = wave * base_rows + min(wave, extra);
    const int nrows = base_rows + (wave < extra ? 1 : 0);
    const int ng = a.np >> 3, tp = (a.np & 7) >> 1;              // full 8-entry groups and tail pairs per row

    auto issue = [&](int t, int buf) {
        const int b = fdiv(t, a.inv_tiles);
        const int q0 = (t - b * tiles) * a.TQ;
        if (a.dmab == 16)
            dma_tile<X, true, 16>(x + (int64_t)b * a.x_sample_stride + q0, lds + buf * a.slab_bytes, a.C,
                                  a.TQ, a.Wf, q0, wave, nwaves, lane, a.inv_Qs);
        else
            dma_tile<X, true, 4>(x + (int64_t)b * a.x_sample_stride + q0, lds + buf * a.slab_bytes, a.C,
                                 a.TQ, a.Wf, q0, wave, nwaves, lane, a.inv_Qs);
    };
    issue(first, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int it = 0;
    for (int t = first; t < total; t += step, ++it) {
        __syncthreads();      // tile t is complete in buffer it&1; the other buffer is free
        if (t + step < total) issue(t + step, (it + 1) & 1);
        if (nrows == 0) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            continue;
        }
        const int b = fdiv(t, a.inv_tiles);
        const int q0 = (t - b * tiles) * a.TQ;
        int out_off[VPT];
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int f = k * 64 + lane;
            out_off[k] = (f < a.TQ && q0 + f < a.Qf) ? q0 + f : -1;
        }
        Y* yd = y + ((int64_t)b * a.D + row0) * a.y_plane;
        const unsigned char* lane_base = lds + (it & 1) * a.slab_bytes + lane * (int)sizeof(X);
        for (int r = 0; r < nrows; ++r) {
            A acc[VPT];
#pragma unroll
            for (int k = 0; k < VPT; ++k) acc[k] = A(0);
            const int2* prow = wl32 + (int64_t)(row0 + r) * a.np;
            auto mac = [&](int wbits, int lam) {
                const WL w = weight_from_bits<DT>(wbits);
                const unsigned char* pj = lane_base + lam;
#pragma unroll
                for (int k = 0; k < VPT; ++k)
                    mac1<DT>(acc[k], w, *reinterpret_cast<const X*>(pj + k * 64 * (int)sizeof(X)));
            };
            for (int g = 0; g < ng; ++g) {
                // no software prefetch on purpose: with nothing else pending on the scalar/LDS
                // counter the eight gathers can be waited for one by one, so the multiply-adds
                // start when the first value arrives; the other waves hide the scalar load
                const int16v c = *(c16_t)(prow + 8 * g);
#pragma unroll
                for (int i = 0; i < 8; ++i) mac(c[2 * i], c[2 * i + 1]);
            }
            if (tp > 0) {
                // the last 1..3 pairs of the row: one more 8-entry load (it reaches into the next
                // row, or into the slack behind the table), of which only the row's pairs are used
                const int16v c = *(c16_t)(prow + 8 * ng);
                mac(c[0], c[1]); mac(c[2], c[3]);
                if (tp > 1) { mac(c[4], c[5]); mac(c[6], c[7]); }
                if (tp > 2) { mac(c[8], c[9]); mac(c[10], c[11]); }
            }
            // before the store of the wave's last row: this wave's share of the next tile and its
            // earlier stores are complete
            if (r == nrows - 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int k = 0; k < VPT; ++k)
                if (out_off[k] >= 0) store_out(yd + out_off[k], narrow<DT>(acc[k]));
            yd += a.y_plane;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Channel-chunked, pipelined form for pointwise layers (tuning.chunk_c > 0).
//
// A tile of TQ pixels is multiplied chunk by chunk: an LDS buffer holds CC input channels of the
// tile, the producers stream chunk i+1 into the other buffer while the consumers work on chunk i,
// and every consumer wave keeps the accumulators of its RPW output channels x VPT positions in
// registers from the first chunk of a tile to the last.  Because a buffer only holds CC channels,
// TQ can be 2..8 waves wide even when C*TQ would not fit LDS: every (theta, lambda) then feeds VPT
// multiply-adds and one paired LDS read serves two of them, and the global loads become long
// contiguous runs.  The weight table is stored as segments (output channel, chunk) -- the entries
// of a row whose input channel lies in the chunk, contiguous because rows are sorted by column --
// each padded to an even length; lambda is the byte offset inside the chunk buffer.
// A workgroup handles DTW output channels (all of them unless tuning.tile_d says otherwise).
// ------------------------------------------------------------------------------------------------
template <sc_dtype_t DT>
__global__ void __launch_bounds__(256)
expand_chunked_kernel(const void* __restrict__ theta, const int32_t* __restrict__ lam,
                      const int32_t* __restrict__ col, const int32_t* __restrict__ seg_off,
                      const int32_t* __restrict__ first_j, int2* __restrict__ out, int D, int n,
                      int RS, int CC, int nch, int copies, int ex, int copy_bytes)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)D * n) return;
    const int d = (int)(i / n), j = (int)(i - (int64_t)d * n);
    const int ch = ((col[i] & 0x7fffffff) / RS) / CC;
    const int l = lam[i];
    const int64_t si = (int64_t)d * nch + ch;
    const int k = j - first_j[si];
    // (a segment built without the fillers is shorter than the entries that map to its chunk: the
    // fillers behind it are dropped; one that lands on a padding slot is a zero weight either way)
    if (k >= seg_off[si + 1] - seg_off[si]) return;
    int lb = l & 0x7fffffff;
    if (copies > 1) {
        // shifted images: an entry s elements past a word boundary reads image s one word-aligned
        const int el = lb / ex, sh = el % copies;
        lb = (el - sh) * ex + sh * copy_bytes;
    }
    out[(int64_t)seg_off[si] + k] = make_int2(weight_bits<DT>(load_weight<DT>(theta, i, l, nullptr)), lb);
}

sc_status_t expand_weights_chunked(const Plan& p, const SlabGeom& g, const int32_t* lam_slab, const int32_t* seg_off,
                                   const int32_t* first_j, int2* wlc_out, hipStream_t stream)
{
    const int64_t cnt = (int64_t)p.L.D * p.n;
    if (cnt == 0) return SC_OK;
    const unsigned blocks = (unsigned)((cnt + 255) / 256);
#define SC_EXPANDC(DT)                                                                             \
    hipLaunchKernelGGL(expand_chunked_kernel<DT>, dim3(blocks), dim3(256), 0, stream, p.d_theta,   \
                       lam_slab, p.d_col, seg_off, first_j, wlc_out, p.L.D, p.n,                   \
                       p.L.R * p.L.S, g.CC, g.nchunks, g.copies, p.ex, g.copy_bytes)
    switch (p.dtype) {
        case SC_F32: SC_EXPANDC(SC_F32); break;
        case SC_F16: SC_EXPANDC(SC_F16); break;
        case SC_I8: SC_EXPANDC(SC_I8); break;
        default: return SC_ERR_UNSUPPORTED;
    }
#undef SC_EXPANDC
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

struct ChunkArgs {
    int C, D, N, Wf, TQ, tiles, CC, nchunks, DTW, ndt, nprod, slab_bytes, dmab;
    int nbuf;                                       // chunk buffers in LDS: 2, or nprod + 1
    float inv_tiles, inv_TQ, inv_ndt;
    int64_t x_sample_stride, y_plane;
};

template <sc_dtype_t DT, int VPT, int RPW, int E>
__global__ void
slab_chunk_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                  const int2* __restrict__ wlc, const int32_t* __restrict__ seg_off, const ChunkArgs a)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = blockDim.x >> 6;
    const int nprod = a.nprod;
    const int ncons = nwaves - nprod;
    const int units = a.N * a.tiles * a.ndt;        // (sample, tile, output-channel block)
    // (XCD-aware: contiguous runs of work items per XCD, see slab_async_kernel)
    const int step = gridDim.x;
    const int first = (step & 7) == 0 ? (int)(blockIdx.x & 7) * (step >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    typedef const int16v __attribute__((address_space(4)))* c16_t;
    typedef const int32_t __attribute__((address_space(4)))* ci_t;
    const ci_t segs = (ci_t)seg_off;                // read through the constant address space
    // unit u -> (sample b, tile, dt); consecutive units share the input tile
    auto decode = [&](int u, int& b, int& q0, int& dt) {
        const int bt = fdiv(u, a.inv_ndt);
        dt = u - bt * a.ndt;
        b = fdiv(bt, a.inv_tiles);
        q0 = (bt - b * a.tiles) * a.TQ;
    };

    if (wave >= ncons) {
        // ------------------------------------------------------------------ producer waves
        __builtin_amdgcn_s_setprio(3);
        const int pw = wave - ncons;
        auto issue = [&](int u, int ch, int buf) {
            int b, q0, dt;
            decode(u, b, q0, dt);
            const int c0 = ch * a.CC;
            dma_tile<X>(x + (int64_t)b * a.x_sample_stride + q0 + (int64_t)c0 * a.Wf,
                        lds + buf * a.slab_bytes, min(a.CC, a.C - c0), a.TQ, a.Wf, q0, pw, nprod, lane,
                        a.inv_TQ);
        };
        if (a.nbuf > 2) {
            // nprod + 1 buffers: item i (a chunk of a tile) belongs to producer wave i % nprod, which
            // copies it alone into buffer i % nbuf, so a wave never has more than one item in flight
            // and "my item has landed" is vmcnt(0).  nprod items are in flight while one is
            // multiplied: the HBM latency of a chunk is spread over nprod phases instead of one.
            auto issue1 = [&](int u, int ch, int buf) {
                int b, q0, dt;
                decode(u, b, q0, dt);
                const int c0 = ch * a.CC;
                dma_tile<X>(x + (int64_t)b * a.x_sample_stride + q0 + (int64_t)c0 * a.Wf,
                            lds + buf * a.slab_bytes, min(a.CC, a.C - c0), a.TQ, a.Wf, q0, 0, 1, lane,
                            a.inv_TQ);
            };
            // item index -> (unit, chunk): items are numbered along this workgroup's units
            auto item = [&](int i, int& u, int& ch) {
                const int q = i / a.nchunks;          // (wave-uniform integer division, once per item)
                ch = i - q * a.nchunks;
                u = first + q * step;
            };
            int nunits = first < units ? (units - first + step - 1) / step : 0;
            const int nitems = nunits * a.nchunks;
            if (pw < nitems) { int u, ch; item(pw, u, ch); issue1(u, ch, pw % a.nbuf); }
            int owner = 0, nxt_buf = nprod % a.nbuf;
            for (int i = 0; i < nitems; ++i) {
                if (owner == pw) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // item i has landed
                // one barrier per phase: it says that item i is in LDS and that every consumer is
                // done with item i - 1, whose buffer the next copy goes to
                __syncthreads();
                if (owner == pw && i + nprod < nitems) { int u, ch; item(i + nprod, u, ch); issue1(u, ch, nxt_buf); }
                if (++owner == nprod) owner = 0;
                if (++nxt_buf == a.nbuf) nxt_buf = 0;
            }
            return;
        }
        if (first < units) issue(first, 0, 0);
        int it = 0;
        for (int u = first; u < units; u += step) {
            for (int ch = 0; ch < a.nchunks; ++ch, ++it) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // item (u, ch) has landed
                __syncthreads();                                   // A
                int un = u, chn = ch + 1;
                if (chn == a.nchunks) { chn = 0; un = u + step; }
                if (un < units) issue(un, chn, (it + 1) & 1);
                __syncthreads();                                   // B
            }
        }
        return;
    }

    // ---------------------------------------------------------------------- consumer waves
    // E > 1 (packed positions): slot k of a lane is the 32-bit word of positions
    // (k * 64 + lane) * E .. + E - 1; rows and tiles are whole words, so a word is valid or not as one
    static_assert(E == 1 || E * (int)sizeof(X) == 4 || E * (int)sizeof(X) == 16, "packed positions: 32- or 128-bit words");
    A acc[RPW][VPT][E];
    int out_off[VPT];
    int it = 0, cbuf = 0;
    for (int u = first; u < units; u += step) {
        int b, q0, dt;
        decode(u, b, q0, dt);
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int f = (k * 64 + lane) * E;
            out_off[k] = (f < a.TQ && q0 + f < a.Wf) ? q0 + f : -1;
        }
#pragma unroll
        for (int r = 0; r < RPW; ++r)
#pragma unroll
            for (int k = 0; k < VPT; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e) acc[r][k][e] = A(0);
        const int d0 = dt * a.DTW;
        const int dend = min(a.D, d0 + a.DTW);
        for (int ch = 0; ch < a.nchunks; ++ch, ++it) {
            const unsigned char* lane_base = lds + cbuf * a.slab_bytes + lane * E * (int)sizeof(X);
            if (++cbuf == a.nbuf) cbuf = 0;
            __syncthreads();  // A
            // one segment per row and chunk, multiplied 8 entries at a time with no software
            // prefetch (the gathers of a group are then waited for one by one, and the other
            // waves hide the scalar loads); a partial last group is loaded whole -- the table has
            // 16 spare entries -- and only its pairs inside the segment are used
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                const int d = d0 + wave + r * ncons;
                if (d < dend) {
                    const int si = d * a.nchunks + ch;
                    const int s0 = segs[si], len = segs[si + 1] - s0;     // even
                    auto mac = [&](int wbits, int lam) {
                        const WL w = weight_from_bits<DT>(wbits);
                        const unsigned char* pj = lane_base + lam;
#pragma unroll
                        for (int k = 0; k < VPT; ++k)
                            mac_slot<DT, E>(acc[r][k], w, pj + k * 64 * E * (int)sizeof(X));
                    };
                    const int2* seg = wlc + s0;
                    int e = 0;
                    for (; e + 8 <= len; e += 8) {
                        const int16v c = *(c16_t)(seg + e);
#pragma unroll
                        for (int i = 0; i < 8; ++i) mac(c[2 * i], c[2 * i + 1]);
                    }
                    const int tail = (len - e) >> 1;                      // 0..3 pairs
                    if (tail > 0) {
                        const int16v c = *(c16_t)(seg + e);
                        mac(c[0], c[1]); mac(c[2], c[3]);
                        if (tail > 1) { mac(c[4], c[5]); mac(c[6], c[7]); }
                        if (tail > 2) { mac(c[8], c[9]); mac(c[10], c[11]); }
                    }
                }
            }
            if (a.nbuf == 2) __syncthreads();  // B (with three or more buffers barrier A of the next phase serves)
        }
        Y* yb = y + (int64_t)b * a.D * a.y_plane;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int d = d0 + wave + r * ncons;
            if (d < dend) {
                Y* yd = yb + (int64_t)d * a.y_plane;
#pragma unroll
                for (int k = 0; k < VPT; ++k)
                    if (out_off[k] >= 0) store_slot<DT, E>(yd + out_off[k], acc[r][k]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Symmetric persistent form with channel chunks (tuning.pipeline = 2, tuning.chunk_c > 0).
//
// As slab_sym_kernel, but an LDS buffer holds only CC input channels of a tile of TQ pixels, so
// tiles 2..4 waves wide fit twice into LDS even for layers with many input channels; one LDS
// instruction then serves two positions of a lane (they are 64 elements apart, which the paired
// read covers) and every scalar-loaded entry feeds VPT multiply-adds.  A workgroup walks over
// (tile, chunk) items; each wave keeps the accumulators of its rows (at most kMaxRowsPerWave) in
// registers from the first chunk of a tile to the last and stores after the last.  The weight
// table holds one segment per (row, chunk), padded with zero weights to whole 8-entry groups.
// ------------------------------------------------------------------------------------------------
template <sc_dtype_t DT, int VPT, int E>
__global__ void
slab_symc_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
                 const int2* __restrict__ wlc, const int32_t* __restrict__ seg_off, const ChunkArgs a)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    typedef const int16v __attribute__((address_space(4)))* c16_t;
    typedef const int32_t __attribute__((address_space(4)))* ci_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int RPW = kMaxRowsPerWave;
    static_assert(E == 1 || E * (int)sizeof(X) == 4 || E * (int)sizeof(X) == 16, "packed positions: 32- or 128-bit words");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = blockDim.x >> 6;
    const int units = a.N * a.tiles * a.ndt;        // (sample, tile, output-channel block)
    // (XCD-aware: contiguous runs of work items per XCD, see slab_async_kernel)
    const int step = gridDim.x;
    const int first = (step & 7) == 0 ? (int)(blockIdx.x & 7) * (step >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    if (first >= units) return;
    auto decode = [&](int u, int& b, int& q0, int& dt) {
        const int bt = fdiv(u, a.inv_ndt);
        dt = u - bt * a.ndt;
        b = fdiv(bt, a.inv_tiles);
        q0 = (bt - b * a.tiles) * a.TQ;
    };
    auto issue = [&](int u, int ch, int buf) {
        int b, q0, dt;
        decode(u, b, q0, dt);
        const int c0 = ch * a.CC;
        if (a.dmab == 16)
            dma_tile<X, true, 16>(x + (int64_t)b * a.x_sample_stride + q0 + (int64_t)c0 * a.Wf,
                                  lds + buf * a.slab_bytes, min(a.CC, a.C - c0), a.TQ, a.Wf, q0, wave,
                                  nwaves, lane, a.inv_TQ);
        else
            dma_tile<X, true, 4>(x + (int64_t)b * a.x_sample_stride + q0 + (int64_t)c0 * a.Wf,
                                 lds + buf * a.slab_bytes, min(a.CC, a.C - c0), a.TQ, a.Wf, q0, wave,
                                 nwaves, lane, a.inv_TQ);
    };
    const ci_t segs = (ci_t)seg_off;
    const c16_t wl = (c16_t)wlc;

    issue(first, 0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int it = 0;
    for (int u = first; u < units; u += step) {
        int b, q0, dt;
        decode(u, b, q0, dt);
        // contiguous row range of this wave inside the output-channel block
        const int d0 = dt * a.DTW, dcnt = min(a.DTW, a.D - d0);
        const int base_rows = dcnt / nwaves, extra = dcnt - base_rows * nwaves;
        const int row0 = d0 + wave * base_rows + min(wave, extra);
        const int nrows = base_rows + (wave < extra ? 1 : 0);
        A acc[RPW][VPT][E];     // E > 1: slot k is the word of positions (k * 64 + lane) * E .. + E - 1
#pragma unroll
        for (int r = 0; r < RPW; ++r)
#pragma unroll
            for (int k = 0; k < VPT; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e) acc[r][k][e] = A(0);
        for (int ch = 0; ch < a.nchunks; ++ch, ++it) {
            __syncthreads();      // item (u, ch) is complete in buffer it&1; the other buffer is free
            {
                int un = u, chn = ch + 1;
                if (chn == a.nchunks) { chn = 0; un = u + step; }
                if (un < units) issue(un, chn, (it + 1) & 1);
            }
            const unsigned char* lane_base = lds + (it & 1) * a.slab_bytes + lane * E * (int)sizeof(X);
#pragma unroll
            for (int r = 0; r < RPW; ++r) {
                if (r < nrows) {
                    const int si = (row0 + r) * a.nchunks + ch;
                    const int s0 = segs[si], s1 = segs[si + 1];       // multiples of 8 entries
                    for (int e = s0; e < s1; e += 8) {
                        const int16v c = wl[e >> 3];
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const WL w = weight_from_bits<DT>(c[2 * i]);
                            const unsigned char* pj = lane_base + c[2 * i + 1];
#pragma unroll
                            for (int k = 0; k < VPT; ++k)
                                mac_slot<DT, E>(acc[r][k], w, pj + k * 64 * E * (int)sizeof(X));
                        }
                    }
                }
            }
            // this wave's share of the next item (and, after a tile's last chunk, nothing younger
            // than stores issued a whole item ago) must be complete before the next barrier
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        Y* yd = y + ((int64_t)b * a.D + row0) * a.y_plane;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            if (r < nrows) {
#pragma unroll
                for (int k = 0; k < VPT; ++k) {
                    const int f = (k * 64 + lane) * E;
                    if (f < a.TQ && q0 + f < a.Wf)
                        store_slot<DT, E>(yd + (int64_t)r * a.y_plane + q0 + f, acc[r][k]);
                }
            }
        }
    }
}

template <sc_dtype_t DT, int VPT, int E = 1>
static sc_status_t launch_symc_one(const Plan& p, const ChunkArgs& a, const void* x, void* y, hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = slab_symc_kernel<DT, VPT, E>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    const int units = a.N * a.tiles * a.ndt;
    const int grid = std::min(units, kNumCU * std::max(1, kMaxLdsBytes / p.geom.lds_bytes));
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(p.tuning.wg_threads), p.geom.lds_bytes, stream,
                       static_cast<const X*>(x), static_cast<Y*>(y), p.d_wlc, p.d_seg_off, a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

// ------------------------------------------------------------------------------------------------
// Channel-chunked one-shot form for any layer shape (tuning.pipeline = 0, tuning.chunk_c > 0).
//
// One workgroup = one sample x one output tile x one block of DTW output channels.  The input
// region of the tile (halo, zero padding and stride phases as in slab_kernel) is staged CC input
// channels at a time; every wave keeps the accumulators of its rows (a contiguous range, at most
// kMaxRowsPerWave) x positions in registers across the chunks and stores after the last.  Because
// only CC channels are resident, layers with many input channels can take tiles several output
// rows high -- all 64 lanes of a wave busy on strided and small-plane layers where a full-channel
// tile is limited by LDS to a fraction of a wave.  Weights: the per-(row, chunk) segments of the
// chunked table, read by scalar loads 8 entries at a time.  Loads and arithmetic of one workgroup
// alternate; two or more workgroups per CU overlap them.
// ------------------------------------------------------------------------------------------------
template <sc_dtype_t DT, int VPT, bool MS, int E, bool LANES, bool FLAT, int ROWB, int SMODE>
__global__ void
slab_cc_kernel(const typename Types<DT>::X* __restrict__ x, typename Types<DT>::Y* __restrict__ y,
               const int2* __restrict__ wlc, const int32_t* __restrict__ seg_off, const SlabArgs a)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    typedef const int16v __attribute__((address_space(4)))* c16_t;
    typedef const int32_t __attribute__((address_space(4)))* ci_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int RPW = kMaxRowsPerWave;
    constexpr int kStageLoads = 4;    // global loads a thread has in flight while staging
    X* slab = reinterpret_cast<X*>(lds);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = nthreads >> 6;

    // workgroup -> (sample, tile, output-channel block); consecutive workgroups share the tile
    const int tiles = a.tiles_p * a.tiles_q;
    // (XCD-aware: workgroups are dealt round-robin to the 8 XCDs; number them so that each XCD gets
    // a contiguous run, and the output-channel blocks of one tile share an L2)
    const int grid = gridDim.x;
    const int wg = (grid & 7) == 0 ? (int)(blockIdx.x & 7) * (grid >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int bt0 = fdiv(wg, a.inv_ndt);
    const int dt = wg - bt0 * a.ndt;
    // (split-K: the chunks of a tile are dealt to ksplit workgroups, each adding its partial sums to
    // y, which the launcher has cleared)
    const int bt = a.ksplit > 1 ? fdiv(bt0, a.inv_ksplit) : bt0;
    const int ks = a.ksplit > 1 ? bt0 - bt * a.ksplit : 0;
    const int ch_lo = a.ksplit > 1 ? ks * a.cps : 0;
    const int ch_hi = a.ksplit > 1 ? min(a.nchunks, ch_lo + a.cps) : a.nchunks;
    const int bg = fdiv(bt, a.inv_tiles);
    const int t = bt - bg * tiles;
    // MS: the workgroup takes VPT samples of a tile of at most 64 positions (slot k of a lane is
    // sample b + k); otherwise one sample, and slot k is position k * 64 + lane
    // (SMODE 1, FSM: the tile is the planes of samples b .. b + a.FS - 1 of a pointwise layer, end
    // to end.  SMODE 2, SI: the workgroup takes E samples, an LDS word holds the same element of all
    // of them and slot k of a lane is position k * 64 + lane of each)
    constexpr bool FSM = SMODE == 1, SI = SMODE == 2;
    static_assert(SMODE == 0 || (E > 1 && !MS && !LANES && !FLAT && (ROWB == 0 || SMODE == 2)), "several samples per packed tile: staged by table, by blocks or (interleaved samples) by rows");
    const int b = MS ? bg * VPT : (FSM ? bg * a.FS : (SI ? bg * E * a.SG : bg));
    // (SI with several sample groups: lane = group * F + position, one slot per lane)
    const int lgrp = (SI && a.SG > 1) ? min(fdiv(lane, 1.0f / (float)a.F), a.SG - 1) : 0;
    const int lpos = (SI && a.SG > 1) ? lane - lgrp * a.F : lane;
    const bool lane_on = !(SI && a.SG > 1) || lane < a.SG * a.F;
    const int tpi = fdiv(t, a.inv_tiles_q);
    const int tqi = t - tpi * a.tiles_q;
    const int p0 = tpi * a.TP, q0 = tqi * a.TQ;
    const int row0 = p0 * a.s_h - a.pad_h, col0 = q0 * a.s_w - a.pad_w;
    const float inv_nsw = 1.0f / (float)a.nsw;
    const X* xb = x + (int64_t)b * a.x_sample_stride;

    // E > 1 (packed positions): slot k of a lane is the 32-bit word of positions
    // (k * 64 + lane) * E .. + E - 1 of the flat tile
    static_assert(E == 1 || (!MS && (E * (int)sizeof(X) == 4 || E * (int)sizeof(X) == 16)), "packed positions: one sample, 32- or 128-bit words");
    int out_off[VPT][E];
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int f = (MS || SI) ? (SI ? k * 64 + lpos : lane) : (k * 64 + lane) * E + e;
            if constexpr (FSM) {
                const int sm = fdiv(f, 1.0f / (float)a.Qf);
                out_off[k][e] = (f < a.F && b + sm < a.N) ? sm * a.D * a.Qf + (f - sm * a.Qf) : -1;
                continue;
            }
            const int tp = fdiv(f, a.inv_Qs);
            const int tq = f - tp * a.Qs;
            const bool ok = f < a.F && tq < a.TQ && q0 + tq < a.Qf && p0 + tp < a.Pf && (!MS || b + k < a.N) &&
                            (!SI || (lane_on && b + lgrp * E + e < a.N));
            out_off[k][e] = ok ? (p0 + tp) * a.Qf + q0 + tq : -1;
        }
    }
    const int img_elems = a.CC * a.chan_pitch;                       // one sample's chunk image
    const int koff = MS ? img_elems * (int)sizeof(X) : 64 * E * (int)sizeof(X);
    const unsigned char* lane_base = lds + (lgrp * img_elems + lpos) * E * (int)sizeof(X);

    // Offset of every element of one staged channel image inside the input plane, or -1 where the
    // image shows zero padding / lies outside the plane: computed once, so that staging a chunk
    // costs one division, one table read and one load per element.
    // (FLAT: a pointwise layer with one tile per plane -- the image of a chunk is one contiguous,
    // 16-byte aligned block of the input and is copied as such, no table.
    // ROWB > 0: unit strides (or strides of two with both phases in use) and a tile as wide as the
    // plane -- the rows of a channel image are whole rows of the input (split by parity into the
    // phase images when the stride is two), and those rows are contiguous in memory: they are
    // copied with ROWB-byte loads, two index divisions per load instead of one per element, no
    // table.  The padding is written once, here: no later store touches it.)
    static_assert(ROWB == 0 || (!MS && !FLAT && ROWB % (int)sizeof(X) == 0), "row runs: one sample, whole elements");
    int* tab = reinterpret_cast<int*>(lds + a.slab_bytes);
    const int plane = a.Hf * a.Wf;
    if constexpr (ROWB > 0) {
        uint4v* z = reinterpret_cast<uint4v*>(lds);
        for (int i = tid; i < (a.slab_bytes >> 4); i += nthreads) z[i] = uint4v{0u, 0u, 0u, 0u};
    }
    constexpr int RV = ROWB > 0 ? ROWB / (int)sizeof(X) : 1;        // elements per load
    const int rlo = max(row0, 0);
    const int rcnt = min(row0 + a.SR * a.s_h, a.Hf) - rlo;          // input rows under the tile (>= 1)
    const int vpr = a.Wf / RV;                                       // loads per row
    const int per_c = rcnt * vpr;                                    // loads per channel
    const float inv_per_c = 1.0f / (float)per_c, inv_vpr = 1.0f / (float)vpr;
    for (int rem = tid; rem < ((FLAT || ROWB > 0) ? 0 : a.chan_pitch); rem += nthreads) {
        if constexpr (FSM) {
            // element rem of a channel image is position rem % plane of sample b + rem / plane
            const int sm = fdiv(rem, 1.0f / (float)plane);
            tab[rem] = (rem < a.F && b + sm < a.N) ? sm * (int)a.x_sample_stride + (rem - sm * plane) : -1;
            continue;
        }
        const int sub = fdiv(rem, a.inv_sub_pitch);
        const int rem2 = rem - sub * a.sub_pitch;
        const int i = fdiv(rem2, a.inv_Qs);
        const int k = rem2 - i * a.Qs;
        const int ph = fdiv(sub, inv_nsw), pw = sub - ph * a.nsw;
        const int row = row0 + i * a.s_h + ph;
        const int col = col0 + k * a.s_w + pw;
        tab[rem] = (row >= 0 && row < a.Hf && col >= 0 && col < a.Wf) ? row * a.Wf + col : -1;
    }
    __syncthreads();

    // contiguous row range of this wave inside the output-channel block
    const int d0 = dt * a.DTW, dcnt = min(a.DTW, a.D - d0);
    const int base_rows = dcnt / nwaves, extra = dcnt - base_rows * nwaves;
    const int drow0 = d0 + wave * base_rows + min(wave, extra);
    const int nrows = base_rows + (wave < extra ? 1 : 0);
    const ci_t segs = (ci_t)seg_off;

    A acc[RPW][VPT][E];
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
        for (int k = 0; k < VPT; ++k)
#pragma unroll
            for (int e = 0; e < E; ++e) acc[r][k][e] = A(0);

    for (int ch = ch_lo; ch < ch_hi; ++ch) {
        const int c0 = ch * a.CC;
        const int elems = min(a.CC, a.C - c0) * a.chan_pitch;
        if (ch > ch_lo) __syncthreads();      // the previous chunk has been consumed
        // four elements per thread and pass, loads first, so that four loads are in flight
        bool staged = false;
        if constexpr (FSM) if (a.fs_vec) {
            staged = true;
            // samples end to end: the chunk of each sample is one contiguous block of the input, read
            // 16 bytes per load; the elements of a load go to their channel rows one by one
            constexpr int EPV = 16 / (int)sizeof(X);
            struct alignas(16) Vec { X e[EPV]; };
            const float inv_plane = 1.0f / (float)plane;
            const int nvec = min(a.CC, a.C - c0) * plane / EPV;
            const float inv_nvec = 1.0f / (float)nvec;
            const int total = min(a.FS, a.N - b) * nvec;
            for (int i0 = tid; i0 < total; i0 += kStageLoads * nthreads) {
                Vec v[kStageLoads];
                int smi[kStageLoads];
#pragma unroll
                for (int u = 0; u < kStageLoads; ++u) {
                    const int i = i0 + u * nthreads;
                    if (i < total) {
                        smi[u] = fdiv(i, inv_nvec);
                        const int iv = i - smi[u] * nvec;
                        v[u] = *reinterpret_cast<const Vec*>(xb + (int64_t)smi[u] * a.x_sample_stride + (int64_t)c0 * plane + iv * EPV);
                        smi[u] *= plane;                       // first position of the sample in a channel row
                    }
                }
#pragma unroll
                for (int u = 0; u < kStageLoads; ++u) {
                    const int i = i0 + u * nthreads;
                    if (i < total) {
                        const int sm = fdiv(i, inv_nvec);
                        const int e0 = (i - sm * nvec) * EPV;
                        int c = fdiv(e0, inv_plane);
                        int pos = e0 - c * plane;
                        int dst = c * a.chan_pitch + smi[u] + pos;
#pragma unroll
                        for (int j = 0; j < EPV; ++j) {
                            slab[dst] = v[u].e[j];
                            // next element: the next position, or the first of the next channel row
                            ++pos; ++dst;
                            if (pos == plane) { pos = 0; dst += a.chan_pitch - plane; }
                        }
                    }
                }
            }
        }
        if constexpr (SI && ROWB > 0) {
            // interleaved samples staged by rows: a thread loads the same ROWB bytes (RV adjacent
            // columns of one input row) of each of the E samples and writes them into RV words, word j
            // holding column j of every sample.  Two index divisions per E loads instead of one per
            // word and load, wide loads along the rows; the padding words were cleared once.
            staged = true;
            struct alignas(ROWB) Vec { X e[RV]; };
            struct alignas(E * sizeof(X)) Word { X e[E]; };
            const int nvec = min(a.CC, a.C - c0) * per_c;
            for (int sg = 0; sg < a.SG; ++sg) {
                Word* wslab = reinterpret_cast<Word*>(lds) + sg * img_elems;
                const X* xc = xb + (int64_t)sg * E * a.x_sample_stride + (int64_t)c0 * plane;
                const int bs = b + sg * E;                       // first sample of this group
                for (int i = tid; i < nvec; i += nthreads) {
                    const int c = fdiv(i, inv_per_c);
                    const int r2 = i - c * per_c;
                    const int ir = fdiv(r2, inv_vpr);
                    const int vv = r2 - ir * vpr;
                    const X* src = xc + (int64_t)c * plane + (rlo + ir) * a.Wf + vv * RV;
                    const int t_r = rlo - row0 + ir;
                    const int tc0 = a.pad_w + vv * RV;
                    const int dsti = a.s_h == 1 ? c * a.chan_pitch + t_r * a.Qs + tc0
                                                : c * a.chan_pitch + (t_r & 1) * 2 * a.sub_pitch + (t_r >> 1) * a.Qs;
                    // all E loads first, then RV word stores.  Lane l writes its columns in the order
                    // (j + l / 4) mod RV: the words of one lane are RV words apart, so without the
                    // rotation every fourth lane would meet on the same LDS banks
                    Vec v[E];
#pragma unroll
                    for (int sm = 0; sm < E; ++sm) {
#pragma unroll
                        for (int j = 0; j < RV; ++j) v[sm].e[j] = X(0);
                        if (bs + sm < a.N) v[sm] = *reinterpret_cast<const Vec*>(src + (int64_t)sm * a.x_sample_stride);
                    }
                    const int rot = (lane >> 2) & (RV - 1);
#pragma unroll
                    for (int j = 0; j < RV; ++j) {
                        const int jj = (j + rot) & (RV - 1);
                        Word w;
#pragma unroll
                        for (int sm = 0; sm < E; ++sm) {
                            X val = v[sm].e[0];
#pragma unroll
                            for (int q = 1; q < RV; ++q) val = jj == q ? v[sm].e[q] : val;
                            w.e[sm] = val;
                        }
                        const int t_c = tc0 + jj;
                        const int dst = a.s_h == 1 ? dsti + jj : dsti + (t_c & 1) * a.sub_pitch + (t_c >> 1);
                        wslab[dst] = w;
                    }
                }
            }
        }
        if constexpr (SI && ROWB == 0) {
            // one word per element of the chunk image: that element of each of the E samples
            // (zero where the image shows padding or the batch has ended)
            staged = true;
            struct alignas(E * sizeof(X)) Word { X e[E]; };
            constexpr int kWords = 2;
            for (int sg = 0; sg < a.SG; ++sg) {
            Word* wslab = reinterpret_cast<Word*>(lds) + sg * img_elems;
            const X* xc = xb + (int64_t)sg * E * a.x_sample_stride + (int64_t)c0 * plane;
            const int bs = b + sg * E;                           // first sample of this group
            for (int e0 = tid; e0 < elems; e0 += kWords * nthreads) {
                Word v[kWords];
#pragma unroll
                for (int u = 0; u < kWords; ++u) {
                    const int e = e0 + u * nthreads;
#pragma unroll
                    for (int sm = 0; sm < E; ++sm) v[u].e[sm] = X(0);
                    if (e < elems) {
                        const int c = fdiv(e, a.inv_chan_pitch);
                        const int o = tab[e - c * a.chan_pitch];
                        if (o >= 0) {
#pragma unroll
                            for (int sm = 0; sm < E; ++sm)
                                if (bs + sm < a.N) v[u].e[sm] = xc[(int64_t)sm * a.x_sample_stride + (int64_t)c * plane + o];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kWords; ++u) {
                    const int e = e0 + u * nthreads;
                    if (e < elems) wslab[e] = v[u];
                }
            }
            }
        }
        if (!staged)
        for (int sm = 0; sm < (MS ? VPT : 1); ++sm) {
        if (MS && b + sm >= a.N) break;
        const X* xc = xb + (int64_t)sm * a.x_sample_stride + (int64_t)c0 * plane;
        X* simg = slab + sm * img_elems;
        if constexpr (FLAT) {
            constexpr int EPV = 16 / (int)sizeof(X);
            const uint4v* src = reinterpret_cast<const uint4v*>(xc);
            uint4v* dst = reinterpret_cast<uint4v*>(simg);
            const int nvec = elems / EPV;                       // elems * sizeof(X) is a multiple of 16
            for (int i0 = tid; i0 < nvec; i0 += kStageLoads * nthreads) {
                uint4v v[kStageLoads];
#pragma unroll
                for (int u = 0; u < kStageLoads; ++u) {
                    const int i = i0 + u * nthreads;
                    if (i < nvec) v[u] = src[i];
                }
#pragma unroll
                for (int u = 0; u < kStageLoads; ++u) {
                    const int i = i0 + u * nthreads;
                    if (i < nvec) dst[i] = v[u];
                }
            }
            continue;
        }
        if constexpr (ROWB > 0) {
            struct alignas(ROWB) Vec { X e[RV]; };
            const int nvec = min(a.CC, a.C - c0) * per_c;
            for (int i0 = tid; i0 < nvec; i0 += kStageLoads * nthreads) {
                Vec v[kStageLoads];
                int dsti[kStageLoads], tc0[kStageLoads];
#pragma unroll
                for (int u = 0; u < kStageLoads; ++u) {
                    const int i = i0 + u * nthreads;
                    if (i < nvec) {
                        const int c = fdiv(i, inv_per_c);
                        const int r2 = i - c * per_c;
                        const int ir = fdiv(r2, inv_vpr);
                        const int vv = r2 - ir * vpr;
                        v[u] = *reinterpret_cast<const Vec*>(xc + (int64_t)c * plane + (rlo + ir) * a.Wf + vv * RV);
                        // unit strides: the row goes to image row t_r behind the left padding;
                        // strides of two: to row t_r / 2 of the phase image of its parity, and its
                        // elements alternate between the two column phases
                        const int t_r = rlo - row0 + ir;
                        tc0[u] = a.pad_w + vv * RV;
                        dsti[u] = a.s_h == 1 ? c * a.chan_pitch + t_r * a.Qs + tc0[u]
                                             : c * a.chan_pitch + (t_r & 1) * 2 * a.sub_pitch + (t_r >> 1) * a.Qs;
                    }
                }
#pragma unroll
                for (int u = 0; u < kStageLoads; ++u) {
                    const int i = i0 + u * nthreads;
                    if (i < nvec) {
#pragma unroll
                        for (int j = 0; j < RV; ++j) {
                            const int t_c = tc0[u] + j;
                            const int dst = a.s_h == 1 ? dsti[u] + j : dsti[u] + (t_c & 1) * a.sub_pitch + (t_c >> 1);
                            simg[dst] = v[u].e[j];
                            if constexpr (E > 1) {
                                if (a.copies > 1) {
#pragma unroll
                                    for (int sh = 1; sh < E; ++sh)
                                        if (dst >= sh)
                                            *reinterpret_cast<X*>(lds + sh * a.copy_bytes + (dst - sh) * (int)sizeof(X)) = v[u].e[j];
                                }
                            }
                        }
                    }
                }
            }
            continue;
        }
        for (int e0 = tid; e0 < elems; e0 += kStageLoads * nthreads) {
            X v[kStageLoads];
#pragma unroll
            for (int u = 0; u < kStageLoads; ++u) {
                const int e = e0 + u * nthreads;
                v[u] = X(0);
                if (e < elems) {
                    const int c = fdiv(e, a.inv_chan_pitch);
                    const int o = tab[e - c * a.chan_pitch];
                    if (o >= 0) v[u] = xc[(int64_t)c * plane + o];
                }
            }
#pragma unroll
            for (int u = 0; u < kStageLoads; ++u) {
                const int e = e0 + u * nthreads;
                if (e < elems) {
                    simg[e] = v[u];
                    if constexpr (E > 1) {
                        // shifted images for the word-aligned packed reads: image s holds element e at e - s
                        if (a.copies > 1) {
#pragma unroll
                            for (int sh = 1; sh < E; ++sh)
                                if (e >= sh) *reinterpret_cast<X*>(lds + sh * a.copy_bytes + (e - sh) * (int)sizeof(X)) = v[u];
                        }
                    }
                }
            }
        }
        }
        // LANES (tuning.wsrc = 3): lane j of the wave holds entry j of the segment being multiplied,
        // loaded by one coalesced vector load and fetched one batch of 64 entries ahead (vector
        // loads have their own counter, so they can be in flight across the gathers), and every
        // entry is broadcast with two v_readlane.  For tables too large for the scalar cache.
        int2 cur2 = make_int2(0, 0);
        if constexpr (LANES) {
            if (nrows > 0) {
                const int si = drow0 * a.nchunks + ch;
                const int s0 = segs[si], len = segs[si + 1] - s0;
                if (lane < len) cur2 = wlc[s0 + lane];
            }
        }
        __syncthreads();                  // chunk staged
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            if (r < nrows) {
                const int si = (drow0 + r) * a.nchunks + ch;
                const int s0 = segs[si], len = segs[si + 1] - s0;     // even
                auto mac = [&](int wbits, int lam) {
                    const WL w = weight_from_bits<DT>(wbits);
                    const unsigned char* pj = lane_base + lam;
#pragma unroll
                    for (int k = 0; k < VPT; ++k) mac_slot<DT, E>(acc[r][k], w, pj + k * koff);
                };
                if constexpr (LANES) {
                    for (int c0 = 0; c0 < len || c0 == 0; c0 += 64) {
                        const int cnt = min(64, len - c0);
                        // next batch: of this segment, or the first of the wave's next row
                        int2 nxt2 = make_int2(0, 0);
                        if (c0 + 64 < len) {
                            if (c0 + 64 + lane < len) nxt2 = wlc[s0 + c0 + 64 + lane];
                        } else if (r + 1 < nrows) {
                            const int sn = segs[si + a.nchunks], lenn = segs[si + a.nchunks + 1] - sn;
                            if (lane < lenn) nxt2 = wlc[sn + lane];
                        }
                        int j = 0;
                        for (; j + 8 <= cnt; j += 8) {
#pragma unroll
                            for (int i = 0; i < 8; ++i)
                                mac(__builtin_amdgcn_readlane(cur2.x, j + i), __builtin_amdgcn_readlane(cur2.y, j + i));
                        }
                        for (; j < cnt; ++j) mac(__builtin_amdgcn_readlane(cur2.x, j), __builtin_amdgcn_readlane(cur2.y, j));
                        cur2 = nxt2;
                    }
                    continue;
                }
                const int2* seg = wlc + s0;
                int e = 0;
                for (; e + 8 <= len; e += 8) {
                    const int16v c = *(c16_t)(seg + e);
#pragma unroll
                    for (int i = 0; i < 8; ++i) mac(c[2 * i], c[2 * i + 1]);
                }
                const int tail = (len - e) >> 1;                      // 0..3 pairs
                if (tail > 0) {
                    const int16v c = *(c16_t)(seg + e);
                    mac(c[0], c[1]); mac(c[2], c[3]);
                    if (tail > 1) { mac(c[4], c[5]); mac(c[6], c[7]); }
                    if (tail > 2) { mac(c[8], c[9]); mac(c[10], c[11]); }
                }
            }
        }
    }
    Y* yd = y + ((int64_t)b * a.D + drow0) * a.y_plane;
    if (a.ksplit > 1) {
        // partial sums of this workgroup's chunks (a loop of its own: the plain stores below keep
        // their registers and schedule)
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            if (r < nrows) {
#pragma unroll
                for (int k = 0; k < VPT; ++k)
#pragma unroll
                    for (int e = 0; e < E; ++e)
                        if (out_off[k][e] >= 0)
                            add_out(yd + (int64_t)(MS ? k : (SI ? lgrp * E + e : 0)) * a.D * a.y_plane + (int64_t)r * a.y_plane + out_off[k][e],
                                    narrow<DT>(acc[r][k][e]));
            }
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        if (r < nrows) {
#pragma unroll
            for (int k = 0; k < VPT; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (out_off[k][e] >= 0)
                        store_out(yd + (int64_t)(MS ? k : (SI ? lgrp * E + e : 0)) * a.D * a.y_plane + (int64_t)r * a.y_plane + out_off[k][e],
                                  narrow<DT>(acc[r][k][e]));
        }
    }
}

template <sc_dtype_t DT, int VPT, bool MS, int E, bool LANES, bool FLAT, int ROWB = 0, int SMODE = 0>
static sc_status_t launch_cc_w(const Plan& p, const SlabArgs& a, const void* x, void* y, int grid,
                               hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = slab_cc_kernel<DT, VPT, MS, E, LANES, FLAT, ROWB, SMODE>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(p.tuning.wg_threads), p.geom.lds_bytes, stream,
                       static_cast<const X*>(x), static_cast<Y*>(y), p.d_wlc, p.d_seg_off, a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

// Bytes per load of the row-run staging this layer, tile and pointer allow (0: stage by table):
// unit strides, a tile as wide as the plane, rows that are a whole number of such loads.
static int row_run_bytes_geom(const Plan& p, const SlabGeom& g, const void* x, bool interleaved)
{
    if (g.tiles_q != 1 || g.TQ != g.Qf || g.ns != 1 || g.fs != 1 || (g.si != 0) != interleaved) return 0;
    if (g.Hf == 1) return 0;                                      // flattened pointwise layers
    if (p.L.stride_h == 1 && p.L.stride_w == 1) {
        if (g.Qs != g.Wf + 2 * p.L.pad_w) return 0;
    } else if (p.L.stride_h == 2 && p.L.stride_w == 2) {
        // both row and both column phases staged, and every input column inside a phase image
        if (g.nsh != 2 || g.nsw != 2 || p.L.pad_w + g.Wf > 2 * g.Qs) return 0;
    } else {
        return 0;
    }
    if (reinterpret_cast<uintptr_t>(x) % 16 != 0) return 0;
    const int row_bytes = g.Wf * p.ex;
    for (int b : {16, 8, 4})
        if (b > p.ex && row_bytes % b == 0) return b;
    return 0;
}
static int row_run_bytes(const Plan& p, const void* x, bool interleaved = false) { return row_run_bytes_geom(p, p.geom, x, interleaved); }
bool slab_rows_stageable(const Plan& p, const SlabGeom& g) { return row_run_bytes_geom(p, g, nullptr, true) >= 8; }

template <sc_dtype_t DT, int VPT, bool MS, int E = 1>
static sc_status_t launch_cc_one(const Plan& p, const SlabArgs& a, const void* x, void* y, int grid,
                                 hipStream_t stream)
{
    if constexpr (E == 1) {
        if (p.tuning.wsrc == 3) return launch_cc_w<DT, VPT, MS, E, true, false>(p, a, x, y, grid, stream);
    }
    if (p.geom.fs > 1) {
        // samples end to end in one packed tile: its own instantiation
        if constexpr (E > 1 && !MS) return launch_cc_w<DT, VPT, MS, E, false, false, 0, 1>(p, a, x, y, grid, stream);
        return SC_ERR_UNSUPPORTED;
    }
    if (p.geom.si) {
        // the same position of E samples in one word: its own instantiation, staged by table or
        // (32-bit activations, rows that are whole 16- or 8-byte loads) by rows
        if constexpr (DT == SC_F32 && E == 4 && !MS) {
            switch (p.geom.srow ? row_run_bytes(p, x, true) : 0) {
                case 16: return launch_cc_w<DT, VPT, MS, E, false, false, 16, 2>(p, a, x, y, grid, stream);
                case 8: return launch_cc_w<DT, VPT, MS, E, false, false, 8, 2>(p, a, x, y, grid, stream);
            }
        }
        if constexpr (E > 1 && !MS) return launch_cc_w<DT, VPT, MS, E, false, false, 0, 2>(p, a, x, y, grid, stream);
        return SC_ERR_UNSUPPORTED;
    }
    {
        // pointwise layer, one tile per plane, chunk images that are whole 16-byte aligned blocks
        // of the input (and, with packed positions, no shifted images): staged as a plain copy
        const SlabGeom& g = p.geom;
        const int64_t chunk_bytes = (int64_t)g.CC * g.chan_pitch * p.ex;
        if (g.fs == 1 && g.Hf == 1 && g.Pf == 1 && g.tiles_q == 1 && g.TQ == g.Wf && g.chan_pitch == g.Wf && chunk_bytes % 16 == 0 &&
            g.copies == 1 && ((int64_t)p.L.C * g.Wf * p.ex) % 16 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0)
            return launch_cc_w<DT, VPT, MS, E, false, true>(p, a, x, y, grid, stream);
    }
    if constexpr (!MS) {
        switch (row_run_bytes(p, x)) {
            case 16: return launch_cc_w<DT, VPT, MS, E, false, false, 16>(p, a, x, y, grid, stream);
            case 8: return launch_cc_w<DT, VPT, MS, E, false, false, 8>(p, a, x, y, grid, stream);
            case 4:
                if constexpr (sizeof(typename Types<DT>::X) < 4)
                    return launch_cc_w<DT, VPT, MS, E, false, false, 4>(p, a, x, y, grid, stream);
                break;
        }
    }
    return launch_cc_w<DT, VPT, MS, E, false, false>(p, a, x, y, grid, stream);
}

template <sc_dtype_t DT>
static sc_status_t launch_cc(const Plan& p, const SlabArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    if (p.geom.ns > 1) {
        switch (p.geom.ns) {
            case 2: return launch_cc_one<DT, 2, true>(p, a, x, y, grid, stream);
            case 3: return launch_cc_one<DT, 3, true>(p, a, x, y, grid, stream);
            case 4: return launch_cc_one<DT, 4, true>(p, a, x, y, grid, stream);
        }
        return SC_ERR_UNSUPPORTED;
    }
    if constexpr (DT == SC_F16 || DT == SC_I8) {
        constexpr int E = 4 / (int)sizeof(typename Types<DT>::X);
        if (p.geom.pack == E) {
            switch (p.geom.vpt) {
                case 1: return launch_cc_one<DT, 1, false, E>(p, a, x, y, grid, stream);
                case 2: return launch_cc_one<DT, 2, false, E>(p, a, x, y, grid, stream);
            }
            if constexpr (E == 2) {
                if (p.geom.vpt == 3) return launch_cc_one<DT, 3, false, E>(p, a, x, y, grid, stream);
                if (p.geom.vpt == 4) return launch_cc_one<DT, 4, false, E>(p, a, x, y, grid, stream);
            }
            return SC_ERR_UNSUPPORTED;
        }
    }
    if constexpr (DT == SC_F32 || DT == SC_F16) {
        constexpr int EW = 16 / (int)sizeof(typename Types<DT>::X);     // 128-bit slots
        if (p.geom.pack == EW) {
            if (p.geom.vpt == 1) return launch_cc_one<DT, 1, false, EW>(p, a, x, y, grid, stream);
            if constexpr (EW == 4) {
                if (p.geom.vpt == 2) return launch_cc_one<DT, 2, false, EW>(p, a, x, y, grid, stream);
            }
            return SC_ERR_UNSUPPORTED;
        }
    }
    if (p.geom.pack != 1) return SC_ERR_UNSUPPORTED;
    switch (p.geom.vpt) {
        case 1: return launch_cc_one<DT, 1, false>(p, a, x, y, grid, stream);
        case 2: return launch_cc_one<DT, 2, false>(p, a, x, y, grid, stream);
        case 3: return launch_cc_one<DT, 3, false>(p, a, x, y, grid, stream);
        case 4: return launch_cc_one<DT, 4, false>(p, a, x, y, grid, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

template <sc_dtype_t DT, int VPT, int RPW, int E = 1>
static sc_status_t launch_chunk_one(const Plan& p, const ChunkArgs& a, const void* x, void* y, hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = slab_chunk_kernel<DT, VPT, RPW, E>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    const int units = a.N * a.tiles * a.ndt;
    const int grid = std::min(units, kNumCU * std::max(1, kMaxLdsBytes / p.geom.lds_bytes));
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(p.tuning.wg_threads), p.geom.lds_bytes, stream,
                       static_cast<const X*>(x), static_cast<Y*>(y), p.d_wlc, p.d_seg_off, a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

template <sc_dtype_t DT, int VPT, int E = 1>
static sc_status_t launch_chunk_rpw(const Plan& p, const ChunkArgs& a, const void* x, void* y, hipStream_t stream)
{
    switch (p.geom.rpw) {
        case 1: return launch_chunk_one<DT, VPT, 1, E>(p, a, x, y, stream);
        case 2: return launch_chunk_one<DT, VPT, 2, E>(p, a, x, y, stream);
        case 3: return launch_chunk_one<DT, VPT, 3, E>(p, a, x, y, stream);
        case 4: return launch_chunk_one<DT, VPT, 4, E>(p, a, x, y, stream);
        case 5: return launch_chunk_one<DT, VPT, 5, E>(p, a, x, y, stream);
        case 6: return launch_chunk_one<DT, VPT, 6, E>(p, a, x, y, stream);
        case 7: return launch_chunk_one<DT, VPT, 7, E>(p, a, x, y, stream);
        case 8: return launch_chunk_one<DT, VPT, 8, E>(p, a, x, y, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

template <sc_dtype_t DT>
static sc_status_t launch_chunk(const Plan& p, const void* x, void* y, int N, hipStream_t stream)
{
    const SlabGeom& g = p.geom;
    ChunkArgs a{};
    a.C = p.L.C; a.D = p.L.D; a.N = N; a.Wf = g.Wf; a.TQ = g.TQ; a.tiles = g.tiles_q;
    a.CC = g.CC; a.nchunks = g.nchunks; a.DTW = g.DTW; a.ndt = g.ndt; a.nprod = p.tuning.producers;
    a.slab_bytes = g.slab_bytes;
    a.dmab = g.dmab;
    a.nbuf = g.nbuf > 2 ? g.nbuf : 2;
    a.inv_tiles = 1.0f / (float)g.tiles_q; a.inv_TQ = 1.0f / (float)g.TQ; a.inv_ndt = 1.0f / (float)g.ndt;
    a.x_sample_stride = (int64_t)p.L.C * g.Wf;
    a.y_plane = (int64_t)g.Qf;
    if ((int64_t)N * g.tiles_q * g.ndt >= (1 << 19)) return SC_ERR_UNSUPPORTED;
    if constexpr (DT == SC_F16 || DT == SC_I8) {
        constexpr int E = 4 / (int)sizeof(typename Types<DT>::X);
        if (g.pack == E) {
            // a lane stores the E results of a word at once: y aligned like such a store
            if (reinterpret_cast<uintptr_t>(y) % (E * sizeof(typename Types<DT>::Y)) != 0) return SC_ERR_UNSUPPORTED;
            const bool sym = p.tuning.pipeline == 2;
            switch (g.vpt) {
                case 1: return sym ? launch_symc_one<DT, 1, E>(p, a, x, y, stream) : launch_chunk_rpw<DT, 1, E>(p, a, x, y, stream);
                case 2: return sym ? launch_symc_one<DT, 2, E>(p, a, x, y, stream) : launch_chunk_rpw<DT, 2, E>(p, a, x, y, stream);
            }
            if constexpr (E == 2) {
                if (g.vpt == 3) return sym ? launch_symc_one<DT, 3, E>(p, a, x, y, stream) : launch_chunk_rpw<DT, 3, E>(p, a, x, y, stream);
                if (g.vpt == 4) return sym ? launch_symc_one<DT, 4, E>(p, a, x, y, stream) : launch_chunk_rpw<DT, 4, E>(p, a, x, y, stream);
            }
            return SC_ERR_UNSUPPORTED;
        }
    }
    if constexpr (DT == SC_F32 || DT == SC_F16) {
        constexpr int EW = 16 / (int)sizeof(typename Types<DT>::X);     // 128-bit slots
        if (g.pack == EW) {
            if (reinterpret_cast<uintptr_t>(y) % 16 != 0) return SC_ERR_UNSUPPORTED;   // 16-byte stores
            const bool sym = p.tuning.pipeline == 2;
            if (g.vpt == 1) return sym ? launch_symc_one<DT, 1, EW>(p, a, x, y, stream) : launch_chunk_rpw<DT, 1, EW>(p, a, x, y, stream);
            if constexpr (EW == 4) {
                if (g.vpt == 2) return sym ? launch_symc_one<DT, 2, EW>(p, a, x, y, stream) : launch_chunk_rpw<DT, 2, EW>(p, a, x, y, stream);
            }
            return SC_ERR_UNSUPPORTED;
        }
    }
    if (g.pack != 1) return SC_ERR_UNSUPPORTED;
    if (p.tuning.pipeline == 2) {
        switch (g.vpt) {
            case 1: return launch_symc_one<DT, 1>(p, a, x, y, stream);
            case 2: return launch_symc_one<DT, 2>(p, a, x, y, stream);
            case 3: return launch_symc_one<DT, 3>(p, a, x, y, stream);
            case 4: return launch_symc_one<DT, 4>(p, a, x, y, stream);
        }
        return SC_ERR_UNSUPPORTED;
    }
    switch (g.vpt) {
        case 1: return launch_chunk_rpw<DT, 1>(p, a, x, y, stream);
        case 2: return launch_chunk_rpw<DT, 2>(p, a, x, y, stream);
        case 3: return launch_chunk_rpw<DT, 3>(p, a, x, y, stream);
        case 4: return launch_chunk_rpw<DT, 4>(p, a, x, y, stream);
        case 5: return launch_chunk_rpw<DT, 5>(p, a, x, y, stream);
        case 6: return launch_chunk_rpw<DT, 6>(p, a, x, y, stream);
        case 7: return launch_chunk_rpw<DT, 7>(p, a, x, y, stream);
        case 8: return launch_chunk_rpw<DT, 8>(p, a, x, y, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

int slab_grid_size(const Plan& p, const SlabGeom& g, int N)
{
    (void)p;
    return N * g.tiles_p * g.tiles_q;
}

sc_status_t expand_weights(const Plan& p, const int32_t* lam_slab, int2* wl32_out, hipStream_t stream)
{
    const int64_t cnt = (int64_t)p.L.D * p.np;
    if (cnt == 0 || !wl32_out) return SC_OK;
    const unsigned blocks = (unsigned)((cnt + 255) / 256);
#define SC_EXPAND(DT)                                                                              \
    hipLaunchKernelGGL(expand_weights_kernel<DT>, dim3(blocks), dim3(256), 0, stream, p.d_theta,   \
                       lam_slab, wl32_out, p.L.D, p.n, p.np)
    switch (p.dtype) {
        case SC_F32: SC_EXPAND(SC_F32); break;
        case SC_F16: SC_EXPAND(SC_F16); break;
        case SC_I8: SC_EXPAND(SC_I8); break;
        default: return SC_ERR_UNSUPPORTED;
    }
#undef SC_EXPAND
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

template <sc_dtype_t DT, int VPT, int WSRC, int E = 1>
static sc_status_t launch_one(const Plan& p, const SlabArgs& a, const void* x, void* y, int grid,
                              hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = slab_kernel<DT, VPT, WSRC, E>;
    // a workgroup may use more than the default 64 KB of LDS: raise the limit once per kernel
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(p.tuning.wg_threads), p.geom.lds_bytes, stream,
                       static_cast<const X*>(x), static_cast<Y*>(y), p.d_theta, p.d_lam_slab, p.d_wl32,
                       p.d_codebook, a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

template <sc_dtype_t DT, int WSRC>
static sc_status_t launch_vpt(const Plan& p, const SlabArgs& a, const void* x, void* y, int grid,
                              hipStream_t stream)
{
    if constexpr ((DT == SC_F32 || DT == SC_F16) && WSRC == 1) {
        // tuning.pack = 2 (pointwise layers): positions packed by the 128-bit word, 16-byte stores
        constexpr int EW = 16 / (int)sizeof(typename Types<DT>::X);
        if (p.geom.pack == EW) {
            if (reinterpret_cast<uintptr_t>(y) % 16 != 0) return SC_ERR_UNSUPPORTED;
            if (p.geom.vpt == 1) return launch_one<DT, 1, WSRC, EW>(p, a, x, y, grid, stream);
            if constexpr (EW == 4) {
                if (p.geom.vpt == 2) return launch_one<DT, 2, WSRC, EW>(p, a, x, y, grid, stream);
            }
            return SC_ERR_UNSUPPORTED;
        }
    }
    if (p.geom.pack != 1) return SC_ERR_UNSUPPORTED;
    switch (p.geom.vpt) {
        case 1: return launch_one<DT, 1, WSRC>(p, a, x, y, grid, stream);
        case 2: return launch_one<DT, 2, WSRC>(p, a, x, y, grid, stream);
        case 3: return launch_one<DT, 3, WSRC>(p, a, x, y, grid, stream);
        case 4: return launch_one<DT, 4, WSRC>(p, a, x, y, grid, stream);
        case 5: return launch_one<DT, 5, WSRC>(p, a, x, y, grid, stream);
        case 6: return launch_one<DT, 6, WSRC>(p, a, x, y, grid, stream);
        case 7: return launch_one<DT, 7, WSRC>(p, a, x, y, grid, stream);
        case 8: return launch_one<DT, 8, WSRC>(p, a, x, y, grid, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

template <sc_dtype_t DT, int VPT, int WSRC, int E = 1>
static sc_status_t launch_async_one(const Plan& p, const SlabArgs& a, const void* x, void* y,
                                    hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = slab_async_kernel<DT, VPT, WSRC, E>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    const int total = a.N * a.tiles_q;
    const int grid = std::min(total, kNumCU * std::max(1, kMaxLdsBytes / p.geom.lds_bytes));
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(p.tuning.wg_threads), p.geom.lds_bytes, stream,
                       static_cast<const X*>(x), static_cast<Y*>(y), p.d_wl32, a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

template <sc_dtype_t DT, int WSRC>
static sc_status_t launch_async_w(const Plan& p, const SlabArgs& a, const void* x, void* y, hipStream_t stream)
{
    if constexpr ((DT == SC_F32 || DT == SC_F16) && WSRC == 1) {
        // tuning.pack = 2: positions packed by the 128-bit word, 16-byte stores
        constexpr int EW = 16 / (int)sizeof(typename Types<DT>::X);
        if (p.geom.pack == EW) {
            if (p.geom.vpt == 1) return launch_async_one<DT, 1, WSRC, EW>(p, a, x, y, stream);
            if constexpr (EW == 4) {
                if (p.geom.vpt == 2) return launch_async_one<DT, 2, WSRC, EW>(p, a, x, y, stream);
            }
            return SC_ERR_UNSUPPORTED;
        }
    }
    if (p.geom.pack != 1) return SC_ERR_UNSUPPORTED;
    if constexpr (DT != SC_F32 && WSRC == 1) {
        // positions packed by the dword: the kernel's count is dwords per lane
        constexpr int E = 4 / (int)sizeof(typename Types<DT>::X);
        switch ((p.geom.TQ + 64 * E - 1) / (64 * E)) {
            case 1: return launch_async_one<DT, 1, WSRC, E>(p, a, x, y, stream);
            case 2: return launch_async_one<DT, 2, WSRC, E>(p, a, x, y, stream);
            case 3: return launch_async_one<DT, 3, WSRC, E>(p, a, x, y, stream);
            case 4: return launch_async_one<DT, 4, WSRC, E>(p, a, x, y, stream);
        }
        return SC_ERR_UNSUPPORTED;
    }
    switch (p.geom.vpt) {
        case 1: return launch_async_one<DT, 1, WSRC>(p, a, x, y, stream);
        case 2: return launch_async_one<DT, 2, WSRC>(p, a, x, y, stream);
        case 3: return launch_async_one<DT, 3, WSRC>(p, a, x, y, stream);
        case 4: return launch_async_one<DT, 4, WSRC>(p, a, x, y, stream);
        case 5: return launch_async_one<DT, 5, WSRC>(p, a, x, y, stream);
        case 6: return launch_async_one<DT, 6, WSRC>(p, a, x, y, stream);
        case 7: return launch_async_one<DT, 7, WSRC>(p, a, x, y, stream);
        case 8: return launch_async_one<DT, 8, WSRC>(p, a, x, y, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

template <sc_dtype_t DT>
static sc_status_t launch_async(const Plan& p, const SlabArgs& a, const void* x, void* y, hipStream_t stream)
{
    if (p.tuning.wsrc == 3) return launch_async_w<DT, 3>(p, a, x, y, stream);
    return p.tuning.wsrc == 2 ? launch_async_w<DT, 2>(p, a, x, y, stream)
                              : launch_async_w<DT, 1>(p, a, x, y, stream);
}

template <sc_dtype_t DT, int VPT>
static sc_status_t launch_sym_one(const Plan& p, const SlabArgs& a, const void* x, void* y, hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    auto kernel = slab_sym_kernel<DT, VPT>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    });
    if (attr_err != hipSuccess) return SC_ERR_HIP;
    const int total = a.N * a.tiles_q;
    const int grid = std::min(total, kNumCU * std::max(1, kMaxLdsBytes / p.geom.lds_bytes));
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(p.tuning.wg_threads), p.geom.lds_bytes, stream,
                       static_cast<const X*>(x), static_cast<Y*>(y), p.d_wl32, a);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

template <sc_dtype_t DT>
static sc_status_t launch_sym(const Plan& p, const SlabArgs& a, const void* x, void* y, hipStream_t stream)
{
    switch (p.geom.vpt) {
        case 1: return launch_sym_one<DT, 1>(p, a, x, y, stream);
        case 2: return launch_sym_one<DT, 2>(p, a, x, y, stream);
        case 3: return launch_sym_one<DT, 3>(p, a, x, y, stream);
        case 4: return launch_sym_one<DT, 4>(p, a, x, y, stream);
        case 5: return launch_sym_one<DT, 5>(p, a, x, y, stream);
        case 6: return launch_sym_one<DT, 6>(p, a, x, y, stream);
        case 7: return launch_sym_one<DT, 7>(p, a, x, y, stream);
        case 8: return launch_sym_one<DT, 8>(p, a, x, y, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

template <sc_dtype_t DT>
static sc_status_t launch_dt(const Plan& p, const SlabArgs& a, const void* x, void* y, int grid,
                             hipStream_t stream)
{
    if constexpr (!kCodebook<DT>) {
        if (p.tuning.pipeline == 2) {
            // as for pipeline 1: an unaligned x takes the one-shot kernel
            if (a.dmab) return launch_sym<DT>(p, a, x, y, stream);
        }
        if (p.tuning.pipeline == 1) {
            // the direct-to-LDS copy needs 16-byte aligned rows: checked at tuning time for the
            // layer, here for the caller's pointer (an unaligned x takes the one-shot kernel)
            if (a.vec) return launch_async<DT>(p, a, x, y, stream);
        }
        if (p.tuning.wsrc == 2) return launch_vpt<DT, 2>(p, a, x, y, grid, stream);
        if (p.tuning.wsrc == 3) return launch_vpt<DT, 3>(p, a, x, y, grid, stream);
    }
    if constexpr (!kCodebook<DT>) {
        if (p.tuning.wsrc == 1) return launch_vpt<DT, 1>(p, a, x, y, grid, stream);
    }
    return launch_vpt<DT, 0>(p, a, x, y, grid, stream);
}

__global__ void __launch_bounds__(256) clear_kernel(uint32_t* __restrict__ dst, int64_t words)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride) dst[i] = 0u;
}

sc_status_t launch_slab(const Plan& p, const void* x, void* y, int N, hipStream_t stream)
{
    const SlabGeom& g = p.geom;
    if (p.tuning.chunk_c > 0 && p.tuning.pipeline >= 1) {
        // direct-to-LDS copies: the caller's pointer must be aligned like the rows
        if (reinterpret_cast<uintptr_t>(x) % (uintptr_t)std::max(g.dmab, 1) != 0) return SC_ERR_UNSUPPORTED;
        switch (p.dtype) {
            case SC_F32: return launch_chunk<SC_F32>(p, x, y, N, stream);
            case SC_F16: return launch_chunk<SC_F16>(p, x, y, N, stream);
            case SC_I8: return launch_chunk<SC_I8>(p, x, y, N, stream);
            default: return SC_ERR_UNSUPPORTED;
        }
    }
    const int64_t grid64 = (int64_t)N * g.tiles_p * g.tiles_q;
    if (grid64 >= (1 << 19)) return SC_ERR_UNSUPPORTED;  // fdiv() range for the tile decode
    SlabArgs a{};
    a.C = p.L.C; a.D = p.L.D; a.n = p.n; a.N = N;
    a.Hf = g.Hf; a.Wf = g.Wf; a.Pf = g.Pf; a.Qf = g.Qf;
    a.s_h = p.L.stride_h; a.s_w = p.L.stride_w; a.pad_h = p.L.pad_h; a.pad_w = p.L.pad_w;
    a.TP = g.TP; a.TQ = g.TQ; a.tiles_p = g.tiles_p; a.tiles_q = g.tiles_q;
    a.nsw = g.nsw; a.Qs = g.Qs; a.sub_pitch = g.sub_pitch; a.chan_pitch = g.chan_pitch; a.F = g.F;
    a.slab_elems = p.L.C * g.chan_pitch;
    a.slab_bytes = g.slab_bytes; a.wcap = g.wcap; a.DS = g.DS; a.JC = g.JC; a.np = p.np; a.nprod = p.tuning.producers;
    // 16-byte staging also needs a 16-byte aligned input pointer
    // (the packed 16- and 8-bit stream also stores 4 / 16 bytes per lane: y aligned like x)
    a.vec = (g.vec && reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0) ? 1 : 0;
    a.dmab = (g.dmab && reinterpret_cast<uintptr_t>(x) % (uintptr_t)g.dmab == 0) ? g.dmab : 0;
    a.inv_chan_pitch = g.inv_chan_pitch; a.inv_sub_pitch = g.inv_sub_pitch; a.inv_Qs = g.inv_Qs;
    a.inv_tiles = 1.0f / (float)(g.tiles_p * g.tiles_q);
    a.inv_tiles_q = 1.0f / (float)g.tiles_q;
    a.x_sample_stride = (int64_t)p.L.C * g.Hf * g.Wf;
    a.y_plane = (int64_t)g.Pf * g.Qf;
    if (p.tuning.chunk_c > 0) {
        a.CC = g.CC; a.nchunks = g.nchunks; a.DTW = g.DTW; a.ndt = g.ndt;
        a.copies = g.copies; a.copy_bytes = g.copy_bytes; a.SR = g.SR; a.FS = g.fs;
        {
            const int64_t plane_bytes = (int64_t)g.Hf * g.Wf * p.ex;
            a.fs_vec = (g.fs > 1 && reinterpret_cast<uintptr_t>(x) % 16 == 0 && (p.L.C * plane_bytes) % 16 == 0 &&
                        (g.CC * plane_bytes) % 16 == 0) ? 1 : 0;
        }
        a.inv_ndt = 1.0f / (float)g.ndt;
        const int per_wg = g.si ? g.pack * std::max(g.sg, 1) : (g.ns > 1 ? g.ns : g.fs);
        a.SG = g.si ? std::max(g.sg, 1) : 1;
        a.ksplit = std::max(g.ksplit, 1);
        a.cps = (g.nchunks + a.ksplit - 1) / a.ksplit;
        a.inv_ksplit = 1.0f / (float)a.ksplit;
        const int64_t gridc = (int64_t)((N + per_wg - 1) / per_wg) * g.tiles_p * g.tiles_q * g.ndt * a.ksplit;
        if (gridc >= (1 << 19)) return SC_ERR_UNSUPPORTED;
        if (a.ksplit > 1) {
            // partial sums are added into y: clear it first (a fill kernel, so that the launch can be
            // captured in a graph)
            const int64_t words = ((int64_t)N * p.L.D * g.Pf * g.Qf * p.ey + 3) / 4;
            if (p.ey != 4) return SC_ERR_UNSUPPORTED;
            hipLaunchKernelGGL(clear_kernel, dim3((unsigned)std::min<int64_t>((words + 1023) / 1024, 4096)), dim3(256), 0, stream,
                               static_cast<uint32_t*>(y), words);
            if (hipGetLastError() != hipSuccess) return SC_ERR_HIP;
        }
        switch (p.dtype) {
            case SC_F32: return launch_cc<SC_F32>(p, a, x, y, (int)gridc, stream);
            case SC_F16: return launch_cc<SC_F16>(p, a, x, y, (int)gridc, stream);
            case SC_I8: return launch_cc<SC_I8>(p, a, x, y, (int)gridc, stream);
            default: return SC_ERR_UNSUPPORTED;
        }
    }
    switch (p.dtype) {
        case SC_F32: return launch_dt<SC_F32>(p, a, x, y, (int)grid64, stream);
        case SC_F16: return launch_dt<SC_F16>(p, a, x, y, (int)grid64, stream);
        case SC_I8: return launch_dt<SC_I8>(p, a, x, y, (int)grid64, stream);
        case SC_CB4_I8: return launch_dt<SC_CB4_I8>(p, a, x, y, (int)grid64, stream);
        case SC_CB4_F16: return launch_dt<SC_CB4_F16>(p, a, x, y, (int)grid64, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

}  // namespace sc
