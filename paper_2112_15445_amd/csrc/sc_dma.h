// Direct-to-LDS tile copies (global_load_lds of gfx950) shared by the kernels whose LDS image of a
// tile is the tile as it lies in memory: the persistent pointwise gather kernels and the
// natural-layout form of the matrix-core tile.
#pragma once

#include <cstdint>

#include "sc_device.h"

namespace sc {

// floor(e / d) for 0 <= e < 2^19 given inv = 1.0f / d (exact: the half-integer bias keeps the
// product at least 1/(2d) away from every integer, well above the two float roundings)
__device__ inline int fdiv(int e, float inv) { return (int)(((float)e + 0.5f) * inv); }

// ------------------------------------------------------------------------------------------------
// Producer-side tile copy, global -> LDS, with the direct-to-LDS loads of gfx950 (16 bytes per lane,
// 1 KB per instruction, no VGPR staging; 4 bytes per lane for rows that are not 16-byte aligned).  Copies nch channel rows of TQ elements (global row pitch
// Wf elements, tb = address of channel 0 / column q0 of the tile, wave-uniform) to the flat
// [channel][TQ] image at dst; the instructions are dealt round-robin to the nprod producer waves.
// When one instruction covers whole channel rows (or a row is a whole number of instructions), a
// lane's byte offset from the instruction's base address never changes, so the base is advanced
// with scalar arithmetic and the loop body holds no vector ALU work at all; other tile widths take
// the generic incremental path.  Lanes whose pixels lie past the end of the plane load nothing.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// (All copies carry the non-temporal hint: the input is streamed once, and keeping it out of the
// caches is worth 10 % of the kernel time on the HBM-bound layers.)
// One copy instruction: BYTES (16 or 4) per lane from base + lane_off (base wave-uniform) to the
// LDS image at dst + BYTES * lane.  HAND = true issues it as inline assembly, which keeps it out of
// the compiler's bookkeeping: a wave that both copies tile i+1 and reads tile i would otherwise be
// made to wait for the copy before its first LDS read.  The caller then waits on vmcnt itself.
template <bool HAND, int BYTES>
__device__ __forceinline__ void dma16(const char* base, uint32_t lane_off, unsigned char* dst)
{
    static_assert(BYTES == 16 || BYTES == 4, "copy width");
    if constexpr (HAND) {
        // (M0 carries the LDS address of the copy; the compiler reserves that register for its own
        // use, so its value is put back before the statement ends)
        const uint32_t l = (uint32_t)(uintptr_t)(lptr_t)dst;
        uint32_t keep;
        if constexpr (BYTES == 16)
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt\n\ts_mov_b32 m0, %0"
                         : "=&s"(keep) : "v"(lane_off), "s"(base), "s"(l) : "memory");
        else
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2 nt\n\ts_mov_b32 m0, %0"
                         : "=&s"(keep) : "v"(lane_off), "s"(base), "s"(l) : "memory");
    } else {
        if constexpr (BYTES == 16) __builtin_amdgcn_global_load_lds((gptr_t)(base + lane_off), (lptr_t)dst, 16, 0, 2);
        else __builtin_amdgcn_global_load_lds((gptr_t)(base + lane_off), (lptr_t)dst, 4, 0, 2);
    }
}
template <bool HAND, int BYTES>
__device__ __forceinline__ void dma16_ptr(const void* src, unsigned char* dst)
{
    if constexpr (HAND) {
        const uint32_t l = (uint32_t)(uintptr_t)(lptr_t)dst;
        uint32_t keep;
        if constexpr (BYTES == 16)
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt\n\ts_mov_b32 m0, %0"
                         : "=&s"(keep) : "v"(src), "s"(l) : "memory");
        else
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %1, off nt\n\ts_mov_b32 m0, %0"
                         : "=&s"(keep) : "v"(src), "s"(l) : "memory");
    } else {
        if constexpr (BYTES == 16) __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 16, 0, 2);
        else __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 4, 0, 2);
    }
}

template <typename X, bool HAND = false, int BYTES = 16>
__device__ __forceinline__ void
dma_tile(const X* tb, unsigned char* dst, int nch, int TQ, int Wf, int q0, int pw, int nprod, int lane,
         float inv_TQ)
{
    constexpr int EPV = BYTES / (int)sizeof(X);
    constexpr int EW = 64 * EPV;                          // elements per copy instruction
    constexpr int IB = 64 * BYTES;                        // bytes per copy instruction
    const int e = lane * EPV;
    if ((TQ & (TQ - 1)) == 0 && TQ <= EW) {
        // one instruction = cpi whole channel rows
        const int sh = __builtin_ctz(TQ);
        const int cpi = EW >> sh;
        const int c_sub = e >> sh;
        const int col = e - (c_sub << sh);
        const uint32_t lane_off = (uint32_t)(c_sub * Wf + col) * (uint32_t)sizeof(X);
        const int nfull = nch >> __builtin_ctz(cpi);
        const int64_t gstride = (int64_t)cpi * Wf * (int64_t)sizeof(X);
        const char* base = reinterpret_cast<const char*>(tb);
        if (q0 + col < Wf) {
            int g = pw;
            for (; g < nfull; g += nprod) dma16<HAND, BYTES>(base + g * gstride, lane_off, dst + g * IB);
            // a last, partial group of channel rows falls to the wave whose turn it is
            if (g == nfull && c_sub < nch - nfull * cpi)
                dma16<HAND, BYTES>(base + nfull * gstride, lane_off, dst + nfull * IB);
        }
        return;
    }
    if (TQ % EW == 0) {
        // one channel row = ipc whole instructions
        const int ipc = TQ / EW;
        const int64_t cstride = (int64_t)Wf * (int64_t)sizeof(X);
        for (int seg = 0; seg < ipc; ++seg) {
            if (q0 + seg * EW + e < Wf) {
                const char* base = reinterpret_cast<const char*>(tb + seg * EW);
                for (int c = pw; c < nch; c += nprod)
                    dma16<HAND, BYTES>(base + c * cstride, (uint32_t)(e * (int)sizeof(X)), dst + (c * ipc + seg) * IB);
            }
        }
        return;
    }
    if (TQ % EPV == 0 && 2 * TQ > EW) {
        // one channel row = ipc instructions, the last of them partly filled (its lanes past the
        // end of the row copy nothing): a constant lane offset again, the base advances by rows
        const int ipc = (TQ + EW - 1) / EW;
        const int64_t cstride = (int64_t)Wf * (int64_t)sizeof(X);
        for (int seg = 0; seg < ipc; ++seg) {
            const int col = seg * EW + e;
            if (col < TQ && q0 + col < Wf) {
                const char* base = reinterpret_cast<const char*>(tb + seg * EW);
                for (int c = pw; c < nch; c += nprod)
                    dma16<HAND, BYTES>(base + c * cstride, (uint32_t)(e * (int)sizeof(X)), dst + (c * TQ + seg * EW) * (int)sizeof(X));
            }
        }
        return;
    }
    // generic: the (channel, column) of a lane's bytes advances by a fixed step from one
    // instruction to the next, so the division is done once and the rest is increments
    const int E = nch * TQ;
    const int stepE = EW * nprod;
    const int qstep = stepE / TQ, rstep = stepE - qstep * TQ;
    int idx = pw * EW + e;
    int c = fdiv(idx, inv_TQ);
    int col = idx - c * TQ;
    const X* src = tb + (int64_t)c * Wf + col;
    for (int i = pw; i * EW < E; i += nprod) {
        if (idx < E && q0 + col < Wf) dma16_ptr<HAND, BYTES>(src, dst + i * IB);
        idx += stepE;
        col += rstep;
        src += (int64_t)qstep * Wf + rstep;
        if (col >= TQ) {
            col -= TQ;
            src += Wf - TQ;
        }
    }
}

}  // namespace sc
