// Device-side element types and conversions shared by the gather and slab kernels.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparse_conv.h"

namespace sc {

// X: activation storage, Y: output storage, A: accumulator, WL: weight as held in LDS / registers
template <sc_dtype_t DT> struct Types;
template <> struct Types<SC_F32> { using X = float; using Y = float; using A = float; using WL = float; };
template <> struct Types<SC_F16> { using X = __half; using Y = __half; using A = float; using WL = float; };
template <> struct Types<SC_I8> { using X = int8_t; using Y = int32_t; using A = int32_t; using WL = int32_t; };
template <> struct Types<SC_CB4_I8> { using X = int8_t; using Y = int32_t; using A = int32_t; using WL = int32_t; };
template <> struct Types<SC_CB4_F16> { using X = __half; using Y = __half; using A = float; using WL = float; };

template <sc_dtype_t DT> constexpr bool kHalfActs = DT == SC_F16 || DT == SC_CB4_F16;   // f16 in, f32 acc, f16 out
template <sc_dtype_t DT> constexpr bool kCodebook = DT == SC_CB4_I8 || DT == SC_CB4_F16; // weights are 4-bit indices

// Weight i of the flat [D*n] table, widened to the accumulator type.  For the 4-bit codebook
// variant the table holds two indices per byte (even entry in the low nibble) and the value is
// looked up in the 16-entry codebook (i8 or f16 centroids) the workgroup keeps in LDS; bit 31 of
// the entry's offset marks a zero-valued filler of a padded row.
template <sc_dtype_t DT>
__device__ inline typename Types<DT>::WL load_weight(const void* theta, int64_t i, int lam,
                                                     const void* cb_lds)
{
    if constexpr (DT == SC_F32) return static_cast<const float*>(theta)[i];
    else if constexpr (DT == SC_F16) return __half2float(static_cast<const __half*>(theta)[i]);
    else if constexpr (DT == SC_I8) return (int32_t) static_cast<const int8_t*>(theta)[i];
    else {
        const uint8_t byte = static_cast<const uint8_t*>(theta)[i >> 1];
        const int idx = (byte >> ((i & 1) * 4)) & 15;
        if constexpr (DT == SC_CB4_I8) return lam < 0 ? 0 : (int32_t) static_cast<const int8_t*>(cb_lds)[idx];
        else return lam < 0 ? 0.0f : __half2float(static_cast<const __half*>(cb_lds)[idx]);
    }
}

// Bytes of the 16-entry codebook of a clustered variant.
template <sc_dtype_t DT> constexpr int kCodebookBytes = DT == SC_CB4_F16 ? 32 : 16;

template <sc_dtype_t DT> __device__ inline typename Types<DT>::A widen(typename Types<DT>::X v)
{
    if constexpr (kHalfActs<DT>) return __half2float(v);
    else return (typename Types<DT>::A)v;
}

// acc += w * x for one gathered element.  The integer variants multiply 8-bit values: the 24-bit
// multiply-add runs at the full rate, the generic 32-bit integer multiply at a quarter of it.
template <sc_dtype_t DT>
__device__ __forceinline__ void mac1(typename Types<DT>::A& acc, typename Types<DT>::WL w, typename Types<DT>::X x)
{
    if constexpr (DT == SC_I8 || DT == SC_CB4_I8) acc += __mul24(w, (int)x);
    else acc += w * widen<DT>(x);
}

template <sc_dtype_t DT> __device__ inline typename Types<DT>::Y narrow(typename Types<DT>::A v)
{
    if constexpr (kHalfActs<DT>) return __float2half_rn(v);
    else return v;
}

// An input element that the kernel reads once: load it with the non-temporal hint.
__device__ inline float load_in(const float* p) { return __builtin_nontemporal_load(p); }
__device__ inline int8_t load_in(const int8_t* p) { return __builtin_nontemporal_load(p); }
__device__ inline __half load_in(const __half* p)
{
    return __ushort_as_half(__builtin_nontemporal_load(reinterpret_cast<const unsigned short*>(p)));
}

// Output values are written once and never read back by the kernels: store them with the
// non-temporal hint so that they do not displace the input stream from the caches.
__device__ inline void store_out(float* p, float v) { __builtin_nontemporal_store(v, p); }
__device__ inline void store_out(int32_t* p, int32_t v) { __builtin_nontemporal_store(v, p); }
__device__ inline void store_out(uint32_t* p, uint32_t v) { __builtin_nontemporal_store(v, p); }
__device__ inline void store_out(__half* p, __half v)
{
    __builtin_nontemporal_store(__half_as_ushort(v), reinterpret_cast<unsigned short*>(p));
}
// Partial sums of one output from several workgroups meet in memory: hardware atomic adds (the
// floating-point one returns nothing and rounds once per add: the order of the adds is the order in
// which the workgroups arrive, so fp32 results of such a launch shape can differ in the last bits
// from run to run; integer sums cannot).
__device__ inline void add_out(float* p, float v) { unsafeAtomicAdd(p, v); }
__device__ inline void add_out(int32_t* p, int32_t v) { atomicAdd(p, v); }
__device__ inline void add_out(__half*, __half) {}      // (never selected: refused at tuning time)
__device__ inline void store_out4(int32_t* p, int32_t a, int32_t b, int32_t c, int32_t d)
{
    typedef int int4v __attribute__((ext_vector_type(4)));
    int4v v = {a, b, c, d};
    __builtin_nontemporal_store(v, reinterpret_cast<int4v*>(p));
}

}  // namespace sc
