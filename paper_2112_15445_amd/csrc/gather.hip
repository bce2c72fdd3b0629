// GATHER variant: the launch shape of the paper's Algorithm 3, written for 64-wide wavefronts.
//
// One workgroup computes one output channel d for a tile of output positions.  The (theta, lambda)
// row of channel d is staged in LDS in chunks; each thread keeps its accumulators in registers,
// reads every (theta, lambda) pair once from LDS, reuses it for its sub_batch output positions
// (the role the paper's sub-batch sb_S plays: shared-memory reads are amortised over several
// outputs, and the grid shrinks to D * positions / (threads * sub_batch) workgroups, the analogue
// of N_B = b_S * D / sb_S), and gathers the input straight from global memory at
// sample_base + p*s_h*Wp + q*s_w + lambda.  The input it reads is the physically zero-padded
// tensor: when the layer has padding, a small pre-pass writes it into the caller's workspace first
// (the paper feeds its kernel pre-padded inputs).
#include <mutex>
#include <type_traits>

#include "sc_device.h"
#include "sc_internal.h"

// Scratch memory of sparse_conv_forward_static: the padded copy of the input that this variant
// materialises when the layer has padding.  One array per GPU (the code object is loaded on each),
// held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress;
// the address kernels and copies use is the one that call returns.
static __device__ __align__(256) unsigned char scratch[SC_STATIC_WORKSPACE_BYTES];

namespace sc {

constexpr int kRowChunk = 1024;  // (theta, lambda) pairs staged per pass

template <typename T>
__global__ void __launch_bounds__(256)
pad_input_kernel(const T* __restrict__ x, T* __restrict__ xp, int64_t total, int H, int W, int Hp,
                 int Wp, int ph, int pw)
{
    // one thread per element of the padded tensor [N*C][Hp][Wp]
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t plane = i / ((int64_t)Hp * Wp);
        const int rem = (int)(i - plane * ((int64_t)Hp * Wp));
        const int hp = rem / Wp, wp = rem - hp * Wp;
        const int h = hp - ph, w = wp - pw;
        T v = T(0);
        if (h >= 0 && h < H && w >= 0 && w < W) v = x[(plane * H + h) * W + w];
        xp[i] = v;
    }
}

// One workgroup = one output channel d (blockIdx.y) x a tile of output positions.  Positions are
// numbered flat over (sample, p, q), so layers with tiny output planes still fill every lane when
// the batch is large.  The 256 threads are laid out as (256 / NSPLIT) position slots x NSPLIT entry
// slices: a thread owns VPT positions (slot, slot + 256/NSPLIT, ...) and, when NSPLIT > 1, only the
// stored entries j = slice (mod NSPLIT); the NSPLIT partial sums of one output sit in adjacent
// lanes and are combined with a butterfly of cross-lane shuffles (wavefront-level reduction), which
// is what keeps the lanes busy when there are fewer output positions than lanes.
template <sc_dtype_t DT, int VPT, int NSPLIT>
__global__ void __launch_bounds__(256)
gather_kernel(const typename Types<DT>::X* __restrict__ xp, const void* __restrict__ theta,
              const int32_t* __restrict__ lam, const void* __restrict__ codebook,
              typename Types<DT>::Y* __restrict__ y, int64_t total_pos, int D, int n, int PQ, int Q,
              int s_h, int s_w, int Wp, int64_t X_size)
{
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    __shared__ WL theta_s[kRowChunk];
    __shared__ int32_t lam_s[kRowChunk];
    __shared__ __attribute__((aligned(4))) unsigned char cb_s[32];
    constexpr int SLOTS = 256 / NSPLIT;

    const int d = blockIdx.y;
    const int slice = threadIdx.x % NSPLIT;
    const int slot = threadIdx.x / NSPLIT;
    const int64_t g0 = (int64_t)blockIdx.x * (SLOTS * VPT) + slot;

    if constexpr (kCodebook<DT>) {
        if (threadIdx.x < kCodebookBytes<DT>) cb_s[threadIdx.x] = static_cast<const unsigned char*>(codebook)[threadIdx.x];
    }
    // positions past the end re-read position 0; their results are not stored
    const typename Types<DT>::X* xs[VPT];
    int64_t yoff[VPT];
    A acc[VPT];
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const int64_t g = g0 + (int64_t)k * SLOTS;
        const bool live = g < total_pos;
        const int64_t gc = live ? g : 0;
        const int64_t b = gc / PQ;
        const int f = (int)(gc - b * PQ);
        const int p = f / Q, q = f - p * Q;
        xs[k] = xp + b * X_size + (int64_t)p * s_h * Wp + q * s_w;
        yoff[k] = live ? (b * D + d) * (int64_t)PQ + f : -1;
        acc[k] = A(0);
    }

    for (int j0 = 0; j0 < n; j0 += kRowChunk) {
        const int jc = min(kRowChunk, n - j0);
        __syncthreads();
        for (int j = threadIdx.x; j < jc; j += 256) {
            const int64_t i = (int64_t)d * n + j0 + j;
            const int l = lam[i];
            theta_s[j] = load_weight<DT>(theta, i, l, cb_s);
            lam_s[j] = l & 0x7fffffff;
        }
        __syncthreads();
#pragma unroll 4
        for (int j = slice; j < jc; j += NSPLIT) {
            const WL w = theta_s[j];
            const int l = lam_s[j];
#pragma unroll
            for (int k = 0; k < VPT; ++k) mac1<DT>(acc[k], w, xs[k][l]);
        }
    }
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        A v = acc[k];
#pragma unroll
        for (int m = NSPLIT / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
        if (slice == 0 && yoff[k] >= 0) store_out(y + yoff[k], narrow<DT>(v));
    }
}

// The same gather with the layer's fused epilogue (ReLU, 2 x 2 max-pooling, requantisation): a thread
// owns one element of y -- with pooling the four convolution outputs of its window, accumulated
// side by side from the same (theta, lambda) reads -- and applies max / ReLU / the requantisation
// multiplier of its channel before the one store.
template <sc_dtype_t DT, bool POOL>
__global__ void __launch_bounds__(256)
gather_epi_kernel(const typename Types<DT>::X* __restrict__ xp, const void* __restrict__ theta,
                  const int32_t* __restrict__ lam, const void* __restrict__ codebook, void* __restrict__ y,
                  int64_t total_out, int D, int n, int Po, int Qo, int s_h, int s_w, int Wp, int64_t X_size,
                  int relu, const float* __restrict__ requant)
{
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    using Y = typename Types<DT>::Y;
    __shared__ WL theta_s[kRowChunk];
    __shared__ int32_t lam_s[kRowChunk];
    __shared__ __attribute__((aligned(4))) unsigned char cb_s[32];
    constexpr int NWIN = POOL ? 4 : 1;
    const int d = blockIdx.y;
    if constexpr (kCodebook<DT>) {
        if (threadIdx.x < kCodebookBytes<DT>) cb_s[threadIdx.x] = static_cast<const unsigned char*>(codebook)[threadIdx.x];
    }
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = g < total_out;
    const int64_t gc = live ? g : 0;                  // (past the end: element 0 again, not stored)
    const int PQo = Po * Qo;
    const int64_t b = gc / PQo;
    const int f = (int)(gc - b * PQo);
    const int pp = f / Qo, qq = f - pp * Qo;
    const typename Types<DT>::X* xs[NWIN];
    A acc[NWIN];
#pragma unroll
    for (int w = 0; w < NWIN; ++w) {
        const int p = POOL ? 2 * pp + (w >> 1) : pp, q = POOL ? 2 * qq + (w & 1) : qq;
        xs[w] = xp + b * X_size + (int64_t)p * s_h * Wp + q * s_w;
        acc[w] = A(0);
    }
    for (int j0 = 0; j0 < n; j0 += kRowChunk) {
        const int jc = min(kRowChunk, n - j0);
        __syncthreads();
        for (int j = threadIdx.x; j < jc; j += 256) {
            const int64_t i = (int64_t)d * n + j0 + j;
            const int l = lam[i];
            theta_s[j] = load_weight<DT>(theta, i, l, cb_s);
            lam_s[j] = l & 0x7fffffff;
        }
        __syncthreads();
#pragma unroll 4
        for (int j = 0; j < jc; ++j) {
            const WL wgt = theta_s[j];
            const int l = lam_s[j];
#pragma unroll
            for (int w = 0; w < NWIN; ++w) mac1<DT>(acc[w], wgt, xs[w][l]);
        }
    }
    A v = acc[0];
    if constexpr (POOL) v = max(max(acc[0], acc[1]), max(acc[2], acc[3]));
    if (relu) v = max(v, A(0));
    if (!live) return;
    const int64_t off = (b * D + d) * (int64_t)PQo + f;
    if constexpr (std::is_same<A, int32_t>::value) {
        if (requant) {
            const float r = rintf(__int2float_rn(v) * requant[d]);
            static_cast<int8_t*>(y)[off] = (int8_t)(int)fminf(fmaxf(r, -127.0f), 127.0f);
            return;
        }
    }
    store_out(static_cast<Y*>(y) + off, narrow<DT>(v));
}

size_t gather_workspace_bytes(const Plan& p, int N)
{
    if (p.L.pad_h == 0 && p.L.pad_w == 0) return 0;
    return (size_t)N * (size_t)p.X_size * (size_t)p.ex;
}

int gather_grid_size(const Plan& p, const sc_tuning_t& t, int N)
{
    const int64_t total = (int64_t)N * p.P * p.Q;
    const int per_wg = (256 / t.split_n) * t.sub_batch;
    return (int)((total + per_wg - 1) / per_wg) * p.L.D;
}

template <sc_dtype_t DT, int VPT>
static void launch_gather_split(const Plan& p, dim3 grid, hipStream_t stream,
                                const typename Types<DT>::X* xp, typename Types<DT>::Y* y, int64_t total)
{
#define SC_GATHER_LAUNCH(NS)                                                                      \
    hipLaunchKernelGGL((gather_kernel<DT, VPT, NS>), grid, dim3(256), 0, stream, xp, p.d_theta,   \
                       p.d_lam, p.d_codebook, y, total, p.L.D, p.n, p.P * p.Q, p.Q, p.L.stride_h, \
                       p.L.stride_w, p.Wp, p.X_size)
    switch (p.tuning.split_n) {
        case 1: SC_GATHER_LAUNCH(1); break;
        case 4: SC_GATHER_LAUNCH(4); break;
        case 16: SC_GATHER_LAUNCH(16); break;
        case 64: SC_GATHER_LAUNCH(64); break;
        default: break;
    }
#undef SC_GATHER_LAUNCH
}

template <sc_dtype_t DT>
static sc_status_t launch_gather_t(const Plan& p, const void* x, void* y, int N, void* ws,
                                   hipStream_t stream)
{
    using X = typename Types<DT>::X;
    using Y = typename Types<DT>::Y;
    const X* xp = static_cast<const X*>(x);
    if (p.L.pad_h || p.L.pad_w) {
        const int64_t total = (int64_t)N * p.X_size;
        const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 1 << 20);
        hipLaunchKernelGGL(pad_input_kernel<X>, dim3(blocks), dim3(256), 0, stream, xp,
                           static_cast<X*>(ws), total, p.L.H, p.L.W, p.Hp, p.Wp, p.L.pad_h, p.L.pad_w);
        xp = static_cast<const X*>(ws);
    }
    if (has_epilogue(p)) {
        if (p.tuning.split_n != 1) return SC_ERR_UNSUPPORTED;
        const int64_t total_out = (int64_t)N * p.Po * p.Qo;
        const int64_t gx = (total_out + 255) / 256;
        if (gx >= (1ll << 31) || p.L.D > 65535) return SC_ERR_UNSUPPORTED;
        dim3 grid((unsigned)gx, p.L.D, 1);
        if (p.epi.pool)
            hipLaunchKernelGGL((gather_epi_kernel<DT, true>), grid, dim3(256), 0, stream, xp, p.d_theta, p.d_lam, p.d_codebook, y,
                               total_out, p.L.D, p.n, p.Po, p.Qo, p.L.stride_h, p.L.stride_w, p.Wp, p.X_size, p.epi.relu,
                               p.epi.requant ? p.d_requant : nullptr);
        else
            hipLaunchKernelGGL((gather_epi_kernel<DT, false>), grid, dim3(256), 0, stream, xp, p.d_theta, p.d_lam, p.d_codebook, y,
                               total_out, p.L.D, p.n, p.Po, p.Qo, p.L.stride_h, p.L.stride_w, p.Wp, p.X_size, p.epi.relu,
                               p.epi.requant ? p.d_requant : nullptr);
        return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
    }
    const int64_t total = (int64_t)N * p.P * p.Q;
    const int vpt = p.tuning.sub_batch, ns = p.tuning.split_n;
    if (ns != 1 && ns != 4 && ns != 16 && ns != 64) return SC_ERR_UNSUPPORTED;
    const int per_wg = (256 / ns) * vpt;
    const int64_t gx = (total + per_wg - 1) / per_wg;
    if (gx >= (1ll << 31) || p.L.D > 65535) return SC_ERR_UNSUPPORTED;
    dim3 grid((unsigned)gx, p.L.D, 1);
    switch (vpt) {
        case 1: launch_gather_split<DT, 1>(p, grid, stream, xp, static_cast<Y*>(y), total); break;
        case 2: launch_gather_split<DT, 2>(p, grid, stream, xp, static_cast<Y*>(y), total); break;
        case 4: launch_gather_split<DT, 4>(p, grid, stream, xp, static_cast<Y*>(y), total); break;
        case 8: launch_gather_split<DT, 8>(p, grid, stream, xp, static_cast<Y*>(y), total); break;
        default: return SC_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_HIP;
}

sc_status_t launch_gather(const Plan& p, const void* x, void* y, int N, void* ws, size_t ws_bytes,
                          hipStream_t stream)
{
    const size_t need = gather_workspace_bytes(p, N);
    if (need && (!ws || ws_bytes < need)) return SC_ERR_WORKSPACE;
    switch (p.dtype) {
        case SC_F32: return launch_gather_t<SC_F32>(p, x, y, N, ws, stream);
        case SC_F16: return launch_gather_t<SC_F16>(p, x, y, N, ws, stream);
        case SC_I8: return launch_gather_t<SC_I8>(p, x, y, N, ws, stream);
        case SC_CB4_I8: return launch_gather_t<SC_CB4_I8>(p, x, y, N, ws, stream);
        case SC_CB4_F16: return launch_gather_t<SC_CB4_F16>(p, x, y, N, ws, stream);
    }
    return SC_ERR_UNSUPPORTED;
}

}  // namespace sc

// ------------------------------------------------------------------------------------------------
// Entry point that allocates nothing and takes no workspace: the padded input copy lives in the
// file-scope scratch array above.
// ------------------------------------------------------------------------------------------------
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on every GPU seen so far

// Address of this GPU's copy of the scratch array, resolved once per device with that device current.
sc_status_t scratch_address(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SC_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SC_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SC_OK;
}
}  // namespace

extern "C" sc_status_t sparse_conv_forward_static(const sparse_conv_plan_t* plan, const void* x_dev,
                                                  void* y_dev, int32_t N, void* stream)
{
    if (!plan || !x_dev || !y_dev) return SC_ERR_NULL;
    if (N <= 0) return SC_ERR_SHAPE;
    const sc::Plan* p = reinterpret_cast<const sc::Plan*>(plan);
    if (p->path == SC_PATH_LIBRARY) return SC_ERR_UNSUPPORTED;      // the dense library brings its own workspace needs
    if (p->tuning.variant == SC_VARIANT_SLAB) return sc::launch_slab(*p, x_dev, y_dev, N, (hipStream_t)stream);
    if (p->tuning.variant == SC_VARIANT_DENSE) return sc::launch_mfma(*p, x_dev, y_dev, N, (hipStream_t)stream);
    const size_t need = sc::gather_workspace_bytes(*p, N);
    if (need > (size_t)SC_STATIC_WORKSPACE_BYTES) return SC_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need) {
        const sc_status_t st = scratch_address(&ws);
        if (st != SC_OK) return st;
    }
    // every byte of the padded copy (zeros included) is rewritten by the pad pass of this call, so
    // what an earlier call left in the array never shows
    return sc::launch_gather(*p, x_dev, y_dev, N, ws, need, (hipStream_t)stream);
}
