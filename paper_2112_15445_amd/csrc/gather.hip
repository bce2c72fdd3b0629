// GATHER variant: the launch shape of the paper's Algorithm 3, written for 64-wide wavefronts.
//
// One workgroup computes one output channel d for a tile of output pixels and SB consecutive
// samples (the paper's sub-batch sb_S, so the grid has pixel_tiles * D * ceil(N / SB) workgroups,
// the analogue of N_B = b_S * D / sb_S).  The (theta, lambda) row of channel d is staged in LDS in
// chunks; each thread owns one output pixel, keeps one accumulator per sample in registers, reads
// every (theta, lambda) pair once from LDS and reuses it for the SB samples, and gathers the input
// straight from global memory at  sample_base + p*s_h*Wp + q*s_w + lambda.  The input it reads is
// the physically zero-padded tensor: when the layer has padding, a small pre-pass writes it into
// the caller's workspace first (the paper feeds its kernel pre-padded inputs).
#include "sc_device.h"
#include "sc_internal.h"

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

template <sc_dtype_t DT, int SB>
__global__ void __launch_bounds__(256)
gather_kernel(const typename Types<DT>::X* __restrict__ xp, const void* __restrict__ theta,
              const int32_t* __restrict__ lam, const int8_t* __restrict__ codebook,
              typename Types<DT>::Y* __restrict__ y, int N, int D, int n, int P, int Q, int s_h,
              int s_w, int Wp, int64_t X_size)
{
    using A = typename Types<DT>::A;
    using WL = typename Types<DT>::WL;
    __shared__ WL theta_s[kRowChunk];
    __shared__ int32_t lam_s[kRowChunk];
    __shared__ int8_t cb_s[16];

    const int d = blockIdx.y;
    const int b0 = blockIdx.z * SB;
    const int pix = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = pix < P * Q;
    const int p = live ? pix / Q : 0;
    const int q = live ? pix - p * Q : 0;
    const int base = p * s_h * Wp + q * s_w;

    if constexpr (DT == SC_CB4_I8) {
        if (threadIdx.x < 16) cb_s[threadIdx.x] = codebook[threadIdx.x];
    }
    A acc[SB];
#pragma unroll
    for (int t = 0; t < SB; ++t) acc[t] = A(0);
    // samples past the end of the batch re-read the last one; their results are not stored
    const typename Types<DT>::X* xs[SB];
#pragma unroll
    for (int t = 0; t < SB; ++t) xs[t] = xp + (int64_t)min(b0 + t, N - 1) * X_size + base;

    for (int j0 = 0; j0 < n; j0 += kRowChunk) {
        const int jc = min(kRowChunk, n - j0);
        __syncthreads();
        for (int j = threadIdx.x; j < jc; j += blockDim.x) {
            const int64_t i = (int64_t)d * n + j0 + j;
            const int l = lam[i];
            theta_s[j] = load_weight<DT>(theta, i, l, cb_s);
            lam_s[j] = l & 0x7fffffff;
        }
        __syncthreads();
        for (int j = 0; j < jc; ++j) {
            const WL w = theta_s[j];
            const int l = lam_s[j];
#pragma unroll
            for (int t = 0; t < SB; ++t) acc[t] += w * widen<DT>(xs[t][l]);
        }
    }
    if (!live) return;
#pragma unroll
    for (int t = 0; t < SB; ++t)
        if (b0 + t < N) y[((int64_t)(b0 + t) * D + d) * ((int64_t)P * Q) + pix] = narrow<DT>(acc[t]);
}

size_t gather_workspace_bytes(const Plan& p, int N)
{
    if (p.L.pad_h == 0 && p.L.pad_w == 0) return 0;
    return (size_t)N * (size_t)p.X_size * (size_t)p.ex;
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
    const int threads = 256;
    const int pix = p.P * p.Q;
    const int sb = p.tuning.sub_batch;
    dim3 grid((pix + threads - 1) / threads, p.L.D, (N + sb - 1) / sb);
    if (grid.y > 65535 || grid.z > 65535) return SC_ERR_UNSUPPORTED;
#define SC_GATHER_LAUNCH(SB)                                                                       \
    hipLaunchKernelGGL((gather_kernel<DT, SB>), grid, dim3(threads), 0, stream, xp, p.d_theta,    \
                       p.d_lam, p.d_codebook, static_cast<Y*>(y), N, p.L.D, p.n, p.P, p.Q,        \
                       p.L.stride_h, p.L.stride_w, p.Wp, p.X_size)
    switch (sb) {
        case 1: SC_GATHER_LAUNCH(1); break;
        case 2: SC_GATHER_LAUNCH(2); break;
        case 4: SC_GATHER_LAUNCH(4); break;
        case 8: SC_GATHER_LAUNCH(8); break;
        default: return SC_ERR_UNSUPPORTED;
    }
#undef SC_GATHER_LAUNCH
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
    }
    return SC_ERR_UNSUPPORTED;
}

}  // namespace sc
