// The dense library as the third contender of the per-layer dispatch (steps 3 and 4 of the paper's
// "Main scheme": compare the sparse layer with the dense library's convolution, then configure the
// network layer by layer).  MIOpen is not linked: it is looked up at run time -- first among the
// libraries already in the process (an application that holds device memory through a framework
// has one loaded), then by name -- so the library loads and works without it, and the dispatch then
// simply has no such leg.  32- and 16-bit floating-point layers only.
#include <dlfcn.h>

#include <mutex>
#include <new>

#include <miopen/miopen.h>

#include "sc_device.h"
#include "sc_internal.h"

namespace sc {

namespace {
struct Api {
    void* so = nullptr;
    bool tried = false;
    decltype(&miopenCreateWithStream) CreateWithStream = nullptr;
    decltype(&miopenDestroy) Destroy = nullptr;
    decltype(&miopenSetStream) SetStream = nullptr;
    decltype(&miopenCreateTensorDescriptor) CreateTensorDescriptor = nullptr;
    decltype(&miopenSet4dTensorDescriptor) Set4dTensorDescriptor = nullptr;
    decltype(&miopenDestroyTensorDescriptor) DestroyTensorDescriptor = nullptr;
    decltype(&miopenCreateConvolutionDescriptor) CreateConvolutionDescriptor = nullptr;
    decltype(&miopenInitConvolutionDescriptor) InitConvolutionDescriptor = nullptr;
    decltype(&miopenDestroyConvolutionDescriptor) DestroyConvolutionDescriptor = nullptr;
    decltype(&miopenConvolutionForwardGetWorkSpaceSize) ConvolutionForwardGetWorkSpaceSize = nullptr;
    decltype(&miopenFindConvolutionForwardAlgorithm) FindConvolutionForwardAlgorithm = nullptr;
    decltype(&miopenConvolutionForward) ConvolutionForward = nullptr;
};
Api g_api;
std::mutex g_api_mutex;

bool load_api()
{
    std::lock_guard<std::mutex> lock(g_api_mutex);
    if (g_api.tried) return g_api.so != nullptr;
    g_api.tried = true;
    void* so = nullptr;
    for (const char* name : {"libMIOpen.so", "libMIOpen.so.1"})
        if (!so) so = dlopen(name, RTLD_NOW | RTLD_NOLOAD);           // the copy already in the process
    for (const char* name : {"libMIOpen.so.1", "libMIOpen.so", "/opt/rocm/lib/libMIOpen.so.1"})
        if (!so) so = dlopen(name, RTLD_NOW | RTLD_LOCAL);
    if (!so) return false;
    bool ok = true;
#define SC_SYM(field, sym) ok = ok && (g_api.field = reinterpret_cast<decltype(g_api.field)>(dlsym(so, #sym))) != nullptr
    SC_SYM(CreateWithStream, miopenCreateWithStream);
    SC_SYM(Destroy, miopenDestroy);
    SC_SYM(SetStream, miopenSetStream);
    SC_SYM(CreateTensorDescriptor, miopenCreateTensorDescriptor);
    SC_SYM(Set4dTensorDescriptor, miopenSet4dTensorDescriptor);
    SC_SYM(DestroyTensorDescriptor, miopenDestroyTensorDescriptor);
    SC_SYM(CreateConvolutionDescriptor, miopenCreateConvolutionDescriptor);
    SC_SYM(InitConvolutionDescriptor, miopenInitConvolutionDescriptor);
    SC_SYM(DestroyConvolutionDescriptor, miopenDestroyConvolutionDescriptor);
    SC_SYM(ConvolutionForwardGetWorkSpaceSize, miopenConvolutionForwardGetWorkSpaceSize);
    SC_SYM(FindConvolutionForwardAlgorithm, miopenFindConvolutionForwardAlgorithm);
    SC_SYM(ConvolutionForward, miopenConvolutionForward);
#undef SC_SYM
    if (!ok) return false;
    g_api.so = so;
    return true;
}
}  // namespace

struct LibraryConv {
    miopenHandle_t handle = nullptr;
    miopenTensorDescriptor_t xd = nullptr, wd = nullptr, yd = nullptr;
    miopenConvolutionDescriptor_t cd = nullptr;
    void* d_w = nullptr;            // dense weights [D][C][R][S] in the layer's floating-point type
    int N = 0;
    miopenConvFwdAlgorithm_t algo{};
    size_t ws_bytes = 0;
};

// Dense OIHW weights from the unified table (fillers, j >= len[d], carry no value).
template <typename T>
__global__ void __launch_bounds__(256)
densify_oihw_kernel(const T* __restrict__ theta, const int32_t* __restrict__ col, const int32_t* __restrict__ len,
                    T* __restrict__ out, int D, int n, int64_t K)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)D * n) return;
    const int d = (int)(i / n), j = (int)(i - (int64_t)d * n);
    if (j >= len[d]) return;
    out[(int64_t)d * K + (col[i] & 0x7fffffff)] = theta[i];
}

void library_conv_destroy(LibraryConv* c)
{
    if (!c) return;
    if (g_api.so) {
        if (c->xd) (void)g_api.DestroyTensorDescriptor(c->xd);
        if (c->wd) (void)g_api.DestroyTensorDescriptor(c->wd);
        if (c->yd) (void)g_api.DestroyTensorDescriptor(c->yd);
        if (c->cd) (void)g_api.DestroyConvolutionDescriptor(c->cd);
        if (c->handle) (void)g_api.Destroy(c->handle);
    }
    if (c->d_w) (void)hipFree(c->d_w);
    delete c;
}

size_t library_conv_workspace(const LibraryConv* c) { return c ? c->ws_bytes : 0; }
int library_conv_batch(const LibraryConv* c) { return c ? c->N : 0; }

// Set the dense library's convolution up for this layer and batch size and let it pick its
// algorithm by running its candidates on the caller's buffers (y is overwritten).
// SC_ERR_UNSUPPORTED: no library in reach, a dtype it is not used for here, duplicate columns.
sc_status_t library_conv_create(const Plan& p, const void* x, void* y, int N, hipStream_t stream, LibraryConv** out)
{
    *out = nullptr;
    if (p.dtype != SC_F32 && p.dtype != SC_F16) return SC_ERR_UNSUPPORTED;
    if (p.has_dup || p.n == 0) return SC_ERR_UNSUPPORTED;
    if (!load_api()) return SC_ERR_UNSUPPORTED;
    LibraryConv* c = new (std::nothrow) LibraryConv();
    if (!c) return SC_ERR_OOM;
    auto fail = [&](sc_status_t st) { library_conv_destroy(c); return st; };
    const miopenDataType_t dt = p.dtype == SC_F32 ? miopenFloat : miopenHalf;
    const int64_t K = (int64_t)p.L.C * p.L.R * p.L.S;
    const size_t wbytes = (size_t)p.L.D * K * p.ex;
    if (hipMalloc(&c->d_w, wbytes) != hipSuccess) return fail(SC_ERR_OOM);
    if (hipMemsetAsync(c->d_w, 0, wbytes, stream) != hipSuccess) return fail(SC_ERR_HIP);
    {
        const int64_t cnt = (int64_t)p.L.D * p.n;
        const unsigned blocks = (unsigned)((cnt + 255) / 256);
        if (p.dtype == SC_F32)
            hipLaunchKernelGGL(densify_oihw_kernel<float>, dim3(blocks), dim3(256), 0, stream, static_cast<const float*>(p.d_theta),
                               p.d_col, p.d_len, static_cast<float*>(c->d_w), p.L.D, p.n, K);
        else
            hipLaunchKernelGGL(densify_oihw_kernel<__half>, dim3(blocks), dim3(256), 0, stream, static_cast<const __half*>(p.d_theta),
                               p.d_col, p.d_len, static_cast<__half*>(c->d_w), p.L.D, p.n, K);
        if (hipGetLastError() != hipSuccess) return fail(SC_ERR_HIP);
    }
    if (g_api.CreateWithStream(&c->handle, stream) != miopenStatusSuccess) return fail(SC_ERR_UNSUPPORTED);
    if (g_api.CreateTensorDescriptor(&c->xd) != miopenStatusSuccess || g_api.CreateTensorDescriptor(&c->wd) != miopenStatusSuccess ||
        g_api.CreateTensorDescriptor(&c->yd) != miopenStatusSuccess || g_api.CreateConvolutionDescriptor(&c->cd) != miopenStatusSuccess)
        return fail(SC_ERR_UNSUPPORTED);
    if (g_api.Set4dTensorDescriptor(c->xd, dt, N, p.L.C, p.L.H, p.L.W) != miopenStatusSuccess ||
        g_api.Set4dTensorDescriptor(c->wd, dt, p.L.D, p.L.C, p.L.R, p.L.S) != miopenStatusSuccess ||
        g_api.Set4dTensorDescriptor(c->yd, dt, N, p.L.D, p.P, p.Q) != miopenStatusSuccess ||
        g_api.InitConvolutionDescriptor(c->cd, miopenConvolution, p.L.pad_h, p.L.pad_w, p.L.stride_h, p.L.stride_w, 1, 1) != miopenStatusSuccess)
        return fail(SC_ERR_UNSUPPORTED);
    size_t ws = 0;
    if (g_api.ConvolutionForwardGetWorkSpaceSize(c->handle, c->wd, c->xd, c->cd, c->yd, &ws) != miopenStatusSuccess)
        return fail(SC_ERR_UNSUPPORTED);
    void* d_ws = nullptr;
    if (ws && hipMalloc(&d_ws, ws) != hipSuccess) return fail(SC_ERR_OOM);
    miopenConvAlgoPerf_t perf{};
    int returned = 0;
    const miopenStatus_t fs = g_api.FindConvolutionForwardAlgorithm(c->handle, c->xd, x, c->wd, c->d_w, c->cd, c->yd, y, 1, &returned,
                                                                    &perf, d_ws, ws, false);
    (void)hipStreamSynchronize(stream);
    if (d_ws) (void)hipFree(d_ws);
    if (fs != miopenStatusSuccess || returned < 1) return fail(SC_ERR_UNSUPPORTED);
    c->algo = perf.fwd_algo;
    c->ws_bytes = perf.memory;
    c->N = N;
    *out = c;
    return SC_OK;
}

// Y = conv(X) through the library, on `stream`, with the algorithm chosen at set-up.  The
// workspace that algorithm needs (library_conv_workspace) comes from the caller.
sc_status_t library_conv_forward(LibraryConv* c, const void* x, void* y, int N, void* ws, size_t ws_bytes, hipStream_t stream)
{
    if (!c || !g_api.so) return SC_ERR_UNSUPPORTED;
    if (N != c->N) return SC_ERR_SHAPE;               // the descriptors are those of the dispatch's batch size
    if (c->ws_bytes && (!ws || ws_bytes < c->ws_bytes)) return SC_ERR_WORKSPACE;
    if (g_api.SetStream(c->handle, stream) != miopenStatusSuccess) return SC_ERR_HIP;
    const float alpha = 1.0f, beta = 0.0f;
    const miopenStatus_t st = g_api.ConvolutionForward(c->handle, &alpha, c->xd, x, c->wd, c->d_w, c->cd, c->algo, &beta, c->yd, y, ws,
                                                       c->ws_bytes);
    return st == miopenStatusSuccess ? SC_OK : SC_ERR_HIP;
}

}  // namespace sc
