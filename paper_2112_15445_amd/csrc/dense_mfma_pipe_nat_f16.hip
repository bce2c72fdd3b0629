// DENSE variant, 16-bit activations (SC_F16, SC_CB4_F16): v_mfma_f32_16x16x32_f16 instantiations of the pipelined form on the natural layout
// (pointwise layers: direct-to-LDS copies, transposing LDS reads).
#include "dense_mfma_kernel.h"

namespace sc {
sc_status_t launch_mfma_pipe_nat_f16(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    return launch_mfma_typed<SC_F16, 3>(p, a, x, y, grid, stream);
}
}  // namespace sc
