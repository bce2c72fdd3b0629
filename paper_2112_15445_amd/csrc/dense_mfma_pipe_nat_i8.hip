// DENSE variant, 8-bit activations (SC_I8, SC_CB4_I8): v_mfma_i32_16x16x64_i8 instantiations of the pipelined form on the natural layout
// (pointwise layers: direct-to-LDS copies, transposing LDS reads).
#include "dense_mfma_kernel.h"

namespace sc {
sc_status_t launch_mfma_pipe_nat_i8(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    return launch_mfma_typed<SC_I8, 3>(p, a, x, y, grid, stream);
}
}  // namespace sc
