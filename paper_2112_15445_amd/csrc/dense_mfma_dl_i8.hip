// DENSE variant, 8-bit activations: instantiations of the one-shot form that walks over several blocks of
// output channels per workgroup (tuning.split_n), on the transposed and on the natural layout.
#include "dense_mfma_kernel.h"

namespace sc {
sc_status_t launch_mfma_dl_i8(const Plan& p, const MfmaArgs& a, const void* x, void* y, int grid, hipStream_t stream)
{
    return p.mg.nat ? launch_mfma_typed<SC_I8, 5>(p, a, x, y, grid, stream) : launch_mfma_typed<SC_I8, 4>(p, a, x, y, grid, stream);
}
}  // namespace sc
