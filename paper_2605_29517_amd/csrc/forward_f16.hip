// Forward kernels of one element type (f16), all supported embedding widths; see forward_impl.h.
#include "forward_impl.h"

namespace maxsim {
hipError_t forward_run_f16(const FwdParams &p, int nu, bool argmax, bool tile, int x, int grid, hipStream_t s)
{
    return run_dtype<MAXSIM_F16>(p, nu, argmax, tile, x, grid, s);
}
} // namespace maxsim
