// Scalar (4-byte access) instantiations of the dense Local AdaAlter kernels: the path taken when a pointer is not
// 16-byte aligned or d is not a multiple of 4.  A translation unit of its own so that it compiles beside the
// vector path.
#include "laa_dense.inl"

namespace laa {

hipError_t launch_step_scalar(const StepArgs &a, dim3 grid, hipStream_t s) { return launch_step_wt<1>(a, grid, s); }

hipError_t launch_mean_scalar(float *x, float *acc, float *snap, int64_t d, int64_t pitch, int32_t W, int32_t wt,
                              bool x_only, bool collapse, dim3 grid, hipStream_t s)
{
    return launch_mean_wt<1>(x, acc, snap, d, pitch, W, wt, x_only, collapse, grid, s);
}

}  // namespace laa
