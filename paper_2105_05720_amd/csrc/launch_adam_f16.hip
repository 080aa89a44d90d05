// Launches of the fused Adam kernels for fp16 gradient slices.
#include "launch_adam.inc.hpp"

namespace ccf {

void launch_fused_adam_f16(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode)
{
    launch_fused_adam<false>(p, s, flag, st, mode);
}

namespace {

template <int MODE, class MEM>
void launch_flat_r(const DevTensor &t, int R, unsigned grid, const StepScalars &s, FlagScratch *fs, int32_t *flag, hipStream_t st)
{
    switch (R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_adam_flat_kernel<r, MODE, kSmallBlock, false, 2, MEM>), dim3(grid), dim3(kSmallBlock), 0, st, t, s, fs, flag); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
}

template <class MEM>
void launch_flat_mode(const DevTensor &t, int R, unsigned grid, const StepScalars &s, FlagScratch *fs, int32_t *flag, hipStream_t st, int mode)
{
    switch (mode) {
        case 0: launch_flat_r<0, MEM>(t, R, grid, s, fs, flag, st); break;
        case 1: launch_flat_r<1, MEM>(t, R, grid, s, fs, flag, st); break;
        case 2: launch_flat_r<2, MEM>(t, R, grid, s, fs, flag, st); break;
        default: launch_flat_r<3, MEM>(t, R, grid, s, fs, flag, st); break;
    }
}

}  // namespace

void launch_fused_adam_flat_f16(const DevTensor &t, int R, unsigned grid, int32_t mem, const StepScalars &s, FlagScratch *fs,
                                int32_t *flag, hipStream_t st, int mode)
{
    if (mem == CC_CACHE_RESIDENT) launch_flat_mode<Resident>(t, R, grid, s, fs, flag, st, mode);
    else if (mem == CC_CACHE_WRITE_THROUGH) launch_flat_mode<WriteThrough>(t, R, grid, s, fs, flag, st, mode);
    else launch_flat_mode<Streaming>(t, R, grid, s, fs, flag, st, mode);
}

}  // namespace ccf
