// Launches of the fused Adam kernels for fp32 gradient slices (every R, mode, schedule and workgroup size).
#include "plan.hpp"

namespace ccf {

namespace {

template <int MODE, int BLK, bool GF32>
void launch_fused_adam_r(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    if (p->ordered) {
        const dim3 grid(ordered_grid(p)), block(kBigBlock);
        switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_adam_ordered_kernel<r, MODE, kBigBlock, GF32>), grid, block, 0, st, ORDERED_ARGS(p, kSpanAdam), s, p->d_queue, flag); break;
            FOR_EACH_R(CASE)
#undef CASE
        }
        return;
    }
    const dim3 grid((unsigned)p->chunks), block(BLK);
    if (p->single >= 0) {                  // one tensor: no table, descriptor in the kernel arguments
        const DevTensor &t = p->host_tensors[(size_t)p->single];
        switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_adam_flat_kernel<r, MODE, BLK, GF32>), grid, block, 0, st, t, s, p->d_flag_scratch, flag); break;
            FOR_EACH_R(CASE)
#undef CASE
        }
        return;
    }
    switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_adam_kernel<r, MODE, BLK, GF32>), grid, block, 0, st, p->d_tensors, p->d_chunks, s, p->d_flag_scratch, flag); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
}

template <int BLK, bool GF32>
void launch_mode(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode)
{
    switch (mode) {
        case 0: launch_fused_adam_r<0, BLK, GF32>(p, s, flag, st); break;
        case 1: launch_fused_adam_r<1, BLK, GF32>(p, s, flag, st); break;
        case 2: launch_fused_adam_r<2, BLK, GF32>(p, s, flag, st); break;
        default: launch_fused_adam_r<3, BLK, GF32>(p, s, flag, st); break;
    }
}

}  // namespace

void launch_fused_adam_f32(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode)
{
    BY_BLOCK(p, (launch_mode<BLK, true>(p, s, flag, st, mode)));
}

}  // namespace ccf
