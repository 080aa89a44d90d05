// Launches of the fused Adam kernels for one gradient element type (every R, mode, schedule, workgroup size and cache
// policy).  Included by launch_adam_f16.hip and launch_adam_f32.hip, which exist as two sources only so that the two
// element types compile side by side.
#pragma once

#include "plan.hpp"

namespace ccf {

namespace {

template <int MODE, int BLK, bool GF32, class MEM>
void launch_fused_adam_r(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    const Layout &L = p->lay();
    if (p->ordered) {
        const dim3 grid(ordered_grid(p)), block(kBigBlock);
        switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_adam_ordered_kernel<r, MODE, kBigBlock, GF32>), grid, block, 0, st, ORDERED_ARGS(p, kSpanAdam), s, p->d_queue, flag); break;
            FOR_EACH_R(CASE)
#undef CASE
        }
        return;
    }
    const dim3 grid((unsigned)L.chunks), block(BLK);
    if (p->single >= 0) {                  // one tensor: no table, descriptor in the kernel arguments
        const DevTensor &t = L.host_tensors[(size_t)p->single];
        switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_adam_flat_kernel<r, MODE, BLK, GF32, 2, MEM>), grid, block, 0, st, t, s, p->d_flag_scratch, flag); break;
            FOR_EACH_R(CASE)
#undef CASE
        }
        return;
    }
    switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_adam_kernel<r, MODE, BLK, GF32, 2, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, p->d_flag_scratch, flag); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
}

template <int BLK, bool GF32, class MEM>
void launch_mode(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode)
{
    switch (mode) {
        case 0: launch_fused_adam_r<0, BLK, GF32, MEM>(p, s, flag, st); break;
        case 1: launch_fused_adam_r<1, BLK, GF32, MEM>(p, s, flag, st); break;
        case 2: launch_fused_adam_r<2, BLK, GF32, MEM>(p, s, flag, st); break;
        default: launch_fused_adam_r<3, BLK, GF32, MEM>(p, s, flag, st); break;
    }
}

template <bool GF32>
void launch_fused_adam(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode)
{
    BY_BLOCK(p, (launch_mode<BLK, GF32, MEM>(p, s, flag, st, mode)));
}

}  // namespace

}  // namespace ccf
