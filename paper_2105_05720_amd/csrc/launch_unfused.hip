// Launches of the unfused pipelines' kernels (reduce, optimizer from the stored sum, cast) and of the flag-clearing kernel.
#include "plan.hpp"

namespace ccf {

namespace {

template <int BLK, bool GF32, class MEM>
void launch_reduce_r(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    const Layout &L = p->lay();
    if (p->ordered) {
        const dim3 grid(ordered_grid(p)), block(kBigBlock);
        switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((reduce_ordered_kernel<r, kBigBlock, GF32>), grid, block, 0, st, ORDERED_ARGS(p, kSpanReduce), s, p->d_queue, flag); break;
            FOR_EACH_R(CASE)
#undef CASE
        }
        return;
    }
    const dim3 grid((unsigned)L.chunks), block(BLK);
    switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((reduce_kernel<r, BLK, GF32, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, p->d_flag_scratch, flag); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
}

template <int BLK, class MEM>
void launch_reduce_half_b(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    const Layout &L = p->lay();
    if (p->ordered) {
        const dim3 grid(ordered_grid(p)), block(kBigBlock);
        switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((reduce_half_ordered_kernel<r, kBigBlock>), grid, block, 0, st, ORDERED_ARGS(p, kSpanReduce), s, p->d_queue, flag); break;
            FOR_EACH_R(CASE)
#undef CASE
        }
        return;
    }
    const dim3 grid((unsigned)L.chunks), block(BLK);
    switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((reduce_half_kernel<r, BLK, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, p->d_flag_scratch, flag); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
}

template <int BLK, bool SUM16, class MEM>
void launch_adam_from_sum_b(const cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st, int mode)
{
    const Layout &L = p->lay();
    if (p->ordered) {
        const dim3 grid(ordered_grid(p)), block(kBigBlock);
        switch (mode) {
            case 0: hipLaunchKernelGGL((adam_from_sum_ordered_kernel<0, kBigBlock, SUM16>), grid, block, 0, st, ORDERED_ARGS(p, kSpanFromSum), s, p->d_queue, flag); break;
            case 1: hipLaunchKernelGGL((adam_from_sum_ordered_kernel<1, kBigBlock, SUM16>), grid, block, 0, st, ORDERED_ARGS(p, kSpanFromSum), s, p->d_queue, flag); break;
            case 2: hipLaunchKernelGGL((adam_from_sum_ordered_kernel<2, kBigBlock, SUM16>), grid, block, 0, st, ORDERED_ARGS(p, kSpanFromSum), s, p->d_queue, flag); break;
            default: hipLaunchKernelGGL((adam_from_sum_ordered_kernel<3, kBigBlock, SUM16>), grid, block, 0, st, ORDERED_ARGS(p, kSpanFromSum), s, p->d_queue, flag); break;
        }
        return;
    }
    const dim3 grid((unsigned)L.chunks), block(BLK);
    switch (mode) {
        case 0: hipLaunchKernelGGL((adam_from_sum_kernel<0, BLK, SUM16, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, flag); break;
        case 1: hipLaunchKernelGGL((adam_from_sum_kernel<1, BLK, SUM16, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, flag); break;
        case 2: hipLaunchKernelGGL((adam_from_sum_kernel<2, BLK, SUM16, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, flag); break;
        default: hipLaunchKernelGGL((adam_from_sum_kernel<3, BLK, SUM16, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, flag); break;
    }
}

}  // namespace

void launch_reduce(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    if (p->grad_f32) BY_BLOCK(p, (launch_reduce_r<BLK, true, MEM>(p, s, flag, st)));
    else BY_BLOCK(p, (launch_reduce_r<BLK, false, MEM>(p, s, flag, st)));
}

void launch_reduce_half(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    BY_BLOCK(p, (launch_reduce_half_b<BLK, MEM>(p, s, flag, st)));
}

void launch_adam_from_sum(const cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st, int mode, bool sum16)
{
    if (sum16) BY_BLOCK(p, (launch_adam_from_sum_b<BLK, true, MEM>(p, s, flag, st, mode)));
    else BY_BLOCK(p, (launch_adam_from_sum_b<BLK, false, MEM>(p, s, flag, st, mode)));
}

// A plan without chunks launches no streaming kernel, so the flag is cleared by a one-thread kernel (a kernel
// rather than a memset node, so that the call can still be captured into a HIP graph).
int clear_flag(int32_t *flag, hipStream_t st)
{
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    return launched("clear_flag_kernel");
}

int cast_launch(cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st, int guarded)
{
    if (p->ordered) {
        hipLaunchKernelGGL((cast_ordered_kernel<kBigBlock>), dim3(ordered_grid(p)), dim3(kBigBlock), 0, st, ORDERED_ARGS(p, kSpanCast), s, p->d_queue, flag, guarded);
        return launched("cast_ordered_kernel");
    }
    const dim3 grid((unsigned)p->chunks());
    BY_BLOCK(p, hipLaunchKernelGGL((cast_kernel<BLK, MEM>), grid, dim3(BLK), 0, st, p->lay().table_tensors(), p->lay().table_chunks(), s, flag, guarded));
    return launched("cast_kernel");
}

}  // namespace ccf
