// Launches of the LAMB kernels: phase 1 (fused and from the stored sum), the per-tensor second level, phase 2.
#include "plan.hpp"

namespace ccf {

namespace {

template <int BLK, bool GF32, class MEM>
void launch_lamb_phase1_r(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    const Layout &L = p->lay();
    if (p->ordered) {
        const dim3 grid(ordered_grid(p)), block(kBigBlock);
        switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((lamb_phase1_ordered_kernel<r, kBigBlock, GF32>), grid, block, 0, st, ORDERED_ARGS(p, kSpanPhase1), s, p->d_partials, p->d_queue, flag); break;
            FOR_EACH_R(CASE)
#undef CASE
        }
        return;
    }
    const dim3 grid((unsigned)L.chunks), block(BLK);
    switch (p->R) {
#define CASE(r) case r: hipLaunchKernelGGL((lamb_phase1_kernel<r, BLK, GF32, MEM>), grid, block, 0, st, L.table_tensors(), L.table_chunks(), s, p->d_partials, p->d_flag_scratch, flag); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
}

}  // namespace

void launch_lamb_phase1(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st)
{
    if (p->grad_f32) BY_BLOCK_MEM(p, p->mem_lamb, (launch_lamb_phase1_r<BLK, true, MEM>(p, s, flag, st)));
    else BY_BLOCK_MEM(p, p->mem_lamb, (launch_lamb_phase1_r<BLK, false, MEM>(p, s, flag, st)));
}

void launch_lamb_phase1_from_sum(const cc_plan *p, const StepScalars &s, hipStream_t st)
{
    const Layout &L = p->lay();
    const dim3 grid((unsigned)L.chunks);
    if (p->ordered) hipLaunchKernelGGL((lamb_phase1_from_sum_ordered_kernel<kBigBlock>), dim3(ordered_grid(p)), dim3(kBigBlock), 0, st, ORDERED_ARGS(p, kSpanFromSum), s, p->d_partials, p->d_queue);
    else BY_BLOCK_MEM(p, p->mem_lamb, hipLaunchKernelGGL((lamb_phase1_from_sum_kernel<BLK, MEM>), grid, dim3(BLK), 0, st, L.table_tensors(), L.table_chunks(), s, p->d_partials));
}

int lamb_phase2_impl(cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st, bool emit16)
{
    const Layout &L = p->lay();
    if (L.chunks == 0) return CC_OK;
    if (p->ordered) {
        const dim3 grid(ordered_grid(p)), block(kBigBlock);
        if (emit16) hipLaunchKernelGGL((lamb_phase2_ordered_kernel<true, kBigBlock>), grid, block, 0, st, ORDERED_ARGS(p, kSpanPhase2), s, p->d_sums, p->d_queue, flag);
        else hipLaunchKernelGGL((lamb_phase2_ordered_kernel<false, kBigBlock>), grid, block, 0, st, ORDERED_ARGS(p, kSpanPhase2), s, p->d_sums, p->d_queue, flag);
        return launched("lamb_phase2_ordered_kernel");
    }
    const dim3 grid((unsigned)L.chunks);
    if (emit16) BY_BLOCK_MEM(p, p->mem_lamb, hipLaunchKernelGGL((lamb_phase2_kernel<true, BLK, MEM>), grid, dim3(BLK), 0, st, L.table_tensors(), L.table_chunks(), s, p->d_sums, flag));
    else BY_BLOCK_MEM(p, p->mem_lamb, hipLaunchKernelGGL((lamb_phase2_kernel<false, BLK, MEM>), grid, dim3(BLK), 0, st, L.table_tensors(), L.table_chunks(), s, p->d_sums, flag));
    return launched("lamb_phase2_kernel");
}

int lamb_phase2_with_norms(cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st)
{
    const Layout &L = p->lay();
    const dim3 grid((unsigned)L.chunks);
    BY_BLOCK_MEM(p, p->mem_lamb, hipLaunchKernelGGL((lamb_phase2_with_norms_kernel<true, BLK, MEM>), grid, dim3(BLK), 0, st, L.table_tensors(), L.table_chunks(), s, p->d_partials, p->d_sums, flag));
    return launched("lamb_phase2_with_norms_kernel");
}

int lamb_norms(cc_plan *p, hipStream_t st)
{
    hipLaunchKernelGGL(lamb_norms_kernel, dim3((unsigned)p->T), dim3(kNormBlock), 0, st, p->lay().d_tensors, p->d_partials, p->d_sums);
    return launched("lamb_norms_kernel");
}

}  // namespace ccf
