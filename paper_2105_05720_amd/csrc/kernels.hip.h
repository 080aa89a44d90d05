// Device side of ccfused: streaming kernels for gfx950 (wave64).
//
// Every kernel here is bound by HBM bandwidth: per parameter the fused Adam step moves 2R bytes of fp16
// gradients and 26 bytes of fp32/fp16 state against ~R + 30 scalar flops, so there is no contraction and no
// MFMA.  The shape follows from what the memory system rewards:
//
//   * One workgroup per chunk of one tensor; the chunk table replaces a per-thread search over the scattered
//     tensors (Section 5.4).  The table entry and the tensor descriptor are uniform, so they arrive through
//     scalar loads and every buffer is addressed as scalar base + 32-bit lane offset.
//   * Ownership is chosen so that EVERY access instruction of a wave covers one contiguous span: a lane owns
//     4 consecutive elements per group, i.e. one 16-byte access per fp32 array (1 KiB per wave instruction)
//     and one 8-byte access per fp16 array (512 B per wave instruction).  Letting a lane own 8 consecutive
//     elements instead would split each fp32 row of a wave into two half-filled store instructions, and HBM
//     pays dearly for partially written lines (measured: 2.5 TB/s against 5.8 TB/s for the stores alone).
//   * Two groups per sweep, all loads of both groups issued before the first use, so that each wave keeps
//     2 x (R + 3) independent requests in flight.
//   * The reduced gradient stays in registers (Section 3.3, AllReduce Fuse: the output of the reduction is
//     handed to the computation directly, never through memory).
//   * Large shards run under the ordered persistent schedule (ordered_stream below): one workgroup per compute
//     unit, chunks handed out in table order from one counter, the next chunk's loads in flight while the current
//     one is computed.  What it buys is on the DRAM side: the addresses in flight at any moment form a narrow
//     window that slides through each stream, instead of the wide, drifting set that a grid of independent
//     workgroups produces.  Small shards keep one workgroup per chunk (more parallel start-up, no ticket latency).
#pragma once
// (Kernels that are not templates are `static`: this header is included by several translation units.)

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "ccfused.h"

namespace ccf {

constexpr uint32_t kStatePack = 4;     // consecutive elements a lane owns per group wherever an fp32 array is written

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One tensor of the shard as the kernels see it.
struct DevTensor {
    uint64_t numel;
    const float *w_in, *m_in, *v_in;
    float *w_out, *m_out, *v_out;
    uint16_t *w16;
    const void *grad[CC_MAX_R];   // fp16 bit patterns, or fp32 values when the plan says so
    float *gsum;              // unfused pipelines only: fp32 reduced gradient of this tensor
    float wd;
    uint32_t first_chunk;     // position of this tensor's first chunk in the table
    uint32_t num_chunks;
    uint32_t tensor;          // index of this tensor in the plan's list
    uint32_t chunk_index;     // per-chunk copies of the descriptor only (see locate_at): which chunk of the tensor
    uint32_t pad_;
};

// Chunk table entry: which tensor, and which chunk_elems-sized piece of it.
struct Chunk {
    uint32_t tensor;
    uint32_t index;
};

// Scalars of one step, precomputed on the host in double and rounded once.
struct StepScalars {
    double inv_div;           // 1 / (loss_scale * (average ? R : 1))
    double beta1, beta2;      // the interface's fp32 values, promoted
    double omb1, omb2;        // 1 - beta, exact in double
    float rc1, rc2;           // 1 / (1 - beta^t)
    float eps, lr;
    uint32_t chunk_elems;
};

enum : int { kModeGuard = 1, kModeL2 = 2 };

__device__ __forceinline__ bool not_finite(float x) { return !(__builtin_fabsf(x) <= 3.402823466e+38f); }

// Moments of one element from the reduced sum S (Fig. 4a: the m and v updates), each formed in double from the fp32
// inputs and rounded to fp32 once, so that the stored moments are the correctly rounded values of their definitions
// (up to double rounding).  In fp32 the terms would be rounded one by one, and where they cancel (the two terms of
// m', or S / (loss_scale D) against wd w in L2 mode) the result carries those roundings at full size: random cases
// put a few elements at 1.3 x the parity bound that way.  Eight double-precision operations per element, which
// neither the HBM-bound nor the launch-bound kernels notice.
template <int MODE>
__device__ __forceinline__ void moments(float S, float w, float wd, const StepScalars &s, float &m, float &v)
{
    double g = (double)S * s.inv_div;
    if (MODE & kModeL2) g = __builtin_fma((double)wd, (double)w, g);
    m = (float)__builtin_fma(s.beta1, (double)m, s.omb1 * g);
    v = (float)__builtin_fma(s.beta2, (double)v, (s.omb2 * g) * g);
}

// Update direction u from the new moments (Fig. 4a: bias corrections and the quotient), plus decoupled decay.
template <int MODE>
__device__ __forceinline__ float direction(float w, float wd, float m, float v, const StepScalars &s)
{
    const float mh = m * s.rc1;
    const float vh = v * s.rc2;
    // v_sqrt_f32 and v_rcp_f32, each within 1 ulp: the quotient is off by at most ~3 x 2^-24 relative, which moves
    // w by lr |u| 2e-7, two orders below the 2e-6 parity bound; the IEEE sequences cost 20 more instructions per
    // element, which a small (launch-bound) shard pays in full.
    float u = mh * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(vh) + s.eps);
    if (!(MODE & kModeL2)) u = __builtin_fmaf(wd, w, u);
    return u;
}

// ---- memory access: every buffer is device memory, addressed as uniform base + 32-bit byte offset ----------
#define CCF_GLOBAL __attribute__((address_space(1)))
typedef const CCF_GLOBAL char *gcbytes;
typedef CCF_GLOBAL char *gbytes;

// Base of a chunk inside one of a tensor's arrays (generic pointers from the descriptor become global ones).
__device__ __forceinline__ gcbytes chunk_base(const void *p, uint64_t byte_off) { return (gcbytes)p + byte_off; }
__device__ __forceinline__ gbytes chunk_base(void *p, uint64_t byte_off) { return (gbytes)p + byte_off; }

// Cache policy of a kernel's vector accesses.
//   Streaming:    non-temporal hints on every access.  Right for shards far beyond what the chip holds: the data is
//                 not touched again before it has left every cache (+3 % with one workgroup per chunk, +7 % on the
//                 stores under the ordered schedule).
//   Resident:     plain loads, and stores that are written through to the device's coherence point (the sc1 bit), for
//                 shards whose whole step (inputs and outputs of two consecutive steps, which ping-pong between two
//                 copies) fits the 256 MB Infinity Cache.  The next step then finds what this one wrote on chip, and
//                 no dirty lines are left in the L2s for the end of the kernel to write back.  On the memory pattern
//                 of a 2^20-element step: 5.2 us, against 6.6-6.8 us for every combination of plain or non-temporal
//                 loads with plain or non-temporal stores on the same machine.
//   WriteThrough: non-temporal loads with the written-through stores, for shards of a few times the Infinity Cache.
//                 Memory pattern of a 2^24-element step with four slices (570 MB): 72 us, against 93 us for Streaming
//                 and 102 us for Resident; at 2^20 elements it is the slowest of the three (7.1 us), at 2^26 it is 2 %
//                 behind Streaming.
// The compiler has no spelling for a vector store with the sc1 bit, hence the asm; the s_nop behind each store is the
// wait the hardware asks for between a store of more than 64 bits and a vector instruction that overwrites the
// registers holding its data, which the compiler inserts for its own stores but cannot for one it does not see.
struct Streaming { static constexpr bool kLoadNonTemporal = true, kStoreThrough = false; };
struct Resident { static constexpr bool kLoadNonTemporal = false, kStoreThrough = true; };
struct WriteThrough { static constexpr bool kLoadNonTemporal = true, kStoreThrough = true; };

template <class Mem> __device__ __forceinline__ f32x4 ld_f32x4(gcbytes b, uint32_t off)
{
    if (Mem::kLoadNonTemporal) return __builtin_nontemporal_load((const CCF_GLOBAL f32x4 *)(b + off));
    return *(const CCF_GLOBAL f32x4 *)(b + off);
}
template <class Mem> __device__ __forceinline__ f16x4 ld_f16x4(gcbytes b, uint32_t off)
{
    if (Mem::kLoadNonTemporal) return __builtin_nontemporal_load((const CCF_GLOBAL f16x4 *)(b + off));
    return *(const CCF_GLOBAL f16x4 *)(b + off);
}
template <class Mem> __device__ __forceinline__ void st_f32x4(gbytes b, uint32_t off, f32x4 x)
{
    if (!Mem::kStoreThrough) __builtin_nontemporal_store(x, (CCF_GLOBAL f32x4 *)(b + off));
    else asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(b + off), "v"(x) : "memory");
}
template <class Mem> __device__ __forceinline__ void st_f16x4(gbytes b, uint32_t off, f16x4 x)
{
    if (!Mem::kStoreThrough) __builtin_nontemporal_store(x, (CCF_GLOBAL f16x4 *)(b + off));
    else asm volatile("global_store_dwordx2 %0, %1, off sc1\n\ts_nop 1" : : "v"(b + off), "v"(x) : "memory");
}
__device__ __forceinline__ float ld_f32(gcbytes b, uint32_t off) { return *(const CCF_GLOBAL float *)(b + off); }
__device__ __forceinline__ float ld_f16(gcbytes b, uint32_t off) { return (float)*(const CCF_GLOBAL _Float16 *)(b + off); }
__device__ __forceinline__ void st_f32(gbytes b, uint32_t off, float x) { *(CCF_GLOBAL float *)(b + off) = x; }

// fp32 -> fp16, round to nearest even, of the fp32 value as stored.  The empty asm pins x in a register so
// that the compiler cannot merge the conversion with the fma that produced x into one mixed-precision fma
// (v_fma_mixlo_f16 rounds the exact product-sum straight to fp16, which can differ from rounding the fp32
// result by one fp16 ulp).
__device__ __forceinline__ _Float16 to_half(float x)
{
    asm volatile("" : "+v"(x));
    return (_Float16)x;
}
__device__ __forceinline__ void st_f16(gbytes b, uint32_t off, float x) { *(CCF_GLOBAL _Float16 *)(b + off) = to_half(x); }

template <class Mem> __device__ __forceinline__ void ld_f32x4(gcbytes b, uint32_t off, float (&x)[4])
{
    const f32x4 t = ld_f32x4<Mem>(b, off);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}
template <class Mem> __device__ __forceinline__ void st_f32x4(gbytes b, uint32_t off, const float (&x)[4])
{
    st_f32x4<Mem>(b, off, f32x4{x[0], x[1], x[2], x[3]});
}
template <class Mem> __device__ __forceinline__ void st_f16x4(gbytes b, uint32_t off, const float (&x)[4])
{
    st_f16x4<Mem>(b, off, f16x4{to_half(x[0]), to_half(x[1]), to_half(x[2]), to_half(x[3])});
}

// ---- where a workgroup works -----------------------------------------------------------------------------------
struct Where {
    const DevTensor *t;
    uint32_t tensor;          // index of t in the plan's tensor list
    uint32_t slot;            // position of the chunk in tensor order (first_chunk + index): where its LAMB partials go
    uint32_t index;           // which chunk of the tensor
    uint64_t base;            // first element of the chunk inside the tensor
    uint32_t len;             // elements in this chunk (the tensor's last chunk may be short)
};

// What is left to derive once the descriptor and the chunk's index are known.
__device__ __forceinline__ void finish_where(Where &wh, uint32_t chunk_elems)
{
    wh.slot = wh.t->first_chunk + wh.index;
    wh.base = (uint64_t)wh.index * chunk_elems;
    const uint64_t rem = wh.t->numel - wh.base;
    wh.len = rem < chunk_elems ? (uint32_t)rem : chunk_elems;
}

// Table entry `entry` (uniform over the workgroup) resolved through the tensor descriptor.
__device__ __forceinline__ Where locate_at(const DevTensor *__restrict__ tensors, const Chunk *__restrict__ chunks,
                                           uint32_t entry, uint32_t chunk_elems)
{
    const Chunk c = chunks[entry];
    Where wh;
    wh.t = tensors + c.tensor;
    wh.tensor = c.tensor;
    wh.index = c.index;
    finish_where(wh, chunk_elems);
    return wh;
}

// The chunk of this workgroup under the one-workgroup-per-chunk launches.  Plans of few chunks pass chunks == nullptr
// and, as `tensors`, one copy of the descriptor per chunk with the chunk's index in it: the workgroup then knows where
// its data is after one trip to memory instead of two dependent ones (entry, then descriptor): 2-4 % of a launch-bound
// step (same machine, with / without: 4.70 / 4.90 us on 398 tensors in 571 chunks, 9.60 / 9.90 us on 10 tensors in
// 1280 chunks).
__device__ __forceinline__ Where locate(const DevTensor *__restrict__ tensors, const Chunk *__restrict__ chunks,
                                        uint32_t chunk_elems)
{
    if (chunks != nullptr) return locate_at(tensors, chunks, blockIdx.x, chunk_elems);
    Where wh;
    wh.t = tensors + blockIdx.x;
    wh.tensor = wh.t->tensor;
    wh.index = wh.t->chunk_index;
    finish_where(wh, chunk_elems);
    return wh;
}

// The overflow flag is produced by the same launch that does the work, with no clearing launch in front of it and
// with nothing on the path between a wave's loads and its stores.
//
// What has to happen: the caller's flag must read 0 after a launch in which no wave saw an inf/NaN and 1 otherwise,
// and the scratch words must be ready for the next launch.  Counting FINISHED workgroups (the obvious way to find
// "the last one", who then writes the flag) puts two dependent atomic round trips behind the last wave's loads, and a
// returning atomic issued after the stores is only seen once those stores are acknowledged (the memory counter is
// in order): measured 0.9-1.7 us on a 6 us step.  So ARRIVALS are counted instead:
//
//   * Lane 0 of every wave adds 1 to one of kFlagSlots slot words as its very first act, before any load.  The
//     result comes back while the loads are in flight.  The high half of a slot word is the launch's phase p (the
//     same in every slot between launches), so the one atomic tells a wave p and whether it is the last arrival in
//     its slot.  That wave puts the slot back to (p+1, 0) and adds 1 to the top word; the wave that completes the top
//     word is the last arrival of the launch: every wave has arrived, none will touch the counters again, so it can
//     zero the top word and move the slots this launch did not use to p+1 as well.
//   * The last arrival clears the caller's flag with a returning exchange issued before its own update and stores,
//     and, behind its stores, once that exchange has returned (so the 0 has been performed at the device's coherence
//     point), exchanges the state word to (p+1, CLEARED).  If this second exchange returns (p+1, BAD), a wave had
//     reported an inf/NaN before, and the last arrival sets the flag to 1 itself.  (A release on the second exchange
//     would state the same order in the language's terms, but costs a write-back of the whole L2 in the middle of
//     the kernel on the one wave that everybody ends up waiting for: measured +0.7 to +1.3 us per step.  The order is
//     enforced in the source instead: the second exchange takes an operand that depends on the first one's result.)
//   * A wave that saw an inf/NaN (rare) moves the state word to (p+1, BAD) with a compare-exchange loop, unless it
//     finds (p+1, CLEARED) there: then the flag's 0 was performed before, and it stores 1 into the flag itself.
//     Either the last arrival's exchange comes first in the state word's modification order, and the reporting wave
//     sees CLEARED and writes 1 after the 0; or the report comes first, and the exchange returns it.  Both can write 1.
//   * Values of older launches in the state word carry another phase and are ignored, so nothing has to be reset at
//     the end of a launch, which is what would need a count of finished waves.
//
// Nothing waits on another wave.  Per launch every wave issues one atomic; one wave per slot issues three more; one
// wave issues the handful around the flag.  Phases are 32 bits and wrap; a report that is exactly 2^32 launches old
// would be taken for a new one.
constexpr uint32_t kFlagSlots = 128;
struct FlagScratch {
    struct alignas(128) Line { unsigned long long word; } slot[kFlagSlots], top, state;
};
constexpr unsigned long long kStateBad = 1ull, kStateCleared = 2ull;

template <int BLOCK>
struct FlagCount {
    unsigned long long prev = 0ull, tprev = 0ull;
    uint32_t slot = 0, in_slot = 0, used = 0;
    int32_t flag_before = 0;
    bool slot_last = false, launch_last = false;

    __device__ __forceinline__ bool counting_lane() const { return (threadIdx.x & 63u) == 0u; }
    __device__ __forceinline__ uint32_t tag() const { return (uint32_t)(prev >> 32) + 1u; }          // this launch's p + 1

    // First act of a kernel: the wave's arrival.  Nothing is waited for here.
    __device__ __forceinline__ void arrive(FlagScratch *fs)
    {
        if (counting_lane()) {
            constexpr uint32_t kWaves = BLOCK / 64;
            const uint32_t waves = gridDim.x * kWaves;
            const uint32_t me = blockIdx.x * kWaves + (threadIdx.x >> 6);
            slot = me % kFlagSlots;
            in_slot = (waves - slot + kFlagSlots - 1) / kFlagSlots;      // waves w with w % kFlagSlots == slot
            used = waves < kFlagSlots ? waves : kFlagSlots;
            prev = atomicAdd(&fs->slot[slot].word, 1ull);
        }
    }
    // Once the arrival's result is needed (behind the issue of the loads): the last arrival in a slot moves on to the top word.
    __device__ __forceinline__ void slot_level(FlagScratch *fs)
    {
        if (counting_lane()) {
            slot_last = (uint32_t)prev == in_slot - 1;
            if (slot_last) {
                atomicExch(&fs->slot[slot].word, (unsigned long long)tag() << 32);
                tprev = atomicAdd(&fs->top.word, 1ull);
            }
        }
    }
    // Before the wave's stores: the last arrival of the launch tidies the counters and starts clearing the flag.  Every
    // lane of the wave calls this.  The slots a small launch did not use are moved on by all 64 lanes at once, behind
    // the flag's exchange: one lane doing it slot by slot, in front of the exchange, cost a launch of one workgroup 2 us.
    __device__ __forceinline__ void top_level(FlagScratch *fs, int32_t *flag)
    {
        if (counting_lane() && slot_last) {
            launch_last = (uint32_t)tprev == used - 1;
            if (launch_last) {
                atomicExch(&fs->top.word, 0ull);
                flag_before = __hip_atomic_exchange(flag, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (__builtin_amdgcn_ballot_w64(launch_last) != 0ull) {            // uniform: this wave holds the last arrival
            const uint32_t first_unused = (uint32_t)__builtin_amdgcn_readfirstlane((int)used);
            const uint32_t next_tag = (uint32_t)__builtin_amdgcn_readfirstlane((int)tag());
            for (uint32_t k = first_unused + (threadIdx.x & 63u); k < kFlagSlots; k += 64u)
                atomicExch(&fs->slot[k].word, (unsigned long long)next_tag << 32);
        }
    }
    // After the wave's stores have been issued: reports.
    __device__ __forceinline__ void finish(bool bad, FlagScratch *fs, int32_t *flag)
    {
        const bool any = __builtin_amdgcn_ballot_w64(bad) != 0ull;
        if (counting_lane()) {
            const unsigned long long mine_bad = ((unsigned long long)tag() << 2) | kStateBad;
            const unsigned long long cleared = ((unsigned long long)tag() << 2) | kStateCleared;
            if (launch_last) {
                unsigned long long mark = cleared;
                asm volatile("" : "+v"(mark) : "v"(flag_before));     // not before the flag's exchange has returned
                const unsigned long long sprev = __hip_atomic_exchange(&fs->state.word, mark, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (sprev == mine_bad) __hip_atomic_store(flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (any) {
                unsigned long long cur = __hip_atomic_load(&fs->state.word, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                while (true) {
                    if (cur == cleared) {                 // the flag was cleared before: this store comes after the 0
                        __hip_atomic_store(flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    if (cur == mine_bad) break;           // another wave has reported for this launch already
                    if (__hip_atomic_compare_exchange_strong(&fs->state.word, &cur, mine_bad, __ATOMIC_ACQ_REL, __ATOMIC_ACQUIRE,
                                                             __HIP_MEMORY_SCOPE_AGENT))
                        break;                            // the last arrival's exchange will return this report
                }
            }
        }
    }
    // Everything behind the arrival at once, for kernels that do not place the stages themselves.
    __device__ __forceinline__ void settle(bool bad, FlagScratch *fs, int32_t *flag)
    {
        slot_level(fs);
        top_level(fs, flag);
        finish(bad, fs, flag);
    }
};

// Only for a plan without any chunk: nothing else would write the flag.
[[maybe_unused]] static __global__ void clear_flag_kernel(int32_t *flag) { *flag = 0; }

// ---- the streaming skeleton --------------------------------------------------------------------------------------
// An Op describes one kernel's per-element work:
//   static constexpr uint32_t kPack;               consecutive elements a lane owns per group
//   struct Regs;                                   registers of one group (kPack elements of this lane)
//   void load(Regs&, uint32_t e) const;            vector loads of elements e .. e+kPack-1 of the chunk
//   void compute(Regs&);                           arithmetic on the group
//   void store(const Regs&, uint32_t e) const;     vector stores
//   void single(uint32_t j);                       one element, scalar accesses (ragged end of a tensor)
// A sweep is two groups BLOCK*kPack elements apart.  A full sweep issues the loads of both groups, then computes
// and stores; the ragged end of a chunk (only a tensor's last chunk has one) falls back group by group.
template <int BLOCK, class Op, int GROUPS = 2>
__device__ __forceinline__ void stream_chunk(Op &op, uint32_t len)
{
    constexpr uint32_t kLanePack = Op::kPack;      // consecutive elements a lane owns per group
    constexpr uint32_t kGroup = BLOCK * kLanePack;
    constexpr uint32_t kSweep = GROUPS * kGroup;
    const uint32_t lane_e = threadIdx.x * kLanePack;
    uint32_t s0 = 0;
    for (; s0 + kSweep <= len; s0 += kSweep) {
        typename Op::Regs x[GROUPS];
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) op.load(x[g], s0 + g * kGroup + lane_e);
        __builtin_amdgcn_sched_barrier(0);         // keep all loads of the sweep ahead of the first use
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            op.compute(x[g]);
            op.store(x[g], s0 + g * kGroup + lane_e);
        }
    }
    for (uint32_t e = s0 + lane_e; e < len; e += kGroup) {
        if (e + kLanePack <= len) {
            typename Op::Regs a;
            op.load(a, e);
            op.compute(a);
            op.store(a, e);
        } else {
            for (uint32_t j = e; j < len; ++j) op.single(j);
        }
    }
}

// One workgroup per chunk, for an Op that raises the flag.  `fc` has arrived already (first act of the kernel).  When
// the chunk is exactly one sweep (the launch shapes the plans use), the stages of the count are placed where their
// results are free: the slot level behind the issue of the loads, the top level behind the sums, the reports behind
// the stores.  The waves of a workgroup never wait for each other here.
template <int BLOCK, int GROUPS, class Op>
__device__ __forceinline__ void sweep_and_publish(Op &op, uint32_t len, FlagCount<BLOCK> &fc, FlagScratch *fs, int32_t *flag)
{
    constexpr uint32_t kGroup = BLOCK * Op::kPack;
    if (len == GROUPS * kGroup) {
        const uint32_t lane_e = threadIdx.x * Op::kPack;
        typename Op::Regs x[GROUPS];
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) op.load(x[g], g * kGroup + lane_e);
        __builtin_amdgcn_sched_barrier(0);
        fc.slot_level(fs);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) op.reduce(x[g]);
        fc.top_level(fs, flag);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) { op.update(x[g]); op.store(x[g], g * kGroup + lane_e); }
        __builtin_amdgcn_sched_barrier(0);
        fc.finish(op.bad, fs, flag);
    } else {
        stream_chunk<BLOCK, Op, GROUPS>(op, len);
        fc.settle(op.bad, fs, flag);
    }
}

// ---- the ordered persistent schedule -------------------------------------------------------------------------------
// gridDim.x workgroups (one per compute unit) share the chunk table through one counter.  The table is cut into
// blocks of `span` consecutive entries.  Workgroup b starts with blocks b and b + G (G = gridDim.x) and then takes
// block 2G + ticket, ticket = atomic increment of `next`: blocks are started in table order by whichever workgroup
// is free, so the chunks in flight are always ~2G span consecutive ones.  (A counter that every workgroup of the
// device increments serves about one ticket per 12 ns; span is chosen per kernel so that a ticket covers enough
// bytes for that not to matter.)  The table lists every full chunk first (nfull of them, in address order) and
// the short last chunks of tensors behind them; full chunks go through a two-stage pipeline (loads of the next
// chunk are issued before the current chunk is computed and stored), the few short ones through stream_chunk.
// Nothing waits on another workgroup: a workgroup leaves when its entries are past the table, so the grid drains
// whatever its size.  `done` counts finished workgroups in its low half and those that saw an inf/NaN in its high
// half (one atomic, so no fence has to order two words); the workgroup that completes the count writes the
// caller's flag and zeroes the queue for the next launch.
struct WorkQueue {
    struct alignas(128) Next { uint32_t v; } next;
    struct alignas(128) Done { unsigned long long v; } done;
};

// The increasing sequence of table entries one workgroup works through.  The ticket for the block after the next
// one is requested when a block is entered and only looked at when that later block is entered, a block's worth of
// work later; the one wave that issues the atomic waits for it there and then, the others never do.  Its value
// reaches them through LDS (two slots used in turn: one barrier per block).
struct Entries {
    WorkQueue *q;
    uint32_t *slots;          // LDS, 2 words
    uint32_t span, blk, j, second, ticket;
    bool second_pending;      // the workgroup's second block (blockIdx.x + gridDim.x) has not been entered yet
    int turn;
    __device__ __forceinline__ void init(WorkQueue *queue, uint32_t *lds_slots, uint32_t span_)
    {
        q = queue; slots = lds_slots; span = span_;
        blk = blockIdx.x; second = blockIdx.x + gridDim.x;    // the two blocks every workgroup owns without asking
        second_pending = true;
        j = 0; turn = 0; ticket = 0;
    }
    // every thread of the workgroup calls next() at the same point
    __device__ __forceinline__ uint32_t next()
    {
        if (j == span) {                                      // enter the next block
            j = 0;
            if (second_pending) {
                blk = second;
                second_pending = false;
            } else {
                if (threadIdx.x == 0) slots[turn] = 2 * gridDim.x + ticket;
                __syncthreads();
                blk = (uint32_t)__builtin_amdgcn_readfirstlane((int)slots[turn]);
                turn ^= 1;
            }
            if (threadIdx.x == 0) ticket = atomicAdd(&q->next.v, 1u);      // for the block after the next one
        }
        return blk * span + j++;
    }
};

// An Op used here also provides   template <int BLOCK> void end_chunk(uint32_t slot);   called once per chunk after
// its last store (LAMB phase 1 writes the chunk's partial sums there; the others do nothing).
// bind(op, entry) points op at table entry `entry` and returns its Where.
template <int BLOCK, int GROUPS, class Op, class Bind>
__device__ __forceinline__ void ordered_stream(Op &opa, Op &opb, Bind bind, uint32_t nfull, uint32_t nchunks, uint32_t span,
                                               WorkQueue *q)
{
    __shared__ uint32_t ticket_slots[2];
    constexpr uint32_t kGroup = BLOCK * Op::kPack;
    const uint32_t lane_e = threadIdx.x * Op::kPack;
    Entries en;
    en.init(q, ticket_slots, span);
    uint32_t e = en.next(), n = en.next();         // current and next entry, e < n
    if (e < nfull) {
        typename Op::Regs xa[GROUPS], xb[GROUPS];
        Where wa = bind(opa, e), wb;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) opa.load(xa[g], g * kGroup + lane_e);
        while (true) {
            if (n < nfull) {                       // past the full chunks there is nothing to fetch ahead
                wb = bind(opb, n);
#pragma unroll
                for (int g = 0; g < GROUPS; ++g) opb.load(xb[g], g * kGroup + lane_e);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) { opa.compute(xa[g]); opa.store(xa[g], g * kGroup + lane_e); }
            opa.template end_chunk<BLOCK>(wa.slot);
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t n2 = en.next();
            if (n >= nfull) { e = n; n = n2; break; }
            if (n2 < nfull) {
                wa = bind(opa, n2);
#pragma unroll
                for (int g = 0; g < GROUPS; ++g) opa.load(xa[g], g * kGroup + lane_e);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) { opb.compute(xb[g]); opb.store(xb[g], g * kGroup + lane_e); }
            opb.template end_chunk<BLOCK>(wb.slot);
            __builtin_amdgcn_sched_barrier(0);
            e = n2;
            n = en.next();
            if (e >= nfull) break;
        }
    }
    while (e < nchunks) {                          // short chunks, one at a time
        const Where wh = bind(opa, e);
        stream_chunk<BLOCK, Op, GROUPS>(opa, wh.len);
        opa.template end_chunk<BLOCK>(wh.slot);
        e = n;
        n = en.next();
    }
}

// Last act of a workgroup under the ordered schedule: count itself (and whether it saw an inf/NaN); the workgroup
// that completes the count writes the flag (RAISE) and zeroes the queue.
// Why `next` is exactly 0 when the next launch starts: every increment of `next` is issued by thread 0 of some
// workgroup (Entries::next), the same thread that later adds to `done` here, so the increment is sequenced before
// that add.  The add releases and acquires at device scope: the add of the workgroup that completes the count reads
// from the release sequence formed by all the earlier adds, hence every increment of `next` by any workgroup happens
// before the exchange below, which is therefore the last modification of `next` in this launch, also for a
// workgroup whose last ticket was requested but never looked at.  One such add per workgroup per launch costs nothing.
template <bool RAISE>
__device__ __forceinline__ void leave_queue(bool bad, WorkQueue *q, int32_t *flag)
{
    const int any = RAISE ? __syncthreads_or(bad ? 1 : 0) : 0;
    if (threadIdx.x == 0) {
        const unsigned long long mine = 1ull | (any ? (1ull << 32) : 0ull);
        const unsigned long long prev = __hip_atomic_fetch_add(&q->done.v, mine, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)prev == gridDim.x - 1) {
            if (RAISE) *flag = ((prev + mine) >> 32) != 0ull ? 1 : 0;
            atomicExch(&q->done.v, 0ull);
            atomicExch(&q->next.v, 0u);
        }
    }
}

// The gradient source of a kernel: R slices reduced in registers in fixed rank order; the reduced value is an fp32.
// The slices are fp16 (fp16 -> fp32 is exact, subnormals included; 8 bytes per lane and slice) or fp32 (16 bytes per
// lane and slice); either way the terms are added in double and rounded to fp32 once (see below).
// The unfused pipelines read the fp32 sum that a reduce kernel stored instead (GradSum).
template <int R, bool F32, class MemT = Streaming>
struct GradSlices;

template <int R, class MemT>
struct GradSlices<R, false, MemT> {
    typedef MemT Mem;
    gcbytes g[R];
    struct Regs { f16x4 g[R]; };
    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base)
    {
#pragma unroll
        for (int r = 0; r < R; ++r) g[r] = chunk_base(t->grad[r], base * 2);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
#pragma unroll
        for (int r = 0; r < R; ++r) x.g[r] = ld_f16x4<Mem>(g[r], e * 2);
    }
    // The sum is formed in double and rounded to fp32 once, in rank order.  Up to 16 fp16 values add exactly in double,
    // so S is the correctly rounded sum whatever the order.  An fp32 running sum is exact only while every partial sum
    // stays below 1 (fp16 values are multiples of 2^-24); with loss-scaled gradients of magnitude ~1 a small addend
    // loses its low bits against a large partial sum (up to 2^-22 absolute per add), and where the slices cancel to
    // |S| ~ 1e-3 that is a relative error of 1e-4 in the reduced gradient.  On the few elements per 10^8 where the
    // unscaled gradient is also comparable with epsilon, u = g/(|g| + eps) turns it into an error of w of 1.8 x the
    // 2e-6 parity bound (measured on the 80 M element embedding of the GPT-2 list).
    __device__ __forceinline__ void sum(const Regs &x, float (&S)[4]) const
    {
        double a = (double)(float)x.g[0].x, b = (double)(float)x.g[0].y, c = (double)(float)x.g[0].z, d = (double)(float)x.g[0].w;
#pragma unroll
        for (int r = 1; r < R; ++r) {
            a += (double)(float)x.g[r].x; b += (double)(float)x.g[r].y; c += (double)(float)x.g[r].z; d += (double)(float)x.g[r].w;
        }
        S[0] = (float)a; S[1] = (float)b; S[2] = (float)c; S[3] = (float)d;
    }
    __device__ __forceinline__ float sum1(uint32_t j) const
    {
        double S = (double)ld_f16(g[0], j * 2);
#pragma unroll
        for (int r = 1; r < R; ++r) S += (double)ld_f16(g[r], j * 2);
        return (float)S;
    }
};

template <int R, class MemT>
struct GradSlices<R, true, MemT> {
    typedef MemT Mem;
    gcbytes g[R];
    struct Regs { f32x4 g[R]; };
    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base)
    {
#pragma unroll
        for (int r = 0; r < R; ++r) g[r] = chunk_base(t->grad[r], base * 4);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
#pragma unroll
        for (int r = 0; r < R; ++r) x.g[r] = ld_f32x4<Mem>(g[r], e * 4);
    }
    // fp32 slices are added in double and rounded to fp32 once: an fp32 running sum would carry up to
    // (R-1) 2^-24 max|g| of rounding, which a near-zero sum turns into a large relative error of g^2 and, through
    // elements with a small second moment, into an error of w above the 2e-6 bar.  16 fp64 operations per
    // element stay far below the memory time.  A finite sum that does not fit fp32 becomes inf and raises the flag.
    __device__ __forceinline__ void sum(const Regs &x, float (&S)[4]) const
    {
        double a = x.g[0].x, b = x.g[0].y, c = x.g[0].z, d = x.g[0].w;
#pragma unroll
        for (int r = 1; r < R; ++r) { a += (double)x.g[r].x; b += (double)x.g[r].y; c += (double)x.g[r].z; d += (double)x.g[r].w; }
        S[0] = (float)a; S[1] = (float)b; S[2] = (float)c; S[3] = (float)d;
    }
    __device__ __forceinline__ float sum1(uint32_t j) const
    {
        double S = ld_f32(g[0], j * 4);
#pragma unroll
        for (int r = 1; r < R; ++r) S += (double)ld_f32(g[r], j * 4);
        return (float)S;
    }
};

template <class MemT = Streaming>
struct GradSum {
    typedef MemT Mem;
    gcbytes s;
    struct Regs { float s[4]; };
    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base) { s = chunk_base((const void *)t->gsum, base * 4); }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const { ld_f32x4<Mem>(s, e * 4, x.s); }
    __device__ __forceinline__ void sum(const Regs &x, float (&S)[4]) const { S[0] = x.s[0]; S[1] = x.s[1]; S[2] = x.s[2]; S[3] = x.s[3]; }
    __device__ __forceinline__ float sum1(uint32_t j) const { return ld_f32(s, j * 4); }
};

// The reduced sum as an fp16 all-reduce hands it over: fp16 values in the first half of the tensor's sum buffer.
template <class MemT = Streaming>
struct GradSumHalf {
    typedef MemT Mem;
    gcbytes s;
    struct Regs { f16x4 s; };
    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base) { s = chunk_base((const void *)t->gsum, base * 2); }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const { x.s = ld_f16x4<Mem>(s, e * 2); }
    __device__ __forceinline__ void sum(const Regs &x, float (&S)[4]) const { S[0] = (float)x.s.x; S[1] = (float)x.s.y; S[2] = (float)x.s.z; S[3] = (float)x.s.w; }
    __device__ __forceinline__ float sum1(uint32_t j) const { return ld_f16(s, j * 2); }
};

// ---------------------------------------------------------------------------------------------------
// Adam: reduce (or read the reduced sum) + moments + weight update (+ fp16 emission when fused).
// One pass, 2R + 26 bytes per parameter when fused.
// ---------------------------------------------------------------------------------------------------
template <class Grad, int MODE, bool EMIT16>
struct AdamOp {
    static constexpr uint32_t kPack = kStatePack;
    typedef typename Grad::Mem Mem;
    Grad grad;
    gcbytes w_in, m_in, v_in;
    gbytes w_out, m_out, v_out, w16;
    StepScalars s;
    float wd;
    bool bad = false;
    struct Regs { typename Grad::Regs g; float S[4], w[4], m[4], v[4]; };

    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base, const StepScalars &sc)
    {
        grad.init(t, base);
        w_in = chunk_base((const void *)t->w_in, base * 4); m_in = chunk_base((const void *)t->m_in, base * 4);
        v_in = chunk_base((const void *)t->v_in, base * 4);
        w_out = chunk_base((void *)t->w_out, base * 4); m_out = chunk_base((void *)t->m_out, base * 4);
        v_out = chunk_base((void *)t->v_out, base * 4);
        w16 = chunk_base((void *)t->w16, base * 2);
        s = sc;
        wd = t->wd;
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
        grad.load(x.g, e);
        ld_f32x4<Mem>(w_in, e * 4, x.w); ld_f32x4<Mem>(m_in, e * 4, x.m); ld_f32x4<Mem>(v_in, e * 4, x.v);
    }
    __device__ __forceinline__ void one(float S, float &w, float &m, float &v)
    {
        const bool nf = not_finite(S);
        bad |= nf;
        float mk = m, vk = v;
        moments<MODE>(S, w, wd, s, mk, vk);
        const float wk = __builtin_fmaf(-s.lr, direction<MODE>(w, wd, mk, vk, s), w);
        if (!(MODE & kModeGuard) || !nf) { m = mk; v = vk; w = wk; }
    }
    // compute = reduce (the sums, which settle `bad`) + update (everything else)
    __device__ __forceinline__ void reduce(Regs &x)
    {
        grad.sum(x.g, x.S);
        bad = bad || not_finite(x.S[0]) || not_finite(x.S[1]) || not_finite(x.S[2]) || not_finite(x.S[3]);
    }
    __device__ __forceinline__ void update(Regs &x)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) one(x.S[k], x.w[k], x.m[k], x.v[k]);
    }
    __device__ __forceinline__ void compute(Regs &x)
    {
        reduce(x);
        update(x);
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const
    {
        st_f32x4<Mem>(m_out, e * 4, x.m); st_f32x4<Mem>(v_out, e * 4, x.v); st_f32x4<Mem>(w_out, e * 4, x.w);
        if (EMIT16) st_f16x4<Mem>(w16, e * 2, x.w);
    }
    __device__ __forceinline__ void single(uint32_t j)
    {
        float w = ld_f32(w_in, j * 4), m = ld_f32(m_in, j * 4), v = ld_f32(v_in, j * 4);
        one(grad.sum1(j), w, m, v);
        st_f32(m_out, j * 4, m); st_f32(v_out, j * 4, v); st_f32(w_out, j * 4, w);
        if (EMIT16) st_f16(w16, j * 2, w);
    }
    template <int BLOCK> __device__ __forceinline__ void end_chunk(uint32_t) {}
};

template <int R, int MODE, int BLOCK, bool GF32 = false, int GROUPS = 2, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void fused_adam_kernel(const DevTensor *__restrict__ tensors,
                                                           const Chunk *__restrict__ chunks, StepScalars s,
                                                           FlagScratch *__restrict__ fs, int32_t *__restrict__ flag)
{
    FlagCount<BLOCK> fc;
    fc.arrive(fs);
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    AdamOp<GradSlices<R, GF32, Mem>, MODE, true> op;
    op.init(wh.t, wh.base, s);
    sweep_and_publish<BLOCK, GROUPS>(op, wh.len, fc, fs, flag);
}

// A plan with a single tensor (the contiguous case of Table 2 and of the standalone sweep of Section 6.1.1) needs
// no table: workgroup b takes chunk b, and the descriptor travels in the kernel arguments, so the two dependent
// scalar loads (table entry, then descriptor) in front of the first vector load fall away.  ~1 us of a launch-bound
// step.
template <int R, int MODE, int BLOCK, bool GF32 = false, int GROUPS = 2, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void fused_adam_flat_kernel(DevTensor t, StepScalars s, FlagScratch *__restrict__ fs,
                                                                int32_t *__restrict__ flag)
{
    FlagCount<BLOCK> fc;
    fc.arrive(fs);
    const uint64_t base = (uint64_t)blockIdx.x * s.chunk_elems;
    const uint64_t rem = t.numel - base;
    AdamOp<GradSlices<R, GF32, Mem>, MODE, true> op;
    op.init(&t, base, s);
    sweep_and_publish<BLOCK, GROUPS>(op, rem < s.chunk_elems ? (uint32_t)rem : s.chunk_elems, fc, fs, flag);
}

// The same step under the ordered persistent schedule (chunk_elems == BLOCK * 4 * GROUPS).
template <int R, int MODE, int BLOCK, bool GF32 = false, int GROUPS = 2>
__global__ __launch_bounds__(BLOCK) void fused_adam_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                                   const Chunk *__restrict__ chunks, uint32_t nfull,
                                                                   uint32_t nchunks, uint32_t span, StepScalars s,
                                                                   WorkQueue *__restrict__ q, int32_t *__restrict__ flag)
{
    typedef AdamOp<GradSlices<R, GF32>, MODE, true> Op;
    Op a, b;
    auto bind = [&](Op &op, uint32_t entry) {
        const Where wh = locate_at(tensors, chunks, entry, s.chunk_elems);
        op.init(wh.t, wh.base, s);
        return wh;
    };
    ordered_stream<BLOCK, GROUPS>(a, b, bind, nfull, nchunks, span, q);
    leave_queue<true>(a.bad | b.bad, q, flag);
}

// Unfused pipeline, optimizer stage: the same update from the stored fp32 sum; the cast kernel emits fp16.
// In whole-step-skip mode the flag is already final here (the reduce kernel set it), so an overflowed step
// writes nothing.
template <int MODE, int BLOCK, bool SUM16 = false, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void adam_from_sum_kernel(const DevTensor *__restrict__ tensors,
                                                              const Chunk *__restrict__ chunks, StepScalars s,
                                                              const int32_t *__restrict__ flag)
{
    if (!(MODE & kModeGuard) && *flag != 0) return;
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    AdamOp<typename std::conditional<SUM16, GradSumHalf<Mem>, GradSum<Mem>>::type, MODE, false> op;
    op.init(wh.t, wh.base, s);
    stream_chunk<BLOCK>(op, wh.len);
}

template <int MODE, int BLOCK, bool SUM16 = false>
__global__ __launch_bounds__(BLOCK) void adam_from_sum_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                                      const Chunk *__restrict__ chunks, uint32_t nfull,
                                                                      uint32_t nchunks, uint32_t span, StepScalars s,
                                                                      WorkQueue *__restrict__ q, const int32_t *__restrict__ flag)
{
    if (!(MODE & kModeGuard) && *flag != 0) return;
    typedef AdamOp<typename std::conditional<SUM16, GradSumHalf<>, GradSum<>>::type, MODE, false> Op;
    Op a, b;
    auto bind = [&](Op &op, uint32_t entry) {
        const Where wh = locate_at(tensors, chunks, entry, s.chunk_elems);
        op.init(wh.t, wh.base, s);
        return wh;
    };
    ordered_stream<BLOCK, 2>(a, b, bind, nfull, nchunks, span, q);
    leave_queue<false>(false, q, nullptr);
}

// ---------------------------------------------------------------------------------------------------
// Block-wide sum of two doubles: wave butterfly, then LDS across the waves.  Same order every run.
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

template <int BLOCK>
__device__ __forceinline__ void block_sum2(double &a, double &b)
{
    constexpr int kWaves = BLOCK / 64;
    a = wave_sum(a);
    b = wave_sum(b);
    if (kWaves > 1) {
        __shared__ double lds[2][kWaves];
        const int wave = threadIdx.x >> 6;
        __syncthreads();                 // a persistent workgroup calls this once per chunk: the last call's reads are over
        if ((threadIdx.x & 63) == 0) { lds[0][wave] = a; lds[1][wave] = b; }
        __syncthreads();
        a = lds[0][0];
        b = lds[1][0];
#pragma unroll
        for (int k = 1; k < kWaves; ++k) { a += lds[0][k]; b += lds[1][k]; }
    }
}

// ---------------------------------------------------------------------------------------------------
// LAMB phase 1: reduce, moments (written), and this chunk's sum(w^2), sum(u^2).
// ---------------------------------------------------------------------------------------------------
template <class Grad>
struct LambPhase1Op {
    static constexpr uint32_t kPack = kStatePack;
    typedef typename Grad::Mem Mem;
    Grad grad;
    gcbytes w_in, m_in, v_in;
    gbytes m_out, v_out;
    StepScalars s;
    float wd;
    bool bad = false;
    float sw = 0.f, su = 0.f;        // per lane: at most chunk_elems / BLOCK terms each, then double
    double *partials = nullptr;      // 2 per chunk, indexed by the chunk's position in tensor order
    struct Regs { typename Grad::Regs g; float S[4], w[4], m[4], v[4]; };

    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base, const StepScalars &sc)
    {
        grad.init(t, base);
        w_in = chunk_base((const void *)t->w_in, base * 4); m_in = chunk_base((const void *)t->m_in, base * 4);
        v_in = chunk_base((const void *)t->v_in, base * 4);
        m_out = chunk_base((void *)t->m_out, base * 4); v_out = chunk_base((void *)t->v_out, base * 4);
        s = sc;
        wd = t->wd;
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
        grad.load(x.g, e);
        ld_f32x4<Mem>(w_in, e * 4, x.w); ld_f32x4<Mem>(m_in, e * 4, x.m); ld_f32x4<Mem>(v_in, e * 4, x.v);
    }
    __device__ __forceinline__ void one(float S, float w, float &m, float &v)
    {
        bad |= not_finite(S);
        moments<0>(S, w, wd, s, m, v);
        const float u = direction<0>(w, wd, m, v, s);
        sw = __builtin_fmaf(w, w, sw);
        su = __builtin_fmaf(u, u, su);
    }
    __device__ __forceinline__ void reduce(Regs &x)
    {
        grad.sum(x.g, x.S);
        bad = bad || not_finite(x.S[0]) || not_finite(x.S[1]) || not_finite(x.S[2]) || not_finite(x.S[3]);
    }
    __device__ __forceinline__ void update(Regs &x)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) one(x.S[k], x.w[k], x.m[k], x.v[k]);
    }
    __device__ __forceinline__ void compute(Regs &x)
    {
        reduce(x);
        update(x);
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const
    {
        st_f32x4<Mem>(m_out, e * 4, x.m); st_f32x4<Mem>(v_out, e * 4, x.v);
    }
    __device__ __forceinline__ void single(uint32_t j)
    {
        const float w = ld_f32(w_in, j * 4);
        float m = ld_f32(m_in, j * 4), v = ld_f32(v_in, j * 4);
        one(grad.sum1(j), w, m, v);
        st_f32(m_out, j * 4, m); st_f32(v_out, j * 4, v);
    }
    // The chunk's two partial sums: lanes in fp32, then wave butterfly and LDS in double, always in the same order.
    template <int BLOCK> __device__ __forceinline__ void end_chunk(uint32_t slot)
    {
        double dw = sw, du = su;
        block_sum2<BLOCK>(dw, du);
        if (threadIdx.x == 0) {
            partials[2 * (uint64_t)slot] = dw;
            partials[2 * (uint64_t)slot + 1] = du;
        }
        sw = su = 0.f;
    }
};

template <class Grad, bool RAISE, int BLOCK>
__device__ __forceinline__ void lamb_phase1_body(const DevTensor *__restrict__ tensors, const Chunk *__restrict__ chunks,
                                                 const StepScalars &s, double *__restrict__ partials,
                                                 FlagScratch *__restrict__ fs, int32_t *__restrict__ flag)
{
    FlagCount<BLOCK> fc;
    if (RAISE) fc.arrive(fs);
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    LambPhase1Op<Grad> op;
    op.init(wh.t, wh.base, s);
    op.partials = partials;
    if (RAISE) {
        sweep_and_publish<BLOCK, 2>(op, wh.len, fc, fs, flag);
    } else {
        stream_chunk<BLOCK>(op, wh.len);
    }
    op.template end_chunk<BLOCK>(wh.slot);
}

template <class Grad, bool RAISE, int BLOCK>
__device__ __forceinline__ void lamb_phase1_ordered_body(const DevTensor *__restrict__ tensors, const Chunk *__restrict__ chunks,
                                                         uint32_t nfull, uint32_t nchunks, uint32_t span, const StepScalars &s,
                                                         double *__restrict__ partials, WorkQueue *__restrict__ q,
                                                         int32_t *__restrict__ flag)
{
    typedef LambPhase1Op<Grad> Op;
    Op a, b;
    a.partials = b.partials = partials;
    auto bind = [&](Op &op, uint32_t entry) {
        const Where wh = locate_at(tensors, chunks, entry, s.chunk_elems);
        op.init(wh.t, wh.base, s);
        return wh;
    };
    ordered_stream<BLOCK, 2>(a, b, bind, nfull, nchunks, span, q);
    leave_queue<RAISE>(a.bad | b.bad, q, flag);
}

template <int R, int BLOCK, bool GF32 = false>
__global__ __launch_bounds__(BLOCK) void lamb_phase1_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                                    const Chunk *__restrict__ chunks, uint32_t nfull,
                                                                    uint32_t nchunks, uint32_t span, StepScalars s,
                                                                    double *__restrict__ partials, WorkQueue *__restrict__ q,
                                                                    int32_t *__restrict__ flag)
{
    lamb_phase1_ordered_body<GradSlices<R, GF32>, true, BLOCK>(tensors, chunks, nfull, nchunks, span, s, partials, q, flag);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void lamb_phase1_from_sum_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                                             const Chunk *__restrict__ chunks, uint32_t nfull,
                                                                             uint32_t nchunks, uint32_t span, StepScalars s,
                                                                             double *__restrict__ partials,
                                                                             WorkQueue *__restrict__ q)
{
    lamb_phase1_ordered_body<GradSum<>, false, BLOCK>(tensors, chunks, nfull, nchunks, span, s, partials, q, nullptr);
}

template <int R, int BLOCK, bool GF32 = false, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void lamb_phase1_kernel(const DevTensor *__restrict__ tensors,
                                                            const Chunk *__restrict__ chunks, StepScalars s,
                                                            double *__restrict__ partials, FlagScratch *__restrict__ fs,
                                                            int32_t *__restrict__ flag)
{
    lamb_phase1_body<GradSlices<R, GF32, Mem>, true, BLOCK>(tensors, chunks, s, partials, fs, flag);
}

template <int BLOCK, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void lamb_phase1_from_sum_kernel(const DevTensor *__restrict__ tensors,
                                                                     const Chunk *__restrict__ chunks, StepScalars s,
                                                                     double *__restrict__ partials)
{
    lamb_phase1_body<GradSum<Mem>, false, BLOCK>(tensors, chunks, s, partials, nullptr, nullptr);
}

// LAMB second level: a tensor's chunk partials are added in a fixed order, so the result does not change between runs
// or between the launch shapes below.  The order is that of 1024 lanes: lane v adds the chunks v, v + 1024, ... into four
// independent strided partial sums, the lanes of each 64-wide wave are added by a butterfly and the 16 wave totals one
// after the other.  A workgroup of BLOCK < 1024 threads plays 1024 / BLOCK lanes per thread: its wave w stands for the
// waves w, w + BLOCK / 64, ... of the wide one, so every addition has the same operands.
constexpr int kNormBlock = 1024;
template <int BLOCK>
__device__ __forceinline__ void tensor_sums(const double *__restrict__ p, uint32_t n, double &sa, double &sb)
{
    constexpr int kRealWaves = BLOCK / 64, kWaves = kNormBlock / 64, kPlayed = kNormBlock / BLOCK;
    static_assert(kNormBlock % BLOCK == 0 && BLOCK % 64 == 0, "a workgroup plays whole waves");
    __shared__ double lds[2][kWaves];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();                     // a caller may use the function twice: the last call's reads are over
    if (n <= (uint32_t)kNormBlock) {
        // At most one chunk per lane: the lane's four strided sums are that chunk's value and zeros, i.e. the value
        // itself, so all loads can be issued at once (a lane that plays eight would otherwise wait eight times).
        double ta[kPlayed], tb[kPlayed];
#pragma unroll
        for (int j = 0; j < kPlayed; ++j) {
            const uint32_t c = (wave + j * kRealWaves) * 64 + lane;
            ta[j] = c < n ? p[2 * (uint64_t)c] : 0.0;
            tb[j] = c < n ? p[2 * (uint64_t)c + 1] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < kPlayed; ++j) {
            const uint32_t played_wave = wave + j * kRealWaves;
            if (played_wave * 64 < n) { ta[j] = wave_sum(ta[j]); tb[j] = wave_sum(tb[j]); }
            if (lane == 0) { lds[0][played_wave] = ta[j]; lds[1][played_wave] = tb[j]; }
        }
    } else
#pragma unroll
    for (int j = 0; j < kPlayed; ++j) {
        const uint32_t played_wave = wave + j * kRealWaves;
        double ta = 0.0, tb = 0.0;
        if (played_wave * 64 < n) {      // a wave without chunks adds up zeros: the same +0.0, without the work
            double a[4] = {0.0, 0.0, 0.0, 0.0}, b[4] = {0.0, 0.0, 0.0, 0.0};
            uint32_t c = played_wave * 64 + lane;
            for (; c + 3 * kNormBlock < n; c += 4 * kNormBlock) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    a[k] += p[2 * (uint64_t)(c + k * kNormBlock)];
                    b[k] += p[2 * (uint64_t)(c + k * kNormBlock) + 1];
                }
            }
            for (int k = 0; c < n; c += kNormBlock, ++k) {
                a[k] += p[2 * (uint64_t)c];
                b[k] += p[2 * (uint64_t)c + 1];
            }
            ta = wave_sum((a[0] + a[1]) + (a[2] + a[3]));
            tb = wave_sum((b[0] + b[1]) + (b[2] + b[3]));
        }
        if (lane == 0) { lds[0][played_wave] = ta; lds[1][played_wave] = tb; }
    }
    __syncthreads();
    sa = lds[0][0];
    sb = lds[1][0];
#pragma unroll
    for (int k = 1; k < kWaves; ++k) { sa += lds[0][k]; sb += lds[1][k]; }
}

// One workgroup per tensor.
[[maybe_unused]] static __global__ __launch_bounds__(kNormBlock) void lamb_norms_kernel(const DevTensor *__restrict__ tensors,
                                                                const double *__restrict__ partials,
                                                                double *__restrict__ sums)
{
    const DevTensor *t = tensors + blockIdx.x;
    double sa, sb;
    tensor_sums<kNormBlock>(partials + 2 * (uint64_t)t->first_chunk, t->num_chunks, sa, sb);
    if (threadIdx.x == 0) {
        sums[2 * (uint64_t)blockIdx.x] = sa;
        sums[2 * (uint64_t)blockIdx.x + 1] = sb;
    }
}

// LAMB phase 2: the same u from the stored moments, scaled by the tensor's ratio.  EMIT16 = false in the
// unfused pipeline, where a separate cast kernel writes the fp16 copy.
template <bool EMIT16, class Mem = Streaming>
struct LambPhase2Op {
    static constexpr uint32_t kPack = kStatePack;
    gcbytes w_in, m_new, v_new;
    gbytes w_out, w16;
    StepScalars s;
    float wd, step;
    struct Regs { float w[4], m[4], v[4]; };

    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base, const StepScalars &sc, float ratio)
    {
        w_in = chunk_base((const void *)t->w_in, base * 4);
        m_new = chunk_base((const void *)t->m_out, base * 4); v_new = chunk_base((const void *)t->v_out, base * 4);
        w_out = chunk_base((void *)t->w_out, base * 4); w16 = chunk_base((void *)t->w16, base * 2);
        s = sc;
        wd = t->wd;
        step = sc.lr * ratio;
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
        ld_f32x4<Mem>(w_in, e * 4, x.w); ld_f32x4<Mem>(m_new, e * 4, x.m); ld_f32x4<Mem>(v_new, e * 4, x.v);
    }
    __device__ __forceinline__ float one(float w, float m, float v) const
    {
        return __builtin_fmaf(-step, direction<0>(w, wd, m, v, s), w);
    }
    __device__ __forceinline__ void compute(Regs &x)
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) x.w[k] = one(x.w[k], x.m[k], x.v[k]);
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const
    {
        st_f32x4<Mem>(w_out, e * 4, x.w);
        if (EMIT16) st_f16x4<Mem>(w16, e * 2, x.w);
    }
    __device__ __forceinline__ void single(uint32_t j)
    {
        const float wn = one(ld_f32(w_in, j * 4), ld_f32(m_new, j * 4), ld_f32(v_new, j * 4));
        st_f32(w_out, j * 4, wn);
        if (EMIT16) st_f16(w16, j * 2, wn);
    }
    template <int BLOCK> __device__ __forceinline__ void end_chunk(uint32_t) {}
};

template <bool EMIT16, int BLOCK, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void lamb_phase2_kernel(const DevTensor *__restrict__ tensors,
                                                            const Chunk *__restrict__ chunks, StepScalars s,
                                                            const double *__restrict__ sums,
                                                            const int32_t *__restrict__ flag)
{
    if (*flag != 0) return;              // whole-step skip: w and w16 stay as they were
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    const double sw = sums[2 * (uint64_t)wh.tensor], su = sums[2 * (uint64_t)wh.tensor + 1];
    const float ratio = (sw > 0.0 && su > 0.0) ? (float)(__builtin_sqrt(sw) / __builtin_sqrt(su)) : 1.0f;
    LambPhase2Op<EMIT16, Mem> op;
    op.init(wh.t, wh.base, s, ratio);
    stream_chunk<BLOCK>(op, wh.len);
}

// Phase 2 of a plan whose tensors have few chunks each, with the second level folded in: every workgroup adds up the
// partials of its own tensor (the same additions in the same order as lamb_norms_kernel, so the same bits), which
// costs 16 bytes per chunk of the tensor from the L2 and saves a launch.  The workgroup of a tensor's first chunk
// also stores the sums, so that they can be read back as after the separate kernel.
template <bool EMIT16, int BLOCK, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void lamb_phase2_with_norms_kernel(const DevTensor *__restrict__ tensors,
                                                                       const Chunk *__restrict__ chunks, StepScalars s,
                                                                       const double *__restrict__ partials,
                                                                       double *__restrict__ sums,
                                                                       const int32_t *__restrict__ flag)
{
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    double sw, su;
    tensor_sums<BLOCK>(partials + 2 * (uint64_t)wh.t->first_chunk, wh.t->num_chunks, sw, su);
    if (wh.index == 0 && threadIdx.x == 0) {
        sums[2 * (uint64_t)wh.tensor] = sw;
        sums[2 * (uint64_t)wh.tensor + 1] = su;
    }
    if (*flag != 0) return;              // whole-step skip: w and w16 stay as they were
    const float ratio = (sw > 0.0 && su > 0.0) ? (float)(__builtin_sqrt(sw) / __builtin_sqrt(su)) : 1.0f;
    LambPhase2Op<EMIT16, Mem> op;
    op.init(wh.t, wh.base, s, ratio);
    stream_chunk<BLOCK>(op, wh.len);
}

template <bool EMIT16, int BLOCK>
__global__ __launch_bounds__(BLOCK) void lamb_phase2_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                                    const Chunk *__restrict__ chunks, uint32_t nfull,
                                                                    uint32_t nchunks, uint32_t span, StepScalars s,
                                                                    const double *__restrict__ sums, WorkQueue *__restrict__ q,
                                                                    const int32_t *__restrict__ flag)
{
    if (*flag != 0) return;
    typedef LambPhase2Op<EMIT16> Op;
    Op a, b;
    auto bind = [&](Op &op, uint32_t entry) {
        const Where wh = locate_at(tensors, chunks, entry, s.chunk_elems);
        const double sw = sums[2 * (uint64_t)wh.tensor], su = sums[2 * (uint64_t)wh.tensor + 1];
        const float ratio = (sw > 0.0 && su > 0.0) ? (float)(__builtin_sqrt(sw) / __builtin_sqrt(su)) : 1.0f;
        op.init(wh.t, wh.base, s, ratio);
        return wh;
    };
    ordered_stream<BLOCK, 2>(a, b, bind, nfull, nchunks, span, q);
    leave_queue<false>(false, q, nullptr);
}

// ---------------------------------------------------------------------------------------------------
// Unfused pipeline pieces: reduce to an fp32 buffer, and the fp32 -> fp16 cast.
// ---------------------------------------------------------------------------------------------------
template <int R, bool GF32, class Mem = Streaming>
struct ReduceOp {
    static constexpr uint32_t kPack = kStatePack;
    GradSlices<R, GF32, Mem> grad;
    gbytes gsum;
    bool bad = false;
    struct Regs { typename GradSlices<R, GF32, Mem>::Regs g; float S[4]; };
    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base)
    {
        grad.init(t, base);
        gsum = chunk_base((void *)t->gsum, base * 4);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const { grad.load(x.g, e); }
    __device__ __forceinline__ void compute(Regs &x)
    {
        grad.sum(x.g, x.S);
        bad = bad || not_finite(x.S[0]) || not_finite(x.S[1]) || not_finite(x.S[2]) || not_finite(x.S[3]);
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const { st_f32x4<Mem>(gsum, e * 4, x.S); }
    __device__ __forceinline__ void single(uint32_t j)
    {
        const float S = grad.sum1(j);
        bad |= not_finite(S);
        st_f32(gsum, j * 4, S);
    }
    template <int BLOCK> __device__ __forceinline__ void end_chunk(uint32_t) {}
};

template <int R, int BLOCK, bool GF32 = false, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void reduce_kernel(const DevTensor *__restrict__ tensors,
                                                       const Chunk *__restrict__ chunks, StepScalars s,
                                                       FlagScratch *__restrict__ fs, int32_t *__restrict__ flag)
{
    FlagCount<BLOCK> fc;
    fc.arrive(fs);
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    ReduceOp<R, GF32, Mem> op;
    op.init(wh.t, wh.base);
    stream_chunk<BLOCK>(op, wh.len);
    fc.settle(op.bad, fs, flag);
}

template <int R, int BLOCK, bool GF32 = false>
__global__ __launch_bounds__(BLOCK) void reduce_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                               const Chunk *__restrict__ chunks, uint32_t nfull,
                                                               uint32_t nchunks, uint32_t span, StepScalars s, WorkQueue *__restrict__ q,
                                                               int32_t *__restrict__ flag)
{
    typedef ReduceOp<R, GF32> Op;
    Op a, b;
    auto bind = [&](Op &op, uint32_t entry) {
        const Where wh = locate_at(tensors, chunks, entry, s.chunk_elems);
        op.init(wh.t, wh.base);
        return wh;
    };
    ordered_stream<BLOCK, 2>(a, b, bind, nfull, nchunks, span, q);
    leave_queue<true>(a.bad | b.bad, q, flag);
}

// The reduce stage of the fp16 all-reduce baseline: the sum of the R fp16 slices leaves as fp16.  The slices are
// added in double (exact for up to 16 fp16 values) and rounded to fp32, then to fp16, so that the stored value is
// fp16(fp32(sum)) whatever the order of the additions.  The flag is decided on the fp16 value: a finite sum beyond
// 65504 comes back as inf, as it would from an fp16 collective.
template <int R, class Mem = Streaming>
struct ReduceHalfOp {
    static constexpr uint32_t kPack = kStatePack;
    GradSlices<R, false, Mem> grad;
    gbytes gsum;
    bool bad = false;
    struct Regs { typename GradSlices<R, false, Mem>::Regs g; float S[4]; };
    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base)
    {
        grad.init(t, base);
        gsum = chunk_base((void *)t->gsum, base * 2);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const { grad.load(x.g, e); }
    static __device__ __forceinline__ float through_half(double s, bool &bad)
    {
        const float h = (float)to_half((float)s);
        bad = bad || not_finite(h);
        return h;
    }
    __device__ __forceinline__ void compute(Regs &x)
    {
        double a = (double)(float)x.g.g[0].x, b = (double)(float)x.g.g[0].y, c = (double)(float)x.g.g[0].z, d = (double)(float)x.g.g[0].w;
#pragma unroll
        for (int r = 1; r < R; ++r) {
            a += (double)(float)x.g.g[r].x; b += (double)(float)x.g.g[r].y; c += (double)(float)x.g.g[r].z; d += (double)(float)x.g.g[r].w;
        }
        x.S[0] = through_half(a, bad); x.S[1] = through_half(b, bad); x.S[2] = through_half(c, bad); x.S[3] = through_half(d, bad);
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const { st_f16x4<Mem>(gsum, e * 2, x.S); }
    __device__ __forceinline__ void single(uint32_t j)
    {
        double S = (double)ld_f16(grad.g[0], j * 2);
#pragma unroll
        for (int r = 1; r < R; ++r) S += (double)ld_f16(grad.g[r], j * 2);
        st_f16(gsum, j * 2, through_half(S, bad));
    }
    template <int BLOCK> __device__ __forceinline__ void end_chunk(uint32_t) {}
};

template <int R, int BLOCK, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void reduce_half_kernel(const DevTensor *__restrict__ tensors,
                                                            const Chunk *__restrict__ chunks, StepScalars s,
                                                            FlagScratch *__restrict__ fs, int32_t *__restrict__ flag)
{
    FlagCount<BLOCK> fc;
    fc.arrive(fs);
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    ReduceHalfOp<R, Mem> op;
    op.init(wh.t, wh.base);
    stream_chunk<BLOCK>(op, wh.len);
    fc.settle(op.bad, fs, flag);
}

template <int R, int BLOCK>
__global__ __launch_bounds__(BLOCK) void reduce_half_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                                    const Chunk *__restrict__ chunks, uint32_t nfull,
                                                                    uint32_t nchunks, uint32_t span, StepScalars s, WorkQueue *__restrict__ q,
                                                                    int32_t *__restrict__ flag)
{
    typedef ReduceHalfOp<R> Op;
    Op a, b;
    auto bind = [&](Op &op, uint32_t entry) {
        const Where wh = locate_at(tensors, chunks, entry, s.chunk_elems);
        op.init(wh.t, wh.base);
        return wh;
    };
    ordered_stream<BLOCK, 2>(a, b, bind, nfull, nchunks, span, q);
    leave_queue<true>(a.bad | b.bad, q, flag);
}

template <class Mem = Streaming>
struct CastOp {
    static constexpr uint32_t kPack = kStatePack;
    gcbytes w_new;
    gbytes w16;
    struct Regs { float w[4]; };
    __device__ __forceinline__ void init(const DevTensor *t, uint64_t base)
    {
        w_new = chunk_base((const void *)t->w_out, base * 4);
        w16 = chunk_base((void *)t->w16, base * 2);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const { ld_f32x4<Mem>(w_new, e * 4, x.w); }
    __device__ __forceinline__ void compute(Regs &) {}
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const { st_f16x4<Mem>(w16, e * 2, x.w); }
    __device__ __forceinline__ void single(uint32_t j) { st_f16(w16, j * 2, ld_f32(w_new, j * 4)); }
    template <int BLOCK> __device__ __forceinline__ void end_chunk(uint32_t) {}
};

// fp32 master weights -> fp16 copy.  `guarded`: leave w16 alone on overflow (whole-step skip).
template <int BLOCK, class Mem = Streaming>
__global__ __launch_bounds__(BLOCK) void cast_kernel(const DevTensor *__restrict__ tensors,
                                                     const Chunk *__restrict__ chunks, StepScalars s,
                                                     const int32_t *__restrict__ flag, int guarded)
{
    if (guarded && *flag != 0) return;
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    CastOp<Mem> op;
    op.init(wh.t, wh.base);
    stream_chunk<BLOCK>(op, wh.len);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void cast_ordered_kernel(const DevTensor *__restrict__ tensors,
                                                             const Chunk *__restrict__ chunks, uint32_t nfull,
                                                             uint32_t nchunks, uint32_t span, StepScalars s, WorkQueue *__restrict__ q,
                                                             const int32_t *__restrict__ flag, int guarded)
{
    if (guarded && *flag != 0) return;
    CastOp<> a, b;
    auto bind = [&](CastOp<> &op, uint32_t entry) {
        const Where wh = locate_at(tensors, chunks, entry, s.chunk_elems);
        op.init(wh.t, wh.base);
        return wh;
    };
    ordered_stream<BLOCK, 2>(a, b, bind, nfull, nchunks, span, q);
    leave_queue<false>(false, q, nullptr);
}

// ---------------------------------------------------------------------------------------------------
// Model-parallel epilogue (Fig. 3 with the schedule of Fig. 5, program 3) on one rank's slice:
//     out = Dropout(partial_0 + ... + partial_{R-1} + bias, p) + residual,  every tensor fp16.
// All streams are fp16, so a lane owns 8 consecutive elements and every access is 16 bytes (1 KiB per wave
// instruction).  2R + 4 bytes per element.  The dropout mask is a counter-based generator of the global element
// index (Philox4x32 with 10 rounds: counter = index / 4, key = seed, word index % 4), so that it does not depend on
// how the tensor is sliced or chunked; an element is kept iff its word >= floor(p 2^32).
// ---------------------------------------------------------------------------------------------------
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

struct EpilogueArgs {
    uint64_t numel;           // elements of this slice
    uint64_t first;           // global index of the slice's first element (multiple of 8)
    uint32_t hidden;          // H: the bias column of global element i is i % H (multiple of 8)
    uint32_t threshold;       // floor(p 2^32)
    uint32_t key0, key1;      // seed, low and high half
    float scale;              // 1 / (1 - p)
    const uint16_t *partial[CC_MAX_R];
    const uint16_t *bias;
    const uint16_t *residual;
    uint16_t *out;
    float *sum;               // unfused pipeline only: fp32 reduced partial outputs
};

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                              uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;      // the key schedule; the bump after the last round is unused
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The pointwise part for one element whose reduced sum is x_sum (fp32).
__device__ __forceinline__ float epilogue_value(float x_sum, float bias, float residual, bool keep, float scale)
{
    const float x = x_sum + bias;
    return (keep ? x * scale : 0.0f) + residual;
}

__device__ __forceinline__ f16x8 ld_f16x8(gcbytes b, uint32_t off) { return __builtin_nontemporal_load((const CCF_GLOBAL f16x8 *)(b + off)); }
__device__ __forceinline__ void st_f16x8(gbytes b, uint32_t off, f16x8 x) { __builtin_nontemporal_store(x, (CCF_GLOBAL f16x8 *)(b + off)); }

// Common part of the fused kernel and of the unfused pipeline's pointwise kernel: mask, bias column, output.
struct EpilogueTail {
    gcbytes res, bias;
    gbytes out;
    uint64_t gbase;           // global index of the chunk's first element
    uint32_t col_base;        // bias column of the chunk's first element
    uint32_t hidden, threshold, k0, k1;
    float scale;
    __device__ __forceinline__ void init(const EpilogueArgs &a, uint64_t base)
    {
        res = chunk_base((const void *)a.residual, base * 2);
        bias = (gcbytes)a.bias;
        out = chunk_base((void *)a.out, base * 2);
        gbase = a.first + base;
        col_base = (uint32_t)(gbase % a.hidden);
        hidden = a.hidden; threshold = a.threshold; k0 = a.key0; k1 = a.key1; scale = a.scale;
    }
    // words of the Philox block that holds global elements 4q .. 4q+3, q = (gbase + e) / 4
    __device__ __forceinline__ void words(uint32_t e, uint32_t (&w)[4]) const
    {
        const uint64_t block = (gbase + e) >> 2;
        philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), 0u, 0u, k0, k1, w);
    }
    __device__ __forceinline__ uint32_t column(uint32_t e) const { return (col_base + e) % hidden; }
    __device__ __forceinline__ void single(uint32_t j, float x_sum) const
    {
        uint32_t w[4];
        words(j, w);
        const bool keep = w[(gbase + j) & 3] >= threshold;
        st_f16(out, j * 2, epilogue_value(x_sum, ld_f16(bias, column(j) * 2), ld_f16(res, j * 2), keep, scale));
    }
};

template <int R>
struct FusedEpilogueOp {
    static constexpr uint32_t kPack = 8;
    gcbytes part[R];
    EpilogueTail t;
    struct Regs { f16x8 p[R]; f16x8 r; f16x8 b; uint32_t e; };
    __device__ __forceinline__ void init(const EpilogueArgs &a, uint64_t base)
    {
#pragma unroll
        for (int r = 0; r < R; ++r) part[r] = chunk_base((const void *)a.partial[r], base * 2);
        t.init(a, base);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
#pragma unroll
        for (int r = 0; r < R; ++r) x.p[r] = ld_f16x8(part[r], e * 2);
        x.r = ld_f16x8(t.res, e * 2);
        x.b = *(const CCF_GLOBAL f16x8 *)(t.bias + t.column(e) * 2);     // 8 columns never wrap: H and e are multiples of 8
        x.e = e;
    }
    __device__ __forceinline__ void compute(Regs &x)
    {
        uint32_t w[8];
        uint32_t lo[4], hi[4];
        t.words(x.e, lo);
        t.words(x.e + 4, hi);
#pragma unroll
        for (int k = 0; k < 4; ++k) { w[k] = lo[k]; w[4 + k] = hi[k]; }
        f16x8 o;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            float sum = (float)x.p[0][k];
#pragma unroll
            for (int r = 1; r < R; ++r) sum += (float)x.p[r][k];
            o[k] = to_half(epilogue_value(sum, (float)x.b[k], (float)x.r[k], w[k] >= t.threshold, t.scale));
        }
        x.r = o;
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const { st_f16x8(t.out, e * 2, x.r); }
    __device__ __forceinline__ void single(uint32_t j)
    {
        float sum = ld_f16(part[0], j * 2);
#pragma unroll
        for (int r = 1; r < R; ++r) sum += ld_f16(part[r], j * 2);
        t.single(j, sum);
    }
};

template <int R, int BLOCK, int GROUPS>
__global__ __launch_bounds__(BLOCK) void fused_epilogue_kernel(EpilogueArgs a)
{
    constexpr uint32_t kChunk = BLOCK * 8 * GROUPS;
    const uint64_t base = (uint64_t)blockIdx.x * kChunk;
    const uint64_t rem = a.numel - base;
    FusedEpilogueOp<R> op;
    op.init(a, base);
    stream_chunk<BLOCK, FusedEpilogueOp<R>, GROUPS>(op, rem < kChunk ? (uint32_t)rem : kChunk);
}

// Unfused pipeline: reduce the R partial outputs into an fp32 buffer (a lane owns 4 elements, so that the fp32
// stores of a wave are contiguous), then the pointwise kernel on that buffer.
template <int R>
struct EpilogueReduceOp {
    static constexpr uint32_t kPack = 4;
    gcbytes part[R];
    gbytes sum;
    struct Regs { f16x4 p[R]; float S[4]; };
    __device__ __forceinline__ void init(const EpilogueArgs &a, uint64_t base)
    {
#pragma unroll
        for (int r = 0; r < R; ++r) part[r] = chunk_base((const void *)a.partial[r], base * 2);
        sum = chunk_base((void *)a.sum, base * 4);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
#pragma unroll
        for (int r = 0; r < R; ++r) x.p[r] = ld_f16x4<Streaming>(part[r], e * 2);
    }
    __device__ __forceinline__ void compute(Regs &x)
    {
        x.S[0] = (float)x.p[0].x; x.S[1] = (float)x.p[0].y; x.S[2] = (float)x.p[0].z; x.S[3] = (float)x.p[0].w;
#pragma unroll
        for (int r = 1; r < R; ++r) { x.S[0] += (float)x.p[r].x; x.S[1] += (float)x.p[r].y; x.S[2] += (float)x.p[r].z; x.S[3] += (float)x.p[r].w; }
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const { st_f32x4<Streaming>(sum, e * 4, x.S); }
    __device__ __forceinline__ void single(uint32_t j)
    {
        float S = ld_f16(part[0], j * 2);
#pragma unroll
        for (int r = 1; r < R; ++r) S += ld_f16(part[r], j * 2);
        st_f32(sum, j * 4, S);
    }
};

struct EpiloguePointwiseOp {
    static constexpr uint32_t kPack = 4;
    gcbytes sum;
    EpilogueTail t;
    struct Regs { float S[4]; f16x4 r; f16x4 b; uint32_t e; };
    __device__ __forceinline__ void init(const EpilogueArgs &a, uint64_t base)
    {
        sum = chunk_base((const void *)a.sum, base * 4);
        t.init(a, base);
    }
    __device__ __forceinline__ void load(Regs &x, uint32_t e) const
    {
        ld_f32x4<Streaming>(sum, e * 4, x.S);
        x.r = ld_f16x4<Streaming>(t.res, e * 2);
        x.b = *(const CCF_GLOBAL f16x4 *)(t.bias + t.column(e) * 2);
        x.e = e;
    }
    __device__ __forceinline__ void compute(Regs &x)
    {
        uint32_t w[4];
        t.words(x.e, w);
        const float b[4] = {(float)x.b.x, (float)x.b.y, (float)x.b.z, (float)x.b.w};
        const float r[4] = {(float)x.r.x, (float)x.r.y, (float)x.r.z, (float)x.r.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) x.S[k] = epilogue_value(x.S[k], b[k], r[k], w[k] >= t.threshold, t.scale);
    }
    __device__ __forceinline__ void store(const Regs &x, uint32_t e) const { st_f16x4<Streaming>(t.out, e * 2, x.S); }
    __device__ __forceinline__ void single(uint32_t j) { t.single(j, ld_f32(sum, j * 4)); }
};

template <int R, int BLOCK>
__global__ __launch_bounds__(BLOCK) void epilogue_reduce_kernel(EpilogueArgs a)
{
    constexpr uint32_t kChunk = BLOCK * 4 * 2;
    const uint64_t base = (uint64_t)blockIdx.x * kChunk;
    const uint64_t rem = a.numel - base;
    EpilogueReduceOp<R> op;
    op.init(a, base);
    stream_chunk<BLOCK>(op, rem < kChunk ? (uint32_t)rem : kChunk);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void epilogue_pointwise_kernel(EpilogueArgs a)
{
    constexpr uint32_t kChunk = BLOCK * 4 * 2;
    const uint64_t base = (uint64_t)blockIdx.x * kChunk;
    const uint64_t rem = a.numel - base;
    EpiloguePointwiseOp op;
    op.init(a, base);
    stream_chunk<BLOCK>(op, rem < kChunk ? (uint32_t)rem : kChunk);
}

// Measurement aid: the memory pattern of the small-shard fused Adam step (one workgroup of BLOCK per BLOCK x 8 elements
// of one flat tensor, R fp16 + 3 fp32 streams in, 3 fp32 + 1 fp16 streams out) with parts taken away, to see where a
// launch-bound step's time goes.  WHAT 0: nothing (an empty workgroup), 1: the loads only, 2: the stores only,
// 3: loads and stores without the update arithmetic and without the flag.
template <int R, int WHAT, int BLOCK, class Mem>
__global__ __launch_bounds__(BLOCK) void pattern_probe_kernel(DevTensor t, StepScalars s, int32_t *__restrict__ sink)
{
    if (WHAT == 0) return;
    typedef AdamOp<GradSlices<R, false, Mem>, 0, true> Op;
    constexpr uint32_t kGroup = BLOCK * Op::kPack;
    Op op;
    op.init(&t, (uint64_t)blockIdx.x * (2 * kGroup), s);
    const uint32_t lane_e = threadIdx.x * Op::kPack;
    typename Op::Regs x[2];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        if (WHAT != 2) {
            op.load(x[g], g * kGroup + lane_e);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) { x[g].w[k] = (float)threadIdx.x; x[g].m[k] = (float)blockIdx.x; x[g].v[k] = 1.f; }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (WHAT == 1) {
        float acc = 0.f;
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            op.grad.sum(x[g].g, x[g].S);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc += x[g].S[k] + x[g].w[k] + x[g].m[k] + x[g].v[k];
        }
        if (acc == 123.456f) *sink = 1;              // keeps the loads alive; never true for the probe's data
        return;
    }
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        if (WHAT == 3) {
            op.grad.sum(x[g].g, x[g].S);
#pragma unroll
            for (int k = 0; k < 4; ++k) x[g].w[k] += x[g].S[k];
        }
        op.store(x[g], g * kGroup + lane_e);
    }
}

// Plain streaming copy, 16 bytes per lane, four accesses in flight per lane.
constexpr int kCopyBlock = 256;
[[maybe_unused]] static __global__ __launch_bounds__(kCopyBlock) void copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                          uint64_t n16)
{
    const uint64_t base = (uint64_t)blockIdx.x * (kCopyBlock * 4) + threadIdx.x;
    u32x4 x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t i = base + (uint64_t)k * kCopyBlock;
        if (i < n16) x[k] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t i = base + (uint64_t)k * kCopyBlock;
        if (i < n16) __builtin_nontemporal_store(x[k], dst + i);
    }
}

}  // namespace ccf
