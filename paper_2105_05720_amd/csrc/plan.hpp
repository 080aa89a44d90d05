// Shared by the host-side translation units of ccfused: the plan, the error helpers and the launch entry points of
// each kernel family.  The library is built from several sources only so that they compile in parallel; nothing
// here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "ccfused.h"
#include "kernels.hip.h"

namespace ccf {

constexpr int32_t kDefaultChunkElems = 4096;     // one sweep of a 512-thread workgroup (2 groups x 512 lanes x 4 elements)
constexpr int32_t kSmallChunkElems = 1024;       // one sweep of a 128-thread workgroup: more workgroups for small shards
constexpr int32_t kLargeChunkElems = 16384;      // four sweeps of a 512-thread workgroup: a quarter of the table and of the launches
constexpr uint64_t kSmallShardElems = 64u << 20; // below this many elements the default chunk is the small one (size sweep)
constexpr int32_t kMaxChunkElems = 1 << 24;      // lane offsets inside a chunk are 32-bit byte offsets
constexpr int kBigBlock = 512, kSmallBlock = 128;
constexpr int64_t kPerChunkDescriptorsMax = 2048; // chunks up to which a small-chunk layout keeps a descriptor per chunk (224 B each)
constexpr int kOrderedMaxF32Slices = 8;           // fp32 slices: the ordered schedule wins up to 8 (config-2 list: 3.18 against 3.41 ms), at 16 two chunks spill
constexpr int64_t kOrderedMinChunksPerCu = 8;    // below this many chunks per compute unit a plan keeps one workgroup per chunk
// AUTO cache policy: plain loads and write-through stores instead of non-temporal accesses while the step's buffers (R
// gradient slices, both copies of w, m, v and of the fp16 weights) total between these bounds, i.e. fit the 256 MB
// Infinity Cache.  Size sweep at R = 8, us per step: 6.2 against 7.9 at 2^20 elements (44 MB), 14.9 against 15.8 at 2^21
// (88 MB), 27.6 against 29.6 at 2^22 (176 MB), but 68.1 against 60.2 at 2^23 (352 MB).  Below 2^17 elements the
// non-temporal accesses are the faster ones by 1-6 % (LAMB at 2^14: 7.7 against 8.0 us), hence the lower bound.
constexpr uint64_t kResidentMinBytes = 4ull << 20, kResidentMaxBytes = 200ull << 20;
// ... and from there on non-temporal loads with write-through stores while one kernel stores less than this (see
// WriteThrough): what a launch writes then about fits the Infinity Cache.  Fused Adam (14 B stored per element) at
// R = 8: 141 against 147 us at 20 Mi elements, 160 against 157 us at 22 Mi; fused LAMB (8 B in its first sweep, 6 B in
// its second): 318 against 338 us at 36 Mi elements, 373 against 368 us at 40 Mi.
constexpr uint64_t kWriteThroughMaxStoreBytes = 288ull << 20;
constexpr uint32_t kAdamStoreBytes = 14, kLambStoreBytes = 8;      // per element: w', m', v', w16 / m', v'
inline int32_t auto_cache_policy(uint64_t footprint, uint64_t stored)
{
    if (footprint < kResidentMinBytes) return CC_CACHE_STREAMING;
    return footprint < kResidentMaxBytes ? CC_CACHE_RESIDENT : stored < kWriteThroughMaxStoreBytes ? CC_CACHE_WRITE_THROUGH : CC_CACHE_STREAMING;
}


// Records the message for cc_last_error() on this thread and returns the code.
int fail(cc_status code, const char *fmt, ...);
// CC_OK, or CC_ERR_HIP with the runtime's message if the last launch failed.
int launched(const char *what);

// One chunking of a plan's tensor list: the table (Section 5.4) and the descriptors that go with it.
struct Layout {
    int32_t chunk_elems = 0;
    int block = kBigBlock;                       // threads per workgroup of the streaming kernels
    int64_t chunks = 0;
    uint32_t nfull = 0;                          // full chunks; the ordered table lists them first, short last chunks behind
    uint32_t most_tensor_chunks = 0;             // chunks of the tensor that has the most
    std::vector<DevTensor> host_tensors;         // host mirror of the device descriptors (first_chunk / num_chunks of this chunking)
    DevTensor *d_tensors = nullptr;
    Chunk *d_chunks = nullptr;                   // tensor order
    std::vector<DevTensor> host_per_chunk;       // few chunks only: the descriptor once per chunk (see locate_at), else empty
    DevTensor *d_per_chunk = nullptr;
    // what the one-workgroup-per-chunk kernels take as their table
    const DevTensor *table_tensors() const { return d_per_chunk ? d_per_chunk : d_tensors; }
    const Chunk *table_chunks() const { return d_per_chunk ? nullptr : d_chunks; }
    Chunk *d_chunks_ordered = nullptr;           // the ordered schedule's order; only for kDefaultChunkElems
};

}  // namespace ccf

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess) return ccf::fail(CC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));     \
    } while (0)

struct cc_plan {
    int32_t T = 0, R = 0;
    std::vector<ccf::Layout> layouts;       // one per chunk size the plan was prepared for
    int active = 0;                         // the layout the step calls use
    int32_t chunk_choice = 0;               // what the caller asked for (0 = the size rule)
    ccf::FlagScratch *d_flag_scratch = nullptr;  // zero between launches
    bool ordered = false;                   // large shards: persistent workgroups take chunks in table order
    int32_t schedule = CC_SCHEDULE_AUTO;    // what the caller asked for
    unsigned ordered_grid = 0;              // workgroups of the ordered schedule (one per compute unit unless set)
    int32_t mem = CC_CACHE_STREAMING;       // the policy in use (other than STREAMING: small-chunk layouts only)
    int32_t mem_lamb = CC_CACHE_STREAMING;  // ... by LAMB's sweeps, which store fewer bytes per element
    int32_t cache_policy = CC_CACHE_AUTO;   // what the caller asked for
    int32_t cus = 0;                        // compute units of the device the plan was created on
    int32_t single = -1;                    // index of the only tensor with elements, or -1 if there are several (or none)
    ccf::WorkQueue *d_queue = nullptr;      // zero between launches
    uint64_t numel = 0;
    bool in_place = false;                  // some tensor has out == in
    bool grad_f32 = false;                  // gradient slices are fp32 instead of fp16
    std::vector<uint64_t> gsum_offset;      // element offset of each tensor in the unfused fp32 buffer
    uint64_t gsum_elems = 0;
    double *d_partials = nullptr;           // 2 per chunk of the finest layout (LAMB)
    double *d_sums = nullptr;               // 2 per tensor (LAMB)
    float *d_gsum = nullptr;                // unfused pipelines: cc_plan_reserve_unfused

    const ccf::Layout &lay() const { return layouts[(size_t)active]; }
    int64_t chunks() const { return lay().chunks; }
};

namespace ccf {

// Workgroups of an ordered launch: one per compute unit unless the caller chose a number; never more than there
// are pairs of chunks (every workgroup owns two entries without asking).
inline unsigned ordered_grid(const cc_plan *p)
{
    unsigned g = p->ordered_grid ? p->ordered_grid : (unsigned)p->cus;
    const unsigned most = (unsigned)((p->chunks() + 1) / 2);
    if (g > most) g = most;
    return g ? g : 1u;
}

#define FOR_EACH_R(X) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16)

// Every per-chunk streaming kernel exists for two workgroup sizes, and the small one for every cache policy; the
// plan's layout and policy pick one.  The statement given sees BLK (int) and MEM (Streaming, Resident or WriteThrough).
#define BY_BLOCK(p, ...) BY_BLOCK_MEM(p, (p)->mem, __VA_ARGS__)
#define BY_BLOCK_MEM(p, mem_, ...)                                                          \
    do {                                                                                    \
        if ((p)->lay().block == kBigBlock) { constexpr int BLK = kBigBlock; typedef Streaming MEM; __VA_ARGS__; }        \
        else if ((mem_) == CC_CACHE_RESIDENT) { constexpr int BLK = kSmallBlock; typedef Resident MEM; __VA_ARGS__; }    \
        else if ((mem_) == CC_CACHE_WRITE_THROUGH) { constexpr int BLK = kSmallBlock; typedef WriteThrough MEM; __VA_ARGS__; } \
        else { constexpr int BLK = kSmallBlock; typedef Streaming MEM; __VA_ARGS__; }                                    \
    } while (0)

// Chunks per ticket of the ordered schedule, by how many bytes a kernel moves per element: one counter serves the
// whole device at about one ticket per 12 ns, so a ticket has to stand for well over 100 KB of traffic.
enum SpanKind { kSpanAdam, kSpanPhase1, kSpanPhase2, kSpanReduce, kSpanFromSum, kSpanCast, kSpanKinds };
inline uint32_t span_of(SpanKind k)
{
    static const uint32_t chunks_per_ticket[kSpanKinds] = {1, 1, 2, 2, 1, 4};      // measured on the BERT-Large list
    return chunks_per_ticket[k];
}

// Arguments every ordered kernel starts with.
#define ORDERED_ARGS(p, kind) (p)->lay().d_tensors, (p)->lay().d_chunks_ordered, (p)->lay().nfull, (uint32_t)(p)->chunks(), ccf::span_of(kind)


// Launch entry points, one family per source file.  `mode` = kModeGuard | kModeL2 bits.
void launch_fused_adam_f16(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode);
void launch_fused_adam_f32(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode);
void launch_lamb_phase1(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st);
void launch_lamb_phase1_from_sum(const cc_plan *p, const StepScalars &s, hipStream_t st);
int lamb_phase2_impl(cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st, bool emit16);
int lamb_norms(cc_plan *p, hipStream_t st);
// Whether cc_fused_lamb_step lets every phase-2 workgroup add up its own tensor's partials instead of launching the
// second level: one workgroup per chunk, and no tensor with more chunks than kFoldNormsMaxChunks.  A workgroup reads 16
// bytes per chunk of its tensor, so the extra traffic grows with the square of a tensor's chunks.  One flat tensor,
// R = 8, us per step folded / three launches: 7.1 / 8.9 at one chunk, 9.2 / 10.7 at 128, 9.6 / 10.9 at 256, 11.4 / 11.6
// at 512, but 16.5 / 14.3 at 1024.
constexpr uint32_t kFoldNormsMaxChunks = 512;
inline bool norms_fold_into_phase2(const cc_plan *p)
{
    const Layout &L = p->lay();
    return !p->ordered && L.block == kSmallBlock && L.chunks > 0 && L.most_tensor_chunks <= kFoldNormsMaxChunks;
}
int lamb_phase2_with_norms(cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st);
void launch_reduce(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st);
void launch_reduce_half(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st);
void launch_adam_from_sum(const cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st, int mode, bool sum16);
int cast_launch(cc_plan *p, const StepScalars &s, const int32_t *flag, hipStream_t st, int guarded);
int clear_flag(int32_t *flag, hipStream_t st);
// One fp16-slice tensor, no plan: one workgroup of kSmallBlock per kSmallChunkElems elements, counted on `fs`.
void launch_fused_adam_flat_f16(const DevTensor &t, int R, unsigned grid, int32_t mem, const StepScalars &s, FlagScratch *fs,
                                int32_t *flag, hipStream_t st, int mode);

}  // namespace ccf
