// Host side of ccfused: argument checks, the chunk table (Section 5.4), step scalars, kernel launches.
// Everything that touches a parameter runs in the kernels of kernels.hip.h; nothing here computes an update.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "plan.hpp"

using namespace ccf;

namespace {

thread_local char g_err[512] = "";

}  // namespace

namespace ccf {

int fail(cc_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return (int)code;
}

int launched(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(CC_ERR_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
    return CC_OK;
}

}  // namespace ccf

namespace {

int32_t resolve_chunk(int32_t chunk_elems, uint64_t total_elems = ~0ull)
{
    if (chunk_elems == 0) return total_elems < kSmallShardElems ? kSmallChunkElems : kDefaultChunkElems;
    if (chunk_elems < 0 || chunk_elems % 1024 != 0 || chunk_elems > kMaxChunkElems) return -1;
    return chunk_elems;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// One buffer of one tensor, for the overlap check of a plan.
struct Span {
    uintptr_t begin, end;
    int32_t tensor;
    int8_t kind;        // 0..2: w, m, v (in or out), 3: w16_out, 4: a gradient slice
    bool output;
};

const char *span_name(const Span &x)
{
    static const char *in_names[5] = {"w_in", "m_in", "v_in", "?", "grad"}, *out_names[4] = {"w_out", "m_out", "v_out", "w16_out"};
    return x.output ? out_names[x.kind] : in_names[x.kind];
}

// Rejects every overlap that involves an output buffer, within a tensor and across tensors, except an input that is
// exactly its own output (in place).  Sorting the buffers by start address makes one pass enough: an overlapping pair
// shows when the later one starts before the furthest end seen so far in the class it may not touch.
int check_overlaps(const cc_tensor *tensors, int32_t T, int32_t R, size_t grad_bytes, bool *in_place)
{
    std::vector<Span> spans;
    *in_place = false;
    try {
        spans.reserve((size_t)T * (size_t)(7 + R));
        for (int32_t t = 0; t < T; ++t) {
            const cc_tensor &x = tensors[t];
            if (x.numel == 0) continue;
            const void *ins[3] = {x.w_in, x.m_in, x.v_in};
            void *outs[3] = {x.w_out, x.m_out, x.v_out};
            for (int k = 0; k < 3; ++k) {
                const uintptr_t o = reinterpret_cast<uintptr_t>(outs[k]), i = reinterpret_cast<uintptr_t>(ins[k]);
                spans.push_back(Span{o, o + x.numel * 4, t, (int8_t)k, true});
                if (i == o) *in_place = true;                       // the input IS the output: one buffer
                else spans.push_back(Span{i, i + x.numel * 4, t, (int8_t)k, false});
            }
            const uintptr_t h = reinterpret_cast<uintptr_t>(x.w16_out);
            spans.push_back(Span{h, h + x.numel * 2, t, 3, true});
            for (int r = 0; r < R; ++r) {
                const uintptr_t g = reinterpret_cast<uintptr_t>(x.grad[r]);
                spans.push_back(Span{g, g + x.numel * grad_bytes, t, 4, false});
            }
        }
        std::sort(spans.begin(), spans.end(), [](const Span &a, const Span &b) { return a.begin < b.begin; });
    } catch (const std::bad_alloc &) {
        return fail(CC_ERR_NOMEM, "cc_plan_create: out of host memory");
    }
    const Span *far_out = nullptr, *far_in = nullptr;           // the output / input seen so far that ends last
    for (const Span &x : spans) {
        const Span *hit = nullptr;
        if (far_out && x.begin < far_out->end) hit = far_out;
        else if (x.output && far_in && x.begin < far_in->end) hit = far_in;
        if (hit)
            return fail(CC_ERR_ALIAS, "tensor %d %s overlaps tensor %d %s (only an input that is exactly its own output may share memory with an output)",
                        x.tensor, span_name(x), hit->tensor, span_name(*hit));
        if (x.output) { if (!far_out || x.end > far_out->end) far_out = &x; }
        else if (!far_in || x.end > far_in->end) far_in = &x;
    }
    return CC_OK;
}

// Settles what the step calls will use (layout, schedule, cache policy) from what the caller asked for.
void resolve_schedule(cc_plan *p)
{
    int want = p->chunk_choice;
    if (want == 0) want = p->numel < kSmallShardElems ? kSmallChunkElems : kDefaultChunkElems;
    p->active = 0;
    for (size_t i = 0; i < p->layouts.size(); ++i)
        if (p->layouts[i].chunk_elems == want) p->active = (int)i;
    const Layout &L = p->lay();
    if (p->schedule == CC_SCHEDULE_ORDERED) p->ordered = true;
    else if (p->schedule == CC_SCHEDULE_PER_CHUNK) p->ordered = false;
    else p->ordered = L.chunks >= kOrderedMinChunksPerCu * (int64_t)p->cus && !(p->grad_f32 && p->R > kOrderedMaxF32Slices);
    if (L.chunk_elems != kDefaultChunkElems || L.chunks == 0) p->ordered = false;
    if (p->cache_policy != CC_CACHE_AUTO) p->mem = p->mem_lamb = p->cache_policy;
    else {
        const uint64_t footprint = p->numel * ((p->grad_f32 ? 4u : 2u) * (uint64_t)p->R + 12u + 14u);
        p->mem = auto_cache_policy(footprint, p->numel * kAdamStoreBytes);
        p->mem_lamb = auto_cache_policy(footprint, p->numel * kLambStoreBytes);
    }
    if (L.block != kSmallBlock || p->ordered) p->mem = p->mem_lamb = CC_CACHE_STREAMING;
}

void free_layout(Layout &L)
{
    if (L.d_tensors) (void)hipFree(L.d_tensors);
    if (L.d_chunks) (void)hipFree(L.d_chunks);
    if (L.d_chunks_ordered) (void)hipFree(L.d_chunks_ordered);
    if (L.d_per_chunk) (void)hipFree(L.d_per_chunk);
    L.d_tensors = nullptr; L.d_chunks = nullptr; L.d_chunks_ordered = nullptr; L.d_per_chunk = nullptr;
}

}  // namespace

extern "C" {

const char *cc_last_error(void) { return g_err; }
int cc_version(void) { return CC_VERSION; }
int32_t cc_default_chunk_elems(void) { return kDefaultChunkElems; }

int64_t cc_chunk_count(const uint64_t *numels, int32_t T, int32_t chunk_elems)
{
    if (!numels && T > 0) return fail(CC_ERR_NULL, "cc_chunk_count: numels is NULL");
    if (T < 0) return fail(CC_ERR_ARG, "cc_chunk_count: T = %d", T);
    const int32_t ce = resolve_chunk(chunk_elems);
    if (ce < 0) return fail(CC_ERR_ARG, "chunk_elems = %d is not a positive multiple of 1024 up to 2^24", chunk_elems);
    int64_t total = 0;
    for (int32_t t = 0; t < T; ++t) {
        const uint64_t c = (numels[t] + (uint64_t)ce - 1) / (uint64_t)ce;
        if (c > 0xffffffffull) return fail(CC_ERR_ARG, "tensor %d has too many chunks", t);
        total += (int64_t)c;
    }
    if (total > 0x7fffffffll) return fail(CC_ERR_ARG, "%lld chunks exceed one launch; use a larger chunk_elems", (long long)total);
    return total;
}

int64_t cc_chunk_table_fill(const uint64_t *numels, int32_t T, int32_t chunk_elems, uint32_t *table, int64_t capacity)
{
    const int64_t need = cc_chunk_count(numels, T, chunk_elems);
    if (need < 0) return need;
    if (!table && need > 0) return fail(CC_ERR_NULL, "cc_chunk_table_fill: table is NULL");
    if (capacity < need) return fail(CC_ERR_ARG, "table capacity %lld < %lld chunks", (long long)capacity, (long long)need);
    const uint64_t ce = (uint64_t)resolve_chunk(chunk_elems);
    int64_t k = 0;
    for (int32_t t = 0; t < T; ++t) {
        const uint64_t c = (numels[t] + ce - 1) / ce;
        for (uint64_t i = 0; i < c; ++i, ++k) {
            table[2 * k] = (uint32_t)t;
            table[2 * k + 1] = (uint32_t)i;
        }
    }
    return k;
}

int64_t cc_ordered_table_fill(const uint64_t *numels, int32_t T, int32_t chunk_elems, uint32_t *table, int64_t capacity,
                              int64_t *full_chunks)
{
    const int64_t need = cc_chunk_count(numels, T, chunk_elems);
    if (need < 0) return need;
    if (!table && need > 0) return fail(CC_ERR_NULL, "cc_ordered_table_fill: table is NULL");
    if (capacity < need) return fail(CC_ERR_ARG, "table capacity %lld < %lld chunks", (long long)capacity, (long long)need);
    const uint64_t ce = (uint64_t)resolve_chunk(chunk_elems);
    int64_t k = 0, nfull = 0;
    for (int pass = 0; pass < 2; ++pass) {             // full chunks in tensor order, then the short last chunks
        for (int32_t t = 0; t < T; ++t) {
            const uint64_t full = numels[t] / ce, all = (numels[t] + ce - 1) / ce;
            for (uint64_t i = pass == 0 ? 0 : full; i < (pass == 0 ? full : all); ++i, ++k) {
                table[2 * k] = (uint32_t)t;
                table[2 * k + 1] = (uint32_t)i;
            }
        }
        if (pass == 0) nfull = k;
    }
    if (full_chunks) *full_chunks = nfull;
    return k;
}

int cc_plan_create(const cc_tensor *tensors, int32_t T, int32_t R, int32_t chunk_elems, cc_plan **out)
{
    return cc_plan_create_ex(tensors, T, R, chunk_elems, CC_GRAD_F16, out);
}

int cc_plan_create_ex(const cc_tensor *tensors, int32_t T, int32_t R, int32_t chunk_elems, int32_t grad_dtype, cc_plan **out)
{
    if (!out) return fail(CC_ERR_NULL, "cc_plan_create: out is NULL");
    *out = nullptr;
    if (!tensors) return fail(CC_ERR_NULL, "cc_plan_create: tensors is NULL");
    if (T <= 0) return fail(CC_ERR_ARG, "cc_plan_create: T = %d must be positive", T);
    if (R < 1 || R > CC_MAX_R) return fail(CC_ERR_ARG, "cc_plan_create: R = %d outside 1..%d", R, CC_MAX_R);
    if (grad_dtype != CC_GRAD_F16 && grad_dtype != CC_GRAD_F32) return fail(CC_ERR_ARG, "cc_plan_create: grad_dtype = %d", grad_dtype);
    if (resolve_chunk(chunk_elems) < 0) return fail(CC_ERR_ARG, "chunk_elems = %d is not a positive multiple of 1024 up to 2^24", chunk_elems);
    std::vector<uint64_t> numels;
    try {
        numels.resize((size_t)T);
    } catch (const std::bad_alloc &) {
        return fail(CC_ERR_NOMEM, "cc_plan_create: out of host memory");
    }
    for (int32_t t = 0; t < T; ++t) {
        const cc_tensor &x = tensors[t];
        numels[(size_t)t] = x.numel;
        if (x.numel == 0) continue;
        if (x.numel > (1ull << 40)) return fail(CC_ERR_ARG, "tensor %d: numel = %llu exceeds 2^40", t, (unsigned long long)x.numel);
        if (!std::isfinite(x.weight_decay)) return fail(CC_ERR_ARG, "tensor %d: weight_decay is not finite", t);
        const void *ptrs[7] = {x.w_in, x.m_in, x.v_in, x.w_out, x.m_out, x.v_out, x.w16_out};
        static const char *names[7] = {"w_in", "m_in", "v_in", "w_out", "m_out", "v_out", "w16_out"};
        for (int k = 0; k < 7; ++k) {
            if (!ptrs[k]) return fail(CC_ERR_NULL, "tensor %d: %s is NULL", t, names[k]);
            if (misaligned(ptrs[k])) return fail(CC_ERR_ALIGN, "tensor %d: %s is not 16-byte aligned", t, names[k]);
        }
        for (int r = 0; r < R; ++r) {
            if (!x.grad[r]) return fail(CC_ERR_NULL, "tensor %d: grad[%d] is NULL", t, r);
            if (misaligned(x.grad[r])) return fail(CC_ERR_ALIGN, "tensor %d: grad[%d] is not 16-byte aligned", t, r);
        }
    }
    bool in_place = false;
    {
        const int rc = check_overlaps(tensors, T, R, grad_dtype == CC_GRAD_F32 ? 4u : 2u, &in_place);
        if (rc) return rc;
    }
    // chunk sizes the plan is prepared for: the caller's, or the three the tuner chooses among (a size whose table
    // would not fit one launch is left out)
    int32_t sizes[3];
    int nsizes = 0;
    if (chunk_elems != 0) {
        const int64_t c = cc_chunk_count(numels.data(), T, chunk_elems);
        if (c < 0) return (int)c;
        sizes[nsizes++] = chunk_elems;
    } else {
        for (int32_t ce : {kSmallChunkElems, kDefaultChunkElems, kLargeChunkElems})
            if (cc_chunk_count(numels.data(), T, ce) >= 0) sizes[nsizes++] = ce;
        if (nsizes == 0) return (int)cc_chunk_count(numels.data(), T, kLargeChunkElems);     // leaves the message
    }

    cc_plan *p = new (std::nothrow) cc_plan;
    if (!p) return fail(CC_ERR_NOMEM, "cc_plan_create: out of host memory");
    p->T = T; p->R = R; p->in_place = in_place; p->chunk_choice = chunk_elems;
    p->grad_f32 = grad_dtype == CC_GRAD_F32;
    try {
        p->gsum_offset.resize((size_t)T);
        p->layouts.resize((size_t)nsizes);
        for (int i = 0; i < nsizes; ++i) p->layouts[(size_t)i].host_tensors.resize((size_t)T);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(CC_ERR_NOMEM, "cc_plan_create: out of host memory");
    }
    {
        uint64_t goff = 0, total = 0;
        int32_t nonempty = 0;
        for (int32_t t = 0; t < T; ++t) {
            p->gsum_offset[(size_t)t] = goff;
            goff += (tensors[t].numel + 7) / 8 * 8;            // every tensor starts 32-byte aligned in the fp32 buffer
            total += tensors[t].numel;
            if (tensors[t].numel > 0) { ++nonempty; p->single = t; }
        }
        if (nonempty != 1) p->single = -1;
        p->numel = total;
        p->gsum_elems = goff;
    }

#define PLAN_TRY(expr)                                                                             \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            fail(CC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));                              \
            cc_plan_destroy(p);                                                                    \
            return CC_ERR_HIP;                                                                     \
        }                                                                                          \
    } while (0)
    int64_t most_chunks = 0;
    for (int i = 0; i < nsizes; ++i) {
        Layout &L = p->layouts[(size_t)i];
        const int32_t ce = sizes[i];
        L.chunk_elems = ce;
        L.block = ce >= kDefaultChunkElems ? kBigBlock : kSmallBlock;
        L.chunks = cc_chunk_count(numels.data(), T, ce);
        if (L.chunks > most_chunks) most_chunks = L.chunks;
        uint64_t first = 0;
        for (int32_t t = 0; t < T; ++t) {
            const cc_tensor &x = tensors[t];
            DevTensor &d = L.host_tensors[(size_t)t];
            std::memset(&d, 0, sizeof(d));
            d.numel = x.numel;
            d.w_in = x.w_in; d.m_in = x.m_in; d.v_in = x.v_in;
            d.w_out = x.w_out; d.m_out = x.m_out; d.v_out = x.v_out;
            d.w16 = x.w16_out;
            for (int r = 0; r < R; ++r) d.grad[r] = x.grad[r];
            d.wd = x.weight_decay;
            d.first_chunk = (uint32_t)first;
            d.tensor = (uint32_t)t;
            d.num_chunks = (uint32_t)((x.numel + (uint64_t)ce - 1) / (uint64_t)ce);
            if (d.num_chunks > L.most_tensor_chunks) L.most_tensor_chunks = d.num_chunks;
            first += d.num_chunks;
        }
        std::vector<uint32_t> table;
        try {
            table.resize((size_t)(2 * L.chunks) + 2);
        } catch (const std::bad_alloc &) {
            cc_plan_destroy(p);
            return fail(CC_ERR_NOMEM, "cc_plan_create: out of host memory");
        }
        PLAN_TRY(hipMalloc((void **)&L.d_tensors, sizeof(DevTensor) * (size_t)T));
        PLAN_TRY(hipMemcpy(L.d_tensors, L.host_tensors.data(), sizeof(DevTensor) * (size_t)T, hipMemcpyHostToDevice));
        cc_chunk_table_fill(numels.data(), T, ce, table.data(), L.chunks);
        PLAN_TRY(hipMalloc((void **)&L.d_chunks, sizeof(Chunk) * (size_t)(L.chunks + 1)));
        if (L.chunks > 0) PLAN_TRY(hipMemcpy(L.d_chunks, table.data(), sizeof(Chunk) * (size_t)L.chunks, hipMemcpyHostToDevice));
        if (L.block == kSmallBlock && L.chunks > 0 && L.chunks <= kPerChunkDescriptorsMax) {
            try {
                L.host_per_chunk.reserve((size_t)L.chunks);
                for (int32_t t = 0; t < T; ++t)
                    for (uint32_t i = 0; i < L.host_tensors[(size_t)t].num_chunks; ++i) {
                        L.host_per_chunk.push_back(L.host_tensors[(size_t)t]);
                        L.host_per_chunk.back().chunk_index = i;
                    }
            } catch (const std::bad_alloc &) {
                cc_plan_destroy(p);
                return fail(CC_ERR_NOMEM, "cc_plan_create: out of host memory");
            }
            PLAN_TRY(hipMalloc((void **)&L.d_per_chunk, sizeof(DevTensor) * (size_t)L.chunks));
            PLAN_TRY(hipMemcpy(L.d_per_chunk, L.host_per_chunk.data(), sizeof(DevTensor) * (size_t)L.chunks, hipMemcpyHostToDevice));
        }
        if (ce == kDefaultChunkElems) {
            // The ordered schedule's table: the same entries, full chunks first (tensor order = address order inside
            // each arena), then the short last chunks, which take the unpipelined path.
            int64_t nfull = 0;
            cc_ordered_table_fill(numels.data(), T, ce, table.data(), L.chunks, &nfull);
            L.nfull = (uint32_t)nfull;
            PLAN_TRY(hipMalloc((void **)&L.d_chunks_ordered, sizeof(Chunk) * (size_t)(L.chunks + 1)));
            if (L.chunks > 0) PLAN_TRY(hipMemcpy(L.d_chunks_ordered, table.data(), sizeof(Chunk) * (size_t)L.chunks, hipMemcpyHostToDevice));
        }
    }
    PLAN_TRY(hipMalloc((void **)&p->d_partials, sizeof(double) * 2 * (size_t)(most_chunks + 1)));
    PLAN_TRY(hipMalloc((void **)&p->d_sums, sizeof(double) * 2 * (size_t)T));
    PLAN_TRY(hipMemset(p->d_sums, 0, sizeof(double) * 2 * (size_t)T));
    PLAN_TRY(hipMalloc((void **)&p->d_flag_scratch, sizeof(FlagScratch)));
    PLAN_TRY(hipMemset(p->d_flag_scratch, 0, sizeof(FlagScratch)));
    PLAN_TRY(hipMalloc((void **)&p->d_queue, sizeof(WorkQueue)));
    PLAN_TRY(hipMemset(p->d_queue, 0, sizeof(WorkQueue)));
    {
        int dev = 0, cus = 0;
        PLAN_TRY(hipGetDevice(&dev));
        PLAN_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        p->cus = cus > 0 ? cus : 1;
    }
#undef PLAN_TRY
    resolve_schedule(p);
    *out = p;
    return CC_OK;
}

int cc_plan_set_schedule(cc_plan *p, int32_t schedule, int32_t workgroups)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_set_schedule: plan is NULL");
    if (schedule != CC_SCHEDULE_AUTO && schedule != CC_SCHEDULE_PER_CHUNK && schedule != CC_SCHEDULE_ORDERED)
        return fail(CC_ERR_ARG, "cc_plan_set_schedule: schedule = %d", schedule);
    if (workgroups < 0 || workgroups > 65536) return fail(CC_ERR_ARG, "cc_plan_set_schedule: workgroups = %d outside 0..65536", workgroups);
    if (schedule == CC_SCHEDULE_ORDERED && p->lay().chunk_elems != kDefaultChunkElems)
        return fail(CC_ERR_ARG, "the ordered schedule needs chunk_elems = %d (plan uses %d)", kDefaultChunkElems, p->lay().chunk_elems);
    p->schedule = schedule;
    p->ordered_grid = (unsigned)workgroups;
    resolve_schedule(p);
    return CC_OK;
}

int cc_plan_set_chunk_elems(cc_plan *p, int32_t chunk_elems)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_set_chunk_elems: plan is NULL");
    if (chunk_elems != 0) {
        bool have = false;
        for (const Layout &L : p->layouts) have = have || L.chunk_elems == chunk_elems;
        if (!have) return fail(CC_ERR_ARG, "cc_plan_set_chunk_elems: the plan was not prepared for chunks of %d elements", chunk_elems);
        if (p->schedule == CC_SCHEDULE_ORDERED && chunk_elems != kDefaultChunkElems)
            return fail(CC_ERR_ARG, "the ordered schedule needs chunk_elems = %d", kDefaultChunkElems);
    }
    p->chunk_choice = chunk_elems;
    resolve_schedule(p);
    return CC_OK;
}

int cc_plan_layout(const cc_plan *p, int32_t *chunk_elems, int32_t *block_threads, int32_t *cache_policy)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_layout: plan is NULL");
    if (chunk_elems) *chunk_elems = p->lay().chunk_elems;
    if (block_threads) *block_threads = p->lay().block;
    if (cache_policy) *cache_policy = p->mem;
    return CC_OK;
}

int cc_plan_set_cache_policy(cc_plan *p, int32_t policy)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_set_cache_policy: plan is NULL");
    if (policy != CC_CACHE_AUTO && policy != CC_CACHE_STREAMING && policy != CC_CACHE_RESIDENT && policy != CC_CACHE_WRITE_THROUGH)
        return fail(CC_ERR_ARG, "cc_plan_set_cache_policy: policy = %d", policy);
    p->cache_policy = policy;
    resolve_schedule(p);
    return CC_OK;
}

int cc_plan_reserve_unfused(cc_plan *p)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_reserve_unfused: plan is NULL");
    if (p->d_gsum) return CC_OK;
    float *buf = nullptr;
    HIP_TRY(hipMalloc((void **)&buf, sizeof(float) * (size_t)(p->gsum_elems + 8)));
    for (Layout &L : p->layouts) {
        for (int32_t t = 0; t < p->T; ++t) L.host_tensors[(size_t)t].gsum = buf + p->gsum_offset[(size_t)t];
        hipError_t e = hipMemcpy(L.d_tensors, L.host_tensors.data(), sizeof(DevTensor) * (size_t)p->T, hipMemcpyHostToDevice);
        if (e == hipSuccess && L.d_per_chunk) {
            for (DevTensor &c : L.host_per_chunk) c.gsum = L.host_tensors[(size_t)c.tensor].gsum;
            e = hipMemcpy(L.d_per_chunk, L.host_per_chunk.data(), sizeof(DevTensor) * L.host_per_chunk.size(), hipMemcpyHostToDevice);
        }
        if (e != hipSuccess) {
            (void)hipFree(buf);
            return fail(CC_ERR_HIP, "cc_plan_reserve_unfused: %s", hipGetErrorString(e));
        }
    }
    p->d_gsum = buf;
    return CC_OK;
}

int cc_plan_queue_state(cc_plan *p, uint32_t *next_ticket, uint64_t *done_word, void *stream)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_queue_state: plan is NULL");
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    WorkQueue q;
    HIP_TRY(hipMemcpy(&q, p->d_queue, sizeof(q), hipMemcpyDeviceToHost));
    if (next_ticket) *next_ticket = q.next.v;
    if (done_word) *done_word = q.done.v;
    return CC_OK;
}

int cc_plan_schedule(const cc_plan *p, int32_t *schedule, int32_t *workgroups)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_schedule: plan is NULL");
    if (schedule) *schedule = p->ordered ? CC_SCHEDULE_ORDERED : CC_SCHEDULE_PER_CHUNK;
    if (workgroups) *workgroups = p->ordered ? (int32_t)ordered_grid(p) : (int32_t)p->chunks();
    return CC_OK;
}

int cc_plan_destroy(cc_plan *p)
{
    if (!p) return CC_OK;
    for (Layout &L : p->layouts) free_layout(L);
    if (p->d_partials) (void)hipFree(p->d_partials);
    if (p->d_sums) (void)hipFree(p->d_sums);
    if (p->d_gsum) (void)hipFree(p->d_gsum);
    if (p->d_flag_scratch) (void)hipFree(p->d_flag_scratch);
    if (p->d_queue) (void)hipFree(p->d_queue);
    delete p;
    return CC_OK;
}

int cc_plan_info(const cc_plan *p, uint64_t *numel, int64_t *chunks, uint64_t *table_bytes)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_info: plan is NULL");
    if (numel) *numel = p->numel;
    if (chunks) *chunks = p->chunks();
    if (table_bytes)      // of the layout and schedule in use
        *table_bytes = sizeof(Chunk) * (uint64_t)p->chunks() + sizeof(DevTensor) * (uint64_t)p->T
                       + sizeof(DevTensor) * (uint64_t)p->lay().host_per_chunk.size();
    return CC_OK;
}

int cc_lamb_norm_buffer(cc_plan *p, double **d_sums)
{
    if (!p || !d_sums) return fail(CC_ERR_NULL, "cc_lamb_norm_buffer: NULL argument");
    *d_sums = p->d_sums;
    return CC_OK;
}

int cc_lamb_norms_read(cc_plan *p, double *h_sums, void *stream)
{
    if (!p || !h_sums) return fail(CC_ERR_NULL, "cc_lamb_norms_read: NULL argument");
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    HIP_TRY(hipMemcpy(h_sums, p->d_sums, sizeof(double) * 2 * (size_t)p->T, hipMemcpyDeviceToHost));
    return CC_OK;
}

}  // extern "C"

namespace {

enum class Opt { Adam, Lamb };

int check_hparams(const cc_hparams *hp, const void *flag, Opt opt, int32_t R, bool in_place, int32_t chunk_elems, StepScalars *s)
{
    if (!hp) return fail(CC_ERR_NULL, "hparams is NULL");
    if (!flag) return fail(CC_ERR_NULL, "d_overflow_flag is NULL");
    if (hp->step < 1) return fail(CC_ERR_ARG, "step = %d must be >= 1", hp->step);
    if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f)) return fail(CC_ERR_ARG, "beta1 = %g outside [0, 1)", (double)hp->beta1);
    if (!(hp->beta2 >= 0.f && hp->beta2 < 1.f)) return fail(CC_ERR_ARG, "beta2 = %g outside [0, 1)", (double)hp->beta2);
    if (!(hp->loss_scale > 0.f) || !std::isfinite(hp->loss_scale)) return fail(CC_ERR_ARG, "loss_scale = %g must be positive and finite", (double)hp->loss_scale);
    if (!std::isfinite(hp->lr)) return fail(CC_ERR_ARG, "lr is not finite");
    if (!(hp->eps >= 0.f) || !std::isfinite(hp->eps)) return fail(CC_ERR_ARG, "eps = %g must be >= 0 and finite", (double)hp->eps);
    if (hp->grad_average != 0 && hp->grad_average != 1) return fail(CC_ERR_ARG, "grad_average = %d", hp->grad_average);
    if (hp->adam_mode != 0 && hp->adam_mode != 1) return fail(CC_ERR_ARG, "adam_mode = %d", hp->adam_mode);
    if (hp->skip_mode != 0 && hp->skip_mode != 1) return fail(CC_ERR_ARG, "skip_mode = %d", hp->skip_mode);
    if (opt == Opt::Lamb && (hp->adam_mode != 1 || hp->skip_mode != 0))
        return fail(CC_ERR_ARG, "LAMB supports adam_mode = 1 and skip_mode = 0 only");
    if (hp->skip_mode == 0 && in_place)
        return fail(CC_ERR_ALIAS, "skip_mode 0 (whole-step skip) needs out buffers distinct from the in buffers");
    const double b1 = hp->beta1, b2 = hp->beta2;
    const double c1 = 1.0 - std::pow(b1, (double)hp->step), c2 = 1.0 - std::pow(b2, (double)hp->step);
    s->beta1 = b1;
    s->beta2 = b2;
    s->omb1 = 1.0 - b1;
    s->omb2 = 1.0 - b2;
    s->rc1 = (float)(1.0 / c1);
    s->rc2 = (float)(1.0 / c2);
    s->eps = hp->eps;
    s->lr = hp->lr;
    s->inv_div = 1.0 / ((double)hp->loss_scale * (hp->grad_average ? (double)R : 1.0));
    s->chunk_elems = (uint32_t)chunk_elems;
    return CC_OK;
}

int check_step(const cc_plan *p, const cc_hparams *hp, const void *flag, Opt opt, StepScalars *s)
{
    if (!p) return fail(CC_ERR_NULL, "plan is NULL");
    return check_hparams(hp, flag, opt, p->R, p->in_place, p->lay().chunk_elems, s);
}

// The unfused pipelines need the plan's fp32 reduced-gradient buffer; a step call does not allocate it.
int ensure_gsum(const cc_plan *p)
{
    if (p->d_gsum) return CC_OK;
    return fail(CC_ERR_ARG, "the unfused pipelines need cc_plan_reserve_unfused(plan) first: step calls never allocate");
}

}  // namespace

extern "C" {

int cc_fused_adam_step(cc_plan *p, const cc_hparams *hp, int32_t *flag, void *stream)
{
    StepScalars s;
    int rc = check_step(p, hp, flag, Opt::Adam, &s);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (p->chunks() == 0) return clear_flag(flag, st);
    const int mode = (hp->skip_mode == 1 ? kModeGuard : 0) | (hp->adam_mode == 0 ? kModeL2 : 0);
    if (p->grad_f32) launch_fused_adam_f32(p, s, flag, st, mode);
    else launch_fused_adam_f16(p, s, flag, st, mode);
    return launched("fused_adam_kernel");
}

}  // extern "C"

// ---- a fused Adam step that allocates nothing ------------------------------------------------------------------------
// The only memory the small-shard kernel needs beyond the caller's buffers are the counting words of the overflow
// flag (FlagScratch).  For callers that cannot allocate they live in this array, one copy per device, for as long as
// the process runs.  In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device, and that pointer is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[sizeof(ccf::FlagScratch)];

namespace {

constexpr uint64_t kStaticMaxElems = 64ull << 20;        // 65536 workgroups of 1024 elements
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
ccf::FlagScratch *g_static_scratch[kMaxDevices] = {};

// The device address of this device's copy of `scratch` (looked up on the first call on each device).
int static_scratch(ccf::FlagScratch **out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CC_ERR_ARG, "device %d is outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_scratch[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(CC_ERR_HIP, "hipGetSymbolAddress returned no address for the scratch array");
        g_static_scratch[dev] = (ccf::FlagScratch *)ptr;
    }
    *out = g_static_scratch[dev];
    return CC_OK;
}

}  // namespace

extern "C" {

int cc_fused_adam_step_static(const cc_tensor *t, int32_t R, const cc_hparams *hp, int32_t *flag, void *stream)
{
    if (!t) return fail(CC_ERR_NULL, "cc_fused_adam_step_static: tensor is NULL");
    if (R < 1 || R > CC_MAX_R) return fail(CC_ERR_ARG, "cc_fused_adam_step_static: R = %d outside 1..%d", R, CC_MAX_R);
    if (t->numel > kStaticMaxElems)
        return fail(CC_ERR_ARG, "cc_fused_adam_step_static: numel = %llu exceeds the maximum of %llu elements; use a plan",
                    (unsigned long long)t->numel, (unsigned long long)kStaticMaxElems);
    bool in_place = false;
    if (t->numel > 0) {
        if (!std::isfinite(t->weight_decay)) return fail(CC_ERR_ARG, "weight_decay is not finite");
        const void *ptrs[7] = {t->w_in, t->m_in, t->v_in, t->w_out, t->m_out, t->v_out, t->w16_out};
        static const char *names[7] = {"w_in", "m_in", "v_in", "w_out", "m_out", "v_out", "w16_out"};
        for (int k = 0; k < 7; ++k) {
            if (!ptrs[k]) return fail(CC_ERR_NULL, "%s is NULL", names[k]);
            if (misaligned(ptrs[k])) return fail(CC_ERR_ALIGN, "%s is not 16-byte aligned", names[k]);
        }
        for (int r = 0; r < R; ++r) {
            if (!t->grad[r]) return fail(CC_ERR_NULL, "grad[%d] is NULL", r);
            if (misaligned(t->grad[r])) return fail(CC_ERR_ALIGN, "grad[%d] is not 16-byte aligned", r);
        }
        // the same overlap rule as a plan's, on this one tensor's buffers (a fixed array: nothing is allocated)
        struct Buf { uintptr_t begin, end; bool output; } bufs[7 + CC_MAX_R];
        int n = 0;
        for (int k = 0; k < 3; ++k) {
            const uintptr_t i = reinterpret_cast<uintptr_t>(ptrs[k]), o = reinterpret_cast<uintptr_t>(ptrs[3 + k]);
            bufs[n++] = Buf{o, o + t->numel * 4, true};
            if (i == o) in_place = true;
            else bufs[n++] = Buf{i, i + t->numel * 4, false};
        }
        const uintptr_t h = reinterpret_cast<uintptr_t>(t->w16_out);
        bufs[n++] = Buf{h, h + t->numel * 2, true};
        for (int r = 0; r < R; ++r) {
            const uintptr_t g = reinterpret_cast<uintptr_t>(t->grad[r]);
            bufs[n++] = Buf{g, g + t->numel * 2, false};
        }
        for (int a = 0; a < n; ++a)
            for (int b = a + 1; b < n; ++b)
                if ((bufs[a].output || bufs[b].output) && bufs[a].begin < bufs[b].end && bufs[b].begin < bufs[a].end)
                    return fail(CC_ERR_ALIAS, "two of the tensor's buffers overlap and one of them is an output");
    }
    StepScalars s;
    int rc = check_hparams(hp, flag, Opt::Adam, R, in_place, kSmallChunkElems, &s);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (t->numel == 0) return clear_flag(flag, st);
    FlagScratch *fs = nullptr;
    if ((rc = static_scratch(&fs))) return rc;
    DevTensor d;
    std::memset(&d, 0, sizeof(d));
    d.numel = t->numel;
    d.w_in = t->w_in; d.m_in = t->m_in; d.v_in = t->v_in;
    d.w_out = t->w_out; d.m_out = t->m_out; d.v_out = t->v_out;
    d.w16 = t->w16_out;
    for (int r = 0; r < R; ++r) d.grad[r] = t->grad[r];
    d.wd = t->weight_decay;
    const unsigned grid = (unsigned)((t->numel + (uint64_t)kSmallChunkElems - 1) / (uint64_t)kSmallChunkElems);
    const int mode = (hp->skip_mode == 1 ? kModeGuard : 0) | (hp->adam_mode == 0 ? kModeL2 : 0);
    const int32_t mem = auto_cache_policy(t->numel * (2u * (uint64_t)R + 26u), t->numel * kAdamStoreBytes);   // the plans' AUTO rule
    launch_fused_adam_flat_f16(d, R, grid, mem, s, fs, flag, st, mode);
    return launched("fused_adam_flat_kernel");
}

int cc_fused_lamb_phase1(cc_plan *p, const cc_hparams *hp, int32_t *flag, void *stream)
{
    StepScalars s;
    int rc = check_step(p, hp, flag, Opt::Lamb, &s);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (p->chunks() == 0) {
        if ((rc = clear_flag(flag, st))) return rc;
    } else {
        launch_lamb_phase1(p, s, flag, st);
        if ((rc = launched("lamb_phase1_kernel"))) return rc;
    }
    return lamb_norms(p, st);
}

int cc_fused_lamb_phase2(cc_plan *p, const cc_hparams *hp, const int32_t *flag, void *stream)
{
    StepScalars s;
    int rc = check_step(p, hp, flag, Opt::Lamb, &s);
    if (rc) return rc;
    return lamb_phase2_impl(p, s, flag, (hipStream_t)stream, true);
}

int cc_fused_lamb_step(cc_plan *p, const cc_hparams *hp, int32_t *flag, void *stream)
{
    StepScalars s;
    int rc = check_step(p, hp, flag, Opt::Lamb, &s);
    if (rc) return rc;
    if (norms_fold_into_phase2(p)) {
        // two launches instead of three: nobody reads the sums between the phases here
        hipStream_t st = (hipStream_t)stream;
        launch_lamb_phase1(p, s, flag, st);
        if ((rc = launched("lamb_phase1_kernel"))) return rc;
        return lamb_phase2_with_norms(p, s, flag, st);
    }
    if ((rc = cc_fused_lamb_phase1(p, hp, flag, stream))) return rc;
    return cc_fused_lamb_phase2(p, hp, flag, stream);
}

int cc_unfused_adam_step(cc_plan *p, const cc_hparams *hp, int32_t *flag, void *stream)
{
    return cc_unfused_adam_step_ex(p, hp, flag, stream, CC_GRAD_F32);
}

int cc_unfused_adam_step_ex(cc_plan *p, const cc_hparams *hp, int32_t *flag, void *stream, int32_t sum_dtype)
{
    StepScalars s;
    int rc = check_step(p, hp, flag, Opt::Adam, &s);
    if (rc) return rc;
    if (sum_dtype != CC_GRAD_F32 && sum_dtype != CC_GRAD_F16) return fail(CC_ERR_ARG, "sum_dtype = %d", sum_dtype);
    const bool sum16 = sum_dtype == CC_GRAD_F16;
    if (sum16 && p->grad_f32) return fail(CC_ERR_ARG, "an fp16 intermediate needs fp16 gradient slices");
    if ((rc = ensure_gsum(p))) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (p->chunks() == 0) return clear_flag(flag, st);
    if (sum16) launch_reduce_half(p, s, flag, st);
    else launch_reduce(p, s, flag, st);
    if ((rc = launched("reduce_kernel"))) return rc;
    const int mode = (hp->skip_mode == 1 ? kModeGuard : 0) | (hp->adam_mode == 0 ? kModeL2 : 0);
    launch_adam_from_sum(p, s, flag, st, mode, sum16);
    if ((rc = launched("adam_from_sum_kernel"))) return rc;
    return cast_launch(p, s, flag, st, hp->skip_mode == 0 ? 1 : 0);
}

int cc_unfused_lamb_step(cc_plan *p, const cc_hparams *hp, int32_t *flag, void *stream)
{
    StepScalars s;
    int rc = check_step(p, hp, flag, Opt::Lamb, &s);
    if (rc) return rc;
    if ((rc = ensure_gsum(p))) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (p->chunks() == 0) {
        if ((rc = clear_flag(flag, st))) return rc;
        return lamb_norms(p, st);
    }
    launch_reduce(p, s, flag, st);
    if ((rc = launched("reduce_kernel"))) return rc;
    launch_lamb_phase1_from_sum(p, s, st);
    if ((rc = launched("lamb_phase1_from_sum_kernel"))) return rc;
    if ((rc = lamb_norms(p, st))) return rc;
    if ((rc = lamb_phase2_impl(p, s, flag, st, false))) return rc;
    return cast_launch(p, s, flag, st, 1);
}

namespace {

int check_epilogue(const cc_epilogue *e, EpilogueArgs *a)
{
    if (!e) return fail(CC_ERR_NULL, "epilogue arguments are NULL");
    if (e->R < 1 || e->R > CC_MAX_R) return fail(CC_ERR_ARG, "epilogue: R = %d outside 1..%d", e->R, CC_MAX_R);
    if (e->hidden == 0 || e->hidden % 8 != 0) return fail(CC_ERR_ARG, "epilogue: hidden = %u must be a positive multiple of 8", e->hidden);
    if (e->first % 8 != 0) return fail(CC_ERR_ARG, "epilogue: first = %llu must be a multiple of 8", (unsigned long long)e->first);
    if (!(e->dropout_p >= 0.f && e->dropout_p < 1.f)) return fail(CC_ERR_ARG, "epilogue: dropout_p = %g outside [0, 1)", (double)e->dropout_p);
    if (e->numel > 0) {
        const void *ptrs[3] = {e->bias, e->residual, e->out};
        static const char *names[3] = {"bias", "residual", "out"};
        for (int k = 0; k < 3; ++k) {
            if (!ptrs[k]) return fail(CC_ERR_NULL, "epilogue: %s is NULL", names[k]);
            if (misaligned(ptrs[k])) return fail(CC_ERR_ALIGN, "epilogue: %s is not 16-byte aligned", names[k]);
        }
        for (int r = 0; r < e->R; ++r) {
            if (!e->partial[r]) return fail(CC_ERR_NULL, "epilogue: partial[%d] is NULL", r);
            if (misaligned(e->partial[r])) return fail(CC_ERR_ALIGN, "epilogue: partial[%d] is not 16-byte aligned", r);
        }
    }
    std::memset(a, 0, sizeof(*a));
    a->numel = e->numel; a->first = e->first; a->hidden = e->hidden;
    a->threshold = (uint32_t)std::floor((double)e->dropout_p * 4294967296.0);
    a->key0 = (uint32_t)e->seed; a->key1 = (uint32_t)(e->seed >> 32);
    a->scale = (float)(1.0 / (1.0 - (double)e->dropout_p));
    for (int r = 0; r < e->R; ++r) a->partial[r] = e->partial[r];
    a->bias = e->bias; a->residual = e->residual; a->out = e->out;
    return CC_OK;
}

constexpr int kEpilogueBlock = 512;             // the unfused pipeline's kernels (64, 128 and 256 threads are 2-8 % slower)
// The fused kernel spends about half as long on the mask generator's integer arithmetic as on its memory traffic, and
// overlaps the two best as single-wave workgroups that come and go independently: 78.0 us against 86.0 us with 512
// threads on the [8, 1024, 3072] tensor (256 threads: 78.5 us; 128: 81.8 us).  Two groups of 8 elements per lane where
// the call is bound by HBM, one where it stays in the Infinity Cache (its 1/8 slices: 10.0 and 20.9 us against 10.4
// and 22.3 us with two).
constexpr int kEpilogueFusedBlock = 64;
constexpr uint64_t kEpilogueCachedBytes = 200ull << 20;

int epilogue_grid(uint64_t numel, uint32_t chunk, unsigned *grid)
{
    const uint64_t g = (numel + chunk - 1) / chunk;
    if (g > 0x7fffffffull) return fail(CC_ERR_ARG, "epilogue: too many elements for one launch");
    *grid = (unsigned)g;
    return CC_OK;
}

}  // namespace

int cc_fused_epilogue(const cc_epilogue *e, void *stream)
{
    EpilogueArgs a;
    int rc = check_epilogue(e, &a);
    if (rc) return rc;
    if (e->numel == 0) return CC_OK;
    const int groups = e->numel * (2u * (uint64_t)e->R + 4u) < kEpilogueCachedBytes ? 1 : 2;
    unsigned grid;
    if ((rc = epilogue_grid(e->numel, (uint32_t)(kEpilogueFusedBlock * 8 * groups), &grid))) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (groups == 2) switch (e->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_epilogue_kernel<r, kEpilogueFusedBlock, 2>), dim3(grid), dim3(kEpilogueFusedBlock), 0, st, a); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
    else switch (e->R) {
#define CASE(r) case r: hipLaunchKernelGGL((fused_epilogue_kernel<r, kEpilogueFusedBlock, 1>), dim3(grid), dim3(kEpilogueFusedBlock), 0, st, a); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
    return launched("fused_epilogue_kernel");
}

int cc_unfused_epilogue(const cc_epilogue *e, float *d_sum, void *stream)
{
    EpilogueArgs a;
    int rc = check_epilogue(e, &a);
    if (rc) return rc;
    if (e->numel == 0) return CC_OK;
    if (!d_sum) return fail(CC_ERR_NULL, "epilogue: d_sum_scratch is NULL");
    if (misaligned(d_sum)) return fail(CC_ERR_ALIGN, "epilogue: d_sum_scratch is not 16-byte aligned");
    a.sum = d_sum;
    unsigned grid;
    if ((rc = epilogue_grid(e->numel, kEpilogueBlock * 4 * 2, &grid))) return rc;
    hipStream_t st = (hipStream_t)stream;
    switch (e->R) {
#define CASE(r) case r: hipLaunchKernelGGL((epilogue_reduce_kernel<r, kEpilogueBlock>), dim3(grid), dim3(kEpilogueBlock), 0, st, a); break;
        FOR_EACH_R(CASE)
#undef CASE
    }
    if ((rc = launched("epilogue_reduce_kernel"))) return rc;
    hipLaunchKernelGGL((epilogue_pointwise_kernel<kEpilogueBlock>), dim3(grid), dim3(kEpilogueBlock), 0, st, a);
    return launched("epilogue_pointwise_kernel");
}

int cc_plan_autotune(cc_plan *p, const cc_hparams *hp, int32_t optimizer, int32_t *flag, void *stream, float *best_ms,
                     float *per_chunk_ms)
{
    if (!p) return fail(CC_ERR_NULL, "cc_plan_autotune: plan is NULL");
    if (optimizer != 0 && optimizer != 1) return fail(CC_ERR_ARG, "cc_plan_autotune: optimizer = %d", optimizer);
    if (p->in_place) return fail(CC_ERR_ALIAS, "cc_plan_autotune needs out buffers distinct from the in buffers");
    {
        StepScalars s;
        const int rc = check_step(p, hp, flag, optimizer == 0 ? Opt::Adam : Opt::Lamb, &s);
        if (rc) return rc;
    }
    hipStream_t st = (hipStream_t)stream;
    struct Candidate { int32_t chunk_elems, schedule; unsigned workgroups; int32_t cache; };
    const Candidate keep{p->chunk_choice, p->schedule, p->ordered_grid, p->cache_policy};
    // one workgroup per chunk under the plan's current layout first: its time is what per_chunk_ms reports
    std::vector<Candidate> cand;
    try {
        const int32_t current = p->lay().chunk_elems;
        cand.push_back(Candidate{current, CC_SCHEDULE_PER_CHUNK, 0u, CC_CACHE_STREAMING});
        if (p->lay().block == kSmallBlock)
            for (int32_t c : {CC_CACHE_RESIDENT, CC_CACHE_WRITE_THROUGH}) cand.push_back(Candidate{current, CC_SCHEDULE_PER_CHUNK, 0u, c});
        for (const Layout &L : p->layouts) {
            if (L.chunks == 0) continue;
            if (L.chunk_elems != current) {
                cand.push_back(Candidate{L.chunk_elems, CC_SCHEDULE_PER_CHUNK, 0u, CC_CACHE_STREAMING});
                if (L.block == kSmallBlock)
                    for (int32_t c : {CC_CACHE_RESIDENT, CC_CACHE_WRITE_THROUGH}) cand.push_back(Candidate{L.chunk_elems, CC_SCHEDULE_PER_CHUNK, 0u, c});
            }
            if (L.chunk_elems == kDefaultChunkElems) {
                const unsigned cus = (unsigned)p->cus;
                for (unsigned w : {cus, cus > 1 ? cus / 2 : 1u, cus * 2}) cand.push_back(Candidate{L.chunk_elems, CC_SCHEDULE_ORDERED, w, CC_CACHE_STREAMING});
            }
        }
    } catch (const std::bad_alloc &) {
        return fail(CC_ERR_NOMEM, "cc_plan_autotune: out of host memory");
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(CC_ERR_HIP, "hipEventCreate failed"); }
    auto apply = [&](const Candidate &c) {
        p->chunk_choice = c.chunk_elems; p->schedule = c.schedule; p->ordered_grid = c.workgroups; p->cache_policy = c.cache;
        resolve_schedule(p);
    };
    int rc = CC_OK, best = -1;
    float best_time = 0.f;
    constexpr int kTrials = 3;
    for (size_t c = 0; c < cand.size() && rc == CC_OK; ++c) {
        apply(cand[c]);
        float ms = 0.f;
        for (int i = 0; i <= kTrials && rc == CC_OK; ++i) {          // the first run warms up
            if (i == 1 && hipEventRecord(e0, st) != hipSuccess) rc = fail(CC_ERR_HIP, "hipEventRecord failed");
            if (rc == CC_OK) rc = optimizer == 0 ? cc_fused_adam_step(p, hp, flag, stream) : cc_fused_lamb_step(p, hp, flag, stream);
        }
        if (rc == CC_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                            hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
            rc = fail(CC_ERR_HIP, "timing a trial step failed");
        if (rc != CC_OK) break;
        ms /= (float)kTrials;
        if (c == 0 && per_chunk_ms) *per_chunk_ms = ms;
        if (best < 0 || ms < best_time) { best = (int)c; best_time = ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != CC_OK) {
        apply(keep);
        return rc;
    }
    apply(cand[(size_t)best]);
    if (best_ms) *best_ms = best_time;
    return CC_OK;
}

int cc_device_info(int32_t *cus, int32_t *clock_khz, int32_t *bus_bits, uint64_t *total_bytes)
{
    int dev = 0, v = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (cus) { HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev)); *cus = v; }
    if (clock_khz) { HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMemoryClockRate, dev)); *clock_khz = v; }
    if (bus_bits) { HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMemoryBusWidth, dev)); *bus_bits = v; }
    if (total_bytes) {
        size_t free_b = 0, total_b = 0;
        HIP_TRY(hipMemGetInfo(&free_b, &total_b));
        *total_bytes = (uint64_t)total_b;
    }
    return CC_OK;
}

int cc_pattern_probe(const cc_tensor *t, int32_t R, int32_t what, int32_t cache_policy, int32_t *d_sink, void *stream)
{
    if (!t || !d_sink) return fail(CC_ERR_NULL, "cc_pattern_probe: NULL argument");
    if (R != 4 && R != 8) return fail(CC_ERR_ARG, "cc_pattern_probe: R = %d (4 or 8)", R);
    if (what < 0 || what > 3) return fail(CC_ERR_ARG, "cc_pattern_probe: what = %d outside 0..3", what);
    if (cache_policy != CC_CACHE_STREAMING && cache_policy != CC_CACHE_RESIDENT && cache_policy != CC_CACHE_WRITE_THROUGH)
        return fail(CC_ERR_ARG, "cc_pattern_probe: cache_policy = %d", cache_policy);
    if (t->numel == 0 || t->numel % kSmallChunkElems != 0 || t->numel / kSmallChunkElems > 0x7fffffffull)
        return fail(CC_ERR_ARG, "cc_pattern_probe: numel = %llu must be a positive multiple of %d", (unsigned long long)t->numel, kSmallChunkElems);
    const void *ptrs[7] = {t->w_in, t->m_in, t->v_in, t->w_out, t->m_out, t->v_out, t->w16_out};
    for (const void *q : ptrs)
        if (!q || misaligned(q)) return fail(CC_ERR_ALIGN, "cc_pattern_probe: a state pointer is NULL or not 16-byte aligned");
    for (int r = 0; r < R; ++r)
        if (!t->grad[r] || misaligned(t->grad[r])) return fail(CC_ERR_ALIGN, "cc_pattern_probe: grad[%d] is NULL or not 16-byte aligned", r);
    DevTensor d;
    std::memset(&d, 0, sizeof(d));
    d.numel = t->numel;
    d.w_in = t->w_in; d.m_in = t->m_in; d.v_in = t->v_in;
    d.w_out = t->w_out; d.m_out = t->m_out; d.v_out = t->v_out;
    d.w16 = t->w16_out;
    for (int r = 0; r < R; ++r) d.grad[r] = t->grad[r];
    StepScalars s;
    std::memset(&s, 0, sizeof(s));
    s.chunk_elems = (uint32_t)kSmallChunkElems;
    const dim3 grid((unsigned)(t->numel / kSmallChunkElems)), block(kSmallBlock);
    hipStream_t st = (hipStream_t)stream;
#define PROBE(r, w, M) hipLaunchKernelGGL((pattern_probe_kernel<r, w, kSmallBlock, M>), grid, block, 0, st, d, s, d_sink)
#define PROBE_W(r, M) switch (what) { case 0: PROBE(r, 0, M); break; case 1: PROBE(r, 1, M); break; case 2: PROBE(r, 2, M); break; default: PROBE(r, 3, M); break; }
    if (cache_policy == CC_CACHE_RESIDENT) { if (R == 4) { PROBE_W(4, Resident) } else { PROBE_W(8, Resident) } }
    else if (cache_policy == CC_CACHE_WRITE_THROUGH) { if (R == 4) { PROBE_W(4, WriteThrough) } else { PROBE_W(8, WriteThrough) } }
    else { if (R == 4) { PROBE_W(4, Streaming) } else { PROBE_W(8, Streaming) } }
#undef PROBE_W
#undef PROBE
    return launched("pattern_probe_kernel");
}

int cc_copy_probe(void *dst, const void *src, uint64_t bytes, void *stream)
{
    if (!dst || !src) return fail(CC_ERR_NULL, "cc_copy_probe: NULL pointer");
    if (bytes % 16 != 0) return fail(CC_ERR_ARG, "cc_copy_probe: bytes = %llu is not a multiple of 16", (unsigned long long)bytes);
    if (misaligned(dst) || misaligned(src)) return fail(CC_ERR_ALIGN, "cc_copy_probe: pointers must be 16-byte aligned");
    if (bytes == 0) return CC_OK;
    const uint64_t n16 = bytes / 16;
    const uint64_t per_block = (uint64_t)kCopyBlock * 4;
    const uint64_t blocks = (n16 + per_block - 1) / per_block;
    if (blocks > 0x7fffffffull) return fail(CC_ERR_ARG, "cc_copy_probe: too large for one launch");
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(kCopyBlock), 0, (hipStream_t)stream, (u32x4 *)dst, (const u32x4 *)src, n16);
    return launched("copy_kernel");
}

}  // extern "C"
