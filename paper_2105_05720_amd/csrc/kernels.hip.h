// Device side of ccfused: streaming kernels for gfx950 (wave64, 128-bit global accesses).
//
// Every kernel here is bound by HBM bandwidth: per parameter it moves 2R bytes of fp16 gradients and
// 26 bytes of fp32/fp16 state against ~R + 30 scalar flops, so there is no contraction and no MFMA.
// The shape follows from that: one workgroup per chunk of one tensor (the chunk table replaces the
// per-thread tensor search of Section 5.4), every lane owns 8 consecutive elements per sweep so that
// one fp16 slice is one 16-byte load and each fp32 array is two, all loads of a sweep are issued before
// the first use, and results leave through 16-byte stores.  The reduced gradient stays in registers
// (Section 3.3, AllReduce Fuse: the output of the reduction is handed to the computation directly).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ccfused.h"

namespace ccf {

constexpr int kBlock = 256;            // 4 waves
constexpr int kPack = 8;               // elements per lane per sweep
constexpr int kSweep = kBlock * kPack; // elements one workgroup covers per sweep

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One tensor of the shard as the kernels see it.  Read through scalar loads: the index is uniform.
struct DevTensor {
    uint64_t numel;
    const float *w_in, *m_in, *v_in;
    float *w_out, *m_out, *v_out;
    uint16_t *w16;
    const uint16_t *grad[CC_MAX_R];
    float *gsum;              // unfused pipelines only: fp32 reduced gradient of this tensor
    float wd;
    uint32_t first_chunk;     // position of this tensor's first chunk in the table
    uint32_t num_chunks;
    uint32_t pad_;
};

// Chunk table entry: which tensor, and which chunk_elems-sized piece of it.
struct Chunk {
    uint32_t tensor;
    uint32_t index;
};

// Scalars of one step, precomputed on the host in double and rounded once.
struct StepScalars {
    float beta1, beta2;
    float omb1, omb2;         // 1 - beta
    float rc1, rc2;           // 1 / (1 - beta^t)
    float eps, lr;
    float inv_div;            // 1 / (loss_scale * (average ? R : 1))
    uint32_t chunk_elems;
};

enum : int { kModeGuard = 1, kModeL2 = 2 };

__device__ __forceinline__ bool not_finite(float x) { return !(__builtin_fabsf(x) <= 3.402823466e+38f); }

// Moments of one element from the reduced sum S (Fig. 4a, second and third statement).
template <int MODE>
__device__ __forceinline__ void moments(float S, float w, float wd, const StepScalars &s, float &m, float &v)
{
    float g = S * s.inv_div;
    if (MODE & kModeL2) g = __builtin_fmaf(wd, w, g);
    m = __builtin_fmaf(s.beta1, m, s.omb1 * g);
    v = __builtin_fmaf(s.beta2, v, (s.omb2 * g) * g);
}

// Update direction u from the new moments (Fig. 4a, bias corrections and the quotient), plus decoupled decay.
template <int MODE>
__device__ __forceinline__ float direction(float w, float wd, float m, float v, const StepScalars &s)
{
    const float mh = m * s.rc1;
    const float vh = v * s.rc2;
    float u = mh / (__builtin_sqrtf(vh) + s.eps);
    if (!(MODE & kModeL2)) u = __builtin_fmaf(wd, w, u);
    return u;
}

// Pointers read from a descriptor are generic; every buffer here is device memory, so address it as global
// (global_load/global_store instead of flat accesses, which also have to test for the LDS aperture).
#define CCF_GLOBAL __attribute__((address_space(1)))
typedef const CCF_GLOBAL float *gcf32;
typedef CCF_GLOBAL float *gf32;
typedef const CCF_GLOBAL uint16_t *gcu16;
typedef CCF_GLOBAL uint16_t *gu16;

__device__ __forceinline__ gcf32 as_global(const float *p) { return (gcf32)p; }
__device__ __forceinline__ gf32 as_global(float *p) { return (gf32)p; }
__device__ __forceinline__ gcu16 as_global(const uint16_t *p) { return (gcu16)p; }
__device__ __forceinline__ gu16 as_global(uint16_t *p) { return (gu16)p; }

__device__ __forceinline__ f32x4 ld4(gcf32 p) { return __builtin_nontemporal_load((const CCF_GLOBAL f32x4 *)p); }
__device__ __forceinline__ void st4(gf32 p, f32x4 x) { __builtin_nontemporal_store(x, (CCF_GLOBAL f32x4 *)p); }
__device__ __forceinline__ f16x8 ld8h(gcu16 p) { return __builtin_nontemporal_load((const CCF_GLOBAL f16x8 *)p); }
__device__ __forceinline__ void st8h(gu16 p, f16x8 x) { __builtin_nontemporal_store(x, (CCF_GLOBAL f16x8 *)p); }
__device__ __forceinline__ float ldh(gcu16 p) { return (float)*(const CCF_GLOBAL _Float16 *)p; }

// fp32 -> fp16, round to nearest even, of the fp32 value as stored.  The empty asm pins x in a register so
// that the compiler cannot merge the conversion with the fma that produced x into one mixed-precision fma
// (v_fma_mixlo_f16 rounds the exact product-sum straight to fp16, which can differ from rounding the fp32
// result by one fp16 ulp).
__device__ __forceinline__ _Float16 to_half(float x)
{
    asm volatile("" : "+v"(x));
    return (_Float16)x;
}
__device__ __forceinline__ void sth(gu16 p, float x) { *(CCF_GLOBAL _Float16 *)p = to_half(x); }

// Where a workgroup works: resolves its chunk to a tensor and an element range.
struct Where {
    const DevTensor *t;
    uint32_t tensor;          // index of t in the plan's tensor list
    uint64_t base;            // first element of the chunk inside the tensor
    uint32_t len;             // elements in this chunk (the tensor's last chunk may be short)
};

__device__ __forceinline__ Where locate(const DevTensor *__restrict__ tensors, const Chunk *__restrict__ chunks,
                                        uint32_t chunk_elems)
{
    const Chunk c = chunks[blockIdx.x];
    Where wh;
    wh.t = tensors + c.tensor;
    wh.tensor = c.tensor;
    wh.base = (uint64_t)c.index * chunk_elems;
    const uint64_t rem = wh.t->numel - wh.base;
    wh.len = rem < chunk_elems ? (uint32_t)rem : chunk_elems;
    return wh;
}

// Wave-level OR of a per-lane predicate, then at most one atomic per wave (and none in the normal case).
__device__ __forceinline__ void raise_flag(bool bad, int32_t *flag)
{
    const unsigned long long any = __builtin_amdgcn_ballot_w64(bad);
    if (any != 0ull && (threadIdx.x & 63) == 0) atomicOr(flag, 1);
}

__global__ void clear_flag_kernel(int32_t *flag) { *flag = 0; }

// Sum of the R slices for the 8 elements at p[r] + i, fixed rank order, fp32.
template <int R>
__device__ __forceinline__ void load_grads(const gcu16 *gp, uint32_t i, f16x8 (&g)[R])
{
#pragma unroll
    for (int r = 0; r < R; ++r) g[r] = ld8h(gp[r] + i);
}

template <int R>
__device__ __forceinline__ void reduce_grads(const f16x8 (&g)[R], float (&S)[kPack])
{
#pragma unroll
    for (int k = 0; k < kPack; ++k) S[k] = (float)g[0][k];
#pragma unroll
    for (int r = 1; r < R; ++r)
#pragma unroll
        for (int k = 0; k < kPack; ++k) S[k] += (float)g[r][k];
}

template <int R>
__device__ __forceinline__ float reduce_one(const gcu16 *gp, uint32_t j)
{
    float S = ldh(gp[0] + j);
#pragma unroll
    for (int r = 1; r < R; ++r) S += ldh(gp[r] + j);
    return S;
}

__device__ __forceinline__ void unpack(const f32x4 &a, const f32x4 &b, float (&x)[kPack])
{
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

__device__ __forceinline__ void store8(gf32 p, const float (&x)[kPack])
{
    st4(p, f32x4{x[0], x[1], x[2], x[3]});
    st4(p + 4, f32x4{x[4], x[5], x[6], x[7]});
}

__device__ __forceinline__ void store8h(gu16 p, const float (&x)[kPack])
{
    f16x8 h;
#pragma unroll
    for (int k = 0; k < kPack; ++k) h[k] = to_half(x[k]);    // v_cvt_f16_f32: round to nearest even, subnormals kept
    st8h(p, h);
}

// ---------------------------------------------------------------------------------------------------
// Fused reduce + Adam + fp16 emission: one pass, 2R + 26 bytes per parameter.
// ---------------------------------------------------------------------------------------------------
template <int R, int MODE>
__global__ __launch_bounds__(kBlock) void fused_adam_kernel(const DevTensor *__restrict__ tensors,
                                                            const Chunk *__restrict__ chunks, StepScalars s,
                                                            int32_t *__restrict__ flag)
{
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    const DevTensor *t = wh.t;
    const float wd = t->wd;
    gcu16 gp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) gp[r] = as_global(t->grad[r]) + wh.base;
    const gcf32 w_in = as_global(t->w_in) + wh.base, m_in = as_global(t->m_in) + wh.base, v_in = as_global(t->v_in) + wh.base;
    const gf32 w_out = as_global(t->w_out) + wh.base, m_out = as_global(t->m_out) + wh.base, v_out = as_global(t->v_out) + wh.base;
    const gu16 w16 = as_global(t->w16) + wh.base;

    bool bad = false;
    for (uint32_t i = threadIdx.x * kPack; i < wh.len; i += kSweep) {
        if (i + kPack <= wh.len) {
            f16x8 g[R];
            load_grads<R>(gp, i, g);
            const f32x4 w0 = ld4(w_in + i), w1 = ld4(w_in + i + 4);
            const f32x4 m0 = ld4(m_in + i), m1 = ld4(m_in + i + 4);
            const f32x4 v0 = ld4(v_in + i), v1 = ld4(v_in + i + 4);
            float S[kPack], w[kPack], m[kPack], v[kPack];
            reduce_grads<R>(g, S);
            unpack(w0, w1, w);
            unpack(m0, m1, m);
            unpack(v0, v1, v);
#pragma unroll
            for (int k = 0; k < kPack; ++k) {
                const bool nf = not_finite(S[k]);
                bad |= nf;
                float mk = m[k], vk = v[k];
                moments<MODE>(S[k], w[k], wd, s, mk, vk);
                const float u = direction<MODE>(w[k], wd, mk, vk, s);
                const float wk = __builtin_fmaf(-s.lr, u, w[k]);
                if (!(MODE & kModeGuard) || !nf) { m[k] = mk; v[k] = vk; w[k] = wk; }
            }
            store8(m_out + i, m);
            store8(v_out + i, v);
            store8(w_out + i, w);
            store8h(w16 + i, w);
        } else {
            for (uint32_t j = i; j < wh.len; ++j) {
                const float S = reduce_one<R>(gp, j);
                const bool nf = not_finite(S);
                bad |= nf;
                const float w = w_in[j];
                float m = m_in[j], v = v_in[j];
                float wn = w;
                if (!(MODE & kModeGuard) || !nf) {
                    moments<MODE>(S, w, wd, s, m, v);
                    wn = __builtin_fmaf(-s.lr, direction<MODE>(w, wd, m, v, s), w);
                }
                m_out[j] = m;
                v_out[j] = v;
                w_out[j] = wn;
                sth(w16 + j, wn);
            }
        }
    }
    raise_flag(bad, flag);
}

// ---------------------------------------------------------------------------------------------------
// Block-wide sum of two doubles: wave butterfly, then LDS across the 4 waves.  Same order every run.
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ void block_sum2(double &a, double &b)
{
    __shared__ double lds[2][kBlock / 64];
    a = wave_sum(a);
    b = wave_sum(b);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { lds[0][wave] = a; lds[1][wave] = b; }
    __syncthreads();
    a = lds[0][0] + lds[0][1] + lds[0][2] + lds[0][3];
    b = lds[1][0] + lds[1][1] + lds[1][2] + lds[1][3];
}

// ---------------------------------------------------------------------------------------------------
// LAMB phase 1: reduce, moments (written), and this chunk's sum(w^2), sum(u^2).
// FROM_SUM: the reduced gradient is read from the fp32 buffer of the unfused pipeline instead.
// ---------------------------------------------------------------------------------------------------
template <int R, bool FROM_SUM>
__global__ __launch_bounds__(kBlock) void lamb_phase1_kernel(const DevTensor *__restrict__ tensors,
                                                             const Chunk *__restrict__ chunks, StepScalars s,
                                                             double *__restrict__ partials,
                                                             int32_t *__restrict__ flag)
{
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    const DevTensor *t = wh.t;
    const float wd = t->wd;
    gcu16 gp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) gp[r] = FROM_SUM ? (gcu16)nullptr : as_global(t->grad[r]) + wh.base;
    const gcf32 gsum = FROM_SUM ? as_global((const float *)t->gsum) + wh.base : (gcf32)nullptr;
    const gcf32 w_in = as_global(t->w_in) + wh.base, m_in = as_global(t->m_in) + wh.base, v_in = as_global(t->v_in) + wh.base;
    const gf32 m_out = as_global(t->m_out) + wh.base, v_out = as_global(t->v_out) + wh.base;

    bool bad = false;
    float sw = 0.f, su = 0.f;            // per lane: at most chunk_elems / 256 terms each, then double
    for (uint32_t i = threadIdx.x * kPack; i < wh.len; i += kSweep) {
        if (i + kPack <= wh.len) {
            float S[kPack], w[kPack], m[kPack], v[kPack];
            if (FROM_SUM) {
                const f32x4 s0 = ld4(gsum + i), s1 = ld4(gsum + i + 4);
                const f32x4 w0 = ld4(w_in + i), w1 = ld4(w_in + i + 4);
                const f32x4 m0 = ld4(m_in + i), m1 = ld4(m_in + i + 4);
                const f32x4 v0 = ld4(v_in + i), v1 = ld4(v_in + i + 4);
                unpack(s0, s1, S); unpack(w0, w1, w); unpack(m0, m1, m); unpack(v0, v1, v);
            } else {
                f16x8 g[R];
                load_grads<R>(gp, i, g);
                const f32x4 w0 = ld4(w_in + i), w1 = ld4(w_in + i + 4);
                const f32x4 m0 = ld4(m_in + i), m1 = ld4(m_in + i + 4);
                const f32x4 v0 = ld4(v_in + i), v1 = ld4(v_in + i + 4);
                reduce_grads<R>(g, S);
                unpack(w0, w1, w); unpack(m0, m1, m); unpack(v0, v1, v);
            }
#pragma unroll
            for (int k = 0; k < kPack; ++k) {
                bad |= not_finite(S[k]);
                moments<0>(S[k], w[k], wd, s, m[k], v[k]);
                const float u = direction<0>(w[k], wd, m[k], v[k], s);
                sw = __builtin_fmaf(w[k], w[k], sw);
                su = __builtin_fmaf(u, u, su);
            }
            store8(m_out + i, m);
            store8(v_out + i, v);
        } else {
            for (uint32_t j = i; j < wh.len; ++j) {
                const float S = FROM_SUM ? gsum[j] : reduce_one<R>(gp, j);
                bad |= not_finite(S);
                const float w = w_in[j];
                float m = m_in[j], v = v_in[j];
                moments<0>(S, w, wd, s, m, v);
                const float u = direction<0>(w, wd, m, v, s);
                sw = __builtin_fmaf(w, w, sw);
                su = __builtin_fmaf(u, u, su);
                m_out[j] = m;
                v_out[j] = v;
            }
        }
    }
    double dw = sw, du = su;
    block_sum2(dw, du);
    if (threadIdx.x == 0) {
        partials[2 * (uint64_t)blockIdx.x] = dw;
        partials[2 * (uint64_t)blockIdx.x + 1] = du;
    }
    if (!FROM_SUM) raise_flag(bad, flag);
}

// LAMB second level: one workgroup per tensor adds that tensor's chunk partials in a fixed order.
__global__ __launch_bounds__(kBlock) void lamb_norms_kernel(const DevTensor *__restrict__ tensors,
                                                            const double *__restrict__ partials,
                                                            double *__restrict__ sums)
{
    const DevTensor *t = tensors + blockIdx.x;
    const uint32_t first = t->first_chunk, n = t->num_chunks;
    double a = 0.0, b = 0.0;
    for (uint32_t c = threadIdx.x; c < n; c += kBlock) {
        a += partials[2 * (uint64_t)(first + c)];
        b += partials[2 * (uint64_t)(first + c) + 1];
    }
    block_sum2(a, b);
    if (threadIdx.x == 0) {
        sums[2 * (uint64_t)blockIdx.x] = a;
        sums[2 * (uint64_t)blockIdx.x + 1] = b;
    }
}

// LAMB phase 2: the same u from the stored moments, scaled by the tensor's ratio.  EMIT16 = false in the
// unfused pipeline, where a separate cast kernel writes the fp16 copy.
template <bool EMIT16>
__global__ __launch_bounds__(kBlock) void lamb_phase2_kernel(const DevTensor *__restrict__ tensors,
                                                             const Chunk *__restrict__ chunks, StepScalars s,
                                                             const double *__restrict__ sums,
                                                             const int32_t *__restrict__ flag)
{
    if (*flag != 0) return;              // whole-step skip: w and w16 stay as they were
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    const DevTensor *t = wh.t;
    const float wd = t->wd;
    const double sw = sums[2 * (uint64_t)wh.tensor], su = sums[2 * (uint64_t)wh.tensor + 1];
    const float ratio = (sw > 0.0 && su > 0.0) ? (float)(__builtin_sqrt(sw) / __builtin_sqrt(su)) : 1.0f;
    const float step = s.lr * ratio;
    const gcf32 w_in = as_global(t->w_in) + wh.base;
    const gcf32 m_new = as_global((const float *)t->m_out) + wh.base, v_new = as_global((const float *)t->v_out) + wh.base;
    const gf32 w_out = as_global(t->w_out) + wh.base;
    const gu16 w16 = as_global(t->w16) + wh.base;
    for (uint32_t i = threadIdx.x * kPack; i < wh.len; i += kSweep) {
        if (i + kPack <= wh.len) {
            const f32x4 w0 = ld4(w_in + i), w1 = ld4(w_in + i + 4);
            const f32x4 m0 = ld4(m_new + i), m1 = ld4(m_new + i + 4);
            const f32x4 v0 = ld4(v_new + i), v1 = ld4(v_new + i + 4);
            float w[kPack], m[kPack], v[kPack];
            unpack(w0, w1, w); unpack(m0, m1, m); unpack(v0, v1, v);
#pragma unroll
            for (int k = 0; k < kPack; ++k) w[k] = __builtin_fmaf(-step, direction<0>(w[k], wd, m[k], v[k], s), w[k]);
            store8(w_out + i, w);
            if (EMIT16) store8h(w16 + i, w);
        } else {
            for (uint32_t j = i; j < wh.len; ++j) {
                const float w = w_in[j];
                const float wn = __builtin_fmaf(-step, direction<0>(w, wd, m_new[j], v_new[j], s), w);
                w_out[j] = wn;
                if (EMIT16) sth(w16 + j, wn);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Unfused pipeline pieces: reduce to an fp32 buffer, optimizer on that buffer, cast.
// ---------------------------------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(kBlock) void reduce_kernel(const DevTensor *__restrict__ tensors,
                                                        const Chunk *__restrict__ chunks, StepScalars s,
                                                        int32_t *__restrict__ flag)
{
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    const DevTensor *t = wh.t;
    gcu16 gp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) gp[r] = as_global(t->grad[r]) + wh.base;
    const gf32 gsum = as_global(t->gsum) + wh.base;
    bool bad = false;
    for (uint32_t i = threadIdx.x * kPack; i < wh.len; i += kSweep) {
        if (i + kPack <= wh.len) {
            f16x8 g[R];
            load_grads<R>(gp, i, g);
            float S[kPack];
            reduce_grads<R>(g, S);
#pragma unroll
            for (int k = 0; k < kPack; ++k) bad |= not_finite(S[k]);
            store8(gsum + i, S);
        } else {
            for (uint32_t j = i; j < wh.len; ++j) {
                const float S = reduce_one<R>(gp, j);
                bad |= not_finite(S);
                gsum[j] = S;
            }
        }
    }
    raise_flag(bad, flag);
}

template <int MODE>
__global__ __launch_bounds__(kBlock) void adam_from_sum_kernel(const DevTensor *__restrict__ tensors,
                                                               const Chunk *__restrict__ chunks, StepScalars s,
                                                               const int32_t *__restrict__ flag)
{
    if (!(MODE & kModeGuard) && *flag != 0) return;
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    const DevTensor *t = wh.t;
    const float wd = t->wd;
    const gcf32 gsum = as_global((const float *)t->gsum) + wh.base;
    const gcf32 w_in = as_global(t->w_in) + wh.base, m_in = as_global(t->m_in) + wh.base, v_in = as_global(t->v_in) + wh.base;
    const gf32 w_out = as_global(t->w_out) + wh.base, m_out = as_global(t->m_out) + wh.base, v_out = as_global(t->v_out) + wh.base;
    for (uint32_t i = threadIdx.x * kPack; i < wh.len; i += kSweep) {
        if (i + kPack <= wh.len) {
            const f32x4 s0 = ld4(gsum + i), s1 = ld4(gsum + i + 4);
            const f32x4 w0 = ld4(w_in + i), w1 = ld4(w_in + i + 4);
            const f32x4 m0 = ld4(m_in + i), m1 = ld4(m_in + i + 4);
            const f32x4 v0 = ld4(v_in + i), v1 = ld4(v_in + i + 4);
            float S[kPack], w[kPack], m[kPack], v[kPack];
            unpack(s0, s1, S); unpack(w0, w1, w); unpack(m0, m1, m); unpack(v0, v1, v);
#pragma unroll
            for (int k = 0; k < kPack; ++k) {
                const bool nf = not_finite(S[k]);
                float mk = m[k], vk = v[k];
                moments<MODE>(S[k], w[k], wd, s, mk, vk);
                const float wk = __builtin_fmaf(-s.lr, direction<MODE>(w[k], wd, mk, vk, s), w[k]);
                if (!(MODE & kModeGuard) || !nf) { m[k] = mk; v[k] = vk; w[k] = wk; }
            }
            store8(m_out + i, m);
            store8(v_out + i, v);
            store8(w_out + i, w);
        } else {
            for (uint32_t j = i; j < wh.len; ++j) {
                const float S = gsum[j];
                const float w = w_in[j];
                float m = m_in[j], v = v_in[j];
                float wn = w;
                if (!(MODE & kModeGuard) || !not_finite(S)) {
                    moments<MODE>(S, w, wd, s, m, v);
                    wn = __builtin_fmaf(-s.lr, direction<MODE>(w, wd, m, v, s), w);
                }
                m_out[j] = m;
                v_out[j] = v;
                w_out[j] = wn;
            }
        }
    }
}

// fp32 master weights -> fp16 copy.  `guarded`: leave w16 alone on overflow (whole-step skip).
__global__ __launch_bounds__(kBlock) void cast_kernel(const DevTensor *__restrict__ tensors,
                                                      const Chunk *__restrict__ chunks, StepScalars s,
                                                      const int32_t *__restrict__ flag, int guarded)
{
    if (guarded && *flag != 0) return;
    const Where wh = locate(tensors, chunks, s.chunk_elems);
    const DevTensor *t = wh.t;
    const gcf32 w_new = as_global((const float *)t->w_out) + wh.base;
    const gu16 w16 = as_global(t->w16) + wh.base;
    for (uint32_t i = threadIdx.x * kPack; i < wh.len; i += kSweep) {
        if (i + kPack <= wh.len) {
            const f32x4 w0 = ld4(w_new + i), w1 = ld4(w_new + i + 4);
            float w[kPack];
            unpack(w0, w1, w);
            store8h(w16 + i, w);
        } else {
            for (uint32_t j = i; j < wh.len; ++j) sth(w16 + j, w_new[j]);
        }
    }
}

// Plain streaming copy, 16 bytes per lane, four accesses in flight per lane.
__global__ __launch_bounds__(kBlock) void copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                      uint64_t n16)
{
    const uint64_t base = (uint64_t)blockIdx.x * (kBlock * 4) + threadIdx.x;
    u32x4 x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t i = base + (uint64_t)k * kBlock;
        if (i < n16) x[k] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t i = base + (uint64_t)k * kBlock;
        if (i < n16) __builtin_nontemporal_store(x[k], dst + i);
    }
}

}  // namespace ccf
