// Streaming kernels of the OSP synchronization step for gfx950 (MI355X):
// PS aggregate + SGD-momentum update with fused PGP importance, worker-side
// stage install, and LGP.  All three are HBM-bound (< 0.5 flop per byte).
//
// Shape that measured fastest on MI355X: one-wavefront workgroups (64 lanes),
// each lane issues ALL its 16-byte loads, computes, issues its stores and the
// wave ends.  A wave that ends does not wait for its stores, so the slot is
// reused at once and stores cost no occupancy; small workgroups also keep the
// set of DRAM pages that are open at any moment small.  With the default chunk
// of 256 elements a lane handles exactly one float4 position.
//
// Work decomposition: a chunk is a run of at most chunk_elems consecutive
// elements of ONE tensor.  Chunk starts are multiples of 4 elements, so every
// 16-byte access is aligned and never straddles a bitmap word; only the last
// float4 of a tensor can be ragged.  For a layer-granular GIB the chunks of
// each stage are listed in a compact index list (ascending addresses), so a
// launch has no idle workgroups.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// one IEEE rounding per operator: parameters must come out bit-identical to a
// plain CPU evaluation, and the element-granular partition depends on it
#pragma clang fp contract(off)

namespace osp {

constexpr int kBlock = 64;             // one wavefront per workgroup
constexpr int kVec = 4;                // fp32 per 16-byte access
constexpr int kStride = kBlock * kVec; // elements covered by one block-wide access

struct Chunk {
    long long start;                   // arena element index, multiple of 4
    int len;                           // 1 .. chunk_elems
    int layer;
};

using f4 = __attribute__((ext_vector_type(4))) float;
using u4 = __attribute__((ext_vector_type(4))) unsigned int;

__device__ __forceinline__ f4 ld_stream(const float *p)
{   // read-once data (gradients): keep it from displacing reusable lines
    return __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
}
__device__ __forceinline__ f4 ld_keep(const float *p)
{
    return *reinterpret_cast<const f4 *>(p);
}
__device__ __forceinline__ void st_keep(float *p, f4 v)
{
    *reinterpret_cast<f4 *>(p) = v;
}
__device__ __forceinline__ void st_stream(float *p, f4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(p));
}

// Which of the 4 elements at chunk position i does this call touch?
// Bit j set = element i+j is inside the chunk and (if MASKED) in the stage.
template <bool MASKED>
__device__ __forceinline__ unsigned lane_mask(int rem, long long e, int stage,
                                              const uint32_t *__restrict__ bitmap)
{
    unsigned m = rem >= kVec ? 0xFu : ((1u << rem) - 1u);
    if (MASKED) {
        const unsigned word = bitmap[e >> 5];
        const unsigned imp = (word >> (unsigned)(e & 31)) & 0xFu; // 1 = important = stage 1
        m &= (stage == 1) ? imp : (~imp & 0xFu);
    }
    return m;
}

// Which chunk does workgroup `b` own?  With a stage list (layer-granular GIB,
// stage 1 or 2) the b-th entry of the list; otherwise chunk b itself.
__device__ __forceinline__ Chunk owned_chunk(const Chunk *__restrict__ chunks,
                                             const int *__restrict__ stage_list, unsigned b)
{
    return chunks[stage_list ? stage_list[b] : (int)b];
}
__device__ __forceinline__ int owned_chunk_index(const int *__restrict__ stage_list, unsigned b)
{
    return stage_list ? stage_list[b] : (int)b;
}

// Deterministic sum of one double per lane over the wavefront (fixed butterfly).
// The result is valid in lane 0.
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x += __shfl_down(x, off, 64);
    return x;
}

__device__ __forceinline__ uint32_t importance_key(float q)
{   // q >= 0 or NaN: the bit pattern orders like the value; one canonical NaN on top
    return (q != q) ? 0x7FC00000u : (__float_as_uint(q) & 0x7FFFFFFFu);
}

// ---------------------------------------------------------------------------
// PS aggregate + update (+ PGP importance), one stage.
// ---------------------------------------------------------------------------
struct AggArgs {
    const Chunk *chunks;
    const int *stage_list;             // chunk indices of this stage, or null = every chunk
    const uint32_t *bitmap;            // bit per element (element-granular GIB), when MASKED
    float *P;
    float *V;
    const float *grads;
    long long worker_stride;
    const float *weights;              // [N] device, used when WEIGHTED
    double *partial;                   // [n_chunks] importance partial of this stage
    uint32_t *key;                     // [arena] when KEYS
    int n_workers;
    int stage;
    float inv_n, lr, mu;
};

constexpr int kWorkerBlock = 16;       // gradient streams loaded before they are summed

template <bool MASKED, bool WEIGHTED, bool KEYS>
__global__ __launch_bounds__(kBlock) void k_aggregate_update(const AggArgs a)
{
    const int ci = owned_chunk_index(a.stage_list, blockIdx.x);
    const Chunk c = a.chunks[ci];
    const int N = a.n_workers;
    double imp = 0.0;
    for (int i = threadIdx.x * kVec; i < c.len; i += kStride) {
        const long long e = c.start + i;
        const unsigned m = lane_mask<MASKED>(c.len - i, e, a.stage, a.bitmap);
        if (m == 0)
            continue;
        const f4 p = ld_stream(a.P + e);
        const f4 v = ld_stream(a.V + e);
        const float *gp = a.grads + e;
        f4 acc;
        for (int w0 = 0; w0 < N; w0 += kWorkerBlock) {
            f4 g[kWorkerBlock];
#pragma unroll
            for (int j = 0; j < kWorkerBlock; ++j)
                if (w0 + j < N)
                    g[j] = ld_stream(gp + (long long)(w0 + j) * a.worker_stride);
#pragma unroll
            for (int j = 0; j < kWorkerBlock; ++j)
                if (w0 + j < N) {
                    f4 term = g[j];
                    if (WEIGHTED)
                        term = term * a.weights[w0 + j];
                    if (w0 + j == 0)
                        acc = term;
                    else
                        acc = acc + term;
                }
        }
        const f4 gbar = WEIGHTED ? acc : acc * a.inv_n;
        const f4 prod = gbar * p;
        f4 q;
        q.x = __builtin_fabsf(prod.x); q.y = __builtin_fabsf(prod.y);
        q.z = __builtin_fabsf(prod.z); q.w = __builtin_fabsf(prod.w);
        const f4 mv = v * a.mu;
        const f4 vn = mv + gbar;
        const f4 step = vn * a.lr;
        const f4 pn = p - step;
        if (m == 0xFu) {
            imp += (double)q.x; imp += (double)q.y; imp += (double)q.z; imp += (double)q.w;
            st_stream(a.V + e, vn);
            st_stream(a.P + e, pn);
            if (KEYS) {
                u4 k;
                k.x = importance_key(q.x); k.y = importance_key(q.y);
                k.z = importance_key(q.z); k.w = importance_key(q.w);
                *reinterpret_cast<u4 *>(a.key + e) = k;
            }
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j)
                if (m & (1u << j)) {
                    imp += (double)q[j];
                    a.V[e + j] = vn[j];
                    a.P[e + j] = pn[j];
                    if (KEYS)
                        a.key[e + j] = importance_key(q[j]);
                }
        }
    }
    const double total = wave_sum(imp);
    if (threadIdx.x == 0)
        a.partial[ci] = total;
}

// ---------------------------------------------------------------------------
// Install a stage's global parameters on every worker replica.
// ---------------------------------------------------------------------------
struct ApplyArgs {
    const Chunk *chunks;
    const int *stage_list;
    const uint32_t *bitmap;
    const float *P;
    float *Pw;
    long long param_stride;
    int n_workers;
    int stage;
};

template <bool MASKED>
__global__ __launch_bounds__(kBlock) void k_apply_stage(const ApplyArgs a)
{
    const Chunk c = owned_chunk(a.chunks, a.stage_list, blockIdx.x);
    const int N = a.n_workers;
    for (int i = threadIdx.x * kVec; i < c.len; i += kStride) {
        const long long e = c.start + i;
        const unsigned m = lane_mask<MASKED>(c.len - i, e, a.stage, a.bitmap);
        if (m == 0)
            continue;
        const f4 p = ld_keep(a.P + e);
        float *dst = a.Pw + e;
        if (m == 0xFu) {
            for (int w = 0; w < N; ++w)
                st_stream(dst + (long long)w * a.param_stride, p);
        } else {
            for (int w = 0; w < N; ++w)
#pragma unroll
                for (int j = 0; j < kVec; ++j)
                    if (m & (1u << j))
                        dst[(long long)w * a.param_stride + j] = p[j];
        }
    }
}

// ---------------------------------------------------------------------------
// LGP: stage-2 parameters of every replica advance by the local gradient.
// ---------------------------------------------------------------------------
struct LgpArgs {
    const Chunk *chunks;
    const int *stage_list;             // stage-2 chunks, or null = every chunk (MASKED)
    const uint32_t *bitmap;
    float *Pw;
    long long param_stride;
    const float *grads;
    long long worker_stride;
    float lr;
};

// grid = (chunks of stage 2, workers): one workgroup moves one chunk of ONE
// replica, so the whole GPU sweeps one worker's arena at a time (three streams).
template <bool MASKED>
__global__ __launch_bounds__(kBlock) void k_lgp_correct(const LgpArgs a)
{
    const Chunk c = owned_chunk(a.chunks, a.stage_list, blockIdx.x);
    const long long w = blockIdx.y;
    float *pw = a.Pw + w * a.param_stride;
    const float *gw = a.grads + w * a.worker_stride;
    for (int i = threadIdx.x * kVec; i < c.len; i += kStride) {
        const long long e = c.start + i;
        const unsigned m = lane_mask<MASKED>(c.len - i, e, 2, a.bitmap);
        if (m == 0)
            continue;
        const f4 p = ld_stream(pw + e);
        const f4 g = ld_stream(gw + e);
        const f4 step = g * a.lr;
        const f4 pn = p - step;
        if (m == 0xFu) {
            st_stream(pw + e, pn);
        } else {
#pragma unroll
            for (int t = 0; t < kVec; ++t)
                if (m & (1u << t))
                    pw[e + t] = pn[t];
        }
    }
}

} // namespace osp
