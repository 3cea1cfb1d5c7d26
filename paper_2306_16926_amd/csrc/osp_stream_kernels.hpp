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
// float4 of a tensor can be ragged.  A launch walks a table of 16-byte spans,
// each covering up to 64 consecutive chunks of one tensor: 64 consecutive
// workgroups share one span (one scalar load, an L2 hit for all but the first
// workgroup on each XCD) and keep the address order of the chunks, which the
// DRAM likes.  The table is either that of all chunks or, for a layer-granular
// GIB, the compact table of one stage's spans, so a launch has next to no idle
// workgroups (at most 63 per tensor).
//
// Addressing: every stream is "uniform base + 32-bit lane offset", which keeps
// the 16 gradient bases in scalar registers instead of 32 vector registers.
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

constexpr int kSpanChunks = 64;        // workgroups that share one table entry

struct Span {
    long long start;                   // arena element index of the first chunk, multiple of 4
    int n_elems;                       // elements covered: 1 .. 64 * chunk_elems
    int chunk_base;                    // index of the first chunk (slot of its importance partial)
};

struct Piece {                         // the chunk one workgroup owns
    long long start;
    int len;
    int chunk;
};

// Launches over the table of all spans: workgroup b owns chunk (b % 64) of span (b / 64);
// false if the span is shorter.
__device__ __forceinline__ bool owned_piece(const Span *__restrict__ spans, int chunk_elems,
                                            Piece &p)
{
    const Span s = spans[blockIdx.x / kSpanChunks];
    const int j = blockIdx.x % kSpanChunks;
    const int off = j * chunk_elems;
    if (off >= s.n_elems)
        return false;
    p.start = s.start + off;
    p.len = s.n_elems - off < chunk_elems ? s.n_elems - off : chunk_elems;
    p.chunk = s.chunk_base + j;
    return true;
}

// Group g of a launch is chunk (g % 64) of span (g / 64) of the launch's table.  A stage table
// (layer-granular GIB) is written on the device by the split, and no launch over it waits for
// its length to reach the host: every table has room for all spans, the entries behind the
// stage's last span are cleared (n_elems == 0), and a workgroup walks groups blockIdx.x,
// blockIdx.x + gridDim.x, ... until it meets a cleared entry or the table's capacity.  The host
// sizes the grid from the last length it has seen; when that was right every workgroup owns
// exactly one group, when it was too small some own a second one, when it was too large the
// surplus workgroups return at once.  The grid never exceeds 64 * capacity.
struct GroupWalk {
    const Span *spans;
    Span s;                            // entry of group g
    unsigned g, cap_groups;
    int chunk_elems;

    __device__ __forceinline__ GroupWalk(const Span *__restrict__ table, unsigned cap_spans, int chunk)
        : spans(table), chunk_elems(chunk)
    {
        g = blockIdx.x;
        cap_groups = cap_spans * kSpanChunks;
        s = table[g / kSpanChunks];
    }

    // The next chunk this workgroup owns; false when there is none.
    __device__ __forceinline__ bool next(Piece &p)
    {
        while (s.n_elems != 0) {
            const int j = g % kSpanChunks;
            const int off = j * chunk_elems;
            const bool ok = off < s.n_elems;      // (false: the span is shorter than 64 chunks)
            if (ok) {
                p.start = s.start + off;
                p.len = s.n_elems - off < chunk_elems ? s.n_elems - off : chunk_elems;
                p.chunk = s.chunk_base + j;
            }
            g += gridDim.x;
            if (g < cap_groups)
                s = spans[g / kSpanChunks];
            else
                s.n_elems = 0;
            if (ok)
                return true;
        }
        return false;
    }
};

using f4 = __attribute__((ext_vector_type(4))) float;
using u4 = __attribute__((ext_vector_type(4))) unsigned int;

__device__ __forceinline__ f4 ld_stream(const float *p)
{   // read-once data: keep it from displacing reusable lines
    return __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
}
// Gradient arenas hold fp32 or bfloat16 values.  A bfloat16 is the upper half of
// the fp32 with the same value, so widening is exact and the arithmetic that
// follows is the fp32 arithmetic on those values; a lane's 4 elements are one
// 8-byte load.
using bf16_t = unsigned short;
using u2 = __attribute__((ext_vector_type(2))) unsigned int;

// A lane's 4 gradient elements as they come from memory (GradRaw) and widened to fp32.
// Kernels whose gradient loads sit behind a test of the worker count load all the raw values
// first and widen afterwards: widening inside such a branch makes the compiler wait for each
// load where it is issued, one round trip to memory per worker.
template <typename GT>
struct GradRaw;
template <>
struct GradRaw<float> { using type = f4; };
template <>
struct GradRaw<bf16_t> { using type = u2; };

__device__ __forceinline__ f4 ld_grad_raw(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
}
__device__ __forceinline__ u2 ld_grad_raw(const bf16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u2 *>(p));
}
__device__ __forceinline__ f4 widen(f4 r) { return r; }
__device__ __forceinline__ f4 widen(u2 r)
{
    f4 f;
    f.x = __uint_as_float(r.x << 16);
    f.y = __uint_as_float(r.x & 0xFFFF0000u);
    f.z = __uint_as_float(r.y << 16);
    f.w = __uint_as_float(r.y & 0xFFFF0000u);
    return f;
}

template <typename GT>
__device__ __forceinline__ f4 ld_grad(const GT *p)
{
    return widen(ld_grad_raw(p));
}

__device__ __forceinline__ f4 ld_keep(const float *p)
{
    return *reinterpret_cast<const f4 *>(p);
}
__device__ __forceinline__ void st_stream(float *p, f4 v)
{   // write-once data: streaming, written through at system scope.  Measured on
    // MI355X this policy is the fastest for all three kernels (the 16-replica
    // install gains about 7 % over a plain store, 12 % over "nt" alone).
    // The compiler has no way to ask for this policy on a 16-byte store, hence
    // the inline instruction.  Two things the compiler would otherwise do for a
    // store of its own:
    //  * a store of more than 8 bytes reads its data registers for up to two
    //    cycles after issue, and the compiler does not look inside an asm block
    //    when it reuses registers, so the two wait states (s_nop 1) are part of
    //    the block;
    //  * no wait on the memory counter is needed: nothing in the kernels reads
    //    back what they store, and a count the compiler does not know of only
    //    makes its own waits conservative (the counter retires in order).
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1"
                 :
                 : "v"(p), "v"(v)
                 : "memory");
}

// Which of the 4 elements at chunk position i does this call touch?
// Bit j set = element i+j is inside the chunk and (if MASKED) in the stage.
//
// Element-granular stages select scattered elements, but every 16-byte group
// that holds a selected element is read whole anyway.  When all four elements
// of a group are real (rem >= 4) the kernels therefore write the group back
// whole, unselected components with the value they already had: full-width
// streaming stores instead of up to four 4-byte ones.  This relies on the calls
// of one context never running concurrently with each other (they share the
// buffers they update); padding is still never written, because a ragged
// last group (rem < 4) takes the per-element path.  All lanes of a wave take
// the same store instruction whatever their masks are, so a wave still writes
// its 1 KiB as whole lines.
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

// Per component: bit j of m set -> a[j], else b[j].
__device__ __forceinline__ f4 blend(unsigned m, f4 a, f4 b)
{
    f4 r;
    r.x = (m & 1u) ? a.x : b.x;
    r.y = (m & 2u) ? a.y : b.y;
    r.z = (m & 4u) ? a.z : b.z;
    r.w = (m & 8u) ? a.w : b.w;
    return r;
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

__device__ __forceinline__ f4 abs4(f4 x)
{
    f4 q;
    q.x = __builtin_fabsf(x.x); q.y = __builtin_fabsf(x.y);
    q.z = __builtin_fabsf(x.z); q.w = __builtin_fabsf(x.w);
    return q;
}

__device__ __forceinline__ f4 keys4(f4 q)
{
    u4 k;
    k.x = importance_key(q.x); k.y = importance_key(q.y);
    k.z = importance_key(q.z); k.w = importance_key(q.w);
    return __builtin_bit_cast(f4, k);
}

__device__ __forceinline__ double masked_sum(unsigned m, f4 q)
{
    double s = 0.0;
    if (m & 1u) s += (double)q.x;
    if (m & 2u) s += (double)q.y;
    if (m & 4u) s += (double)q.z;
    if (m & 8u) s += (double)q.w;
    return s;
}

// ---------------------------------------------------------------------------
// PS aggregate + update (+ PGP importance), one stage.
// ---------------------------------------------------------------------------
// (The span table of a launch is a kernel parameter of its own, declared restrict: the
// walkers read it inside their loops, behind the kernel's stores, and only a table that
// provably none of these stores can touch is read through the scalar path.)
struct AggArgs {
    unsigned cap_spans;                // entries the table has room for (see GroupWalk)
    int chunk_elems;
    const uint32_t *bitmap;            // bit per element (element-granular GIB), when MASKED
    float *P;
    float *V;
    const void *grads;                 // fp32 or bfloat16 arenas (template parameter GT)
    long long worker_stride;
    const float *weights;              // [N] device, used when WEIGHTED
    double *partial;                   // [n_chunks] importance partial of this stage
    double *partial_other;             // [n_chunks] partial of the other stage (with stash)
    uint32_t *key;                     // [arena] when KEYS
    float *stash;                      // [arena] or null: see k_aggregate_update
    int n_workers;
    int stage;
    float inv_n, lr, mu;
};

// Add B consecutive workers' gradients (w0 .. w0+B-1) to the running sum, in
// ascending worker order; with w0 == 0 worker 0 starts the sum.  All B loads
// are issued before the first add.
template <int B, bool WEIGHTED, typename GT = float>
__device__ __forceinline__ void add_workers(f4 &acc, int w0, const GT *__restrict__ g0,
                                            long long worker_stride, unsigned i,
                                            const float *__restrict__ weights)
{
    float wgt[B];
    if (WEIGHTED) {
#pragma unroll
        for (int j = 0; j < B; ++j)
            wgt[j] = weights[w0 + j];
    }
    f4 g[B];
#pragma unroll
    for (int j = 0; j < B; ++j)
        g[j] = ld_grad<GT>(g0 + (long long)(w0 + j) * worker_stride + i);
    if (WEIGHTED) {
#pragma unroll
        for (int j = 0; j < B; ++j)
            g[j] = g[j] * wgt[j];
    }
    f4 s = g[0];
    if (w0 != 0)
        s = acc + s;
#pragma unroll
    for (int j = 1; j < B; ++j)
        s = s + g[j];
    acc = s;
}

constexpr int kWorkerBlock = 16;       // most gradient streams in flight per lane

template <bool MASKED, bool WEIGHTED, bool KEYS, typename GT = float>
__global__ __launch_bounds__(kBlock) void k_aggregate_update(const Span *__restrict__ table, const AggArgs a)
{
    GroupWalk walk(table, a.cap_spans, a.chunk_elems);
    Piece c;
    while (walk.next(c)) {
    const int N = a.n_workers;
    // uniform bases of this chunk in every stream
    float *Pc = a.P + c.start;
    float *Vc = a.V + c.start;
    const GT *Gc = static_cast<const GT *>(a.grads) + c.start;
    double imp = 0.0, imp_other = 0.0;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        // (masked: the data loads do not wait for the bitmap word; a group with no
        // selected element is written back unchanged)
        const unsigned m = lane_mask<MASKED>(c.len - (int)i, c.start + i, a.stage, a.bitmap);
        const f4 p = ld_stream(Pc + i);
        const f4 v = ld_stream(Vc + i);
        // workers in blocks of 16, then 8, 4, 2, 1 (N in binary): ascending order,
        // few branches, and for N = 16 all gradient loads in flight at once
        f4 acc;
        int w = 0;
        for (; w + kWorkerBlock <= N; w += kWorkerBlock)
            add_workers<kWorkerBlock, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights);
        const int rest = N - w;
        if (rest & 8) { add_workers<8, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 8; }
        if (rest & 4) { add_workers<4, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 4; }
        if (rest & 2) { add_workers<2, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 2; }
        if (rest & 1) { add_workers<1, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); }
        const f4 gbar = WEIGHTED ? acc : acc * a.inv_n;
        const f4 prod = gbar * p;
        f4 q;
        q.x = __builtin_fabsf(prod.x); q.y = __builtin_fabsf(prod.y);
        q.z = __builtin_fabsf(prod.z); q.w = __builtin_fabsf(prod.w);
        const f4 mv = v * a.mu;
        const f4 vn = mv + gbar;
        const f4 step = vn * a.lr;
        const f4 pn = p - step;
        const int rem = (int)c.len - (int)i;
        const bool whole = MASKED ? rem >= kVec : m == 0xFu;
        // Element-granular stage 1 with a stash: every group that holds a stage-1 element is
        // read whole, so the aggregate of its stage-2 elements is at hand too.  It is kept
        // (stash), together with their keys and importance, which depend only on the aggregate
        // and on PS values that stay untouched until stage 2; the stage-2 call of the same
        // gradients then needs one stream instead of N (k_update_from_stash).
        const bool stashing = MASKED && a.stash != nullptr;
        const unsigned valid = rem >= kVec ? 0xFu : ((1u << rem) - 1u);
        const unsigned other = stashing ? (valid & ~m) : 0u;
        if (whole) {
            if (m & 1u) imp += (double)q.x;
            if (m & 2u) imp += (double)q.y;
            if (m & 4u) imp += (double)q.z;
            if (m & 8u) imp += (double)q.w;
            if (other & 1u) imp_other += (double)q.x;
            if (other & 2u) imp_other += (double)q.y;
            if (other & 4u) imp_other += (double)q.z;
            if (other & 8u) imp_other += (double)q.w;
            st_stream(Vc + i, MASKED ? blend(m, vn, v) : vn);
            st_stream(Pc + i, MASKED ? blend(m, pn, p) : pn);
            if (KEYS) {
                u4 k;
                k.x = importance_key(q.x); k.y = importance_key(q.y);
                k.z = importance_key(q.z); k.w = importance_key(q.w);
                f4 kf = __builtin_bit_cast(f4, k);
                float *kp = reinterpret_cast<float *>(a.key + c.start + i);
                if (MASKED && !stashing)
                    kf = blend(m, kf, ld_stream(kp));
                st_stream(kp, kf);
            }
            if (stashing)
                st_stream(a.stash + c.start + i, gbar);
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                if (m & (1u << j)) {
                    imp += (double)q[j];
                    Vc[i + j] = vn[j];
                    Pc[i + j] = pn[j];
                    if (KEYS)
                        a.key[c.start + i + j] = importance_key(q[j]);
                }
                if (other & (1u << j)) {
                    imp_other += (double)q[j];
                    a.key[c.start + i + j] = importance_key(q[j]);
                    a.stash[c.start + i + j] = gbar[j];
                }
            }
        }
    }
    const double total = wave_sum(imp);
    if (threadIdx.x == 0)
        a.partial[c.chunk] = total;
    if (MASKED && a.stash != nullptr) {
        const double total_other = wave_sum(imp_other);
        if (threadIdx.x == 0)
            a.partial_other[c.chunk] = total_other;
    }
    }
}

// Stage 2 of an iteration whose aggregate is already in the stash (left there by an
// element-granular stage 1, or by LGP over a layer-granular stage 2): V = mu V + gbar,
// P = P - lr V on the stage-2 elements; their keys and importance were written with it.
// MASKED: element-granular GIB over all spans; otherwise the stage-2 span table.
struct StashArgs {
    unsigned cap_spans;                // entries the table has room for
    int chunk_elems;
    const uint32_t *bitmap;
    float *P;
    float *V;
    const float *stash;
    float lr, mu;
};

template <bool MASKED>
__global__ __launch_bounds__(kBlock) void k_update_from_stash(const Span *__restrict__ table, const StashArgs a)
{
    GroupWalk walk(table, a.cap_spans, a.chunk_elems);
    Piece c;
    while (walk.next(c)) {
    float *Pc = a.P + c.start;
    float *Vc = a.V + c.start;
    const float *Sc = a.stash + c.start;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        const int rem = (int)c.len - (int)i;
        const unsigned m = lane_mask<MASKED>(rem, c.start + i, 2, a.bitmap);
        const f4 p = ld_stream(Pc + i);
        const f4 v = ld_stream(Vc + i);
        const f4 gbar = ld_stream(Sc + i);
        const f4 mv = v * a.mu;
        const f4 vn = mv + gbar;
        const f4 step = vn * a.lr;
        const f4 pn = p - step;
        if (rem >= kVec) {
            st_stream(Vc + i, MASKED ? blend(m, vn, v) : vn);
            st_stream(Pc + i, MASKED ? blend(m, pn, p) : pn);
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j)
                if (m & (1u << j)) {
                    Vc[i + j] = vn[j];
                    Pc[i + j] = pn[j];
                }
        }
    }
    }
}

// ---------------------------------------------------------------------------
// Install a stage's global parameters on every worker replica: one read
// stream, N write streams.  Two shapes, chosen by N on the host:
//
//  * sweep (N > 4): writing all N from one workgroup keeps 16+ DRAM write
//    streams open at once (measured 5.7 TB/s at N = 16).  Instead the table is
//    cut into blocks of about 16 MB of parameters and, block after block, the GPU
//    writes one replica at a time: the parameter block is read from HBM once and
//    served from cache to the other N-1 sweeps, and the writes form a single
//    stream.  Workgroups of 256 lanes: with one wavefront per KiB the launch
//    rate of workgroups would be the limit here.
//  * fan-out (N <= 4): one wavefront per chunk reads its float4 once and writes
//    it to all N replicas; with few replicas this is as fast and launches fewer
//    workgroups.
// ---------------------------------------------------------------------------
constexpr int kApplyBlock = 256;
constexpr int kPiece = kApplyBlock * kVec;     // elements per workgroup

struct ApplyArgs {
    const uint32_t *bitmap;
    const float *P;
    float *Pw;
    long long param_stride;
    unsigned cap_spans;                // entries the table has room for (all spans)
    unsigned pieces_per_span;          // 64 * chunk_elems / (T * kPiece)
    int pieces_shift;                  // log2(pieces_per_span) if it is a power of two, else -1
    unsigned spans_per_block;
    int stage;
};

// Sweep kernels: grid = (pieces of a block, workers, blocks), dispatched in that order (x
// fastest), so the kernel needs no division to find its place.  A workgroup lives about as
// long as two dependent cache hits (its span entry, then its parameters): each lane moves T
// float4, T * 4 KiB per workgroup, to keep enough bytes in flight over that latency.
// As in GroupWalk the table ends at its first cleared entry: a workgroup owns its piece of
// blocks blockIdx.z, blockIdx.z + gridDim.z, ... (one block each when the host sized the grid
// from the right length).
template <int T>
struct SweepWalk {
    const Span *spans;
    Span s;
    unsigned si, cap_spans, stride_spans;
    int off0;                          // the lane's first element inside its span

    __device__ __forceinline__ SweepWalk(const Span *__restrict__ table, unsigned cap,
                                         unsigned spb, unsigned pieces_per_span, int pieces_shift)
        : spans(table), cap_spans(cap)
    {
        const unsigned q = blockIdx.x;
        const unsigned sp = pieces_shift >= 0 ? q >> pieces_shift : q / pieces_per_span;
        off0 = (int)(q - sp * pieces_per_span) * (kPiece * T) + (int)threadIdx.x * kVec;
        si = blockIdx.z * spb + sp;
        stride_spans = gridDim.z * spb;
        s.n_elems = 0;
        if (si < cap)
            s = table[si];
    }

    // The span of the next block this workgroup has a piece in; false when there is none.
    __device__ __forceinline__ bool next(Span &out)
    {
        while (s.n_elems != 0) {
            out = s;
            const bool ok = off0 < s.n_elems;
            si += stride_spans;
            if (si < cap_spans)
                s = spans[si];
            else
                s.n_elems = 0;
            if (ok)
                return true;
        }
        return false;
    }
};

template <bool MASKED, int T>
__global__ __launch_bounds__(kApplyBlock) void k_apply_stage_sweep(const Span *__restrict__ table, const ApplyArgs a)
{
    SweepWalk<T> walk(table, a.cap_spans, a.spans_per_block, a.pieces_per_span, a.pieces_shift);
    const int off0 = walk.off0;
    Span s;
    while (walk.next(s)) {
    const float *src = a.P + s.start;
    float *dst = a.Pw + (long long)blockIdx.y * a.param_stride + s.start;
    f4 p[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int off = off0 + t * kPiece;
        if (off < s.n_elems)
            p[t] = ld_keep(src + off);         // kept in cache for the other replicas' sweeps
    }
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int off = off0 + t * kPiece;
        if (off >= s.n_elems)
            continue;
        const int rem = s.n_elems - off;
        const unsigned m = lane_mask<MASKED>(rem, s.start + off, a.stage, a.bitmap);
        if (!MASKED && m == 0xFu) {
            st_stream(dst + off, p[t]);
        } else if (MASKED && rem >= kVec) {
            st_stream(dst + off, blend(m, p[t], ld_stream(dst + off)));
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j)
                if (m & (1u << j))
                    dst[off + j] = p[t][j];
        }
    }
    }
}

struct FanoutArgs {
    unsigned cap_spans;                // entries the table has room for
    int chunk_elems;
    const uint32_t *bitmap;
    const float *P;
    float *Pw;
    long long param_stride;
    int n_workers;
    int stage;
};

template <bool MASKED>
__global__ __launch_bounds__(kBlock) void k_apply_stage_fanout(const Span *__restrict__ table, const FanoutArgs a)
{
    GroupWalk walk(table, a.cap_spans, a.chunk_elems);
    Piece c;
    while (walk.next(c)) {
    const int N = a.n_workers;
    const float *Pc = a.P + c.start;
    float *Wc = a.Pw + c.start;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        const unsigned m = lane_mask<MASKED>(c.len - (int)i, c.start + i, a.stage, a.bitmap);
        const f4 p = ld_keep(Pc + i);
        if (!MASKED && m == 0xFu) {
            for (int w = 0; w < N; ++w)
                st_stream(Wc + (long long)w * a.param_stride + i, p);
        } else if (MASKED && (int)c.len - (int)i >= kVec) {
            // all old values first (they do not wait for the bitmap word), then all stores
            for (int w0 = 0; w0 < N; w0 += 8) {
                f4 old[8];
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (w0 + j < N)
                        old[j] = ld_stream(Wc + (long long)(w0 + j) * a.param_stride + i);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (w0 + j < N)
                        st_stream(Wc + (long long)(w0 + j) * a.param_stride + i, blend(m, p, old[j]));
            }
        } else {
            for (int w = 0; w < N; ++w)
#pragma unroll
                for (int j = 0; j < kVec; ++j)
                    if (m & (1u << j))
                        Wc[(long long)w * a.param_stride + i + j] = p[j];
        }
    }
    }
}

// ---------------------------------------------------------------------------
// LGP: stage-2 parameters of every replica advance by the local gradient.
// ---------------------------------------------------------------------------
struct LgpArgs {                       // (table: stage-2 spans, or all spans when MASKED)
    unsigned cap_spans;                // entries the table has room for
    int chunk_elems;
    const uint32_t *bitmap;
    float *Pw;
    long long param_stride;
    const void *grads;                 // fp32 or bfloat16 arenas (template parameter GT)
    long long worker_stride;
    float lr;
};

// grid = (chunks of stage 2, workers): one workgroup moves one chunk of ONE
// replica, so the whole GPU sweeps one worker's arena at a time (three streams).
template <bool MASKED, typename GT = float>
__global__ __launch_bounds__(kBlock) void k_lgp_correct(const Span *__restrict__ table, const LgpArgs a)
{
    GroupWalk walk(table, a.cap_spans, a.chunk_elems);
    Piece c;
    while (walk.next(c)) {
    const long long w = blockIdx.y;
    float *pw = a.Pw + w * a.param_stride + c.start;
    const GT *gw = static_cast<const GT *>(a.grads) + w * a.worker_stride + c.start;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        const unsigned m = lane_mask<MASKED>(c.len - (int)i, c.start + i, 2, a.bitmap);
        const f4 p = ld_stream(pw + i);
        const f4 g = ld_grad<GT>(gw + i);
        const f4 step = g * a.lr;
        const f4 pn = p - step;
        if (!MASKED && m == 0xFu) {
            st_stream(pw + i, pn);
        } else if (MASKED && (int)c.len - (int)i >= kVec) {
            st_stream(pw + i, blend(m, pn, p));
        } else {
#pragma unroll
            for (int t = 0; t < kVec; ++t)
                if (m & (1u << t))
                    pw[i + t] = pn[t];
        }
    }
    }
}

// ---------------------------------------------------------------------------
// LGP that keeps the stage-2 aggregate (layer-granular GIB, replicas in sync).
// LGP reads every worker's stage-2 gradients, and so does the stage-2 aggregate
// a little later.  Here one workgroup owns a chunk of ALL workers: with a block
// of gradients in registers it writes each replica's estimate P - lr g_w (P: the
// PS arena, which holds the replicas' stale values), adds the block to the
// aggregate in the aggregate's own order, and finally leaves the aggregate, its
// importance and keys in the workspace.  The stage-2 call on the same gradient
// arenas then needs one stream instead of N (k_update_from_stash).
// ---------------------------------------------------------------------------
struct LgpKeepArgs {                   // (table: stage-2 spans)
    unsigned cap_spans;                // entries the table has room for
    int chunk_elems;
    const float *P;
    float *Pw;
    long long param_stride;
    const void *grads;                 // fp32 or bfloat16 arenas (template parameter GT)
    long long worker_stride;
    const float *weights;              // WEIGHTED
    double *partial;                   // [n_chunks] importance partial of stage 2
    uint32_t *key;                     // KEYS
    float *stash;
    int n_workers;
    float inv_n, lr;
};

// B consecutive workers: their replicas' LGP values are stored (m: which of the lane's 4
// elements exist), then their gradients join the running sum as in add_workers.
template <int B, bool WEIGHTED, typename GT>
__device__ __forceinline__ void lgp_and_add(f4 &acc, int w0, const GT *__restrict__ g0,
                                            long long worker_stride, unsigned i,
                                            const float *__restrict__ weights, f4 p, float lr,
                                            float *__restrict__ w_base, long long param_stride,
                                            unsigned m)
{
    float wgt[B];
    if (WEIGHTED) {                    // (ahead of the stores: a load issued behind them waits for them)
#pragma unroll
        for (int j = 0; j < B; ++j)
            wgt[j] = weights[w0 + j];
    }
    f4 g[B];
#pragma unroll
    for (int j = 0; j < B; ++j)
        g[j] = ld_grad<GT>(g0 + (long long)(w0 + j) * worker_stride + i);
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const f4 step = g[j] * lr;
        const f4 pn = p - step;
        float *dst = w_base + (long long)(w0 + j) * param_stride + i;
        if (m == 0xFu) {
            st_stream(dst, pn);
        } else {
#pragma unroll
            for (int t = 0; t < kVec; ++t)
                if (m & (1u << t))
                    dst[t] = pn[t];
        }
    }
    if (WEIGHTED) {
#pragma unroll
        for (int j = 0; j < B; ++j)
            g[j] = g[j] * wgt[j];
    }
    f4 s = g[0];
    if (w0 != 0)
        s = acc + s;
#pragma unroll
    for (int j = 1; j < B; ++j)
        s = s + g[j];
    acc = s;
}

constexpr int kKeepBlock = 16;         // workers whose gradients a lane holds at once (8: 4 % slower)

template <bool WEIGHTED, bool KEYS, typename GT = float>
__global__ __launch_bounds__(kBlock) void k_lgp_keep(const Span *__restrict__ table, const LgpKeepArgs a)
{
    GroupWalk walk(table, a.cap_spans, a.chunk_elems);
    Piece c;
    while (walk.next(c)) {
    const int N = a.n_workers;
    const float *Pc = a.P + c.start;
    float *Wc = a.Pw + c.start;
    const GT *Gc = static_cast<const GT *>(a.grads) + c.start;
    double imp = 0.0;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        const int rem = (int)c.len - (int)i;
        const unsigned m = rem >= kVec ? 0xFu : ((1u << rem) - 1u);
        const f4 p = ld_stream(Pc + i);
        f4 acc;
        int w = 0;
        for (; w + kKeepBlock <= N; w += kKeepBlock)
            lgp_and_add<kKeepBlock, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights, p, a.lr,
                                                  Wc, a.param_stride, m);
        const int rest = N - w;
        if (kKeepBlock > 8 && (rest & 8)) { lgp_and_add<8, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights, p, a.lr, Wc, a.param_stride, m); w += 8; }
        if (rest & 4) { lgp_and_add<4, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights, p, a.lr, Wc, a.param_stride, m); w += 4; }
        if (rest & 2) { lgp_and_add<2, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights, p, a.lr, Wc, a.param_stride, m); w += 2; }
        if (rest & 1) { lgp_and_add<1, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights, p, a.lr, Wc, a.param_stride, m); }
        const f4 gbar = WEIGHTED ? acc : acc * a.inv_n;
        const f4 prod = gbar * p;
        const f4 q = abs4(prod);
        if (m & 1u) imp += (double)q.x;        // (the order k_aggregate_update adds them in)
        if (m & 2u) imp += (double)q.y;
        if (m & 4u) imp += (double)q.z;
        if (m & 8u) imp += (double)q.w;
        if (m == 0xFu) {
            st_stream(a.stash + c.start + i, gbar);
            if (KEYS)
                st_stream(reinterpret_cast<float *>(a.key + c.start + i), keys4(q));
        } else {
#pragma unroll
            for (int t = 0; t < kVec; ++t)
                if (m & (1u << t)) {
                    a.stash[c.start + i + t] = gbar[t];
                    if (KEYS)
                        a.key[c.start + i + t] = importance_key(q[t]);
                }
        }
    }
    const double total = wave_sum(imp);
    if (threadIdx.x == 0)
        a.partial[c.chunk] = total;
    }
}

// ---------------------------------------------------------------------------
// Plain copy with the same access shape as the kernels above (one wavefront per
// 1 KiB, one streaming 16-byte load and one written-through 16-byte store per
// lane).  Reference line for bandwidth and calibration of traffic counters.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_stream_copy(float *__restrict__ dst,
                                                        const float *__restrict__ src,
                                                        long long n_vec)
{
    const long long v = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (v < n_vec)
        st_stream(dst + v * kVec, ld_stream(src + v * kVec));
}

// ---------------------------------------------------------------------------
// Reference traffic of the aggregate's shape, without its arithmetic: n_read
// streams are read and summed, n_rw streams (1 or 2) are read and written back
// with the sum added, one wavefront per KiB of every stream.  What this reaches
// is the ceiling of k_aggregate_update's access pattern on the machine at hand.
// ---------------------------------------------------------------------------
struct PatternArgs {
    const float *reads;
    long long read_stride;
    float *rw;
    long long rw_stride;
    long long n_vec;
    int n_read;
    int n_rw;
};

__global__ __launch_bounds__(kBlock) void k_stream_pattern(const PatternArgs a)
{
    const long long v = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (v >= a.n_vec)
        return;
    const unsigned i = threadIdx.x * kVec;
    const float *R = a.reads + (long long)blockIdx.x * kStride;
    float *W = a.rw + (long long)blockIdx.x * kStride;
    f4 old[2];
    old[0] = ld_stream(W + i);
    if (a.n_rw > 1)
        old[1] = ld_stream(W + a.rw_stride + i);
    f4 acc;
    int w = 0;
    for (; w + kWorkerBlock <= a.n_read; w += kWorkerBlock)
        add_workers<kWorkerBlock, false>(acc, w, R, a.read_stride, i, nullptr);
    const int rest = a.n_read - w;
    if (rest & 8) { add_workers<8, false>(acc, w, R, a.read_stride, i, nullptr); w += 8; }
    if (rest & 4) { add_workers<4, false>(acc, w, R, a.read_stride, i, nullptr); w += 4; }
    if (rest & 2) { add_workers<2, false>(acc, w, R, a.read_stride, i, nullptr); w += 2; }
    if (rest & 1) { add_workers<1, false>(acc, w, R, a.read_stride, i, nullptr); }
    st_stream(W + i, old[0] + acc);
    if (a.n_rw > 1)
        st_stream(W + a.rw_stride + i, old[1] + acc);
}

// ---------------------------------------------------------------------------
// LGP when every replica is known to equal the PS on the stage-2 elements (the
// previous iteration installed both stages and nothing else writes replicas):
// P_w = P - lr g_w then gives bit for bit what P_w = P_w - lr g_w gives, and the
// N reads of stale replica values become one read of the PS values.  Same
// blocked per-replica sweep as the install: the parameter block comes from HBM
// once and from cache N-1 times; per replica one gradient stream in, one
// parameter stream out.
// Element-granular GIB (MASKED): legal once this iteration's stage 1 has been
// installed; the unselected elements of a group then already equal the PS, so
// the group is written whole as "P, minus lr g on the stage-2 elements".
// ---------------------------------------------------------------------------
struct LgpSweepArgs {
    const uint32_t *bitmap;
    const float *P;
    float *Pw;
    long long param_stride;
    const void *grads;                 // fp32 or bfloat16 arenas (template parameter GT)
    long long worker_stride;
    unsigned cap_spans;                // entries the table has room for (all spans)
    unsigned pieces_per_span;
    int pieces_shift;
    unsigned spans_per_block;
    float lr;
};

template <bool MASKED, typename GT, int T>
__global__ __launch_bounds__(kApplyBlock) void k_lgp_sweep(const Span *__restrict__ table, const LgpSweepArgs a)
{
    SweepWalk<T> walk(table, a.cap_spans, a.spans_per_block, a.pieces_per_span, a.pieces_shift);
    const int off0 = walk.off0;
    Span s;
    while (walk.next(s)) {
    const long long w = blockIdx.y;
    const float *src = a.P + s.start;
    const GT *grad = static_cast<const GT *>(a.grads) + w * a.worker_stride + s.start;
    float *dst = a.Pw + w * a.param_stride + s.start;
    f4 p[T], g[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int off = off0 + t * kPiece;
        if (off < s.n_elems) {
            p[t] = ld_keep(src + off);         // kept in cache for the other replicas' sweeps
            g[t] = ld_grad<GT>(grad + off);
        }
    }
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int off = off0 + t * kPiece;
        if (off >= s.n_elems)
            continue;
        const int rem = s.n_elems - off;
        const unsigned m = lane_mask<MASKED>(rem, s.start + off, 2, a.bitmap);
        const f4 step = g[t] * a.lr;
        const f4 pn = p[t] - step;
        if (!MASKED && m == 0xFu) {
            st_stream(dst + off, pn);
        } else if (MASKED && rem >= kVec) {
            st_stream(dst + off, blend(m, pn, p[t]));
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j)
                if (m & (1u << j))
                    dst[off + j] = pn[j];
        }
    }
    }
}

} // namespace osp
