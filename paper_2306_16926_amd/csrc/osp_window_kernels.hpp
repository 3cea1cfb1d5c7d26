// Fused kernels for the two synchronization windows of one OSP iteration
// (Sec. 3.1): the RS window (stage-1 aggregate + update, install of stage 1 in
// every replica, LGP on stage 2: Sec. 2.1.1, Eq. 6) and the ICS window (stage-2
// aggregate + update and install, Eq. 7).  Each writes exactly what the
// sequence of single-stage kernels writes, with the same separately rounded
// fp32 operations; what is saved is launches and the re-reading of data a lane
// already holds.
//
// Both rely on what the replicas hold when the window begins:
//  * RS: every replica equals the PS arena (the previous iteration ended with
//    both installs), so the stale stage-2 value LGP starts from is the PS's.
//  * ICS (element-granular): stage 1 of this iteration is installed, so writing
//    a whole 16-byte group of PS values into a replica changes only its
//    stage-2 elements.
// The host checks these conditions and otherwise runs the single-stage kernels.
#pragma once
#include "osp_stream_kernels.hpp"

#pragma clang fp contract(off)

namespace osp {

// ---------------------------------------------------------------------------
// Element-granular GIB, RS window.  A lane holds the N gradients of its group
// in registers: it forms the aggregate (ascending workers), updates the stage-1
// elements on the PS, stores keys and importance of all four elements and the
// aggregate itself (for the ICS window), and writes each replica's group:
// the new PS value where the element is in stage 1, stale value - lr * g_w
// where it is in stage 2.  NB = register capacity in workers (N <= NB).
// ---------------------------------------------------------------------------
struct RsElementArgs {
    const Span *spans;
    int chunk_elems;
    const uint32_t *bitmap;
    float *P;
    float *V;
    const void *grads;                 // fp32 or bfloat16 arenas (template parameter GT)
    long long worker_stride;
    const float *weights;
    double *partial1;                  // [n_chunks] importance of stage-1 elements
    double *partial2;                  // [n_chunks] importance of stage-2 elements
    uint32_t *key;
    float *stash;
    float *Pw;
    long long param_stride;
    int n_workers;
    float inv_n, lr, mu;
};

template <int NB, bool WEIGHTED, typename GT = float>
__global__ __launch_bounds__(kBlock) void k_rs_window_element(const RsElementArgs a)
{
    Piece c;
    if (!owned_piece(a.spans, a.chunk_elems, c))
        return;
    const int N = a.n_workers;
    float *Pc = a.P + c.start;
    float *Vc = a.V + c.start;
    const GT *Gc = static_cast<const GT *>(a.grads) + c.start;
    float *Wc = a.Pw + c.start;
    double imp1 = 0.0, imp2 = 0.0;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        const int rem = (int)c.len - (int)i;
        const unsigned m = lane_mask<true>(rem, c.start + i, 1, a.bitmap);
        const unsigned valid = rem >= kVec ? 0xFu : ((1u << rem) - 1u);
        const unsigned other = valid & ~m;
        const f4 p = ld_stream(Pc + i);
        const f4 v = ld_stream(Vc + i);
        typename GradRaw<GT>::type raw[NB];
        float wgt[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j)
            if (j < N) {
                raw[j] = ld_grad_raw(Gc + (long long)j * a.worker_stride + i);
                if (WEIGHTED)
                    wgt[j] = a.weights[j];
            }
        f4 g[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j)
            if (j < N)
                g[j] = widen(raw[j]);
        f4 acc = WEIGHTED ? g[0] * wgt[0] : g[0];
#pragma unroll
        for (int j = 1; j < NB; ++j)
            if (j < N) {
                const f4 t = WEIGHTED ? g[j] * wgt[j] : g[j];
                acc = acc + t;
            }
        const f4 gbar = WEIGHTED ? acc : acc * a.inv_n;
        const f4 prod = gbar * p;
        const f4 q = abs4(prod);
        const f4 mv = v * a.mu;
        const f4 vn = mv + gbar;
        const f4 step = vn * a.lr;
        const f4 pn = p - step;
        if (rem >= kVec) {
            imp1 += masked_sum(m, q);
            imp2 += masked_sum(other, q);
            st_stream(Vc + i, blend(m, vn, v));
            st_stream(Pc + i, blend(m, pn, p));
            st_stream(reinterpret_cast<float *>(a.key + c.start + i), keys4(q));
            st_stream(a.stash + c.start + i, gbar);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                if (j < N) {
                    const f4 ls = g[j] * a.lr;
                    const f4 pl = p - ls;
                    st_stream(Wc + (long long)j * a.param_stride + i, blend(m, pn, pl));
                }
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                if (!(valid & (1u << e)))
                    continue;
                const bool first = (m >> e) & 1u;
                a.key[c.start + i + e] = importance_key(q[e]);
                if (first) {
                    imp1 += (double)q[e];
                    Vc[i + e] = vn[e];
                    Pc[i + e] = pn[e];
                } else {
                    imp2 += (double)q[e];
                    a.stash[c.start + i + e] = gbar[e];
                }
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (j < N) {
                        const float ls = g[j][e] * a.lr;
                        Wc[(long long)j * a.param_stride + i + e] = first ? pn[e] : p[e] - ls;
                    }
            }
        }
    }
    const double t1 = wave_sum(imp1);
    const double t2 = wave_sum(imp2);
    if (threadIdx.x == 0) {
        a.partial1[c.chunk] = t1;
        a.partial2[c.chunk] = t2;
    }
}

// ---------------------------------------------------------------------------
// Element-granular GIB, ICS window: stage-2 update on the PS from the kept
// aggregate (STASH) or from the N gradient arenas, then the whole group of PS
// values into every replica.
// ---------------------------------------------------------------------------
struct IcsElementArgs {
    const Span *spans;
    int chunk_elems;
    const uint32_t *bitmap;
    float *P;
    float *V;
    const float *stash;                // STASH
    const void *grads;                 // !STASH; fp32 or bfloat16 (GT)
    long long worker_stride;
    const float *weights;
    double *partial2;                  // !STASH
    uint32_t *key;                     // !STASH
    float *Pw;
    long long param_stride;
    int n_workers;
    float inv_n, lr, mu;
};

template <bool STASH, bool WEIGHTED, typename GT = float>
__global__ __launch_bounds__(kBlock) void k_ics_window_element(const IcsElementArgs a)
{
    Piece c;
    if (!owned_piece(a.spans, a.chunk_elems, c))
        return;
    const int N = a.n_workers;
    float *Pc = a.P + c.start;
    float *Vc = a.V + c.start;
    float *Wc = a.Pw + c.start;
    double imp = 0.0;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        const int rem = (int)c.len - (int)i;
        const unsigned m = lane_mask<true>(rem, c.start + i, 2, a.bitmap);
        const f4 p = ld_stream(Pc + i);
        const f4 v = ld_stream(Vc + i);
        f4 gbar;
        if (STASH) {
            gbar = ld_stream(a.stash + c.start + i);
        } else {
            const GT *Gc = static_cast<const GT *>(a.grads) + c.start;
            f4 acc;
            int w = 0;
            for (; w + kWorkerBlock <= N; w += kWorkerBlock)
                add_workers<kWorkerBlock, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights);
            const int rest = N - w;
            if (rest & 8) { add_workers<8, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 8; }
            if (rest & 4) { add_workers<4, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 4; }
            if (rest & 2) { add_workers<2, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 2; }
            if (rest & 1) { add_workers<1, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); }
            gbar = WEIGHTED ? acc : acc * a.inv_n;
        }
        const f4 prod = gbar * p;
        const f4 q = abs4(prod);
        const f4 mv = v * a.mu;
        const f4 vn = mv + gbar;
        const f4 step = vn * a.lr;
        const f4 pn = p - step;
        if (rem >= kVec) {
            const f4 pb = blend(m, pn, p);
            st_stream(Vc + i, blend(m, vn, v));
            st_stream(Pc + i, pb);
            if (!STASH) {
                imp += masked_sum(m, q);
                float *kp = reinterpret_cast<float *>(a.key + c.start + i);
                st_stream(kp, blend(m, keys4(q), ld_stream(kp)));
            }
            for (int j = 0; j < N; ++j)
                st_stream(Wc + (long long)j * a.param_stride + i, pb);
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                if (!(m & (1u << e)))
                    continue;
                Vc[i + e] = vn[e];
                Pc[i + e] = pn[e];
                if (!STASH) {
                    imp += (double)q[e];
                    a.key[c.start + i + e] = importance_key(q[e]);
                }
                for (int j = 0; j < N; ++j)
                    Wc[(long long)j * a.param_stride + i + e] = pn[e];
            }
        }
    }
    if (!STASH) {
        const double total = wave_sum(imp);
        if (threadIdx.x == 0)
            a.partial2[c.chunk] = total;
    }
}

// ---------------------------------------------------------------------------
// Layer-granular GIB, either window, for N <= 8 replicas and small models (above
// that the per-replica install and LGP sweeps of the single-stage kernels are
// as fast or faster, and launches no longer matter).
// One launch of two kinds of workgroups:
//   the first n_agg_groups own the chunks of the window's stage: aggregate +
//   update + importance, and the new values go into every replica at once;
//   the others (RS window only) own the stage-2 chunks: LGP on every replica
//   from the PS's stale values.
// The two kinds touch disjoint elements, so their order does not matter.
// ---------------------------------------------------------------------------
struct WindowLayerArgs {
    const Span *agg_spans;             // span table of the window's stage
    const int *n_agg_spans;            // device: length of agg_spans.  The launch covers as many
                                       // groups as all spans have, so a window is enqueued right
                                       // behind a split whose table lengths the host does not
                                       // know yet (RS window: both tables, whose lengths add up
                                       // to the number of all spans)
    const Span *lgp_spans;             // stage-2 span table (RS window), or null (ICS window)
    int chunk_elems;
    float *P;
    float *V;
    const void *grads;                 // fp32 or bfloat16 arenas (template parameter GT)
    long long worker_stride;
    const float *weights;
    double *partial;
    uint32_t *key;                     // KEYS
    float *Pw;
    long long param_stride;
    int n_workers;
    float inv_n, lr, mu;
};

constexpr int kWindowMaxWorkers = 8;

__device__ __forceinline__ bool piece_at(const Span *__restrict__ spans, int chunk_elems,
                                         unsigned b, Piece &p)
{
    const Span s = spans[b / kSpanChunks];
    const int j = b % kSpanChunks;
    const int off = j * chunk_elems;
    if (off >= s.n_elems)
        return false;
    p.start = s.start + off;
    p.len = s.n_elems - off < chunk_elems ? s.n_elems - off : chunk_elems;
    p.chunk = s.chunk_base + j;
    return true;
}

template <bool WEIGHTED, bool KEYS, typename GT = float>
__global__ __launch_bounds__(kBlock) void k_window_layer(const WindowLayerArgs a)
{
    const int N = a.n_workers;
    const unsigned n_agg = (unsigned)*a.n_agg_spans * kSpanChunks;
    Piece c;
    if (blockIdx.x < n_agg) {
        if (!piece_at(a.agg_spans, a.chunk_elems, blockIdx.x, c))
            return;
        float *Pc = a.P + c.start;
        float *Vc = a.V + c.start;
        float *Wc = a.Pw + c.start;
        const GT *Gc = static_cast<const GT *>(a.grads) + c.start;
        double imp = 0.0;
        for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
            const int rem = (int)c.len - (int)i;
            const f4 p = ld_stream(Pc + i);
            const f4 v = ld_stream(Vc + i);
            f4 acc;
            int w = 0;
            const int rest = N;        // N <= 8
            if (rest & 8) { add_workers<8, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 8; }
            if (rest & 4) { add_workers<4, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 4; }
            if (rest & 2) { add_workers<2, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); w += 2; }
            if (rest & 1) { add_workers<1, WEIGHTED, GT>(acc, w, Gc, a.worker_stride, i, a.weights); }
            const f4 gbar = WEIGHTED ? acc : acc * a.inv_n;
            const f4 prod = gbar * p;
            const f4 q = abs4(prod);
            const f4 mv = v * a.mu;
            const f4 vn = mv + gbar;
            const f4 step = vn * a.lr;
            const f4 pn = p - step;
            if (rem >= kVec) {
                imp += masked_sum(0xFu, q);
                st_stream(Vc + i, vn);
                st_stream(Pc + i, pn);
                if (KEYS)
                    st_stream(reinterpret_cast<float *>(a.key + c.start + i), keys4(q));
                for (int j = 0; j < N; ++j)
                    st_stream(Wc + (long long)j * a.param_stride + i, pn);
            } else {
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    if (e >= rem)
                        continue;
                    imp += (double)q[e];
                    Vc[i + e] = vn[e];
                    Pc[i + e] = pn[e];
                    if (KEYS)
                        a.key[c.start + i + e] = importance_key(q[e]);
                    for (int j = 0; j < N; ++j)
                        Wc[(long long)j * a.param_stride + i + e] = pn[e];
                }
            }
        }
        const double total = wave_sum(imp);
        if (threadIdx.x == 0)
            a.partial[c.chunk] = total;
    } else {
        if (!a.lgp_spans || !piece_at(a.lgp_spans, a.chunk_elems, blockIdx.x - n_agg, c))
            return;
        const float *Pc = a.P + c.start;
        float *Wc = a.Pw + c.start;
        const GT *Gc = static_cast<const GT *>(a.grads) + c.start;
        for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
            const int rem = (int)c.len - (int)i;
            const f4 p = ld_stream(Pc + i);
            typename GradRaw<GT>::type raw[kWindowMaxWorkers];
#pragma unroll
            for (int j = 0; j < kWindowMaxWorkers; ++j)
                if (j < N)
                    raw[j] = ld_grad_raw(Gc + (long long)j * a.worker_stride + i);
#pragma unroll
            for (int j = 0; j < kWindowMaxWorkers; ++j)
                if (j < N) {
                    const f4 ls = widen(raw[j]) * a.lr;
                    const f4 pl = p - ls;
                    float *dst = Wc + (long long)j * a.param_stride + i;
                    if (rem >= kVec) {
                        st_stream(dst, pl);
                    } else {
#pragma unroll
                        for (int e = 0; e < kVec; ++e)
                            if (e < rem)
                                dst[e] = pl[e];
                    }
                }
        }
    }
}

} // namespace osp
