// Gradient splitter (Sec. 4.5) for gfx950: each worker's gradient arena is cut
// by the GIB into two dense arrays, G^i (stage 1) and G^u (stage 2), holding the
// stage's elements in arena order; and the PS-side aggregate + update fed by
// such dense arrays.  This is the payload a transport would carry; with all
// workers resident on one GPU the in-place kernels are faster, so nothing else
// in the library depends on these.
//
// Position of an element inside its dense array = number of elements of the
// same stage before it.  That is kept per chunk (pack index: two exclusive
// prefix sums over the chunks, built once per GIB) and finished inside the
// wavefront that owns the chunk with a prefix sum over the lanes' counts.
#pragma once
#include "osp_stream_kernels.hpp"

#pragma clang fp contract(off)

namespace osp {

constexpr int kScanBlock = 1024;       // chunks per workgroup of the index scans

// Stage-1 selection of the 4 elements at chunk position i (bit j = element
// i+j is in stage 1), and which of the 4 exist at all.
__device__ __forceinline__ void group_stages(bool element, bool layer_important, int rem,
                                             long long e, const uint32_t *__restrict__ bitmap,
                                             unsigned &first, unsigned &valid)
{
    valid = rem >= kVec ? 0xFu : ((1u << rem) - 1u);
    if (element) {
        const unsigned word = bitmap[e >> 5];
        first = (word >> (unsigned)(e & 31)) & valid;
    } else {
        first = layer_important ? valid : 0u;
    }
}

// Inclusive prefix sum over the wavefront of two small counts packed as
// lo | hi << 16 (each total stays below 65536: at most 256 per wavefront pass).
__device__ __forceinline__ unsigned wave_scan_pair(unsigned x)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned up = __shfl_up(x, off, 64);
        if (lane >= off)
            x += up;
    }
    return x;
}

struct PackIndexArgs {
    const Span *spans;
    const int *span_layer;             // layer of each span
    const uint8_t *gib_layer;          // layer-granular GIB
    const uint32_t *bitmap;            // element-granular GIB
    int chunk_elems;
    int element;                       // granularity of the current GIB
    long long *base1;                  // [n_chunks + 1]
    long long *base2;                  // [n_chunks + 1]
};

// Step 1: per chunk, the number of its elements in stage 1 and in stage 2.
__global__ __launch_bounds__(kBlock) void k_pack_count(const PackIndexArgs a)
{
    Piece c;
    if (!owned_piece(a.spans, a.chunk_elems, c))
        return;
    const bool important = a.element ? false : a.gib_layer[a.span_layer[blockIdx.x / kSpanChunks]] != 0;
    unsigned n1 = 0;
    for (unsigned i = threadIdx.x * kVec; i < (unsigned)c.len; i += kStride) {
        unsigned first, valid;
        group_stages(a.element != 0, important, c.len - (int)i, c.start + i, a.bitmap, first, valid);
        n1 += __popc(first);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        n1 += __shfl_down(n1, off, 64);
    if (threadIdx.x == 0) {
        a.base1[c.chunk] = n1;
        a.base2[c.chunk] = c.len - (int)n1;
    }
}

template <int BLOCK>
__device__ __forceinline__ long long block_total(long long x)
{
    __shared__ long long part[BLOCK / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x += __shfl_down(x, off, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        part[threadIdx.x >> 6] = x;
    __syncthreads();
    long long s = 0;
#pragma unroll
    for (int i = 0; i < BLOCK / 64; ++i)
        s += part[i];
    return s;
}

// Exclusive prefix sum over a workgroup in thread order; all threads call it.
template <int BLOCK>
__device__ __forceinline__ long long block_prefix(long long x, long long *total)
{
    __shared__ long long wave_tot[BLOCK / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    long long incl = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const long long up = __shfl_up(incl, off, 64);
        if (lane >= off)
            incl += up;
    }
    __syncthreads();
    if (lane == 63)
        wave_tot[wave] = incl;
    __syncthreads();
    long long base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < BLOCK / 64; ++w) {
        if (w < wave)
            base += wave_tot[w];
        sum += wave_tot[w];
    }
    if (total)
        *total = sum;
    return base + incl - x;
}

// Step 2: totals of each block of kScanBlock chunks.
__global__ __launch_bounds__(kScanBlock) void k_pack_block_totals(
    long long n_chunks, const long long *__restrict__ base1, const long long *__restrict__ base2,
    long long *__restrict__ tot1, long long *__restrict__ tot2)
{
    const long long c = (long long)blockIdx.x * kScanBlock + threadIdx.x;
    const long long x1 = c < n_chunks ? base1[c] : 0, x2 = c < n_chunks ? base2[c] : 0;
    const long long s1 = block_total<kScanBlock>(x1);
    const long long s2 = block_total<kScanBlock>(x2);
    if (threadIdx.x == 0) {
        tot1[blockIdx.x] = s1;
        tot2[blockIdx.x] = s2;
    }
}

// Step 3 (one workgroup): exclusive prefix sums of the block totals, in place;
// the grand totals go behind the last chunk's entry.
__global__ __launch_bounds__(kScanBlock) void k_pack_scan_totals(
    long long n_blocks, long long n_chunks, long long *__restrict__ tot1,
    long long *__restrict__ tot2, long long *__restrict__ base1, long long *__restrict__ base2)
{
    long long carry1 = 0, carry2 = 0;
    for (long long b0 = 0; b0 < n_blocks; b0 += kScanBlock) {
        const long long b = b0 + threadIdx.x;
        const long long x1 = b < n_blocks ? tot1[b] : 0, x2 = b < n_blocks ? tot2[b] : 0;
        long long s1, s2;
        const long long e1 = block_prefix<kScanBlock>(x1, &s1);
        const long long e2 = block_prefix<kScanBlock>(x2, &s2);
        if (b < n_blocks) {
            tot1[b] = carry1 + e1;
            tot2[b] = carry2 + e2;
        }
        carry1 += s1;
        carry2 += s2;
    }
    if (threadIdx.x == 0) {
        base1[n_chunks] = carry1;
        base2[n_chunks] = carry2;
    }
}

// Step 4: per block, exclusive prefix sums of the chunk counts plus the block's offset, in place.
__global__ __launch_bounds__(kScanBlock) void k_pack_scan_chunks(
    long long n_chunks, const long long *__restrict__ tot1, const long long *__restrict__ tot2,
    long long *__restrict__ base1, long long *__restrict__ base2)
{
    const long long c = (long long)blockIdx.x * kScanBlock + threadIdx.x;
    const long long x1 = c < n_chunks ? base1[c] : 0, x2 = c < n_chunks ? base2[c] : 0;
    const long long e1 = block_prefix<kScanBlock>(x1, nullptr);
    const long long e2 = block_prefix<kScanBlock>(x2, nullptr);
    if (c < n_chunks) {
        base1[c] = tot1[blockIdx.x] + e1;
        base2[c] = tot2[blockIdx.x] + e2;
    }
}

// ---------------------------------------------------------------------------
// The splitter: grid (chunk groups, workers).
// ---------------------------------------------------------------------------
struct SplitGradArgs {
    const Span *spans;
    const int *span_layer;
    const uint8_t *gib_layer;
    const uint32_t *bitmap;
    int chunk_elems;
    int element;
    const long long *base1;
    const long long *base2;
    const float *grads;
    long long worker_stride;
    float *g_i;                        // or null
    long long stride_i;
    float *g_u;                        // or null
    long long stride_u;
};

__global__ __launch_bounds__(kBlock) void k_split_gradients(const SplitGradArgs a)
{
    Piece c;
    if (!owned_piece(a.spans, a.chunk_elems, c))
        return;
    const bool important = a.element ? false : a.gib_layer[a.span_layer[blockIdx.x / kSpanChunks]] != 0;
    const long long w = blockIdx.y;
    const float *G = a.grads + w * a.worker_stride + c.start;
    float *out1 = a.g_i ? a.g_i + w * a.stride_i + a.base1[c.chunk] : nullptr;
    float *out2 = a.g_u ? a.g_u + w * a.stride_u + a.base2[c.chunk] : nullptr;
    // The 4 elements of a lane land at consecutive dense positions, but those are not 16-byte
    // aligned in general, and four 4-byte stores per lane would each touch every line of the run
    // a little.  So a pass (256 elements) is put in dense order in LDS first and written out with
    // lane k storing element k, k+64, ...: every store instruction covers 256 consecutive bytes.
    __shared__ float dense1[kStride], dense2[kStride];
    unsigned carry1 = 0, carry2 = 0;   // elements of each stage in earlier passes over the chunk
    // every lane takes every pass (inactive ones count nothing): the prefix sum is wave-wide
    for (unsigned i0 = 0; i0 < (unsigned)c.len; i0 += kStride) {
        const unsigned i = i0 + threadIdx.x * kVec;
        const int rem = (int)c.len - (int)i;
        unsigned first = 0, valid = 0;
        f4 g = {0.f, 0.f, 0.f, 0.f};
        if (rem > 0) {
            group_stages(a.element != 0, important, rem, c.start + i, a.bitmap, first, valid);
            g = ld_stream(G + i);
        }
        const unsigned second = valid & ~first;
        const unsigned mine = (unsigned)__popc(first) | ((unsigned)__popc(second) << 16);
        const unsigned incl = wave_scan_pair(mine);
        const unsigned excl = incl - mine;
        unsigned p1 = excl & 0xFFFFu, p2 = excl >> 16;
#pragma unroll
        for (int j = 0; j < kVec; ++j) {
            if (first & (1u << j))
                dense1[p1++] = g[j];
            else if (second & (1u << j))
                dense2[p2++] = g[j];
        }
        const unsigned tot = __shfl(incl, 63, 64);
        const unsigned n1 = tot & 0xFFFFu, n2 = tot >> 16;
        __syncthreads();
        if (out1)
            for (unsigned k = threadIdx.x; k < n1; k += kBlock)
                __builtin_nontemporal_store(dense1[k], out1 + carry1 + k);
        if (out2)
            for (unsigned k = threadIdx.x; k < n2; k += kBlock)
                __builtin_nontemporal_store(dense2[k], out2 + carry2 + k);
        __syncthreads();               // the next pass reuses the two buffers
        carry1 += n1;
        carry2 += n2;
    }
}

// ---------------------------------------------------------------------------
// PS aggregate + update of one stage from dense arrays: same arithmetic, in the
// same order, as k_aggregate_update.
// ---------------------------------------------------------------------------
struct PackedAggArgs {
    const Span *spans;
    const int *span_layer;
    const uint8_t *gib_layer;
    const uint32_t *bitmap;
    int chunk_elems;
    int element;
    const long long *base;             // pack index of this stage
    float *P;
    float *V;
    const float *packed;
    long long packed_stride;
    const float *weights;
    double *partial;
    uint32_t *key;                     // KEYS
    int n_workers;
    int stage;
    float inv_n, lr, mu;
};

template <bool WEIGHTED, bool KEYS>
__global__ __launch_bounds__(kBlock) void k_aggregate_update_packed(const PackedAggArgs a)
{
    Piece c;
    if (!owned_piece(a.spans, a.chunk_elems, c))
        return;
    const long long base = a.base[c.chunk];
    if (a.base[c.chunk + 1] == base) { // no element of this chunk is in the stage
        if (threadIdx.x == 0)
            a.partial[c.chunk] = 0.0;
        return;
    }
    const bool important = a.element ? false : a.gib_layer[a.span_layer[blockIdx.x / kSpanChunks]] != 0;
    const int N = a.n_workers;
    float *Pc = a.P + c.start;
    float *Vc = a.V + c.start;
    const float *src = a.packed + base;
    double imp = 0.0;
    unsigned carry = 0;
    for (unsigned i0 = 0; i0 < (unsigned)c.len; i0 += kStride) {
        const unsigned i = i0 + threadIdx.x * kVec;
        const int rem = (int)c.len - (int)i;
        unsigned first = 0, valid = 0;
        if (rem > 0)
            group_stages(a.element != 0, important, rem, c.start + i, a.bitmap, first, valid);
        const unsigned m = a.stage == 1 ? first : (valid & ~first);
        const unsigned mine = (unsigned)__popc(m);
        const unsigned incl = wave_scan_pair(mine);
        const unsigned pos = carry + incl - mine;
        carry += __shfl(incl, 63, 64);
        if (rem <= 0)
            continue;                  // (this lane; the next pass's scan is still wave-wide)
        // slot of component j inside this lane's run of the dense array
        const unsigned r1 = m & 1u, r2 = r1 + ((m >> 1) & 1u), r3 = r2 + ((m >> 2) & 1u);
        const f4 p = ld_stream(Pc + i);
        const f4 v = ld_stream(Vc + i);
        f4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < N; ++w) {
            const float *s = src + (long long)w * a.packed_stride + pos;
            f4 g = {0.f, 0.f, 0.f, 0.f};
            if (m & 1u) g.x = __builtin_nontemporal_load(s);
            if (m & 2u) g.y = __builtin_nontemporal_load(s + r1);
            if (m & 4u) g.z = __builtin_nontemporal_load(s + r2);
            if (m & 8u) g.w = __builtin_nontemporal_load(s + r3);
            if (WEIGHTED)
                g = g * a.weights[w];
            acc = w == 0 ? g : acc + g;
        }
        const f4 gbar = WEIGHTED ? acc : acc * a.inv_n;
        const f4 prod = gbar * p;
        const f4 q = abs4(prod);
        const f4 mv = v * a.mu;
        const f4 vn = mv + gbar;
        const f4 step = vn * a.lr;
        const f4 pn = p - step;
        imp += masked_sum(m, q);
        if (rem >= kVec) {
            // whole groups are written back whole, as in k_aggregate_update
            st_stream(Vc + i, blend(m, vn, v));
            st_stream(Pc + i, blend(m, pn, p));
            if (KEYS) {
                float *kp = reinterpret_cast<float *>(a.key + c.start + i);
                f4 kf = keys4(q);
                if (a.element)
                    kf = blend(m, kf, ld_stream(kp));
                st_stream(kp, kf);
            }
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j)
                if (m & (1u << j)) {
                    Vc[i + j] = vn[j];
                    Pc[i + j] = pn[j];
                    if (KEYS)
                        a.key[c.start + i + j] = importance_key(q[j]);
                }
        }
    }
    const double total = wave_sum(imp);
    if (threadIdx.x == 0)
        a.partial[c.chunk] = total;
}

} // namespace osp
