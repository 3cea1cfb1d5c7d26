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
    const void *grads;                 // fp32 or bfloat16 arenas
    long long worker_stride;
    void *g_i;                         // or null; same element type as grads
    long long stride_i;
    void *g_u;                         // or null
    long long stride_u;
};

// The splitter moves values as they are stored: a lane's 4 consecutive elements are one
// 16-byte (fp32) or 8-byte (bfloat16) group.
template <typename GT> struct GroupOf;
template <> struct GroupOf<float> { using type = f4; };
template <> struct GroupOf<bf16_t> { using type = u2; };

__device__ __forceinline__ f4 get_group(const float *src) { return ld_stream(src); }
__device__ __forceinline__ void put_group(float *dst, f4 v) { st_stream(dst, v); }
__device__ __forceinline__ float group_elem(f4 v, int j) { return v[j]; }
__device__ __forceinline__ u2 get_group(const bf16_t *src)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u2 *>(src));
}
__device__ __forceinline__ void put_group(bf16_t *dst, u2 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<u2 *>(dst));
}
__device__ __forceinline__ bf16_t group_elem(u2 v, int j)
{
    return (bf16_t)(v[j >> 1] >> ((j & 1) * 16));
}

template <typename GT>
__global__ __launch_bounds__(kBlock) void k_split_gradients(const SplitGradArgs a)
{
    using group_t = typename GroupOf<GT>::type;
    // A workgroup lives for one short chain of dependent loads, so the chain is kept flat:
    // the span entry, then data, pack index and bitmap word together.
    const int span_idx = blockIdx.x / kSpanChunks;
    const Span sp = a.spans[span_idx];
    const int jchunk = blockIdx.x % kSpanChunks;
    const int off = jchunk * a.chunk_elems;
    if (off >= sp.n_elems)
        return;
    const long long start = sp.start + off;
    const unsigned len = (unsigned)(sp.n_elems - off < a.chunk_elems ? sp.n_elems - off : a.chunk_elems);
    const int chunk = sp.chunk_base + jchunk;
    const long long w = blockIdx.y;
    const GT *G = static_cast<const GT *>(a.grads) + w * a.worker_stride + start;
    const unsigned i_first = threadIdx.x * kVec;
    // (a group that straddles the tensor's end is read whole: tensors start on multiples of
    // 4 elements, so the bytes are inside the arena)
    group_t next = {};
    if (i_first < len)
        next = get_group(G + i_first);
    const long long b1 = a.base1[chunk], b1_next = a.base1[chunk + 1], b2 = a.base2[chunk];
    asm volatile("" ::"s"(b2));        // (requested here, with the others, not where it is used)
    // layer-granular GIB: a chunk lies in one stage, and the pack index says which
    const bool layer_important = b1_next != b1;
    GT *out1 = a.g_i ? static_cast<GT *>(a.g_i) + w * a.stride_i + b1 : nullptr;
    GT *out2 = a.g_u ? static_cast<GT *>(a.g_u) + w * a.stride_u + b2 : nullptr;
    if (!a.element) {
        // Layer-granular GIB: the whole chunk goes to one part, at consecutive positions.  Where
        // that run starts on a lane's 4-element boundary (tensor sizes that are multiples of 4:
        // the usual case) this is a plain copy with full-width loads and stores.
        GT *out = layer_important ? out1 : out2;
        if (!out)
            return;
        if ((reinterpret_cast<uintptr_t>(out) & (4 * sizeof(GT) - 1)) == 0) {
            for (unsigned i = i_first; i < len; i += kStride) {
                const group_t cur = next;
                if (i + kStride < len)
                    next = get_group(G + i + kStride);
                if (len - i >= (unsigned)kVec)
                    put_group(out + i, cur);
                else
                    for (unsigned j = 0; j < len - i; ++j)
                        out[i + j] = group_elem(cur, (int)j);
            }
            return;
        }
    }
    // The 4 elements of a lane land at consecutive dense positions, but those are not aligned
    // to the group in general, and four single-element stores per lane would each touch every
    // line of the run a little.  So a pass (256 elements) is put in dense order in LDS first and
    // written out with lane k storing element k, k+64, ...: every store instruction covers
    // consecutive bytes.
    __shared__ GT dense1[kStride], dense2[kStride];
    unsigned carry1 = 0, carry2 = 0;   // elements of each stage in earlier passes over the chunk
    // every lane takes every pass (inactive ones count nothing): the prefix sum is wave-wide
    for (unsigned i0 = 0; i0 < len; i0 += kStride) {
        const unsigned i = i0 + i_first;
        const int rem = (int)len - (int)i;
        const group_t cur = next;
        if (i + kStride < len)
            next = get_group(G + i + kStride);
        unsigned first = 0, valid = 0;
        if (rem > 0)
            group_stages(a.element != 0, layer_important, rem, start + i, a.bitmap, first, valid);
        const unsigned second = valid & ~first;
        const unsigned mine = (unsigned)__popc(first) | ((unsigned)__popc(second) << 16);
        const unsigned incl = wave_scan_pair(mine);
        const unsigned excl = incl - mine;
        unsigned p1 = excl & 0xFFFFu, p2 = excl >> 16;
#pragma unroll
        for (int j = 0; j < kVec; ++j) {
            if (first & (1u << j))
                dense1[p1++] = group_elem(cur, j);
            else if (second & (1u << j))
                dense2[p2++] = group_elem(cur, j);
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
    const void *packed;                // fp32 or bfloat16 dense arrays
    long long packed_stride;
    const float *weights;
    double *partial;
    uint32_t *key;                     // KEYS
    int n_workers;
    int stage;
    float inv_n, lr, mu;
};

template <typename GT>
__device__ __forceinline__ float ld_packed(const GT *p);
template <>
__device__ __forceinline__ float ld_packed<float>(const float *p)
{
    return __builtin_nontemporal_load(p);
}
template <>
__device__ __forceinline__ float ld_packed<bf16_t>(const bf16_t *p)
{
    return __uint_as_float((unsigned)__builtin_nontemporal_load(p) << 16);
}

template <bool WEIGHTED, bool KEYS, typename GT>
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
    // layer-granular GIB: a chunk lies in one stage, so one that has elements of this stage
    // lies in it whole
    const bool important = a.stage == 1;
    const int N = a.n_workers;
    float *Pc = a.P + c.start;
    float *Vc = a.V + c.start;
    const GT *src = static_cast<const GT *>(a.packed) + base;
    // Layer-granular GIB: the chunk's elements sit at consecutive positions from src; if every
    // worker's run starts on a lane's 4-element boundary they are read with full-width loads.
    const bool dense_run = !a.element;
    const bool wide = dense_run && (reinterpret_cast<uintptr_t>(src) & (4 * sizeof(GT) - 1)) == 0 &&
                      (a.packed_stride & 3) == 0;
    double imp = 0.0;
    unsigned carry = 0;
    for (unsigned i0 = 0; i0 < (unsigned)c.len; i0 += kStride) {
        const unsigned i = i0 + threadIdx.x * kVec;
        const int rem = (int)c.len - (int)i;
        unsigned first = 0, valid = 0;
        if (rem > 0)
            group_stages(a.element != 0, important, rem, c.start + i, a.bitmap, first, valid);
        const unsigned m = a.stage == 1 ? first : (valid & ~first);
        unsigned pos = i;
        if (!dense_run) {
            const unsigned mine = (unsigned)__popc(m);
            const unsigned incl = wave_scan_pair(mine);
            pos = carry + incl - mine;
            carry += __shfl(incl, 63, 64);
        }
        if (rem <= 0)
            continue;                  // (this lane; the next pass's scan is still wave-wide)
        // slot of component j inside this lane's run of the dense array
        const unsigned r1 = m & 1u, r2 = r1 + ((m >> 1) & 1u), r3 = r2 + ((m >> 2) & 1u);
        const f4 p = ld_stream(Pc + i);
        const f4 v = ld_stream(Vc + i);
        f4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < N; ++w) {
            const GT *s = src + (long long)w * a.packed_stride + pos;
            f4 g = {0.f, 0.f, 0.f, 0.f};
            if (wide && rem >= kVec) {
                g = ld_grad<GT>(s);
            } else {
                if (m & 1u) g.x = ld_packed<GT>(s);
                if (m & 2u) g.y = ld_packed<GT>(s + r1);
                if (m & 4u) g.z = ld_packed<GT>(s + r2);
                if (m & 8u) g.w = ld_packed<GT>(s + r3);
            }
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
