// Split kernels: turn this iteration's importances into the next GIB.
//
// Layer granularity: finish the per-layer fp64 sums from the per-chunk partials
// (fixed order, so the result is reproducible), rank the L layers by
// (importance, index) and take the longest prefix that fits the budget.
//
// Element granularity: exact selection of the `budget` smallest 32-bit keys
// with ties broken by arena index: two radix passes (11 + 11 bits, most
// significant first) with per-workgroup LDS histograms find the upper 22 bits
// of the threshold key, a third pass writes the bitmap and lists the few keys
// that share those bits, and one workgroup decides among them.  Integer
// arithmetic only.
#pragma once
#include "osp_stream_kernels.hpp"

namespace osp {

constexpr int kSplitBlock = 256;       // 4 wavefronts
constexpr int kSplitStride = kSplitBlock * kVec;

// Written by the device into pinned host memory: the lengths of the two stage
// tables and the number of stage-2 elements, then a sequence number (released
// at system scope) that tells the host which split they belong to.
struct StageCounts {
    int n[2];
    long long n_stage2;
    unsigned int seq;
    unsigned int pad;
};

__device__ __forceinline__ void publish_counts(StageCounts *out, int n1, int n2,
                                               long long n_stage2, unsigned seq)
{
    out->n[0] = n1;
    out->n[1] = n2;
    out->n_stage2 = n_stage2;
    __hip_atomic_store(&out->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// One value from device memory into host memory the device can write (pinned, mapped).
__global__ void k_publish_i64(const long long *__restrict__ src, long long *__restrict__ dst_host)
{
    __hip_atomic_store(dst_host, *src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

struct SplitState {                    // one per context, in the workspace
    long long n_stage2;                // elements in stage 2 under the current GIB
    int stage_spans[2][2];             // [table set][stage - 1]: spans in that set's stage table
                                       // (layer GIB; two sets of tables, written alternately)
    // element split: what radix pass p decided (recorded by workgroup 0 of the launch after it)
    unsigned long long k_rem[3];       // rank still to be found inside the bucket pass p chose
    unsigned int prefix[3];            // key bits decided after pass p (right-aligned)
    unsigned int threshold;            // T
    unsigned long long ties_to_take;   // r: how many of the keys equal to T go to stage 2
    unsigned int done;                 // 1: budget 0, nothing is selected
    unsigned int all_ties;             // 1: every key equal to T is taken
    unsigned int collect;              // 1: few keys share the threshold's 22-bit prefix; the bitmap
                                       // pass lists them and one workgroup decides among them
    unsigned int next_guess;           // 1 + the first digit of the last split's threshold (0: none):
                                       // the bucket the next split's first pass refines on spec
    unsigned int layer_ticket;         // workgroups of k_layer_split_lds that have summed their segments
    long long *log;                    // caller's log of stage-2 sizes, or null (osp_set_stage2_log)
    long long log_cap;
    unsigned long long n_splits;       // splits since the log was set
};

// Every split leaves the size of its stage 2 in the caller's log (if there is one).
__device__ __forceinline__ void log_stage2(SplitState *st, long long n_stage2)
{
    if (st->log != nullptr)
        st->log[st->n_splits % (unsigned long long)st->log_cap] = n_stage2;
    st->n_splits += 1;
}

__global__ void k_set_stage2_log(SplitState *st, long long *log, long long cap)
{
    st->log = log;
    st->log_cap = cap;
    st->n_splits = 0;
}

// Keys that share the threshold's upper 22 bits, listed by the bitmap pass when there are few of
// them (the usual case): one workgroup then decides among them instead of more passes over all
// keys.
struct TieCandidate {
    unsigned long long index;          // arena index of the element
    unsigned int key;
    unsigned int pad;
};
constexpr unsigned kTieCandidates = 65536;    // capacity of the list

// "Last workgroup done" without memory fences.  A fence at device scope writes back and
// invalidates the whole L2 of the compute die on this GPU; a thousand workgroups doing that
// cost more than the pass they belong to.  Instead everything that one workgroup hands to the
// last one goes through device-scope atomics that RETURN a value: the value comes back once
// the operation has been performed where every compute die sees it, so when a workgroup's
// threads have all got their values back (wait_for) and passed the barrier, its ticket is drawn
// after its data is in place; the workgroup that draws the last ticket then reads the data with
// device-scope loads.  No workgroup waits for another.
__device__ __forceinline__ void wait_for(unsigned long long returned)
{   // the compiler may not drop or delay what produced `returned`
    asm volatile("" ::"v"(returned) : "memory");
}

__device__ __forceinline__ unsigned long long load_device_scope(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ double load_device_scope(const double *p)
{
    return __longlong_as_double((long long)__hip_atomic_load(
        reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// Store one double where every compute die sees it; returns when it is there.
__device__ __forceinline__ void store_device_scope(double *p, double x)
{
    wait_for(__hip_atomic_exchange(reinterpret_cast<unsigned long long *>(p),
                                   (unsigned long long)__double_as_longlong(x), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT));
}

// True in exactly one workgroup of the launch: the one whose threads all get here last.  Every
// thread must have waited (wait_for) for the device-scope atomics it wants the last workgroup
// to see.  The ticket counter is left at zero.
__device__ __forceinline__ bool last_workgroup(unsigned int *ticket)
{
    __shared__ bool last;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = t == gridDim.x - 1;
        if (last)
            __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    return last;
}

// ---------------------------------------------------------------------------
// layer granularity
// ---------------------------------------------------------------------------

// Deterministic sum of one double per thread over a workgroup of BLOCK threads:
// fixed butterfly inside each wavefront, then the wavefront totals in order.
// The result is valid in thread 0.
template <int BLOCK>
__device__ __forceinline__ double block_sum(double x)
{
    __shared__ double wave_part[BLOCK / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x += __shfl_down(x, off, 64);
    if ((threadIdx.x & 63) == 0)
        wave_part[threadIdx.x >> 6] = x;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < BLOCK / 64; ++i)
        s += wave_part[i];
    return s;
}

// The per-chunk partials of a layer are summed in two fixed-order levels:
// segments of at most kSegChunks consecutive chunks of one layer, one workgroup
// each, then the segment sums of a layer in ascending order.
constexpr int kSegChunks = 2048;

struct Segment {
    int begin, end;                    // chunk index range [begin, end)
    int layer;
    int pad;
};

// mode 0: partials of a stage-0 (single pass) aggregate are in slot 0;
// mode 1: layer-granular GIB, layer l was aggregated by stage gib[l] ? 1 : 2;
// mode 2: element-granular GIB, both stages visited every chunk.
__global__ __launch_bounds__(kSplitBlock) void k_segment_importance(
    const Segment *__restrict__ segs, const double *__restrict__ partial_s1,
    const double *__restrict__ partial_s2, const uint8_t *__restrict__ gib_layer, int mode,
    double *__restrict__ seg_sum)
{
    const Segment sg = segs[blockIdx.x];
    const double *src = partial_s1;
    if (mode == 1 && gib_layer[sg.layer] == 0)
        src = partial_s2;
    double s = 0.0;
    for (int c = sg.begin + (int)threadIdx.x; c < sg.end; c += kSplitBlock) {
        double x = src[c];
        if (mode == 2)
            x += partial_s2[c];
        s += x;
    }
    const double total = block_sum<kSplitBlock>(s);
    if (threadIdx.x == 0)
        seg_sum[blockIdx.x] = total;
}

__device__ __forceinline__ unsigned long long importance_rank_key(double x)
{   // x >= 0, +Inf or NaN: the bit pattern orders like the value; all NaNs
    // collapse to one pattern above +Inf
    return (x != x) ? 0x7FF8000000000000ull
                    : ((unsigned long long)__double_as_longlong(x) & 0x7FFFFFFFFFFFFFFFull);
}

constexpr int kRankBlock = 1024;
// Up to this many spans the ranking workgroup fills the stage tables itself (one launch less).
constexpr int kRankFillMaxSpans = 4096;

// Exclusive scan of one value per thread over a workgroup of BLOCK threads, in
// thread order (shuffles inside a wavefront, wavefront totals through LDS).
// total (may be null) gets the sum.  All threads of the workgroup must call it.
template <int BLOCK, class T>
__device__ __forceinline__ T block_scan_exclusive(T x, T *total)
{
    __shared__ T wave_tot[BLOCK / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    T incl = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const T up = __shfl_up(incl, off, 64);
        if (lane >= off)
            incl += up;
    }
    __syncthreads();                   // wave_tot may still be read from a previous call
    if (lane == 63)
        wave_tot[wave] = incl;
    __syncthreads();
    T base = 0, sum = 0;
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

constexpr int kRankTile = 2048;        // importance keys staged in LDS per pass of the ranking
constexpr int kFewSegments = 16;       // up to here one thread sums a layer's segments

// One workgroup: finish the layer importances (Eq. 4), rank the layers by
// (importance, index), cut the ranking where the running size first exceeds
// the budget, write the layer GIB and the bases of the two stage tables.
// scratch: [L] long long.
__global__ __launch_bounds__(kRankBlock) void k_layer_rank(
    int L, const double *__restrict__ seg_sum, const int *__restrict__ layer_seg_begin,
    const int *__restrict__ big_layers, int n_big, double *__restrict__ imp, const long long *__restrict__ numel,
    const int *__restrict__ layer_span_begin, long long budget,
    uint8_t *__restrict__ gib_layer, int *__restrict__ order, int *__restrict__ layer_base,
    long long *__restrict__ scratch, SplitState *__restrict__ st,
    StageCounts *__restrict__ counts_out, unsigned seq, int set)
{
    __shared__ __align__(16) unsigned long long tile[kRankTile];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // I^l = sum of the layer's segment sums (fixed order per layer).  Layers with
    // few segments: one thread each, ascending.  Layers with many: one wavefront
    // each, lanes take segments lane, lane+64, ... in order, then a fixed butterfly.
    for (int l = threadIdx.x; l < L; l += kRankBlock) {
        const int g0 = layer_seg_begin[l], g1 = layer_seg_begin[l + 1];
        if (g1 - g0 <= kFewSegments) {
            double s = 0.0;
            for (int g = g0; g < g1; ++g)
                s += seg_sum[g];
            imp[l] = s;
        }
    }
    for (int i = wave; i < n_big; i += kRankBlock / 64) {
        const int l = big_layers[i];   // the layers with more than kFewSegments segments
        const int g0 = layer_seg_begin[l], g1 = layer_seg_begin[l + 1];
        double s = 0.0;
        for (int g = g0 + lane; g < g1; g += 64)
            s += seg_sum[g];
        s = wave_sum(s);
        if (lane == 0)
            imp[l] = s;
    }
    __syncthreads();

    const int per = (L + kRankBlock - 1) / kRankBlock;
    {
        // rank[l] = number of layers that come before l in the order (importance, index);
        // a thread owns layers t, t+1024, ...; all keys pass through LDS in tiles
        for (int rep = 0; rep < per; ++rep) {
            const int l = rep * kRankBlock + (int)threadIdx.x;
            const unsigned long long mine = l < L ? importance_rank_key(imp[l]) : 0ull;
            int rank = 0;
            for (int t0 = 0; t0 < L; t0 += kRankTile) {
                const int tn = L - t0 < kRankTile ? L - t0 : kRankTile;
                __syncthreads();
                for (int j = threadIdx.x; j < tn; j += kRankBlock)
                    tile[j] = importance_rank_key(imp[t0 + j]);
                __syncthreads();
                if (l < L) {
                    // every thread reads the same keys (LDS broadcast); four per iteration as two
                    // 16-byte reads, so the loop is not bound by the latency of one read per key
                    int j = 0;
                    for (; j + 4 <= tn; j += 4) {
                        const ulonglong2 a = *reinterpret_cast<const ulonglong2 *>(&tile[j]);
                        const ulonglong2 b = *reinterpret_cast<const ulonglong2 *>(&tile[j + 2]);
                        rank += (a.x < mine) || (a.x == mine && t0 + j < l);
                        rank += (a.y < mine) || (a.y == mine && t0 + j + 1 < l);
                        rank += (b.x < mine) || (b.x == mine && t0 + j + 2 < l);
                        rank += (b.y < mine) || (b.y == mine && t0 + j + 3 < l);
                    }
                    for (; j < tn; ++j) {
                        const unsigned long long other = tile[j];
                        rank += (other < mine) || (other == mine && t0 + j < l);
                    }
                }
            }
            if (l < L) {
                order[rank] = l;
                scratch[rank] = numel[l];
            }
        }
    }
    if (threadIdx.x == 0)
        st->n_stage2 = 0;
    __syncthreads();

    // running size along the ranking; sizes are positive, so "cumulative size <= budget"
    // holds exactly on a prefix: the prefix rule needs no further test
    long long carry = 0;
    for (int rep = 0; rep < per; ++rep) {
        const int r = rep * kRankBlock + (int)threadIdx.x;
        const long long mine = r < L ? scratch[r] : 0;
        long long total;
        const long long incl = carry + block_scan_exclusive<kRankBlock, long long>(mine, &total) + mine;
        if (r < L) {
            const bool fits = incl <= budget;
            gib_layer[order[r]] = fits ? 0 : 1;
            const bool last = r == L - 1 || incl + scratch[r + 1] > budget;
            if (fits && last)
                st->n_stage2 = incl;
        }
        carry += total;
    }
    __syncthreads();

    // bases of the two stage tables: exclusive scans over the layers, in layer order
    int carry1 = 0, carry2 = 0;
    for (int rep = 0; rep < per; ++rep) {
        const int l = rep * kRankBlock + (int)threadIdx.x;
        int ns = 0;
        bool important = true;
        if (l < L) {
            ns = layer_span_begin[l + 1] - layer_span_begin[l];
            important = gib_layer[l] != 0;
        }
        int tot1, tot2;
        const int b1 = block_scan_exclusive<kRankBlock, int>(important ? ns : 0, &tot1);
        const int b2 = block_scan_exclusive<kRankBlock, int>(important ? 0 : ns, &tot2);
        if (l < L)
            layer_base[l] = important ? carry1 + b1 : carry2 + b2;
        carry1 += tot1;
        carry2 += tot2;
    }
    if (threadIdx.x == 0) {
        st->stage_spans[set][0] = carry1;
        st->stage_spans[set][1] = carry2;
        log_stage2(st, st->n_stage2);
        publish_counts(counts_out, carry1, carry2, st->n_stage2, seq);   // a hint for the host's next grids
    }
}

// The same for L <= kRankTile (every model of the paper), with all intermediate
// arrays in LDS: a bitonic sort of (importance, index) pairs instead of the
// all-pairs count, and no global round trip between the phases.  If n_spans > 0
// the workgroup also fills the two stage tables (what k_stage_lists does), after
// it has published their lengths.  Run by one workgroup of BLOCK threads (the one
// of k_layer_split_lds that finishes last).  (Measured with BLOCK = 256 for small
// L: 1 us less at L = 62, 6 us more at L = 467; kRankBlock throughout.)
template <int BLOCK>
__device__ __forceinline__ void layer_rank_in_lds(
    int L, const double *__restrict__ seg_sum, const int *__restrict__ layer_seg_begin,
    const int *__restrict__ big_layers, int n_big, double *__restrict__ imp,
    const long long *__restrict__ numel, const int *__restrict__ layer_span_begin, long long budget,
    uint8_t *__restrict__ gib_layer, int *__restrict__ order, int *__restrict__ layer_base,
    SplitState *__restrict__ st, StageCounts *__restrict__ counts_out, unsigned seq, int set,
    int n_spans, const Span *__restrict__ spans, const int *__restrict__ span_layer,
    Span *__restrict__ list_s1, Span *__restrict__ list_s2)
{
    __shared__ __align__(16) unsigned long long key[kRankTile];
    __shared__ long long numel_of_layer[kRankTile];
    __shared__ int sorted_layer[kRankTile];
    __shared__ int base_of_layer[kRankTile];
    __shared__ int first_span_of_layer[kRankTile];
    __shared__ uint8_t important_layer[kRankTile];
    __shared__ long long n_stage2_found;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int n = 1;
    while (n < L)
        n <<= 1;

    // Everything the later phases read from global memory that does not depend on the ranking
    // is requested here, so that its latency passes behind the importance sums and the sort
    // instead of adding one round trip per phase (the kernel is a chain of short phases).
    constexpr int kLayersPer = kRankTile / BLOCK, kSpansPer = kRankFillMaxSpans / BLOCK;
    static_assert(kRankTile % BLOCK == 0 && kRankFillMaxSpans % BLOCK == 0, "whole rounds per thread");
    long long my_numel[kLayersPer];
    int my_first[kLayersPer], my_end[kLayersPer];
#pragma unroll
    for (int rep = 0; rep < kLayersPer; ++rep) {
        const int l = rep * BLOCK + (int)threadIdx.x;
        my_numel[rep] = l < L ? numel[l] : 0;
        my_first[rep] = l < L ? layer_span_begin[l] : 0;
        my_end[rep] = l < L ? layer_span_begin[l + 1] : 0;
    }
    Span my_span[kSpansPer];
    int my_span_layer[kSpansPer];
#pragma unroll
    for (int j = 0; j < kSpansPer; ++j) {
        const int k = j * BLOCK + (int)threadIdx.x;
        if (k < n_spans) {
            my_span[j] = spans[k];
            my_span_layer[j] = span_layer[k];
        }
    }

    // I^l (same two summation schemes as k_layer_rank), straight into the sort keys
    for (int l = threadIdx.x; l < n; l += BLOCK) {
        sorted_layer[l] = l;
        if (l >= L) {
            key[l] = ~0ull;            // padding sorts behind every layer, NaN ones included
            continue;
        }
        const int g0 = layer_seg_begin[l], g1 = layer_seg_begin[l + 1];
        if (g1 - g0 <= kFewSegments) {
            double s = 0.0;
            for (int g = g0; g < g1; ++g)
                s += load_device_scope(&seg_sum[g]);   // (written by this launch)
            imp[l] = s;
            key[l] = importance_rank_key(s);
        }
    }
    for (int i = wave; i < n_big; i += BLOCK / 64) {
        const int l = big_layers[i];
        const int g0 = layer_seg_begin[l], g1 = layer_seg_begin[l + 1];
        double s = 0.0;
        for (int g = g0 + lane; g < g1; g += 64)
            s += load_device_scope(&seg_sum[g]);   // (written by this launch)
        s = wave_sum(s);
        if (lane == 0) {
            imp[l] = s;
            key[l] = importance_rank_key(s);
        }
    }
    if (threadIdx.x == 0)
        n_stage2_found = 0;
    __syncthreads();

    for (int k = 2; k <= n; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (n >> 1); t += BLOCK) {
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));   // bit j of i is clear
                const int p = i | j;
                const bool ascending = (i & k) == 0;
                const unsigned long long a = key[i], b = key[p];
                const int la = sorted_layer[i], lb = sorted_layer[p];
                const bool a_after_b = a > b || (a == b && la > lb);
                if (a_after_b == ascending) {
                    key[i] = b; key[p] = a;
                    sorted_layer[i] = lb; sorted_layer[p] = la;
                }
            }
            __syncthreads();
        }

#pragma unroll
    for (int rep = 0; rep < kLayersPer; ++rep) {
        const int l = rep * BLOCK + (int)threadIdx.x;
        if (l < L) {
            numel_of_layer[l] = my_numel[rep];
            first_span_of_layer[l] = my_first[rep];
            order[l] = sorted_layer[l];     // (position l of the ranking)
        }
    }
    __syncthreads();

    // running size along the ranking (sizes are positive: "fits" holds exactly on a prefix)
    long long carry = 0;
#pragma unroll
    for (int rep = 0; rep < kLayersPer; ++rep) {
        if (rep * BLOCK >= L)
            break;
        const int r = rep * BLOCK + (int)threadIdx.x;
        const long long mine = r < L ? numel_of_layer[sorted_layer[r]] : 0;
        long long total;
        const long long incl = carry + block_scan_exclusive<BLOCK, long long>(mine, &total) + mine;
        if (r < L) {
            const bool fits = incl <= budget;
            const int l = sorted_layer[r];
            important_layer[l] = fits ? 0 : 1;
            gib_layer[l] = fits ? 0 : 1;
            const bool last = r == L - 1 || incl + numel_of_layer[sorted_layer[r + 1]] > budget;
            if (fits && last)
                n_stage2_found = incl;
        }
        carry += total;
    }
    __syncthreads();

    // bases of the two stage tables: exclusive scans over the layers, in layer order
    int carry1 = 0, carry2 = 0;
#pragma unroll
    for (int rep = 0; rep < kLayersPer; ++rep) {
        if (rep * BLOCK >= L)
            break;
        const int l = rep * BLOCK + (int)threadIdx.x;
        int ns = 0;
        bool important = true;
        if (l < L) {
            ns = my_end[rep] - my_first[rep];
            important = important_layer[l] != 0;
        }
        int tot1, tot2;
        const int b1 = block_scan_exclusive<BLOCK, int>(important ? ns : 0, &tot1);
        const int b2 = block_scan_exclusive<BLOCK, int>(important ? 0 : ns, &tot2);
        if (l < L) {
            const int base = important ? carry1 + b1 : carry2 + b2;
            base_of_layer[l] = base;
            layer_base[l] = base;
        }
        carry1 += tot1;
        carry2 += tot2;
    }
    if (threadIdx.x == 0) {
        st->n_stage2 = n_stage2_found;
        st->stage_spans[set][0] = carry1;
        st->stage_spans[set][1] = carry2;
        log_stage2(st, n_stage2_found);
        publish_counts(counts_out, carry1, carry2, n_stage2_found, seq);
    }
    __syncthreads();
    // Span k goes to its place in its stage's table; the same place behind the other table's
    // last entry is cleared (the two lengths add up to the number of spans, so this clears
    // exactly the unused entries: a table ends at its first cleared entry).
    Span cleared;
    cleared.start = 0; cleared.n_elems = 0; cleared.chunk_base = 0;
#pragma unroll
    for (int j = 0; j < kSpansPer; ++j) {
        const int k = j * BLOCK + (int)threadIdx.x;
        if (k < n_spans) {
            const int l = my_span_layer[j];
            const int pos = base_of_layer[l] + (k - first_span_of_layer[l]);
            if (important_layer[l]) {
                list_s1[pos] = my_span[j];
                list_s2[carry2 + pos] = cleared;
            } else {
                list_s2[pos] = my_span[j];
                list_s1[carry1 + pos] = cleared;
            }
        }
    }
}

// The same for at most 64 layers (VGG-16, ResNet-18): the ranking runs in ONE wavefront, a layer
// per lane, with cross-lane shuffles where the LDS version has barriers (a bitonic sort of 64
// keys is 21 compare-exchange rounds: 21 barriers of a 1024-thread workgroup there, none here);
// one barrier before the whole workgroup fills the stage tables.  Same sums, same order of
// operations per layer, same results.
constexpr int kRankWaveLayers = 64;

template <int BLOCK>
__device__ __forceinline__ void layer_rank_in_wave(
    int L, const double *__restrict__ seg_sum, const int *__restrict__ layer_seg_begin,
    const int *__restrict__ big_layers, int n_big, double *__restrict__ imp,
    const long long *__restrict__ numel, const int *__restrict__ layer_span_begin, long long budget,
    uint8_t *__restrict__ gib_layer, int *__restrict__ order, int *__restrict__ layer_base,
    SplitState *__restrict__ st, StageCounts *__restrict__ counts_out, unsigned seq, int set,
    int n_spans, const Span *__restrict__ spans, const int *__restrict__ span_layer,
    Span *__restrict__ list_s1, Span *__restrict__ list_s2)
{
    __shared__ int w_base[kRankWaveLayers], w_first[kRankWaveLayers], w_total[2];
    __shared__ uint8_t w_important[kRankWaveLayers];
    // (requested up front, as in the LDS version)
    constexpr int kSpansPer = kRankFillMaxSpans / BLOCK;
    Span my_span[kSpansPer];
    int my_span_layer[kSpansPer];
#pragma unroll
    for (int j = 0; j < kSpansPer; ++j) {
        const int k = j * BLOCK + (int)threadIdx.x;
        if (k < n_spans) {
            my_span[j] = spans[k];
            my_span_layer[j] = span_layer[k];
        }
    }
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const bool live = lane < L;
        const long long my_numel = live ? numel[lane] : 0;
        const int first = live ? layer_span_begin[lane] : 0;
        const int n_my_spans = live ? layer_span_begin[lane + 1] - first : 0;
        // I^l: layers of few segments by their own lane, in order; layers of many by the whole
        // wavefront, one layer at a time (lanes take segments lane, lane+64, ..., then the butterfly)
        double s = 0.0;
        if (live) {
            const int g0 = layer_seg_begin[lane], g1 = layer_seg_begin[lane + 1];
            if (g1 - g0 <= kFewSegments)
                for (int g = g0; g < g1; ++g)
                    s += load_device_scope(&seg_sum[g]);   // (written by this launch)
        }
        for (int i = 0; i < n_big; ++i) {
            const int lb = big_layers[i];
            const int g0 = layer_seg_begin[lb], g1 = layer_seg_begin[lb + 1];
            double t = 0.0;
            for (int g = g0 + lane; g < g1; g += 64)
                t += load_device_scope(&seg_sum[g]);
            t = __shfl(wave_sum(t), 0, 64);
            if (lane == lb)
                s = t;
        }
        if (live)
            imp[lane] = s;
        // bitonic sort of (importance, layer) over the 64 lanes; padding lanes sort last
        unsigned long long key = live ? importance_rank_key(s) : ~0ull;
        int idx = lane;
#pragma unroll
        for (int k = 2; k <= 64; k <<= 1)
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1) {
                const unsigned long long o_key = __shfl_xor(key, j, 64);
                const int o_idx = __shfl_xor(idx, j, 64);
                const bool other_first = o_key < key || (o_key == key && o_idx < idx);
                const bool keep_first = ((lane & j) == 0) == ((lane & k) == 0);
                if (keep_first == other_first) {
                    key = o_key;
                    idx = o_idx;
                }
            }
        // lane r now holds the layer ranked r-th: running size along the ranking (sizes are
        // positive, so "fits" holds exactly on a prefix)
        const long long size_r = __shfl(my_numel, idx, 64);
        long long incl = size_r;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long up = __shfl_up(incl, off, 64);
            if (lane >= off)
                incl += up;
        }
        const bool fits = lane < L && incl <= budget;
        long long n_stage2 = fits ? incl : 0;              // the largest fitting prefix
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const long long other = __shfl_xor(n_stage2, off, 64);
            n_stage2 = other > n_stage2 ? other : n_stage2;
        }
        if (lane < L) {
            order[lane] = idx;
            w_important[idx] = fits ? 0 : 1;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const bool important = live ? w_important[lane] != 0 : true;
        if (live)
            gib_layer[lane] = important ? 1 : 0;
        // bases of the two stage tables: exclusive scans over the layers, in layer order
        int in1 = important ? n_my_spans : 0, in2 = important ? 0 : n_my_spans;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int u1 = __shfl_up(in1, off, 64), u2 = __shfl_up(in2, off, 64);
            if (lane >= off) {
                in1 += u1;
                in2 += u2;
            }
        }
        const int tot1 = __shfl(in1, 63, 64), tot2 = __shfl(in2, 63, 64);
        if (live) {
            const int base = important ? in1 - n_my_spans : in2 - n_my_spans;
            w_base[lane] = base;
            w_first[lane] = first;
            layer_base[lane] = base;
        }
        if (lane == 0) {
            w_total[0] = tot1;
            w_total[1] = tot2;
            st->n_stage2 = n_stage2;
            st->stage_spans[set][0] = tot1;
            st->stage_spans[set][1] = tot2;
            log_stage2(st, n_stage2);
            publish_counts(counts_out, tot1, tot2, n_stage2, seq);
        }
    }
    __syncthreads();
    const int carry1 = w_total[0], carry2 = w_total[1];
    Span cleared;
    cleared.start = 0; cleared.n_elems = 0; cleared.chunk_base = 0;
#pragma unroll
    for (int j = 0; j < kSpansPer; ++j) {
        const int k = j * BLOCK + (int)threadIdx.x;
        if (k < n_spans) {
            const int l = my_span_layer[j];
            const int pos = w_base[l] + (k - w_first[l]);
            if (w_important[l]) {
                list_s1[pos] = my_span[j];
                list_s2[carry2 + pos] = cleared;
            } else {
                list_s2[pos] = my_span[j];
                list_s1[carry1 + pos] = cleared;
            }
        }
    }
}

// The whole layer-granular split in one launch for L <= kRankTile: every workgroup sums four
// segments of per-chunk importance partials (each by 256 threads, in k_segment_importance's
// order, so the sums are the same bit for bit), and the workgroup that finishes last ranks
// the layers and writes the GIB and the stage tables.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_layer_split_lds(
    const Segment *__restrict__ segs, int n_segments, const double *__restrict__ partial_s1,
    const double *__restrict__ partial_s2, int mode, double *__restrict__ seg_sum,
    int L, const int *__restrict__ layer_seg_begin, const int *__restrict__ big_layers, int n_big,
    double *__restrict__ imp, const long long *__restrict__ numel,
    const int *__restrict__ layer_span_begin, long long budget, uint8_t *__restrict__ gib_layer,
    int *__restrict__ order, int *__restrict__ layer_base, SplitState *__restrict__ st,
    StageCounts *__restrict__ counts_out, unsigned seq, int set, int n_spans,
    const Span *__restrict__ spans, const int *__restrict__ span_layer,
    Span *__restrict__ list_s1, Span *__restrict__ list_s2)
{
    static_assert(BLOCK % kSplitBlock == 0, "whole segments per workgroup");
    constexpr int kPer = BLOCK / kSplitBlock;              // segments per workgroup
    __shared__ double wave_part[BLOCK / 64];
    {
        const int quarter = threadIdx.x / kSplitBlock, t = threadIdx.x % kSplitBlock;
        const int g = blockIdx.x * kPer + quarter;
        double x = 0.0;
        if (g < n_segments) {
            const Segment sg = segs[g];
            const double *src = partial_s1;
            if (mode == 1 && gib_layer[sg.layer] == 0)
                src = partial_s2;
            for (int c = sg.begin + t; c < sg.end; c += kSplitBlock) {
                double v = src[c];
                if (mode == 2)
                    v += partial_s2[c];
                x += v;
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1)
            x += __shfl_down(x, off, 64);
        if ((threadIdx.x & 63) == 0)
            wave_part[threadIdx.x >> 6] = x;
        __syncthreads();
        if (t == 0 && g < n_segments) {
            double total = 0.0;
#pragma unroll
            for (int i = 0; i < kSplitBlock / 64; ++i)
                total += wave_part[quarter * (kSplitBlock / 64) + i];
            store_device_scope(&seg_sum[g], total);
        }
    }
    if (!last_workgroup(&st->layer_ticket))
        return;
    if (L <= kRankWaveLayers)
        layer_rank_in_wave<BLOCK>(L, seg_sum, layer_seg_begin, big_layers, n_big, imp, numel,
                                  layer_span_begin, budget, gib_layer, order, layer_base, st,
                                  counts_out, seq, set, n_spans, spans, span_layer, list_s1, list_s2);
    else
        layer_rank_in_lds<BLOCK>(L, seg_sum, layer_seg_begin, big_layers, n_big, imp, numel,
                                 layer_span_begin, budget, gib_layer, order, layer_base, st, counts_out,
                                 seq, set, n_spans, spans, span_layer, list_s1, list_s2);
}

// After a GIB was uploaded from the host: only the table bases are needed.
__global__ void k_stage_bases(int L, const uint8_t *__restrict__ gib_layer,
                              const int *__restrict__ layer_span_begin,
                              int *__restrict__ layer_base, SplitState *__restrict__ st,
                              StageCounts *__restrict__ counts_out, unsigned seq, int set)
{
    if (blockIdx.x != 0 || threadIdx.x != 0)
        return;
    int n1 = 0, n2 = 0;
    for (int l = 0; l < L; ++l) {
        const int ns = layer_span_begin[l + 1] - layer_span_begin[l];
        if (gib_layer[l]) {
            layer_base[l] = n1;
            n1 += ns;
        } else {
            layer_base[l] = n2;
            n2 += ns;
        }
    }
    st->stage_spans[set][0] = n1;
    st->stage_spans[set][1] = n2;
    publish_counts(counts_out, n1, n2, st->n_stage2, seq);
}

// Fill the two stage tables: span k of layer l goes to position
// layer_base[l] + (k - first span of l) of the table of l's stage, and the same position
// behind the other table's last entry is cleared (see k_layer_rank_lds).
__global__ __launch_bounds__(kSplitBlock) void k_stage_lists(
    int n_spans, const Span *__restrict__ spans, const int *__restrict__ span_layer,
    const uint8_t *__restrict__ gib_layer, const int *__restrict__ layer_span_begin,
    const int *__restrict__ layer_base, const SplitState *__restrict__ st, int set,
    Span *__restrict__ list_s1, Span *__restrict__ list_s2)
{
    const int k = blockIdx.x * kSplitBlock + threadIdx.x;
    if (k >= n_spans)
        return;
    const int l = span_layer[k];
    const int pos = layer_base[l] + (k - layer_span_begin[l]);
    Span cleared;
    cleared.start = 0; cleared.n_elems = 0; cleared.chunk_base = 0;
    if (gib_layer[l]) {
        list_s1[pos] = spans[k];
        list_s2[st->stage_spans[set][1] + pos] = cleared;
    } else {
        list_s2[pos] = spans[k];
        list_s1[st->stage_spans[set][0] + pos] = cleared;
    }
}

// ---------------------------------------------------------------------------
// element granularity
//
// Exact selection of the `budget` smallest 32-bit keys, ties broken by arena index, in six
// launches and three passes over the keys:
//   1. histogram of the top 11 bits;
//   2. histogram of the next 11 bits inside the bucket of the budget-th smallest key;
//   3. bitmap pass: with P = the upper 22 bits of the threshold, a key whose upper 22 bits are
//      below P goes to stage 2, above P to stage 1; the (few) keys with exactly P are listed as
//      candidates and left in stage 1 for now;
//   4. one workgroup picks, among the candidates, the ones that still belong to stage 2 (by
//      their low 10 bits, then by arena index) and clears their bits.
// When more than kTieCandidates keys share P (long runs of equal keys: zeros, quantised
// gradients) launch 4 is instead the histogram of the last 10 bits over all keys, and two more
// launches count the ties per tile and write the bitmap again.  Those two launches are always
// enqueued and return at once when not needed, so the host never has to know.
// Which bucket a finished histogram puts the budget-th smallest key in is worked out by every
// workgroup of the NEXT launch for itself (16 KB of counts from L2 and one scan: a few
// microseconds, no launch of its own, no workgroup waiting for another); workgroup 0 also
// records it for the launches after that.  A histogram is left zeroed by the launch after the
// one that read it.  Integer arithmetic only.
// ---------------------------------------------------------------------------
constexpr int kRadixBins = 2048;
constexpr int kSelectHistograms = 4;   // three digits, and the second digit under a guessed first one
// pass 0: bits 31..21, pass 1: bits 20..10, pass 2: bits 9..0
__device__ __forceinline__ constexpr int radix_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ constexpr int radix_bits(int pass) { return pass == 2 ? 10 : 11; }

constexpr int kSelTile = 8192;         // keys per tile of the bitmap / tie-count passes

__global__ __launch_bounds__(kSplitBlock) void k_fill_u32(uint32_t *p, long long n, uint32_t v)
{
    for (long long i = (long long)blockIdx.x * kSplitBlock + threadIdx.x; i < n;
         i += (long long)gridDim.x * kSplitBlock)
        p[i] = v;
}

// Exclusive scan of one unsigned long long per thread over the 256-thread
// workgroup, in thread order.  total (may be null) gets the sum.
__device__ __forceinline__ unsigned long long block_exclusive_scan(unsigned long long x,
                                                                   unsigned long long *total)
{
    __shared__ unsigned long long wave_tot[kSplitBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long incl = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long up = __shfl_up(incl, off, 64);
        if (lane >= off)
            incl += up;
    }
    __syncthreads();                   // wave_tot may still be read from a previous call
    if (lane == 63)
        wave_tot[wave] = incl;
    __syncthreads();
    unsigned long long base = 0;
    for (int w = 0; w < wave; ++w)
        base += wave_tot[w];
    if (total)
        *total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    return base + incl - x;
}

// The bin that holds the want-th smallest item (want >= 1) of a histogram whose counts are
// spread over the workgroup, PER consecutive bins per thread: the unique bin with
// below < want <= below + count.  Every thread gets the answer; bin < 0 if want exceeds the
// total.  All threads of the workgroup must call it.
template <int PER, int BLOCK = kSplitBlock>
__device__ __forceinline__ void find_rank_bin(const unsigned long long (&c)[PER],
                                              unsigned long long want, int &bin,
                                              unsigned long long &below, unsigned long long &count)
{
    __shared__ int s_bin;
    __shared__ unsigned long long s_below, s_count;
    unsigned long long mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j)
        mine += c[j];
    if (threadIdx.x == 0)
        s_bin = -1;
    const unsigned long long before =
        block_scan_exclusive<BLOCK, unsigned long long>(mine, nullptr);       // (barriers inside)
    if (before < want && want <= before + mine) {
        unsigned long long run = before;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (run < want && want <= run + c[j]) {
                s_bin = (int)threadIdx.x * PER + j;
                s_below = run;
                s_count = c[j];
            }
            run += c[j];
        }
    }
    __syncthreads();
    bin = s_bin;
    below = s_below;
    count = s_count;
    __syncthreads();                   // the shared slots are free for the next call
}

// What radix pass PASS has decided, worked out by a whole workgroup from that pass's finished
// histogram (written by an earlier launch) and from what the pass before it recorded.
struct Picked {
    unsigned prefix;                   // key bits decided so far, right-aligned
    unsigned long long k_rem;          // rank of the wanted key inside the chosen bucket, >= 1
    unsigned long long count;          // keys in the chosen bucket
    bool ok;                           // false: budget beyond the number of keys (cannot happen)
};

template <int PASS, int BLOCK = kSplitBlock>
__device__ __forceinline__ Picked pick_bucket(long long budget,
                                              const unsigned long long *__restrict__ hist,
                                              const SplitState *__restrict__ st)
{
    constexpr int per = kRadixBins / BLOCK;                // consecutive bins per thread
    unsigned long long c[per];
#pragma unroll
    for (int j = 0; j < per; ++j)
        c[j] = hist[threadIdx.x * per + j];
    const unsigned long long k = PASS == 0 ? (unsigned long long)budget : st->k_rem[PASS - 1];
    const unsigned prefix = PASS == 0 ? 0u : st->prefix[PASS - 1];
    int bin;
    unsigned long long below, count;
    find_rank_bin<per, BLOCK>(c, k, bin, below, count);
    Picked r;
    r.ok = bin >= 0;
    r.prefix = (prefix << radix_bits(PASS)) | (unsigned)(bin < 0 ? 0 : bin);
    r.k_rem = k - below;
    r.count = count;
    return r;
}

// Workgroup 0 leaves what a pass decided for the launches after the next one.
template <int PASS>
__device__ __forceinline__ void record_pick(SplitState *__restrict__ st, const Picked &r)
{
    if (blockIdx.x != 0 || threadIdx.x != 0)
        return;
    st->prefix[PASS] = r.prefix;
    st->k_rem[PASS] = r.k_rem;
    if (PASS == 1)                     // few keys share the 22-bit prefix: the bitmap pass lists them
        st->collect = r.ok && r.count <= kTieCandidates ? 1u : 0u;
    if (PASS == 2) {
        st->threshold = r.prefix;
        st->ties_to_take = r.k_rem;
        // (distinct keys around the threshold: all keys equal to T are taken)
        st->all_ties = r.k_rem == r.count ? 1u : 0u;
    }
}

__device__ __forceinline__ void zero_histogram(unsigned long long *__restrict__ hist)
{   // one workgroup, after the last launch that reads it
    for (int b = threadIdx.x; b < kRadixBins; b += blockDim.x)
        hist[b] = 0;
}

// Histogram of one radix digit over all keys (PASS 0), or over the keys whose higher bits
// equal `prefix`; per-workgroup counts in LDS, flushed with one global atomic per non-empty
// bin (nobody waits for them: the next launch reads the sums).  The flush is what a pass over
// few keys costs (the second digit fills nearly all 2048 bins of every workgroup, and the GPU
// retires some 40 G such atomics per second), hence few workgroups of kHistBlock threads.
constexpr int kHistBlock = 1024;
constexpr int kHistVecPerThread = 16;  // 16-byte groups a thread reads (when the grid is not capped)
constexpr int kHistMaxGrid = 512;

//
// SPEC (first pass only): the threshold's first digit rarely moves from one iteration to the
// next, so the pass also counts the second digit of the keys whose first digit is `guess`, into
// hist_guess.  If the guess turns out right that is the second pass's histogram, and the second
// pass over the keys is not made.
template <int PASS, int BLOCK, bool SPEC = false>
__device__ __forceinline__ void select_histogram(const uint32_t *__restrict__ key, long long n_vec,
                                                 unsigned prefix,
                                                 unsigned long long *__restrict__ hist,
                                                 unsigned guess = 0,
                                                 unsigned long long *__restrict__ hist_guess = nullptr)
{
    static_assert(!SPEC || PASS == 0, "only the first pass guesses");
    __shared__ unsigned int h[kRadixBins];
    __shared__ unsigned int hg[SPEC ? kRadixBins : 1];
    for (int b = threadIdx.x; b < kRadixBins; b += BLOCK) {
        h[b] = 0;
        if (SPEC)
            hg[b] = 0;
    }
    __syncthreads();
    constexpr int shift = radix_shift(PASS);
    constexpr unsigned mask = (1u << radix_bits(PASS)) - 1u;
    constexpr int hi = shift + radix_bits(PASS);      // bits above this pass's digit
    const u4 *kv = reinterpret_cast<const u4 *>(key);
    // eight 16-byte loads in flight per thread; keys of one group that fall into one bin
    // (the rule in the first pass, whose digit is mostly exponent) cost one LDS atomic
    constexpr int kUnroll = 8;
    const long long stride = (long long)gridDim.x * BLOCK;
    for (long long v0 = (long long)blockIdx.x * BLOCK + threadIdx.x; v0 < n_vec;
         v0 += kUnroll * stride) {
        u4 k[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long long v = v0 + u * stride;
            if (v < n_vec)
                k[u] = __builtin_nontemporal_load(kv + v);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (v0 + u * stride >= n_vec)
                continue;
            unsigned bin[kVec];
            bool in[kVec];
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const unsigned x = k[u][j];
                in[j] = PASS == 0 || (x >> hi) == prefix;
                bin[j] = (x >> shift) & mask;
            }
            if (in[0] && in[1] && in[2] && in[3] && bin[0] == bin[1] && bin[0] == bin[2] &&
                bin[0] == bin[3]) {
                atomicAdd(&h[bin[0]], 4u);
            } else {
#pragma unroll
                for (int j = 0; j < kVec; ++j)
                    if (in[j])
                        atomicAdd(&h[bin[j]], 1u);
            }
            if (SPEC) {
                constexpr int shift1 = radix_shift(1);
                constexpr unsigned mask1 = (1u << radix_bits(1)) - 1u;
#pragma unroll
                for (int j = 0; j < kVec; ++j)
                    if (bin[j] == guess)
                        atomicAdd(&hg[(k[u][j] >> shift1) & mask1], 1u);
            }
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kRadixBins; b += BLOCK) {
        if (h[b])
            atomicAdd(&hist[b], (unsigned long long)h[b]);
        if (SPEC && hg[b])
            atomicAdd(&hist_guess[b], (unsigned long long)hg[b]);
    }
}

// Launch 1: the top 11 bits.
__global__ __launch_bounds__(kHistBlock) void k_select_histogram0(
    const uint32_t *__restrict__ key, long long n_vec, long long budget,
    SplitState *__restrict__ st, unsigned long long *__restrict__ hist0,
    unsigned long long *__restrict__ hist_guess)
{
    const unsigned next_guess = st->next_guess;      // (written by the last split's launch 4 only)
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st->n_stage2 = budget;
        log_stage2(st, budget);
        st->done = budget == 0 ? 1u : 0u;
        if (budget == 0) {
            st->threshold = 0;
            st->ties_to_take = 0;
            st->all_ties = 0;
            st->collect = 0;
        }
    }
    if (next_guess != 0 && budget != 0)
        select_histogram<0, kHistBlock, true>(key, n_vec, 0u, hist0, next_guess - 1u, hist_guess);
    else
        select_histogram<0, kHistBlock>(key, n_vec, 0u, hist0);
}

// Launch 2: the next 11 bits inside the bucket the first histogram points to.
__global__ __launch_bounds__(kHistBlock) void k_select_histogram1(
    const uint32_t *__restrict__ key, long long n_vec, long long budget,
    SplitState *__restrict__ st, const unsigned long long *__restrict__ hist0,
    unsigned long long *__restrict__ hist1)
{
    if (budget == 0)
        return;                        // nothing is selected; hist0 is zeroed by the bitmap pass
    const Picked p0 = pick_bucket<0, kHistBlock>(budget, hist0, st);
    record_pick<0>(st, p0);
    if (!p0.ok)
        return;
    if (st->next_guess == p0.prefix + 1u)
        return;                        // launch 1 guessed this bucket: its histogram is there already
    select_histogram<1, kHistBlock>(key, n_vec, p0.prefix, hist1);
}

__device__ __forceinline__ u4 load_keys_or_pad(const uint32_t *__restrict__ key, long long v,
                                               long long n_vec)
{
    if (v < n_vec)
        return reinterpret_cast<const u4 *>(key)[v];
    u4 pad;
    pad.x = pad.y = pad.z = pad.w = 0xFFFFFFFFu;
    return pad;
}

// Eight neighbouring lanes hold 4 bits each of one 32-bit bitmap word (bit = 1: important).
__device__ __forceinline__ void store_bitmap_word(unsigned sel, long long v, long long n_words,
                                                  uint32_t *__restrict__ bitmap)
{
    unsigned word = (~sel & 0xFu) << ((threadIdx.x & 7) * 4);
    word |= __shfl_xor(word, 1, 64);
    word |= __shfl_xor(word, 2, 64);
    word |= __shfl_xor(word, 4, 64);
    const long long w = v >> 3;        // 8 lanes x 4 keys = one 32-bit word
    if ((threadIdx.x & 7) == 0 && w < n_words)
        bitmap[w] = word;
}

// Launch 3: the bitmap from the 22-bit prefix P of the threshold.  Upper 22 bits below P:
// stage 2.  Equal to P: listed as a candidate (when few keys share P) and left in stage 1 until
// k_select_finish has decided; above P: stage 1.  Workgroups walk the tiles in rounds of the
// grid, so the prologue (P from the second histogram) is paid once per workgroup.
__global__ __launch_bounds__(kSplitBlock) void k_select_bitmap(
    const uint32_t *__restrict__ key, long long n_vec, long long n_words, long long n_tiles,
    long long budget, SplitState *__restrict__ st, unsigned long long *__restrict__ hist0,
    const unsigned long long *__restrict__ hist1, const unsigned long long *__restrict__ hist_guess,
    TieCandidate *__restrict__ cand, unsigned int *__restrict__ n_cand, uint32_t *__restrict__ bitmap)
{
    bool none = budget == 0;
    bool collect = false;
    unsigned P = 0;
    if (!none) {
        // (launch 1 guessed the bucket launch 2 found: the second digit's counts are in hist_guess)
        const bool guessed = st->next_guess == st->prefix[0] + 1u;
        const Picked p1 = pick_bucket<1>(budget, guessed ? hist_guess : hist1, st);
        record_pick<1>(st, p1);
        none = !p1.ok;                 // (cannot happen)
        collect = p1.count <= kTieCandidates;
        P = p1.prefix;
    }
    if (blockIdx.x == 0)
        zero_histogram(hist0);         // (read by launch 2 only)
    constexpr int kIters = kSelTile / kSplitStride;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long long v0 = tile * (kSelTile / kVec);
        u4 keys[kIters];               // all of the tile's loads in flight at once
#pragma unroll
        for (int it = 0; it < kIters; ++it)
            keys[it] = load_keys_or_pad(key, v0 + it * kSplitBlock + threadIdx.x, n_vec);
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const long long v = v0 + it * kSplitBlock + threadIdx.x;
            const u4 k = keys[it];
            unsigned sel = 0;          // bit j: element j goes to stage 2
            if (!none) {
#pragma unroll
                for (int j = 0; j < kVec; ++j) {
                    const unsigned hi = k[j] >> 10;
                    sel |= (hi < P ? 1u : 0u) << j;
                    if (hi == P && collect && v < n_vec) {
                        // (at most kTieCandidates keys share P, so every slot exists)
                        const unsigned slot = atomicAdd(n_cand, 1u);
                        if (slot < kTieCandidates) {
                            TieCandidate tc;
                            tc.index = (unsigned long long)v * kVec + j;
                            tc.key = k[j];
                            tc.pad = 0;
                            cand[slot] = tc;
                        }
                    }
                }
            }
            store_bitmap_word(sel, v, n_words, bitmap);
        }
    }
}

// Launch 4.  Few keys share the prefix (st->collect): workgroup 0 takes, among the listed
// candidates, the r smallest in the order (low 10 bits, arena index) and clears their bits;
// the other workgroups return.  Otherwise: the histogram of the last 10 bits over all keys.
constexpr int kIndexDigit = 11;        // arena indices are cut by four digits of 11 bits (< 2^44)

__global__ __launch_bounds__(kHistBlock) void k_select_finish(
    const uint32_t *__restrict__ key, long long n_vec, long long budget,
    SplitState *__restrict__ st, unsigned long long *__restrict__ hist1,
    unsigned long long *__restrict__ hist_guess, unsigned long long *__restrict__ hist2,
    const TieCandidate *__restrict__ cand, unsigned int *__restrict__ n_cand,
    uint32_t *__restrict__ bitmap)
{
    if (blockIdx.x == gridDim.x - 1) {
        zero_histogram(hist1);         // (both read by launch 3 only)
        zero_histogram(hist_guess);
        // the next split's guess; launches 1 to 3 of this one, which read the old one, are done
        if (threadIdx.x == 0 && budget != 0)
            st->next_guess = st->prefix[0] + 1u;
    }
    if (budget == 0)
        return;
    const unsigned P = st->prefix[1];
    if (!st->collect) {
        select_histogram<2, kHistBlock>(key, n_vec, P, hist2);
        return;
    }
    if (blockIdx.x != 0)
        return;
    constexpr int B = kHistBlock;
    __shared__ unsigned int lh[kRadixBins];
    const unsigned n = *n_cand < kTieCandidates ? *n_cand : kTieCandidates;
    const unsigned long long r = st->k_rem[1];              // 1 <= r <= n
    for (int b = threadIdx.x; b < kRadixBins; b += B)
        lh[b] = 0;
    __syncthreads();
    for (unsigned c = threadIdx.x; c < n; c += B)
        atomicAdd(&lh[cand[c].key & 1023u], 1u);
    __syncthreads();
    int low;                                                // the threshold's last 10 bits
    unsigned long long below, count;
    {
        unsigned long long c1[1];
        c1[0] = lh[threadIdx.x];
        find_rank_bin<1, B>(c1, r, low, below, count);
    }
    if (low < 0)                                            // (the list is incomplete: cannot happen)
        return;
    const unsigned long long r2 = r - below;                // ties to take, 1 <= r2 <= count
    const bool all = r2 == count;
    // Ties that are not all taken: the first r2 of them in index order are.  `cut` = the r2-th
    // smallest index among the ties, found digit by digit from the top.
    unsigned long long cut = ~0ull;
    if (!all) {
        unsigned long long idx_prefix = 0, want = r2;
        for (int round = 0; round < 4; ++round) {
            const int shift = kIndexDigit * (3 - round);
            for (int b = threadIdx.x; b < kRadixBins; b += B)
                lh[b] = 0;
            __syncthreads();
            for (unsigned c = threadIdx.x; c < n; c += B) {
                const TieCandidate tc = cand[c];
                if ((tc.key & 1023u) == (unsigned)low &&
                    (round == 0 || (tc.index >> (shift + kIndexDigit)) == idx_prefix))
                    atomicAdd(&lh[(tc.index >> shift) & (kRadixBins - 1)], 1u);
            }
            __syncthreads();
            unsigned long long c2[2];
            c2[0] = lh[threadIdx.x * 2];
            c2[1] = lh[threadIdx.x * 2 + 1];
            int digit;
            unsigned long long d_below, d_count;
            find_rank_bin<2, B>(c2, want, digit, d_below, d_count);
            if (digit < 0)
                return;                                     // (cannot happen)
            idx_prefix = (idx_prefix << kIndexDigit) | (unsigned long long)digit;
            want -= d_below;
        }
        cut = idx_prefix;
    }
    for (unsigned c = threadIdx.x; c < n; c += B) {
        const TieCandidate tc = cand[c];
        const unsigned l = tc.key & 1023u;
        if (l < (unsigned)low || (l == (unsigned)low && (all || tc.index <= cut)))
            atomicAnd(&bitmap[tc.index >> 5], ~(1u << (unsigned)(tc.index & 31)));
    }
    if (threadIdx.x == 0) {
        st->threshold = (P << 10) | (unsigned)low;
        st->ties_to_take = r2;
        st->all_ties = all ? 1u : 0u;
        *n_cand = 0;
    }
}

// Launch 5 (works only when many keys share the threshold's prefix): the threshold T from the
// third histogram, then per tile how many keys equal T.
__global__ __launch_bounds__(kSplitBlock) void k_select_count_ties(
    const uint32_t *__restrict__ key, long long n_vec, long long n_tiles, long long budget,
    SplitState *__restrict__ st, const unsigned long long *__restrict__ hist2,
    unsigned int *__restrict__ tile_ties)
{
    if (budget == 0 || st->collect)    // uniform over the launch
        return;
    const Picked p2 = pick_bucket<2>(budget, hist2, st);
    record_pick<2>(st, p2);
    if (!p2.ok || p2.k_rem == p2.count)     // all keys equal to T are taken: no counts needed
        return;
    const unsigned T = p2.prefix;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long long v0 = tile * (kSelTile / kVec);
        unsigned long long n = 0;
        for (int it = 0; it < kSelTile / kSplitStride; ++it) {
            const u4 k = load_keys_or_pad(key, v0 + it * kSplitBlock + threadIdx.x, n_vec);
            n += (k.x == T) + (k.y == T) + (k.z == T) + (k.w == T);
        }
        unsigned long long total;
        block_exclusive_scan(n, &total);
        if (threadIdx.x == 0)
            tile_ties[tile] = (unsigned int)total;
    }
}

// Launch 6 (same condition): the bitmap from the full threshold T; of the keys equal to T the
// first r in index order go to stage 2.  A tile adds up the tie counts of the tiles before it.
__global__ __launch_bounds__(kSplitBlock) void k_select_write_bitmap(
    const uint32_t *__restrict__ key, long long n_vec, long long n_words, long long n_tiles,
    long long budget, const SplitState *__restrict__ st, unsigned long long *__restrict__ hist2,
    const unsigned int *__restrict__ tile_ties, uint32_t *__restrict__ bitmap)
{
    if (budget == 0 || st->collect)
        return;
    if (blockIdx.x == 0)
        zero_histogram(hist2);         // (read by launch 5 only)
    const unsigned T = st->threshold;
    const unsigned long long r = st->ties_to_take;
    const bool all = st->all_ties != 0;
    for (long long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        unsigned long long before = 0, ties = 0;
        if (!all) {
            unsigned long long mine = 0;
            for (long long t = threadIdx.x; t < tile; t += kSplitBlock)
                mine += tile_ties[t];
            block_exclusive_scan(mine, &before);
            ties = tile_ties[tile];
        }
        // 0: no tie of this tile is taken, 1: all are, 2: the boundary is inside
        int tie_mode;
        if (all)
            tie_mode = 1;
        else if (ties == 0 || before >= r)
            tie_mode = 0;
        else if (before + ties <= r)
            tie_mode = 1;
        else
            tie_mode = 2;
        unsigned long long run = before;
        const long long v0 = tile * (kSelTile / kVec);
        for (int it = 0; it < kSelTile / kSplitStride; ++it) {
            const long long v = v0 + it * kSplitBlock + threadIdx.x;
            const u4 k = load_keys_or_pad(key, v, n_vec);
            unsigned sel = 0;          // bit j: element j goes to stage 2
            unsigned long long my_before = 0;
            if (tie_mode == 2) {
                const unsigned long long n = (k.x == T) + (k.y == T) + (k.z == T) + (k.w == T);
                unsigned long long total;
                my_before = run + block_exclusive_scan(n, &total);
                run += total;
            }
#pragma unroll
            for (int j = 0; j < kVec; ++j) {
                const unsigned x = k[j];
                bool s = x < T;
                if (x == T) {
                    if (tie_mode == 1)
                        s = true;
                    else if (tie_mode == 2) {
                        s = my_before < r;
                        ++my_before;
                    }
                }
                sel |= (s ? 1u : 0u) << j;
            }
            store_bitmap_word(sel, v, n_words, bitmap);
        }
    }
}

} // namespace osp
