// C ABI of the OSP synchronization step (declared in include/osp.h):
// context, argument validation, the per-iteration order-of-calls state machine,
// workspace layout, and the kernel launches.  Host logic here never touches
// the GPU before osp_bind, so creation, validation and ordering errors can be
// exercised on a machine without one.
#include "../../include/osp.h"
#include "osp_split_kernels.hpp"
#include "osp_window_kernels.hpp"
#include "osp_pack_kernels.hpp"

#include <cstdarg>
#include <cstdio>
#include <chrono>
#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <thread>
#include <vector>

using namespace osp;

namespace {

constexpr int kDefaultChunkElems = kStride;     // one float4 per lane
constexpr size_t kAlign = 256;
constexpr int kFanoutMaxWorkers = 4;           // install: fan-out kernel up to here, sweep above
constexpr int kLgpKeepMinWorkers = 4;          // LGP keeps the stage-2 aggregate from here up

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

thread_local std::string g_create_error;

} // namespace

struct osp_ctx {
    // ---- configuration (copied) ----
    int n_workers = 0, n_tensors = 0;
    std::vector<long long> numel, offset;
    long long arena = 0, n_params = 0;
    float lr = 0.f, mu = 0.f;
    bool weighted = false;
    std::vector<float> weights;
    bool element_keys = false;
    int chunk_elems = kDefaultChunkElems;

    // ---- derived host tables ----
    std::vector<Span> spans;                   // every span, ascending addresses
    std::vector<int> span_layer;               // [n_spans]
    std::vector<int> layer_span_begin;         // [L+1]
    std::vector<int> layer_chunk_begin;        // [L+1] (host only)
    long long n_chunks = 0;
    std::vector<Segment> segments;             // fixed-order reduction tree, level 1
    std::vector<int> layer_seg_begin;          // [L+1]
    std::vector<int> big_layers;               // layers with more than kFewSegments segments
    long long n_vec = 0, n_words = 0, n_tiles = 0;

    // ---- workspace layout (byte offsets) ----
    size_t off_spans = 0, off_slayer = 0, off_lsp = 0, off_numel = 0, off_lists = 0, off_partial = 0, off_imp = 0,
           off_order = 0, off_lbase = 0, off_rscratch = 0, off_segs = 0, off_lsb = 0, off_big = 0, off_segsum = 0, off_gib = 0, off_state = 0, off_weights = 0, off_key = 0, off_stash = 0, off_pack = 0,
           off_bitmap = 0, off_hist = 0, off_cand = 0, off_tile_ties = 0, ws_bytes = 0;

    // ---- bound buffers ----
    bool bound = false;
    float *P = nullptr, *V = nullptr, *Pw = nullptr;
    long long param_stride = 0;
    char *ws = nullptr;

    // ---- iteration state machine ----
    bool have_gib = false;
    int gib_gran = OSP_GRAN_LAYER;
    bool agg1 = false, agg2 = false, single_pass = false, lgp_done = false, applied1 = false,
         applied2 = false;
    bool have_layer_importance = false;
    // replicas_synced: every replica equals the PS on every element (after an iteration that
    // installed both stages, or by the caller's word at bind).  iter_synced: that held when
    // the current iteration began, i.e. the stage-2 replica values are the PS's stale ones.
    bool replicas_synced = false, iter_synced = false, last_lgp_shared = false, last_lgp_kept = false;
    // element-granular stage 1 leaves the aggregate of the stage-2 elements in the stash;
    // valid for a stage-2 call on the same gradient arenas
    bool pack_index_valid = false;      // the pack index matches the current GIB
    int windows_fused = 0;              // bit 0: last RS window ran fused, bit 1: last ICS window
    bool stash_valid = false;
    bool keep_stage2 = true;            // LGP over a layer-granular stage 2 keeps its aggregate
    const void *stash_grads = nullptr;
    long long stash_stride = 0;
    bool stash_bf16 = false;

    // ---- stage-table lengths (layer-granular GIB) ----
    // The split runs on the device and leaves the lengths of the two stage tables in device
    // memory, where the kernels that walk the tables read them: no call waits for a split.
    // The ranking kernel also publishes the lengths, the stage-2 size and a sequence number in
    // pinned host memory; the host uses them to size grids (a hint: any grid is correct) and
    // to answer osp_n_stage2.  counts_pending: a split with sequence number split_seq has been
    // enqueued and its lengths have not been seen yet; stage_spans are the last ones seen.
    int stage_spans[2] = {0, 0};
    int tables = 0;                     // which of the two sets of stage tables is current
    bool counts_pending = false;
    unsigned split_seq = 0;
    StageCounts *pinned_counts = nullptr;      // hipHostMalloc (mapped)
    StageCounts *pinned_counts_dev = nullptr;  // the same memory as the device sees it
    long long n_stage2_host = 0;        // stage-2 elements under the current GIB (see counts_pending)

    std::string err;

    template <class T> T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
    Span *d_spans() const { return at<Span>(off_spans); }
    int *d_slayer() const { return at<int>(off_slayer); }
    int *d_lsp() const { return at<int>(off_lsp); }
    long long *d_numel() const { return at<long long>(off_numel); }
    double *d_partial(int slot) const { return at<double>(off_partial) + (size_t)slot * (size_t)n_chunks; }
    double *d_imp() const { return at<double>(off_imp); }
    int *d_order() const { return at<int>(off_order); }
    int *d_lbase() const { return at<int>(off_lbase); }
    long long *d_rscratch() const { return at<long long>(off_rscratch); }
    Segment *d_segs() const { return at<Segment>(off_segs); }
    int *d_lsb() const { return at<int>(off_lsb); }
    int *d_big() const { return at<int>(off_big); }
    double *d_segsum() const { return at<double>(off_segsum); }
    // stage tables of the current GIB; there are two sets, written alternately, so that a split
    // may be enqueued while a launch over the old tables is still to come
    Span *d_list(int stage) const
    {
        return at<Span>(off_lists) + (size_t)(tables * 2 + stage - 1) * spans.size();
    }
    uint8_t *d_gib() const { return at<uint8_t>(off_gib); }
    SplitState *d_state() const { return at<SplitState>(off_state); }
    float *d_weights() const { return at<float>(off_weights); }
    uint32_t *d_key() const { return at<uint32_t>(off_key); }
    float *d_stash() const { return at<float>(off_stash); }
    // pack index: base1 [n_chunks+1], base2 [n_chunks+1], block totals 2 x [n_pack_blocks]
    long long n_pack_blocks() const { return (n_chunks + kScanBlock - 1) / kScanBlock; }
    long long *d_pack_base(int stage) const { return at<long long>(off_pack) + (size_t)(stage - 1) * (size_t)(n_chunks + 1); }
    long long *d_pack_tot(int stage) const { return at<long long>(off_pack) + 2 * (size_t)(n_chunks + 1) + (size_t)(stage - 1) * (size_t)n_pack_blocks(); }
    uint32_t *d_bitmap() const { return at<uint32_t>(off_bitmap); }
    unsigned long long *d_hist(int pass) const
    {
        return at<unsigned long long>(off_hist) + (size_t)pass * kRadixBins;
    }
    unsigned int *d_n_cand() const { return reinterpret_cast<unsigned int *>(d_hist(kSelectHistograms)); }
    TieCandidate *d_cand() const { return at<TieCandidate>(off_cand); }
    unsigned int *d_tile_ties() const { return at<unsigned int>(off_tile_ties); }
};

namespace {

osp_status fail(osp_ctx *ctx, osp_status s, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx)
        ctx->err = buf;
    else
        g_create_error = buf;
    return s;
}

osp_status hip_fail(osp_ctx *ctx, hipError_t e, const char *what)
{
    return fail(ctx, OSP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define OSP_HIP(call)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return hip_fail(ctx, e_, #call);                                                   \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

void layout_workspace(osp_ctx *c)
{
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes);
        return at;
    };
    // The arena-sized arrays start on 4 KiB boundaries of the workspace (tensor offsets are
    // multiples of 4 KiB in the measured layouts): the 1 KiB a wavefront loads or stores is
    // then one aligned piece of them, as it is of the caller's arenas.
    auto take_arena = [&](size_t bytes) {
        o = (o + 4095) / 4096 * 4096;
        return take(bytes);
    };
    const size_t nc = (size_t)c->n_chunks, ns = c->spans.size();
    c->off_spans = take(ns * sizeof(Span));
    c->off_slayer = take(ns * sizeof(int));
    c->off_lsp = take((size_t)(c->n_tensors + 1) * sizeof(int));
    c->off_numel = take((size_t)c->n_tensors * sizeof(long long));
    c->off_segs = take(c->segments.size() * sizeof(Segment));
    c->off_lsb = take((size_t)(c->n_tensors + 1) * sizeof(int));
    c->off_big = take((size_t)(c->big_layers.size() + 1) * sizeof(int));
    c->off_lists = take(4 * ns * sizeof(Span));
    c->off_partial = take_arena(2 * nc * sizeof(double));
    c->off_segsum = take(c->segments.size() * sizeof(double));
    c->off_imp = take((size_t)c->n_tensors * sizeof(double));
    c->off_order = take((size_t)c->n_tensors * sizeof(int));
    c->off_lbase = take((size_t)c->n_tensors * sizeof(int));
    c->off_rscratch = take((size_t)c->n_tensors * sizeof(long long));
    c->off_gib = take((size_t)c->n_tensors);
    c->off_state = take(sizeof(SplitState));
    c->off_weights = take((size_t)c->n_workers * sizeof(float));
    c->off_pack = take((2 * (nc + 1) + 2 * (size_t)c->n_pack_blocks()) * sizeof(long long));
    c->off_stash = take_arena((size_t)c->arena * sizeof(float));
    if (c->element_keys) {
        c->off_key = take_arena((size_t)c->arena * sizeof(uint32_t));
        c->off_bitmap = take_arena((size_t)c->n_words * sizeof(uint32_t));
        // four histograms, then the length of the tie-candidate list (zero between splits)
        c->off_hist = take(((size_t)kSelectHistograms * kRadixBins + 1) * sizeof(unsigned long long));
        c->off_cand = take((size_t)kTieCandidates * sizeof(TieCandidate));
        c->off_tile_ties = take((size_t)c->n_tiles * sizeof(unsigned int));
    }
    c->ws_bytes = o;
}

osp_status check_grads(osp_ctx *ctx, const void *grads, int64_t stride, bool bf16 = false)
{
    if (!grads)
        return fail(ctx, OSP_ERR_INVALID_ARG, "grads is NULL");
    if (bf16 ? reinterpret_cast<uintptr_t>(grads) % 8 != 0 : !aligned16(grads))
        return fail(ctx, OSP_ERR_INVALID_ARG, "grads must be %d-byte aligned", bf16 ? 8 : 16);
    if (stride < ctx->arena || stride % 4 != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG,
                    "worker_stride %lld must be a multiple of 4 and >= arena_elems %lld",
                    (long long)stride, ctx->arena);
    return OSP_OK;
}

bool stage2_pending(const osp_ctx *c) { return c->agg1 && !c->agg2; }

// Enqueue the fill of both stage lists (bases must already be on the device).
osp_status enqueue_stage_lists(osp_ctx *ctx, hipStream_t s)
{
    const int ns = (int)ctx->spans.size();
    k_stage_lists<<<(ns + kSplitBlock - 1) / kSplitBlock, kSplitBlock, 0, s>>>(
        ns, ctx->d_spans(), ctx->d_slayer(), ctx->d_gib(), ctx->d_lsp(), ctx->d_lbase(),
        ctx->d_state(), ctx->tables, ctx->d_list(1), ctx->d_list(2));
    // (the table lengths were written straight into pinned host memory by the kernel before)
    ctx->counts_pending = true;
    return OSP_OK;
}

// Take over the lengths the last split published, if it has published them.  Never waits.
bool refresh_counts(osp_ctx *ctx)
{
    if (!ctx->counts_pending)
        return true;
    if (__atomic_load_n(&ctx->pinned_counts->seq, __ATOMIC_ACQUIRE) != ctx->split_seq)
        return false;
    const int n1 = ctx->pinned_counts->n[0], n2 = ctx->pinned_counts->n[1];
    if (n1 < 0 || n2 < 0 || (long long)n1 + n2 != (long long)ctx->spans.size())
        return false;                   // (stage_counts reports this)
    ctx->stage_spans[0] = n1;
    ctx->stage_spans[1] = n2;
    ctx->n_stage2_host = ctx->pinned_counts->n_stage2;
    ctx->counts_pending = false;
    return true;
}

// The same for the calls that need the sizes on the HOST (osp_n_stage2, the gradient
// splitter's and the packed aggregate's stride checks): waits for the split that produces
// them, first polling the sequence number (the lengths are published by the ranking kernel,
// before the table-filling work behind it), yielding the core between polls; after 2 s it
// waits for the device instead, which also surfaces a device error instead of spinning on it.
osp_status stage_counts(osp_ctx *ctx)
{
    if (!ctx->counts_pending)
        return OSP_OK;
    const auto t0 = std::chrono::steady_clock::now();
    unsigned spins = 0;
    while (__atomic_load_n(&ctx->pinned_counts->seq, __ATOMIC_ACQUIRE) != ctx->split_seq) {
        if (++spins < 4096u) {
            __builtin_ia32_pause();
            continue;
        }
        std::this_thread::yield();
        if ((spins & 255u) == 0 && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) {
            OSP_HIP(hipDeviceSynchronize());
            if (__atomic_load_n(&ctx->pinned_counts->seq, __ATOMIC_ACQUIRE) != ctx->split_seq)
                return fail(ctx, OSP_ERR_HIP, "the split did not publish its stage-table lengths");
            break;
        }
    }
    if (!refresh_counts(ctx))
        return fail(ctx, OSP_ERR_HIP, "stage tables are inconsistent (%d + %d != %lld spans)",
                    ctx->pinned_counts->n[0], ctx->pinned_counts->n[1], (long long)ctx->spans.size());
    return OSP_OK;
}

bool stream_is_capturing(hipStream_t s)
{
    if (!s)
        return false;                   // the default stream cannot be captured
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

// How to launch over the table of one stage of the current layer-granular GIB.  The kernels
// find the table's end on the device (its first cleared entry) and cope with any grid;
// grid_spans is what the grid is sized for: the exact length when the host has seen it (0: the
// stage is empty, nothing to launch), otherwise the last published length, and never less than
// an eighth of all spans, so that a stage that has grown since is still walked by many
// workgroups (a surplus workgroup costs a few per cent of a working one).  A launch that is
// being captured into a graph is sized the same way: replays may meet other lengths.
struct StageLaunch {
    const Span *table;
    unsigned grid_spans;
};

StageLaunch stage_launch(osp_ctx *ctx, int stage, hipStream_t s)
{
    StageLaunch L;
    L.table = ctx->d_list(stage);
    const unsigned total = (unsigned)ctx->spans.size();
    const bool exact = refresh_counts(ctx) && !stream_is_capturing(s);
    if (exact) {
        L.grid_spans = (unsigned)ctx->stage_spans[stage - 1];
    } else {
        int hint = ctx->counts_pending ? ctx->pinned_counts->n[stage - 1] : ctx->stage_spans[stage - 1];
        if (hint < 0)
            hint = 0;
        unsigned g = (unsigned)hint > (total + 7) / 8 ? (unsigned)hint : (total + 7) / 8;
        L.grid_spans = g > total ? total : g;
    }
    return L;
}

osp_status launch_check(osp_ctx *ctx, const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return hip_fail(ctx, e, what);
    return OSP_OK;
}

} // namespace

// How many one-wavefront workgroups of a wide kernel a compute unit should hold.  A wavefront
// of the aggregate has (N + 2) KB of loads in flight, and a compute unit takes as many
// wavefronts as their registers allow (16-20 at N = 16): over 70 MB in flight on the whole
// GPU, several times what keeps the memory busy, and measurably worse than less (the requests
// of one moment then spread over more DRAM pages).  The launch therefore asks for dynamic LDS
// that no kernel touches, sized so that only `target_bytes / bytes_per_wave` workgroups fit
// into a compute unit.  Measured on VGG-16- (N = 16) and ResNet-shaped (N = 8) steps, best
// count per compute unit and time against the unbounded launch:
//   aggregate              N = 16: 4-5 (1.31 -> 1.27 ms)   N = 8: 7 (0.136 -> 0.130 ms)
//   k_lgp_keep             N = 16: 6-7 (0.87 -> 0.85 ms)   N = 8: unbounded is best
//   element RS window      N = 16: 4 (3.92 -> 3.56 ms)     N = 8: 5-6 (0.95 -> 0.87 ms)
//   element ICS window                                     N = 8: 6-8 (0.74 -> 0.65 ms)
// which the three byte targets below reproduce.  Fewer than 4 is never asked for (3 ran 35 %
// slower than 4); above `most` (10; 8 for the RS window, whose (N + 4) KB of stores per
// wavefront count as well: bfloat16 arenas at N = 8, 0.78 -> 0.74 ms) the launch is left
// alone.  The sweep kernels (one load per lane) and k_update_from_stash lose from any bound.
constexpr size_t kLoadsInFlightPerCu = 70u * 1024u;
constexpr size_t kKeepStoresInFlightPerCu = 110u * 1024u;
constexpr size_t kWindowBytesInFlightPerCu = 62u * 1024u;

// Dynamic LDS per one-wavefront workgroup that leaves room for exactly `waves` of them in a
// compute unit (measured with a kernel that counts its resident workgroups per compute unit:
// the 160 KB do not divide evenly, 32 KB fit 4 times and 16 KB 9 times).
static unsigned lds_for_waves(size_t waves)
{
    static const unsigned lds[] = {40960, 30720, 26624, 22528, 20480, 16384, 14336};   // 4 .. 10
    return lds[waves - 4];
}

static unsigned occupancy_lds(size_t bytes_per_wave, size_t target_bytes, size_t most = 10,
                              bool always = false)
{
    size_t waves = (target_bytes + bytes_per_wave / 2) / bytes_per_wave;
    if (waves > most) {
        if (!always)
            return 0;
        waves = most;
    }
    if (waves < 4)
        waves = 4;
    return lds_for_waves(waves);
}

// Bytes one wavefront moves per pass over a group of chunks: `n_grad` gradient streams of
// `grad_bytes` per element (at most kWorkerBlock of them at once) and `n_f32` fp32 streams,
// 4 elements per lane.
static size_t wave_bytes(int n_grad, size_t grad_bytes, int n_f32)
{
    const int g = n_grad < kWorkerBlock ? n_grad : kWorkerBlock;
    return (size_t)kBlock * kVec * ((size_t)g * grad_bytes + (size_t)n_f32 * sizeof(float));
}

template <typename GT>
static void launch_aggregate(int variant, dim3 grid, dim3 block, hipStream_t s, const Span *table,
                             const AggArgs &a, int n_workers)
{
    const unsigned lds = occupancy_lds(wave_bytes(n_workers, sizeof(GT), 2), kLoadsInFlightPerCu);
    switch (variant) {
    case 0: k_aggregate_update<false, false, false, GT><<<grid, block, lds, s>>>(table, a); break;
    case 1: k_aggregate_update<false, false, true, GT><<<grid, block, lds, s>>>(table, a); break;
    case 2: k_aggregate_update<false, true, false, GT><<<grid, block, lds, s>>>(table, a); break;
    case 3: k_aggregate_update<false, true, true, GT><<<grid, block, lds, s>>>(table, a); break;
    case 5: k_aggregate_update<true, false, true, GT><<<grid, block, lds, s>>>(table, a); break;
    default: k_aggregate_update<true, true, true, GT><<<grid, block, lds, s>>>(table, a); break;
    }
}

// Shape of a sweep launch (install or LGP over a span table): blocks of about 16 MB of
// parameters, each swept replica after replica; grid = (pieces of a block, workers, blocks).
// The block has to stay in the L2s (8 x 4 MB) while the N replicas are written: 16 and 20 MB
// measure 0.5-1.5 % faster than 8 MB on every workload, 28 MB is slower on some, 32 MB on all
// (VGG-16-shaped install 1.05 -> 1.41 ms).
constexpr long long kSweepBlockBytes = 16LL << 20;
constexpr int kSweepVec = 1;            // float4 per lane in the sweep kernels (2 measured slower)
struct SweepShape {
    unsigned pieces_per_span, spans_per_block, n_blocks;
    int pieces_shift;
};

static SweepShape sweep_shape(const osp_ctx *ctx, unsigned n_spans)
{
    SweepShape sh;
    sh.pieces_per_span = (unsigned)(kSpanChunks * ctx->chunk_elems / (kPiece * kSweepVec));
    sh.pieces_shift = -1;
    for (int b = 0; b < 31; ++b)
        if (sh.pieces_per_span == (1u << b))
            sh.pieces_shift = b;
    const long long span_bytes = (long long)kSpanChunks * ctx->chunk_elems * 4;
    sh.spans_per_block = (unsigned)(kSweepBlockBytes / span_bytes > 0 ? kSweepBlockBytes / span_bytes : 1);
    sh.n_blocks = (n_spans + sh.spans_per_block - 1) / sh.spans_per_block;
    return sh;
}

template <typename GT>
static void launch_window_layer_t(const osp_ctx *ctx, const WindowLayerArgs &a, unsigned n_groups,
                                  hipStream_t s)
{
    const dim3 grid(n_groups), block(kBlock);
    const int variant = (ctx->weighted ? 2 : 0) | (ctx->element_keys ? 1 : 0);
    switch (variant) {
    case 0: k_window_layer<false, false, GT><<<grid, block, 0, s>>>(a); break;
    case 1: k_window_layer<false, true, GT><<<grid, block, 0, s>>>(a); break;
    case 2: k_window_layer<true, false, GT><<<grid, block, 0, s>>>(a); break;
    default: k_window_layer<true, true, GT><<<grid, block, 0, s>>>(a); break;
    }
}

static void launch_window_layer(const osp_ctx *ctx, const WindowLayerArgs &a, unsigned n_groups,
                                hipStream_t s, bool bf16)
{
    if (n_groups == 0)
        return;
    if (bf16)
        launch_window_layer_t<bf16_t>(ctx, a, n_groups, s);
    else
        launch_window_layer_t<float>(ctx, a, n_groups, s);
}

template <typename GT>
static void launch_rs_window_element(const osp_ctx *ctx, const RsElementArgs &a, dim3 grid, hipStream_t s)
{
    const dim3 block(kBlock);
    const int N = ctx->n_workers;
    const int cap = N <= 4 ? 4 : (N <= 8 ? 8 : 16);
    const unsigned lds = occupancy_lds(wave_bytes(N, sizeof(GT), 2), kWindowBytesInFlightPerCu, 8, true);
    if (ctx->weighted) {
        if (cap == 4) k_rs_window_element<4, true, GT><<<grid, block, lds, s>>>(a);
        else if (cap == 8) k_rs_window_element<8, true, GT><<<grid, block, lds, s>>>(a);
        else k_rs_window_element<16, true, GT><<<grid, block, lds, s>>>(a);
    } else {
        if (cap == 4) k_rs_window_element<4, false, GT><<<grid, block, lds, s>>>(a);
        else if (cap == 8) k_rs_window_element<8, false, GT><<<grid, block, lds, s>>>(a);
        else k_rs_window_element<16, false, GT><<<grid, block, lds, s>>>(a);
    }
}

template <typename GT>
static void launch_aggregate_packed(int variant, dim3 grid, dim3 block, hipStream_t s,
                                    const PackedAggArgs &a)
{
    switch (variant) {
    case 0: k_aggregate_update_packed<false, false, GT><<<grid, block, 0, s>>>(a); break;
    case 1: k_aggregate_update_packed<false, true, GT><<<grid, block, 0, s>>>(a); break;
    case 2: k_aggregate_update_packed<true, false, GT><<<grid, block, 0, s>>>(a); break;
    default: k_aggregate_update_packed<true, true, GT><<<grid, block, 0, s>>>(a); break;
    }
}

template <typename GT>
static void launch_lgp_keep(const osp_ctx *ctx, const Span *table, const LgpKeepArgs &a,
                            unsigned n_groups, hipStream_t s)
{
    const dim3 grid(n_groups), block(kBlock);
    const int variant = (ctx->weighted ? 2 : 0) | (ctx->element_keys ? 1 : 0);
    // (counted on the (N + 1) KB a wavefront stores, whatever the gradients' type)
    const unsigned lds = occupancy_lds(wave_bytes(ctx->n_workers, sizeof(float), 1), kKeepStoresInFlightPerCu);
    switch (variant) {
    case 0: k_lgp_keep<false, false, GT><<<grid, block, lds, s>>>(table, a); break;
    case 1: k_lgp_keep<false, true, GT><<<grid, block, lds, s>>>(table, a); break;
    case 2: k_lgp_keep<true, false, GT><<<grid, block, lds, s>>>(table, a); break;
    default: k_lgp_keep<true, true, GT><<<grid, block, lds, s>>>(table, a); break;
    }
}

// The launches of one element-granular selection: `budget` smallest keys in the order
// (key, index) -> bitmap.  Everything but `key` and `bitmap` is scratch: the split state,
// hist = (4 * kRadixBins + 1) counters of 8 bytes (four histograms, then the length of the
// candidate list; all zero on entry and left zero), the candidate list, the per-tile tie
// counts.
struct SelectScratch {
    SplitState *state;
    unsigned long long *hist;
    TieCandidate *cand;
    unsigned int *tile_ties;
};

static void enqueue_element_select(const uint32_t *key, long long n_vec, long long n_words,
                                   long long n_tiles, long long budget, const SelectScratch &w,
                                   uint32_t *bitmap, hipStream_t s)
{
    unsigned long long *h0 = w.hist, *h1 = w.hist + kRadixBins, *h2 = w.hist + 2 * kRadixBins;
    unsigned long long *hg = w.hist + 3 * kRadixBins;      // the second digit under the guessed first
    unsigned int *n_cand = reinterpret_cast<unsigned int *>(w.hist + kSelectHistograms * kRadixBins);
    // histogram passes: few, large workgroups (see select_histogram)
    const long long per_wg = (long long)kHistBlock * kHistVecPerThread;
    long long want = (n_vec + per_wg - 1) / per_wg;
    const unsigned hist_grid = (unsigned)(want < kHistMaxGrid ? (want < 1 ? 1 : want) : kHistMaxGrid);
    // the tile passes walk their tiles in rounds of the grid: their prologue is paid per workgroup
    const unsigned tgrid = (unsigned)(n_tiles < 8192 ? (n_tiles < 1 ? 1 : n_tiles) : 8192);
    k_select_histogram0<<<hist_grid, kHistBlock, 0, s>>>(key, n_vec, budget, w.state, h0, hg);
    k_select_histogram1<<<hist_grid, kHistBlock, 0, s>>>(key, n_vec, budget, w.state, h0, h1);
    k_select_bitmap<<<tgrid, kSplitBlock, 0, s>>>(key, n_vec, n_words, n_tiles, budget, w.state, h0, h1,
                                                 hg, w.cand, n_cand, bitmap);
    k_select_finish<<<hist_grid, kHistBlock, 0, s>>>(key, n_vec, budget, w.state, h1, hg, h2, w.cand,
                                                    n_cand, bitmap);
    // (the last two return at once unless many keys share the threshold's upper 22 bits:
    // small grids, so that returning costs little)
    const unsigned fgrid = tgrid < 1024 ? tgrid : 1024;
    k_select_count_ties<<<fgrid, kSplitBlock, 0, s>>>(key, n_vec, n_tiles, budget, w.state, h2, w.tile_ties);
    k_select_write_bitmap<<<fgrid, kSplitBlock, 0, s>>>(key, n_vec, n_words, n_tiles, budget, w.state, h2,
                                                       w.tile_ties, bitmap);
}

// ---------------------------------------------------------------------------
// Scratch of osp_split_element_static: one array per GPU, held until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress;
// the address kernels are given is looked up once per device.
// ---------------------------------------------------------------------------
constexpr long long kStaticMaxElems = 1LL << 28;
constexpr size_t kStaticOffHist = 256;                                   // SplitState first
constexpr size_t kStaticOffCand = kStaticOffHist + 65792;                // (4 * 2048 + 1) * 8, rounded up
constexpr size_t kStaticOffTies = kStaticOffCand + (size_t)kTieCandidates * sizeof(TieCandidate);
constexpr size_t kStaticTiles = (size_t)(kStaticMaxElems / kSelTile);
constexpr size_t kStaticScratchBytes = kStaticOffTies + kStaticTiles * sizeof(unsigned int);
static_assert(sizeof(SplitState) <= kStaticOffHist, "state fits in front of the histograms");
static_assert(((size_t)kSelectHistograms * kRadixBins + 1) * sizeof(unsigned long long) <= kStaticOffCand - kStaticOffHist,
              "histograms fit");
static_assert(kStaticOffCand % 256 == 0 && kStaticOffTies % 256 == 0,
              "every part starts on a 256-byte boundary");

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static unsigned char *g_scratch_ptr[kMaxDevices];      // device address of `scratch`, per device

// Device address of this process's scratch array on the current device (looked up on the
// first call per device; a race between two first calls stores the same value twice).
static hipError_t static_scratch(unsigned char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= kMaxDevices)
        return hipErrorInvalidDevice;
    unsigned char *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return e;
        if (!p)
            return hipErrorInvalidSymbol;
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return hipSuccess;
}

extern "C" {

osp_status osp_create(const osp_config *cfg, osp_ctx **out)
{
    if (out)
        *out = nullptr;
    osp_ctx *ctx = nullptr;                    // fail() records into the thread-local slot
    if (!cfg || !out)
        return fail(ctx, OSP_ERR_INVALID_ARG, "cfg and out must not be NULL");
    if (cfg->n_workers < 1)
        return fail(ctx, OSP_ERR_INVALID_ARG, "n_workers must be >= 1 (got %d)", cfg->n_workers);
    if (cfg->n_tensors < 1)
        return fail(ctx, OSP_ERR_INVALID_ARG, "n_tensors must be >= 1 (got %d)", cfg->n_tensors);
    if (!cfg->numel || !cfg->offset)
        return fail(ctx, OSP_ERR_INVALID_ARG, "numel and offset must not be NULL");
    if (cfg->arena_elems <= 0 || cfg->arena_elems % 4 != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG, "arena_elems must be a positive multiple of 4");
    if (!(cfg->lr == cfg->lr) || !(cfg->momentum >= 0.f && cfg->momentum < 1.f))
        return fail(ctx, OSP_ERR_INVALID_ARG, "lr must be a number and 0 <= momentum < 1");
    int chunk = cfg->chunk_elems == 0 ? kDefaultChunkElems : cfg->chunk_elems;
    if (chunk < kStride || chunk % kStride != 0 || chunk > (1 << 24))
        return fail(ctx, OSP_ERR_INVALID_ARG, "chunk_elems must be a multiple of %d in [%d, %d]",
                    kStride, kStride, 1 << 24);
    long long prev_end = 0, total = 0;
    for (int l = 0; l < cfg->n_tensors; ++l) {
        const long long n = cfg->numel[l], o = cfg->offset[l];
        if (n <= 0)
            return fail(ctx, OSP_ERR_INVALID_ARG, "numel[%d] must be > 0", l);
        if (o < prev_end || o % 4 != 0)
            return fail(ctx, OSP_ERR_INVALID_ARG,
                        "offset[%d]=%lld must be a multiple of 4 and not overlap tensor %d", l, o,
                        l - 1);
        if (n > cfg->arena_elems - o)
            return fail(ctx, OSP_ERR_INVALID_ARG, "tensor %d ends past arena_elems", l);
        prev_end = o + n;
        total += n;
    }
    osp_ctx *c = new (std::nothrow) osp_ctx;
    if (!c)
        return fail(ctx, OSP_ERR_NOMEM, "out of host memory");
    try {
        c->n_workers = cfg->n_workers;
        c->n_tensors = cfg->n_tensors;
        c->numel.assign(cfg->numel, cfg->numel + cfg->n_tensors);
        c->offset.assign(cfg->offset, cfg->offset + cfg->n_tensors);
        c->arena = cfg->arena_elems;
        c->n_params = total;
        c->lr = cfg->lr;
        c->mu = cfg->momentum;
        c->weighted = cfg->worker_weight != nullptr;
        if (c->weighted)
            c->weights.assign(cfg->worker_weight, cfg->worker_weight + cfg->n_workers);
        else
            c->weights.assign((size_t)cfg->n_workers, 1.0f / (float)cfg->n_workers);
        c->element_keys = cfg->element_keys != 0;
        c->chunk_elems = chunk;
        for (int l = 0; l < c->n_tensors; ++l) {
            c->layer_chunk_begin.push_back((int)c->n_chunks);
            c->layer_span_begin.push_back((int)c->spans.size());
            const long long per_span = (long long)chunk * kSpanChunks;
            for (long long b = 0; b < c->numel[l]; b += per_span) {
                Span sp;
                sp.start = c->offset[l] + b;
                sp.n_elems = (int)(c->numel[l] - b < per_span ? c->numel[l] - b : per_span);
                sp.chunk_base = (int)c->n_chunks;
                c->spans.push_back(sp);
                c->span_layer.push_back(l);
                c->n_chunks += (sp.n_elems + chunk - 1) / chunk;
                if (c->n_chunks > 0x7FFFFF00LL || c->spans.size() > (size_t)(0x7FFFFF00 / kSpanChunks)) {
                    delete c;
                    return fail(ctx, OSP_ERR_UNSUPPORTED, "more than 2^31 chunks; raise chunk_elems");
                }
            }
        }
        c->layer_chunk_begin.push_back((int)c->n_chunks);
        c->layer_span_begin.push_back((int)c->spans.size());
        for (int l = 0; l < c->n_tensors; ++l) {
            c->layer_seg_begin.push_back((int)c->segments.size());
            for (int b = c->layer_chunk_begin[l]; b < c->layer_chunk_begin[l + 1]; b += kSegChunks) {
                Segment sg;
                sg.begin = b;
                sg.end = b + kSegChunks < c->layer_chunk_begin[l + 1] ? b + kSegChunks
                                                                      : c->layer_chunk_begin[l + 1];
                sg.layer = l;
                sg.pad = 0;
                c->segments.push_back(sg);
            }
        }
        c->layer_seg_begin.push_back((int)c->segments.size());
        for (int l = 0; l < c->n_tensors; ++l)
            if (c->layer_seg_begin[l + 1] - c->layer_seg_begin[l] > kFewSegments)
                c->big_layers.push_back(l);
    } catch (const std::bad_alloc &) {
        delete c;
        return fail(ctx, OSP_ERR_NOMEM, "out of host memory");
    }
    c->n_vec = c->arena / 4;
    c->n_words = (c->arena + 31) / 32;
    c->n_tiles = (c->arena + kSelTile - 1) / kSelTile;
    layout_workspace(c);
    *out = c;
    return OSP_OK;
}

void osp_destroy(osp_ctx *ctx)
{
    if (!ctx)
        return;
    if (ctx->pinned_counts)
        (void)hipHostFree(ctx->pinned_counts);
    delete ctx;
}

size_t osp_workspace_bytes(const osp_ctx *ctx) { return ctx ? ctx->ws_bytes : 0; }

int32_t osp_chunk_elems(const osp_ctx *ctx) { return ctx ? ctx->chunk_elems : 0; }

int32_t osp_lgp_read_shared(const osp_ctx *ctx) { return ctx && ctx->last_lgp_shared ? 1 : 0; }

int32_t osp_windows_fused(const osp_ctx *ctx) { return ctx ? ctx->windows_fused : 0; }

int32_t osp_lgp_kept_aggregate(const osp_ctx *ctx) { return ctx && ctx->last_lgp_kept ? 1 : 0; }

osp_status osp_set_keep_stage2_aggregate(osp_ctx *ctx, int32_t on)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE, "the option cannot change between the two stages");
    ctx->keep_stage2 = on != 0;
    return OSP_OK;
}

osp_status osp_drop_kept_aggregate(osp_ctx *ctx)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    ctx->stash_valid = false;
    return OSP_OK;
}

int64_t osp_n_chunks(const osp_ctx *ctx) { return ctx ? (int64_t)ctx->n_chunks : 0; }

const char *osp_last_error(const osp_ctx *ctx)
{
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

osp_status osp_set_hyper(osp_ctx *ctx, float lr, float momentum)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (!(lr == lr) || !(momentum >= 0.f && momentum < 1.f))
        return fail(ctx, OSP_ERR_INVALID_ARG, "lr must be a number and 0 <= momentum < 1");
    if (stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE, "hyper-parameters cannot change between the two stages");
    ctx->lr = lr;
    ctx->mu = momentum;
    return OSP_OK;
}

osp_status osp_bind(osp_ctx *ctx, const osp_buffers *buf, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (!buf)
        return fail(ctx, OSP_ERR_INVALID_ARG, "buffers is NULL");
    if (!buf->ps_param || !buf->ps_momentum || !buf->worker_param || !buf->workspace)
        return fail(ctx, OSP_ERR_INVALID_ARG, "ps_param, ps_momentum, worker_param and workspace must not be NULL");
    if (!aligned16(buf->ps_param) || !aligned16(buf->ps_momentum) || !aligned16(buf->worker_param))
        return fail(ctx, OSP_ERR_INVALID_ARG, "parameter buffers must be 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(buf->workspace) % kAlign != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (buf->worker_param_stride < ctx->arena || buf->worker_param_stride % 4 != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG,
                    "worker_param_stride must be a multiple of 4 and >= arena_elems");
    if (buf->workspace_bytes < ctx->ws_bytes)
        return fail(ctx, OSP_ERR_INVALID_ARG, "workspace has %zu bytes, %zu needed",
                    buf->workspace_bytes, ctx->ws_bytes);
    if (stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE, "cannot rebind while a stage 2 is pending");
    hipStream_t s = (hipStream_t)stream;
    ctx->bound = false;
    if (!ctx->pinned_counts) {
        OSP_HIP(hipHostMalloc((void **)&ctx->pinned_counts, sizeof(StageCounts), hipHostMallocMapped));
        OSP_HIP(hipHostGetDevicePointer((void **)&ctx->pinned_counts_dev, ctx->pinned_counts, 0));
        ctx->pinned_counts->n[0] = ctx->pinned_counts->n[1] = 0;
        ctx->pinned_counts->n_stage2 = 0;
        ctx->pinned_counts->seq = 0;
        ctx->split_seq = 0;
    }
    ctx->counts_pending = false;
    ctx->tables = 0;
    ctx->ws = (char *)buf->workspace;
    OSP_HIP(hipMemcpyAsync(ctx->d_spans(), ctx->spans.data(), ctx->spans.size() * sizeof(Span),
                           hipMemcpyHostToDevice, s));
    OSP_HIP(hipMemcpyAsync(ctx->d_slayer(), ctx->span_layer.data(),
                           ctx->span_layer.size() * sizeof(int), hipMemcpyHostToDevice, s));
    OSP_HIP(hipMemcpyAsync(ctx->d_lsp(), ctx->layer_span_begin.data(),
                           ctx->layer_span_begin.size() * sizeof(int), hipMemcpyHostToDevice, s));
    OSP_HIP(hipMemcpyAsync(ctx->d_segs(), ctx->segments.data(), ctx->segments.size() * sizeof(Segment),
                           hipMemcpyHostToDevice, s));
    OSP_HIP(hipMemcpyAsync(ctx->d_lsb(), ctx->layer_seg_begin.data(),
                           ctx->layer_seg_begin.size() * sizeof(int), hipMemcpyHostToDevice, s));
    if (!ctx->big_layers.empty())
        OSP_HIP(hipMemcpyAsync(ctx->d_big(), ctx->big_layers.data(), ctx->big_layers.size() * sizeof(int),
                               hipMemcpyHostToDevice, s));
    OSP_HIP(hipMemcpyAsync(ctx->d_numel(), ctx->numel.data(), ctx->numel.size() * sizeof(long long),
                           hipMemcpyHostToDevice, s));
    OSP_HIP(hipMemcpyAsync(ctx->d_weights(), ctx->weights.data(), ctx->weights.size() * sizeof(float),
                           hipMemcpyHostToDevice, s));
    // partials, importances, ranking, GIB, split state start at zero
    const size_t zero_bytes = ctx->off_weights - ctx->off_partial;
    k_fill_u32<<<256, kSplitBlock, 0, s>>>(ctx->at<uint32_t>(ctx->off_partial),
                                           (long long)(zero_bytes / 4), 0u);
    if (ctx->element_keys) {
        // padding keys stay 0xFFFFFFFF for good: above every real key, never selected
        k_fill_u32<<<1024, kSplitBlock, 0, s>>>(ctx->d_key(), ctx->arena, 0xFFFFFFFFu);
        k_fill_u32<<<256, kSplitBlock, 0, s>>>(ctx->d_bitmap(), ctx->n_words, 0xFFFFFFFFu);
        // histograms and the candidate count start at zero; every split leaves them so
        k_fill_u32<<<24, kSplitBlock, 0, s>>>(reinterpret_cast<uint32_t *>(ctx->d_hist(0)),
                                             (long long)(kSelectHistograms * kRadixBins + 1) * 2, 0u);
    }
    osp_status st = launch_check(ctx, "bind fill kernels");
    if (st != OSP_OK)
        return st;
    OSP_HIP(hipStreamSynchronize(s));
    ctx->P = buf->ps_param;
    ctx->V = buf->ps_momentum;
    ctx->Pw = buf->worker_param;
    ctx->param_stride = buf->worker_param_stride;
    ctx->bound = true;
    ctx->replicas_synced = buf->replicas_in_sync != 0;
    ctx->iter_synced = false;
    ctx->stash_valid = false;
    ctx->last_lgp_kept = false;
    ctx->pack_index_valid = false;
    ctx->windows_fused = 0;
    ctx->have_gib = false;
    ctx->agg1 = ctx->agg2 = ctx->single_pass = ctx->lgp_done = ctx->applied1 = ctx->applied2 = false;
    ctx->have_layer_importance = false;
    return OSP_OK;
}

osp_status osp_set_gib(osp_ctx *ctx, int granularity, const void *gib_host, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (granularity != OSP_GRAN_LAYER && granularity != OSP_GRAN_ELEMENT)
        return fail(ctx, OSP_ERR_INVALID_ARG, "unknown granularity %d", granularity);
    if (!gib_host)
        return fail(ctx, OSP_ERR_INVALID_ARG, "gib_host is NULL");
    if (granularity == OSP_GRAN_ELEMENT && !ctx->element_keys)
        return fail(ctx, OSP_ERR_UNSUPPORTED, "element granularity needs cfg.element_keys");
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE, "the GIB cannot change while a stage 2 is pending");
    hipStream_t s = (hipStream_t)stream;
    long long n2 = 0;
    if (granularity == OSP_GRAN_LAYER) {
        const uint8_t *g = (const uint8_t *)gib_host;
        std::vector<uint8_t> norm((size_t)ctx->n_tensors);
        for (int l = 0; l < ctx->n_tensors; ++l) {
            norm[l] = g[l] ? 1 : 0;
            if (!g[l])
                n2 += ctx->numel[l];
        }
        OSP_HIP(hipMemcpyAsync(ctx->d_gib(), norm.data(), norm.size(), hipMemcpyHostToDevice, s));
        OSP_HIP(hipMemcpyAsync(&ctx->d_state()->n_stage2, &n2, sizeof n2, hipMemcpyHostToDevice, s));
        ctx->tables ^= 1;               // the new GIB's tables go into the other set
        k_stage_bases<<<1, 64, 0, s>>>(ctx->n_tensors, ctx->d_gib(), ctx->d_lsp(), ctx->d_lbase(),
                                       ctx->d_state(), ctx->pinned_counts_dev, ++ctx->split_seq,
                                       ctx->tables);
        osp_status st = enqueue_stage_lists(ctx, s);
        if (st != OSP_OK)
            return st;
        st = launch_check(ctx, "stage list kernels");
        if (st != OSP_OK)
            return st;
        OSP_HIP(hipStreamSynchronize(s));
        st = stage_counts(ctx);         // (published by now)
        if (st != OSP_OK)
            return st;
    } else {
        const uint32_t *g = (const uint32_t *)gib_host;
        std::vector<uint32_t> bits;
        try {
            bits.assign((size_t)ctx->n_words, 0xFFFFFFFFu);
        } catch (const std::bad_alloc &) {
            return fail(ctx, OSP_ERR_NOMEM, "out of host memory");
        }
        for (int l = 0; l < ctx->n_tensors; ++l)       // padding bits stay 1
            for (long long k = ctx->offset[l]; k < ctx->offset[l] + ctx->numel[l]; ++k)
                if (!((g[k >> 5] >> (k & 31)) & 1u)) {
                    bits[(size_t)(k >> 5)] &= ~(1u << (k & 31));
                    ++n2;
                }
        OSP_HIP(hipMemcpyAsync(ctx->d_bitmap(), bits.data(), bits.size() * sizeof(uint32_t),
                               hipMemcpyHostToDevice, s));
        OSP_HIP(hipMemcpyAsync(&ctx->d_state()->n_stage2, &n2, sizeof n2, hipMemcpyHostToDevice, s));
        OSP_HIP(hipStreamSynchronize(s));
        ctx->counts_pending = false;
        ctx->n_stage2_host = n2;
    }
    ctx->have_gib = true;
    ctx->pack_index_valid = false;
    ctx->gib_gran = granularity;
    ctx->agg1 = ctx->agg2 = ctx->single_pass = ctx->lgp_done = ctx->applied1 = ctx->applied2 = false;
    return OSP_OK;
}

osp_status osp_get_gib(osp_ctx *ctx, uint8_t *layer_gib, uint32_t *elem_bitmap, int64_t *n_stage2,
                       void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (!ctx->bound || !ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "no GIB yet (osp_set_gib or osp_split first)");
    hipStream_t s = (hipStream_t)stream;
    long long n2 = 0;
    if (layer_gib && ctx->gib_gran == OSP_GRAN_LAYER)
        OSP_HIP(hipMemcpyAsync(layer_gib, ctx->d_gib(), (size_t)ctx->n_tensors, hipMemcpyDeviceToHost, s));
    if (elem_bitmap && ctx->gib_gran == OSP_GRAN_ELEMENT)
        OSP_HIP(hipMemcpyAsync(elem_bitmap, ctx->d_bitmap(), (size_t)ctx->n_words * sizeof(uint32_t),
                               hipMemcpyDeviceToHost, s));
    OSP_HIP(hipMemcpyAsync(&n2, &ctx->d_state()->n_stage2, sizeof n2, hipMemcpyDeviceToHost, s));
    OSP_HIP(hipStreamSynchronize(s));
    if (n_stage2)
        *n_stage2 = n2;
    return OSP_OK;
}

osp_status osp_read_n_stage2_async(osp_ctx *ctx, int64_t *out_host, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (!out_host)
        return fail(ctx, OSP_ERR_INVALID_ARG, "out_host is NULL");
    if (!ctx->bound || !ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "no GIB yet (osp_set_gib or osp_split first)");
    // Pinned (mapped) host memory is written by a one-lane kernel: a few microseconds of stream
    // time and a node that can be captured into a graph, where a copy of 8 bytes through the
    // copy path costs several times that.  Any other host memory takes the copy.
    void *dev = nullptr;
    if (hipHostGetDevicePointer(&dev, out_host, 0) == hipSuccess && dev) {
        k_publish_i64<<<1, 1, 0, (hipStream_t)stream>>>(&ctx->d_state()->n_stage2,
                                                        static_cast<long long *>(dev));
        return launch_check(ctx, "k_publish_i64");
    }
    (void)hipGetLastError();
    OSP_HIP(hipMemcpyAsync(out_host, &ctx->d_state()->n_stage2, sizeof(int64_t),
                           hipMemcpyDeviceToHost, (hipStream_t)stream));
    return OSP_OK;
}

osp_status osp_set_stage2_log(osp_ctx *ctx, int64_t *log, int64_t capacity, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (log && capacity < 1)
        return fail(ctx, OSP_ERR_INVALID_ARG, "capacity must be >= 1 (got %lld)", (long long)capacity);
    if (reinterpret_cast<uintptr_t>(log) % 8 != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG, "log must be 8-byte aligned");
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    k_set_stage2_log<<<1, 1, 0, (hipStream_t)stream>>>(ctx->d_state(), reinterpret_cast<long long *>(log),
                                                      log ? (long long)capacity : 1);
    return launch_check(ctx, "k_set_stage2_log");
}

osp_status osp_n_stage2(osp_ctx *ctx, int64_t *n_stage2)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (!n_stage2)
        return fail(ctx, OSP_ERR_INVALID_ARG, "n_stage2 is NULL");
    if (!ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "there is no GIB");
    osp_status st = stage_counts(ctx);
    if (st != OSP_OK)
        return st;
    *n_stage2 = ctx->n_stage2_host;
    return OSP_OK;
}

static osp_status aggregate_update(osp_ctx *ctx, int stage, const void *grads, int64_t worker_stride,
                                   void *stream, bool bf16)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (stage < 0 || stage > 2)
        return fail(ctx, OSP_ERR_INVALID_ARG, "stage must be 0, 1 or 2 (got %d)", stage);
    osp_status st = check_grads(ctx, grads, worker_stride, bf16);
    if (st != OSP_OK)
        return st;
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (stage != 0 && !ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "a staged call needs a GIB (osp_set_gib or osp_split)");
    if (stage != 2 && stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE,
                    "stage 2 of the previous iteration is still pending (ICS must complete first)");
    if (stage == 2 && !stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE, "stage 2 needs this iteration's stage 1 first");

    const bool masked = stage != 0 && ctx->gib_gran == OSP_GRAN_ELEMENT;
    const bool listed = stage != 0 && ctx->gib_gran == OSP_GRAN_LAYER;
    hipStream_t s = (hipStream_t)stream;
    unsigned n_groups = (unsigned)ctx->spans.size() * kSpanChunks;
    AggArgs a;
    const Span *table = ctx->d_spans();
    a.cap_spans = (unsigned)ctx->spans.size();
    if (listed) {
        const StageLaunch L = stage_launch(ctx, stage, s);
        table = L.table;
        n_groups = L.grid_spans * kSpanChunks;
    }
    a.chunk_elems = ctx->chunk_elems;
    a.bitmap = ctx->element_keys ? ctx->d_bitmap() : nullptr;
    a.P = ctx->P;
    a.V = ctx->V;
    a.grads = grads;
    a.worker_stride = worker_stride;
    a.weights = ctx->d_weights();
    a.partial = ctx->d_partial(stage == 2 ? 1 : 0);
    a.key = ctx->element_keys ? ctx->d_key() : nullptr;
    a.partial_other = nullptr;
    a.stash = nullptr;
    if (masked && stage == 1) {
        a.stash = ctx->d_stash();
        a.partial_other = ctx->d_partial(1);
    }
    const bool from_stash = (masked || listed) && stage == 2 && ctx->stash_valid &&
                            ctx->stash_grads == grads &&
                            ctx->stash_stride == (long long)worker_stride && ctx->stash_bf16 == bf16;
    a.n_workers = ctx->n_workers;
    a.stage = stage;
    a.inv_n = 1.0f / (float)ctx->n_workers;
    a.lr = ctx->lr;
    a.mu = ctx->mu;
    const dim3 grid(n_groups), block(kBlock);
    const int variant = (masked ? 4 : 0) | (ctx->weighted ? 2 : 0) | (ctx->element_keys ? 1 : 0);
    if (from_stash) {
        StashArgs sa;
        sa.cap_spans = a.cap_spans;
        sa.chunk_elems = a.chunk_elems;
        sa.bitmap = a.bitmap;
        sa.P = ctx->P;
        sa.V = ctx->V;
        sa.stash = ctx->d_stash();
        sa.lr = ctx->lr;
        sa.mu = ctx->mu;
        if (masked)
            k_update_from_stash<true><<<grid, block, 0, s>>>(table, sa);
        else if (n_groups > 0)
            k_update_from_stash<false><<<grid, block, 0, s>>>(table, sa);
    } else if (n_groups > 0) {        // an empty stage launches nothing
        if (variant == 4 || variant == 6)
            return fail(ctx, OSP_ERR_UNSUPPORTED, "element-granular GIB without element_keys");
        if (bf16)
            launch_aggregate<bf16_t>(variant, grid, block, s, table, a, ctx->n_workers);
        else
            launch_aggregate<float>(variant, grid, block, s, table, a, ctx->n_workers);
    }
    st = launch_check(ctx, "k_aggregate_update");
    if (st != OSP_OK)
        return st;
    if (stage != 2) {                   // a new iteration begins: the PS moves away from the replicas
        ctx->iter_synced = ctx->replicas_synced;
        ctx->replicas_synced = false;
        ctx->stash_valid = masked && stage == 1;
        ctx->stash_grads = grads;
        ctx->stash_stride = (long long)worker_stride;
        ctx->stash_bf16 = bf16;
    }
    if (stage == 1) {
        ctx->agg1 = true;
        ctx->agg2 = ctx->single_pass = ctx->lgp_done = ctx->applied1 = ctx->applied2 = false;
    } else if (stage == 2) {
        ctx->agg2 = true;
    } else {
        ctx->agg1 = ctx->agg2 = ctx->single_pass = true;
        ctx->lgp_done = ctx->applied1 = ctx->applied2 = false;
    }
    return OSP_OK;
}

osp_status osp_ps_aggregate_update(osp_ctx *ctx, int stage, const float *grads,
                                   int64_t worker_stride, void *stream)
{
    return aggregate_update(ctx, stage, grads, worker_stride, stream, false);
}

osp_status osp_ps_aggregate_update_bf16(osp_ctx *ctx, int stage, const uint16_t *grads,
                                        int64_t worker_stride, void *stream)
{
    return aggregate_update(ctx, stage, grads, worker_stride, stream, true);
}

static osp_status lgp_correct(osp_ctx *ctx, const void *grads, int64_t worker_stride, void *stream,
                              bool bf16)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    osp_status st = check_grads(ctx, grads, worker_stride, bf16);
    if (st != OSP_OK)
        return st;
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (!ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "LGP needs a GIB");
    if (!ctx->agg1 || ctx->single_pass)
        return fail(ctx, OSP_ERR_BAD_STATE, "LGP belongs after this iteration's stage 1 aggregate");
    if (ctx->lgp_done)
        return fail(ctx, OSP_ERR_BAD_STATE, "LGP already applied in this iteration");
    if (ctx->applied2)
        return fail(ctx, OSP_ERR_BAD_STATE, "LGP after the stage-2 correction would undo it");
    const bool masked = ctx->gib_gran == OSP_GRAN_ELEMENT;
    hipStream_t s = (hipStream_t)stream;
    unsigned n_spans = (unsigned)ctx->spans.size();
    const Span *table = ctx->d_spans();
    const unsigned cap_spans = (unsigned)ctx->spans.size();
    if (!masked) {
        const StageLaunch L = stage_launch(ctx, 2, s);
        table = L.table;
        n_spans = L.grid_spans;
    }
    const uint32_t *bitmap = ctx->element_keys ? ctx->d_bitmap() : nullptr;
    // The replicas' stage-2 values are still the PS's (stale) ones: read them once from the PS.
    // Needs the PS's stage-2 values untouched (stage 2 not aggregated yet) and, for an
    // element-granular GIB, this iteration's stage 1 already installed.
    const bool shared_read = ctx->iter_synced && !ctx->agg2 && (!masked || ctx->applied1);
    ctx->last_lgp_shared = shared_read;
    // Layer-granular stage 2, several workers: the pass that has every worker's stage-2
    // gradients in hand also leaves their aggregate for the stage-2 call (one read of the N
    // arenas' stage-2 part per iteration instead of two).
    const bool keep = shared_read && !masked && ctx->keep_stage2 && ctx->n_workers >= kLgpKeepMinWorkers;
    ctx->last_lgp_kept = keep;
    if (keep) {
        LgpKeepArgs a;
        a.cap_spans = cap_spans;
        a.chunk_elems = ctx->chunk_elems;
        a.P = ctx->P;
        a.Pw = ctx->Pw;
        a.param_stride = ctx->param_stride;
        a.grads = grads;
        a.worker_stride = worker_stride;
        a.weights = ctx->d_weights();
        a.partial = ctx->d_partial(1);
        a.key = ctx->element_keys ? ctx->d_key() : nullptr;
        a.stash = ctx->d_stash();
        a.n_workers = ctx->n_workers;
        a.inv_n = 1.0f / (float)ctx->n_workers;
        a.lr = ctx->lr;
        const unsigned n_groups = n_spans * kSpanChunks;
        if (n_groups > 0) {
            if (bf16)
                launch_lgp_keep<bf16_t>(ctx, table, a, n_groups, s);
            else
                launch_lgp_keep<float>(ctx, table, a, n_groups, s);
        }
        ctx->stash_valid = true;
        ctx->stash_grads = grads;
        ctx->stash_stride = (long long)worker_stride;
        ctx->stash_bf16 = bf16;
    } else if (shared_read) {
        LgpSweepArgs a;
        a.cap_spans = cap_spans;
        a.bitmap = bitmap;
        a.P = ctx->P;
        a.Pw = ctx->Pw;
        a.param_stride = ctx->param_stride;
        a.grads = grads;
        a.worker_stride = worker_stride;
        const SweepShape sh = sweep_shape(ctx, n_spans);
        a.pieces_per_span = sh.pieces_per_span;
        a.pieces_shift = sh.pieces_shift;
        a.spans_per_block = sh.spans_per_block;
        a.lr = ctx->lr;
        if (sh.n_blocks > 65535u || ctx->n_workers > 65535)
            return fail(ctx, OSP_ERR_UNSUPPORTED, "LGP launch of %u blocks x %d workers exceeds the grid limit",
                        sh.n_blocks, ctx->n_workers);
        const dim3 grid(sh.spans_per_block * sh.pieces_per_span, (unsigned)ctx->n_workers, sh.n_blocks);
        const dim3 block(kApplyBlock);
        if (sh.n_blocks > 0) {
            if (bf16) {
                if (masked)
                    k_lgp_sweep<true, bf16_t, kSweepVec><<<grid, block, 0, s>>>(table, a);
                else
                    k_lgp_sweep<false, bf16_t, kSweepVec><<<grid, block, 0, s>>>(table, a);
            } else {
                if (masked)
                    k_lgp_sweep<true, float, kSweepVec><<<grid, block, 0, s>>>(table, a);
                else
                    k_lgp_sweep<false, float, kSweepVec><<<grid, block, 0, s>>>(table, a);
            }
        }
    } else {
        LgpArgs a;
        a.cap_spans = cap_spans;
        a.chunk_elems = ctx->chunk_elems;
        a.bitmap = bitmap;
        a.Pw = ctx->Pw;
        a.param_stride = ctx->param_stride;
        a.grads = grads;
        a.worker_stride = worker_stride;
        a.lr = ctx->lr;
        const unsigned n_groups = n_spans * kSpanChunks;
        if (n_groups > 0) {
            // grid.y is limited to 65535: sweep the workers in slabs of that size
            for (int w0 = 0; w0 < ctx->n_workers; w0 += 65535) {
                const int nw = ctx->n_workers - w0 < 65535 ? ctx->n_workers - w0 : 65535;
                LgpArgs b = a;
                b.Pw = a.Pw + (long long)w0 * a.param_stride;
                b.grads = static_cast<const char *>(a.grads) +
                          (long long)w0 * a.worker_stride * (bf16 ? 2 : 4);
                const dim3 grid(n_groups, (unsigned)nw), block(kBlock);
                if (bf16) {
                    if (masked)
                        k_lgp_correct<true, bf16_t><<<grid, block, 0, s>>>(table, b);
                    else
                        k_lgp_correct<false, bf16_t><<<grid, block, 0, s>>>(table, b);
                } else {
                    if (masked)
                        k_lgp_correct<true><<<grid, block, 0, s>>>(table, b);
                    else
                        k_lgp_correct<false><<<grid, block, 0, s>>>(table, b);
                }
            }
        }
    }
    st = launch_check(ctx, "k_lgp_correct");
    if (st != OSP_OK)
        return st;
    ctx->lgp_done = true;
    return OSP_OK;
}

osp_status osp_lgp_correct(osp_ctx *ctx, const float *grads, int64_t worker_stride, void *stream)
{
    return lgp_correct(ctx, grads, worker_stride, stream, false);
}

osp_status osp_lgp_correct_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride,
                                void *stream)
{
    return lgp_correct(ctx, grads, worker_stride, stream, true);
}

// Install launch over a span table: every replica receives the PS values of the table's spans
// (masked: of their elements in `stage` under the element-granular GIB).
static osp_status launch_install(osp_ctx *ctx, const Span *table, unsigned n_spans, int stage,
                                 bool masked, hipStream_t s)
{
    const uint32_t *bitmap = ctx->element_keys ? ctx->d_bitmap() : nullptr;
    if (ctx->n_workers > kFanoutMaxWorkers) {
        ApplyArgs a;
        a.cap_spans = (unsigned)ctx->spans.size();
        a.bitmap = bitmap;
        a.P = ctx->P;
        a.Pw = ctx->Pw;
        a.param_stride = ctx->param_stride;
        const SweepShape sh = sweep_shape(ctx, n_spans);
        a.pieces_per_span = sh.pieces_per_span;
        a.pieces_shift = sh.pieces_shift;
        a.spans_per_block = sh.spans_per_block;
        a.stage = stage;
        if (sh.n_blocks > 65535u || ctx->n_workers > 65535)
            return fail(ctx, OSP_ERR_UNSUPPORTED,
                        "install launch of %u blocks x %d workers exceeds the grid limit", sh.n_blocks,
                        ctx->n_workers);
        const dim3 grid(sh.spans_per_block * sh.pieces_per_span, (unsigned)ctx->n_workers, sh.n_blocks);
        const dim3 block(kApplyBlock);
        if (sh.n_blocks > 0) {
            if (masked)
                k_apply_stage_sweep<true, kSweepVec><<<grid, block, 0, s>>>(table, a);
            else
                k_apply_stage_sweep<false, kSweepVec><<<grid, block, 0, s>>>(table, a);
        }
    } else {
        FanoutArgs a;
        a.cap_spans = (unsigned)ctx->spans.size();
        a.chunk_elems = ctx->chunk_elems;
        a.bitmap = bitmap;
        a.P = ctx->P;
        a.Pw = ctx->Pw;
        a.param_stride = ctx->param_stride;
        a.n_workers = ctx->n_workers;
        a.stage = stage;
        const dim3 grid(n_spans * kSpanChunks), block(kBlock);
        if (n_spans > 0) {
            if (masked)
                k_apply_stage_fanout<true><<<grid, block, 0, s>>>(table, a);
            else
                k_apply_stage_fanout<false><<<grid, block, 0, s>>>(table, a);
        }
    }
    return launch_check(ctx, "k_apply_stage");
}

osp_status osp_apply_stage(osp_ctx *ctx, int stage, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (stage < 0 || stage > 2)
        return fail(ctx, OSP_ERR_INVALID_ARG, "stage must be 0, 1 or 2 (got %d)", stage);
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (stage != 0 && !ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "a staged call needs a GIB");
    if (stage == 1 && !ctx->agg1)
        return fail(ctx, OSP_ERR_BAD_STATE, "stage 1 has not been aggregated in this iteration");
    if (stage != 1 && !(ctx->agg1 && ctx->agg2))
        return fail(ctx, OSP_ERR_BAD_STATE, "stage 2 has not been aggregated in this iteration");
    // Element-granular GIB: two situations in which writing ALL elements gives the same result
    // as writing the stage's elements only, with full-width stores and no read of old values:
    //  * stage 2 after this iteration's stage 1 was installed: the stage-1 elements of every
    //    replica already equal the PS and have not changed since;
    //  * stage 1 when the replicas were in sync as the iteration began and neither LGP nor the
    //    stage-2 aggregate has run yet: the stage-2 elements of every replica still equal the
    //    PS's (both hold the stale value).
    const bool element = ctx->gib_gran == OSP_GRAN_ELEMENT;
    const bool overwrite_all =
        element && ((stage == 2 && ctx->applied1) ||
                    (stage == 1 && ctx->iter_synced && !ctx->agg2 && !ctx->lgp_done));
    const bool masked = stage != 0 && ctx->gib_gran == OSP_GRAN_ELEMENT && !overwrite_all;
    const bool listed = stage != 0 && ctx->gib_gran == OSP_GRAN_LAYER;
    unsigned n_spans = (unsigned)ctx->spans.size();
    const Span *table = ctx->d_spans();
    if (listed) {
        const StageLaunch L = stage_launch(ctx, stage, (hipStream_t)stream);
        table = L.table;
        n_spans = L.grid_spans;
    }
    osp_status st = launch_install(ctx, table, n_spans, stage, masked, (hipStream_t)stream);
    if (st != OSP_OK)
        return st;
    if (stage != 1)
        ctx->applied2 = true;
    if (stage != 2)
        ctx->applied1 = true;
    if (ctx->applied1 && ctx->applied2)
        ctx->replicas_synced = true;    // every element of every replica equals the PS again
    return OSP_OK;
}

// Largest N for which the element-granular RS window keeps all gradients of a group in registers.
constexpr int kRsElementMaxWorkers = 16;
// Layer-granular windows run fused up to this many gradient elements (N x parameters), where a
// step is bound by its launches.  Above, the single-stage kernels win: LGP there keeps the
// stage-2 aggregate, which the fused launch does not (it reads the stage-2 gradients twice).
constexpr long long kWindowLayerMaxGradElems = 32LL << 20;

static bool layer_window_fused(const osp_ctx *ctx)
{
    return ctx->n_workers <= kWindowMaxWorkers &&
           (long long)ctx->n_workers * ctx->n_params <= kWindowLayerMaxGradElems;
}

static osp_status rs_window(osp_ctx *ctx, const void *grads, int64_t worker_stride, void *stream,
                            bool bf16)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    osp_status st = check_grads(ctx, grads, worker_stride, bf16);
    if (st != OSP_OK)
        return st;
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (!ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "a staged call needs a GIB (osp_set_gib or osp_split)");
    if (stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE,
                    "stage 2 of the previous iteration is still pending (ICS must complete first)");
    const bool element = ctx->gib_gran == OSP_GRAN_ELEMENT;
    const int N = ctx->n_workers;
    // The fused kernels take LGP's stale values from the PS arena: every replica must equal it.
    const bool fused = ctx->replicas_synced &&
                       (element ? N <= kRsElementMaxWorkers : layer_window_fused(ctx));
    ctx->windows_fused = fused ? 1 : 0;
    if (!fused) {
        st = aggregate_update(ctx, 1, grads, worker_stride, stream, bf16);
        if (st == OSP_OK)
            st = osp_apply_stage(ctx, 1, stream);
        if (st == OSP_OK)
            st = lgp_correct(ctx, grads, worker_stride, stream, bf16);
        return st;
    }
    hipStream_t s = (hipStream_t)stream;
    if (element) {
        RsElementArgs a;
        a.spans = ctx->d_spans();
        a.chunk_elems = ctx->chunk_elems;
        a.bitmap = ctx->d_bitmap();
        a.P = ctx->P;
        a.V = ctx->V;
        a.grads = grads;
        a.worker_stride = worker_stride;
        a.weights = ctx->d_weights();
        a.partial1 = ctx->d_partial(0);
        a.partial2 = ctx->d_partial(1);
        a.key = ctx->d_key();
        a.stash = ctx->d_stash();
        a.Pw = ctx->Pw;
        a.param_stride = ctx->param_stride;
        a.n_workers = N;
        a.inv_n = 1.0f / (float)N;
        a.lr = ctx->lr;
        a.mu = ctx->mu;
        const dim3 grid((unsigned)ctx->spans.size() * kSpanChunks);
        if (bf16)
            launch_rs_window_element<bf16_t>(ctx, a, grid, s);
        else
            launch_rs_window_element<float>(ctx, a, grid, s);
    } else {
        // No wait for the table lengths of a split that may still be running: the launch covers
        // both tables (all spans), and the kernel reads where the first one ends.
        WindowLayerArgs a;
        a.agg_spans = ctx->d_list(1);
        a.n_agg_spans = &ctx->d_state()->stage_spans[ctx->tables][0];
        a.lgp_spans = ctx->d_list(2);
        a.chunk_elems = ctx->chunk_elems;
        a.P = ctx->P;
        a.V = ctx->V;
        a.grads = grads;
        a.worker_stride = worker_stride;
        a.weights = ctx->d_weights();
        a.partial = ctx->d_partial(0);
        a.key = ctx->element_keys ? ctx->d_key() : nullptr;
        a.Pw = ctx->Pw;
        a.param_stride = ctx->param_stride;
        a.n_workers = N;
        a.inv_n = 1.0f / (float)N;
        a.lr = ctx->lr;
        a.mu = ctx->mu;
        const unsigned n_groups = (unsigned)ctx->spans.size() * kSpanChunks;
        launch_window_layer(ctx, a, n_groups, s, bf16);
    }
    st = launch_check(ctx, "osp_rs_window");
    if (st != OSP_OK)
        return st;
    ctx->iter_synced = true;
    ctx->replicas_synced = false;
    ctx->stash_valid = element;
    ctx->stash_grads = grads;
    ctx->stash_stride = (long long)worker_stride;
    ctx->stash_bf16 = bf16;
    ctx->agg1 = ctx->applied1 = ctx->lgp_done = ctx->last_lgp_shared = true;
    ctx->last_lgp_kept = false;
    ctx->agg2 = ctx->single_pass = ctx->applied2 = false;
    return OSP_OK;
}

osp_status osp_rs_window(osp_ctx *ctx, const float *grads, int64_t worker_stride, void *stream)
{
    return rs_window(ctx, grads, worker_stride, stream, false);
}

osp_status osp_rs_window_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride, void *stream)
{
    return rs_window(ctx, grads, worker_stride, stream, true);
}

static osp_status ics_window(osp_ctx *ctx, const void *grads, int64_t worker_stride, int granularity,
                             int64_t budget_elems, void *stream, bool bf16)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    osp_status st = check_grads(ctx, grads, worker_stride, bf16);
    if (st != OSP_OK)
        return st;
    // the split's arguments are checked before anything is launched
    if (granularity != OSP_GRAN_LAYER && granularity != OSP_GRAN_ELEMENT)
        return fail(ctx, OSP_ERR_INVALID_ARG, "unknown granularity %d", granularity);
    if (budget_elems < 0 || budget_elems > ctx->n_params)
        return fail(ctx, OSP_ERR_INVALID_ARG, "budget %lld outside [0, %lld]",
                    (long long)budget_elems, ctx->n_params);
    if (granularity == OSP_GRAN_ELEMENT && !ctx->element_keys)
        return fail(ctx, OSP_ERR_UNSUPPORTED, "element granularity needs cfg.element_keys");
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (!stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE, "stage 2 needs this iteration's stage 1 first");
    const bool element = ctx->gib_gran == OSP_GRAN_ELEMENT;
    const int N = ctx->n_workers;
    // element-granular: whole groups of PS values go into the replicas, which is an install of
    // stage 2 only if stage 1 is in place there
    // (above 8 replicas the per-replica install sweep beats writing them all from one lane)
    const bool fused = element ? (ctx->applied1 && N <= kWindowMaxWorkers) : layer_window_fused(ctx);
    ctx->windows_fused = (ctx->windows_fused & 1) | (fused ? 2 : 0);
    hipStream_t s = (hipStream_t)stream;
    if (!fused && !element && !stream_is_capturing(s)) {
        // Layer-granular GIB: the split only needs the stage-2 aggregate, and it writes the new
        // stage tables into the other set.  Enqueued ahead of the install, it publishes the new
        // table lengths while the install still runs, so a host that keeps pace with the GPU
        // sizes the next iteration's grids exactly.  (Not while a graph is being captured: a
        // captured split writes the set of tables its own iteration read, see osp_split.)
        st = aggregate_update(ctx, 2, grads, worker_stride, stream, bf16);
        if (st != OSP_OK)
            return st;
        const StageLaunch old2 = stage_launch(ctx, 2, s);    // the tables this iteration ran on
        const bool stage1_installed = ctx->applied1;
        st = osp_split(ctx, granularity, budget_elems, stream);
        if (st != OSP_OK)
            return st;
        st = launch_install(ctx, old2.table, old2.grid_spans, 2, false, s);
        if (st != OSP_OK)
            return st;
        if (stage1_installed)
            ctx->replicas_synced = true;    // every element of every replica equals the PS again
        return OSP_OK;
    }
    if (!fused) {
        st = aggregate_update(ctx, 2, grads, worker_stride, stream, bf16);
        if (st == OSP_OK)
            st = osp_apply_stage(ctx, 2, stream);
        if (st != OSP_OK)
            return st;
    } else {
        if (element) {
            const bool from_stash = ctx->stash_valid && ctx->stash_grads == grads &&
                                    ctx->stash_stride == (long long)worker_stride && ctx->stash_bf16 == bf16;
            IcsElementArgs a;
            a.spans = ctx->d_spans();
            a.chunk_elems = ctx->chunk_elems;
            a.bitmap = ctx->d_bitmap();
            a.P = ctx->P;
            a.V = ctx->V;
            a.stash = ctx->d_stash();
            a.grads = grads;
            a.worker_stride = worker_stride;
            a.weights = ctx->d_weights();
            a.partial2 = ctx->d_partial(1);
            a.key = ctx->d_key();
            a.Pw = ctx->Pw;
            a.param_stride = ctx->param_stride;
            a.n_workers = N;
            a.inv_n = 1.0f / (float)N;
            a.lr = ctx->lr;
            a.mu = ctx->mu;
            const dim3 grid((unsigned)ctx->spans.size() * kSpanChunks), block(kBlock);
            // (N + 2) KB of stores per wavefront; bounded like the loads of the RS window
            const unsigned lds = occupancy_lds(wave_bytes(N, sizeof(float), 2), kWindowBytesInFlightPerCu);
            if (from_stash)
                k_ics_window_element<true, false><<<grid, block, lds, s>>>(a);
            else if (bf16 && ctx->weighted)
                k_ics_window_element<false, true, bf16_t><<<grid, block, lds, s>>>(a);
            else if (bf16)
                k_ics_window_element<false, false, bf16_t><<<grid, block, lds, s>>>(a);
            else if (ctx->weighted)
                k_ics_window_element<false, true><<<grid, block, lds, s>>>(a);
            else
                k_ics_window_element<false, false><<<grid, block, lds, s>>>(a);
        } else {
            // (the launch covers all groups; the kernel reads the stage-2 table's length)
            WindowLayerArgs a;
            a.agg_spans = ctx->d_list(2);
            a.n_agg_spans = &ctx->d_state()->stage_spans[ctx->tables][1];
            a.lgp_spans = nullptr;
            a.chunk_elems = ctx->chunk_elems;
            a.P = ctx->P;
            a.V = ctx->V;
            a.grads = grads;
            a.worker_stride = worker_stride;
            a.weights = ctx->d_weights();
            a.partial = ctx->d_partial(1);
            a.key = ctx->element_keys ? ctx->d_key() : nullptr;
            a.Pw = ctx->Pw;
            a.param_stride = ctx->param_stride;
            a.n_workers = N;
            a.inv_n = 1.0f / (float)N;
            a.lr = ctx->lr;
            a.mu = ctx->mu;
            launch_window_layer(ctx, a, (unsigned)ctx->spans.size() * kSpanChunks, s, bf16);
        }
        st = launch_check(ctx, "osp_ics_window");
        if (st != OSP_OK)
            return st;
        ctx->agg2 = ctx->applied2 = true;
        if (ctx->applied1)
            ctx->replicas_synced = true;
    }
    return osp_split(ctx, granularity, budget_elems, stream);
}

osp_status osp_ics_window(osp_ctx *ctx, const float *grads, int64_t worker_stride, int granularity,
                          int64_t budget_elems, void *stream)
{
    return ics_window(ctx, grads, worker_stride, granularity, budget_elems, stream, false);
}

osp_status osp_ics_window_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride,
                               int granularity, int64_t budget_elems, void *stream)
{
    return ics_window(ctx, grads, worker_stride, granularity, budget_elems, stream, true);
}

osp_status osp_sync_step(osp_ctx *ctx, const float *grads, int64_t worker_stride, int granularity,
                         int64_t budget_elems, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    // the split's arguments are checked before the RS window changes anything
    if (granularity != OSP_GRAN_LAYER && granularity != OSP_GRAN_ELEMENT)
        return fail(ctx, OSP_ERR_INVALID_ARG, "unknown granularity %d", granularity);
    if (budget_elems < 0 || budget_elems > ctx->n_params)
        return fail(ctx, OSP_ERR_INVALID_ARG, "budget %lld outside [0, %lld]",
                    (long long)budget_elems, ctx->n_params);
    if (granularity == OSP_GRAN_ELEMENT && !ctx->element_keys)
        return fail(ctx, OSP_ERR_UNSUPPORTED, "element granularity needs cfg.element_keys");
    osp_status st = osp_rs_window(ctx, grads, worker_stride, stream);
    if (st != OSP_OK)
        return st;
    return osp_ics_window(ctx, grads, worker_stride, granularity, budget_elems, stream);
}

// Build the pack index of the current GIB if it is not there yet (four small launches).
static osp_status ensure_pack_index(osp_ctx *ctx, hipStream_t s)
{
    if (ctx->pack_index_valid)
        return OSP_OK;
    PackIndexArgs a;
    a.spans = ctx->d_spans();
    a.span_layer = ctx->d_slayer();
    a.gib_layer = ctx->d_gib();
    a.bitmap = ctx->element_keys ? ctx->d_bitmap() : nullptr;
    a.chunk_elems = ctx->chunk_elems;
    a.element = ctx->gib_gran == OSP_GRAN_ELEMENT ? 1 : 0;
    a.base1 = ctx->d_pack_base(1);
    a.base2 = ctx->d_pack_base(2);
    const unsigned n_groups = (unsigned)ctx->spans.size() * kSpanChunks;
    const unsigned nb = (unsigned)ctx->n_pack_blocks();
    k_pack_count<<<n_groups, kBlock, 0, s>>>(a);
    k_pack_block_totals<<<nb, kScanBlock, 0, s>>>(ctx->n_chunks, a.base1, a.base2,
                                                 ctx->d_pack_tot(1), ctx->d_pack_tot(2));
    k_pack_scan_totals<<<1, kScanBlock, 0, s>>>((long long)nb, ctx->n_chunks, ctx->d_pack_tot(1),
                                               ctx->d_pack_tot(2), a.base1, a.base2);
    k_pack_scan_chunks<<<nb, kScanBlock, 0, s>>>(ctx->n_chunks, ctx->d_pack_tot(1), ctx->d_pack_tot(2),
                                                a.base1, a.base2);
    osp_status st = launch_check(ctx, "pack index kernels");
    if (st != OSP_OK)
        return st;
    ctx->pack_index_valid = true;
    return OSP_OK;
}

static osp_status split_gradients(osp_ctx *ctx, const void *grads, int64_t worker_stride,
                                  void *g_important, int64_t important_stride,
                                  void *g_unimportant, int64_t unimportant_stride, void *stream,
                                  bool bf16)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    osp_status st = check_grads(ctx, grads, worker_stride, bf16);
    if (st != OSP_OK)
        return st;
    if (!g_important && !g_unimportant)
        return fail(ctx, OSP_ERR_INVALID_ARG, "both outputs are NULL");
    const uintptr_t elem = bf16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(g_important) % elem != 0 ||
        reinterpret_cast<uintptr_t>(g_unimportant) % elem != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG, "outputs must be %d-byte aligned", (int)elem);
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (!ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "the splitter needs a GIB");
    st = stage_counts(ctx);             // the stage-2 size of a split that may still be running
    if (st != OSP_OK)
        return st;
    const long long e2 = ctx->n_stage2_host, e1 = ctx->n_params - e2;
    if (g_important && important_stride < e1)
        return fail(ctx, OSP_ERR_INVALID_ARG, "important_stride %lld is below the %lld stage-1 elements",
                    (long long)important_stride, e1);
    if (g_unimportant && unimportant_stride < e2)
        return fail(ctx, OSP_ERR_INVALID_ARG, "unimportant_stride %lld is below the %lld stage-2 elements",
                    (long long)unimportant_stride, e2);
    hipStream_t s = (hipStream_t)stream;
    st = ensure_pack_index(ctx, s);
    if (st != OSP_OK)
        return st;
    SplitGradArgs a;
    a.spans = ctx->d_spans();
    a.span_layer = ctx->d_slayer();
    a.gib_layer = ctx->d_gib();
    a.bitmap = ctx->element_keys ? ctx->d_bitmap() : nullptr;
    a.chunk_elems = ctx->chunk_elems;
    a.element = ctx->gib_gran == OSP_GRAN_ELEMENT ? 1 : 0;
    a.base1 = ctx->d_pack_base(1);
    a.base2 = ctx->d_pack_base(2);
    a.worker_stride = worker_stride;
    a.stride_i = important_stride;
    a.stride_u = unimportant_stride;
    const unsigned n_groups = (unsigned)ctx->spans.size() * kSpanChunks;
    for (int w0 = 0; w0 < ctx->n_workers; w0 += 65535) {   // grid.y is limited to 65535
        const int nw = ctx->n_workers - w0 < 65535 ? ctx->n_workers - w0 : 65535;
        const long long esz = (long long)elem;
        a.grads = static_cast<const char *>(grads) + (long long)w0 * worker_stride * esz;
        a.g_i = g_important ? static_cast<char *>(g_important) + (long long)w0 * important_stride * esz
                            : nullptr;
        a.g_u = g_unimportant
                    ? static_cast<char *>(g_unimportant) + (long long)w0 * unimportant_stride * esz
                    : nullptr;
        if (bf16)
            k_split_gradients<bf16_t><<<dim3(n_groups, (unsigned)nw), kBlock, 0, s>>>(a);
        else
            k_split_gradients<float><<<dim3(n_groups, (unsigned)nw), kBlock, 0, s>>>(a);
    }
    return launch_check(ctx, "k_split_gradients");
}

osp_status osp_split_gradients(osp_ctx *ctx, const float *grads, int64_t worker_stride,
                               float *g_important, int64_t important_stride,
                               float *g_unimportant, int64_t unimportant_stride, void *stream)
{
    return split_gradients(ctx, grads, worker_stride, g_important, important_stride, g_unimportant,
                           unimportant_stride, stream, false);
}

osp_status osp_split_gradients_bf16(osp_ctx *ctx, const uint16_t *grads, int64_t worker_stride,
                                    uint16_t *g_important, int64_t important_stride,
                                    uint16_t *g_unimportant, int64_t unimportant_stride,
                                    void *stream)
{
    return split_gradients(ctx, grads, worker_stride, g_important, important_stride, g_unimportant,
                           unimportant_stride, stream, true);
}

static osp_status aggregate_update_packed(osp_ctx *ctx, int stage, const void *packed,
                                          int64_t packed_stride, void *stream, bool bf16)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (stage != 1 && stage != 2)
        return fail(ctx, OSP_ERR_INVALID_ARG, "stage must be 1 or 2 (got %d)", stage);
    if (!packed)
        return fail(ctx, OSP_ERR_INVALID_ARG, "packed is NULL");
    if (reinterpret_cast<uintptr_t>(packed) % (bf16 ? 2 : 4) != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG, "packed must be %d-byte aligned", bf16 ? 2 : 4);
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (!ctx->have_gib)
        return fail(ctx, OSP_ERR_BAD_STATE, "a staged call needs a GIB (osp_set_gib or osp_split)");
    if (stage == 1 && stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE,
                    "stage 2 of the previous iteration is still pending (ICS must complete first)");
    if (stage == 2 && !stage2_pending(ctx))
        return fail(ctx, OSP_ERR_BAD_STATE, "stage 2 needs this iteration's stage 1 first");
    osp_status st = stage_counts(ctx);
    if (st != OSP_OK)
        return st;
    const long long e2 = ctx->n_stage2_host, need = stage == 1 ? ctx->n_params - e2 : e2;
    if (packed_stride < need)
        return fail(ctx, OSP_ERR_INVALID_ARG, "packed_stride %lld is below the %lld elements of stage %d",
                    (long long)packed_stride, need, stage);
    hipStream_t s = (hipStream_t)stream;
    st = ensure_pack_index(ctx, s);
    if (st != OSP_OK)
        return st;
    PackedAggArgs a;
    a.spans = ctx->d_spans();
    a.span_layer = ctx->d_slayer();
    a.gib_layer = ctx->d_gib();
    a.bitmap = ctx->element_keys ? ctx->d_bitmap() : nullptr;
    a.chunk_elems = ctx->chunk_elems;
    a.element = ctx->gib_gran == OSP_GRAN_ELEMENT ? 1 : 0;
    a.base = ctx->d_pack_base(stage);
    a.P = ctx->P;
    a.V = ctx->V;
    a.packed = packed;
    a.packed_stride = packed_stride;
    a.weights = ctx->d_weights();
    a.partial = ctx->d_partial(stage == 2 ? 1 : 0);
    a.key = ctx->element_keys ? ctx->d_key() : nullptr;
    a.n_workers = ctx->n_workers;
    a.stage = stage;
    a.inv_n = 1.0f / (float)ctx->n_workers;
    a.lr = ctx->lr;
    a.mu = ctx->mu;
    const dim3 grid((unsigned)ctx->spans.size() * kSpanChunks), block(kBlock);
    // an empty stage launches nothing, unless the GIB is element-granular: a layer split sums
    // both stages' importance partials of every chunk, so each call has to leave its own
    if (need > 0 || a.element) {
        const int variant = (ctx->weighted ? 2 : 0) | (ctx->element_keys ? 1 : 0);
        if (bf16)
            launch_aggregate_packed<bf16_t>(variant, grid, block, s, a);
        else
            launch_aggregate_packed<float>(variant, grid, block, s, a);
    }
    st = launch_check(ctx, "k_aggregate_update_packed");
    if (st != OSP_OK)
        return st;
    if (stage == 1) {                   // a new iteration begins: the PS moves away from the replicas
        ctx->iter_synced = ctx->replicas_synced;
        ctx->replicas_synced = false;
        ctx->stash_valid = false;       // the stage-2 gradients were not at hand
        ctx->agg1 = true;
        ctx->agg2 = ctx->single_pass = ctx->lgp_done = ctx->applied1 = ctx->applied2 = false;
    } else {
        ctx->agg2 = true;
    }
    return OSP_OK;
}

osp_status osp_ps_aggregate_update_packed(osp_ctx *ctx, int stage, const float *packed,
                                          int64_t packed_stride, void *stream)
{
    return aggregate_update_packed(ctx, stage, packed, packed_stride, stream, false);
}

osp_status osp_ps_aggregate_update_packed_bf16(osp_ctx *ctx, int stage, const uint16_t *packed,
                                               int64_t packed_stride, void *stream)
{
    return aggregate_update_packed(ctx, stage, packed, packed_stride, stream, true);
}

osp_status osp_split(osp_ctx *ctx, int granularity, int64_t budget_elems, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (granularity != OSP_GRAN_LAYER && granularity != OSP_GRAN_ELEMENT)
        return fail(ctx, OSP_ERR_INVALID_ARG, "unknown granularity %d", granularity);
    if (budget_elems < 0 || budget_elems > ctx->n_params)
        return fail(ctx, OSP_ERR_INVALID_ARG, "budget %lld outside [0, %lld]",
                    (long long)budget_elems, ctx->n_params);
    if (granularity == OSP_GRAN_ELEMENT && !ctx->element_keys)
        return fail(ctx, OSP_ERR_UNSUPPORTED, "element granularity needs cfg.element_keys");
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    if (!(ctx->agg1 && ctx->agg2))
        return fail(ctx, OSP_ERR_BAD_STATE,
                    "split needs the importances of a complete iteration (stage 2 or stage 0 aggregate)");
    hipStream_t s = (hipStream_t)stream;
    const int old_tables = ctx->tables;
    const bool old_pending = ctx->counts_pending;
    if (granularity == OSP_GRAN_LAYER) {
        const int mode = ctx->single_pass ? 0 : (ctx->gib_gran == OSP_GRAN_LAYER ? 1 : 2);
        const int ns = (int)ctx->spans.size();
        // The new GIB's tables go into the other set, so that a launch over the old ones may
        // still follow.  A split captured into a graph stays on its set: every replay reads
        // the tables the replay before it wrote (the captured launches name one set for good),
        // and nothing that reads the old tables is captured behind it.
        if (!stream_is_capturing(s))
            ctx->tables ^= 1;
        if (ctx->n_tensors <= kRankTile) {
            // one launch: segment sums in every workgroup, then the last one ranks in LDS and,
            // unless the tables are long, fills them as well
            const bool fill = ns <= kRankFillMaxSpans;
            const int n_seg = (int)ctx->segments.size();
            constexpr int kPer = kRankBlock / kSplitBlock;
            k_layer_split_lds<kRankBlock><<<(unsigned)((n_seg + kPer - 1) / kPer), kRankBlock, 0, s>>>(
                ctx->d_segs(), n_seg, ctx->d_partial(0), ctx->d_partial(1), mode, ctx->d_segsum(),
                ctx->n_tensors, ctx->d_lsb(), ctx->d_big(), (int)ctx->big_layers.size(),
                ctx->d_imp(), ctx->d_numel(), ctx->d_lsp(), (long long)budget_elems, ctx->d_gib(),
                ctx->d_order(), ctx->d_lbase(), ctx->d_state(), ctx->pinned_counts_dev, ++ctx->split_seq,
                ctx->tables, fill ? ns : 0, ctx->d_spans(), ctx->d_slayer(), ctx->d_list(1),
                ctx->d_list(2));
            if (fill) {
                ctx->counts_pending = true;
            } else {
                osp_status ls = enqueue_stage_lists(ctx, s);
                if (ls != OSP_OK)
                    return ls;
            }
        } else {
            k_segment_importance<<<(unsigned)ctx->segments.size(), kSplitBlock, 0, s>>>(
                ctx->d_segs(), ctx->d_partial(0), ctx->d_partial(1), ctx->d_gib(), mode, ctx->d_segsum());
            k_layer_rank<<<1, kRankBlock, 0, s>>>(ctx->n_tensors, ctx->d_segsum(), ctx->d_lsb(),
                                                  ctx->d_big(), (int)ctx->big_layers.size(),
                                                  ctx->d_imp(), ctx->d_numel(),
                                                  ctx->d_lsp(), (long long)budget_elems, ctx->d_gib(),
                                                  ctx->d_order(), ctx->d_lbase(), ctx->d_rscratch(),
                                                  ctx->d_state(), ctx->pinned_counts_dev, ++ctx->split_seq,
                                                  ctx->tables);
            osp_status ls = enqueue_stage_lists(ctx, s);
            if (ls != OSP_OK)
                return ls;
        }
        ctx->have_layer_importance = true;
    } else {
        SelectScratch w;
        w.state = ctx->d_state();
        w.hist = ctx->d_hist(0);
        w.cand = ctx->d_cand();
        w.tile_ties = ctx->d_tile_ties();
        enqueue_element_select(ctx->d_key(), ctx->n_vec, ctx->n_words, ctx->n_tiles,
                               (long long)budget_elems, w, ctx->d_bitmap(), s);
        ctx->counts_pending = false;    // stage tables belong to layer-granular GIBs only
        ctx->n_stage2_host = budget_elems;
    }
    osp_status st = launch_check(ctx, "split kernels");
    if (st != OSP_OK) {
        // The old GIB stays current with its set of tables, whose lengths on the device the
        // failed split did not touch (it works on the other set).  Sequence numbers are not
        // reused: part of the split may have been enqueued.
        ctx->tables = old_tables;
        ctx->counts_pending = old_pending;
        return st;
    }
    ctx->have_gib = true;
    ctx->pack_index_valid = false;
    ctx->gib_gran = granularity;
    ctx->agg1 = ctx->agg2 = ctx->single_pass = ctx->lgp_done = ctx->applied1 = ctx->applied2 = false;
    return OSP_OK;
}

osp_status osp_split_element_static(const uint32_t *keys, int64_t n_elems, int64_t budget_elems,
                                    uint32_t *elem_bitmap, void *stream)
{
    osp_ctx *ctx = nullptr;                    // messages go to the thread's slot (osp_last_error(NULL))
    if (!keys || !elem_bitmap)
        return fail(ctx, OSP_ERR_INVALID_ARG, "keys and elem_bitmap must not be NULL");
    if (!aligned16(keys) || reinterpret_cast<uintptr_t>(elem_bitmap) % 4 != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG, "keys must be 16-byte and elem_bitmap 4-byte aligned");
    if (n_elems <= 0 || n_elems % 4 != 0)
        return fail(ctx, OSP_ERR_INVALID_ARG, "n_elems must be a positive multiple of 4 (got %lld)",
                    (long long)n_elems);
    if (n_elems > kStaticMaxElems)
        return fail(ctx, OSP_ERR_UNSUPPORTED,
                    "n_elems %lld exceeds the %lld keys the built-in scratch is sized for",
                    (long long)n_elems, kStaticMaxElems);
    if (budget_elems < 0 || budget_elems > n_elems)
        return fail(ctx, OSP_ERR_INVALID_ARG, "budget %lld outside [0, %lld]",
                    (long long)budget_elems, (long long)n_elems);
    unsigned char *base = nullptr;
    OSP_HIP(static_scratch(&base));
    SelectScratch w;
    w.state = reinterpret_cast<SplitState *>(base);
    w.hist = reinterpret_cast<unsigned long long *>(base + kStaticOffHist);
    w.cand = reinterpret_cast<TieCandidate *>(base + kStaticOffCand);
    w.tile_ties = reinterpret_cast<unsigned int *>(base + kStaticOffTies);
    const long long n_tiles = (n_elems + kSelTile - 1) / kSelTile;
    // The array keeps what the last call on this GPU left: the split state (its tickets) and
    // the histograms must start at zero, whatever became of that call.
    k_fill_u32<<<24, kSplitBlock, 0, (hipStream_t)stream>>>(reinterpret_cast<uint32_t *>(base),
                                                            (long long)(kStaticOffCand / 4), 0u);
    enqueue_element_select(keys, n_elems / 4, (n_elems + 31) / 32, n_tiles, (long long)budget_elems,
                           w, elem_bitmap, (hipStream_t)stream);
    return launch_check(ctx, "element select kernels");
}

osp_status osp_stream_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0)
        return OSP_ERR_INVALID_ARG;
    const long long n_vec = (long long)(bytes / 16);
    const long long groups = (n_vec + kBlock - 1) / kBlock;
    if (groups > 0x7FFFFFFFLL)
        return OSP_ERR_INVALID_ARG;
    if (groups > 0)
        k_stream_copy<<<(unsigned)groups, kBlock, 0, (hipStream_t)stream>>>((float *)dst,
                                                                           (const float *)src, n_vec);
    return hipGetLastError() == hipSuccess ? OSP_OK : OSP_ERR_HIP;
}

osp_status osp_stream_pattern(const float *reads, int32_t n_read, int64_t read_stride, float *rw,
                              int32_t n_rw, int64_t rw_stride, int64_t n_elems, void *stream)
{
    if (!reads || !rw || !aligned16(reads) || !aligned16(rw) || n_read < 1 || n_rw < 1 || n_rw > 2 ||
        n_elems < 0 || n_elems % 4 != 0 || read_stride % 4 != 0 || rw_stride % 4 != 0 ||
        read_stride < n_elems || rw_stride < n_elems)
        return OSP_ERR_INVALID_ARG;
    PatternArgs a;
    a.reads = reads;
    a.read_stride = read_stride;
    a.rw = rw;
    a.rw_stride = rw_stride;
    a.n_vec = n_elems / 4;
    a.n_read = n_read;
    a.n_rw = n_rw;
    const long long groups = (a.n_vec + kBlock - 1) / kBlock;
    if (groups > 0x7FFFFFFFLL)
        return OSP_ERR_INVALID_ARG;
    if (groups > 0) {
        // bounded like the aggregate whose traffic it stands for
        const unsigned lds = occupancy_lds(wave_bytes(n_read, sizeof(float), n_rw), kLoadsInFlightPerCu);
        k_stream_pattern<<<(unsigned)groups, kBlock, lds, (hipStream_t)stream>>>(a);
    }
    return hipGetLastError() == hipSuccess ? OSP_OK : OSP_ERR_HIP;
}

double osp_ics_upper_bound(double bandwidth_elems_per_s, double loss_rate, double t_compute_s,
                           int32_t n_workers)
{
    if (!(std::isfinite(bandwidth_elems_per_s) && bandwidth_elems_per_s >= 0.0) ||
        !(std::isfinite(loss_rate) && loss_rate >= 0.0) ||
        !(std::isfinite(t_compute_s) && t_compute_s >= 0.0) || n_workers < 1)
        return 0.0;
    return bandwidth_elems_per_s * (1.0 + loss_rate) * t_compute_s / (double)n_workers;
}

int64_t osp_tune_budget(int32_t epoch, double loss_i, double loss_1, double u_max,
                        int64_t model_elems)
{
    if (epoch < 1 || model_elems < 0 || !std::isfinite(loss_i) || !std::isfinite(loss_1) ||
        !(loss_1 > 0.0) || !std::isfinite(u_max) || u_max < 0.0)
        return -1;
    const double cap = 0.8 * (double)model_elems;
    const double u = u_max < cap ? u_max : cap;
    if (epoch == 1)
        return 0;
    double s = (1.0 - loss_i / loss_1) * u;
    if (!(s > 0.0))
        s = 0.0;
    if (s > u)
        s = u;
    return (int64_t)std::floor(s);
}

osp_status osp_get_importance(osp_ctx *ctx, double *imp_host, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (!imp_host)
        return fail(ctx, OSP_ERR_INVALID_ARG, "imp_host is NULL");
    if (!ctx->bound || !ctx->have_layer_importance)
        return fail(ctx, OSP_ERR_BAD_STATE, "no layer importances yet (osp_split with OSP_GRAN_LAYER first)");
    hipStream_t s = (hipStream_t)stream;
    OSP_HIP(hipMemcpyAsync(imp_host, ctx->d_imp(), (size_t)ctx->n_tensors * sizeof(double),
                           hipMemcpyDeviceToHost, s));
    OSP_HIP(hipStreamSynchronize(s));
    return OSP_OK;
}

osp_status osp_get_keys(osp_ctx *ctx, uint32_t *key_host, void *stream)
{
    if (!ctx)
        return OSP_ERR_INVALID_ARG;
    if (!key_host)
        return fail(ctx, OSP_ERR_INVALID_ARG, "key_host is NULL");
    if (!ctx->element_keys)
        return fail(ctx, OSP_ERR_UNSUPPORTED, "keys need cfg.element_keys");
    if (!ctx->bound)
        return fail(ctx, OSP_ERR_BAD_STATE, "osp_bind first");
    hipStream_t s = (hipStream_t)stream;
    OSP_HIP(hipMemcpyAsync(key_host, ctx->d_key(), (size_t)ctx->arena * sizeof(uint32_t),
                           hipMemcpyDeviceToHost, s));
    OSP_HIP(hipStreamSynchronize(s));
    return OSP_OK;
}

} // extern "C"
