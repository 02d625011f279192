// C interface of libs2v.so: argument checks, workspace layout and the order of kernel launches.
// See include/s2v.h for the contract of every entry point.
#include <cmath>
#include <mutex>
#include <new>
#include <cstdlib>
#include <vector>

#include "../../include/s2v.h"
#include "internal.h"
#include "loop_util.h"

using namespace s2v;

namespace {

struct Prepared {
    const void *ws;
    const int32_t *rowptr;
    const int32_t *colidx;
    const float *w;      // the edge sums in the head of ws were formed from these weights
    int32_t N;
    int64_t nnz;
    int32_t G;
    int32_t n_chunks;
    int32_t n_hubs;
    int32_t n_segs;
    bool has_neg;   // some stored weight is negative
    int32_t max_graph_nodes;   // nodes of the largest graph of the batch
    int32_t max_hub_segs;      // segments of the longest row
    // s2v_mvc_inference keeps the single-state node records (and q+-) in the head of the workspace over its
    // steps: the state update refreshes the records of the rows it changes, so they are not rebuilt per evaluation
    mutable bool rec_keep = false;      // the loop is running on this workspace
    mutable bool rec_current = false;   // ... and the records in the head match x, s+ and s-
};

// Carves consecutive 256-byte aligned pieces out of a byte range.
struct Carver {
    size_t off;
    explicit Carver(size_t start) : off(align_up(start)) {}
    size_t take(size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes);
        return at;
    }
};

struct HeadLayout {
    size_t s_pos, s_neg, nbr_sp, nbr_spw, chunk_begin, chunk_end, graph_chunk_off;
    size_t hub_rows, hub_seg_off, seg_row, seg_begin, seg_end, touched, hub_of, epoch, loop_ctr, rec, qkeep, jobs, end;
    int max_chunks, max_hubs, max_segs;
};

// Bounds on hub rows and segments from the shape alone: a hub has more than kHubDegree entries,
// and a hub of d entries has ceil(d / kHubSegment) <= d / kHubSegment + 1 segments.
void hub_bounds(int64_t nnz, int *hubs, int *segs) {
    *hubs = (int)(nnz / (kHubDegree + 1));
    *segs = (int)(nnz / kHubSegment) + *hubs;
}

// Exact counts from the row pointers (host copy).
void hub_counts(const std::vector<int32_t> &rp, int *hubs, int *segs) {
    int h = 0, sg = 0;
    for (size_t v = 0; v + 1 < rp.size(); ++v) {
        const int d = rp[v + 1] - rp[v];
        if (d > kHubDegree) {
            ++h;
            sg += (d + kHubSegment - 1) / kHubSegment;
        }
    }
    *hubs = h;
    *segs = sg;
}

// The head holds room for `hubs` hub rows and `segs` segments: the exact counts once the graph is
// prepared, an upper bound when only its shape is known.
HeadLayout head_layout(int64_t N, int64_t G, int hubs, int segs) {
    HeadLayout h;
    h.max_chunks = (int)((N + kChunkNodes - 1) / kChunkNodes + G);
    h.max_hubs = hubs;
    h.max_segs = segs;
    Carver c(0);
    h.s_pos = c.take(sizeof(float) * N);
    h.s_neg = c.take(sizeof(float) * N);
    h.nbr_sp = c.take(sizeof(float) * N);   // per row: s_pos summed over its neighbours (see NodeInfo::xbits)
    h.nbr_spw = c.take(sizeof(float) * N);  // the same, each neighbour weighted by its edge weight
    h.chunk_begin = c.take(sizeof(int32_t) * h.max_chunks);
    h.chunk_end = c.take(sizeof(int32_t) * h.max_chunks);
    h.graph_chunk_off = c.take(sizeof(int32_t) * (G + 1));
    h.hub_rows = c.take(sizeof(int32_t) * h.max_hubs);
    h.hub_seg_off = c.take(sizeof(int32_t) * (h.max_hubs + 1));
    h.seg_row = c.take(sizeof(int32_t) * h.max_segs);
    h.seg_begin = c.take(sizeof(int32_t) * h.max_segs);
    h.seg_end = c.take(sizeof(int32_t) * h.max_segs);
    h.touched = c.take(sizeof(int32_t) * N);        // per-node words of the incremental state update
    h.hub_of = c.take(sizeof(int32_t) * (hubs > 0 ? N : 0));   // per node: its index among the long rows
    h.epoch = c.take(sizeof(int32_t) * 2);          // number of incremental updates so far; a flag of the preparation
    h.loop_ctr = c.take(sizeof(unsigned long long) * 2);   // counters of s2v_mvc_inference
    h.rec = c.take(sizeof(float) * 5 * N);          // its node records {x, s+, s-, 0} and the 4-byte table behind them
    h.qkeep = c.take(sizeof(float) * 2 * 128);      // its q+-
    h.jobs = c.take(sizeof(int32_t) * 2 * kUpdateJobs);   // row ranges handed from the first to the second half of an update
    h.end = c.off;
    return h;
}

struct FwdLayout { size_t qvec, info, xbits, tmp, gpart, hub_part, hub_sum, end; };
FwdLayout fwd_layout(const HeadLayout &h, int64_t N, int p, int S, bool need_tmp, size_t start = 0) {
    FwdLayout f;
    Carver c(start ? start : h.end);   // (start: behind the backward pass's pieces when both run in one call)
    f.qvec = c.take(sizeof(float) * 2 * p);
    f.info = c.take(sizeof(float) * (size_t)N * nodeinfo_stride(S));
    f.xbits = c.take(S == 1 ? sizeof(unsigned long long) * (size_t)((N + 63) / 64)
                            : (S % 16 == 0 ? sizeof(unsigned short) * (size_t)N * (S / 16) : 0));
    size_t part_rows = (size_t)h.max_chunks * S;
    const size_t fused_rows = (size_t)kRoundGridMax * (S == 16 ? 16 : 1);   // partials of a fused graph sum
    if (part_rows < fused_rows) part_rows = fused_rows;
    f.gpart = c.take(sizeof(float) * part_rows * p);
    f.tmp = c.take(need_tmp ? sizeof(float) * (size_t)N * S * p : 0);
    f.hub_part = c.take(sizeof(float) * (size_t)h.max_segs * S * p);
    f.hub_sum = c.take(sizeof(float) * (size_t)h.max_hubs * S * p);
    f.end = c.off;
    return f;
}

struct QLayout { size_t qa, end; };
QLayout q_layout(const HeadLayout &h, int S, int G) {
    QLayout q;
    Carver c(h.end);
    q.qa = c.take(sizeof(float) * (size_t)S * G);
    q.end = c.off;
    return q;
}

struct SelLayout { size_t part_val, part_idx, hist, state, blk, keys0, keys1, ids0, ids1, sort_cnt, end; };
SelLayout sel_layout(const HeadLayout &h, int64_t N, int64_t k) {
    SelLayout s;
    Carver c(h.end);
    const size_t n_scan_blk = (size_t)((N + kScanBlock - 1) / kScanBlock);
    const size_t n_sort_blk = (size_t)((k + kSortTile - 1) / kSortTile);
    s.part_val = c.take(sizeof(float) * h.max_chunks * kSmallK);
    s.part_idx = c.take(sizeof(int32_t) * h.max_chunks * kSmallK);
    s.hist = c.take(sizeof(uint32_t) * 4 * 256);
    s.state = c.take(sizeof(uint32_t) * 16);
    s.blk = c.take(sizeof(uint32_t) * 4 * n_scan_blk);
    s.keys0 = c.take(sizeof(uint32_t) * k);
    s.keys1 = c.take(sizeof(uint32_t) * k);
    s.ids0 = c.take(sizeof(int32_t) * k);
    s.ids1 = c.take(sizeof(int32_t) * k);
    s.sort_cnt = c.take(sizeof(uint32_t) * 256 * n_sort_blk);
    s.end = c.off;
    return s;
}

struct BwdLayout {
    size_t dg, da, glo, ghi, head_part, dz0, dz1, maskT, rec, flags16, qvec, dc_part, d2_part, dvec, red_tmp, hub_part,
        hub_sum, hub_part4, hub_sum4, end;
    int dc_rows, d2_rows;
};
BwdLayout bwd_layout(const HeadLayout &h, int64_t N, int p, int T, int S) {
    BwdLayout b;
    Carver c(h.end);
    // partial rows: the mask/seed kernel, every reversed round, and the action-node fix-up
    // (a reversed round keeps a compensated pair of rows per workgroup: kBwdRoundRows = 2 * kBwdGrid)
    b.dc_rows = kBwdHeadGrid + (T - 1) * kBwdRoundRows + (T >= 2 ? S * kFixSplit : 0);
    b.d2_rows = (T - 1) * kBwdRoundRows + (T >= 2 ? S * kFixSplit : 0);
    const size_t width = (size_t)(3 * p > p * p ? 3 * p : p * p);
    const size_t segs = (size_t)(b.dc_rows + 63) / 64;
    b.dg = c.take(sizeof(float) * (size_t)S * p);
    b.da = c.take(sizeof(float) * (size_t)S * p);
    b.glo = c.take(sizeof(int32_t) * S);
    b.ghi = c.take(sizeof(int32_t) * S);
    b.head_part = c.take(sizeof(float) * (size_t)S * (2 * p + 2 * p * p + 1));
    b.dz0 = c.take(T >= 3 ? sizeof(float) * (size_t)N * S * p : 0);
    // (in node mode the last two reversed rounds run as one, so dz^2 is never stored)
    b.dz1 = c.take((T >= 5 || (T == 4 && S % 16 != 0)) ? sizeof(float) * (size_t)N * S * p : 0);
    b.maskT = c.take(T >= 2 ? sizeof(unsigned long long) * (size_t)N * S : 0);
    b.rec = c.take(sizeof(float) * (size_t)N * nodeinfo_stride(S));
    b.flags16 = c.take(S % 16 == 0 ? sizeof(unsigned short) * (size_t)N * (S / 16) : 0);
    b.qvec = c.take(sizeof(float) * 2 * p);
    b.dc_part = c.take(sizeof(float) * (size_t)b.dc_rows * 3 * p);
    b.d2_part = c.take(sizeof(float) * (size_t)b.d2_rows * p * p);
    b.dvec = c.take(sizeof(float) * 3 * p);
    b.red_tmp = c.take(sizeof(float) * segs * width);
    b.hub_part = c.take(sizeof(float) * (size_t)h.max_segs * S * p);
    b.hub_sum = c.take(sizeof(float) * (size_t)h.max_hubs * S * p);
    // the scalar form of the last reversed round keeps four sums per long row
    const size_t four = T >= 3 ? 4 : 0;
    b.hub_part4 = c.take(sizeof(float) * (size_t)h.max_segs * S * p * four);
    b.hub_sum4 = c.take(sizeof(float) * (size_t)h.max_hubs * S * p * four);
    b.end = c.off;
    return b;
}

template <class T>
T *at(void *ws, size_t off) {
    return reinterpret_cast<T *>(static_cast<char *>(ws) + off);
}

bool p_supported(int p) { return p == 32 || p == 64; }

}  // namespace

// ---- scratch of s2v_select_topk_noalloc: device memory the library owns, so that the call allocates nothing ----
// Layout for the largest supported call (N = S2V_NOALLOC_MAX_NODES, k = S2V_NOALLOC_MAX_K); a smaller call uses
// the front part of every piece.
namespace {
struct NoallocLayout {
    size_t chunk_begin, chunk_end, graph_chunk_off, part_val, part_idx, hist, state, blk, keys0, keys1, ids0, ids1,
        sort_cnt, end;
};
constexpr NoallocLayout noalloc_layout() {
    constexpr size_t n = S2V_NOALLOC_MAX_NODES, k = S2V_NOALLOC_MAX_K;
    constexpr size_t chunks = (n + kChunkNodes - 1) / kChunkNodes;
    NoallocLayout l{};
    size_t off = 0;
    auto take = [&off](size_t bytes) { const size_t at = off; off = align_up(off + bytes); return at; };
    l.chunk_begin = take(sizeof(int32_t) * chunks);
    l.chunk_end = take(sizeof(int32_t) * chunks);
    l.graph_chunk_off = take(sizeof(int32_t) * 2);
    l.part_val = take(sizeof(float) * chunks * kSmallK);
    l.part_idx = take(sizeof(int32_t) * chunks * kSmallK);
    l.hist = take(sizeof(uint32_t) * 4 * 256);
    l.state = take(sizeof(uint32_t) * 16);
    l.blk = take(sizeof(uint32_t) * 4 * ((n + kScanBlock - 1) / kScanBlock));
    l.keys0 = take(sizeof(uint32_t) * k);
    l.keys1 = take(sizeof(uint32_t) * k);
    l.ids0 = take(sizeof(int32_t) * k);
    l.ids1 = take(sizeof(int32_t) * k);
    l.sort_cnt = take(sizeof(uint32_t) * 256 * ((k + kSortTile - 1) / kSortTile));
    l.end = off;
    return l;
}
constexpr size_t kNoallocScratchBytes = (size_t)5 << 20;   // 5 MiB per GPU, held until the process ends
static_assert(noalloc_layout().end <= kNoallocScratchBytes, "scratch array too small for the largest call");
}  // namespace

// In host code this name is only a handle for hipGetSymbolAddress; kernels and copies get the address that call returns.
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU this process has used
}  // namespace

struct ProfSpan {
    hipEvent_t start, stop;
    int kind;
};

struct s2v_ctx {
    hipStream_t stream;
    int32_t last_hip;
    size_t max_lds_per_block = 0;  // of the device that was current in s2v_create
    int device = -1;               // the device that was current in s2v_create
    void *noalloc_scratch = nullptr;   // that device's copy of the library-owned scratch array
    std::vector<Prepared> prepared;
    // Embedding matrices of at least this many bytes ([N][S][p] floats, S a multiple of 16) have the rounds
    // that read them visit their rows state by state instead of node by node: one state's rows then fit the
    // last-level cache where all states' rows do not.  Measured on scale-free graphs of average degree 16
    // with S = 16, p = 64: 2.39 against 2.63 ms per round for a 1 GB matrix (node by node is faster),
    // 5.62 against 5.16 ms at 2 GB, 12.3 against 11.2 ms at 4 GB.  The two orders add the neighbours in a
    // different sequence, so their results differ in the last float32 bits.
    // s2v_set_sliced_min_bytes overrides the default.
    size_t sliced_min_bytes = (size_t)3 << 29;
    int32_t single_launch = S2V_SINGLE_LAUNCH_AUTO;   // s2v_set_single_launch
    // optional timing of the two gather kernels (s2v_profile_begin / s2v_profile_end)
    bool profiling = false;
    std::vector<ProfSpan> spans;   // pre-created event pairs
    size_t spans_used = 0;
};

namespace {

int32_t hip_fail(s2v_ctx *ctx, hipError_t e) {
    ctx->last_hip = (int32_t)e;
    return S2V_ERR_HIP;
}

#define S2V_TRY(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return hip_fail(ctx, e_); \
    } while (0)

// Brackets one kernel launch with events on the context's stream while profiling is on.
struct SpanGuard {
    s2v_ctx *ctx;
    ProfSpan *span = nullptr;
    SpanGuard(s2v_ctx *c, int kind) : ctx(c) {
        if (c->profiling && c->spans_used < c->spans.size()) {
            span = &c->spans[c->spans_used++];
            span->kind = kind;
            (void)hipEventRecord(span->start, c->stream);
        }
    }
    ~SpanGuard() {
        if (span) (void)hipEventRecord(span->stop, ctx->stream);
    }
};

int32_t check_graph(const s2v_graph *g) {
    if (!g) return S2V_ERR_INVALID_ARG;
    if (g->n_nodes < 0 || g->nnz < 0 || g->n_graphs < 1) return S2V_ERR_INVALID_ARG;
    if (g->nnz >= ((int64_t)1 << 31)) return S2V_ERR_UNSUPPORTED;
    if (!g->rowptr) return S2V_ERR_INVALID_ARG;
    if (g->nnz > 0 && !g->colidx) return S2V_ERR_INVALID_ARG;
    if (g->n_graphs > 1 && !g->graph_off) return S2V_ERR_INVALID_ARG;
    return S2V_OK;
}

int32_t check_params(const s2v_params *t) {
    if (!t) return S2V_ERR_INVALID_ARG;
    if (!p_supported(t->p)) return S2V_ERR_UNSUPPORTED;
    if (!t->theta1 || !t->theta2 || !t->theta3 || !t->theta4 || !t->theta5 || !t->theta6 || !t->theta7)
        return S2V_ERR_INVALID_ARG;
    return S2V_OK;
}

int32_t check_ws(const void *ws) {
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return S2V_ERR_INVALID_ARG;
    return S2V_OK;
}

// One past the last live entry of every row: the caller's row_end, or rowptr shifted by one.
const int32_t *row_end_of(const s2v_graph *g) { return g->row_end ? g->row_end : g->rowptr + 1; }

const Prepared *find_prepared(const s2v_ctx *ctx, const s2v_graph *g, const void *ws) {
    for (const Prepared &pr : ctx->prepared)
        if (pr.ws == ws && pr.rowptr == g->rowptr && pr.colidx == g->colidx && pr.w == g->w && pr.N == g->n_nodes &&
            pr.nnz == g->nnz && pr.G == g->n_graphs)
            return &pr;
    return nullptr;
}

HubTable hub_table(void *ws, const HeadLayout &h, const Prepared &pr) {
    HubTable ht;
    ht.n_hubs = pr.n_hubs;
    ht.n_segs = pr.n_segs;
    ht.hub_rows = at<int32_t>(ws, h.hub_rows);
    ht.hub_of = at<int32_t>(ws, h.hub_of);
    ht.fold = 0;
    ht.hub_seg_off = at<int32_t>(ws, h.hub_seg_off);
    ht.seg_row = at<int32_t>(ws, h.seg_row);
    ht.seg_begin = at<int32_t>(ws, h.seg_begin);
    ht.seg_end = at<int32_t>(ws, h.seg_end);
    return ht;
}

ChunkTable chunk_table(void *ws, const HeadLayout &h, const Prepared &pr) {
    ChunkTable ct;
    ct.n_chunks = pr.n_chunks;
    ct.chunk_begin = at<int32_t>(ws, h.chunk_begin);
    ct.chunk_end = at<int32_t>(ws, h.chunk_end);
    ct.graph_chunk_off = at<int32_t>(ws, h.graph_chunk_off);
    return ct;
}

}  // namespace

extern "C" {

const char *s2v_status_str(int32_t status) {
    switch (status) {
        case S2V_OK: return "ok";
        case S2V_ERR_INVALID_ARG: return "invalid argument";
        case S2V_ERR_UNSUPPORTED: return "unsupported configuration";
        case S2V_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case S2V_ERR_HIP: return "HIP runtime error";
        case S2V_ERR_NO_DEVICE: return "no usable GPU";
        case S2V_ERR_NOT_PREPARED: return "graph not prepared with this workspace";
        case S2V_ERR_TOO_LARGE: return "size beyond the fixed maximum of an entry point that allocates nothing";
        default: return "unknown status";
    }
}

int32_t s2v_create(void *hip_stream, s2v_ctx **out) {
    if (!out) return S2V_ERR_INVALID_ARG;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return S2V_ERR_NO_DEVICE;
    }
    s2v_ctx *ctx = new (std::nothrow) s2v_ctx;
    if (!ctx) return S2V_ERR_INVALID_ARG;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->last_hip = 0;
    // this device's copy of the scratch array of s2v_select_topk_noalloc, looked up once per device
    // (the symbol is named here, in a function with external linkage: the device-side compilation keeps a
    //  file-scope device variable visible to the runtime only when such a function refers to it)
    if (hipGetDevice(&ctx->device) == hipSuccess) {
        int lds = 0;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, ctx->device) == hipSuccess && lds > 0)
            ctx->max_lds_per_block = (size_t)lds;
        else
            (void)hipGetLastError();
    }
    if (ctx->device >= 0 && ctx->device < kMaxDevices) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[ctx->device]) {
            void *ptr = nullptr;
            const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e == hipSuccess) g_scratch_ptr[ctx->device] = ptr;
            else ctx->last_hip = (int32_t)e;   // only s2v_select_topk_noalloc is affected
        }
        ctx->noalloc_scratch = g_scratch_ptr[ctx->device];
    } else {
        (void)hipGetLastError();
    }
    *out = ctx;
    return S2V_OK;
}

static void drop_spans(s2v_ctx *ctx) {
    for (ProfSpan &sp : ctx->spans) {
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    ctx->spans.clear();
    ctx->spans_used = 0;
    ctx->profiling = false;
}

int32_t s2v_destroy(s2v_ctx *ctx) {
    if (ctx) drop_spans(ctx);
    delete ctx;
    return S2V_OK;
}

int32_t s2v_profile_begin(s2v_ctx *ctx, int32_t max_launches) {
    if (!ctx || max_launches < 1) return S2V_ERR_INVALID_ARG;
    drop_spans(ctx);
    ctx->spans.reserve(max_launches);
    for (int i = 0; i < max_launches; ++i) {
        ProfSpan sp;
        sp.kind = 0;
        S2V_TRY(hipEventCreate(&sp.start));
        hipError_t e = hipEventCreate(&sp.stop);
        if (e != hipSuccess) {
            (void)hipEventDestroy(sp.start);
            return hip_fail(ctx, e);
        }
        ctx->spans.push_back(sp);
    }
    ctx->profiling = true;
    return S2V_OK;
}

int32_t s2v_profile_end(s2v_ctx *ctx, int32_t *n_launches, float *total_ms) {
    if (!ctx || !n_launches || !total_ms) return S2V_ERR_INVALID_ARG;
    for (int k = 0; k < S2V_PROFILE_KINDS; ++k) {
        n_launches[k] = 0;
        total_ms[k] = 0.f;
    }
    ctx->profiling = false;
    S2V_TRY(hipStreamSynchronize(ctx->stream));
    for (size_t i = 0; i < ctx->spans_used; ++i) {
        float ms = 0.f;
        S2V_TRY(hipEventElapsedTime(&ms, ctx->spans[i].start, ctx->spans[i].stop));
        const int k = ctx->spans[i].kind;
        n_launches[k] += 1;
        total_ms[k] += ms;
    }
    drop_spans(ctx);
    return S2V_OK;
}

int32_t s2v_last_hip_error(const s2v_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

int32_t s2v_set_sliced_min_bytes(s2v_ctx *ctx, size_t bytes) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    ctx->sliced_min_bytes = bytes;
    return S2V_OK;
}

int32_t s2v_set_single_launch(s2v_ctx *ctx, int32_t mode) {
    if (!ctx || mode < S2V_SINGLE_LAUNCH_AUTO || mode > S2V_SINGLE_LAUNCH_NEVER) return S2V_ERR_INVALID_ARG;
    ctx->single_launch = mode;
    return S2V_OK;
}

int32_t s2v_stream_read(s2v_ctx *ctx, const void *src, size_t bytes, float *out) {
    if (!ctx || !src || !out || (bytes & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u)) return S2V_ERR_INVALID_ARG;
    S2V_TRY(launch_stream_read(ctx->stream, src, bytes, out));
    return S2V_OK;
}

int32_t s2v_workspace_bytes(s2v_ctx *ctx, const s2v_graph *g, int32_t p, int32_t T, int32_t S, int32_t k_max,
                            int32_t training, size_t *out) {
    if (!g || !out || g->n_nodes < 0 || g->n_graphs < 1 || T < 1 || S < 1 || k_max < 0) return S2V_ERR_INVALID_ARG;
    if (!p_supported(p)) return S2V_ERR_UNSUPPORTED;
    if ((int64_t)g->n_nodes * S >= ((int64_t)1 << 31)) return S2V_ERR_UNSUPPORTED;
    int hubs = 0, segs = 0;
    if (ctx && g->rowptr && g->n_nodes > 0) {
        // exact hub counts from the graph itself (reads rowptr back: waits for the stream)
        std::vector<int32_t> rp((size_t)g->n_nodes + 1);
        S2V_TRY(hipMemcpyAsync(rp.data(), g->rowptr, sizeof(int32_t) * rp.size(), hipMemcpyDeviceToHost, ctx->stream));
        S2V_TRY(hipStreamSynchronize(ctx->stream));
        hub_counts(rp, &hubs, &segs);
    } else {
        hub_bounds(g->nnz, &hubs, &segs);
    }
    const HeadLayout h = head_layout(g->n_nodes, g->n_graphs, hubs, segs);
    size_t need = fwd_layout(h, g->n_nodes, p, S, true).end;
    const size_t q_end = q_layout(h, S, g->n_graphs).end;
    const size_t s_end = sel_layout(h, g->n_nodes, k_max > 0 ? k_max : 1).end;
    if (q_end > need) need = q_end;
    if (s_end > need) need = s_end;
    const size_t sm_end = align_up(h.end) + align_up(sizeof(float) * (size_t)g->n_nodes * p);   // s2v_policy_select
    if (sm_end > need) need = sm_end;
    const size_t t_end = align_up(align_up(h.end) + align_up(sizeof(float) * (size_t)S * h.max_chunks) +
                                  sizeof(int32_t) * (size_t)S * h.max_chunks);
    if (t_end > need) need = t_end;
    if (training) {
        const size_t b_end = bwd_layout(h, g->n_nodes, p, T, S).end;
        if (b_end > need) need = b_end;
        // s2v_loss_grad keeps the forward pass's pieces behind the backward pass's
        const size_t fb_end = fwd_layout(h, g->n_nodes, p, S, false, b_end).end;
        if (fb_end > need) need = fb_end;
    }
    *out = need;
    return S2V_OK;
}

int32_t s2v_graph_prepare(s2v_ctx *ctx, const s2v_graph *g, void *ws, size_t ws_bytes) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_graph(g);
    if (rc != S2V_OK) return rc;
    rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    const int32_t N = g->n_nodes, G = g->n_graphs;
    // Long rows and their segments.  A kernel counts them and checks the row pointers; only a graph that has
    // long rows gets its row pointers copied to the host, where the (ordered) tables are built.
    // (the first words of the workspace serve as the kernel's output: the head is written after this)
    if (ws_bytes < 256) return S2V_ERR_WORKSPACE_TOO_SMALL;
    int32_t row_stats[3] = {0, 0, 0};
    if (N > 0) {
        S2V_TRY(launch_zero_i32(ctx->stream, 4, static_cast<int32_t *>(ws)));
        S2V_TRY(launch_row_stats(ctx->stream, N, (long)g->nnz, g->rowptr, static_cast<int32_t *>(ws)));
        S2V_TRY(hipMemcpyAsync(row_stats, ws, sizeof(row_stats), hipMemcpyDeviceToHost, ctx->stream));
        S2V_TRY(hipStreamSynchronize(ctx->stream));
        if (row_stats[2] != 0) return S2V_ERR_INVALID_ARG;
    } else if (g->nnz != 0) {
        return S2V_ERR_INVALID_ARG;
    }
    // Hub rows are those that are long in STORAGE: rows only shrink afterwards, and the kernels test
    // the live length, so a stored-long row that became short is simply handled as an ordinary row.
    const int n_hubs = row_stats[0], n_segs = row_stats[1];
    std::vector<int32_t> rp;
    if (n_hubs > 0) {
        rp.resize((size_t)N + 1);
        S2V_TRY(hipMemcpyAsync(rp.data(), g->rowptr, sizeof(int32_t) * ((size_t)N + 1), hipMemcpyDeviceToHost, ctx->stream));
        S2V_TRY(hipStreamSynchronize(ctx->stream));
    }
    const HeadLayout h = head_layout(N, G, n_hubs, n_segs);
    if (ws_bytes < h.end) return S2V_ERR_WORKSPACE_TOO_SMALL;

    // graph offsets to the host: the chunk table is built here, once per graph
    std::vector<int32_t> off(G + 1);
    if (G > 1) {
        S2V_TRY(hipMemcpyAsync(off.data(), g->graph_off, sizeof(int32_t) * (G + 1), hipMemcpyDeviceToHost, ctx->stream));
        S2V_TRY(hipStreamSynchronize(ctx->stream));
        if (off[0] != 0 || off[G] != N) return S2V_ERR_INVALID_ARG;
        for (int b = 0; b < G; ++b)
            if (off[b + 1] < off[b]) return S2V_ERR_INVALID_ARG;
    } else {
        off[0] = 0;
        off[1] = N;
    }
    std::vector<int32_t> cb, ce, gco(G + 1);
    for (int b = 0; b < G; ++b) {
        gco[b] = (int32_t)cb.size();
        for (int32_t v = off[b]; v < off[b + 1]; v += kChunkNodes) {
            cb.push_back(v);
            ce.push_back(v + kChunkNodes < off[b + 1] ? v + kChunkNodes : off[b + 1]);
        }
    }
    gco[G] = (int32_t)cb.size();
    const int n_chunks = (int)cb.size();
    if (n_chunks > h.max_chunks) return S2V_ERR_INVALID_ARG;
    if (n_chunks > 0) {
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.chunk_begin), cb.data(), sizeof(int32_t) * n_chunks, hipMemcpyHostToDevice, ctx->stream));
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.chunk_end), ce.data(), sizeof(int32_t) * n_chunks, hipMemcpyHostToDevice, ctx->stream));
    }
    S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.graph_chunk_off), gco.data(), sizeof(int32_t) * (G + 1), hipMemcpyHostToDevice, ctx->stream));
    std::vector<int32_t> hub_rows, hub_seg_off, seg_row, seg_begin, seg_end;
    for (int32_t v = 0; n_hubs > 0 && v < N; ++v) {
        if (rp[v + 1] - rp[v] > kHubDegree) {
            hub_rows.push_back(v);
            hub_seg_off.push_back((int32_t)seg_begin.size());
            for (int32_t b = rp[v]; b < rp[v + 1]; b += kHubSegment) {
                seg_row.push_back(v);
                seg_begin.push_back(b);
                seg_end.push_back(b + kHubSegment < rp[v + 1] ? b + kHubSegment : rp[v + 1]);
            }
        }
    }
    hub_seg_off.push_back((int32_t)seg_begin.size());
    int32_t max_hub_segs = 0;
    for (size_t i = 0; i + 1 < hub_seg_off.size(); ++i)
        if (hub_seg_off[i + 1] - hub_seg_off[i] > max_hub_segs) max_hub_segs = hub_seg_off[i + 1] - hub_seg_off[i];
    if ((int)hub_rows.size() != n_hubs || (int)seg_begin.size() != n_segs) return S2V_ERR_INVALID_ARG;
    if (n_hubs > 0) {
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.hub_rows), hub_rows.data(), sizeof(int32_t) * n_hubs, hipMemcpyHostToDevice, ctx->stream));
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.hub_seg_off), hub_seg_off.data(), sizeof(int32_t) * (n_hubs + 1), hipMemcpyHostToDevice, ctx->stream));
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.seg_row), seg_row.data(), sizeof(int32_t) * n_segs, hipMemcpyHostToDevice, ctx->stream));
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.seg_begin), seg_begin.data(), sizeof(int32_t) * n_segs, hipMemcpyHostToDevice, ctx->stream));
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.seg_end), seg_end.data(), sizeof(int32_t) * n_segs, hipMemcpyHostToDevice, ctx->stream));
    }
    // per node its index among the long rows (any value for other nodes): the round kernels look it up
    std::vector<int32_t> hub_of;
    if (n_hubs > 0) {
        hub_of.assign((size_t)N, -1);
        for (int i = 0; i < n_hubs; ++i) hub_of[hub_rows[i]] = i;
        S2V_TRY(hipMemcpyAsync(at<int32_t>(ws, h.hub_of), hub_of.data(), sizeof(int32_t) * (size_t)N, hipMemcpyHostToDevice, ctx->stream));
    }
    S2V_TRY(launch_zero_i32(ctx->stream, N, at<int32_t>(ws, h.touched)));
    // whether any weight is negative: a word beside the update counter serves as the flag
    int32_t *neg_flag = at<int32_t>(ws, h.epoch) + 1;
    int32_t has_neg = 0;
    S2V_TRY(launch_zero_i32(ctx->stream, 2, at<int32_t>(ws, h.epoch)));
    S2V_TRY(launch_prepare_s(ctx->stream, N, g->rowptr, row_end_of(g), g->w, at<float>(ws, h.s_pos), at<float>(ws, h.s_neg),
                             neg_flag));
    S2V_TRY(launch_prepare_nbr(ctx->stream, N, g->rowptr, row_end_of(g), g->colidx, g->w, at<float>(ws, h.s_pos),
                               at<float>(ws, h.nbr_sp), at<float>(ws, h.nbr_spw)));
    S2V_TRY(hipMemcpyAsync(&has_neg, neg_flag, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    S2V_TRY(hipStreamSynchronize(ctx->stream));  // the host vectors above must outlive the copies

    int32_t max_graph_nodes = 0;
    for (int b = 0; b < G; ++b)
        if (off[b + 1] - off[b] > max_graph_nodes) max_graph_nodes = off[b + 1] - off[b];
    Prepared pr{ws, g->rowptr, g->colidx, g->w, N, g->nnz, G, n_chunks, n_hubs, n_segs, has_neg != 0, max_graph_nodes, max_hub_segs};
    for (Prepared &old : ctx->prepared)
        if (old.ws == ws) { old = pr; return S2V_OK; }
    ctx->prepared.push_back(pr);
    return S2V_OK;
}

// Alg. 1 for all states.  q_node != NULL asks the last round to leave the node term of Eq. 2 in
// q_node [S][N] as well; *q_node_done says whether it did (only the row-mode round kernel can).
// fused != NULL: the backward pass follows in the same call (s2v_loss_grad, which has checked that the
// shape allows it).  The workspace pieces then start at fused->layout_start, round 1 is not written (no
// reversed round reads it) and the last round leaves relu-mask words, the action nodes' rows and the
// graph sums instead of mu^T.
struct FusedTrain {
    size_t layout_start;
    unsigned long long *mask_words;
    const int32_t *action;
};
// defer != NULL (one state, one graph, T >= 2: the last round leaves per-workgroup partial rows of the graph sum):
// the second stage of the graph sum is left to the caller, who gets the partial rows here.
struct DeferredGsum {
    const float *gpart;
    int rows;
};
static int32_t embed_fwd_impl(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                              int32_t S, float *mu_out, float *mu_saved, float *gsum, void *ws, size_t ws_bytes,
                              float *q_node, bool *q_node_done, const FusedTrain *fused = nullptr,
                              DeferredGsum *defer = nullptr) {
    if (q_node_done) *q_node_done = false;
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_graph(g);
    if (rc != S2V_OK) return rc;
    rc = check_params(params);
    if (rc != S2V_OK) return rc;
    rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    if (T < 1 || S < 1) return S2V_ERR_INVALID_ARG;
    const int32_t N = g->n_nodes, G = g->n_graphs, p = params->p;
    if (N > 0 && !mu_out && !mu_saved) return S2V_ERR_INVALID_ARG;
    if (N > 0 && !x) return S2V_ERR_INVALID_ARG;
    if ((int64_t)N * S >= ((int64_t)1 << 31)) return S2V_ERR_UNSUPPORTED;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    const bool need_tmp = !mu_saved && T >= 3;  // round 2 reads no embedding from memory
    const FwdLayout f = fwd_layout(h, N, p, S, need_tmp, fused ? fused->layout_start : 0);
    if (ws_bytes < f.end) return S2V_ERR_WORKSPACE_TOO_SMALL;

    hipStream_t st = ctx->stream;
    const float *s_pos = at<float>(ws, h.s_pos), *s_neg = at<float>(ws, h.s_neg);
    // (inside s2v_mvc_inference: records and q+- live in the head and are kept current by the state update)
    const bool keep = pr->rec_keep && S == 1 && !g->state_residual && !fused;
    float *qvec = keep ? at<float>(ws, h.qkeep) : at<float>(ws, f.qvec);
    float *tmp = at<float>(ws, f.tmp);
    const size_t nsp = (size_t)N * S * p;
    // destination of round t (1-based): the saved slot, or ping-pong so that round T lands in mu_out
    auto dest = [&](int t) -> float * {
        if (mu_saved) return mu_saved + (size_t)(t - 1) * nsp;
        return ((T - t) % 2 == 0) ? mu_out : tmp;
    };
    // Round 1 has no neighbour term (mu^0 = 0).  Its result is written out only when somebody reads
    // it from memory: the caller (mu_saved) or, when T == 1, the output itself.  Round 2 recomputes
    // the neighbours' round-1 rows from the per-node scalars instead of gathering them.
    float *info = keep ? at<float>(ws, h.rec) : at<float>(ws, f.info);
    float *gpart = at<float>(ws, f.gpart);
    const HubTable ht = hub_table(ws, h, *pr);
    // per-(node, state) scalar records; with per-state residual graphs they hold each state's own edge sums
    const float *x_res = g->state_residual ? x : nullptr;
    const float *wagg = g->weighted_sum ? g->w : nullptr;   // NULL weights mean w = 1: the plain sum
    // S = 1 without negative weights: round 2 reads a 4-byte table first (see gather_tile_mu1_single)
    float *compact = (S == 1 && !pr->has_neg) ? info + (size_t)N * 4 : nullptr;
    // ... and on a graph whose rows do not shrink (the per-row totals of s_pos date from s2v_graph_prepare)
    // flag bits come first and the table is not needed at all (see gather_tile_mu1_single, mode 2)
    // (for S a multiple of 16 the same with one 16-bit flag word per node and block of 16 states)
    const bool by_bits = (S == 1 || S % 16 == 0) && !pr->has_neg && !g->row_end && !x_res && T >= 2;
    unsigned long long *xbits = by_bits ? at<unsigned long long>(ws, f.xbits) : nullptr;
    if (by_bits) compact = nullptr;
    if (x_res) {
        S2V_TRY(launch_qvec(st, p, params->theta3, params->theta4, qvec));
        S2V_TRY(launch_stateinfo_residual(st, N, S, ht, g->rowptr, row_end_of(g), g->colidx, g->w, x, info, compact));
    } else if (!(keep && pr->rec_current)) {
        // (q+- = theta3 relu(+-theta4) comes out of the same launch as the records)
        if (keep) pr->rec_current = true;
        S2V_TRY(launch_nodeinfo(st, N, S, x, s_pos, s_neg, info, compact,
                                by_bits ? at<float>(ws, wagg ? h.nbr_spw : h.nbr_sp) : nullptr, xbits, p, params->theta3,
                                params->theta4, qvec));
    }
    NodeInfo ninfo = make_nodeinfo(info, S, x_res != nullptr);
    ninfo.compact = compact;
    if (S == 1) ninfo.xbits = reinterpret_cast<const unsigned *>(xbits);
    else ninfo.flags16 = reinterpret_cast<const unsigned short *>(xbits);
    if ((mu_saved && !fused) || T == 1)
        S2V_TRY(launch_round1(st, p, N, S, ninfo, x_res, T == 1, params->theta1, qvec, dest(1)));
    const bool fuse_gsum = gsum && (S == 1 || S == 16) && G == 1 && T >= 2 && N > 0;
    const bool fuse_q = q_node && T >= 2 && N > 0 && round_fuses_qnode(S, T);
    float *hub_part = at<float>(ws, f.hub_part), *hub_sum = at<float>(ws, f.hub_sum);
    const bool by_state = S > 1 && nsp * sizeof(float) >= ctx->sliced_min_bytes;
    // one state and at most four segments per long row: no combine pass, the round kernel adds the segments
    HubTable htf = ht;
    htf.fold = (S == 1 && pr->n_segs != pr->n_hubs && pr->max_hub_segs <= 4) ? 1 : 0;
    for (int t = 2; t <= T; ++t) {
        QHead qh{params->theta5, params->theta7, (fuse_q && t == T) ? q_node : nullptr};
        const float *src = t == 2 ? nullptr : dest(t - 1);
        S2V_TRY(launch_hub_sums(st, p, S, htf, row_end_of(g), g->colidx, wagg, src, ninfo, params->theta1, qvec, nullptr, hub_part, hub_sum));
        SpanGuard span(ctx, (qh.q || (fused && t == T)) ? S2V_PROFILE_FWD_ROUND_Q
                                                            : (t == 2 ? S2V_PROFILE_FWD_ROUND2 : S2V_PROFILE_FWD_ROUND));
        S2V_TRY(launch_round(st, p, N, S, g->rowptr, row_end_of(g), g->colidx, wagg, src, dest(t), ninfo, params->theta1,
                             params->theta2, qvec, t == 2, (fuse_gsum && t == T) ? gpart : nullptr, htf,
                             htf.fold ? hub_part : hub_sum, x_res, t == T, qh,
                             (fused && t == T) ? MaskOut{fused->mask_words, fused->action} : MaskOut{nullptr, nullptr},
                             by_state));
    }
    if (q_node_done) *q_node_done = fuse_q;
    float *muT = dest(T);
    if (mu_saved && mu_out && mu_out != muT && nsp > 0)
        S2V_TRY(hipMemcpyAsync(mu_out, muT, sizeof(float) * nsp, hipMemcpyDeviceToDevice, st));
    if (gsum) {
        if (fuse_gsum && defer) {
            defer->gpart = gpart;
            defer->rows = round_grid((long)N * S);
        } else if (fuse_gsum) {
            S2V_TRY(launch_gsum_from_round(st, p, S, round_grid((long)N * S), gpart, gsum));
        } else {
            const ChunkTable ct = chunk_table(ws, h, *pr);
            S2V_TRY(launch_gsum(st, p, N, S, G, ct, muT, gpart, gsum));
        }
    }
    return S2V_OK;
}

int32_t s2v_embed_fwd(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                      int32_t S, float *mu_out, float *mu_saved, float *gsum, void *ws, size_t ws_bytes) {
    return embed_fwd_impl(ctx, g, params, x, T, S, mu_out, mu_saved, gsum, ws, ws_bytes, nullptr, nullptr);
}

int32_t s2v_policy_eval(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                        int32_t S, float *mu_out, float *gsum, float *q, void *ws, size_t ws_bytes) {
    if (!gsum || (g && g->n_nodes > 0 && (!mu_out || !q))) return S2V_ERR_INVALID_ARG;
    bool q_node_done = false;
    int32_t rc = embed_fwd_impl(ctx, g, params, x, T, S, mu_out, nullptr, gsum, ws, ws_bytes, q, &q_node_done);
    if (rc != S2V_OK) return rc;
    if (!q_node_done) return s2v_q_score(ctx, g, params, mu_out, gsum, S, q, ws, ws_bytes);
    const int32_t N = g->n_nodes, G = g->n_graphs;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    const QLayout ql = q_layout(h, S, G);
    if (ws_bytes < ql.end) return S2V_ERR_WORKSPACE_TOO_SMALL;
    float *qa = at<float>(ws, ql.qa);
    S2V_TRY(launch_qa(ctx->stream, params->p, S, G, params->theta5, params->theta6, gsum, qa));
    S2V_TRY(launch_qfinish(ctx->stream, N, S, G, g->graph_off, qa, q));
    return S2V_OK;
}

// end != NULL (the inference loop): where the selection's last launch can also take the step's decisions and
// begin the state update it does, and *ended says so; otherwise the caller launches them.
static int32_t policy_select_impl(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x,
                                  const uint8_t *cand, int32_t T, int32_t k, float *mu_out, float *gsum, float *q,
                                  int32_t *idx, float *val, int32_t *count, void *ws, size_t ws_bytes,
                                  const StepEnd *end, bool *ended) {
    if (!ctx || !g || !params) return S2V_ERR_INVALID_ARG;
    if (k < 1 || !idx || !val || !count || !gsum) return S2V_ERR_INVALID_ARG;
    if (g->n_graphs > 1 && k > 1) return S2V_ERR_UNSUPPORTED;
    const Prepared *pr = check_ws(ws) == S2V_OK ? find_prepared(ctx, g, ws) : nullptr;
    // One launch for the whole step when every graph's embedding fits the LDS of a compute unit
    // (see small_kernels.hip); plain neighbour sum on the stored graph only.
    // One workgroup per graph uses one compute unit per graph, so it pays for batches, or for graphs small enough
    // that the launches of the general path cost more than the work (measured on scale-free graphs of 250-1000
    // nodes, 1 to 512 per batch: at 64 graphs and more it wins or ties at every size that fits; one graph of
    // 1000 nodes at p = 32 takes 78 us this way and 61 us as a chain of launches, one of 250 nodes at p = 64
    // 66 against 81 us).
    const bool small_pays = pr && ctx->single_launch != S2V_SINGLE_LAUNCH_NEVER &&
                            (ctx->single_launch == S2V_SINGLE_LAUNCH_ALWAYS || g->n_graphs >= 64 ||
                             (int64_t)pr->max_graph_nodes * params->p <= kSmallLdsFloats / 2 ||
                             (params->p <= 32 && g->n_graphs >= 4));
    const bool small = pr && small_pays && p_supported(params->p) && check_params(params) == S2V_OK && T >= 1 && g->n_nodes > 0 &&
                       (int64_t)pr->max_graph_nodes * params->p <= kSmallLdsFloats && k <= kSmallK &&
                       !g->weighted_sum && !g->state_residual && ctx->max_lds_per_block >= kSmallLdsBytes && x && mu_out &&
                       q;
    // One state of one graph with few workgroups in the last round: the tail of the evaluation (graph sum,
    // graph term of Eq. 2, q = graph term + node term) and the first stage of the selection share a launch.
    // Same device functions as the separate kernels: the results are those of the two calls bit for bit.
    const bool tail = !small && pr && g->n_graphs == 1 && T >= 2 && g->n_nodes > 0 && k <= kSmallK && x && mu_out && q &&
                      round_grid((long)g->n_nodes) <= kTailMaxRows && check_params(params) == S2V_OK;
    bool tail_fits = false;
    if (tail) {
        // the selection's partial results and the forward pass's partial rows both start behind the head of the
        // workspace; the fused kernel reads the one while it writes the other, so they must not overlap
        const HeadLayout h = head_layout(g->n_nodes, 1, pr->n_hubs, pr->n_segs);
        const SelLayout sl = sel_layout(h, g->n_nodes, k);
        const FwdLayout f = fwd_layout(h, g->n_nodes, params->p, 1, T >= 3);
        tail_fits = sl.hist <= f.gpart;
    }
    if (tail && tail_fits) {
        const int32_t N = g->n_nodes;
        const HeadLayout h = head_layout(N, 1, pr->n_hubs, pr->n_segs);
        const SelLayout sl = sel_layout(h, N, k);
        if (ws_bytes < sl.end) return S2V_ERR_WORKSPACE_TOO_SMALL;
        DeferredGsum dg{nullptr, 0};
        bool q_node_done = false;
        int32_t rc = embed_fwd_impl(ctx, g, params, x, T, 1, mu_out, nullptr, gsum, ws, ws_bytes, q, &q_node_done, nullptr, &dg);
        if (rc != S2V_OK) return rc;
        if (!q_node_done || !dg.gpart) return S2V_ERR_INVALID_ARG;   // (cannot happen for this shape)
        // (the partial rows live in the forward pass's part of the workspace, the selection's partial results
        //  in its own: sel_layout's first two pieces lie below the forward pass's gpart)
        SelectScratch sc{};
        sc.part_val = at<float>(ws, sl.part_val);
        sc.part_idx = at<int32_t>(ws, sl.part_idx);
        const ChunkTable ct = chunk_table(ws, h, *pr);
        SpanGuard span(ctx, S2V_PROFILE_SELECT);
        S2V_TRY(launch_tail_select(ctx->stream, params->p, dg.rows, k, dg.gpart, params->theta5, params->theta6, gsum, q, x,
                                   cand, ct, sc, idx, val, count, end));
        if (end) *ended = true;
        return S2V_OK;
    }
    if (!small) {
        int32_t rc = s2v_policy_eval(ctx, g, params, x, T, 1, mu_out, gsum, q, ws, ws_bytes);
        if (rc != S2V_OK) return rc;
        return s2v_select_topk(ctx, g, q, x, cand, k, idx, val, count, ws, ws_bytes);
    }
    const int32_t N = g->n_nodes, G = g->n_graphs, p = params->p;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    const size_t agg_off = align_up(h.end);
    if (ws_bytes < agg_off + sizeof(float) * (size_t)N * p) return S2V_ERR_WORKSPACE_TOO_SMALL;
    SmallPolicyArgs a;
    a.N = N; a.G = G; a.T = T; a.k = k;
    a.graph_off = G > 1 ? g->graph_off : nullptr;
    a.rowptr = g->rowptr; a.rowend = row_end_of(g); a.colidx = g->colidx;
    a.x = x; a.s_pos = at<float>(ws, h.s_pos); a.s_neg = at<float>(ws, h.s_neg);
    a.cand = cand;
    a.theta1 = params->theta1; a.theta2 = params->theta2; a.theta3 = params->theta3; a.theta4 = params->theta4;
    a.theta5 = params->theta5; a.theta6 = params->theta6; a.theta7 = params->theta7;
    a.agg = at<float>(ws, agg_off);
    a.mu_out = mu_out; a.gsum = gsum; a.q = q;
    a.idx = idx; a.val = val; a.count = count;
    SpanGuard span(ctx, S2V_PROFILE_SELECT);
    S2V_TRY(launch_small_policy(ctx->stream, p, a));
    return S2V_OK;
}

int32_t s2v_policy_select(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x,
                          const uint8_t *cand, int32_t T, int32_t k, float *mu_out, float *gsum, float *q, int32_t *idx,
                          float *val, int32_t *count, void *ws, size_t ws_bytes) {
    return policy_select_impl(ctx, g, params, x, cand, T, k, mu_out, gsum, q, idx, val, count, ws, ws_bytes, nullptr,
                              nullptr);
}


int32_t s2v_q_score(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *mu,
                    const float *gsum, int32_t S, float *q, void *ws, size_t ws_bytes) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_graph(g);
    if (rc != S2V_OK) return rc;
    rc = check_params(params);
    if (rc != S2V_OK) return rc;
    rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    if (S < 1 || !gsum) return S2V_ERR_INVALID_ARG;
    const int32_t N = g->n_nodes, G = g->n_graphs, p = params->p;
    if (N > 0 && (!mu || !q)) return S2V_ERR_INVALID_ARG;
    if ((int64_t)N * S >= ((int64_t)1 << 31)) return S2V_ERR_UNSUPPORTED;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    const QLayout ql = q_layout(h, S, G);
    if (ws_bytes < ql.end) return S2V_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = ctx->stream;
    float *qa = at<float>(ws, ql.qa);
    S2V_TRY(launch_qa(st, p, S, G, params->theta5, params->theta6, gsum, qa));
    S2V_TRY(launch_qnode(st, p, N, S, G, g->graph_off, params->theta5, params->theta7, mu, qa, q));
    return S2V_OK;
}

int32_t s2v_select_topk(s2v_ctx *ctx, const s2v_graph *g, const float *q, const float *x, const uint8_t *cand,
                        int32_t k, int32_t *idx, float *val, int32_t *count, void *ws, size_t ws_bytes) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_graph(g);
    if (rc != S2V_OK) return rc;
    rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    if (k < 1 || !idx || !val || !count) return S2V_ERR_INVALID_ARG;
    const int32_t N = g->n_nodes, G = g->n_graphs;
    if (N > 0 && (!q || (!x && !cand))) return S2V_ERR_INVALID_ARG;
    if (G > 1 && k > 1) return S2V_ERR_UNSUPPORTED;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    const SelLayout sl = sel_layout(h, N, k);
    if (ws_bytes < sl.end) return S2V_ERR_WORKSPACE_TOO_SMALL;
    SelectScratch sc;
    sc.part_val = at<float>(ws, sl.part_val);
    sc.part_idx = at<int32_t>(ws, sl.part_idx);
    sc.hist = at<uint32_t>(ws, sl.hist);
    sc.state = at<uint32_t>(ws, sl.state);
    sc.blk = at<uint32_t>(ws, sl.blk);
    sc.keys[0] = at<uint32_t>(ws, sl.keys0);
    sc.keys[1] = at<uint32_t>(ws, sl.keys1);
    sc.ids[0] = at<int32_t>(ws, sl.ids0);
    sc.ids[1] = at<int32_t>(ws, sl.ids1);
    sc.sort_cnt = at<uint32_t>(ws, sl.sort_cnt);
    SpanGuard span(ctx, S2V_PROFILE_SELECT);   // the whole chain of selection kernels as one span
    if (k == 1) {
        const ChunkTable ct = chunk_table(ws, h, *pr);
        S2V_TRY(launch_argmax(ctx->stream, N, G, ct, q, x, cand, sc, idx, val, count));
    } else if (k <= kSmallK) {
        const ChunkTable ct = chunk_table(ws, h, *pr);
        S2V_TRY(launch_smallk(ctx->stream, ct, q, x, cand, k, sc, idx, val, count));
    } else {
        S2V_TRY(launch_topk(ctx->stream, N, q, x, cand, k, sc, idx, val, count));
    }
    return S2V_OK;
}

int32_t s2v_select_topk_noalloc(s2v_ctx *ctx, int32_t n_nodes, const float *q, const float *x, const uint8_t *cand,
                                int32_t k, int32_t *idx, float *val, int32_t *count) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    if (n_nodes < 0 || k < 1 || !idx || !val || !count) return S2V_ERR_INVALID_ARG;
    if (n_nodes > 0 && (!q || (!x && !cand))) return S2V_ERR_INVALID_ARG;
    if (n_nodes > S2V_NOALLOC_MAX_NODES || k > S2V_NOALLOC_MAX_K) return S2V_ERR_TOO_LARGE;
    if (!ctx->noalloc_scratch) return S2V_ERR_HIP;   // the lookup in s2v_create failed (see s2v_last_hip_error)
    constexpr NoallocLayout l = noalloc_layout();
    void *base = ctx->noalloc_scratch;   // the device address, never the array's name
    ChunkTable ct;
    ct.n_chunks = (n_nodes + kChunkNodes - 1) / kChunkNodes;
    ct.chunk_begin = at<int32_t>(base, l.chunk_begin);
    ct.chunk_end = at<int32_t>(base, l.chunk_end);
    ct.graph_chunk_off = at<int32_t>(base, l.graph_chunk_off);
    SelectScratch sc;
    sc.part_val = at<float>(base, l.part_val);
    sc.part_idx = at<int32_t>(base, l.part_idx);
    sc.hist = at<uint32_t>(base, l.hist);
    sc.state = at<uint32_t>(base, l.state);
    sc.blk = at<uint32_t>(base, l.blk);
    sc.keys[0] = at<uint32_t>(base, l.keys0);
    sc.keys[1] = at<uint32_t>(base, l.keys1);
    sc.ids[0] = at<int32_t>(base, l.ids0);
    sc.ids[1] = at<int32_t>(base, l.ids1);
    sc.sort_cnt = at<uint32_t>(base, l.sort_cnt);
    // Everything the kernels read from the scratch is written earlier in the same call (the chunk table here,
    // the histograms and the selection state by the chain's first kernel), so the previous call's contents
    // do not matter.
    if (k <= kSmallK) {
        S2V_TRY(launch_chunk_table_single(ctx->stream, n_nodes, ct.n_chunks, at<int32_t>(base, l.chunk_begin),
                                          at<int32_t>(base, l.chunk_end), at<int32_t>(base, l.graph_chunk_off)));
        if (k == 1) S2V_TRY(launch_argmax(ctx->stream, n_nodes, 1, ct, q, x, cand, sc, idx, val, count));
        else S2V_TRY(launch_smallk(ctx->stream, ct, q, x, cand, k, sc, idx, val, count));
    } else {
        S2V_TRY(launch_topk(ctx->stream, n_nodes, q, x, cand, k, sc, idx, val, count));
    }
    return S2V_OK;
}

// words_ready: the forward pass of the same call has left the relu-mask words of mu^T in the workspace
// (and of mu^T itself only the action nodes' rows), see FusedTrain.
static int32_t embed_bwd_impl(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                              int32_t S, const float *mu_saved, const float *gsum, const int32_t *action,
                              const float *target, float *loss, float *q_pred, s2v_params *grads, void *ws,
                              size_t ws_bytes, bool words_ready) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_graph(g);
    if (rc != S2V_OK) return rc;
    rc = check_params(params);
    if (rc != S2V_OK) return rc;
    rc = check_params(grads);
    if (rc != S2V_OK) return rc;
    rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    if (grads->p != params->p || T < 1 || S < 1) return S2V_ERR_INVALID_ARG;
    if (!x || !mu_saved || !gsum || !action || !target || !loss) return S2V_ERR_INVALID_ARG;
    const int32_t N = g->n_nodes, G = g->n_graphs, p = params->p;
    if (N < 1) return S2V_ERR_INVALID_ARG;  // an action node must exist
    if ((int64_t)N * S >= ((int64_t)1 << 31)) return S2V_ERR_UNSUPPORTED;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    const BwdLayout bl = bwd_layout(h, N, p, T, S);
    if (ws_bytes < bl.end) return S2V_ERR_WORKSPACE_TOO_SMALL;

    hipStream_t st = ctx->stream;
    const float *s_pos = at<float>(ws, h.s_pos), *s_neg = at<float>(ws, h.s_neg);
    BwdScratch sc;
    sc.dg = at<float>(ws, bl.dg);
    sc.da = at<float>(ws, bl.da);
    sc.glo = at<int32_t>(ws, bl.glo);
    sc.ghi = at<int32_t>(ws, bl.ghi);
    sc.head_part = at<float>(ws, bl.head_part);
    sc.dz[0] = at<float>(ws, bl.dz0);
    sc.dz[1] = at<float>(ws, bl.dz1);
    sc.maskT = at<unsigned long long>(ws, bl.maskT);
    sc.rec = at<float>(ws, bl.rec);
    sc.dc_part = at<float>(ws, bl.dc_part);
    sc.d2_part = at<float>(ws, bl.d2_part);
    sc.dvec = at<float>(ws, bl.dvec);
    sc.red_tmp = at<float>(ws, bl.red_tmp);

    const size_t nsp = (size_t)N * S * p;
    const float *muT = mu_saved + (size_t)(T - 1) * nsp;
    S2V_TRY(launch_bwd_head(st, p, N, S, G, g->graph_off, params->theta5, params->theta6, params->theta7, muT, gsum,
                            action, target, sc, q_pred));
    S2V_TRY(launch_bwd_head_reduce(st, p, S, sc, loss, grads->theta5, grads->theta6, grads->theta7));
    // dz^T is never materialised: its relu mask and its share of the sums come from one pass over mu^T
    const HubTable ht = hub_table(ws, h, *pr);
    const float *x_res = g->state_residual ? x : nullptr;
    const float *wagg = g->weighted_sum ? g->w : nullptr;   // NULL weights mean w = 1: the plain sum
    if (x_res)
        S2V_TRY(launch_stateinfo_residual(st, N, S, ht, g->rowptr, row_end_of(g), g->colidx, g->w, x, sc.rec, nullptr));
    // (node mode on a static graph without negative weights: the last reversed round -- done inside the round
    //  t = 3, or by k_bwd_first when T = 3 -- works from flag words and the rows' totals of s+ like the
    //  forward's round 2)
    const bool by_flags = S % 16 == 0 && T >= 3 && !pr->has_neg && !g->row_end && !x_res;
    unsigned long long *flags = by_flags ? at<unsigned long long>(ws, bl.flags16) : nullptr;
    if (!x_res)
        S2V_TRY(launch_nodeinfo(st, N, S, x, s_pos, s_neg, sc.rec, nullptr,
                                by_flags ? at<float>(ws, wagg ? h.nbr_spw : h.nbr_sp) : nullptr, flags));
    NodeInfo ninfo = make_nodeinfo(sc.rec, S, x_res != nullptr);
    ninfo.flags16 = reinterpret_cast<const unsigned short *>(flags);
    {
        SpanGuard span(ctx, S2V_PROFILE_BWD_SEED);
        S2V_TRY(launch_bwd_maskT(st, p, N, S, muT, ninfo, x_res, action, sc, T >= 2 ? sc.maskT : nullptr, sc.dc_part,
                                 words_ready));
    }
    float *hub_part = at<float>(ws, bl.hub_part), *hub_sum = at<float>(ws, bl.hub_sum);
    float *hub_part4 = at<float>(ws, bl.hub_part4), *hub_sum4 = at<float>(ws, bl.hub_sum4);
    const bool node = S % 16 == 0 && N > 0;
    int cur = 1;  // the round t = T writes dz[0]
    for (int t = T; t >= 2; --t) {
        const int slot = T - t;  // 0 for the first reversed round
        float *dc_part = sc.dc_part + ((size_t)kBwdHeadGrid + (size_t)slot * kBwdRoundRows) * 3 * p;
        float *d2_part = sc.d2_part + (size_t)slot * kBwdRoundRows * p * p;
        const float *mu_prev = mu_saved + (size_t)(t - 2) * nsp;
        const bool first = t == T;
        const float *dz_in = first ? nullptr : sc.dz[cur];
        float *dz_out = t == 2 ? nullptr : sc.dz[cur ^ 1];  // dz^1 only feeds the sums
        float *qvec = at<float>(ws, bl.qvec);
        if (t == 2 && !first && node && T >= 4) {
            // done inside the round t = 3 (see below): this round's partial rows stay empty
            S2V_TRY(launch_zero_i32(st, (long)kBwdRoundRows * 3 * p, reinterpret_cast<int32_t *>(dc_part)));
            S2V_TRY(launch_zero_i32(st, (long)kBwdRoundRows * p * p, reinterpret_cast<int32_t *>(d2_part)));
            continue;
        }
        if (t == 2 && !first) {
            // (node mode: T == 3; row mode: any T >= 3) the last reversed round streams dz^2 and gathers
            // scalars instead of rows (for T == 2 the round reads mask words, which is cheaper still)
            S2V_TRY(launch_qvec(st, p, params->theta3, params->theta4, qvec));
            S2V_TRY(launch_hub_sums_grad(st, p, S, ht, row_end_of(g), g->colidx, wagg, ninfo, pr->has_neg, params->theta1,
                                         qvec, hub_part4, hub_sum4));
            {
                SpanGuard span(ctx, S2V_PROFILE_BWD_FIRST);
                S2V_TRY(launch_bwd_first(st, p, N, S, g->rowptr, row_end_of(g), g->colidx, wagg, dz_in, ninfo, pr->has_neg,
                                         params->theta1, params->theta2, qvec, dc_part, d2_part, ht, hub_sum4));
            }
            cur ^= 1;
            continue;
        }
        // node mode, T >= 4: the round t = 3 (rows of dz^3 in memory) also does the round t = 2 for each
        // of its tiles while the tile's dz^2 is on chip; dz^2 is neither written nor read
        const bool fuse_last = t == 3 && !first && node;
        BwdFuse bf{params->theta1, qvec, hub_sum4, pr->has_neg};
        if (fuse_last) {
            S2V_TRY(launch_qvec(st, p, params->theta3, params->theta4, qvec));
            S2V_TRY(launch_hub_sums_grad(st, p, S, ht, row_end_of(g), g->colidx, wagg, ninfo, pr->has_neg, params->theta1,
                                         qvec, hub_part4, hub_sum4));
            dz_out = nullptr;
        }
        S2V_TRY(launch_hub_sums(st, p, S, ht, row_end_of(g), g->colidx, wagg, dz_in, ninfo, nullptr, nullptr, first ? sc.maskT : nullptr,
                                hub_part, hub_sum));
        {
            SpanGuard span(ctx, first ? S2V_PROFILE_BWD_ROUND_MASK : S2V_PROFILE_BWD_ROUND);
            S2V_TRY(launch_bwd_round(st, p, N, S, g->rowptr, row_end_of(g), g->colidx, wagg, dz_in, first ? sc.maskT : nullptr, sc, mu_prev,
                                     dz_out, ninfo, params->theta2, dc_part, d2_part, ht, hub_sum, fuse_last ? &bf : nullptr,
                                     nsp * sizeof(float) >= ctx->sliced_min_bytes));
        }
        if (first) {
            float *dc_fix = sc.dc_part + ((size_t)kBwdHeadGrid + (size_t)(T - 1) * kBwdRoundRows) * 3 * p;
            float *d2_fix = sc.d2_part + (size_t)(T - 1) * kBwdRoundRows * p * p;
            S2V_TRY(launch_bwd_action_fix(st, p, S, g->rowptr, row_end_of(g), g->colidx, wagg, action, sc.maskT, sc, params->theta2,
                                          mu_prev, dz_out, ninfo, dc_fix, d2_fix));
        }
        cur ^= 1;
    }
    S2V_TRY(launch_bwd_finish(st, p, bl.dc_rows, bl.d2_rows, sc, params->theta3, params->theta4, grads->theta1,
                              grads->theta2, grads->theta3, grads->theta4));
    return S2V_OK;
}

int32_t s2v_embed_bwd(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                      int32_t S, const float *mu_saved, const float *gsum, const int32_t *action,
                      const float *target, float *loss, float *q_pred, s2v_params *grads, void *ws,
                      size_t ws_bytes) {
    return embed_bwd_impl(ctx, g, params, x, T, S, mu_saved, gsum, action, target, loss, q_pred, grads, ws, ws_bytes,
                          false);
}

int32_t s2v_loss_grad(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, const float *x, int32_t T,
                      int32_t S, float *mu_saved, float *gsum, const int32_t *action, const float *target,
                      float *loss, float *q_pred, s2v_params *grads, void *ws, size_t ws_bytes) {
    if (!ctx || !g || !params || !mu_saved || !gsum || !action) return S2V_ERR_INVALID_ARG;
    // The forward pass can leave out what the backward pass never reads (round 1's rows, and all of mu^T
    // but its relu mask, the action nodes' rows and the graph sums) when the kernels that make do without
    // them apply: 16 states sharing one graph, at least three rounds.  Otherwise the two passes run as
    // they do when called one after the other.
    const bool fuse = S == 16 && g->n_graphs == 1 && T >= 3 && !g->state_residual && g->n_nodes > 0 &&
                      p_supported(params->p);
    if (!fuse) {
        const int32_t rc = embed_fwd_impl(ctx, g, params, x, T, S, nullptr, mu_saved, gsum, ws, ws_bytes, nullptr, nullptr);
        if (rc != S2V_OK) return rc;
        return embed_bwd_impl(ctx, g, params, x, T, S, mu_saved, gsum, action, target, loss, q_pred, grads, ws, ws_bytes,
                              false);
    }
    int32_t rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(g->n_nodes, g->n_graphs, pr->n_hubs, pr->n_segs);
    const BwdLayout bl = bwd_layout(h, g->n_nodes, params->p, T, S);
    const FusedTrain ft{bl.end, at<unsigned long long>(ws, bl.maskT), action};
    rc = embed_fwd_impl(ctx, g, params, x, T, S, nullptr, mu_saved, gsum, ws, ws_bytes, nullptr, nullptr, &ft);
    if (rc != S2V_OK) return rc;
    return embed_bwd_impl(ctx, g, params, x, T, S, mu_saved, gsum, action, target, loss, q_pred, grads, ws, ws_bytes,
                          true);
}

static UpdateState update_state(const s2v_graph *g, const Prepared &pr, const HeadLayout &h, void *ws, float *x, int32_t k,
                                uint8_t *cand, int32_t *stats) {
    UpdateState u{};
    u.G = g->n_graphs;
    u.k = k;
    u.total = g->n_graphs * k;
    u.graph_off = g->graph_off;
    u.rowptr = g->rowptr;
    u.rowend = const_cast<int32_t *>(g->row_end);
    u.x = x;
    u.s_pos = at<float>(ws, h.s_pos);
    u.s_neg = at<float>(ws, h.s_neg);
    u.cand = cand;
    u.stats = stats;
    u.touched = at<int32_t>(ws, h.touched);
    u.epoch = at<int32_t>(ws, h.epoch);   // (the number of incremental updates since s2v_graph_prepare)
    u.jobs = at<int32_t>(ws, h.jobs);
    u.rec = pr.rec_keep ? at<float>(ws, h.rec) : nullptr;
    u.compact = (pr.rec_keep && !pr.has_neg) ? at<float>(ws, h.rec) + (size_t)g->n_nodes * 4 : nullptr;
    return u;
}

static int32_t residual_update_impl(s2v_ctx *ctx, const s2v_graph *g, float *x, const int32_t *sel_idx,
                                    const int32_t *sel_count, int32_t k, uint8_t *cand, int32_t *stats, void *ws,
                                    size_t ws_bytes, bool begun) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_graph(g);
    if (rc != S2V_OK) return rc;
    rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    const int32_t N = g->n_nodes, G = g->n_graphs;
    if (!g->row_end || !cand || !stats || k < 0) return S2V_ERR_INVALID_ARG;
    if (N > 0 && !x) return S2V_ERR_INVALID_ARG;
    if (sel_idx && (!sel_count || k < 1)) return S2V_ERR_INVALID_ARG;
    if (sel_idx && (int64_t)G * k > INT32_MAX) return S2V_ERR_INVALID_ARG;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    if (ws_bytes < h.end) return S2V_ERR_WORKSPACE_TOO_SMALL;
    if (!sel_idx) pr->rec_current = false;   // a full rebuild does not touch the records
    const UpdateState u = update_state(g, *pr, h, ws, x, sel_idx ? k : 0, cand, stats);
    S2V_TRY(launch_residual_update(ctx->stream, N, u, const_cast<int32_t *>(g->colidx), const_cast<float *>(g->w), sel_idx,
                                   sel_count, begun));
    return S2V_OK;
}

int32_t s2v_residual_update(s2v_ctx *ctx, const s2v_graph *g, float *x, const int32_t *sel_idx,
                            const int32_t *sel_count, int32_t k, uint8_t *cand, int32_t *stats, void *ws,
                            size_t ws_bytes) {
    return residual_update_impl(ctx, g, x, sel_idx, sel_count, k, cand, stats, ws, ws_bytes, false);
}

int32_t s2v_mvc_inference(s2v_ctx *ctx, const s2v_graph *g, const s2v_params *params, float *x, int32_t T,
                          int32_t adaptive, int32_t max_steps, float *mu, float *gsum, float *q, uint8_t *cand,
                          int32_t *sel_idx, float *sel_val, int32_t *sel_count, int32_t *stats,
                          int32_t *steps_out, int64_t *picked_out, int64_t *live_out, void *ws, size_t ws_bytes) {
    if (!ctx || !g || !steps_out || !picked_out || !live_out || max_steps < 0) return S2V_ERR_INVALID_ARG;
    if (!mu || !gsum || !q || !cand || !sel_idx || !sel_val || !sel_count || !stats) return S2V_ERR_INVALID_ARG;
    const int32_t N = g->n_nodes, G = g->n_graphs;
    *steps_out = 0;
    *picked_out = 0;
    *live_out = 0;
    // state from the incoming x: drops the edges already covered, fills cand and stats
    int32_t rc = s2v_residual_update(ctx, g, x, nullptr, nullptr, 0, cand, stats, ws, ws_bytes);
    if (rc != S2V_OK) return rc;
    // The loop runs in blocks of steps without reading anything back: which d to use, whether an edge is
    // left, and the counts of evaluations and of added nodes are all decided and kept on the device
    // (k_loop_control).  The host looks at the state once per block; a block that outlasts the solve costs the
    // evaluations it still makes, which change nothing.  Blocks grow 1, 2, 4, ... up to kLoopBlock steps, and
    // never beyond a sixteenth of the candidates the largest graph has left (every step removes at least one).
    constexpr int kLoopBlock = 64;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    unsigned long long *ctr = at<unsigned long long>(ws, h.loop_ctr);
    S2V_TRY(launch_zero_i32(ctx->stream, 4, reinterpret_cast<int32_t *>(ctr)));
    std::vector<int32_t> hstats(2 * (size_t)G);
    unsigned long long hctr[2] = {0ull, 0ull};
    int32_t max_cand = 0;
    auto read_state = [&](int64_t *n_live) -> int32_t {
        S2V_TRY(hipMemcpyAsync(hstats.data(), stats, sizeof(int32_t) * 2 * G, hipMemcpyDeviceToHost, ctx->stream));
        S2V_TRY(hipMemcpyAsync(hctr, ctr, sizeof(hctr), hipMemcpyDeviceToHost, ctx->stream));
        S2V_TRY(hipStreamSynchronize(ctx->stream));
        *n_live = 0;
        max_cand = 0;
        for (int b = 0; b < G; ++b) {
            *n_live += hstats[2 * b + 1];
            if (hstats[2 * b] > max_cand) max_cand = hstats[2 * b];
        }
        return S2V_OK;
    };
    int64_t n_live = 0;
    rc = read_state(&n_live);
    if (rc != S2V_OK) return rc;
    const bool use_rule = adaptive && G == 1;
    const int32_t k_sel = use_rule ? kSmallK : 1;   // the largest d of the rule; the device cuts the count to d
    if (!g->row_end) return S2V_ERR_INVALID_ARG;
    // from here to the return the node records stay in the head of the workspace (see Prepared::rec_keep)
    struct KeepRecords {
        const Prepared *pr;
        explicit KeepRecords(const Prepared *p_) : pr(p_) { pr->rec_keep = true; pr->rec_current = false; }
        ~KeepRecords() { pr->rec_keep = false; pr->rec_current = false; }
    } keep_records(pr);
    const UpdateState upd = update_state(g, *pr, h, ws, x, k_sel, cand, stats);
    const StepEnd end{N, use_rule, ctr, &upd};
    int32_t launched = 0, block = 1;
    while (n_live > 0 && launched < max_steps) {
        int32_t todo = block < max_steps - launched ? block : max_steps - launched;
        if (todo > max_cand / 16) todo = max_cand / 16 > 1 ? max_cand / 16 : 1;
        for (int32_t i = 0; i < todo; ++i) {
            bool ended = false;
            rc = policy_select_impl(ctx, g, params, x, cand, T, k_sel, mu, gsum, q, sel_idx, sel_val, sel_count, ws, ws_bytes,
                                    &end, &ended);
            if (rc != S2V_OK) return rc;
            if (!ended) S2V_TRY(launch_loop_control(ctx->stream, N, use_rule, sel_count, ctr, sel_idx, upd));
            rc = residual_update_impl(ctx, g, x, sel_idx, sel_count, k_sel, cand, stats, ws, ws_bytes, true);
            if (rc != S2V_OK) return rc;
        }
        launched += todo;
        if (block < kLoopBlock) block *= 2;
        rc = read_state(&n_live);
        if (rc != S2V_OK) return rc;
    }
    const int32_t steps = (int32_t)hctr[0];
    const int64_t picked = (int64_t)hctr[1];
    *steps_out = steps;
    *picked_out = picked;
    *live_out = n_live;
    return S2V_OK;
}

int32_t s2v_sgd_step(s2v_ctx *ctx, s2v_params *params, const s2v_params *grads, float lr) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_params(params);
    if (rc != S2V_OK) return rc;
    rc = check_params(grads);
    if (rc != S2V_OK) return rc;
    if (grads->p != params->p) return S2V_ERR_INVALID_ARG;
    float *const th[7] = {params->theta1, params->theta2, params->theta3, params->theta4,
                          params->theta5, params->theta6, params->theta7};
    const float *const gr[7] = {grads->theta1, grads->theta2, grads->theta3, grads->theta4,
                                grads->theta5, grads->theta6, grads->theta7};
    S2V_TRY(launch_sgd(ctx->stream, params->p, th, gr, lr));
    return S2V_OK;
}

int32_t s2v_adam_step(s2v_ctx *ctx, s2v_params *params, const s2v_params *grads, s2v_params *m, s2v_params *v,
                      int32_t step, float lr, float beta1, float beta2, float eps) {
    if (!ctx || step < 1) return S2V_ERR_INVALID_ARG;
    const s2v_params *all[4] = {params, grads, m, v};
    for (const s2v_params *t : all) {
        int32_t rc = check_params(t);
        if (rc != S2V_OK) return rc;
        if (t->p != params->p) return S2V_ERR_INVALID_ARG;
    }
    float *const th[7] = {params->theta1, params->theta2, params->theta3, params->theta4,
                          params->theta5, params->theta6, params->theta7};
    const float *const gr[7] = {grads->theta1, grads->theta2, grads->theta3, grads->theta4,
                                grads->theta5, grads->theta6, grads->theta7};
    float *const mm[7] = {m->theta1, m->theta2, m->theta3, m->theta4, m->theta5, m->theta6, m->theta7};
    float *const vv[7] = {v->theta1, v->theta2, v->theta3, v->theta4, v->theta5, v->theta6, v->theta7};
    const float bias1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    const float bias2_sqrt = (float)std::sqrt(1.0 - std::pow((double)beta2, (double)step));
    S2V_TRY(launch_adam(ctx->stream, params->p, th, gr, mm, vv, lr, beta1, beta2, eps, bias1, bias2_sqrt));
    return S2V_OK;
}

int32_t s2v_q_target(s2v_ctx *ctx, const s2v_graph *g, const float *q_next, const float *x_next,
                     const uint8_t *cand_next, const int32_t *action, const float *reward, float gamma, int32_t S,
                     float *target, void *ws, size_t ws_bytes) {
    if (!ctx) return S2V_ERR_INVALID_ARG;
    int32_t rc = check_graph(g);
    if (rc != S2V_OK) return rc;
    rc = check_ws(ws);
    if (rc != S2V_OK) return rc;
    if (S < 1 || !reward || !target) return S2V_ERR_INVALID_ARG;
    const int32_t N = g->n_nodes, G = g->n_graphs;
    if (N > 0 && (!q_next || (!x_next && !cand_next))) return S2V_ERR_INVALID_ARG;
    if (G > 1 && !action) return S2V_ERR_INVALID_ARG;
    const Prepared *pr = find_prepared(ctx, g, ws);
    if (!pr) return S2V_ERR_NOT_PREPARED;
    const HeadLayout h = head_layout(N, G, pr->n_hubs, pr->n_segs);
    Carver c(h.end);
    const size_t pv = c.take(sizeof(float) * (size_t)S * h.max_chunks);
    const size_t pi = c.take(sizeof(int32_t) * (size_t)S * h.max_chunks);
    if (ws_bytes < c.off) return S2V_ERR_WORKSPACE_TOO_SMALL;
    const ChunkTable ct = chunk_table(ws, h, *pr);
    S2V_TRY(launch_q_target(ctx->stream, N, S, G, g->graph_off, ct, q_next, x_next, cand_next, action, reward, gamma,
                            at<float>(ws, pv), at<int32_t>(ws, pi), target));
    return S2V_OK;
}

int32_t s2v_adaptive_d(int64_t n_candidates, int64_t n_nodes) {
    // compare 2|C| > N, 4|C| > N, 8|C| > N to avoid fractions
    if (2 * n_candidates > n_nodes) return 8;
    if (4 * n_candidates > n_nodes) return 4;
    if (8 * n_candidates > n_nodes) return 2;
    return 1;
}

}  // extern "C"
