// The C boundary (include/tagore_knn.h): argument checks, workspace layout, and the round
// loop of Algorithm 1.  Host code only; every device step is a launcher from tg_kernels.h.
#include "../../include/tagore_knn.h"
#include "tg_device.h"
#include "tg_kernels.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

static thread_local char g_err[256] = "";

static int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
extern "C" const char* tg_last_error(void) { return g_err; }

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(TG_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

static int check_problem(int64_t n, int32_t d, const tg_knn_params* p)
{
    if (!p) return fail(TG_ERR_INVALID_ARG, "params is NULL");
    if (p->k < 1 || p->k > 64) return fail(TG_ERR_INVALID_ARG, "k = %d outside 1..64", p->k);
    if (n <= p->k) return fail(TG_ERR_INVALID_ARG, "need k < n (k = %d, n = %lld)", p->k, (long long)n);
    if (n >= (1ll << 30)) return fail(TG_ERR_INVALID_ARG, "n = %lld must be below 2^30", (long long)n);
    if (d < 1 || d > 4096) return fail(TG_ERR_INVALID_ARG, "d = %d outside 1..4096", d);
    if (p->metric < 0 || p->metric > 2) return fail(TG_ERR_INVALID_ARG, "unknown metric %d", p->metric);
    if (p->it1 < 0 || p->it2 < 0 || p->it1 + p->it2 > TG_MAX_ROUNDS)
        return fail(TG_ERR_INVALID_ARG, "it1 = %d, it2 = %d: need 0 <= it1 + it2 <= %d", p->it1, p->it2, TG_MAX_ROUNDS);
    if (p->S < 1 || p->S > 32) return fail(TG_ERR_INVALID_ARG, "S = %d outside 1..32", p->S);
    if (p->R < 0 || p->R > 32) return fail(TG_ERR_INVALID_ARG, "R = %d outside 0..32", p->R);
    if (p->C < 16 || p->C > 256 || (p->C & (p->C - 1))) return fail(TG_ERR_INVALID_ARG, "C = %d must be 16, 32, 64, 128 or 256", p->C);
    if (p->parts != 1 && p->parts != 2 && p->parts != 4 && p->parts != 8) return fail(TG_ERR_INVALID_ARG, "parts = %d must be 1, 2, 4 or 8", p->parts);
    if (p->m < 1 || p->m > 4) return fail(TG_ERR_INVALID_ARG, "m = %d outside 1..4", p->m);
    if (!(p->delta >= 0.0f && p->delta < 1.0f)) return fail(TG_ERR_INVALID_ARG, "delta must be in [0, 1)");
    if (p->screen != 0 && p->screen != 1) return fail(TG_ERR_INVALID_ARG, "screen = %d must be 0 or 1", p->screen);
    if (p->join_f16 < 0 || p->join_f16 > 2) return fail(TG_ERR_INVALID_ARG, "join_f16 = %d must be 0, 1 or 2", p->join_f16);
    return TG_OK;
}

extern "C" int tg_knn_default_params(int32_t k, int32_t iters, tg_knn_params* p)
{
    if (!p) return fail(TG_ERR_INVALID_ARG, "params is NULL");
    memset(p, 0, sizeof(*p));
    p->k = k;
    p->metric = TG_METRIC_L2;
    p->delta = 0.0f;
    if (iters <= 0) { iters = 16; p->delta = 0.001f; }
    // the first phase converges fastest while the lists are poor (section 4.1): it gets the first four rounds and,
    // beyond eight, every other one
    p->it1 = iters < 4 ? iters : (iters + 1) / 2 > 4 ? (iters + 1) / 2 : 4;
    p->it2 = iters - p->it1;
    p->S = k < 32 ? (k < 1 ? 1 : k) : 32;
    p->R = 32;
    p->C = 256;
    p->parts = 2;
    p->m = 2;
    p->finalize = 1;
    p->screen = 1;
    p->join_f16 = 0;
    p->seed = 1;
    return TG_OK;
}

// ---- workspace layout -----------------------------------------------------------------
struct Carver {
    char* base;
    size_t used;
    template <class T> T* take(size_t count)
    {
        used = (used + 255) & ~(size_t)255;
        T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
        used += count * sizeof(T);
        return p;
    }
};

struct tg_knn_handle {
    tg_knn_params p;
    TgGraph g;
    TgSample sm;
    TgCand cd;
    hipStream_t stream;
    u64* d_updates;      // TG_MAX_ROUNDS x TG_STAT_BINS partial counters (spread to avoid one hot address)
    u64* d_stat_bins;    // TG_MAX_ROUNDS x 2 x TG_STAT_BINS
    float* x_padded;     // own copy of X when the caller's rows are not 16-byte friendly
    uint8_t* xq;         // 8-bit screening copy of X, written when phase 2 begins
    float* xqm;          // its grid (three words, see TgGraph)
    u32* d_screen_on;    // device flag: screening still pays (decided after each screened round)
    u32* d_undefined;    // device counter: rows of X without a defined distance (written with the norms)
    uint16_t* xh;        // fp16 copy of X for the local join (join_f16 = 1, 2)
    u32* d_f16_ok;       // join_f16 = 2: device flag, 1 while every value of X is an fp16 number
    int round;           // rounds run so far (both phases)
    int rounds1, rounds2;
    bool phase2;
    bool norms_done;
    bool lists_ready;    // tg_knn_init or tg_knn_import has written the lists
    // timing
    std::vector<hipEvent_t> ev;
    struct Span { int kind, round, e0, e1; };
    std::vector<Span> spans;
};
enum { SPAN_NORMS, SPAN_INIT, SPAN_SAMPLE, SPAN_ADJ, SPAN_JOIN, SPAN_UPDATE, SPAN_FINALIZE };

static int round_up4(int d) { return (d + 3) & ~3; }

static void carve(tg_knn_handle* h, const float* X, int64_t n, int32_t d, void* ws, size_t* need)
{
    const tg_knn_params& p = h->p;
    Carver c{reinterpret_cast<char*>(ws), 0};
    const int ld = round_up4(d);
    const bool pad = (ld != d) || ((reinterpret_cast<uintptr_t>(X) & 15) != 0);
    h->x_padded = pad ? c.take<float>((size_t)n * ld) : nullptr;
    h->g.n = n; h->g.d = d; h->g.ld = ld; h->g.k = p.k; h->g.metric = p.metric;
    h->g.X = pad ? h->x_padded : X;
    h->g.nrm = c.take<float>(n);
    h->g.rnorm = c.take<float>(n);
    h->g.gid = c.take<u32>((size_t)n * p.k);
    h->g.gid_next = c.take<u32>((size_t)n * p.k);
    h->g.gdist = c.take<float>((size_t)n * p.k);
    h->g.kth = c.take<u64>(n);
    h->g.ldq = (d + 15) & ~15;
    h->xq = p.screen ? c.take<uint8_t>((size_t)n * h->g.ldq) : nullptr;
    h->xqm = c.take<float>(64);          // also where the norms leave the range of the values
    h->g.Xq = h->xq;
    h->g.Xqm = h->xqm;
    h->d_screen_on = c.take<u32>(64);
    h->d_undefined = h->d_screen_on + 32;        // a word of its own line in the same 256 bytes
    // the register-resident join reads 64, 96 or 128 columns per row (4, 6 or 8 steps of 16); longer rows are whole steps of 32
    h->g.ldh = ld <= 64 ? 64 : ld <= 96 ? 96 : ld <= 128 ? 128 : (d + 31) & ~31;
    h->xh = p.join_f16 ? c.take<uint16_t>((size_t)n * h->g.ldh) : nullptr;
    h->d_f16_ok = p.join_f16 == 2 ? c.take<u32>(64) : nullptr;
    h->g.f16_ok = h->d_f16_ok;
    h->g.Xh = h->xh;
    h->sm.S = p.S; h->sm.R = p.R;
    h->sm.bshift = tg_rev_bucket_shift(n);
    h->sm.nbuckets = (n + (1ll << h->sm.bshift) - 1) >> h->sm.bshift;
    h->sm.bcnt = c.take<u32>((size_t)h->sm.nbuckets);
    h->sm.boff = c.take<u64>((size_t)h->sm.nbuckets + 1);
    h->sm.csr = c.take<u32>((size_t)n * p.k);
    {
        const int fwd = p.k < 2 * p.S ? p.k : 2 * p.S;
        h->sm.BC = (fwd + 2 * p.R + 15) & ~15;
    }
    h->sm.blk = c.take<u32>((size_t)n * h->sm.BC);
    h->sm.bsz = c.take<u32>(n);
    h->sm.wl = c.take<u64>((size_t)3 * (n + TG_MAX_PARTS));
    h->sm.wl_cnt = c.take<u32>(TG_WL_LISTS);
    h->sm.scan_tmp = c.take<u64>(tg_scan_tmp_elems(h->sm.nbuckets));
    h->sm.parts = p.parts;
    h->sm.parts_shift = p.parts == 8 ? 3 : p.parts == 4 ? 2 : p.parts == 2 ? 1 : 0;
    h->sm.adj_words = h->sm.BC > 64 ? 4 : 2;
    {
        // the adjacency words of a part and the edges by bucket are never alive together: one place for both
        const size_t adj_bytes = (size_t)((n + p.parts - 1) / p.parts) * h->sm.BC * h->sm.adj_words * sizeof(u32);
        const size_t ebuf_bytes = (size_t)n * p.k * sizeof(u64);
        u64* both = c.take<u64>((adj_bytes > ebuf_bytes ? adj_bytes : ebuf_bytes) / sizeof(u64) + 1);
        h->sm.adj = reinterpret_cast<u32*>(both);
        h->sm.ebuf = both;
    }
    h->cd.C = p.C;
    h->cd.slots = c.take<u64>((size_t)n * p.C);
    h->d_updates = c.take<u64>((size_t)TG_MAX_ROUNDS * TG_STAT_BINS);
    h->d_stat_bins = c.take<u64>((size_t)TG_MAX_ROUNDS * 2 * TG_STAT_BINS);
    *need = (c.used + 255) & ~(size_t)255;
}

extern "C" size_t tg_knn_workspace_bytes(int64_t n, int32_t d, const tg_knn_params* p)
{
    if (check_problem(n, d, p) != TG_OK) return 0;
    tg_knn_handle tmp;
    tmp.p = *p;
    size_t need = 0;
    // rows of a whole number of 16 bytes are used where they are (X is then expected 16-byte aligned); others are copied
    carve(&tmp, reinterpret_cast<const float*>(0), n, d, nullptr, &need);
    return need;
}

static int begin_span(tg_knn_handle* h, int kind, int round)
{
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return -1;        // no timing for this span; the work goes on
    if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return -1;
    }
    h->ev.push_back(a);
    h->ev.push_back(b);
    h->spans.push_back({kind, round, (int)h->ev.size() - 2, (int)h->ev.size() - 1});
    (void)hipEventRecord(a, h->stream);
    return (int)h->spans.size() - 1;
}
static void end_span(tg_knn_handle* h, int span)
{
    if (span >= 0) (void)hipEventRecord(h->ev[h->spans[span].e1], h->stream);
}

extern "C" int tg_knn_create(tg_knn_handle** out, const float* X, int64_t n, int32_t d, const tg_knn_params* p,
                             void* workspace, size_t workspace_bytes, void* stream)
{
    if (!out) return fail(TG_ERR_INVALID_ARG, "handle pointer is NULL");
    *out = nullptr;
    int rc = check_problem(n, d, p);
    if (rc != TG_OK) return rc;
    if (!X) return fail(TG_ERR_INVALID_ARG, "X is NULL");
    if (!workspace) return fail(TG_ERR_INVALID_ARG, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(TG_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    tg_knn_handle* h = new (std::nothrow) tg_knn_handle();
    if (!h) return fail(TG_ERR_OUT_OF_MEMORY, "host allocation failed");
    h->p = *p;
    h->stream = reinterpret_cast<hipStream_t>(stream);
    size_t need = 0;
    carve(h, X, n, d, workspace, &need);
    if (need > workspace_bytes) {
        const bool misaligned = h->x_padded && (d & 3) == 0;
        delete h;
        return fail(TG_ERR_INVALID_ARG, "workspace too small: %zu bytes given, %zu needed%s", workspace_bytes, need,
                    misaligned ? " (X is not 16-byte aligned, so room for an aligned copy of it is needed too)" : "");
    }
    h->round = h->rounds1 = h->rounds2 = 0;
    h->phase2 = false;
    h->norms_done = false;
    h->lists_ready = false;
    if (h->x_padded) tg_launch_pad_rows(X, n, d, h->x_padded, h->g.ld, h->stream);
    tg_launch_fill_u32(h->sm.bcnt, (size_t)h->sm.nbuckets, 0u, h->stream);
    tg_launch_fill_u64(h->cd.slots, (size_t)n * p->C, TG_EMPTY_KEY, h->stream);
    tg_launch_fill_u64(h->d_updates, (size_t)TG_MAX_ROUNDS * TG_STAT_BINS, 0ull, h->stream);
    tg_launch_fill_u64(h->d_stat_bins, (size_t)TG_MAX_ROUNDS * 2 * TG_STAT_BINS, 0ull, h->stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        delete h;
        return fail(TG_ERR_HIP, "launch failed: %s", hipGetErrorString(e));
    }
    *out = h;
    return TG_OK;
}

extern "C" int tg_knn_destroy(tg_knn_handle* h)
{
    if (!h) return TG_OK;
    for (hipEvent_t e : h->ev) (void)hipEventDestroy(e);
    delete h;
    return TG_OK;
}

static int launch_status(const char* what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TG_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return TG_OK;
}

static void ensure_norms(tg_knn_handle* h)
{
    if (h->norms_done) return;
    int sp = begin_span(h, SPAN_NORMS, 0);
    tg_launch_norms(h->g, reinterpret_cast<uint32_t*>(h->xqm), h->d_undefined, h->stream);
    if (h->d_f16_ok) tg_launch_fill_u32(h->d_f16_ok, 1, 1u, h->stream);
    // rounding every row whatever its values (join_f16 = 1): a row with a value beyond +-65504 has no fp16 copy to rank on, and is counted
    if (h->xh) tg_launch_narrow(h->g, h->xh, h->d_f16_ok, h->d_f16_ok ? nullptr : h->d_undefined, h->stream);
    end_span(h, sp);
    h->norms_done = true;
}

extern "C" int tg_knn_init(tg_knn_handle* h)
{
    if (!h) return fail(TG_ERR_INVALID_ARG, "handle is NULL");
    ensure_norms(h);
    int sp = begin_span(h, SPAN_INIT, 0);
    tg_launch_init(h->g, tg_hash_seed(h->p.seed, TG_TAG_INIT), h->stream);
    end_span(h, sp);
    h->round = h->rounds1 = h->rounds2 = 0;
    h->phase2 = false;
    h->lists_ready = true;
    return launch_status("init");
}

static int read_updates(tg_knn_handle* h, int round, int64_t* updates)
{
    std::vector<u64> bins(TG_STAT_BINS);
    HIP_TRY(hipMemcpyAsync(bins.data(), h->d_updates + (size_t)round * TG_STAT_BINS, TG_STAT_BINS * sizeof(u64),
                           hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(hipStreamSynchronize(h->stream));
    u64 v = 0;
    for (u64 b : bins) v += b;
    *updates = (int64_t)v;
    return TG_OK;
}

static int phase1_round(tg_knn_handle* h, int64_t* updates)
{
    if (!h) return fail(TG_ERR_INVALID_ARG, "handle is NULL");
    if (!h->lists_ready) return fail(TG_ERR_INVALID_ARG, "no lists yet: call tg_knn_init or tg_knn_import first");
    if (h->phase2) return fail(TG_ERR_INVALID_ARG, "phase 1 round after the switch to phase 2");
    if (h->round >= TG_MAX_ROUNDS) return fail(TG_ERR_INVALID_ARG, "more than %d rounds", TG_MAX_ROUNDS);
    const int r = h->round;
    int sp = begin_span(h, SPAN_SAMPLE, r);
    tg_launch_reverse(h->g, h->sm, tg_hash_seed(h->p.seed, TG_TAG_REV(r)), h->stream);
    tg_launch_bin(h->g, h->sm, h->p.parts, h->stream);
    end_span(h, sp);
    for (int part = 0; part < h->p.parts; ++part) {
        // the anchors v = part mod parts: their blocks are joined, then every list takes in what it was handed
        sp = begin_span(h, SPAN_ADJ, r);
        tg_launch_adj(h->g, h->sm, part, h->stream);
        end_span(h, sp);
        sp = begin_span(h, SPAN_JOIN, r);
        tg_launch_join(h->g, h->sm, h->cd, part, h->p.parts, tg_hash_seed(h->p.seed, TG_TAG_SLOT(r)),
                       h->d_stat_bins + (size_t)r * 2 * TG_STAT_BINS, h->stream);
        end_span(h, sp);
        sp = begin_span(h, SPAN_UPDATE, r);
        tg_launch_update(h->g, h->sm, h->cd, h->d_updates + (size_t)r * TG_STAT_BINS, part == 0, h->stream);
        end_span(h, sp);
    }
    h->round++;
    h->rounds1++;
    int rc = launch_status("phase-1 round");
    if (rc != TG_OK) return rc;
    return updates ? read_updates(h, r, updates) : TG_OK;
}
extern "C" int tg_knn_phase1_round(tg_knn_handle* h, int64_t* updates) { return phase1_round(h, updates); }

extern "C" int tg_knn_begin_phase2(tg_knn_handle* h)
{
    if (!h) return fail(TG_ERR_INVALID_ARG, "handle is NULL");
    if (!h->lists_ready) return fail(TG_ERR_INVALID_ARG, "no lists yet: call tg_knn_init or tg_knn_import first");
    tg_launch_mark_all_fresh(h->g, h->stream);
    if (h->xq) tg_launch_fill_u32(h->d_screen_on, 1, 1u, h->stream);
    if (!h->phase2 && h->xq) {
        ensure_norms(h);
        int sp = begin_span(h, SPAN_NORMS, 0);
        tg_launch_quantize(h->g, h->xq, h->xqm, h->stream);
        end_span(h, sp);
    }
    h->phase2 = true;
    return launch_status("phase switch");
}

extern "C" int tg_knn_phase2_round(tg_knn_handle* h, int64_t* updates)
{
    if (!h) return fail(TG_ERR_INVALID_ARG, "handle is NULL");
    if (!h->lists_ready) return fail(TG_ERR_INVALID_ARG, "no lists yet: call tg_knn_init or tg_knn_import first");
    if (!h->phase2) return fail(TG_ERR_INVALID_ARG, "phase 2 round before tg_knn_begin_phase2");
    if (h->round >= TG_MAX_ROUNDS) return fail(TG_ERR_INVALID_ARG, "more than %d rounds", TG_MAX_ROUNDS);
    const int r = h->round;
    int sp = begin_span(h, SPAN_JOIN, r);
    tg_launch_phase2(h->g, h->p.m, h->d_updates + (size_t)r * TG_STAT_BINS, h->d_stat_bins + (size_t)r * 2 * TG_STAT_BINS, h->d_screen_on,
                     h->stream);
    end_span(h, sp);
    u32* t = h->g.gid; h->g.gid = h->g.gid_next; h->g.gid_next = t;   // the written lists are current now
    h->round++;
    h->rounds2++;
    int rc = launch_status("phase-2 round");
    if (rc != TG_OK) return rc;
    return updates ? read_updates(h, r, updates) : TG_OK;
}

extern "C" int tg_knn_finalize(tg_knn_handle* h, int32_t* out_ids, float* out_dist)
{
    if (!h) return fail(TG_ERR_INVALID_ARG, "handle is NULL");
    if (!h->lists_ready) return fail(TG_ERR_INVALID_ARG, "no lists yet: call tg_knn_init or tg_knn_import first");
    if (!out_ids) return fail(TG_ERR_INVALID_ARG, "out_ids is NULL");
    int sp = begin_span(h, SPAN_FINALIZE, 0);
    ensure_norms(h);
    tg_launch_finalize(h->g, h->p.finalize, reinterpret_cast<const uint32_t*>(h->xqm), out_ids, out_dist, h->stream);
    end_span(h, sp);
    return launch_status("finalize");
}

extern "C" int tg_knn_get_stats(tg_knn_handle* h, tg_knn_stats* out)
{
    if (!h || !out) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    memset(out, 0, sizeof(*out));
    HIP_TRY(hipStreamSynchronize(h->stream));
    out->rounds_phase1 = h->rounds1;
    out->rounds_phase2 = h->rounds2;
    if (h->norms_done) {
        u32 bad = 0;
        HIP_TRY(hipMemcpy(&bad, h->d_undefined, sizeof(bad), hipMemcpyDeviceToHost));
        out->undefined_rows = (int64_t)bad;
    }
    if (h->round > 0) {
        std::vector<u64> upd((size_t)h->round * TG_STAT_BINS);
        HIP_TRY(hipMemcpy(upd.data(), h->d_updates, upd.size() * sizeof(u64), hipMemcpyDeviceToHost));
        for (int r = 0; r < h->round; ++r) {
            u64 v = 0;
            for (int b = 0; b < TG_STAT_BINS; ++b) v += upd[(size_t)r * TG_STAT_BINS + b];
            out->updates[r] = (int64_t)v;
        }
    }
    if (h->round > 0) {
        std::vector<u64> bins((size_t)h->round * 2 * TG_STAT_BINS);
        HIP_TRY(hipMemcpy(bins.data(), h->d_stat_bins, bins.size() * sizeof(u64), hipMemcpyDeviceToHost));
        for (int r = 0; r < h->round; ++r) {
            double pairs = 0, vecs = 0;
            for (int b = 0; b < TG_STAT_BINS; ++b) {
                pairs += (double)bins[((size_t)r * 2) * TG_STAT_BINS + b];
                vecs += (double)bins[((size_t)r * 2 + 1) * TG_STAT_BINS + b];
            }
            out->join_pairs[r] = pairs;
            out->join_vectors[r] = vecs;
        }
    }
    for (const auto& s : h->spans) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, h->ev[s.e0], h->ev[s.e1]) != hipSuccess) continue;
        switch (s.kind) {
        case SPAN_NORMS: out->ms_norms += ms; break;
        case SPAN_INIT: out->ms_init += ms; break;
        case SPAN_FINALIZE: out->ms_finalize += ms; break;
        case SPAN_SAMPLE: out->ms_sample[s.round] += ms; break;
        case SPAN_ADJ: out->ms_adjacency[s.round] += ms; break;
        case SPAN_JOIN: out->ms_join[s.round] += ms; break;
        case SPAN_UPDATE: out->ms_update[s.round] += ms; break;
        }
    }
    return TG_OK;
}

extern "C" int tg_knn_export(tg_knn_handle* h, int32_t* ids, float* dist, uint8_t* fresh)
{
    if (!h) return fail(TG_ERR_INVALID_ARG, "handle is NULL");
    if (!h->lists_ready) return fail(TG_ERR_INVALID_ARG, "no lists yet: call tg_knn_init or tg_knn_import first");
    tg_launch_export(h->g, ids, dist, fresh, h->stream);
    return launch_status("export");
}

extern "C" int tg_knn_import(tg_knn_handle* h, const int32_t* ids, const float* dist, const uint8_t* fresh)
{
    if (!h || !ids || !dist || !fresh) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    {
        // the lists come from the caller: every id is checked on the host before a kernel follows it
        std::vector<int32_t> hi((size_t)h->g.n * h->g.k);
        HIP_TRY(hipMemcpyAsync(hi.data(), ids, hi.size() * sizeof(int32_t), hipMemcpyDeviceToHost, h->stream));
        HIP_TRY(hipStreamSynchronize(h->stream));
        for (size_t i = 0; i < hi.size(); ++i)
            if (hi[i] < 0 || hi[i] >= h->g.n)
                return fail(TG_ERR_INVALID_ARG, "row %lld: id %d out of range", (long long)(i / h->g.k), hi[i]);
    }
    ensure_norms(h);
    tg_launch_import(h->g, ids, dist, fresh, h->stream);
    h->lists_ready = true;
    return launch_status("import");
}

extern "C" int tg_knn_sample_blocks(tg_knn_handle* h, int32_t* blk, int32_t* sizes)
{
    if (!h || !blk || !sizes) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (!h->lists_ready) return fail(TG_ERR_INVALID_ARG, "no lists yet: call tg_knn_init or tg_knn_import first");
    tg_launch_reverse(h->g, h->sm, tg_hash_seed(h->p.seed, TG_TAG_REV(h->round)), h->stream);
    tg_launch_dump_blocks(h->g, h->sm, blk, sizes, h->stream);
    return launch_status("sample");
}

extern "C" int tg_knn_block_adjacency(tg_knn_handle* h, uint32_t* adj)
{
    if (!h || !adj) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (!h->lists_ready) return fail(TG_ERR_INVALID_ARG, "no lists yet: call tg_knn_init or tg_knn_import first");
    for (int part = 0; part < h->p.parts; ++part) tg_launch_dump_adj(h->g, h->sm, part, adj, h->stream);
    return launch_status("block adjacency");
}

extern "C" int tg_knn_join_distances(tg_knn_handle* h, const int32_t* blk, const int32_t* sizes, int64_t nb, float* out)
{
    if (!h || !blk || !sizes || !out) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (nb < 0) return fail(TG_ERR_INVALID_ARG, "nb < 0");
    if (nb == 0) return TG_OK;
    // the blocks come from the caller: check them on the host side before any kernel trusts them
    std::vector<int32_t> hs((size_t)nb * 2), hb((size_t)nb * TG_BLOCK_COLS);
    HIP_TRY(hipMemcpyAsync(hs.data(), sizes, hs.size() * sizeof(int32_t), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(hipMemcpyAsync(hb.data(), blk, hb.size() * sizeof(int32_t), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(hipStreamSynchronize(h->stream));
    for (int64_t b = 0; b < nb; ++b) {
        const int nN = hs[b * 2], nO = hs[b * 2 + 1];
        if (nN < 0 || nO < 0 || nN > TG_BLOCK_ROWS || nN + nO > TG_BLOCK_COLS)
            return fail(TG_ERR_INVALID_ARG, "block %lld: sizes (%d, %d) outside (<= 64, sum <= 128)", (long long)b, nN, nO);
        for (int i = 0; i < nN + nO; ++i) {
            const int32_t id = hb[b * TG_BLOCK_COLS + i];
            if (id < 0 || id >= h->g.n) return fail(TG_ERR_INVALID_ARG, "block %lld: id %d out of range", (long long)b, id);
        }
    }
    ensure_norms(h);
    tg_launch_join_distances(h->g, blk, sizes, nb, out, h->stream);
    return launch_status("join distances");
}

// ---- whole builds ---------------------------------------------------------------------
static int run_all(tg_knn_handle* h, int32_t* out_ids, float* out_dist)
{
    const tg_knn_params& p = h->p;
    const double stop = (double)p.delta * (double)h->g.n * (double)p.k;
    int rc = tg_knn_init(h);
    if (rc != TG_OK) return rc;
    for (int r = 0; r < p.it1; ++r) {
        int64_t upd = 0;
        rc = phase1_round(h, p.delta > 0.0f ? &upd : nullptr);
        if (rc != TG_OK) return rc;
        if (p.delta > 0.0f && (double)upd < stop) break;
    }
    if (p.it2 > 0) {
        rc = tg_knn_begin_phase2(h);
        if (rc != TG_OK) return rc;
    }
    for (int r = 0; r < p.it2; ++r) {
        int64_t upd = 0;
        rc = tg_knn_phase2_round(h, p.delta > 0.0f ? &upd : nullptr);
        if (rc != TG_OK) return rc;
        if (p.delta > 0.0f && (double)upd < stop) break;
    }
    return tg_knn_finalize(h, out_ids, out_dist);
}

extern "C" int tg_knn_build_ex(const float* X, int64_t n, int32_t d, const tg_knn_params* p, void* workspace,
                               size_t workspace_bytes, int32_t* out_ids, float* out_dist, tg_knn_stats* stats,
                               void* stream)
{
    if (!out_ids) return fail(TG_ERR_INVALID_ARG, "out_ids is NULL");
    tg_knn_handle* h = nullptr;
    int rc = tg_knn_create(&h, X, n, d, p, workspace, workspace_bytes, stream);
    if (rc != TG_OK) return rc;
    rc = run_all(h, out_ids, out_dist);
    if (rc == TG_OK && stats) rc = tg_knn_get_stats(h, stats);
    tg_knn_destroy(h);
    return rc;
}

extern "C" int tg_knn_build(const float* X, int64_t n, int32_t d, int32_t k, int32_t metric, int32_t iters,
                            uint64_t seed, int32_t* out_ids, float* out_dist, void* stream)
{
    tg_knn_params p;
    tg_knn_default_params(k, iters, &p);
    p.metric = metric;
    p.seed = seed;
    int rc = check_problem(n, d, &p);
    if (rc != TG_OK) return rc;
    if (!X) return fail(TG_ERR_INVALID_ARG, "X is NULL");
    if (!out_ids) return fail(TG_ERR_INVALID_ARG, "out_ids is NULL");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // The workspace lives in stream order: taken before the first kernel, given back behind the last one, no wait.
    // Where the defaults' workspace cannot be had (1e8 points), the two parameters that only trade memory for recall per
    // round step down until it can: rounds in 4, then 8 parts, then 128, 64, 32 slots.
    static const int steps[][2] = {{0, 0}, {4, 0}, {8, 0}, {8, 128}, {8, 64}, {8, 32}};
    void* ws = nullptr;
    size_t bytes = 0;
    for (const auto& st : steps) {
        if (st[0]) p.parts = st[0];
        if (st[1]) p.C = st[1];
        // an X that is not 16-byte aligned is copied: room for that on top of what the size query says
        bytes = tg_knn_workspace_bytes(n, d, &p);
        if ((d & 3) == 0 && (reinterpret_cast<uintptr_t>(X) & 15)) bytes += (size_t)n * d * sizeof(float) + 256;
        if (hipMallocAsync(&ws, bytes, s) == hipSuccess) break;
        (void)hipGetLastError();
        ws = nullptr;
    }
    if (!ws) return fail(TG_ERR_OUT_OF_MEMORY, "workspace of %zu bytes could not be allocated", bytes);
    rc = tg_knn_build_ex(X, n, d, &p, ws, bytes, out_ids, out_dist, nullptr, stream);
    const hipError_t e = hipFreeAsync(ws, s);
    if (rc == TG_OK && e != hipSuccess) return fail(TG_ERR_HIP, "releasing the workspace failed: %s", hipGetErrorString(e));
    return rc;
}

extern "C" int tg_exact_knn(const float* X, int64_t n, int32_t d, int32_t k, int32_t metric, const int64_t* query_rows,
                            int64_t nq, int32_t* out_ids, float* out_dist, void* stream)
{
    if (!X || !out_ids) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (k < 1 || k > 64) return fail(TG_ERR_INVALID_ARG, "k = %d outside 1..64", k);
    if (n <= k || n >= (1ll << 30)) return fail(TG_ERR_INVALID_ARG, "need k < n < 2^30");
    if (d < 1 || d > 4096) return fail(TG_ERR_INVALID_ARG, "d = %d outside 1..4096", d);
    if (metric < 0 || metric > 2) return fail(TG_ERR_INVALID_ARG, "unknown metric %d", metric);
    if (nq < 0) return fail(TG_ERR_INVALID_ARG, "nq < 0");
    if (nq == 0) return TG_OK;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (query_rows) {   // the row indices come from the caller: check them before a kernel uses them
        std::vector<int64_t> hr((size_t)nq);
        HIP_TRY(hipMemcpyAsync(hr.data(), query_rows, hr.size() * sizeof(int64_t), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        for (int64_t r : hr)
            if (r < 0 || r >= n) return fail(TG_ERR_INVALID_ARG, "query row %lld out of range", (long long)r);
    } else if (nq > n) {
        return fail(TG_ERR_INVALID_ARG, "nq > n without query_rows");
    }
    const int ld = round_up4(d);
    const bool pad = (ld != d) || ((reinterpret_cast<uintptr_t>(X) & 15) != 0);
    const int slices = tg_exact_slices(n, nq);
    Carver c{nullptr, 0};
    c.take<float>(pad ? (size_t)n * ld : 0);
    c.take<float>(n);
    c.take<float>(n);
    c.take<u64>((size_t)nq * slices * k);
    const size_t bytes = (c.used + 255) & ~(size_t)255;
    void* ws = nullptr;
    if (hipMalloc(&ws, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(TG_ERR_OUT_OF_MEMORY, "scratch of %zu bytes could not be allocated", bytes);
    }
    Carver w{reinterpret_cast<char*>(ws), 0};
    float* xp = w.take<float>(pad ? (size_t)n * ld : 0);
    TgGraph g = {};
    g.n = n; g.d = d; g.ld = ld; g.k = k; g.metric = metric;
    g.X = pad ? xp : X;
    g.nrm = w.take<float>(n);
    g.rnorm = w.take<float>(n);
    u64* partial = w.take<u64>((size_t)nq * slices * k);
    if (pad) tg_launch_pad_rows(X, n, d, xp, ld, s);
    if (metric == 2) tg_launch_norms(g, nullptr, nullptr, s);
    tg_launch_exact_knn(g.X, ld, g.nrm, g.rnorm, n, d, k, metric, query_rows, nq, out_ids, out_dist, partial, slices, s);
    int rc = launch_status("exact k-NN");
    hipError_t e = hipStreamSynchronize(s);
    (void)hipFree(ws);
    if (rc == TG_OK && e != hipSuccess) return fail(TG_ERR_HIP, "exact k-NN failed: %s", hipGetErrorString(e));
    return rc;
}

// ---- exact k-NN without any allocation ------------------------------------------------------------
// The scratch of tg_exact_knn (inverse norms for the cosine, the per-slice partial lists) in device memory
// that belongs to the library: a file-scope array, one copy per GPU, held until the process ends.  Host
// code never uses the array's name as an address: its device address is asked for once per device.
#define TG_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[TG_STATIC_SCRATCH_BYTES];
#define TG_MAX_DEVICES 64
static void* g_scratch_ptr[TG_MAX_DEVICES];      // by device ordinal, filled on first use (under the lock)
static std::mutex g_scratch_lock;

static int static_scratch(void** out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= TG_MAX_DEVICES) return fail(TG_ERR_UNSUPPORTED, "device ordinal %d outside 0..%d", dev, TG_MAX_DEVICES - 1);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(TG_ERR_HIP, "no device address for the static scratch");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TG_OK;
}

extern "C" size_t tg_exact_knn_static_scratch_bytes(void) { return TG_STATIC_SCRATCH_BYTES; }

extern "C" int tg_exact_knn_static(const float* X, int64_t n, int32_t d, int32_t k, int32_t metric, const int64_t* query_rows,
                                   int64_t nq, int32_t* out_ids, float* out_dist, void* stream)
{
    if (!X || !out_ids) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (k < 1 || k > 64) return fail(TG_ERR_INVALID_ARG, "k = %d outside 1..64", k);
    if (n <= k || n >= (1ll << 30)) return fail(TG_ERR_INVALID_ARG, "need k < n < 2^30");
    if (d < 1 || d > 4096) return fail(TG_ERR_INVALID_ARG, "d = %d outside 1..4096", d);
    if (metric < 0 || metric > 2) return fail(TG_ERR_INVALID_ARG, "unknown metric %d", metric);
    if (nq < 0) return fail(TG_ERR_INVALID_ARG, "nq < 0");
    if (!query_rows && nq > n) return fail(TG_ERR_INVALID_ARG, "nq > n without query_rows");
    if ((d & 3) || (reinterpret_cast<uintptr_t>(X) & 15))
        return fail(TG_ERR_UNSUPPORTED, "the allocation-free exact k-NN needs d %% 4 == 0 and a 16-byte aligned X (a padded copy would have to be allocated)");
    if (nq == 0) return TG_OK;
    // layout: inverse norms (cosine only), then the partial lists; fewer slices when they would not fit
    Carver c{nullptr, 0};
    if (metric == 2) { c.take<float>(n); c.take<float>(n); }
    const size_t fixed = (c.used + 255) & ~(size_t)255;
    int slices = tg_exact_slices(n, nq);
    while (slices > 1 && fixed + (size_t)nq * slices * k * sizeof(u64) > TG_STATIC_SCRATCH_BYTES) --slices;
    const size_t need = fixed + (size_t)nq * slices * k * sizeof(u64);
    if (need > TG_STATIC_SCRATCH_BYTES)
        return fail(TG_ERR_INVALID_ARG, "problem too large for the static scratch: %zu bytes needed (%s8 nq k), %u available",
                    need, metric == 2 ? "8 n + " : "", (unsigned)TG_STATIC_SCRATCH_BYTES);
    void* base = nullptr;
    int rc = static_scratch(&base);
    if (rc != TG_OK) return rc;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    Carver w{reinterpret_cast<char*>(base), 0};
    TgGraph g = {};
    g.n = n; g.d = d; g.ld = d; g.k = k; g.metric = metric;
    g.X = X;
    if (metric == 2) {
        g.nrm = w.take<float>(n);
        g.rnorm = w.take<float>(n);
        tg_launch_norms(g, nullptr, nullptr, s);           // writes every word it later reads
    }
    u64* partial = w.take<u64>((size_t)nq * slices * k);   // every word read by the merge is written by the scan
    tg_launch_exact_knn(g.X, g.ld, g.nrm, g.rnorm, n, d, k, metric, query_rows, nq, out_ids, out_dist, partial, slices, s);
    return launch_status("exact k-NN (static scratch)");
}

extern "C" int tg_prune_rank(const int32_t* knn_ids, int64_t n, int32_t k, int32_t d_out, int32_t* out_ids, int32_t* out_counts,
                             void* stream)
{
    if (!knn_ids || !out_ids) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (n < 1 || n >= (1ll << 30)) return fail(TG_ERR_INVALID_ARG, "n = %lld outside 1..2^30-1", (long long)n);
    if (k < 1 || k > 64) return fail(TG_ERR_INVALID_ARG, "k = %d outside 1..64", k);
    if (d_out < 1 || d_out > k) return fail(TG_ERR_INVALID_ARG, "d_out = %d outside 1..k", d_out);
    tg_launch_prune_rank(knn_ids, n, k, d_out, out_ids, out_counts, reinterpret_cast<hipStream_t>(stream));
    return launch_status("rank-based pruning");
}

static int check_filter(const float* X, int64_t n, int32_t d, const int32_t* knn_ids, int32_t k, int32_t hops, int32_t cand_size,
                        int32_t d_out, const int32_t* out_ids)
{
    if (!X || !knn_ids || !out_ids) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (n < 1 || n >= (1ll << 30)) return fail(TG_ERR_INVALID_ARG, "n = %lld outside 1..2^30-1", (long long)n);
    if (d < 1 || d > 4096) return fail(TG_ERR_INVALID_ARG, "d = %d outside 1..4096", d);
    if (k < 1 || k > 64) return fail(TG_ERR_INVALID_ARG, "k = %d outside 1..64", k);
    if (hops != 1 && hops != 2) return fail(TG_ERR_INVALID_ARG, "hops = %d must be 1 or 2", hops);
    if (cand_size < 1 || cand_size > 64) return fail(TG_ERR_INVALID_ARG, "cand_size = %d outside 1..64", cand_size);
    if (d_out < 1 || d_out > 64) return fail(TG_ERR_INVALID_ARG, "d_out = %d outside 1..64", d_out);
    return TG_OK;
}

extern "C" int tg_prune_dist(const float* X, int64_t n, int32_t d, const int32_t* knn_ids, int32_t k, int32_t hops,
                             int32_t cand_size, float alpha, int32_t d_out, int32_t* out_ids, int32_t* out_deg, void* stream)
{
    const int rc = check_filter(X, n, d, knn_ids, k, hops, cand_size, d_out, out_ids);
    if (rc != TG_OK) return rc;
    if (!(alpha >= 1.0f) || !(alpha <= 1e6f)) return fail(TG_ERR_INVALID_ARG, "alpha must be in [1, 1e6]");
    tg_launch_filter(X, n, d, knn_ids, k, hops, cand_size, 0, alpha * alpha, d_out, out_ids, out_deg,
                     reinterpret_cast<hipStream_t>(stream));
    return launch_status("distance-based pruning");
}

extern "C" int tg_prune_angle(const float* X, int64_t n, int32_t d, const int32_t* knn_ids, int32_t k, int32_t hops,
                              int32_t cand_size, float gamma_deg, int32_t d_out, int32_t* out_ids, int32_t* out_deg, void* stream)
{
    const int rc = check_filter(X, n, d, knn_ids, k, hops, cand_size, d_out, out_ids);
    if (rc != TG_OK) return rc;
    if (!(gamma_deg > 0.0f) || !(gamma_deg <= 90.0f)) return fail(TG_ERR_INVALID_ARG, "gamma must be in (0, 90] degrees");
    // 4 cos^2(gamma), formed in double and rounded once; the cosine of 90 degrees is taken as 0
    double cg = cos((double)gamma_deg * 3.14159265358979323846 / 180.0);
    if (fabs(cg) < 1e-12) cg = 0.0;
    tg_launch_filter(X, n, d, knn_ids, k, hops, cand_size, 1, (float)(4.0 * cg * cg), d_out, out_ids, out_deg,
                     reinterpret_cast<hipStream_t>(stream));
    return launch_status("angle-based pruning");
}

extern "C" int tg_prune_dispersion(const float* X, int64_t n, int32_t d, const int32_t* knn_ids, int32_t k, int32_t hops,
                                   int32_t cand_size, int32_t d_out, int32_t* out_ids, int32_t* out_deg, void* stream)
{
    const int rc = check_filter(X, n, d, knn_ids, k, hops, cand_size, d_out, out_ids);
    if (rc != TG_OK) return rc;
    tg_launch_filter(X, n, d, knn_ids, k, hops, cand_size, 2, 0.0f, d_out, out_ids, out_deg, reinterpret_cast<hipStream_t>(stream));
    return launch_status("dispersion pruning");
}

extern "C" int tg_angle_at(const float* a, const float* b, const float* c, float* out, int64_t count, void* stream)
{
    if (count < 0 || count >= (1ll << 31)) return fail(TG_ERR_INVALID_ARG, "count = %lld outside 0..2^31-1", (long long)count);
    if (count == 0) return TG_OK;
    if (!a || !b || !c || !out) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    tg_launch_angle_at(a, b, c, out, count, reinterpret_cast<hipStream_t>(stream));
    return launch_status("angles");
}

extern "C" int tg_merge_local(int32_t* g_ids, float* g_dist, int64_t n, int32_t k, const int32_t* l_ids, const float* l_dist,
                              int64_t n_local, int32_t k_local, const int32_t* local_to_global, void* stream)
{
    if (!g_ids || !g_dist) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (n < 1 || n >= (1ll << 30)) return fail(TG_ERR_INVALID_ARG, "n = %lld outside 1..2^30-1", (long long)n);
    if (n_local < 0 || n_local > n) return fail(TG_ERR_INVALID_ARG, "n_local = %lld outside 0..n", (long long)n_local);
    if (k < 1 || k > 64 || k_local < 1 || k_local > 64) return fail(TG_ERR_INVALID_ARG, "k = %d, k_local = %d outside 1..64", k, k_local);
    if (n_local == 0) return TG_OK;              // an empty local index: nothing to merge, its pointers are not looked at
    if (!l_ids || !l_dist || !local_to_global) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    tg_launch_merge_local(g_ids, g_dist, n, k, l_ids, l_dist, n_local, k_local, local_to_global,
                          reinterpret_cast<hipStream_t>(stream));
    return launch_status("merge of a local index");
}

extern "C" int tg_lists_clear(int32_t* g_ids, float* g_dist, int64_t n, int32_t k, void* stream)
{
    if (!g_ids || !g_dist) return fail(TG_ERR_INVALID_ARG, "NULL argument");
    if (n < 1 || k < 1) return fail(TG_ERR_INVALID_ARG, "n = %lld, k = %d must be positive", (long long)n, k);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    tg_launch_fill_u32(reinterpret_cast<uint32_t*>(g_ids), (size_t)n * k, 0xFFFFFFFFu, s);
    tg_launch_fill_u32(reinterpret_cast<uint32_t*>(g_dist), (size_t)n * k, 0x7F800000u, s);
    return launch_status("clearing lists");
}
