/*
 * tagore_knn.h — C boundary of the MI355X (gfx950) GNN-Descent k-NN graph builder.
 *
 * The library builds an approximate k-nearest-neighbour graph with the two-phase
 * GNN-Descent of the Tagore paper (section 4, Algorithm 1): random neighbour lists,
 * then it1 rounds of shared-sample local joins (phase 1) and it2 rounds of per-node
 * expansion of the closest unvisited neighbours (phase 2), each round followed by a
 * lock-free per-list update (section 4.2).
 *
 * Conventions for every entry point
 *   - Every pointer marked "device" is HIP device memory of the current device and is
 *     owned by the caller; the library never frees or keeps it beyond the call, except
 *     that a handle keeps X and its workspace until tg_knn_destroy.
 *   - All device work is enqueued on the hipStream_t passed as `stream` (NULL = the
 *     default stream).  Calls return after enqueueing unless stated otherwise.
 *   - Return value: TG_OK or a negative tg_status.  Nothing is printed and no C++
 *     exception crosses the boundary; tg_last_error() gives a message for the calling
 *     thread's last failure.  On TG_ERR_INVALID_ARG outputs are untouched.
 *   - Distances: TG_METRIC_L2 is the squared Euclidean distance, TG_METRIC_IP is
 *     -<x,y>, TG_METRIC_COSINE is 1 - <x,y>/(|x||y|)  (the paper leaves "dis" open).
 *     X is expected to hold finite numbers whose squared norms are finite, and no all-zero
 *     row under TG_METRIC_COSINE.  Rows without a defined distance are not refused (the
 *     calls only enqueue work) but counted: tg_knn_stats.undefined_rows.  When it is not
 *     0 the lists are unspecified (such a row can pose as everyone's nearest neighbour),
 *     though every list still holds ids in [0, n), never its own node and no id twice:
 *     no distance is ever turned into an index.
 *   - Lists are ordered by (distance, id) ascending; a list never holds its own node
 *     or the same id twice.
 */
#ifndef TAGORE_KNN_H
#define TAGORE_KNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TG_OK = 0,
    TG_ERR_INVALID_ARG = -1,
    TG_ERR_UNSUPPORTED = -2,
    TG_ERR_OUT_OF_MEMORY = -3,
    TG_ERR_HIP = -4
} tg_status;

typedef enum { TG_METRIC_L2 = 0, TG_METRIC_IP = 1, TG_METRIC_COSINE = 2 } tg_metric;

/*
 * Parameters of Algorithm 1 and of the choices the paper leaves open.
 *   k        list length (degree of the graph), 1 <= k <= 64, k < n
 *   it1,it2  rounds of phase 1 / phase 2 (Algorithm 1 input; the paper sets it1 = it2)
 *   S        forward sample cap per class (new / old) in phase 1, 1 <= S <= 32
 *   R        reverse sample cap per class in phase 1, 0 <= R <= 32
 *   C        candidate slots per node (section 4.2 "candidate list"), a power of two, 16 <= C <= 256.  A block
 *            hands each of its members at most eight candidates: the closest one of every group of eight
 *            consecutive block positions (section 4.2: one closest candidate per node and sub-tile) that is
 *            not in the member's list already and would precede the list's last entry; the eight share one
 *            64-byte line of the member's slots, picked by a hash of (member, anchor), and a slot keeps the
 *            closer candidate when two meet in it
 *   parts    a phase-1 round is carried out in this many parts (1, 2, 4 or 8): part p joins the blocks of
 *            the anchors v = p (mod parts), then every list takes in its candidates, so that the next part
 *            meets the tightened thresholds and the lengthened lists.  More parts: fewer candidates that
 *            cannot stay, so fewer slots do; more list updates
 *   m        neighbours expanded per node and phase-2 round (the paper: m = 2), 1..4
 *   delta    early stop: a phase ends when a round changes fewer than delta*n*k
 *            entries; 0 = run exactly it1 + it2 rounds (never synchronises with the host)
 *   seed     seed of every random decision (initial lists, reverse sampling, slots)
 *   finalize 1: recompute the reported distances directly from the vectors and
 *            re-sort each list before writing the outputs.  Where X holds whole numbers with
 *            2 d max|x|^2 <= 2^24 (byte-valued features of up to 129 dimensions, say; found while
 *            the norms are formed) and the distance is not the cosine, every fp32 sum the rounds
 *            form is exact, the lists hold the directly computed distances already, and nothing is
 *            recomputed
 *   screen   1: a phase-2 round first bounds every candidate's distance from below on an
 *            8-bit copy of the vectors (n x (d + 47) bytes of workspace) and measures in fp32
 *            only those that may still enter the list; the bound is rigorous, so the graph is
 *            the same as with 0, which measures every candidate (section 4.1 as written).
 *            When more than half of a round's candidates pass the bound (real-valued data in
 *            high dimension) the following rounds measure every candidate directly
 *   join_f16 1: the local join of phase 1 forms its inner products on the fp16 matrix
 *            instructions from a copy of the vectors rounded to fp16 (round to nearest even;
 *            n x (64, 96, 128, or d rounded up to 32) x 2 bytes of workspace), accumulating in fp32; norms,
 *            thresholds, phase 2 and the reported distances stay fp32.  Where every value is an
 *            fp16 number (byte-valued features, say) the copy is exact (see 2 for what that
 *            means for the graph); elsewhere the join ranks its candidates on rounded vectors (11 significant
 *            bits), and the list update measures every candidate that enters a list again in fp32
 *            from the vectors, so lists and thresholds hold exact distances.  Values
 *            beyond +-65504 have no fp16 number: such data must not use 1; the rows that hold such a
 *            value are counted in tg_knn_stats.undefined_rows (their lists stay well-formed and hold
 *            exact distances, but which candidates reach them is unspecified).
 *            2: as 1, but only if every value of X turned out to be an fp16 number when the copy
 *            was made (a flag on the device; both variants of the join are launched and the one
 *            whose turn it is not ends at once).  No operand is rounded then, so the join's
 *            products are those of the fp32 join exactly; its fp32 sums are taken in another
 *            order, so the graph is the same as with 0 bit for bit where those sums are exact
 *            (integer-valued data below 2^24) and equally accurate elsewhere.  Default 0
 */
typedef struct tg_knn_params {
    int32_t k;
    int32_t metric;
    int32_t it1, it2;
    int32_t S, R, C;
    int32_t parts;
    int32_t m;
    float delta;
    int32_t finalize;
    int32_t screen;
    int32_t join_f16;
    uint64_t seed;
} tg_knn_params;

#define TG_MAX_ROUNDS 64

/* What a build did; filled by tg_knn_build_ex / tg_knn_get_stats (host memory). */
typedef struct tg_knn_stats {
    int32_t rounds_phase1, rounds_phase2;
    int64_t updates[TG_MAX_ROUNDS];      /* list entries replaced in round r (both phases, in order) */
    float ms_norms, ms_init, ms_finalize; /* ms_norms: norms plus the 8-bit screening copy (screen = 1) */
    float ms_sample[TG_MAX_ROUNDS];      /* reverse-sample build of round r (phase 1)               */
    float ms_join[TG_MAX_ROUNDS];        /* local join (phase 1: the multiplying kernels of every part) or expand+update (phase 2) */
    float ms_adjacency[TG_MAX_ROUNDS];   /* which members of a block already list which (phase 1, every part) */
    float ms_update[TG_MAX_ROUNDS];      /* list update kernel (phase 1)                            */
    double join_pairs[TG_MAX_ROUNDS];    /* pairs the join of round r had to evaluate               */
    double join_vectors[TG_MAX_ROUNDS];  /* vectors the join of round r had to gather               */
    int64_t undefined_rows;              /* rows of X without a defined distance (see "Distances"): 0 for valid input */
} tg_knn_stats;

typedef struct tg_knn_handle tg_knn_handle;

/* Defaults for a given k and total round budget.  From 8 rounds on it1 = ceil(iters/2), it2 = iters - it1
 * (section 7.3: it1 = it2); a smaller budget goes to the first phase first (it1 = min(iters, 4)), which is
 * the one that converges while the lists are poor (section 4.1).  S = min(k,32), R = 32, C = 256,
 * parts = 2, m = 2, delta = 0, finalize = 1, screen = 1, seed = 1.  iters <= 0 selects 16 rounds with
 * delta = 0.001. */
int tg_knn_default_params(int32_t k, int32_t iters, tg_knn_params* p /* host, out */);

/* Device bytes a build of this size needs as workspace, for an X that is 16-byte aligned (rows of d % 4 == 0
 * floats are then used where they are; other rows are copied, which is counted).  An X with d % 4 == 0 that
 * is not 16-byte aligned needs 4 n d + 256 bytes more.  0 if the arguments are invalid. */
size_t tg_knn_workspace_bytes(int64_t n, int32_t d, const tg_knn_params* p);

/*
 * The whole of Algorithm 1.  X: device, row-major n x d fp32.  out_ids: device, n x k
 * int32.  out_dist: device, n x k fp32, may be NULL.  Takes and returns its own workspace in
 * stream order (hipMallocAsync / hipFreeAsync on `stream`: no wait; with iters > 0 the call
 * only enqueues work).  Runs with tg_knn_default_params(k, iters); where the device cannot give the
 * workspace of those (about 3.9 KB per point at k = 32), parts and C step down (parts 4, 8, then C 128,
 * 64, 32) until it can.
 * iters > 0: exactly that many rounds, split as tg_knn_default_params says; iters <= 0: up to
 * 16 rounds with early stop.  Valid iff 1 <= k <= 64, k < n < 2^30, 1 <= d <= 4096.
 */
int tg_knn_build(const float* X, int64_t n, int32_t d, int32_t k, int32_t metric, int32_t iters,
                 uint64_t seed, int32_t* out_ids, float* out_dist, void* stream);

/* As tg_knn_build with explicit parameters and a caller-provided device workspace of at
 * least tg_knn_workspace_bytes() bytes (256-byte aligned).  stats may be NULL; when it is
 * not, the call synchronises the stream before returning so that the timings are final. */
int tg_knn_build_ex(const float* X, int64_t n, int32_t d, const tg_knn_params* p, void* workspace,
                    size_t workspace_bytes, int32_t* out_ids, float* out_dist, tg_knn_stats* stats,
                    void* stream);

/* ---- Algorithm 1 step by step (what tg_knn_build_ex runs, one call per line) ---------- */

/* Binds X, the parameters, a workspace and a stream.  X and workspace must stay valid
 * until tg_knn_destroy.  The handle itself is host memory owned by the library. */
int tg_knn_create(tg_knn_handle** h, const float* X, int64_t n, int32_t d, const tg_knn_params* p,
                  void* workspace, size_t workspace_bytes, void* stream);
int tg_knn_destroy(tg_knn_handle* h);

/* Algorithm 1, initialisation: random lists, their distances, sorted, every entry "new". */
int tg_knn_init(tg_knn_handle* h);
/* Algorithm 1, phase-1 loop: one phase-1 round (sample, local join, update).  updates: host,
 * may be NULL; when given, the call waits for the round and stores the number of list
 * entries it replaced. */
int tg_knn_phase1_round(tg_knn_handle* h, int64_t* updates);
/* Phase switch: every list entry becomes "unvisited". */
int tg_knn_begin_phase2(tg_knn_handle* h);
/* Algorithm 1, phase-2 loop: one phase-2 round. */
int tg_knn_phase2_round(tg_knn_handle* h, int64_t* updates);
/* Writes the graph: with finalize = 1 distances are recomputed directly and rows re-sorted. */
int tg_knn_finalize(tg_knn_handle* h, int32_t* out_ids, float* out_dist);
/* Stats of the rounds run so far on this handle (synchronises the stream). */
int tg_knn_get_stats(tg_knn_handle* h, tg_knn_stats* out);

/* ---- state inspection, for tests of the individual steps ------------------------------ */

/* Current lists as they are (no finalize): ids n x k int32, dist n x k fp32, fresh n x k
 * uint8 (1 = new / unvisited); all device, any may be NULL. */
int tg_knn_export(tg_knn_handle* h, int32_t* ids, float* dist, uint8_t* fresh);
/* Replace the lists (rows must be sorted by (dist,id)); all device.  Ids outside [0, n) are refused
 * (checked on the host: this call synchronises the stream). */
int tg_knn_import(tg_knn_handle* h, const int32_t* ids, const float* dist, const uint8_t* fresh);
/* Step (1) of a phase-1 round on its own (section 3.1.1): draws the reverse samples of
 * the coming round and writes every anchor's block: blk device n x 128 int32 (NEW ids
 * first, then OLD ids), sizes device n x 2 int32 (|NEW|, |OLD|).  Does not advance the round. */
int tg_knn_sample_blocks(tg_knn_handle* h, int32_t* blk, int32_t* sizes);
/* Which members of the blocks last written by tg_knn_sample_blocks already sit in which member's list (the local
 * join offers no node to a list that holds it): adj device n x 128 x 4 uint32; bit x % 32 of word x / 32 of
 * entry (v, p) is set iff the node at position x of anchor v's block is in the list of the node at position p, as
 * the lists stand now.  Entries of positions beyond a block, and of anchors without a join, are 0. */
int tg_knn_block_adjacency(tg_knn_handle* h, uint32_t* adj);
/* The local join's distance tile for explicit blocks, through the same LDS/MFMA core:
 * blk device nb x 128 int32, sizes device nb x 2 (|NEW| <= 64, |NEW|+|OLD| <= 128),
 * out device nb x 64 x 128 fp32; entry (b, r, c) is dist(blk[b][r], blk[b][c]) for
 * r < |NEW|, r < c < |NEW|+|OLD|, and is left untouched elsewhere. */
int tg_knn_join_distances(tg_knn_handle* h, const int32_t* blk, const int32_t* sizes, int64_t nb,
                          float* out);

/*
 * Exact k-NN of selected rows by exhaustive search on the GPU (ground truth for the
 * recall of section 7.1).  query_rows: device int64[nq] row indices into X (NULL = rows
 * 0..nq-1); out_ids device nq x k, out_dist device nq x k (may be NULL).  Order (dist, id).
 * A row index outside [0, n) is refused (checked on the host).
 */
int tg_exact_knn(const float* X, int64_t n, int32_t d, int32_t k, int32_t metric,
                 const int64_t* query_rows, int64_t nq, int32_t* out_ids, float* out_dist,
                 void* stream);

/*
 * tg_exact_knn for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same result as tg_exact_knn, but the scratch (the
 * per-slice partial lists, and for TG_METRIC_COSINE the norms of all n rows) lives in a static device
 * array of tg_exact_knn_static_scratch_bytes() = 16 MiB that every GPU the library runs on holds until
 * the process ends.  The call allocates and frees nothing, never synchronises, and copies nothing to the
 * host; all work is enqueued on `stream`.
 *   - Needs d % 4 == 0 and a 16-byte aligned X (TG_ERR_UNSUPPORTED otherwise: the padded copy
 *     tg_exact_knn makes would have to be allocated).
 *   - Needs 8 nq k (+ 8 n for the cosine, each part rounded up to 256 bytes) <= the scratch size;
 *     larger problems are refused with TG_ERR_INVALID_ARG and a message that says how many bytes were needed.
 *   - query_rows are not checked on the host (that would need a copy and a wait): a row index outside
 *     [0, n) is no query, its output row is k times (-1, +infinity).
 *   - Every call on a GPU uses that GPU's one array and finds the previous call's contents there; each
 *     call writes every word it later reads, so nothing has to be cleared.  Calls that overlap in time
 *     on one GPU (two streams, two threads) race on it: keep them on one stream, or order them.
 */
int tg_exact_knn_static(const float* X, int64_t n, int32_t d, int32_t k, int32_t metric,
                        const int64_t* query_rows, int64_t nq, int32_t* out_ids, float* out_dist,
                        void* stream);
size_t tg_exact_knn_static_scratch_bytes(void);

/*
 * Rank-based pruning of a k-NN graph by detourable routes (section 3.2, the CAGRA row of the
 * table of pruning strategies; section 5.2).  knn_ids: device n x k int32, every row ordered
 * closest first (the output of tg_knn_build); the position of a neighbour in its row stands for
 * its distance.  For node A and its neighbour F at position p, D is a detour of the edge (A, F)
 * when D's positions in A's row and in F's row are both below p.  out_ids: device n x d_out, the
 * d_out neighbours of each row with the smallest (detour count, position), in that order;
 * out_counts: device n x k int32 detour counts by position, or NULL.  1 <= d_out <= k <= 64.
 * Ids outside [0, n) are padding: they have no detours, are no detours, and are kept or dropped
 * by their position alone.  The inputs are not modified; nothing is allocated.
 */
int tg_prune_rank(const int32_t* knn_ids, int64_t n, int32_t k, int32_t d_out, int32_t* out_ids,
                  int32_t* out_counts, void* stream);

/*
 * Distance-based pruning of a k-NN graph by the Collect-Filter-Store procedure (section 5.1), with
 * the serial rule of NSG (alpha = 1) and Vamana (alpha > 1) of section 3.2.  Squared L2 only.
 * X: device n x d fp32 row-major (any alignment; 16-byte aligned rows are faster), knn_ids: device
 * n x k int32.  For every node p:
 *   Collect: hops = 1: p's neighbours; hops = 2: those and the neighbours of each of them (rows of more
 *            than 32 ids take a slower instance of the kernel with a larger id set).
 *            p itself, ids outside [0, n) and repeats are no candidates.  The candidates are ordered
 *            by (dis(p, c), id) and the first cand_size (1..64) go on.
 *   Filter:  closest first, p' is inserted iff dis(p, p') < alpha dis(p*, p') for every p* inserted
 *            before it, until d_out (1..64) are in.  dis is the Euclidean distance: on the squared
 *            values the test is sq(p, p') < alpha^2 sq(p*, p'), taken in fp32 with
 *            sq(p*, p') = |p*|^2 + |p'|^2 - 2 <p*, p'>.
 *   Store:   out_ids device n x d_out: the inserted nodes in insertion order, then -1;
 *            out_deg device n int32: how many were inserted, or NULL.
 * The 'path' Collect of section 5.1 (candidates from a graph search) is not part of this library.
 * The inputs are not modified; nothing is allocated.  Errors: TG_ERR_INVALID_ARG for NULL or
 * out-of-range arguments.
 */
int tg_prune_dist(const float* X, int64_t n, int32_t d, const int32_t* knn_ids, int32_t k,
                  int32_t hops, int32_t cand_size, float alpha, int32_t d_out,
                  int32_t* out_ids, int32_t* out_deg, void* stream);

/*
 * Angle-based pruning of a k-NN graph by the same Collect-Filter-Store procedure (section 5.1) with
 * the serial rule of NSSG (section 3.2).  Everything is as for tg_prune_dist except the Filter:
 * closest first, p' is inserted iff the angle at p between p* and p' exceeds gamma for every p*
 * inserted before it, until d_out are in.  gamma_deg: the angle in degrees, 0 < gamma_deg <= 90
 * (60 is the usual choice).  With a = sq(p, p*), b = sq(p, p'), c = sq(p*, p') and t = (a + b) - c
 * the test is  t < 0  or  t * t < c4 * (a * b),  c4 = 4 cos^2(gamma) rounded to fp32 (exactly 0 at
 * 90 degrees), every operation in fp32 in the order written, c = |p*|^2 + |p'|^2 - 2 <p*, p'>.
 * A candidate at p's own position, or at the position of an inserted node, is never inserted.
 * Errors as for tg_prune_dist, TG_ERR_INVALID_ARG for gamma_deg outside (0, 90].
 */
int tg_prune_angle(const float* X, int64_t n, int32_t d, const int32_t* knn_ids, int32_t k,
                   int32_t hops, int32_t cand_size, float gamma_deg, int32_t d_out,
                   int32_t* out_ids, int32_t* out_deg, void* stream);

/*
 * Dispersion pruning of a k-NN graph by the same Collect-Filter-Store procedure with the rule of DPG
 * (section 3.2: the neighbours of p are to make the sum of their pairwise angles at p large, by
 * greedy insertion; section 5.1 reaches this rule with the angle metric and a threshold of 0).
 * Collect and the cut to cand_size are as for tg_prune_dist.  Filter: the nearest candidate is
 * inserted first; then, until d_out nodes are in or no candidate is left, the candidate whose
 * angles to the inserted nodes add up to the most is inserted; of equal sums the nearer candidate
 * (order (dis, id)) wins.  Nothing is dropped while there is room: with d_out >= the number of
 * candidates the row is a reordering of them.  Store: out_ids in insertion order (not by distance),
 * then -1; out_deg = min(d_out, candidates).  The angle of a pair is tg_angle_at of the squared
 * lengths sq(p, r), sq(p, c), sq(r, c); a candidate's angles are added in fp32 in insertion order.
 * Errors as for tg_prune_dist.
 */
int tg_prune_dispersion(const float* X, int64_t n, int32_t d, const int32_t* knn_ids, int32_t k,
                        int32_t hops, int32_t cand_size, int32_t d_out,
                        int32_t* out_ids, int32_t* out_deg, void* stream);

/*
 * The angle the dispersion rule uses, elementwise on device arrays of `count` values: out[i] is the
 * angle in radians at p between p -> r and p -> c for the squared lengths a[i] = |p r|^2,
 * b[i] = |p c|^2, c[i] = |r c|^2, namely acos(x) with x = ((a + b) - c) / (2 sqrt(a b)) clamped to
 * [-1, 1], and 0 when a b is not positive (a node at p's position has no direction).  The arc cosine
 * is the eight-term polynomial of Abramowitz and Stegun 4.4.46: acos(x) = sqrt(1 - x) (a0 + a1 x +
 * ... + a7 x^7) on [0, 1] (|error| <= 2e-8), pi - acos(-x) below 0; every operation is an fp32
 * operation rounded once (Horner with one fused multiply-add per coefficient), so the result can be
 * reproduced bit for bit on a host.  count = 0 is allowed.
 */
int tg_angle_at(const float* a, const float* b, const float* c, float* out, int64_t count, void* stream);

/*
 * Merge of a local index into the global neighbour lists (section 6.1: a node belongs to several
 * clusters, every cluster gets a local index, and the node's list becomes merge(list so far, its list
 * in the local index)).  g_ids, g_dist: device n x k, updated in place; an unused entry has id -1 and
 * distance +infinity (tg_lists_clear writes a whole array of them).  l_ids, l_dist: device
 * n_local x k_local, the local index in local numbering (the output of tg_knn_build on the
 * cluster's rows); local_to_global: device n_local int32, the global id of every local node, every
 * global id at most once.  For local node i with v = local_to_global[i] the row of v becomes the k
 * entries with the smallest (distance, id) of its old entries and the translated local ones; an id
 * counts once (an old entry wins over a local one, else the first in the row), v itself and ids
 * without a node are no entries, a shorter row ends in -1 / +infinity.  Rows of nodes outside the
 * cluster are not touched; a local node whose global id is outside [0, n) is skipped.
 * 1 <= k, k_local <= 64; n_local = 0 is allowed (nothing happens, the local pointers may be NULL).
 * Nothing is allocated.
 */
int tg_merge_local(int32_t* g_ids, float* g_dist, int64_t n, int32_t k, const int32_t* l_ids,
                   const float* l_dist, int64_t n_local, int32_t k_local,
                   const int32_t* local_to_global, void* stream);
/* Makes every entry of n x k lists unused (id -1, distance +infinity). */
int tg_lists_clear(int32_t* g_ids, float* g_dist, int64_t n, int32_t k, void* stream);

/* Message of the calling thread's last error (static storage, never NULL). */
const char* tg_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TAGORE_KNN_H */
