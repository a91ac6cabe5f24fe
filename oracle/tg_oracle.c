/*
 * CPU oracle for the GNN-Descent k-NN graph initialisation (paper section 4,
 * Algorithm 1; NN-Descent as summarised in section 3.1.1).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded
 * reference used only by the test-suite, the smoke check and the benchmark's
 * CPU-baseline leg.  It shares no code with the HIP library and the product
 * path never calls it.  All distances are accumulated in double precision
 * from the fp32 inputs.
 *
 * Two programs live here:
 *   O-BF   obf_knn()      exact k nearest neighbours by exhaustive search
 *                         (the "ground-truth top-k" of the paper's recall
 *                         definition, section 7.1 Metrics).
 *   O-NND  onnd_*()       two-phase NN-Descent, one function per step of
 *                         Algorithm 1, in the algorithm's order.
 *
 * Where the paper leaves a choice open (sample sizes, reverse neighbours,
 * tie order, visited marks) the reading implemented here is the one the
 * repository's design notes list; every such reading is a parameter or is
 * commented where it is taken.
 *
 * The reference mode of O-NND is the plain method: every pair a block
 * evaluates is offered to both of its nodes, and a node's candidate list is
 * unbounded (retain = 0, C = 0, parts = 1).  The remaining parameters
 * (retain, tile, ng_row, ng_col, C with slot_of(), exclude_listed, parts) do
 * not belong to the method: they model a bounded hand-over of candidates from the blocks to
 * the lists, such as a device with little fast memory per block needs
 * (section 4.2 keeps one closest node per node and warp sub-tile for the same
 * reason).  They are here so that such a build can be followed step by step;
 * what they cost in quality is measured against the reference mode.
 *
 * Pinning: tests/test_oracle_*.py check O-BF against closed forms and an
 * independent full sort, and O-NND against O-BF in the cases where the
 * iteration is exact by construction (k = n-1; one round with every node in
 * every block), plus per-round invariants.  The per-round recall values and
 * update counts of the sampled heuristic itself have no published number to
 * compare against: for those, parity is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Counter-based random numbers: the SplitMix64 output function       */
/* (Steele, Lea, Flood 2014) applied three times to (seed,tag),x,y.   */
/* The HIP library implements the same published function on its own. */
/* ------------------------------------------------------------------ */
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

#define TG_GOLDEN 0x9E3779B97F4A7C15ULL

static uint64_t hash3(uint64_t seed, uint64_t tag, uint64_t x, uint64_t y)
{
    uint64_t h = mix64(seed + tag * TG_GOLDEN);
    h = mix64(h + x);
    h = mix64(h + y);
    return h;
}

/* exported so a test can check the generator against published vectors */
uint64_t oracle_mix64(uint64_t z) { return mix64(z); }
uint64_t oracle_hash3(uint64_t seed, uint64_t tag, uint64_t x, uint64_t y)
{
    return hash3(seed, tag, x, y);
}

/* tags of the three random decisions the method takes */
#define TAG_INIT 1u                       /* x = node, y = draw counter      */
#define TAG_REV(round) (2u + 4u * (uint64_t)(round))  /* x = source, y = dest */
#define TAG_SLOT(round) (3u + 4u * (uint64_t)(round)) /* x = target, y = cand */

/* ------------------------------------------------------------------ */
/* Distances.  metric 0: squared Euclidean; 1: negative inner product; */
/* 2: one minus cosine.  (The paper never names its "dis"; these are   */
/* the three the boundary offers.)                                     */
/* ------------------------------------------------------------------ */
static double distance(const float *X, int64_t d, int metric, int64_t a, int64_t b)
{
    const float *x = X + a * d, *y = X + b * d;
    double s = 0.0;
    if (metric == 0) {
        for (int64_t j = 0; j < d; ++j) {
            double t = (double)x[j] - (double)y[j];
            s += t * t;
        }
        return s;
    }
    double xx = 0.0, yy = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        s += (double)x[j] * (double)y[j];
        xx += (double)x[j] * (double)x[j];
        yy += (double)y[j] * (double)y[j];
    }
    if (metric == 1) return -s;
    return 1.0 - s / sqrt(xx * yy);
}

double oracle_distance(const float *X, int64_t d, int metric, int64_t a, int64_t b)
{
    return distance(X, d, metric, a, b);
}

/* total order used everywhere: distance first, then id */
static int key_less(double da, int32_t ia, double db, int32_t ib)
{
    return da < db || (da == db && ia < ib);
}

/* ------------------------------------------------------------------ */
/* O-BF: exhaustive exact k-NN for the listed rows                     */
/* ------------------------------------------------------------------ */
int obf_knn(const float *X, int64_t n, int64_t d, int k, int metric,
            const int64_t *rows, int64_t nq, int32_t *out_ids, double *out_dist)
{
    if (k < 1 || k >= n) return -1;
    for (int64_t q = 0; q < nq; ++q) {
        int64_t i = rows ? rows[q] : q;
        int32_t *ids = out_ids + q * k;
        double *ds = out_dist + q * k;
        int cnt = 0;
        for (int64_t j = 0; j < n; ++j) {
            if (j == i) continue;
            double dj = distance(X, d, metric, i, j);
            if (cnt == k && !key_less(dj, (int32_t)j, ds[k - 1], ids[k - 1])) continue;
            int p = cnt < k ? cnt : k - 1;          /* insertion sort step */
            while (p > 0 && key_less(dj, (int32_t)j, ds[p - 1], ids[p - 1])) {
                ds[p] = ds[p - 1];
                ids[p] = ids[p - 1];
                --p;
            }
            ds[p] = dj;
            ids[p] = (int32_t)j;
            if (cnt < k) ++cnt;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* O-NND state                                                         */
/* ------------------------------------------------------------------ */
typedef struct {
    double dist;
    int32_t id;
    uint8_t fresh;   /* phase 1: "new" (not yet sampled); phase 2: "unvisited" */
} entry_t;

typedef struct {
    double dist;
    int32_t id;
} cand_t;

typedef struct {
    cand_t *v;
    int64_t len, cap;
} candvec_t;

typedef struct {
    /* problem */
    const float *X;
    int64_t n, d;
    int k, metric;
    /* readings of the open choices */
    int S;            /* forward sample cap per class                          */
    int R;            /* reverse sample cap per class                          */
    int C;            /* candidate slots per node per round; 0 = unbounded     */
    int retain;       /* 0: offer every pair under the threshold
                         1: per target and opponent group keep the closest     */
    int tile;         /* opponent positions are grouped as (pos / tile) % ng   */
    int ng_row;       /* groups of row opponents (seen by a column target)     */
    int ng_col;       /* groups of column opponents (seen by a row target)     */
    int m;            /* neighbours expanded per node per phase-2 round        */
    int all_block;    /* 1: every anchor's block is all of V, all new          */
    int use_threshold;/* 0 switches off the early threshold test (the merge
                         then discards the same candidates)                    */
    int exclude_listed;/* 1: a node that the target's list already holds is no
                         candidate where the pair is met (the merge would drop
                         it anyway; with retention it matters, because such a
                         node would otherwise take the place of a useful one)  */
    int parts;        /* a phase-1 round is carried out in this many parts:
                         part p joins the blocks of the anchors v = p mod parts,
                         and the lists are updated after every part            */
    uint64_t seed;
    /* state */
    entry_t *G;       /* n x k, each row sorted by (dist, id)                  */
    int round;        /* rounds executed so far, both phases                   */
    /* per-round scratch */
    int32_t *new_fwd, *old_fwd;   /* n x S forward samples of this round      */
    int *n_new, *n_old;           /* their lengths                            */
    int32_t *new_rev, *old_rev;   /* n x R reverse samples of this round      */
    int *n_new_rev, *n_old_rev;
    uint8_t *sampled;             /* n x k: entry was taken as a new sample   */
    cand_t *slots;    /* n x C when C > 0                                      */
    candvec_t *bag;   /* n vectors when C == 0                                 */
    /* counters of the last round */
    int64_t pairs, offered, updates;
} onnd_t;

static void bag_push(candvec_t *b, double dist, int32_t id)
{
    if (b->len == b->cap) {
        b->cap = b->cap ? 2 * b->cap : 16;
        b->v = (cand_t *)realloc(b->v, (size_t)b->cap * sizeof(cand_t));
    }
    b->v[b->len].dist = dist;
    b->v[b->len].id = id;
    b->len++;
}

void *onnd_create(const float *X, int64_t n, int64_t d, int k, int metric,
                  int S, int R, int C, int retain, int tile, int ng_row, int ng_col,
                  int m, int all_block, int use_threshold, int exclude_listed, int parts, uint64_t seed)
{
    if (k < 1 || k >= n || (C & (C - 1)) != 0 || parts < 1) return NULL;
    onnd_t *o = (onnd_t *)calloc(1, sizeof(onnd_t));
    o->X = X; o->n = n; o->d = d; o->k = k; o->metric = metric;
    o->S = S; o->R = R; o->C = C; o->retain = retain; o->tile = tile;
    o->ng_row = ng_row; o->ng_col = ng_col; o->m = m;
    o->all_block = all_block; o->use_threshold = use_threshold; o->seed = seed;
    o->exclude_listed = exclude_listed; o->parts = parts;
    o->G = (entry_t *)calloc((size_t)(n * k), sizeof(entry_t));
    if (C > 0) o->slots = (cand_t *)malloc((size_t)(n * C) * sizeof(cand_t));
    else o->bag = (candvec_t *)calloc((size_t)n, sizeof(candvec_t));
    if (!all_block) {
        o->new_fwd = (int32_t *)malloc((size_t)(n * S) * sizeof(int32_t));
        o->old_fwd = (int32_t *)malloc((size_t)(n * S) * sizeof(int32_t));
        o->new_rev = (int32_t *)malloc((size_t)(n * R) * sizeof(int32_t));
        o->old_rev = (int32_t *)malloc((size_t)(n * R) * sizeof(int32_t));
        o->n_new = (int *)calloc((size_t)n, sizeof(int));
        o->n_old = (int *)calloc((size_t)n, sizeof(int));
        o->n_new_rev = (int *)calloc((size_t)n, sizeof(int));
        o->n_old_rev = (int *)calloc((size_t)n, sizeof(int));
        o->sampled = (uint8_t *)calloc((size_t)(n * k), 1);
    }
    return o;
}

void onnd_destroy(void *h)
{
    onnd_t *o = (onnd_t *)h;
    if (!o) return;
    if (o->bag) for (int64_t i = 0; i < o->n; ++i) free(o->bag[i].v);
    free(o->new_fwd); free(o->old_fwd); free(o->new_rev); free(o->old_rev);
    free(o->n_new); free(o->n_old); free(o->n_new_rev); free(o->n_old_rev); free(o->sampled);
    free(o->bag); free(o->slots); free(o->G); free(o);
}

void onnd_export(void *h, int32_t *ids, double *dist, uint8_t *fresh)
{
    onnd_t *o = (onnd_t *)h;
    for (int64_t i = 0; i < o->n * o->k; ++i) {
        if (ids) ids[i] = o->G[i].id;
        if (dist) dist[i] = o->G[i].dist;
        if (fresh) fresh[i] = o->G[i].fresh;
    }
}

/* Overwrite the graph state (rows must be sorted by (dist, id)); lets a test
 * start from a chosen graph. */
void onnd_import(void *h, const int32_t *ids, const double *dist, const uint8_t *fresh)
{
    onnd_t *o = (onnd_t *)h;
    for (int64_t i = 0; i < o->n * o->k; ++i) {
        o->G[i].id = ids[i]; o->G[i].dist = dist[i]; o->G[i].fresh = fresh[i];
    }
}

void onnd_counters(void *h, int64_t *out3)
{
    onnd_t *o = (onnd_t *)h;
    out3[0] = o->pairs; out3[1] = o->offered; out3[2] = o->updates;
}

static int entry_cmp(const void *a, const void *b)
{
    const entry_t *x = (const entry_t *)a, *y = (const entry_t *)b;
    if (key_less(x->dist, x->id, y->dist, y->id)) return -1;
    if (key_less(y->dist, y->id, x->dist, x->id)) return 1;
    return 0;
}

static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (key_less(x->dist, x->id, y->dist, y->id)) return -1;
    if (key_less(y->dist, y->id, x->dist, x->id)) return 1;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Algorithm 1, initialisation: random neighbour lists.                */
/* Node v draws ids  floor(n * U_t)  for t = 0,1,2,...  and keeps the  */
/* first k that differ from v and from each other; their distances are */
/* computed, the list is sorted, and every entry starts as "new".      */
/* ------------------------------------------------------------------ */
void onnd_init(void *h)
{
    onnd_t *o = (onnd_t *)h;
    for (int64_t v = 0; v < o->n; ++v) {
        entry_t *L = o->G + v * o->k;
        int cnt = 0;
        for (uint64_t t = 0; cnt < o->k; ++t) {
            uint64_t u32 = hash3(o->seed, TAG_INIT, (uint64_t)v, t) >> 32;
            int32_t c = (int32_t)((u32 * (uint64_t)o->n) >> 32);
            int dup = (c == v);
            for (int j = 0; j < cnt && !dup; ++j) dup = (L[j].id == c);
            if (dup) continue;
            L[cnt].id = c;
            L[cnt].dist = distance(o->X, o->d, o->metric, v, c);
            L[cnt].fresh = 1;
            ++cnt;
        }
        qsort(L, (size_t)o->k, sizeof(entry_t), entry_cmp);
    }
    o->round = 0;
}

/* ------------------------------------------------------------------ */
/* Candidate hand-over (the "candidate list" of section 4.2).          */
/* ------------------------------------------------------------------ */
static void clear_candidates(onnd_t *o)
{
    if (o->C > 0) {
        for (int64_t i = 0; i < o->n * o->C; ++i) { o->slots[i].id = -1; o->slots[i].dist = 0.0; }
    } else {
        for (int64_t i = 0; i < o->n; ++i) o->bag[i].len = 0;
    }
}

/* Slot of a candidate at target t that anchor v's block found in opponent group g.
 * The C slots of t are C/8 lines of 8; the pair (t, v) picks its line and a rotation from
 * a 32-bit multiply-xorshift hash of v plus a per-(round, target) salt (tagged hash), and
 * group g takes word (g + rotation) mod 8 of that line. */
static uint32_t slot_of(uint64_t seed, int round, int32_t t, int32_t v, int g, int C)
{
    uint32_t salt = (uint32_t)mix64(mix64(seed + TAG_SLOT(round) * TG_GOLDEN) + (uint64_t)t);
    uint32_t h = ((uint32_t)v + salt) * 0x9E3779B1u;
    h ^= h >> 15;
    h *= 0x85EBCA77u;
    h ^= h >> 13;
    int bits = 0;
    while ((8 << bits) < C) ++bits;
    uint32_t line = bits ? h >> (32 - bits) : 0u;
    return line * 8u + (((uint32_t)g + (h & 7u)) & 7u);
}
uint32_t oracle_slot_of(uint64_t seed, int round, int32_t t, int32_t v, int g, int C) { return slot_of(seed, round, t, v, g, C); }

/* A candidate c for target t, found by anchor v's block in opponent group g.  With bounded
 * storage it goes to slot_of(round, t, v, g) and a slot keeps the smaller (dist, id); the
 * same candidate may reach t through several blocks and then sits in several slots (the
 * list update drops the repeats). */
static void emit(onnd_t *o, int32_t t, int32_t c, double dist, int32_t v, int g)
{
    o->offered++;
    if (o->C == 0) { bag_push(&o->bag[t], dist, c); return; }
    uint32_t s = slot_of(o->seed, o->round, t, v, g, o->C);
    cand_t *slot = o->slots + (int64_t)t * o->C + (int64_t)s;
    if (slot->id < 0 || key_less(dist, c, slot->dist, slot->id)) { slot->dist = dist; slot->id = c; }
}

/* Is c, at this distance, a candidate for t's list?  Threshold of section 4.2:
 * only candidates that would precede the last entry of the target's current
 * list are kept; and (exclude_listed) a node the list holds is none. */
static int passes(const onnd_t *o, int32_t t, int32_t c, double dist)
{
    if (o->exclude_listed) {
        const entry_t *L = o->G + (int64_t)t * o->k;
        for (int q = 0; q < o->k; ++q) if (L[q].id == c) return 0;
    }
    if (!o->use_threshold) return 1;
    const entry_t *last = o->G + (int64_t)t * o->k + (o->k - 1);
    return key_less(dist, c, last->dist, last->id);
}

/* ------------------------------------------------------------------ */
/* Neighbour-list update (section 4.2, last paragraph): sort the       */
/* candidates, drop ids the list already holds, merge the two sorted   */
/* sequences, keep the first k; inserted entries are "new".            */
/* Returns how many candidates ended up in the list.                   */
/* ------------------------------------------------------------------ */
static int64_t merge_list(entry_t *L, int k, int64_t t, cand_t *cands, int64_t nc)
{
    qsort(cands, (size_t)nc, sizeof(cand_t), cand_cmp);
    entry_t *M = (entry_t *)malloc((size_t)(k + nc) * sizeof(entry_t));
    int64_t len = 0, i = 0, j = 0, inserted = 0;
    while ((i < k || j < nc) && len < k) {
        if (j < nc) {
            /* skip ids that are the node itself, already listed, or repeated */
            int skip = (cands[j].id == (int32_t)t);
            for (int q = 0; q < k && !skip; ++q) skip = (L[q].id == cands[j].id);
            for (int64_t q = 0; q < len && !skip; ++q) skip = (M[q].id == cands[j].id);
            if (skip) { ++j; continue; }
        }
        int take_list = (j >= nc) || (i < k && key_less(L[i].dist, L[i].id, cands[j].dist, cands[j].id));
        if (take_list) {
            M[len++] = L[i++];
        } else {
            M[len].dist = cands[j].dist; M[len].id = cands[j].id; M[len].fresh = 1;
            ++len; ++j; ++inserted;
        }
    }
    memcpy(L, M, (size_t)k * sizeof(entry_t));
    free(M);
    return inserted;
}

/* The update rule on caller-supplied arrays (for direct testing). */
int64_t oracle_merge_list(int k, int64_t self, int32_t *ids, double *dist, uint8_t *fresh,
                          const int32_t *cid, const double *cdist, int64_t nc)
{
    entry_t *L = (entry_t *)malloc((size_t)k * sizeof(entry_t));
    for (int i = 0; i < k; ++i) { L[i].id = ids[i]; L[i].dist = dist[i]; L[i].fresh = fresh[i]; }
    cand_t *c = (cand_t *)malloc((size_t)(nc ? nc : 1) * sizeof(cand_t));
    for (int64_t j = 0; j < nc; ++j) { c[j].id = cid[j]; c[j].dist = cdist[j]; }
    int64_t ins = merge_list(L, k, self, c, nc);
    for (int i = 0; i < k; ++i) { ids[i] = L[i].id; dist[i] = L[i].dist; fresh[i] = L[i].fresh; }
    free(c); free(L);
    return ins;
}

static int64_t merge_all(onnd_t *o)
{
    int64_t updates = 0;
    cand_t *tmp = (cand_t *)malloc((size_t)(o->C > 0 ? o->C : 1) * sizeof(cand_t));
    for (int64_t t = 0; t < o->n; ++t) {
        if (o->C > 0) {
            int64_t nc = 0;
            for (int s = 0; s < o->C; ++s)
                if (o->slots[t * o->C + s].id >= 0) tmp[nc++] = o->slots[t * o->C + s];
            updates += merge_list(o->G + t * o->k, o->k, t, tmp, nc);
        } else {
            updates += merge_list(o->G + t * o->k, o->k, t, o->bag[t].v, o->bag[t].len);
        }
    }
    free(tmp);
    return updates;
}

/* ------------------------------------------------------------------ */
/* Phase 1 round (Algorithm 1, first loop; steps (1)-(3) of 3.1.1).    */
/* ------------------------------------------------------------------ */
typedef struct { uint32_t prio; int32_t src; } rev_t;

static int rev_cmp(const void *a, const void *b)
{
    const rev_t *x = (const rev_t *)a, *y = (const rev_t *)b;
    if (x->prio != y->prio) return x->prio < y->prio ? -1 : 1;
    return (x->src > y->src) - (x->src < y->src);
}

typedef struct { rev_t *v; int64_t len, cap; } revvec_t;

static void rev_push(revvec_t *r, uint32_t prio, int32_t src)
{
    if (r->len == r->cap) {
        r->cap = r->cap ? 2 * r->cap : 16;
        r->v = (rev_t *)realloc(r->v, (size_t)r->cap * sizeof(rev_t));
    }
    r->v[r->len].prio = prio; r->v[r->len].src = src; r->len++;
}

static int contains(const int32_t *a, int na, int32_t x)
{
    for (int i = 0; i < na; ++i) if (a[i] == x) return 1;
    return 0;
}

/* The local join of one block.  Positions 0..nN-1 are the NEW nodes,
 * nN..nN+nO-1 the OLD nodes.  Every pair (a,b), a<b, with a NEW is
 * evaluated once; both endpoints are targets of the result. */
static void local_join(onnd_t *o, int32_t v, const int32_t *blk, int nN, int nO)
{
    int nT = nN + nO;
    if (nN == 0 || nT < 2) return;
    if (o->retain == 0) {
        for (int a = 0; a < nN; ++a)
            for (int b = a + 1; b < nT; ++b) {
                double dist = distance(o->X, o->d, o->metric, blk[a], blk[b]);
                o->pairs++;
                if (passes(o, blk[a], blk[b], dist)) emit(o, blk[a], blk[b], dist, v, (b / o->tile) % 8);
                if (passes(o, blk[b], blk[a], dist)) emit(o, blk[b], blk[a], dist, v, (a / o->tile) % 8);
            }
        return;
    }
    /* Retention (section 4.2: one closest node per node and warp sub-tile).
     * A row target a keeps, for each group of column positions, the closest
     * column node; a column target b keeps, for each group of row positions,
     * the closest row node.  Group of a position p: (p / tile) mod ng. */
    int ngc = o->ng_col, ngr = o->ng_row;
    cand_t *best_row = (cand_t *)malloc((size_t)nN * ngc * sizeof(cand_t)); /* target = row a */
    cand_t *best_col = (cand_t *)malloc((size_t)nT * ngr * sizeof(cand_t)); /* target = col b */
    for (int i = 0; i < nN * ngc; ++i) best_row[i].id = -1;
    for (int i = 0; i < nT * ngr; ++i) best_col[i].id = -1;
    for (int a = 0; a < nN; ++a)
        for (int b = a + 1; b < nT; ++b) {
            double dist = distance(o->X, o->d, o->metric, blk[a], blk[b]);
            o->pairs++;
            if (passes(o, blk[a], blk[b], dist)) {
                cand_t *s = best_row + a * ngc + (b / o->tile) % ngc;
                if (s->id < 0 || key_less(dist, blk[b], s->dist, s->id)) { s->dist = dist; s->id = blk[b]; }
            }
            if (passes(o, blk[b], blk[a], dist)) {
                cand_t *s = best_col + b * ngr + (a / o->tile) % ngr;
                if (s->id < 0 || key_less(dist, blk[a], s->dist, s->id)) { s->dist = dist; s->id = blk[a]; }
            }
        }
    for (int a = 0; a < nN; ++a)
        for (int g = 0; g < ngc; ++g)
            if (best_row[a * ngc + g].id >= 0) emit(o, blk[a], best_row[a * ngc + g].id, best_row[a * ngc + g].dist, v, g);
    for (int b = 0; b < nT; ++b)
        for (int g = 0; g < ngr; ++g)
            if (best_col[b * ngr + g].id >= 0) emit(o, blk[b], best_col[b * ngr + g].id, best_col[b * ngr + g].dist, v, g);
    free(best_row); free(best_col);
}

/* Step (1) of a phase-1 round: the shared samples of every anchor. */
void onnd_phase1_sample(void *h)
{
    onnd_t *o = (onnd_t *)h;
    int64_t n = o->n;
    int k = o->k, S = o->S, R = o->R;
    /* forward samples: the first S new and the first S old entries of each
     * list, in list order (closest first). */
    memset(o->sampled, 0, (size_t)(n * k));
    for (int64_t v = 0; v < n; ++v) {
        o->n_new[v] = o->n_old[v] = 0;
        for (int j = 0; j < k; ++j) {
            entry_t *e = o->G + v * k + j;
            if (e->fresh) {
                if (o->n_new[v] < S) { o->new_fwd[v * S + o->n_new[v]++] = e->id; o->sampled[v * k + j] = 1; }
            } else if (o->n_old[v] < S) o->old_fwd[v * S + o->n_old[v]++] = e->id;
        }
    }
    /* reverse samples: u receives v for every sampled edge v -> u; of more
     * than R arrivals the R with the smallest (priority, source) stay, in
     * that order, where priority = hash(round, source, dest): a uniform
     * subset that does not depend on the order of arrival. */
    revvec_t *rn = (revvec_t *)calloc((size_t)n, sizeof(revvec_t));
    revvec_t *ro = (revvec_t *)calloc((size_t)n, sizeof(revvec_t));
    for (int64_t v = 0; v < n; ++v) {
        for (int j = 0; j < o->n_new[v]; ++j) {
            int32_t u = o->new_fwd[v * S + j];
            rev_push(&rn[u], (uint32_t)(hash3(o->seed, TAG_REV(o->round), (uint64_t)v, (uint64_t)u) >> 32), (int32_t)v);
        }
        for (int j = 0; j < o->n_old[v]; ++j) {
            int32_t u = o->old_fwd[v * S + j];
            rev_push(&ro[u], (uint32_t)(hash3(o->seed, TAG_REV(o->round), (uint64_t)v, (uint64_t)u) >> 32), (int32_t)v);
        }
    }
    for (int64_t u = 0; u < n; ++u) {
        qsort(rn[u].v, (size_t)rn[u].len, sizeof(rev_t), rev_cmp);
        qsort(ro[u].v, (size_t)ro[u].len, sizeof(rev_t), rev_cmp);
        o->n_new_rev[u] = (int)(rn[u].len > R ? R : rn[u].len);
        o->n_old_rev[u] = (int)(ro[u].len > R ? R : ro[u].len);
        for (int j = 0; j < o->n_new_rev[u]; ++j) o->new_rev[u * R + j] = rn[u].v[j].src;
        for (int j = 0; j < o->n_old_rev[u]; ++j) o->old_rev[u * R + j] = ro[u].v[j].src;
        free(rn[u].v); free(ro[u].v);
    }
    free(rn); free(ro);
}

/* The block of anchor v from the current samples:
 * NEW = new_fwd ++ (new_rev not yet there);
 * OLD = (old_fwd not in NEW) ++ (old_rev in neither).
 * blk must hold 2S+2R ids; sizes[0] = |NEW|, sizes[1] = |OLD|. */
void onnd_block(void *h, int64_t v, int32_t *blk, int *sizes)
{
    onnd_t *o = (onnd_t *)h;
    int S = o->S, R = o->R, nN = 0;
    for (int j = 0; j < o->n_new[v]; ++j) blk[nN++] = o->new_fwd[v * S + j];
    for (int j = 0; j < o->n_new_rev[v]; ++j)
        if (!contains(blk, nN, o->new_rev[v * R + j])) blk[nN++] = o->new_rev[v * R + j];
    int nT = nN;
    for (int j = 0; j < o->n_old[v]; ++j)
        if (!contains(blk, nT, o->old_fwd[v * S + j])) blk[nT++] = o->old_fwd[v * S + j];
    for (int j = 0; j < o->n_old_rev[v]; ++j)
        if (!contains(blk, nT, o->old_rev[v * R + j])) blk[nT++] = o->old_rev[v * R + j];
    sizes[0] = nN; sizes[1] = nT - nN;
}

int64_t onnd_phase1_round(void *h)
{
    onnd_t *o = (onnd_t *)h;
    int64_t n = o->n;
    int k = o->k;
    o->pairs = o->offered = o->updates = 0;
    clear_candidates(o);

    if (o->all_block) {
        /* pin mode: every node meets every other node as NEW */
        int32_t *all = (int32_t *)malloc((size_t)n * sizeof(int32_t));
        for (int64_t i = 0; i < n; ++i) all[i] = (int32_t)i;
        local_join(o, 0, all, (int)n, 0);
        free(all);
        for (int64_t i = 0; i < n * k; ++i) o->G[i].fresh = 0;
        o->updates = merge_all(o);
        o->round++;
        return o->updates;
    }

    /* (1) sample: the blocks of the whole round are fixed here */
    onnd_phase1_sample(h);
    int bw = 2 * o->S + 2 * o->R;
    int32_t *blk = (int32_t *)malloc((size_t)n * bw * sizeof(int32_t));
    int *sizes = (int *)malloc((size_t)n * 2 * sizeof(int));
    for (int64_t v = 0; v < n; ++v) onnd_block(h, v, blk + v * bw, sizes + v * 2);

    /* sampled new entries become old (3.1.1: previously sampled nodes are
     * labelled old) */
    for (int64_t i = 0; i < n * k; ++i) if (o->sampled[i]) o->G[i].fresh = 0;

    for (int p = 0; p < o->parts; ++p) {
        if (p) clear_candidates(o);
        /* (2) local join per anchor of this part */
        for (int64_t v = p; v < n; v += o->parts)
            local_join(o, (int32_t)v, blk + v * bw, sizes[v * 2], sizes[v * 2 + 1]);
        /* (3) update */
        o->updates += merge_all(o);
    }
    free(blk); free(sizes);
    o->round++;
    return o->updates;
}

/* Phase switch: phase 2 starts with every list entry unvisited. */
void onnd_begin_phase2(void *h)
{
    onnd_t *o = (onnd_t *)h;
    for (int64_t i = 0; i < o->n * o->k; ++i) o->G[i].fresh = 1;
}

/* ------------------------------------------------------------------ */
/* Phase 2 round (Algorithm 1, second loop): node v expands its first m */
/* unvisited neighbours u, reads G[u] as it stood when the round began,*/
/* measures v against those nodes, and updates G[v] only.              */
/* ------------------------------------------------------------------ */
int64_t onnd_phase2_round(void *h)
{
    onnd_t *o = (onnd_t *)h;
    int64_t n = o->n;
    int k = o->k;
    o->pairs = o->offered = o->updates = 0;
    int32_t *snap = (int32_t *)malloc((size_t)(n * k) * sizeof(int32_t));
    for (int64_t i = 0; i < n * k; ++i) snap[i] = o->G[i].id;
    cand_t *cands = (cand_t *)malloc((size_t)(o->m * k) * sizeof(cand_t));
    for (int64_t v = 0; v < n; ++v) {
        entry_t *L = o->G + v * k;
        int64_t nc = 0;
        int expanded = 0;
        for (int j = 0; j < k && expanded < o->m; ++j) {
            if (!L[j].fresh) continue;
            L[j].fresh = 0;                      /* non-revisitation */
            ++expanded;
            const int32_t *Nu = snap + (int64_t)L[j].id * k;
            for (int q = 0; q < k; ++q) {
                int32_t c = Nu[q];
                int skip = (c == (int32_t)v);
                for (int p = 0; p < k && !skip; ++p) skip = (L[p].id == c);
                for (int64_t p = 0; p < nc && !skip; ++p) skip = (cands[p].id == c);
                if (skip) continue;
                double dist = distance(o->X, o->d, o->metric, v, c);
                o->pairs++;
                if (passes(o, (int32_t)v, c, dist)) { cands[nc].dist = dist; cands[nc].id = c; ++nc; o->offered++; }
                else { cands[nc].dist = INFINITY; cands[nc].id = c; ++nc; } /* remembered only to skip repeats */
            }
        }
        /* drop the placeholders of rejected candidates */
        int64_t w = 0;
        for (int64_t p = 0; p < nc; ++p) if (cands[p].dist != INFINITY) cands[w++] = cands[p];
        o->updates += merge_list(L, k, v, cands, w);
    }
    free(cands); free(snap);
    o->round++;
    return o->updates;
}

/* Whole Algorithm 1 with optional early stop: a phase ends early when a
 * round changes fewer than delta*n*k entries.  rounds_done[0..1] receive the
 * rounds run in each phase. */
void onnd_run(void *h, int it1, int it2, double delta, int *rounds_done)
{
    onnd_t *o = (onnd_t *)h;
    double stop = delta * (double)o->n * (double)o->k;
    onnd_init(h);
    int r1 = 0, r2 = 0;
    for (; r1 < it1;) { int64_t u = onnd_phase1_round(h); ++r1; if ((double)u < stop) break; }
    onnd_begin_phase2(h);
    for (; r2 < it2;) { int64_t u = onnd_phase2_round(h); ++r2; if ((double)u < stop) break; }
    if (rounds_done) { rounds_done[0] = r1; rounds_done[1] = r2; }
}

/* recall of section 7.1: |G ∩ R| / k averaged over the listed rows */
double oracle_recall(const int32_t *ids, const int32_t *truth, int64_t nq, int k)
{
    int64_t hit = 0;
    for (int64_t q = 0; q < nq; ++q)
        for (int i = 0; i < k; ++i)
            for (int j = 0; j < k; ++j)
                if (ids[q * k + i] == truth[q * k + j]) { ++hit; break; }
    return (double)hit / ((double)nq * k);
}
