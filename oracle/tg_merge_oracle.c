/*
 * CPU oracle for merging a local index into the global one (paper section 6.1: every node
 * goes to its closest clusters, each cluster gets a local index, and the merging workflow
 * replaces a node's neighbour list by merge(list so far, list in the local index)).
 *
 * THIS IS TEST INFRASTRUCTURE: a plain, slow, single-threaded definition written out,
 * used only by the test-suite.  It shares no code with the HIP library.
 *
 * Lists are k-NN lists with distances.  For local node i with global id v = l2g[i]:
 *     merge = the k entries with the smallest (distance, id) of
 *             G[v]  united with  { (l2g[c], dist) : (c, dist) in L[i] },
 * where an id counts once (an id that G[v] holds keeps G[v]'s entry; otherwise the first
 * occurrence), v itself and ids without a node are no entries, and a list shorter than k is
 * filled with id -1 and distance +infinity.  The paper does not define merge(); for lists that
 * approximate "the k nearest" this is the only reading that keeps their meaning.
 *
 * Pinning (tests/test_oracle_merge.py): overlapping intervals of a line merge into the exact
 * global lists, a hand-made example, merging in any order, merging a list with itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct { float dist; int32_t id; } ent_t;

static int ent_less(const void *pa, const void *pb)
{
    const ent_t *a = (const ent_t *)pa, *b = (const ent_t *)pb;
    if (a->dist != b->dist) return a->dist < b->dist ? -1 : 1;
    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

/* g_ids, g_dist: n x k, updated in place.  l_ids, l_dist: n_local x k_local in local numbering,
 * l2g: n_local global ids (every global id at most once).  Returns 0, or -1 on bad arguments. */
int omerge_local(int32_t *g_ids, float *g_dist, int64_t n, int k, const int32_t *l_ids, const float *l_dist,
                 int64_t n_local, int k_local, const int32_t *l2g)
{
    if (!g_ids || !g_dist || !l_ids || !l_dist || !l2g || n < 1 || k < 1 || n_local < 0 || k_local < 1) return -1;
    ent_t *e = (ent_t *)malloc((size_t)(k + k_local) * sizeof(ent_t));
    for (int64_t i = 0; i < n_local; ++i) {
        const int64_t v = l2g[i];
        if (v < 0 || v >= n) { free(e); return -1; }
        int m = 0;
        for (int j = 0; j < k + k_local; ++j) {
            int32_t id;
            float dist;
            if (j < k) { id = g_ids[v * k + j]; dist = g_dist[v * k + j]; }
            else {
                const int32_t c = l_ids[i * k_local + (j - k)];
                if (c < 0 || c >= n_local) continue;
                id = l2g[c]; dist = l_dist[i * k_local + (j - k)];
            }
            if (id < 0 || id >= n || id == v) continue;
            int seen = 0;
            for (int q = 0; q < m && !seen; ++q) seen = (e[q].id == id);
            if (seen) continue;
            e[m].id = id; e[m].dist = dist; ++m;
        }
        qsort(e, (size_t)m, sizeof(ent_t), ent_less);
        for (int j = 0; j < k; ++j) {
            g_ids[v * k + j] = j < m ? e[j].id : -1;
            g_dist[v * k + j] = j < m ? e[j].dist : INFINITY;
        }
    }
    free(e);
    return 0;
}
