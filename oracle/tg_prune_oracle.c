/*
 * CPU oracle for the rank-based ("detourable route") pruning of a k-NN graph
 * (paper section 3.2, the CAGRA row of the table of pruning strategies, and the
 * description of its computing paradigm in section 5.2).
 *
 * THIS IS TEST INFRASTRUCTURE: a plain, slow, single-threaded definition written
 * out, used only by the test-suite.  It shares no code with the HIP library.
 *
 * Input: the graph as n rows of k ids, each row ordered closest first.  The
 * position of a neighbour in a row (1 = first) stands for its distance.
 * For node A and its neighbour F at position p, a node D is a detour of the edge
 * (A, F) when max(dis(A, D), dis(D, F)) < dis(A, F) with
 *     dis(A, D) = position of D in A's row,
 *     dis(D, F) = position of D in F's row      (section 5.2: F's row is scanned
 *                                                for nodes of A's row),
 *     dis(A, F) = p.
 * The edge's count is the number of such D.  Neighbours with more detours are
 * pruned first: the d_out neighbours with the smallest (count, position) stay,
 * written in that order.
 *
 * Pinning (tests/test_oracle_prune.py): the worked example of section 5.2, a
 * closed form on cliques, an independent path enumeration in Python, invariants.
 */
#include <stdint.h>
#include <stdlib.h>

/* Prunes the rows of nodes 0 .. n_do-1 (n_do <= n; the rest of the graph is only read).
 * counts: n_do x k (may be NULL), out_ids: n_do x d_out.  Ids outside [0, n) have no row
 * and are no nodes: they bring no detours and are no detours.  Returns 0, or -1 on bad arguments. */
int oprune_rank(const int32_t *ids, int64_t n, int64_t n_do, int k, int d_out, int32_t *out_ids, int32_t *counts)
{
    if (!ids || !out_ids || n < 1 || n_do < 0 || n_do > n || k < 1 || d_out < 1 || d_out > k) return -1;
    int32_t *cnt = (int32_t *)malloc((size_t)k * sizeof(int32_t));
    uint8_t *taken = (uint8_t *)malloc((size_t)k);
    for (int64_t a = 0; a < n_do; ++a) {
        const int32_t *NA = ids + a * k;
        for (int p = 0; p < k; ++p) {          /* p is the position minus one */
            cnt[p] = 0;
            int32_t f = NA[p];
            if (f < 0 || f >= n) continue;
            const int32_t *NF = ids + (int64_t)f * k;
            for (int r = 0; r < p; ++r) {      /* D = NF[r]: dis(D, F) = r + 1 < p + 1 */
                if (NF[r] < 0 || NF[r] >= n) continue;       /* padding is no node */
                for (int i = 0; i < p; ++i)    /* dis(A, D) = i + 1 < p + 1 */
                    if (NA[i] == NF[r]) { cnt[p]++; break; }
            }
        }
        /* keep the d_out smallest (count, position), in that order */
        for (int p = 0; p < k; ++p) taken[p] = 0;
        for (int t = 0; t < d_out; ++t) {
            int best = -1;
            for (int p = 0; p < k; ++p)
                if (!taken[p] && (best < 0 || cnt[p] < cnt[best])) best = p;
            taken[best] = 1;
            out_ids[a * d_out + t] = NA[best];
        }
        if (counts) for (int p = 0; p < k; ++p) counts[a * k + p] = cnt[p];
    }
    free(cnt); free(taken);
    return 0;
}
