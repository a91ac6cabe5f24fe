// Host-callable launchers of the gfx950 kernels (internal; the public boundary is
// include/tagore_knn.h).  Every launcher only enqueues work on `stream`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define TG_BLOCK_COLS 128   // a join block holds at most 64 NEW rows and 128 rows in total
#define TG_BLOCK_ROWS 64
#define TG_STAT_BINS 1024   // spread of the per-round statistics counters
#define TG_MAX_PARTS 8      // a phase-1 round is carried out in at most this many parts
#define TG_WL_LISTS (3 * TG_MAX_PARTS)   // join work lists of a round: one per part and block-size class

// One launch carries fewer than 2^32 work-items.  Kernels that give every node a wave (or a group
// of lanes) of its own are therefore launched once per chunk of TG_LAUNCH_NODES nodes and told
// where their chunk begins; the chunk size is a multiple of every such group size.
#define TG_LAUNCH_NODES (1ll << 24)
#define TG_RANGE_NONINT 8        // word of the range buffer: set when a value of X is not a whole number
#define TG_REV_BUCKETS 8192      // buckets of reverse edges one launch counts in LDS
#define TG_REV_MAX_SHIFT 11      // a bucket holds at most 2048 targets
#define TG_REV_MAX_W (1 << TG_REV_MAX_SHIFT)
template <class F>
static inline void tg_for_node_chunks(int64_t n, F launch)
{
    for (int64_t v0 = 0; v0 < n; v0 += TG_LAUNCH_NODES) launch(v0, n - v0 < TG_LAUNCH_NODES ? n - v0 : TG_LAUNCH_NODES);
}

struct TgGraph {
    int64_t n;
    int32_t d;        // logical dimension
    int32_t ld;       // row stride of X in floats, multiple of 4, columns d..ld-1 are zero
    int32_t k;
    int32_t metric;
    const float* X;
    float* nrm;       // n: squared norms
    float* rnorm;     // n: 1/|x| (cosine only, else unused)
    uint32_t* gid;    // n x k list words of the current round: id | fresh << 31
    uint32_t* gid_next; // n x k, written by a phase-2 round
    float* gdist;     // n x k
    unsigned long long* kth;   // n: what the join needs of a node besides its vector: ordered distance of its list's last entry
                               // (high word), bits of its squared norm, or inverse norm for cosine (low word)
    const uint8_t* Xq;  // n x ldq bytes: 8-bit codes of every row (phase-2 screening), or null
    const float* Xqm;   // the grid of the codes, three words: ordered bits of the smallest and of the largest value of X, float
                        // bits of the largest distance of a row from its grid point
    int32_t ldq;        // d rounded up to 16: a row of codes never straddles more lines than it must
    const uint16_t* Xh; // n x ldh: the rows rounded to fp16 for the local join, or null (join in fp32)
    int32_t ldh;        // 64, 96 or 128 (the smallest that holds d), d rounded up to 32 beyond: columns d..ldh-1 are zero
    const uint32_t* f16_ok; // device flag, or null: 1 while every value of X has turned out to be an fp16 number.  When set,
                            // both variants of the join are launched and the one the flag does not name ends at once
};

struct TgSample {
    int32_t S, R;
    int32_t bshift;           // reverse edges are brought together in buckets of 2^bshift consecutive targets
    int64_t nbuckets;         // ceil(n / 2^bshift)
    uint32_t* bcnt;           // nbuckets: edges per bucket while a round's reverse samples are built, zero otherwise
    unsigned long long* boff; // nbuckets + 1: where each bucket's edges begin
    unsigned long long* ebuf; // n x k: the sampled edges by bucket, target % 2^bshift << 32 | class << 31 | source
    uint32_t* csr;            // n x k: the same by target, class << 31 | source
    int32_t BC;               // row stride of blk: min(k, 2S) + 2R rounded up to 16
    uint32_t* blk;            // n x BC: this round's block of every anchor, NEW ids then OLD ids
    uint32_t* bsz;            // n: |NEW| | (|NEW|+|OLD|) << 8
    unsigned long long* wl;   // 3 x (n + TG_MAX_PARTS): this round's join work lists (anchor | sizes), by part of the round and block size
    uint32_t* wl_cnt;         // TG_WL_LISTS: their lengths
    unsigned long long* scan_tmp; // block sums of the prefix sum over the buckets
    int32_t parts, parts_shift;   // a round's anchors are joined in `parts` = 1 << parts_shift parts: v goes to part v % parts, slot v / parts
    uint32_t* adj;                // ceil(n / parts) x BC x adj_words: of the part in hand, per anchor slot and member, bit x = the
    int32_t adj_words;            // node at block position x is in that member's list already (2 words for blocks of at most 64, else 4)
};

struct TgCand {
    int32_t C;
    unsigned long long* slots;   // n x C keys, TG_EMPTY_KEY when free
};

// range: two words for the smallest and largest value of X, or NULL; undefined: one word that counts the rows without a defined distance, or NULL
void tg_launch_norms(const TgGraph& g, uint32_t* range, uint32_t* undefined, hipStream_t s);
void tg_launch_init(const TgGraph& g, uint64_t hs_init, hipStream_t s);
void tg_launch_quantize(const TgGraph& g, uint8_t* Xq, float* Xqm, hipStream_t s);
void tg_launch_narrow(const TgGraph& g, uint16_t* Xh, uint32_t* exact_flag /* cleared when a value is no fp16 number, or null */,
                      uint32_t* overflow_rows /* counts the rows with a finite value beyond fp16's range, or null */, hipStream_t s);
void tg_launch_fill_u64(unsigned long long* p, size_t count, unsigned long long v, hipStream_t s);
void tg_launch_fill_u32(uint32_t* p, size_t count, uint32_t v, hipStream_t s);
void tg_launch_reverse(const TgGraph& g, const TgSample& sm, uint64_t hs_rev, hipStream_t s);
int tg_rev_bucket_shift(int64_t n);
// work lists of the coming round from the stored blocks: anchor v goes to part v mod parts
void tg_launch_bin(const TgGraph& g, const TgSample& sm, int parts, hipStream_t s);
// which members of a block sit in which member's list, for the anchors of one part: sm.adj (to run before tg_launch_join of that part);
// the same, copied to n x 128 x 4 words for inspection
void tg_launch_adj(const TgGraph& g, const TgSample& sm, int part, hipStream_t s);
void tg_launch_dump_adj(const TgGraph& g, const TgSample& sm, int part, uint32_t* out, hipStream_t s);
// local join of the blocks of one part (sm.parts parts in all)
void tg_launch_join(const TgGraph& g, const TgSample& sm, const TgCand& c, int part, int parts,
                    uint64_t hs_slot, unsigned long long* stat_bins /* 2 x TG_STAT_BINS or null */,
                    hipStream_t s);
void tg_launch_dump_blocks(const TgGraph& g, const TgSample& sm, int32_t* blk, int32_t* sizes, hipStream_t s);
void tg_launch_join_distances(const TgGraph& g, const int32_t* blk, const int32_t* sizes, int64_t nb,
                              float* out, hipStream_t s);
// flip: the entries sampled as new for this round become old (first update of a round)
void tg_launch_update(const TgGraph& g, const TgSample& sm, const TgCand& c, unsigned long long* updates,
                      bool flip, hipStream_t s);
void tg_launch_mark_all_fresh(const TgGraph& g, hipStream_t s);
void tg_launch_phase2(const TgGraph& g, int m, unsigned long long* updates, unsigned long long* stat_bins,
                      uint32_t* screen_on /* device flag, used when g.Xq is set */, hipStream_t s);
// range: the words tg_launch_norms filled, or null: where they show whole numbers whose fp32 sums are all exact, nothing is recomputed
void tg_launch_finalize(const TgGraph& g, int recompute, const uint32_t* range, int32_t* out_ids, float* out_dist, hipStream_t s);
void tg_launch_export(const TgGraph& g, int32_t* ids, float* dist, uint8_t* fresh, hipStream_t s);
void tg_launch_import(const TgGraph& g, const int32_t* ids, const float* dist, const uint8_t* fresh, hipStream_t s);
void tg_launch_pad_rows(const float* X, int64_t n, int d, float* Xp, int ld, hipStream_t s);
int tg_exact_slices(int64_t n, int64_t nq);
void tg_launch_exact_knn(const float* X, int ld, const float* nrm, const float* rnorm, int64_t n, int d, int k,
                         int metric, const int64_t* rows, int64_t nq, int32_t* out_ids, float* out_dist,
                         unsigned long long* partial /* nq x slices x k */, int nslices, hipStream_t s);
size_t tg_scan_tmp_elems(int64_t n);
void tg_launch_prune_rank(const int32_t* ids, int64_t n, int k, int d_out, int32_t* out_ids, int32_t* counts /* or null */,
                          hipStream_t s);
// rule 0: distance rule, thr = alpha^2; 1: angle rule, thr = 4 cos^2(gamma); 2: dispersion rule, thr unused
void tg_launch_angle_at(const float* a, const float* b, const float* c, float* out, int64_t count, hipStream_t s);
void tg_launch_filter(const float* X, int64_t n, int d, const int32_t* ids, int k, int hops, int cand_size, int rule, float thr,
                           int d_out, int32_t* out_ids, int32_t* out_deg /* or null */, hipStream_t s);
void tg_launch_merge_local(int32_t* g_ids, float* g_dist, int64_t n, int k, const int32_t* l_ids, const float* l_dist,
                           int64_t n_local, int k_local, const int32_t* l2g, hipStream_t s);
