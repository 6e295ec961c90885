/*
 * ldaref.c -- CPU oracle for the LightLDA cycle Metropolis-Hastings token sweep.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, plain-C
 * definition that the GPU library is compared against.  It shares no code,
 * header, table or constant generator with the HIP path, and nothing in the
 * product path may call it.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark load it.
 *
 * What it follows (LightLDA, arXiv 1412.1576):
 *   - target conditional                      : Eq. (1)/(4)
 *   - word-proposal and its acceptance ratio  : Eq. (6)-(8), Sec. 4.2
 *   - alias table (split point + alias / bin) : Sec. 4.2, Fig. 2
 *   - sparsified (mixture) word-proposal      : Sec. 4.2, paragraph after Eq. (8)
 *   - doc-proposal, z-array as alias table    : Eq. (9)-(12), Fig. 3
 *   - cycle of the two proposals              : Eq. (13), Sec. 4.3
 *   - count tables n_kd, n_kw, n_k            : Sec. 3, text after Eq. (1)
 *   - immutable model + delayed updates       : Sec. 6, "Multi-thread Efficiency"
 *
 * Points the paper leaves open are fixed as follows (each is listed again in
 * the repository's design notes):
 *   - Snapshot semantics: every token of a sweep reads z and all counts as they
 *     were at the start of the sweep; the "-di" exclusion removes the token at
 *     its snapshot topic z0, for all three count tables, during its whole chain.
 *   - One MH step = one proposal + one accept test.  Step j of a token is a
 *     word-proposal when j is even and a doc-proposal when j is odd.
 *   - Proposal factors in the ratios use snapshot counts including the token.
 *   - Randomness: Philox4x32-10 (Salmon et al., SC'11), key = 64-bit seed,
 *     counter = (token id low, token id high, sweep index, step index).
 *   - The alias table is an all-integer construction (see alias_from_q0) so
 *     that a sequential and a parallel build give identical tables.
 *   - Accept iff u*den < num with u = (x2 + 0.5) / 2^32; products left to right
 *     in fp64, no fused multiply-add (build with -ffp-contract=off).
 *   - Log-likelihood = collapsed joint log p(w, z | alpha, beta); the paper
 *     names the metric (Sec. 7) but prints no formula: the textbook form is used.
 *
 * Pins (see tests/): Philox known-answer vectors; alias mass reconstruction and
 * closed-form (merge) equivalence; detailed balance of the coded acceptance
 * against Eq. (4) computed independently; exact m-step distribution vs chain
 * histogram; doc-draw histogram vs (n_dk+alpha); count invariants vs numpy
 * recount; log-likelihood vs scipy gammaln and a K=1 closed form.  The two storage
 * options (tables built on first use, n_kw rows counted on first use) are pinned to the
 * plain form bit for bit.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define LDAREF_OK 0
#define LDAREF_ERR_ARG (-1)
#define LDAREF_ERR_STATE (-2)
#define LDAREF_ERR_OOM (-3)
#define LDAREF_ERR_INTERNAL (-4)

enum { ST_COUNTS_VALID = 1, ST_ALIAS_VALID = 2, ST_SWEPT = 3 };

/* ------------------------------------------------------------------------- */
/* Philox4x32-10, as published (Salmon, Moraes, Dror, Shaw, SC'11).           */
/* ------------------------------------------------------------------------- */
void ldaref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static uint32_t mulhi32(uint32_t a, uint32_t b)
{
    return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32);
}

/* uniform in (0,1): (x + 1/2) / 2^32, exact in fp64 */
static double unit_open(uint32_t x)
{
    return ((double)x + 0.5) * (1.0 / 4294967296.0);
}

static void token_random(uint64_t seed, uint64_t g, uint32_t sweep, uint32_t step, uint32_t x[4])
{
    uint32_t ctr[4] = { (uint32_t)g, (uint32_t)(g >> 32), sweep, step };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    ldaref_philox4x32_10(ctr, key, x);
}

/* ------------------------------------------------------------------------- */
/* Alias table (Sec. 4.2, Fig. 2): integer construction.                      */
/*                                                                           */
/* Input: q0[0..n), the bin weights already quantised to integers            */
/* (floor(weight * 2^40), weight in (0,1]).                                   */
/*  1. Q0 = sum q0.  sh = smallest shift with (Q0 >> sh) < n * 2^31.          */
/*  2. q_k = max(1, q0_k >> sh), Q = sum q_k, C = ceil(Q / n) (bin capacity), */
/*     pad = n*C - Q, m_k = q_k + (k < pad)  ==> sum m_k = n*C exactly.       */
/*  3. Lights {m_k < C} and heavies {m_k >= C}, both in ascending k, are      */
/*     paired by a two-pointer sweep: the current heavy fills lights until    */
/*     its residual drops to <= C, keeps that residual as its own split and   */
/*     borrows the rest of its bin from the next heavy.                       */
/* Output: split[k] in [1,C], alias[k]; a draw (bin, rr) with bin uniform in  */
/* [0,n) and rr uniform in [0,C) returns rr < split[bin] ? bin : alias[bin].  */
/* ------------------------------------------------------------------------- */
int ldaref_alias_masses(int32_t n, const uint64_t* q0, uint64_t* m, uint32_t* C_out)
{
    if (n < 1) return LDAREF_ERR_ARG;
    uint64_t Q0 = 0;
    for (int32_t k = 0; k < n; ++k) Q0 += q0[k];
    int sh = 0;
    while ((Q0 >> sh) >= ((uint64_t)n << 31)) ++sh;
    uint64_t Q = 0;
    for (int32_t k = 0; k < n; ++k) {
        uint64_t q = q0[k] >> sh;
        if (q < 1) q = 1;
        m[k] = q;
        Q += q;
    }
    uint64_t C = (Q + (uint64_t)n - 1) / (uint64_t)n;
    uint64_t pad = (uint64_t)n * C - Q;
    for (int32_t k = 0; k < n; ++k)
        if ((uint64_t)k < pad) m[k] += 1;
    if (C > 0xFFFFFFFFull) return LDAREF_ERR_INTERNAL;
    *C_out = (uint32_t)C;
    return LDAREF_OK;
}

int ldaref_alias_from_q0(int32_t n, const uint64_t* q0, uint32_t* split, uint32_t* alias,
                         uint32_t* C_out)
{
    uint64_t* m = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)n);
    if (!m) return LDAREF_ERR_OOM;
    uint32_t C32;
    int rc = ldaref_alias_masses(n, q0, m, &C32);
    if (rc) { free(m); return rc; }
    const uint64_t C = C32;

    int32_t li = 0; /* next light candidate */
    int32_t hi = 0; /* next heavy candidate */
    while (hi < n && m[hi] < C) ++hi;
    if (hi >= n) { free(m); return LDAREF_ERR_INTERNAL; } /* mean is C: a heavy exists */
    int32_t h = hi++;
    uint64_t r = m[h];
    for (;;) {
        if (r > C) {
            while (li < n && m[li] >= C) ++li;
            if (li >= n) { free(m); return LDAREF_ERR_INTERNAL; }
            split[li] = (uint32_t)m[li];
            alias[li] = (uint32_t)h;
            r -= C - m[li];
            ++li;
        } else {
            split[h] = (uint32_t)r;
            while (hi < n && m[hi] < C) ++hi;
            if (hi >= n) {
                if (r != C) { free(m); return LDAREF_ERR_INTERNAL; }
                alias[h] = (uint32_t)h;
                break;
            }
            alias[h] = (r == C) ? (uint32_t)h : (uint32_t)hi;
            r = m[hi] - (C - r);
            h = hi++;
        }
    }
    /* conservation: no light may be left over */
    while (li < n && m[li] >= C) ++li;
    free(m);
    if (li < n) return LDAREF_ERR_INTERNAL;
    *C_out = C32;
    return LDAREF_OK;
}

/* weight -> integer: floor(a * 2^40), a in (0,1] */
static uint64_t quantise40(double a)
{
    return (uint64_t)floor(a * 1099511627776.0);
}

/* Dense word-proposal table for one word: weights (n_kw+beta)/(n_k+betabar), Eq. (6). */
int ldaref_alias_build_dense_row(int32_t K, const int32_t* nkw_row, const int32_t* nk,
                                 double beta, double betabar, uint32_t* split, uint32_t* alias,
                                 uint32_t* C_out)
{
    uint64_t* q0 = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)K);
    if (!q0) return LDAREF_ERR_OOM;
    for (int32_t k = 0; k < K; ++k) {
        double a = ((double)nkw_row[k] + beta) / ((double)nk[k] + betabar);
        q0[k] = quantise40(a);
    }
    int rc = ldaref_alias_from_q0(K, q0, split, alias, C_out);
    free(q0);
    return rc;
}

/* draw from a table: Fig. 2 */
uint32_t ldaref_alias_draw(int32_t n, const uint32_t* split, const uint32_t* alias, uint32_t C,
                           uint32_t x0, uint32_t x1)
{
    uint32_t bin = mulhi32(x0, (uint32_t)n);
    uint32_t rr = mulhi32(x1, C);
    return rr < split[bin] ? bin : alias[bin];
}

/* ------------------------------------------------------------------------- */
/* Doc-proposal draw (Eq. 9, 12; Fig. 3): with probability L/(L + K*alpha)    */
/* copy the snapshot topic of a uniformly chosen token of the document        */
/* (possibly the token itself), otherwise a uniform topic.                    */
/* ------------------------------------------------------------------------- */
int32_t ldaref_doc_draw(int32_t L, int32_t K, double alphabar, const int32_t* z_doc,
                        uint32_t x0, uint32_t x1)
{
    double u0 = unit_open(x0);
    if (u0 * ((double)L + alphabar) < (double)L) {
        uint32_t j = mulhi32(x1, (uint32_t)L);
        return z_doc[j];
    }
    return (int32_t)mulhi32(x1, (uint32_t)K);
}

/* ------------------------------------------------------------------------- */
/* Accept test for a move s -> t (t != s) of a token whose snapshot topic is  */
/* z0.  word_step != 0: Eq. (8); word_step == 0: Eq. (11).                     */
/* n_*s / n_*t are snapshot counts (token included).                          */
/* ------------------------------------------------------------------------- */
int ldaref_mh_accept(int word_step, int32_t s, int32_t t, int32_t z0,
                     int32_t ndk_s, int32_t ndk_t, int32_t nkw_s, int32_t nkw_t,
                     int32_t nk_s, int32_t nk_t, double alpha, double beta, double betabar,
                     uint32_t x2)
{
    const int32_t ms = (s == z0) ? 1 : 0;
    const int32_t mt = (t == z0) ? 1 : 0;
    double num = ((double)(ndk_t - mt) + alpha);
    num = num * ((double)(nkw_t - mt) + beta);
    num = num * ((double)(nk_s - ms) + betabar);
    double den = ((double)(ndk_s - ms) + alpha);
    den = den * ((double)(nkw_s - ms) + beta);
    den = den * ((double)(nk_t - mt) + betabar);
    if (word_step) {
        num = num * ((double)nkw_s + beta);
        num = num * ((double)nk_t + betabar);
        den = den * ((double)nkw_t + beta);
        den = den * ((double)nk_s + betabar);
    } else {
        num = num * ((double)ndk_s + alpha);
        den = den * ((double)ndk_t + alpha);
    }
    double u = unit_open(x2);
    return (u * den < num) ? 1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Context                                                                    */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t n;         /* number of non-zero topics of the word */
    int32_t* topics;   /* ascending */
    uint32_t* split;
    uint32_t* alias;
    uint32_t C;
    uint64_t QS;       /* integer mass of the sparse term */
} sparse_table;

typedef struct ldaref_ctx {
    int64_t D, N;
    int32_t V, K;
    double alpha, beta, alphabar, betabar;
    uint64_t seed;
    int32_t dense_alias_min_count; /* words with corpus count >= this use the dense table; 0: all */
    int32_t proposal_mode;         /* 0 cycle, 1 word only, 2 doc only */
    int32_t lazy_alias;            /* build a word's table on first use in a sweep */
    int64_t* doff;                 /* [D+1] */
    int32_t* word;                 /* [N] */
    int32_t* wcount;               /* [V] corpus frequency */
    int32_t* z;                    /* [N] snapshot */
    int32_t* znew;                 /* [N] */
    /* n_kw: one row of K counts per word, reached through nkw_row[w].  Default: every row
     * lives in one V*K block and is counted by count_all.  With lazy_rows (vocabularies
     * whose V*K table does not fit in memory) a row is allocated and counted from the
     * word's tokens when it is first asked for and dropped when the counts go stale; the
     * numbers in a row are the same either way. */
    int32_t** nkw_row;             /* [V]; NULL = not counted yet (lazy_rows only) */
    int32_t* nkw_block;            /* [V*K] backing store of all rows (not lazy_rows) */
    int32_t lazy_rows;
    int64_t* wtok_off;             /* [V+1] lazy_rows: tokens of word w are            */
    int32_t* wtok;                 /* [N]   wtok[wtok_off[w] .. wtok_off[w+1]), ascending */
    int32_t* nk;                   /* [K] */
    int32_t* doc_scratch;          /* [K] dense n_dk row of the current document */
    /* word-proposal tables */
    uint32_t** split_row;          /* [V] dense form: K bins of word w (lazy_rows: NULL until built) */
    uint32_t** alias_row;          /* [V] */
    uint32_t* split_block;         /* [V*K] backing store (not lazy_rows) */
    uint32_t* alias_block;
    uint32_t* cap;                 /* [V] */
    uint8_t* built;                /* [V] table valid for the current snapshot */
    sparse_table* sparse;          /* [V] mixture form: per-word sparse term */
    uint32_t* bsplit;              /* [K] mixture form: shared beta/(n_k+betabar) table */
    uint32_t* balias;
    uint32_t bC;
    uint64_t QB;
    int beta_table_built;
    int state;
    int prev_valid;                /* znew holds the assignment before the last sweep */
    uint32_t sweep_index;
} ldaref_ctx;

static int word_is_dense(const ldaref_ctx* c, int32_t w)
{
    return c->dense_alias_min_count <= 0 || c->wcount[w] >= c->dense_alias_min_count;
}

static void free_sparse(sparse_table* s)
{
    free(s->topics); free(s->split); free(s->alias);
    memset(s, 0, sizeof(*s));
}

void ldaref_destroy(ldaref_ctx* c)
{
    if (!c) return;
    if (c->sparse)
        for (int32_t w = 0; w < c->V; ++w) free_sparse(&c->sparse[w]);
    free(c->sparse); free(c->bsplit); free(c->balias);
    if (c->lazy_rows) {
        for (int32_t w = 0; w < c->V; ++w) {
            if (c->nkw_row) free(c->nkw_row[w]);
            if (c->split_row) free(c->split_row[w]);
            if (c->alias_row) free(c->alias_row[w]);
        }
    }
    free(c->nkw_row); free(c->nkw_block); free(c->wtok_off); free(c->wtok);
    free(c->split_row); free(c->alias_row); free(c->split_block); free(c->alias_block);
    free(c->doff); free(c->word); free(c->wcount); free(c->z); free(c->znew);
    free(c->nk); free(c->doc_scratch);
    free(c->cap); free(c->built);
    free(c);
}

static void count_all(ldaref_ctx* c)
{
    memset(c->nk, 0, sizeof(int32_t) * (size_t)c->K);
    if (c->lazy_rows) {
        /* rows counted from an older assignment are dropped; nkw_row_of recounts on demand */
        for (int32_t w = 0; w < c->V; ++w) {
            free(c->nkw_row[w]);
            c->nkw_row[w] = NULL;
        }
    } else {
        memset(c->nkw_block, 0, sizeof(int32_t) * (size_t)c->V * (size_t)c->K);
    }
    for (int64_t g = 0; g < c->N; ++g) {
        if (!c->lazy_rows) c->nkw_row[c->word[g]][c->z[g]] += 1;
        c->nk[c->z[g]] += 1;
    }
    /* n_dk rows are formed per document from z when needed (doc_scratch) */
}

/* Row w of n_kw for the current assignment; NULL: out of memory (lazy_rows only). */
static const int32_t* nkw_row_of(ldaref_ctx* c, int32_t w)
{
    if (!c->nkw_row[w]) {
        int32_t* row = (int32_t*)calloc((size_t)c->K, sizeof(int32_t));
        if (!row) return NULL;
        for (int64_t i = c->wtok_off[w]; i < c->wtok_off[w + 1]; ++i) row[c->z[c->wtok[i]]] += 1;
        c->nkw_row[w] = row;
    }
    return c->nkw_row[w];
}

/* lazy_rows != 0: n_kw rows and dense tables are allocated per word on first use (see the
 * context); everything the oracle computes is the same. */
int ldaref_init_ex(ldaref_ctx** out, int64_t D, int32_t V, int32_t K, const int64_t* doc_offsets,
                   const int32_t* word_ids, double alpha, double beta, uint64_t seed,
                   int32_t dense_alias_min_count, int32_t proposal_mode, int32_t lazy_rows)
{
    if (!out || !doc_offsets || D < 1 || V < 1 || K < 1 || !(alpha > 0.0) || !(beta > 0.0))
        return LDAREF_ERR_ARG;
    if (proposal_mode < 0 || proposal_mode > 2 || dense_alias_min_count < 0) return LDAREF_ERR_ARG;
    if (doc_offsets[0] != 0) return LDAREF_ERR_ARG;
    for (int64_t d = 0; d < D; ++d)
        if (doc_offsets[d + 1] < doc_offsets[d]) return LDAREF_ERR_ARG;
    const int64_t N = doc_offsets[D];
    if (N < 1 || N >= 2147483647LL || !word_ids) return LDAREF_ERR_ARG;
    for (int64_t g = 0; g < N; ++g)
        if (word_ids[g] < 0 || word_ids[g] >= V) return LDAREF_ERR_ARG;

    ldaref_ctx* c = (ldaref_ctx*)calloc(1, sizeof(ldaref_ctx));
    if (!c) return LDAREF_ERR_OOM;
    c->D = D; c->N = N; c->V = V; c->K = K;
    c->alpha = alpha; c->beta = beta;
    c->alphabar = (double)K * alpha;
    c->betabar = (double)V * beta;
    c->seed = seed;
    c->dense_alias_min_count = dense_alias_min_count;
    c->proposal_mode = proposal_mode;
    c->lazy_rows = lazy_rows ? 1 : 0;
    const size_t VK = (size_t)V * (size_t)K;
    c->doff = (int64_t*)malloc(sizeof(int64_t) * (size_t)(D + 1));
    c->word = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    c->wcount = (int32_t*)calloc((size_t)V, sizeof(int32_t));
    c->z = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    c->znew = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    c->nkw_row = (int32_t**)calloc((size_t)V, sizeof(int32_t*));
    c->split_row = (uint32_t**)calloc((size_t)V, sizeof(uint32_t*));
    c->alias_row = (uint32_t**)calloc((size_t)V, sizeof(uint32_t*));
    if (c->lazy_rows) {
        c->wtok_off = (int64_t*)calloc((size_t)V + 1, sizeof(int64_t));
        c->wtok = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    } else {
        c->nkw_block = (int32_t*)calloc(VK, sizeof(int32_t));
        c->split_block = (uint32_t*)calloc(VK, sizeof(uint32_t));
        c->alias_block = (uint32_t*)calloc(VK, sizeof(uint32_t));
    }
    c->nk = (int32_t*)calloc((size_t)K, sizeof(int32_t));
    c->doc_scratch = (int32_t*)calloc((size_t)K, sizeof(int32_t));
    c->cap = (uint32_t*)calloc((size_t)V, sizeof(uint32_t));
    c->built = (uint8_t*)calloc((size_t)V, 1);
    c->sparse = (sparse_table*)calloc((size_t)V, sizeof(sparse_table));
    c->bsplit = (uint32_t*)calloc((size_t)K, sizeof(uint32_t));
    c->balias = (uint32_t*)calloc((size_t)K, sizeof(uint32_t));
    const int rows_ok = c->lazy_rows ? (c->wtok_off && c->wtok)
                                     : (c->nkw_block && c->split_block && c->alias_block);
    if (!c->doff || !c->word || !c->wcount || !c->z || !c->znew || !c->nkw_row || !c->nk ||
        !c->doc_scratch || !c->split_row || !c->alias_row || !rows_ok || !c->cap || !c->built ||
        !c->sparse || !c->bsplit || !c->balias) {
        ldaref_destroy(c);
        return LDAREF_ERR_OOM;
    }
    memcpy(c->doff, doc_offsets, sizeof(int64_t) * (size_t)(D + 1));
    memcpy(c->word, word_ids, sizeof(int32_t) * (size_t)N);
    for (int64_t g = 0; g < N; ++g) c->wcount[c->word[g]] += 1;
    if (c->lazy_rows) {
        /* the tokens of every word, in ascending token order (counting sort) */
        for (int32_t w = 0; w < V; ++w) c->wtok_off[w + 1] = c->wtok_off[w] + c->wcount[w];
        int64_t* next = (int64_t*)malloc(sizeof(int64_t) * (size_t)V);
        if (!next) { ldaref_destroy(c); return LDAREF_ERR_OOM; }
        memcpy(next, c->wtok_off, sizeof(int64_t) * (size_t)V);
        for (int64_t g = 0; g < N; ++g) c->wtok[next[c->word[g]]++] = (int32_t)g;
        free(next);
    } else {
        for (int32_t w = 0; w < V; ++w) {
            c->nkw_row[w] = c->nkw_block + (size_t)w * (size_t)K;
            c->split_row[w] = c->split_block + (size_t)w * (size_t)K;
            c->alias_row[w] = c->alias_block + (size_t)w * (size_t)K;
        }
    }
    /* initial assignment: uniform topic from the token's own Philox stream,
       counter (g, 0xFFFFFFFF, 0) */
    for (int64_t g = 0; g < N; ++g) {
        uint32_t x[4];
        token_random(seed, (uint64_t)g, 0xFFFFFFFFu, 0u, x);
        c->z[g] = (int32_t)mulhi32(x[0], (uint32_t)K);
    }
    count_all(c);
    c->state = ST_COUNTS_VALID;
    c->sweep_index = 0;
    *out = c;
    return LDAREF_OK;
}

int ldaref_init(ldaref_ctx** out, int64_t D, int32_t V, int32_t K, const int64_t* doc_offsets,
                const int32_t* word_ids, double alpha, double beta, uint64_t seed,
                int32_t dense_alias_min_count, int32_t proposal_mode)
{
    return ldaref_init_ex(out, D, V, K, doc_offsets, word_ids, alpha, beta, seed,
                          dense_alias_min_count, proposal_mode, 0);
}

/* lazy != 0: ldaref_build_alias builds only the shared table; a word's table is built from
 * the same counts when a draw first needs it.  The tables are the same either way. */
void ldaref_set_lazy_alias(ldaref_ctx* c, int32_t lazy) { c->lazy_alias = lazy ? 1 : 0; }

/* Mixture form (Sec. 4.2): p_w = n_kw/(n_k+betabar) [sparse, per word]
 *                              + beta/(n_k+betabar) [dense, shared by all words]. */
static int build_beta_table(ldaref_ctx* c)
{
    uint64_t* q0 = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)c->K);
    if (!q0) return LDAREF_ERR_OOM;
    uint64_t QB = 0;
    for (int32_t k = 0; k < c->K; ++k) {
        q0[k] = quantise40(c->beta / ((double)c->nk[k] + c->betabar));
        QB += q0[k];
    }
    int rc = ldaref_alias_from_q0(c->K, q0, c->bsplit, c->balias, &c->bC);
    free(q0);
    c->QB = QB;
    c->beta_table_built = 1;
    return rc;
}

static int build_word_table(ldaref_ctx* c, int32_t w)
{
    const int32_t K = c->K;
    const int32_t* row = nkw_row_of(c, w);
    if (!row) return LDAREF_ERR_OOM;
    int rc = LDAREF_OK;
    if (word_is_dense(c, w)) {
        if (!c->split_row[w]) c->split_row[w] = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)K);
        if (!c->alias_row[w]) c->alias_row[w] = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)K);
        if (!c->split_row[w] || !c->alias_row[w]) return LDAREF_ERR_OOM;
        rc = ldaref_alias_build_dense_row(K, row, c->nk, c->beta, c->betabar, c->split_row[w],
                                          c->alias_row[w], &c->cap[w]);
    } else {
        sparse_table* s = &c->sparse[w];
        free_sparse(s);
        int32_t n = 0;
        for (int32_t k = 0; k < K; ++k) n += (row[k] > 0);
        s->n = n;
        s->QS = 0;
        if (n > 0) {
            s->topics = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
            s->split = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)n);
            s->alias = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)n);
            uint64_t* q0 = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)n);
            if (!s->topics || !s->split || !s->alias || !q0) { free(q0); return LDAREF_ERR_OOM; }
            int32_t i = 0;
            for (int32_t k = 0; k < K; ++k) {
                if (row[k] > 0) {
                    s->topics[i] = k;
                    q0[i] = quantise40((double)row[k] / ((double)c->nk[k] + c->betabar));
                    s->QS += q0[i];
                    ++i;
                }
            }
            rc = ldaref_alias_from_q0(n, q0, s->split, s->alias, &s->C);
            free(q0);
        }
    }
    if (rc == LDAREF_OK) c->built[w] = 1;
    return rc;
}

int ldaref_build_alias(ldaref_ctx* c)
{
    if (!c) return LDAREF_ERR_ARG;
    if (c->state != ST_COUNTS_VALID && c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    memset(c->built, 0, (size_t)c->V);
    c->beta_table_built = 0;
    if (c->dense_alias_min_count > 0) {
        int rc = build_beta_table(c);
        if (rc) return rc;
    }
    if (!c->lazy_alias) {
        for (int32_t w = 0; w < c->V; ++w) {
            int rc = build_word_table(c, w);
            if (rc) return rc;
        }
    }
    c->state = ST_ALIAS_VALID;
    return LDAREF_OK;
}

/* word-proposal draw for word w from (x0, x1, x3) into *t */
static int word_draw(ldaref_ctx* c, int32_t w, uint32_t x0, uint32_t x1, uint32_t x3, int32_t* t)
{
    const int32_t K = c->K;
    if (!c->built[w]) {
        int rc = build_word_table(c, w);
        if (rc) return rc;
    }
    if (word_is_dense(c, w)) {
        *t = (int32_t)ldaref_alias_draw(K, c->split_row[w], c->alias_row[w], c->cap[w], x0, x1);
        return LDAREF_OK;
    }
    const sparse_table* s = &c->sparse[w];
    double u3 = unit_open(x3);
    if (u3 * (double)(s->QS + c->QB) < (double)s->QS) {
        uint32_t i = ldaref_alias_draw(s->n, s->split, s->alias, s->C, x0, x1);
        *t = s->topics[i];
        return LDAREF_OK;
    }
    *t = (int32_t)ldaref_alias_draw(K, c->bsplit, c->balias, c->bC, x0, x1);
    return LDAREF_OK;
}

/* One token's chain (Eq. 13): ndk = dense n_dk row of its document, zdoc = the
 * document's snapshot topics, L = document length.  The final topic goes to *out. */
static int token_chain(ldaref_ctx* c, int64_t g, int32_t w, const int32_t* ndk,
                       const int32_t* zdoc, int32_t L, uint32_t sweep, int32_t mh_steps,
                       int32_t* out)
{
    const int32_t K = c->K;
    const int32_t* nkw = nkw_row_of(c, w);
    if (!nkw) return LDAREF_ERR_OOM;
    const int32_t z0 = c->z[g];
    int32_t s = z0;
    for (int32_t j = 0; j < mh_steps; ++j) {
        uint32_t x[4];
        token_random(c->seed, (uint64_t)g, sweep, (uint32_t)j, x);
        int word_step = (c->proposal_mode == 0) ? ((j & 1) == 0) : (c->proposal_mode == 1);
        int32_t t;
        if (word_step) {
            int rc = word_draw(c, w, x[0], x[1], x[3], &t);
            if (rc) return rc;
        } else {
            t = ldaref_doc_draw(L, K, c->alphabar, zdoc, x[0], x[1]);
        }
        if (t != s) {
            if (ldaref_mh_accept(word_step, s, t, z0, ndk[s], ndk[t], nkw[s], nkw[t], c->nk[s],
                                 c->nk[t], c->alpha, c->beta, c->betabar, x[2]))
                s = t;
        }
    }
    *out = s;
    return LDAREF_OK;
}

int ldaref_sweep(ldaref_ctx* c, int32_t mh_steps)
{
    if (!c || mh_steps < 1) return LDAREF_ERR_ARG;
    if (c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    int32_t* ndk = c->doc_scratch;
    for (int64_t d = 0; d < c->D; ++d) {
        const int64_t b = c->doff[d], e = c->doff[d + 1];
        const int32_t L = (int32_t)(e - b);
        int rc = LDAREF_OK;
        for (int64_t g = b; g < e; ++g) ndk[c->z[g]] += 1;
        for (int64_t g = b; g < e && rc == LDAREF_OK; ++g)
            rc = token_chain(c, g, c->word[g], ndk, c->z + b, L, c->sweep_index, mh_steps,
                             &c->znew[g]);
        for (int64_t g = b; g < e; ++g) ndk[c->z[g]] = 0;
        if (rc) return rc;
    }
    int32_t* tmp = c->z; c->z = c->znew; c->znew = tmp;
    c->sweep_index += 1;
    c->state = ST_SWEPT;
    c->prev_valid = 1;
    return LDAREF_OK;
}

/* Sweep with the doc side refreshed after every token (Sec. 4.2, footnote 4: the doc-proposal
 * is not frozen during a document but follows the document's assignments token by token)
 * while the word side -- n_kw, n_k and the word-proposal tables -- stays at the snapshot
 * (Sec. 6, the immutable model slice).  The tokens of a document are visited in order; token
 * i sees the topics that tokens < i of the same document were just given, in n_kd and in the
 * doc-proposal's draw.  Its own entry is still its snapshot topic z0, which is what the "-di"
 * exclusion removes from all three tables.  Documents stay independent of each other. */
int ldaref_sweep_doc_refresh(ldaref_ctx* c, int32_t mh_steps)
{
    if (!c || mh_steps < 1) return LDAREF_ERR_ARG;
    if (c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    int32_t* ndk = c->doc_scratch;
    int32_t maxL = 0;
    for (int64_t d = 0; d < c->D; ++d)
        if (c->doff[d + 1] - c->doff[d] > maxL) maxL = (int32_t)(c->doff[d + 1] - c->doff[d]);
    int32_t* zcur = (int32_t*)malloc(sizeof(int32_t) * (size_t)(maxL > 0 ? maxL : 1));
    if (!zcur) return LDAREF_ERR_OOM;
    for (int64_t d = 0; d < c->D; ++d) {
        const int64_t b = c->doff[d], e = c->doff[d + 1];
        const int32_t L = (int32_t)(e - b);
        int rc = LDAREF_OK;
        for (int64_t g = b; g < e; ++g) {
            zcur[g - b] = c->z[g];
            ndk[c->z[g]] += 1;
        }
        for (int64_t g = b; g < e && rc == LDAREF_OK; ++g) {
            int32_t s;
            rc = token_chain(c, g, c->word[g], ndk, zcur, L, c->sweep_index, mh_steps, &s);
            if (rc == LDAREF_OK) {
                ndk[zcur[g - b]] -= 1;
                ndk[s] += 1;
                zcur[g - b] = s;
                c->znew[g] = s;
            }
        }
        for (int32_t i = 0; i < L; ++i) ndk[zcur[i]] = 0;
        for (int64_t g = b; g < e; ++g) ndk[c->z[g]] = 0;
        if (rc) { free(zcur); return rc; }
    }
    free(zcur);
    int32_t* tmp = c->z; c->z = c->znew; c->znew = tmp;
    c->sweep_index += 1;
    c->state = ST_SWEPT;
    c->prev_valid = 1;
    return LDAREF_OK;
}

/* One token's chain with the document side taken from a caller-given assignment zdoc[0..L)
 * of its document (zdoc at the token's own place must be its snapshot topic); the word side
 * is the snapshot.  Does not change the context. */
int ldaref_chain_with_doc(ldaref_ctx* c, int64_t g, uint32_t sweep_index, int32_t mh_steps,
                          int32_t L, const int32_t* zdoc, int32_t* out)
{
    if (!c || mh_steps < 1 || !zdoc || !out || g < 0 || g >= c->N) return LDAREF_ERR_ARG;
    if (c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    int64_t lo = 0, hi = c->D;
    while (hi - lo > 1) {
        int64_t mid = lo + (hi - lo) / 2;
        if (c->doff[mid] <= g) lo = mid; else hi = mid;
    }
    while (c->doff[lo + 1] <= g) ++lo;
    if (L != (int32_t)(c->doff[lo + 1] - c->doff[lo]) || zdoc[g - c->doff[lo]] != c->z[g])
        return LDAREF_ERR_ARG;
    for (int32_t i = 0; i < L; ++i)
        if (zdoc[i] < 0 || zdoc[i] >= c->K) return LDAREF_ERR_ARG;
    int32_t* ndk = c->doc_scratch;
    for (int32_t i = 0; i < L; ++i) ndk[zdoc[i]] += 1;
    int rc = token_chain(c, g, c->word[g], ndk, zdoc, L, sweep_index, mh_steps, out);
    for (int32_t i = 0; i < L; ++i) ndk[zdoc[i]] = 0;
    return rc;
}

/* Chains of selected tokens only, against the current snapshot, for an
 * arbitrary sweep index; does not change the context's assignment. */
int ldaref_sweep_tokens(ldaref_ctx* c, uint32_t sweep_index, int32_t mh_steps, int64_t n,
                        const int64_t* token_ids, int32_t* out)
{
    if (!c || mh_steps < 1 || n < 0 || (n > 0 && (!token_ids || !out))) return LDAREF_ERR_ARG;
    if (c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    int32_t* ndk = c->doc_scratch;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t g = token_ids[i];
        if (g < 0 || g >= c->N) return LDAREF_ERR_ARG;
        int64_t lo = 0, hi = c->D; /* last d with doff[d] <= g */
        while (hi - lo > 1) {
            int64_t mid = lo + (hi - lo) / 2;
            if (c->doff[mid] <= g) lo = mid; else hi = mid;
        }
        /* skip empty documents that share the offset */
        while (c->doff[lo + 1] <= g) ++lo;
        const int64_t b = c->doff[lo], e = c->doff[lo + 1];
        for (int64_t q = b; q < e; ++q) ndk[c->z[q]] += 1;
        int rc = token_chain(c, g, c->word[g], ndk, c->z + b, (int32_t)(e - b), sweep_index,
                             mh_steps, &out[i]);
        for (int64_t q = b; q < e; ++q) ndk[c->z[q]] = 0;
        if (rc) return rc;
    }
    return LDAREF_OK;
}

int ldaref_rebuild_counts(ldaref_ctx* c)
{
    if (!c) return LDAREF_ERR_ARG;
    count_all(c);
    c->state = ST_COUNTS_VALID;
    c->prev_valid = 0;
    return LDAREF_OK;
}

/* The paper's own way to keep the counts (Sec. 3, text after Eq. 1): when a token moves from
 * topic a to topic b, n_kw[w][a], n_k[a] lose one and n_kw[w][b], n_k[b] gain one (n_kd is
 * formed per document from z here).  Applied after a sweep for every token that moved, from
 * the assignment before the sweep, it must leave the same tables as a recount. */
int ldaref_update_counts(ldaref_ctx* c)
{
    if (!c) return LDAREF_ERR_ARG;
    if (c->state != ST_SWEPT || !c->prev_valid) return LDAREF_ERR_STATE;
    for (int64_t g = 0; g < c->N; ++g) {
        const int32_t a = c->znew[g], b = c->z[g]; /* before, after */
        if (a == b) continue;
        if (!c->lazy_rows) {
            c->nkw_row[c->word[g]][a] -= 1;
            c->nkw_row[c->word[g]][b] += 1;
        }
        c->nk[a] -= 1;
        c->nk[b] += 1;
    }
    if (c->lazy_rows) { /* rows are recounted when next needed */
        for (int32_t w = 0; w < c->V; ++w) {
            free(c->nkw_row[w]);
            c->nkw_row[w] = NULL;
        }
    }
    c->state = ST_COUNTS_VALID;
    c->prev_valid = 0;
    return LDAREF_OK;
}

/* ------------------------------------------------------------------------- */
/* Log-likelihood: log p(w, z | alpha, beta) of the collapsed model,          */
/*   doc  = sum_d [ lgG(K a) - lgG(L_d + K a) + sum_{k: n_dk>0} (lgG(n_dk+a) - lgG(a)) ] */
/*   word = sum_k [ lgG(V b) - lgG(n_k + V b) + sum_{w: n_kw>0} (lgG(n_kw+b) - lgG(b)) ] */
/* compensated (Neumaier) summation in fp64.                                   */
/* ------------------------------------------------------------------------- */
typedef struct { double s, c; } ksum;
static void kadd(ksum* a, double x)
{
    double t = a->s + x;
    if (fabs(a->s) >= fabs(x)) a->c += (a->s - t) + x; else a->c += (x - t) + a->s;
    a->s = t;
}

static int cmp_int32(const void* a, const void* b)
{
    const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

int ldaref_loglik(ldaref_ctx* c, double* total, double* doc_part, double* word_part)
{
    if (!c || !total) return LDAREF_ERR_ARG;
    if (c->state != ST_COUNTS_VALID && c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    const int32_t K = c->K;
    ksum sd = { 0.0, 0.0 }, sw = { 0.0, 0.0 };
    const double lga = lgamma(c->alpha), lgb = lgamma(c->beta);
    const double lgab = lgamma(c->alphabar), lgbb = lgamma(c->betabar);
    int32_t* ndk = c->doc_scratch;
    for (int64_t d = 0; d < c->D; ++d) {
        const int64_t b = c->doff[d], e = c->doff[d + 1];
        kadd(&sd, lgab - lgamma((double)(e - b) + c->alphabar));
        for (int64_t g = b; g < e; ++g) ndk[c->z[g]] += 1;
        for (int64_t g = b; g < e; ++g) {
            int32_t k = c->z[g];
            if (ndk[k] > 0) {
                kadd(&sd, lgamma((double)ndk[k] + c->alpha) - lga);
                ndk[k] = 0; /* each topic of the document once */
            }
        }
    }
    for (int32_t k = 0; k < K; ++k) kadd(&sw, lgbb - lgamma((double)c->nk[k] + c->betabar));
    if (!c->lazy_rows) {
        for (int32_t w = 0; w < c->V; ++w) {
            const int32_t* row = c->nkw_row[w];
            for (int32_t k = 0; k < K; ++k)
                if (row[k] > 0) kadd(&sw, lgamma((double)row[k] + c->beta) - lgb);
        }
    } else {
        /* the same terms in the same order (words ascending, topics ascending) without
           K-entry rows: a word's distinct topics are collected from its tokens and sorted */
        int32_t* cnt = (int32_t*)calloc((size_t)K, sizeof(int32_t));
        int32_t* tl = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
        if (!cnt || !tl) { free(cnt); free(tl); return LDAREF_ERR_OOM; }
        for (int32_t w = 0; w < c->V; ++w) {
            int32_t n = 0;
            for (int64_t i = c->wtok_off[w]; i < c->wtok_off[w + 1]; ++i) {
                const int32_t k = c->z[c->wtok[i]];
                if (cnt[k]++ == 0) tl[n++] = k;
            }
            qsort(tl, (size_t)n, sizeof(int32_t), cmp_int32);
            for (int32_t j = 0; j < n; ++j) {
                kadd(&sw, lgamma((double)cnt[tl[j]] + c->beta) - lgb);
                cnt[tl[j]] = 0;
            }
        }
        free(cnt); free(tl);
    }
    const double dp = sd.s + sd.c, wp = sw.s + sw.c;
    if (doc_part) *doc_part = dp;
    if (word_part) *word_part = wp;
    *total = dp + wp;
    return LDAREF_OK;
}

/* ------------------------------------------------------------------------- */
/* Accessors                                                                  */
/* ------------------------------------------------------------------------- */
int64_t ldaref_num_tokens(const ldaref_ctx* c) { return c ? c->N : -1; }
uint32_t ldaref_sweep_index(const ldaref_ctx* c) { return c ? c->sweep_index : 0; }

int ldaref_get_z(ldaref_ctx* c, int32_t* z)
{
    if (!c || !z) return LDAREF_ERR_ARG;
    memcpy(z, c->z, sizeof(int32_t) * (size_t)c->N);
    return LDAREF_OK;
}

int ldaref_set_z(ldaref_ctx* c, const int32_t* z, int64_t next_sweep_index)
{
    if (!c || !z || next_sweep_index < 0 || next_sweep_index > 0xFFFFFFFELL) return LDAREF_ERR_ARG;
    for (int64_t g = 0; g < c->N; ++g)
        if (z[g] < 0 || z[g] >= c->K) return LDAREF_ERR_ARG;
    memcpy(c->z, z, sizeof(int32_t) * (size_t)c->N);
    c->sweep_index = (uint32_t)next_sweep_index;
    c->state = ST_SWEPT; /* counts are stale until rebuilt */
    c->prev_valid = 0;
    return LDAREF_OK;
}

int ldaref_get_nk(ldaref_ctx* c, int32_t* nk)
{
    if (!c || !nk) return LDAREF_ERR_ARG;
    if (c->state == ST_SWEPT) return LDAREF_ERR_STATE;
    memcpy(nk, c->nk, sizeof(int32_t) * (size_t)c->K);
    return LDAREF_OK;
}

int ldaref_get_nkw_row(ldaref_ctx* c, int32_t w, int32_t* row)
{
    if (!c || !row || w < 0 || w >= c->V) return LDAREF_ERR_ARG;
    if (c->state == ST_SWEPT) return LDAREF_ERR_STATE;
    const int32_t* src = nkw_row_of(c, w);
    if (!src) return LDAREF_ERR_OOM;
    memcpy(row, src, sizeof(int32_t) * (size_t)c->K);
    return LDAREF_OK;
}

int ldaref_get_ndk_row(ldaref_ctx* c, int64_t d, int32_t* row)
{
    if (!c || !row || d < 0 || d >= c->D) return LDAREF_ERR_ARG;
    memset(row, 0, sizeof(int32_t) * (size_t)c->K);
    for (int64_t g = c->doff[d]; g < c->doff[d + 1]; ++g) row[c->z[g]] += 1;
    return LDAREF_OK;
}

/* Dense-form table of word w (the word must use the dense form). */
int ldaref_get_alias_row(ldaref_ctx* c, int32_t w, uint32_t* split, uint32_t* alias, uint32_t* C)
{
    if (!c || !split || !alias || !C || w < 0 || w >= c->V) return LDAREF_ERR_ARG;
    if (c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    if (!word_is_dense(c, w)) return LDAREF_ERR_ARG;
    if (!c->built[w]) { int rc = build_word_table(c, w); if (rc) return rc; }
    memcpy(split, c->split_row[w], sizeof(uint32_t) * (size_t)c->K);
    memcpy(alias, c->alias_row[w], sizeof(uint32_t) * (size_t)c->K);
    *C = c->cap[w];
    return LDAREF_OK;
}

/* Mixture-form tables of word w: the sparse term (n entries, topics ascending)
 * and its integer mass; n_out may exceed cap_entries, then only the count is returned. */
int ldaref_get_sparse_table(ldaref_ctx* c, int32_t w, int32_t cap_entries, int32_t* n_out,
                            int32_t* topics, uint32_t* split, uint32_t* alias, uint32_t* C,
                            uint64_t* QS)
{
    if (!c || !n_out || w < 0 || w >= c->V) return LDAREF_ERR_ARG;
    if (c->state != ST_ALIAS_VALID) return LDAREF_ERR_STATE;
    if (word_is_dense(c, w)) return LDAREF_ERR_ARG;
    if (!c->built[w]) { int rc = build_word_table(c, w); if (rc) return rc; }
    const sparse_table* s = &c->sparse[w];
    *n_out = s->n;
    if (QS) *QS = s->QS;
    if (C) *C = s->C;
    if (s->n <= cap_entries && topics && split && alias) {
        memcpy(topics, s->topics, sizeof(int32_t) * (size_t)s->n);
        memcpy(split, s->split, sizeof(uint32_t) * (size_t)s->n);
        memcpy(alias, s->alias, sizeof(uint32_t) * (size_t)s->n);
    }
    return LDAREF_OK;
}

int ldaref_get_beta_table(ldaref_ctx* c, uint32_t* split, uint32_t* alias, uint32_t* C,
                          uint64_t* QB)
{
    if (!c || !split || !alias || !C || !QB) return LDAREF_ERR_ARG;
    if (c->state != ST_ALIAS_VALID || !c->beta_table_built) return LDAREF_ERR_STATE;
    memcpy(split, c->bsplit, sizeof(uint32_t) * (size_t)c->K);
    memcpy(alias, c->balias, sizeof(uint32_t) * (size_t)c->K);
    *C = c->bC;
    *QB = c->QB;
    return LDAREF_OK;
}
