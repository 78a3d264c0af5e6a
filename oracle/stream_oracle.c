/*
 * CPU oracle for Stream mask estimation and masked attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow implementation used to check
 * the GPU library; nothing on the product path may call it.  It shares no code
 * with the HIP kernels.
 *
 * What it follows:
 *   - Algorithm 2 ("Stream", Appendix C of the paper), step by step in the
 *     listing's order and notation (nodes (f,l), midpoint m, branches B,
 *     validity omega, representative r, score s, top-k indices t, output I),
 *     with the block-level mask C^blk and the padding of the preamble.
 *   - Eq. (2) (masked softmax attention) restricted to the retained blocks, and
 *     the column sums of its probabilities ("vertical attention scores",
 *     Section 4.1).
 *
 * Readings taken where the listing is ambiguous (each is also listed in the
 * design notes of this repository):
 *   - node ranges are ranges of KEY-BLOCK indices: N = T_p / b_k replaces T in
 *     the initialisation, and j runs 0..k-1;
 *   - the midpoint is taken on the half-open range, m = floor((f+l+1)/2), so a
 *     node of n blocks splits into floor(n/2) and ceil(n/2) blocks;
 *   - "top-k indices": larger score first, equal scores -> lower branch
 *     position; the selected branches are stored in positional order;
 *   - log in n_it is base 2;
 *   - k counts key blocks, so I has k entries per query block.
 *
 * Arithmetic: inputs are float arrays holding exactly the values of the
 * workload's dtype (fp32, or bf16 widened); every product and sum is fp64.
 * No blocking, no reuse of a parent's score, no skipped levels.
 *
 * Parity pins (tests/test_oracle_*.py): brute force over dense T x T scores,
 * exact block top-k when N <= 2k, closed forms for monotone scores, the count
 * law cnt = min(k, q+1), causality, scale invariance, a hand-traced example,
 * dense softmax attention when k >= N.  The paper's quality claims (behaviour
 * preserved under 90-99 % pruning) need its models: parity unpinned.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the row loops will use (for reporting next to a timing). */
int stream_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Masks C given by a rule instead of a T x T array (Alg. 2 takes any C; these are the ones
   the models of the paper use: causal layers, sliding-window layers, and no mask = Alg. 1). */
enum { MASK_CAUSAL = 0, MASK_FULL = 1, MASK_SLIDING = 2 };

typedef struct {
    const float *Q;           /* [T, d]  one query head              */
    const float *K;           /* [T, d]  its key head                */
    const unsigned char *C;   /* [T, T] attention mask, or NULL = the rule below */
    long T;                   /* real tokens (before padding)        */
    int d, bq, bk;            /* head dim, query block size b_q, key block size b_k */
    int kind;                 /* MASK_CAUSAL: C[t,u] = 1 iff u <= t; MASK_FULL: all ones;
                                 MASK_SLIDING: u <= t and t - u < window                  */
    long window;
} problem_t;

/* C[t,u] after the preamble's zero padding: rows/cols >= T are 0. */
static int mask_C(const problem_t *p, long t, long u)
{
    if (t >= p->T || u >= p->T) return 0;
    if (p->C) return p->C[t * p->T + u] != 0;
    if (p->kind == MASK_FULL) return 1;
    if (p->kind == MASK_SLIDING) return u <= t && t - u < p->window;
    return u <= t;
}

/* C^blk[q,r] = max_{m,n} C[q,m,r,n]. */
static int mask_Cblk(const problem_t *p, long q, long r)
{
    const int bq = p->bq, bk = p->bk;
    if (!p->C && p->kind == MASK_CAUSAL) {
        /* causal: some real key of block r is <= some real query of block q
           iff the block's first key is <= the block's last real query        */
        long first_key = r * bk;
        long last_query = ((q + 1) * (long)bq < p->T ? (q + 1) * (long)bq : p->T) - 1;
        return first_key < p->T && q * (long)bq < p->T && first_key <= last_query;
    }
    for (int m = 0; m < bq; ++m)
        for (int n = 0; n < bk; ++n)
            if (mask_C(p, q * bq + m, r * bk + n)) return 1;
    return 0;
}

/* s = max over (m,n) with C = 1 of <Q[q,m,:], K[r,n,:]>   (score line of Alg. 2; Eq. (4)) */
static double block_score(const problem_t *p, long q, long r)
{
    const int bq = p->bq, bk = p->bk, d = p->d;
    double s = -INFINITY;
    for (int m = 0; m < bq; ++m) {
        long t = q * bq + m;
        for (int n = 0; n < bk; ++n) {
            long u = r * bk + n;
            if (!mask_C(p, t, u)) continue;
            const float *qv = p->Q + t * d, *kv = p->K + u * d;
            double acc = 0.0;
            for (int i = 0; i < d; ++i) acc += (double)qv[i] * (double)kv[i];
            if (acc > s) s = acc;
        }
    }
    return s;
}

double stream_oracle_block_score(const float *Q, const float *K, const unsigned char *C,
                                 long T, int d, int b, long q, long r)
{
    problem_t p = {Q, K, C, T, d, b, b, MASK_CAUSAL, 0};
    return block_score(&p, q, r);
}

double stream_oracle_block_score_rule(const float *Q, const float *K, int mask_kind, long window,
                                      long T, int d, int b, long q, long r)
{
    problem_t p = {Q, K, NULL, T, d, b, b, mask_kind, window};
    return block_score(&p, q, r);
}

/* The same for b_q x b_k blocks (q counts query blocks of b_q tokens, r key blocks of b_k). */
double stream_oracle_block_score_rect(const float *Q, const float *K, const unsigned char *C,
                                      int mask_kind, long window,
                                      long T, int d, int bq, int bk, long q, long r)
{
    problem_t p = {Q, K, C, T, d, bq, bk, mask_kind, window};
    return block_score(&p, q, r);
}

static long gcd_l(long a, long b) { while (b) { long t = a % b; a = b; b = t; } return a; }

/* T_p of the preamble of Alg. 2: T rounded up to a multiple of lcm(b_q, b_k). */
long stream_oracle_padded_len(long T, int bq, int bk)
{
    const long l = (long)bq / gcd_l(bq, bk) * bk;
    return (T + l - 1) / l * l;
}

static long ceil_log2(long n)
{
    long it = 0, v = 1;
    while (v < n) { v <<= 1; ++it; }
    return it;
}

long stream_oracle_n_it(long T, int b)
{
    long N = (T + b - 1) / b;
    return ceil_log2(N);
}

typedef struct { double s; int pos; } cand_t;

static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

static int int_cmp(const void *a, const void *b)
{
    int x = *(const int *)a, y = *(const int *)b;
    return (x > y) - (x < y);
}

/*
 * Algorithm 2 for the query blocks listed in qlist (rows are independent).
 *
 *   n_levels < 0  -> n_it = ceil(log2(T_p / b_k)) as printed
 *   idx   [nq, k]  retained key-block ids, ascending, padded with -1
 *   cnt   [nq]     number of retained blocks
 *   score [nq, k]  block score of each retained block, padded with -inf (may be NULL)
 *   trace [nq, levels, k, 2]  (f,l) of the nodes kept after each level, or NULL
 *   evals [2]      += finite-score branch evaluations: [0] as executed here,
 *                  [1] those whose representative differs from the parent node's
 *                  (the evaluations that cannot be inherited), may be NULL
 */
int stream_oracle_prune_head_rect(const float *Q, const float *K, const unsigned char *C,
                                  int mask_kind, long window,
                                  long T, int d, int bq, int bk, int k, int n_levels,
                                  const int *qlist, int nq,
                                  int *idx, int *cnt, double *score, int *trace, long long *evals)
{
    if (!Q || !K || T <= 0 || d <= 0 || bq <= 0 || bk <= 0 || k <= 0 || nq < 0) return 1;
    if (mask_kind < MASK_CAUSAL || mask_kind > MASK_SLIDING) return 1;
    if (mask_kind == MASK_SLIDING && window < 1) return 1;
    problem_t p = {Q, K, C, T, d, bq, bk, mask_kind, window};
    /* preamble: pad to a multiple of l = lcm(b_q, b_k); block views are index arithmetic;
       the nodes range over the T_p / b_k key blocks */
    const long T_p = stream_oracle_padded_len(T, bq, bk);
    const long N = T_p / bk;
    const long n_it = n_levels < 0 ? ceil_log2(N) : n_levels;
    long long ev_all = 0, ev_new = 0;

#pragma omp parallel for schedule(dynamic, 1) reduction(+ : ev_all, ev_new)
    for (int qi = 0; qi < nq; ++qi) {
        const long q = qlist[qi];
        long *f = (long *)malloc(sizeof(long) * k), *l = (long *)malloc(sizeof(long) * k);
        long *rep = (long *)malloc(sizeof(long) * k); /* representative of each node, -1 = none yet */
        long *Bf = (long *)malloc(sizeof(long) * 2 * k), *Bl = (long *)malloc(sizeof(long) * 2 * k);
        long *Br = (long *)malloc(sizeof(long) * 2 * k);
        double *s = (double *)malloc(sizeof(double) * 2 * k);
        cand_t *order = (cand_t *)malloc(sizeof(cand_t) * 2 * k);
        int *t = (int *)malloc(sizeof(int) * k);

        /* k nodes: equal split of the key blocks */
        for (int j = 0; j < k; ++j) {
            f[j] = (long)(((long long)j * N) / k);
            l[j] = (long)(((long long)(j + 1) * N) / k) - 1;
            rep[j] = -1;
        }
        for (long i = 0; i < n_it; ++i) {
            /* split every node at its midpoint into two branches */
            for (int j = 0; j < k; ++j) {
                long m = (f[j] + l[j] + 1) / 2; /* an empty node (l = f-1) gives two empty branches */
                Bf[2 * j] = f[j];     Bl[2 * j] = m - 1;
                Bf[2 * j + 1] = m;    Bl[2 * j + 1] = l[j];
            }
            for (int h = 0; h < 2 * k; ++h) {
                /* omega = max_{r in B} C^blk[q,r]; first r with C^blk = 1 */
                long r = -1;
                for (long c = Bf[h]; c <= Bl[h]; ++c)
                    if (mask_Cblk(&p, q, c)) { r = c; break; }
                Br[h] = r;
                if (r < 0) { s[h] = -INFINITY; continue; }
                s[h] = block_score(&p, q, r);
                ev_all += 1;
                if (rep[h / 2] != r) ev_new += 1;
            }
            /* top-k indices of s_1..s_2k */
            for (int h = 0; h < 2 * k; ++h) { order[h].s = s[h]; order[h].pos = h; }
            qsort(order, 2 * k, sizeof(cand_t), cand_cmp);
            for (int j = 0; j < k; ++j) t[j] = order[j].pos;
            qsort(t, k, sizeof(int), int_cmp);
            for (int j = 0; j < k; ++j) { f[j] = Bf[t[j]]; l[j] = Bl[t[j]]; rep[j] = Br[t[j]]; }
            if (trace)
                for (int j = 0; j < k; ++j) {
                    long o = (((long)qi * n_it + i) * k + j) * 2;
                    int live = rep[j] >= 0;
                    trace[o] = live ? (int)f[j] : -1;
                    trace[o + 1] = live ? (int)l[j] : -1;
                }
        }
        /* I_qj = first valid r of the final node, or empty */
        int c_out = 0;
        for (int j = 0; j < k; ++j) {
            long r = -1;
            for (long c = f[j]; c <= l[j]; ++c)
                if (mask_Cblk(&p, q, c)) { r = c; break; }
            if (r >= 0) t[c_out++] = (int)r;
        }
        qsort(t, c_out, sizeof(int), int_cmp);
        for (int j = 0; j < k; ++j) {
            idx[(long)qi * k + j] = j < c_out ? t[j] : -1;
            if (score) score[(long)qi * k + j] = j < c_out ? block_score(&p, q, t[j]) : -INFINITY;
        }
        cnt[qi] = c_out;
        free(f); free(l); free(rep); free(Bf); free(Bl); free(Br); free(s); free(order); free(t);
    }
    if (evals) { evals[0] += ev_all; evals[1] += ev_new; }
    return 0;
}

/* b_q = b_k = b. */
int stream_oracle_prune_head_rule(const float *Q, const float *K, const unsigned char *C,
                                  int mask_kind, long window,
                                  long T, int d, int b, int k, int n_levels,
                                  const int *qlist, int nq,
                                  int *idx, int *cnt, double *score, int *trace, long long *evals)
{
    return stream_oracle_prune_head_rect(Q, K, C, mask_kind, window, T, d, b, b, k, n_levels, qlist, nq,
                                         idx, cnt, score, trace, evals);
}

/* The same with the causal mask (or an explicit C). */
int stream_oracle_prune_head(const float *Q, const float *K, const unsigned char *C,
                             long T, int d, int b, int k, int n_levels,
                             const int *qlist, int nq,
                             int *idx, int *cnt, double *score, int *trace, long long *evals)
{
    return stream_oracle_prune_head_rule(Q, K, C, MASK_CAUSAL, 0, T, d, b, k, n_levels, qlist, nq,
                                         idx, cnt, score, trace, evals);
}

/*
 * Eq. (2) with the mask M given by idx/cnt (block ids per query block) and the
 * mask C (an explicit [T, T] array, else the rule named by mask_kind) inside retained blocks:  for each real query token t of the query
 * blocks in qlist,
 *     S~[t,u] = scale * <Q_t, K_u>   for u in retained blocks of block(t), u <= t
 *     P~ = softmax(S~),  O_t = sum_u P~[t,u] V_u,  lse_t = log sum_u exp(S~[t,u])
 *     mass[u] += P~[t,u]             (column sums: received attention per key)
 * idx is [nq, k] (rows aligned with qlist), O is [T, d] and lse [T] (only rows of
 * the listed blocks are written), mass [T] is accumulated into (caller zeroes).
 */
int stream_oracle_attn_head_mask(const float *Q, const float *K, const float *V,
                                 const unsigned char *C, int mask_kind, long window,
                                 long T, int d, int bq, int bk, int k, double scale,
                                 const int *qlist, int nq, const int *idx, const int *cnt,
                                 double *O, double *lse, double *mass)
{
    if (!Q || !K || !V || !idx || !cnt || T <= 0) return 1;
    if (mask_kind < MASK_CAUSAL || mask_kind > MASK_SLIDING) return 1;
    if (mask_kind == MASK_SLIDING && window < 1) return 1;
    problem_t p = {Q, K, C, T, d, bq, bk, mask_kind, window};
#pragma omp parallel for schedule(dynamic, 1)
    for (int qi = 0; qi < nq; ++qi) {
        const long q = qlist[qi];
        const int c = cnt[qi];
        double *sc = (double *)malloc(sizeof(double) * (size_t)(c > 0 ? c : 1) * bk);
        long *key = (long *)malloc(sizeof(long) * (size_t)(c > 0 ? c : 1) * bk);
        for (int m = 0; m < bq; ++m) {
            const long t = q * bq + m;
            if (t >= T) break;
            long nk = 0;
            double mx = -INFINITY;
            for (int j = 0; j < c; ++j) {
                const long r = idx[(long)qi * k + j];
                for (int n = 0; n < bk; ++n) {
                    const long u = r * bk + n;
                    if (!mask_C(&p, t, u)) continue;
                    double acc = 0.0;
                    for (int i = 0; i < d; ++i) acc += (double)Q[t * d + i] * (double)K[u * d + i];
                    acc *= scale;
                    sc[nk] = acc; key[nk] = u; ++nk;
                    if (acc > mx) mx = acc;
                }
            }
            double *o = O + t * d;
            for (int i = 0; i < d; ++i) o[i] = 0.0;
            if (nk == 0) { if (lse) lse[t] = -INFINITY; continue; }
            double z = 0.0;
            for (long x = 0; x < nk; ++x) z += exp(sc[x] - mx);
            const double L = mx + log(z);
            if (lse) lse[t] = L;
            for (long x = 0; x < nk; ++x) {
                const double pr = exp(sc[x] - L);
                const float *v = V + key[x] * d;
                for (int i = 0; i < d; ++i) o[i] += pr * (double)v[i];
                if (mass) {
#pragma omp atomic
                    mass[key[x]] += pr;
                }
            }
        }
        free(sc); free(key);
    }
    return 0;
}

/* The mask C given by a rule. */
int stream_oracle_attn_head_rect(const float *Q, const float *K, const float *V,
                                 int mask_kind, long window,
                                 long T, int d, int bq, int bk, int k, double scale,
                                 const int *qlist, int nq, const int *idx, const int *cnt,
                                 double *O, double *lse, double *mass)
{
    return stream_oracle_attn_head_mask(Q, K, V, NULL, mask_kind, window, T, d, bq, bk, k, scale, qlist, nq,
                                        idx, cnt, O, lse, mass);
}

int stream_oracle_attn_head_rule(const float *Q, const float *K, const float *V,
                                 int mask_kind, long window,
                                 long T, int d, int b, int k, double scale,
                                 const int *qlist, int nq, const int *idx, const int *cnt,
                                 double *O, double *lse, double *mass)
{
    return stream_oracle_attn_head_rect(Q, K, V, mask_kind, window, T, d, b, b, k, scale, qlist, nq, idx,
                                        cnt, O, lse, mass);
}

int stream_oracle_attn_head(const float *Q, const float *K, const float *V,
                            long T, int d, int b, int k, double scale,
                            const int *qlist, int nq, const int *idx, const int *cnt,
                            double *O, double *lse, double *mass)
{
    return stream_oracle_attn_head_rule(Q, K, V, MASK_CAUSAL, 0, T, d, b, k, scale, qlist, nq, idx, cnt,
                                        O, lse, mass);
}
