/*
 * stand_oracle.c -- plain, slow, single-threaded CPU oracle for the STAND speculation step.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or import this
 * file; it exists so that tests, the smoke check and the CPU-baseline leg of the
 * benchmark have an independent statement of what the method computes.  It shares no
 * code, header, table or constant generator with the HIP library.
 *
 * What it follows (paper = arxiv 2506.04708, "STAND"):
 *   - row distribution p = softmax(logits / T)                 Sec. 4.1, Sec. 5 setup (T = 0.6)
 *   - observation = top-k ids and probabilities of a row       Sec. 4.1 "Efficient logit approximation"
 *   - running-mean merge k/(k+1), 1/(k+1), absent = 0,
 *     truncate to top-k                                         Sec. 4.1 "Efficient logit approximation"
 *   - multi-level lookup, longest order first, first hit wins   Sec. 4.2 "Stochastic tree drafting"
 *   - children of a tree node = samples without replacement
 *     via Gumbel-Top-K, phi' = phi - log(-log U)                Sec. 4.2 "Gumbel-Top-K sampling"
 *   - accept x~q with prob min(1, p/q); on rejection resample
 *     from norm(max(0, p - q))                                  Sec. 3.2
 *   - several children of one node: the single-draft rule applied recursively to the
 *     residual target and to the proposal conditioned on the earlier rejections
 *     (the paper only says the sampled tokens "undergo standard speculative sampling
 *     verification", Sec. 4.2; the recursive reading is this build's).
 *
 * Everything is dense and naive on purpose: a row is a V-vector, top-k is a full sort,
 * the n-gram table is keyed by the full token tuple.
 *
 * Arithmetic.  All probabilities are IEEE binary32.  So that a second implementation can
 * reach the same bits, the transcendental functions are spelled out as fixed sequences of
 * correctly rounded operations (so_exp2, so_log below), the row normaliser is an integer
 * sum (order free), and every other formula is written with one rounding per operation
 * in the order shown.  Build with -ffp-contract=off and without -ffast-math.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SO_MAX_K 32
#define SO_MAX_ORDER 8
#define SO_DT_BF16 0
#define SO_DT_F32 1
#define SO_STREAM_DRAFT 0u
#define SO_STREAM_ACCEPT 1u
#define SO_STREAM_BONUS 2u

/* how the children of a node are drawn from its table entry (Sec. 3.1, Sec. 4.2, Table 5) */
/* which rows of a verified tree are merged into the table (Sec. 4.1) */
#define SO_UPDATE_ACCEPTED_PATH 0 /* the rows that produced committed tokens                       */
#define SO_UPDATE_ALL_NODES 1     /* the row of every drafted node, under the context that node    */
                                  /* would have if its path were accepted (a table stress variant) */
/* what a table update does to an entry that exists (Sec. 4.1; Sec. 5.1 on replacing) */
#define SO_MERGE_MEAN 0    /* running mean of all observations (the method)      */
#define SO_MERGE_REPLACE 1 /* the newest observation only (comparison policy)   */
#define SO_DRAFT_GUMBEL_TOPK 0   /* stochastic, Gumbel-Top-K (the method's own)                */
#define SO_DRAFT_MULTINOMIAL 1   /* stochastic, sequential sampling without replacement        */
#define SO_DRAFT_DETERMINISTIC 2 /* the most probable stored tokens; proposal treated as one-hot */

/* ------------------------------------------------------------------------------------------
 * Counter-based uniforms: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).
 * key = 64-bit seed; counter = (token >> 2, node | stream << 24, step low, b | step high << 20);
 * the word used is token & 3.  U = (2 * (x >> 9) + 1) * 2^-24: an odd 24-bit integer scaled,
 * exact in binary32 and strictly inside (0, 1).
 * ---------------------------------------------------------------------------------------- */
static void philox4x32_10(const uint32_t ctr_in[4], uint64_t seed, uint32_t out[4])
{
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void so_philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t out[4])
{
    uint32_t ctr[4] = {c0, c1, c2, c3};
    philox4x32_10(ctr, seed, out);
}

float so_uniform(uint64_t seed, uint32_t b, uint64_t step, uint32_t node, uint32_t token, uint32_t stream)
{
    uint32_t ctr[4], out[4];
    ctr[0] = token >> 2;
    ctr[1] = node | (stream << 24);
    ctr[2] = (uint32_t)step;
    ctr[3] = b | ((uint32_t)(step >> 32) << 20);
    philox4x32_10(ctr, seed, out);
    uint32_t x = out[token & 3u];
    return (float)(2u * (x >> 9) + 1u) * 0x1p-24f;
}

/* 64 uniform bits of (b, step, node, stream): words 0 and 1 of the block of token group 0. */
uint64_t so_uniform_u64(uint64_t seed, uint32_t b, uint64_t step, uint32_t node, uint32_t stream)
{
    uint32_t ctr[4], out[4];
    ctr[0] = 0u;
    ctr[1] = node | (stream << 24);
    ctr[2] = (uint32_t)step;
    ctr[3] = b | ((uint32_t)(step >> 32) << 20);
    philox4x32_10(ctr, seed, out);
    return ((uint64_t)out[0] << 32) | (uint64_t)out[1];
}

/* ------------------------------------------------------------------------------------------
 * so_exp2(y) ~ 2^y for y <= small positive.  y < -64 gives exactly 0.
 * k = round-half-even(y), f = y - k in [-1/2, 1/2], 2^f = 1 + f*Q(f), Q of degree 5
 * evaluated by Horner with fused multiply-adds; result scaled by 2^k exactly.
 * ---------------------------------------------------------------------------------------- */
float so_exp2(float y)
{
    if (!(y >= -64.0f)) return 0.0f;
    float k = rintf(y);
    float f = y - k;
    float q = 0x1.44138ap-13f;
    q = fmaf(q, f, 0x1.5f0890p-10f);
    q = fmaf(q, f, 0x1.3b2a54p-7f);
    q = fmaf(q, f, 0x1.c6af6cp-5f);
    q = fmaf(q, f, 0x1.ebfbe0p-3f);
    q = fmaf(q, f, 0x1.62e430p-1f);
    float p = fmaf(q, f, 1.0f);
    return ldexpf(p, (int)k);
}

/* ------------------------------------------------------------------------------------------
 * so_log(x) ~ ln x for positive normal x.
 * x = 2^e * m with m in (sqrt(1/2), sqrt 2];  t = m - 1;  s = t / (2 + t);  z = s*s;
 * ln m = 2s + s*z*(2/3 + z*(2/5 + z*(2/7 + z*2/9)));  ln x = e*ln2 + ln m.
 * ---------------------------------------------------------------------------------------- */
float so_log(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, 4);
    int e = (int)(bits >> 23) - 127;
    uint32_t mb = (bits & 0x007FFFFFu) | 0x3F800000u;
    float m;
    memcpy(&m, &mb, 4);
    if (m > 0x1.6a09e6p+0f) { m = m * 0.5f; e += 1; }
    float t = m - 1.0f;
    float s = t / (2.0f + t);
    float z = s * s;
    float w = 0x1.c71c72p-3f;              /* 2/9 */
    w = fmaf(w, z, 0x1.24924ap-2f);        /* 2/7 */
    w = fmaf(w, z, 0x1.99999ap-2f);        /* 2/5 */
    w = fmaf(w, z, 0x1.555556p-1f);        /* 2/3 */
    float lnm = fmaf(s * z, w, 2.0f * s);
    return fmaf((float)e, 0x1.62e430p-1f, lnm);
}

/* ------------------------------------------------------------------------------------------
 * Row distribution, Sec. 4.1 / Sec. 5 (temperature softmax).
 *   c   = (float)(log2(e) / T)          computed in double, rounded once
 *   y_v = (l_v - m) * c                 m = max_v l_v; subtraction, then multiplication
 *   e_v = so_exp2(y_v)
 *   S   = sum_v floor(e_v * 2^F)        integer, F = min(40, 62 - ceil(log2 V)); order free
 *   s   = (float)((double)S * 2^-F)
 *   p_v = e_v / s
 * ---------------------------------------------------------------------------------------- */
static float widen(const void *row, int dtype, int64_t v)
{
    if (dtype == SO_DT_F32) return ((const float *)row)[v];
    uint32_t bits = (uint32_t)((const uint16_t *)row)[v] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

static int fx_bits(int V)
{
    int lg = 0;
    while (((int64_t)1 << lg) < (int64_t)V) ++lg;
    int f = 62 - lg;
    return f > 40 ? 40 : f;
}

float so_scale(float temperature)
{
    return (float)(1.4426950408889634 / (double)temperature);
}

void so_row_softmax(const void *row, int dtype, int V, float temperature,
                    float *p_out /* [V] or NULL */, float *m_out, float *s_out, uint64_t *S_out)
{
    float c = so_scale(temperature);
    float m = widen(row, dtype, 0);
    for (int v = 1; v < V; ++v) {
        float l = widen(row, dtype, v);
        if (l > m) m = l;
    }
    int F = fx_bits(V);
    uint64_t S = 0;
    for (int v = 0; v < V; ++v) {
        float d = widen(row, dtype, v) - m;
        float y = d * c;
        float e = so_exp2(y);
        S += (uint64_t)floor(ldexp((double)e, F));
    }
    float s = (float)ldexp((double)S, -F);
    if (p_out) {
        for (int v = 0; v < V; ++v) {
            float d = widen(row, dtype, v) - m;
            float y = d * c;
            p_out[v] = so_exp2(y) / s;
        }
    }
    if (m_out) *m_out = m;
    if (s_out) *s_out = s;
    if (S_out) *S_out = S;
}

/* The integer terms of S: F_out[v] = floor(e_v * 2^F). */
void so_row_masses(const void *row, int dtype, int V, float temperature, uint64_t *F_out)
{
    float c = so_scale(temperature);
    float m = widen(row, dtype, 0);
    for (int v = 1; v < V; ++v) {
        float l = widen(row, dtype, v);
        if (l > m) m = l;
    }
    int F = fx_bits(V);
    for (int v = 0; v < V; ++v) {
        float d = widen(row, dtype, v) - m;
        float y = d * c;
        F_out[v] = (uint64_t)floor(ldexp((double)so_exp2(y), F));
    }
}

/* ------------------------------------------------------------------------------------------
 * Top-k of a vector by (value descending, id ascending): full sort, keep the first k.
 * -0 and +0 compare equal, so the id decides between them.
 * ---------------------------------------------------------------------------------------- */
typedef struct { float val; int32_t id; } so_pair;

static int pair_cmp(const void *a, const void *b)
{
    const so_pair *x = (const so_pair *)a, *y = (const so_pair *)b;
    if (x->val > y->val) return -1;
    if (x->val < y->val) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

void so_topk(const float *vals, int n, int k, int32_t *idx_out, float *val_out)
{
    so_pair *tmp = (so_pair *)malloc(sizeof(so_pair) * (size_t)n);
    for (int i = 0; i < n; ++i) { tmp[i].val = vals[i]; tmp[i].id = i; }
    qsort(tmp, (size_t)n, sizeof(so_pair), pair_cmp);
    for (int i = 0; i < k; ++i) { idx_out[i] = tmp[i].id; val_out[i] = tmp[i].val; }
    free(tmp);
}

/* Observation of a row (Sec. 4.1): its k largest entries.  The ranking is taken on the
 * raw logits (value desc, id asc) -- the softmax is monotone, so this is the top-k of p,
 * with ties between different logits that round to one probability resolved by the logit. */
void so_row_obs(const void *row, int dtype, int V, float temperature, int K,
                int32_t *idx_out, float *p_out, float *m_out, float *s_out)
{
    float *l = (float *)malloc(sizeof(float) * (size_t)V);
    float *lv = (float *)malloc(sizeof(float) * (size_t)K);
    for (int v = 0; v < V; ++v) l[v] = widen(row, dtype, v);
    so_topk(l, V, K, idx_out, lv);
    float m, s;
    so_row_softmax(row, dtype, V, temperature, NULL, &m, &s, NULL);
    float c = so_scale(temperature);
    for (int i = 0; i < K; ++i) {
        float d = lv[i] - m;
        float y = d * c;
        p_out[i] = so_exp2(y) / s;
    }
    if (m_out) *m_out = m;
    if (s_out) *s_out = s;
    free(l);
    free(lv);
}

/* ------------------------------------------------------------------------------------------
 * Running-mean merge of one table entry with one observation (Sec. 4.1).
 * Entry seen `count` times holds the mean mu over its stored ids.  For every id x in the
 * union:  mu'(x) = (count * mu(x) + obs(x)) / (count + 1), absent terms = 0
 * (the paper's weights k/(k+1) and 1/(k+1) written over a common denominator);
 * keep the K largest by (mu' desc, id asc).  count == 0: the entry becomes the observation.
 * ---------------------------------------------------------------------------------------- */
void so_merge(uint32_t count, const int32_t *ids, const float *mu, int K,
              const int32_t *obs_ids, const float *obs_p, int32_t *ids_out, float *mu_out)
{
    if (count == 0) {
        for (int i = 0; i < K; ++i) { ids_out[i] = obs_ids[i]; mu_out[i] = obs_p[i]; }
        return;
    }
    so_pair u[2 * SO_MAX_K];
    int n = 0;
    float cf = (float)count;
    float denom = cf + 1.0f;
    for (int i = 0; i < K; ++i) {
        float o = 0.0f;
        for (int j = 0; j < K; ++j) if (obs_ids[j] == ids[i]) o = obs_p[j];
        float t = cf * mu[i];
        t = t + o;
        u[n].id = ids[i];
        u[n].val = t / denom;
        ++n;
    }
    for (int j = 0; j < K; ++j) {
        int present = 0;
        for (int i = 0; i < K; ++i) if (ids[i] == obs_ids[j]) present = 1;
        if (present) continue;
        float t = cf * 0.0f;
        t = t + obs_p[j];
        u[n].id = obs_ids[j];
        u[n].val = t / denom;
        ++n;
    }
    qsort(u, (size_t)n, sizeof(so_pair), pair_cmp);
    for (int i = 0; i < K; ++i) { ids_out[i] = u[i].id; mu_out[i] = u[i].val; }
}

/* ------------------------------------------------------------------------------------------
 * 64-bit fingerprint of a key (order n, its n context tokens oldest first).  The table is
 * keyed by the full tuple; the fingerprint is what a fixed-width hash table would store,
 * and is exported so that two implementations can compare key sets.
 * ---------------------------------------------------------------------------------------- */
static uint64_t fmix64(uint64_t h)
{
    h ^= h >> 33; h *= 0xff51afd7ed558ccdULL;
    h ^= h >> 33; h *= 0xc4ceb9fe1a85ec53ULL;
    h ^= h >> 33;
    return h;
}

/* h = fmix64(n * C + sum_i M_i * (x_i + 1)) with x_i the token i positions before the end of the
 * key (x_0 = newest) and M_0..M_7 fixed odd multipliers; 0 is mapped to 1.  The terms do not
 * depend on each other, and keys that share their newest tokens share their first terms. */
static const uint64_t fp_mult[SO_MAX_ORDER] = {
    0x9E3779B97F4A7C15ULL, 0xC2B2AE3D27D4EB4FULL, 0x165667B19E3779F9ULL, 0xD6E8FEB86659FD93ULL,
    0xA0761D6478BD642FULL, 0xE7037ED1A0B428DBULL, 0x8EBC6AF09C88C6E3ULL, 0x589965CC75374CC3ULL};

uint64_t so_fingerprint(int n, const int32_t *tokens)
{
    uint64_t acc = (uint64_t)n * 0x2545F4914F6CDD1DULL;
    for (int i = 0; i < n; ++i)
        acc += fp_mult[i] * ((uint64_t)(uint32_t)tokens[n - 1 - i] + 1u);
    uint64_t h = fmix64(acc);
    return h ? h : 1;
}

/* ------------------------------------------------------------------------------------------
 * Gumbel-Top-K (Sec. 4.2): score_i = ln mu_i - ln(-ln U_i); the c largest scores, in
 * order, are c draws without replacement.  Candidates are the stored ids with mu > 0.
 * Returns the number of tokens written (min(c, #candidates)).
 * ---------------------------------------------------------------------------------------- */
int so_gumbel_topk(const int32_t *ids, const float *mu, int K, int c, const float *U /* [K] */,
                   int32_t *tok_out)
{
    so_pair sc[SO_MAX_K];
    int n = 0;
    for (int i = 0; i < K; ++i) {
        if (!(mu[i] > 0.0f)) continue;
        float g = so_log(-so_log(U[i]));
        sc[n].val = so_log(mu[i]) - g;
        sc[n].id = ids[i];
        ++n;
    }
    qsort(sc, (size_t)n, sizeof(so_pair), pair_cmp);
    int w = c < n ? c : n;
    for (int j = 0; j < w; ++j) tok_out[j] = sc[j].id;
    return w;
}

static float support_sum(const float *x, int K);

/* Sequential sampling without replacement (the "basic stochastic drafting" of Table 5): draw j
 * picks among the candidates not drawn yet with probability proportional to mu.  z = sum of the
 * remaining mu (support_sum's order); t = U_j * z; the pick is the first remaining candidate, in stored
 * order, whose running sum exceeds t (the last remaining one if rounding leaves none).  Same law
 * as Gumbel-Top-K (Plackett-Luce). */
int so_multinomial_wor(const int32_t *ids, const float *mu, int K, int c, const float *U /* [c] */,
                       int32_t *tok_out)
{
    int left[SO_MAX_K];
    int n = 0;
    for (int i = 0; i < K; ++i) { left[i] = mu[i] > 0.0f; n += left[i]; }
    int w = c < n ? c : n;
    for (int j = 0; j < w; ++j) {
        float rest[SO_MAX_K];
        for (int i = 0; i < K; ++i) rest[i] = left[i] ? mu[i] : 0.0f;
        float z = support_sum(rest, K);
        float t = U[j] * z;
        float a = 0.0f;
        int pick = -1, last = -1;
        for (int i = 0; i < K; ++i) {
            if (!left[i]) continue;
            last = i;
            a = a + mu[i];
            if (pick < 0 && t < a) pick = i;
        }
        if (pick < 0) pick = last;
        tok_out[j] = ids[pick];
        left[pick] = 0;
    }
    return w;
}

/* Deterministic drafting (Sec. 3.1): the c most probable stored tokens, (mu desc, id asc). */
int so_top_c(const int32_t *ids, const float *mu, int K, int c, int32_t *tok_out)
{
    so_pair sc[SO_MAX_K];
    int n = 0;
    for (int i = 0; i < K; ++i) {
        if (!(mu[i] > 0.0f)) continue;
        sc[n].val = mu[i];
        sc[n].id = ids[i];
        ++n;
    }
    qsort(sc, (size_t)n, sizeof(so_pair), pair_cmp);
    int w = c < n ? c : n;
    for (int j = 0; j < w; ++j) tok_out[j] = sc[j].id;
    return w;
}

/* ------------------------------------------------------------------------------------------
 * Verification of the children of one node (Sec. 3.2 applied recursively).
 *   p       dense target distribution of the node's row
 *   ids/mu  the table entry the children were drawn from (proposal support)
 *   child_tok[0..nchild)  drafted tokens in rank order (= draw order)
 *   omega[j]              the uniform of child j
 * State:  r_i = residual target on support token i; outside the support the residual is
 *         p(v) * rho;  w_i = proposal, normalised over what has not been rejected yet.
 * Round j:  accept iff omega_j * w_i < r_i  (i.e. omega < r/w, so r >= w always accepts);
 *           else  r <- max(r - w, 0) / Z  with  Z = 1 - sum_i min(r_i, w_i)
 *           (= the mass of max(r - w, 0) when r sums to 1),  w_i <- 0, w renormalised.
 * Returns the rank of the accepted child or -1; leaves the final r_i and rho for the
 * resampling step.
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    float r[SO_MAX_K];
    float w[SO_MAX_K];
    float rho;
    int rounds;
    int near_threshold; /* |omega - r/w| < 1e-6 on some round */
} so_node_state;

/* Sum over the support as a balanced pairwise tree on SO_MAX_K slots (absent slots are +0):
 * neighbours first, then groups of 4, 8, 16, 32 -- one binary32 rounding per addition.  The
 * order is part of the numeric contract (any fixed order would do for the method; this one
 * needs log2 steps on a machine that adds in parallel). */
static float support_sum(const float *x, int K)
{
    float t[SO_MAX_K];
    for (int i = 0; i < SO_MAX_K; ++i) t[i] = i < K ? x[i] : 0.0f;
    for (int n = SO_MAX_K; n > 1; n /= 2)
        for (int i = 0; i < n / 2; ++i) t[i] = t[2 * i] + t[2 * i + 1];
    return t[0];
}

/* onehot != 0 (deterministic drafting, Sec. 3.1): the proposal of round j is the one-hot vector
 * on child j, so the child is accepted with probability r(x) and a rejection removes only x. */
int so_verify_node(const float *p, int K, const int32_t *ids, const float *mu,
                   int nchild, const int32_t *child_tok, const float *omega, so_node_state *st, int onehot)
{
    float zw = 0.0f;
    for (int i = 0; i < K; ++i) { st->w[i] = mu[i] > 0.0f ? mu[i] : 0.0f; }
    zw = support_sum(st->w, K);
    for (int i = 0; i < K; ++i) {
        st->w[i] = zw > 0.0f ? st->w[i] / zw : 0.0f;
        st->r[i] = p[ids[i]];
    }
    st->rho = 1.0f;
    st->rounds = 0;
    st->near_threshold = 0;
    for (int j = 0; j < nchild; ++j) {
        if (child_tok[j] < 0) break;
        int i = -1;
        for (int q = 0; q < K; ++q) if (ids[q] == child_tok[j]) i = q;
        if (i < 0) break; /* cannot happen for a tree drafted from this entry */
        st->rounds++;
        if (onehot) for (int q = 0; q < K; ++q) st->w[q] = q == i ? 1.0f : 0.0f;
        float lhs = omega[j] * st->w[i];
        if (st->w[i] > 0.0f && fabs((double)omega[j] - (double)st->r[i] / (double)st->w[i]) < 1e-6)
            st->near_threshold = 1;
        if (lhs < st->r[i]) return j;
        float mn[SO_MAX_K];
        for (int q = 0; q < K; ++q) mn[q] = st->r[q] < st->w[q] ? st->r[q] : st->w[q];
        float M = support_sum(mn, K);
        float Z = 1.0f - M;
        if (!(Z > 1e-30f)) Z = 1e-30f;
        for (int q = 0; q < K; ++q) {
            float d = st->r[q] - st->w[q];
            if (!(d > 0.0f)) d = 0.0f;
            st->r[q] = d / Z;
        }
        st->rho = st->rho / Z;
        if (onehot) continue;
        st->w[i] = 0.0f;
        float zw2 = support_sum(st->w, K);
        for (int q = 0; q < K; ++q) st->w[q] = zw2 > 0.0f ? st->w[q] / zw2 : 0.0f;
    }
    return -1;
}

/* Dense residual after so_verify_node (or the target itself when st == NULL). */
void so_residual_dense(const float *p, int V, int K, const int32_t *ids, const so_node_state *st,
                       float *r_out)
{
    for (int v = 0; v < V; ++v) r_out[v] = st ? p[v] * st->rho : p[v];
    if (st) for (int i = 0; i < K; ++i) r_out[ids[i]] = st->r[i];
}

/* One token from the residual of a node (Sec. 3.2: on rejection, resample from the normalised
 * positive part of target minus proposal), by inverting its cumulative mass in integers.
 * Unit of mass: 2^-F / s * rho.  In it a token outside the support weighs F(v), the integer term
 * it contributes to S (its residual is p(v) rho = e_v / s * rho); support token i weighs
 * G_i = floor(r_i * (S / rho)), evaluated in binary64 (S and rho converted first, one division,
 * one multiplication).  The entries are laid out as: the support tokens in stored order, then all
 * tokens by id with the support left out.  With T the total mass and u uniform on [0, 2^64), the
 * draw is the entry that covers position floor(u T / 2^64).  st == NULL (no proposal at the node),
 * T == 0 (the residual vanished) or a state with sum_i r_i > 2 or rho not finite: the draw is from
 * the target, i.e. all tokens by id with F.
 * Nothing depends on summation order. */
int32_t so_residual_draw(const uint64_t *F, int V, uint64_t S, int K, const int32_t *ids,
                         const so_node_state *st, uint64_t u)
{
    uint64_t G[SO_MAX_K];
    uint64_t total = 0;
    int use_support = st != NULL;
    /* a state that is no distribution any more (the normalising mass underflowed to the clamp)
     * is not used; otherwise sum_i r_i <= 2 keeps every product below 2^63 */
    if (use_support && (!(support_sum(st->r, K) <= 2.0f) || !(st->rho < INFINITY))) use_support = 0;
    if (use_support) {
        double ratio = (double)S / (double)st->rho;
        for (int i = 0; i < K; ++i) {
            int valid = ids[i] >= 0 && ids[i] < V;
            G[i] = valid ? (uint64_t)floor((double)st->r[i] * ratio) : 0;
            total += G[i];
        }
        for (int v = 0; v < V; ++v) {
            int in_support = 0;
            for (int i = 0; i < K; ++i) if (ids[i] == v) in_support = 1;
            if (!in_support) total += F[v];
        }
        if (total == 0) use_support = 0;
    }
    if (!use_support) {
        total = 0;
        for (int v = 0; v < V; ++v) total += F[v];
    }
    uint64_t t = (uint64_t)(((unsigned __int128)u * (unsigned __int128)total) >> 64);
    if (use_support)
        for (int i = 0; i < K; ++i) {
            if (t < G[i]) return ids[i];
            t -= G[i];
        }
    for (int v = 0; v < V; ++v) {
        if (use_support) {
            int in_support = 0;
            for (int i = 0; i < K; ++i) if (ids[i] == v) in_support = 1;
            if (in_support) continue;
        }
        if (t < F[v]) return v;
        t -= F[v];
    }
    return -1; /* not reached: t < total */
}

/* ==========================================================================================
 * Stateful part: table keyed by token tuples, contexts, pending draft.
 * ======================================================================================== */
typedef struct {
    int32_t vocab;
    int32_t max_batch;
    int32_t order_min, order_max;
    int32_t topk;
    int32_t tree_nodes;
    const int32_t *tree_parent;
    float temperature;
    uint64_t table_capacity;
    int32_t max_probe;
    uint64_t seed;
    int32_t logits_dtype;
    int32_t update_mode;
    int32_t draft_mode;
    int32_t merge_policy;
} so_config;

typedef struct {
    int32_t n;
    int32_t tok[SO_MAX_ORDER];
    uint64_t fp;
    uint32_t count;
    int32_t ids[SO_MAX_K];
    float mu[SO_MAX_K];
    int64_t next; /* chain in the tuple hash */
} so_entry;

typedef struct {
    uint64_t hits[SO_MAX_ORDER + 1];
    uint64_t misses;
    uint64_t inserts, merges, drops;
    uint64_t near_threshold;
    uint64_t tokens_emitted;
    uint64_t fp_collisions;
    uint64_t accept_tests;
} so_stats;

typedef struct so_handle {
    so_config cfg;
    int32_t N, D, K, B, V;
    int32_t *parent, *depth, *nchild, *first_child;
    /* table */
    so_entry *ent;
    int64_t n_ent, cap_ent;
    int64_t *bucket;
    int64_t n_bucket;
    uint64_t *slot_fp; /* model of a fixed-capacity linear-probing table: which slot holds which fingerprint */
    /* per trajectory */
    int32_t **ctx;
    int64_t *ctx_len, *ctx_cap;
    /* pending draft */
    int32_t *draft_tok;   /* [B][N] */
    int32_t *draft_has;   /* [B][N] node has an entry */
    int32_t *draft_qid;   /* [B][N][K] */
    float *draft_qmu;     /* [B][N][K] */
    uint64_t *node_count; /* [N] how often each tree node lay on an accepted path (Sec. 4.3) */
    const uint8_t *ext_drop; /* during so_update_drops: which records of this update are dropped (see there) */
    so_stats st;
} so_handle;

so_handle *so_create(const so_config *cfg)
{
    so_handle *h = (so_handle *)calloc(1, sizeof(so_handle));
    h->cfg = *cfg;
    h->N = cfg->tree_nodes; h->K = cfg->topk; h->B = cfg->max_batch; h->V = cfg->vocab;
    int N = h->N;
    h->parent = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    h->depth = (int32_t *)calloc((size_t)N, sizeof(int32_t));
    h->nchild = (int32_t *)calloc((size_t)N, sizeof(int32_t));
    h->first_child = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    memcpy(h->parent, cfg->tree_parent, sizeof(int32_t) * (size_t)N);
    h->cfg.tree_parent = h->parent;
    h->D = 0;
    for (int u = 0; u < N; ++u) h->first_child[u] = -1;
    for (int u = 1; u < N; ++u) {
        int par = h->parent[u];
        h->depth[u] = h->depth[par] + 1;
        if (h->depth[u] > h->D) h->D = h->depth[u];
        if (h->nchild[par] == 0) h->first_child[par] = u;
        h->nchild[par]++;
    }
    h->n_bucket = 1 << 16;
    h->bucket = (int64_t *)malloc(sizeof(int64_t) * (size_t)h->n_bucket);
    for (int64_t i = 0; i < h->n_bucket; ++i) h->bucket[i] = -1;
    h->cap_ent = 1024;
    h->ent = (so_entry *)malloc(sizeof(so_entry) * (size_t)h->cap_ent);
    h->slot_fp = (uint64_t *)calloc((size_t)cfg->table_capacity, sizeof(uint64_t));
    int B = h->B;
    h->ctx = (int32_t **)calloc((size_t)B, sizeof(int32_t *));
    h->ctx_len = (int64_t *)calloc((size_t)B, sizeof(int64_t));
    h->ctx_cap = (int64_t *)calloc((size_t)B, sizeof(int64_t));
    h->draft_tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * N);
    h->draft_has = (int32_t *)calloc((size_t)B * N, sizeof(int32_t));
    h->draft_qid = (int32_t *)calloc((size_t)B * N * h->K, sizeof(int32_t));
    h->draft_qmu = (float *)calloc((size_t)B * N * h->K, sizeof(float));
    for (int64_t i = 0; i < (int64_t)B * N; ++i) h->draft_tok[i] = -1;
    h->node_count = (uint64_t *)calloc((size_t)N, sizeof(uint64_t));
    return h;
}

void so_destroy(so_handle *h)
{
    if (!h) return;
    for (int b = 0; b < h->B; ++b) free(h->ctx[b]);
    free(h->ctx); free(h->ctx_len); free(h->ctx_cap);
    free(h->parent); free(h->depth); free(h->nchild); free(h->first_child);
    free(h->ent); free(h->bucket); free(h->slot_fp);
    free(h->draft_tok); free(h->draft_has); free(h->draft_qid); free(h->draft_qmu);
    free(h->node_count);
    free(h);
}

int32_t so_depth(const so_handle *h) { return h->D; }

static void ctx_push(so_handle *h, int b, int32_t t)
{
    if (h->ctx_len[b] == h->ctx_cap[b]) {
        h->ctx_cap[b] = h->ctx_cap[b] ? 2 * h->ctx_cap[b] : 256;
        h->ctx[b] = (int32_t *)realloc(h->ctx[b], sizeof(int32_t) * (size_t)h->ctx_cap[b]);
    }
    h->ctx[b][h->ctx_len[b]++] = t;
}

/* Prompt / prefix of trajectory b: replaces its context; nothing is merged, since no
 * distribution exists for prompt positions. */
void so_set_context(so_handle *h, int b, const int32_t *tokens, int n)
{
    h->ctx_len[b] = 0;
    for (int i = 0; i < n; ++i) ctx_push(h, b, tokens[i]);
    for (int u = 0; u < h->N; ++u) { h->draft_tok[(int64_t)b * h->N + u] = -1; h->draft_has[(int64_t)b * h->N + u] = 0; }
}

/* Beam copy: trajectory b continues from the context of src_of[b]; pending drafts are dropped. */
void so_reorder(so_handle *h, const int32_t *src_of)
{
    int B = h->B;
    int32_t **nc = (int32_t **)calloc((size_t)B, sizeof(int32_t *));
    int64_t *nl = (int64_t *)calloc((size_t)B, sizeof(int64_t));
    for (int b = 0; b < B; ++b) {
        int s = src_of[b];
        nl[b] = h->ctx_len[s];
        nc[b] = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nl[b] ? nl[b] : 1));
        memcpy(nc[b], h->ctx[s], sizeof(int32_t) * (size_t)nl[b]);
    }
    for (int b = 0; b < B; ++b) {
        free(h->ctx[b]);
        h->ctx[b] = nc[b]; h->ctx_len[b] = nl[b]; h->ctx_cap[b] = nl[b] ? nl[b] : 1;
        for (int u = 0; u < h->N; ++u) { h->draft_tok[(int64_t)b * h->N + u] = -1; h->draft_has[(int64_t)b * h->N + u] = 0; }
    }
    free(nc); free(nl);
}

int64_t so_context_len(const so_handle *h, int b) { return h->ctx_len[b]; }
void so_context_tail(const so_handle *h, int b, int n, int32_t *out)
{
    for (int i = 0; i < n; ++i) out[i] = h->ctx[b][h->ctx_len[b] - n + i];
}

static uint64_t tuple_bucket(const so_handle *h, int n, const int32_t *tok)
{
    uint64_t x = 1469598103934665603ULL ^ (uint64_t)n;
    for (int i = 0; i < n; ++i) { x ^= (uint64_t)(uint32_t)tok[i]; x *= 1099511628211ULL; }
    return x % (uint64_t)h->n_bucket;
}

static int64_t table_find(const so_handle *h, int n, const int32_t *tok)
{
    for (int64_t e = h->bucket[tuple_bucket(h, n, tok)]; e >= 0; e = h->ent[e].next)
        if (h->ent[e].n == n && memcmp(h->ent[e].tok, tok, sizeof(int32_t) * (size_t)n) == 0) return e;
    return -1;
}

/* Fixed-capacity model: a key lives at the first slot, scanning at most max_probe slots from
 * fingerprint & (capacity-1), that is empty or already holds its fingerprint.  No such slot:
 * the update is dropped and counted.  Returns 1 if the fingerprint got a new slot, 2 if a
 * slot already held it, 0 if there is no slot. */
static int slot_claim(so_handle *h, uint64_t fp)
{
    uint64_t mask = h->cfg.table_capacity - 1;
    uint64_t pos = fp & mask;
    for (int i = 0; i < h->cfg.max_probe; ++i) {
        uint64_t cur = h->slot_fp[(pos + (uint64_t)i) & mask];
        if (cur == fp) return 2;
        if (cur == 0) { h->slot_fp[(pos + (uint64_t)i) & mask] = fp; return 1; }
    }
    return 0;
}

static void table_merge(so_handle *h, int64_t rec, int n, const int32_t *tok, const int32_t *obs_ids, const float *obs_p)
{
    if (h->ext_drop && h->ext_drop[rec]) { h->st.drops++; return; } /* dropped by decree, see so_update_drops */
    int64_t e = table_find(h, n, tok);
    uint64_t fp = so_fingerprint(n, tok);
    if (e < 0) {
        /* with the drops given from outside the capacity model is off: every other record is applied */
        int sc = h->ext_drop ? 1 : slot_claim(h, fp);
        if (sc == 0) { h->st.drops++; return; }
        if (sc == 2) h->st.fp_collisions++; /* a different tuple with the same fingerprint */
        if (h->n_ent == h->cap_ent) {
            h->cap_ent *= 2;
            h->ent = (so_entry *)realloc(h->ent, sizeof(so_entry) * (size_t)h->cap_ent);
        }
        e = h->n_ent++;
        so_entry *en = &h->ent[e];
        memset(en, 0, sizeof(*en));
        en->n = n;
        memcpy(en->tok, tok, sizeof(int32_t) * (size_t)n);
        en->fp = fp;
        en->count = 0;
        uint64_t bk = tuple_bucket(h, n, tok);
        en->next = h->bucket[bk];
        h->bucket[bk] = e;
        h->st.inserts++;
    } else {
        h->st.merges++;
    }
    so_entry *en = &h->ent[e];
    int32_t ids2[SO_MAX_K];
    float mu2[SO_MAX_K];
    /* SO_MERGE_REPLACE: the comparison policy the paper argues against in Sec. 5.1 (a table that
     * keeps only the newest observation of a context); the occurrence count is still kept */
    so_merge(h->cfg.merge_policy == SO_MERGE_REPLACE ? 0u : en->count, en->ids, en->mu, h->K, obs_ids, obs_p, ids2, mu2);
    memcpy(en->ids, ids2, sizeof(int32_t) * (size_t)h->K);
    memcpy(en->mu, mu2, sizeof(float) * (size_t)h->K);
    en->count++;
}

/* Direct insertion of an entry, for tests that build a table by hand. */
int so_table_put(so_handle *h, int n, const int32_t *tok, uint32_t count, const int32_t *ids, const float *mu)
{
    if (table_find(h, n, tok) >= 0) return -1;
    uint64_t fp = so_fingerprint(n, tok);
    if (!slot_claim(h, fp)) return -2;
    if (h->n_ent == h->cap_ent) {
        h->cap_ent *= 2;
        h->ent = (so_entry *)realloc(h->ent, sizeof(so_entry) * (size_t)h->cap_ent);
    }
    int64_t e = h->n_ent++;
    so_entry *en = &h->ent[e];
    memset(en, 0, sizeof(*en));
    en->n = n;
    memcpy(en->tok, tok, sizeof(int32_t) * (size_t)n);
    en->fp = fp;
    en->count = count;
    memcpy(en->ids, ids, sizeof(int32_t) * (size_t)h->K);
    memcpy(en->mu, mu, sizeof(float) * (size_t)h->K);
    uint64_t bk = tuple_bucket(h, n, tok);
    en->next = h->bucket[bk];
    h->bucket[bk] = e;
    return 0;
}

/* Multi-level lookup (Sec. 4.2): longest order first, first hit wins.  ctx/len is the full
 * context of the position being predicted.  Returns the entry index or -1; *order_out = n. */
static int64_t table_lookup(so_handle *h, const int32_t *ctx, int64_t len, int *order_out)
{
    for (int n = h->cfg.order_max; n >= h->cfg.order_min; --n) {
        if (len < n) continue;
        int64_t e = table_find(h, n, ctx + (len - n));
        if (e >= 0 && h->ent[e].count > 0) { *order_out = n; return e; }
    }
    return -1;
}

int so_lookup(so_handle *h, const int32_t *ctx, int64_t len, int32_t *ids_out, float *mu_out, uint32_t *count_out)
{
    int n = 0;
    int64_t e = table_lookup(h, ctx, len, &n);
    if (e < 0) return 0;
    memcpy(ids_out, h->ent[e].ids, sizeof(int32_t) * (size_t)h->K);
    memcpy(mu_out, h->ent[e].mu, sizeof(float) * (size_t)h->K);
    if (count_out) *count_out = h->ent[e].count;
    return n;
}

/* ------------------------------------------------------------------------------------------
 * Draft (Sec. 4.2): walk the static tree breadth first.  The context of node u is the
 * committed context followed by the tokens on the path root -> u (the root is the last
 * committed token itself).  A node with children and a valid token looks its context up;
 * its children receive the Gumbel-Top-K draws in rank order.  A miss, or fewer candidates
 * than children, leaves the remaining children (and their subtrees) invalid (-1).
 * ---------------------------------------------------------------------------------------- */
void so_draft(so_handle *h, uint64_t step, int32_t *draft_tok_out /* [B][N] */)
{
    int N = h->N, K = h->K;
    int32_t *cx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(SO_MAX_ORDER + h->D + 2));
    for (int b = 0; b < h->B; ++b) {
        int32_t *tok = h->draft_tok + (int64_t)b * N;
        int32_t *has = h->draft_has + (int64_t)b * N;
        for (int u = 0; u < N; ++u) { tok[u] = -1; has[u] = 0; }
        if (h->ctx_len[b] > 0) tok[0] = h->ctx[b][h->ctx_len[b] - 1];
        for (int u = 0; u < N; ++u) {
            if (h->nchild[u] == 0 || tok[u] < 0) continue;
            /* context = last order_max committed tokens, then path tokens below the root */
            int64_t take = h->ctx_len[b] < SO_MAX_ORDER ? h->ctx_len[b] : SO_MAX_ORDER;
            int64_t len = 0;
            for (int64_t i = 0; i < take; ++i) cx[len++] = h->ctx[b][h->ctx_len[b] - take + i];
            int d = h->depth[u];
            int32_t path[64];
            int x = u;
            for (int i = d - 1; i >= 0; --i) { path[i] = tok[x]; x = h->parent[x]; }
            for (int i = 0; i < d; ++i) cx[len++] = path[i];
            /* orders need n real tokens; the committed context may be shorter than SO_MAX_ORDER */
            int order = 0;
            int64_t e = table_lookup(h, cx, len, &order);
            if (e < 0) { h->st.misses++; continue; }
            h->st.hits[order]++;
            has[u] = 1;
            int32_t *qid = h->draft_qid + ((int64_t)b * N + u) * K;
            float *qmu = h->draft_qmu + ((int64_t)b * N + u) * K;
            memcpy(qid, h->ent[e].ids, sizeof(int32_t) * (size_t)K);
            memcpy(qmu, h->ent[e].mu, sizeof(float) * (size_t)K);
            float U[SO_MAX_K];
            int32_t drawn[SO_MAX_K];
            int nd;
            if (h->cfg.draft_mode == SO_DRAFT_DETERMINISTIC) {
                nd = so_top_c(qid, qmu, K, h->nchild[u], drawn);
            } else if (h->cfg.draft_mode == SO_DRAFT_MULTINOMIAL) {
                /* the uniform of draw j is keyed by j */
                for (int j = 0; j < h->nchild[u]; ++j)
                    U[j] = so_uniform(h->cfg.seed, (uint32_t)b, step, (uint32_t)u, (uint32_t)j, SO_STREAM_DRAFT);
                nd = so_multinomial_wor(qid, qmu, K, h->nchild[u], U, drawn);
            } else {
                for (int i = 0; i < K; ++i)
                    U[i] = so_uniform(h->cfg.seed, (uint32_t)b, step, (uint32_t)u, (uint32_t)qid[i], SO_STREAM_DRAFT);
                nd = so_gumbel_topk(qid, qmu, K, h->nchild[u], U, drawn);
            }
            for (int j = 0; j < nd; ++j) tok[h->first_child[u] + j] = drawn[j];
        }
        if (draft_tok_out) memcpy(draft_tok_out + (int64_t)b * N, tok, sizeof(int32_t) * (size_t)N);
    }
    free(cx);
}

/* ------------------------------------------------------------------------------------------
 * What the target model needs to score the pending tree in one pass (Sec. 3.2: the drafted
 * tokens are verified "in parallel" by tree attention): node u may attend to node v iff v lies
 * on the path root -> u (u itself included) and both carry a drafted token; the position of
 * node u in the sequence is (number of committed tokens - 1) + depth(u), the root being the
 * last committed token.  mask_out[b][u][v] in {0, 1}; pos_out[b][u] = -1 for undrafted nodes.
 * ---------------------------------------------------------------------------------------- */
void so_tree_packing(const so_handle *h, uint8_t *mask_out /* [B][N][N] */, int64_t *pos_out /* [B][N] */)
{
    int N = h->N;
    for (int b = 0; b < h->B; ++b) {
        const int32_t *tok = h->draft_tok + (int64_t)b * N;
        for (int u = 0; u < N; ++u) {
            uint8_t *row = mask_out + ((int64_t)b * N + u) * N;
            for (int v = 0; v < N; ++v) row[v] = 0;
            pos_out[(int64_t)b * N + u] = -1;
            if (tok[u] < 0) continue;
            for (int v = u; v >= 0; v = h->parent[v]) row[v] = 1;
            pos_out[(int64_t)b * N + u] = h->ctx_len[b] - 1 + h->depth[u];
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Verify (Sec. 3.2, Sec. 4.2): from the root, test the children of the current node in rank
 * order; descend on acceptance; when no child is accepted (or there is none) draw one token
 * from the residual of that node and stop.  out_node[j] is the tree node whose logits row
 * produced out_tok[j] (the root, then each accepted node).  State is not modified.
 * ---------------------------------------------------------------------------------------- */
static const void *row_ptr(const so_handle *h, const void *logits, int b, int u)
{
    size_t es = h->cfg.logits_dtype == SO_DT_F32 ? 4 : 2;
    return (const char *)logits + ((size_t)b * (size_t)h->N + (size_t)u) * (size_t)h->V * es;
}

void so_verify(so_handle *h, uint64_t step, const void *logits,
               int32_t *out_tok /* [B][D+1] */, int32_t *out_node /* [B][D+1] */, int32_t *out_len /* [B] */)
{
    int N = h->N, K = h->K, V = h->V, W = h->D + 1;
    float *p = (float *)malloc(sizeof(float) * (size_t)V);
    uint64_t *F = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
    for (int b = 0; b < h->B; ++b) {
        const int32_t *tok = h->draft_tok + (int64_t)b * N;
        const int32_t *has = h->draft_has + (int64_t)b * N;
        int cur = 0, len = 0;
        for (;;) {
            uint64_t S;
            so_row_softmax(row_ptr(h, logits, b, cur), h->cfg.logits_dtype, V, h->cfg.temperature, p, NULL, NULL, &S);
            int nc = 0;
            if (has[cur])
                for (int j = 0; j < h->nchild[cur]; ++j) { if (tok[h->first_child[cur] + j] < 0) break; nc++; }
            const int32_t *qid = h->draft_qid + ((int64_t)b * N + cur) * K;
            const float *qmu = h->draft_qmu + ((int64_t)b * N + cur) * K;
            so_node_state st;
            int acc = -1;
            if (nc > 0) {
                float om[SO_MAX_K];
                for (int j = 0; j < nc; ++j)
                    om[j] = so_uniform(h->cfg.seed, (uint32_t)b, step, (uint32_t)(h->first_child[cur] + j), 0u, SO_STREAM_ACCEPT);
                acc = so_verify_node(p, K, qid, qmu, nc, tok + h->first_child[cur], om, &st,
                                     h->cfg.draft_mode == SO_DRAFT_DETERMINISTIC);
                h->st.accept_tests += (uint64_t)st.rounds;
                h->st.near_threshold += (uint64_t)st.near_threshold;
            }
            out_node[(int64_t)b * W + len] = cur;
            h->node_count[cur]++; /* this node is on the accepted path of this verification */
            if (acc >= 0) {
                int ch = h->first_child[cur] + acc;
                out_tok[(int64_t)b * W + len] = tok[ch];
                len++;
                cur = ch;
                continue;
            }
            so_row_masses(row_ptr(h, logits, b, cur), h->cfg.logits_dtype, V, h->cfg.temperature, F);
            out_tok[(int64_t)b * W + len] = so_residual_draw(
                F, V, S, K, qid, nc > 0 ? &st : NULL,
                so_uniform_u64(h->cfg.seed, (uint32_t)b, step, (uint32_t)cur, SO_STREAM_BONUS));
            len++;
            break;
        }
        out_len[b] = len;
        for (int j = len; j < W; ++j) { out_tok[(int64_t)b * W + j] = -1; out_node[(int64_t)b * W + j] = -1; }
        h->st.tokens_emitted += (uint64_t)len;
    }
    free(p);
    free(F);
}

/* ------------------------------------------------------------------------------------------
 * Update (Sec. 4.1): for committed token j of trajectory b, produced by the distribution of
 * row commit_row[b][j], and for every order n the context is long enough for, merge the
 * row's observation under the key (n, the n tokens before token j).  Records are applied in
 * the order b, then j, then n ascending; the tokens join the contexts afterwards.
 * ---------------------------------------------------------------------------------------- */
void so_update(so_handle *h, uint64_t step, const void *logits, const int32_t *commit_tok,
               const int32_t *commit_row, const int32_t *commit_len)
{
    (void)step;
    int K = h->K, V = h->V, W = h->D + 1;
    int NO = h->cfg.order_max - h->cfg.order_min + 1; /* records are numbered (b, position or node, order) */
    int32_t obs_id[SO_MAX_K];
    float obs_p[SO_MAX_K];
    if (h->cfg.update_mode == SO_UPDATE_ALL_NODES) {
        /* Every drafted node u: its row is the distribution of the token after the sequence
         * context ++ tokens on the path root -> u (the root is the context's last token).
         * Records in the order b, u, n ascending; the pending draft is the one just verified. */
        int N = h->N;
        int32_t path_tok[64];
        for (int b = 0; b < h->B; ++b) {
            const int32_t *tok = h->draft_tok + (int64_t)b * N;
            int64_t base_len = h->ctx_len[b];
            for (int u = 0; u < N; ++u) {
                if (tok[u] < 0) continue;
                so_row_obs(row_ptr(h, logits, b, u), h->cfg.logits_dtype, V, h->cfg.temperature, K, obs_id, obs_p, NULL, NULL);
                int d = h->depth[u];
                for (int x = u, i = d; x > 0; x = h->parent[x]) path_tok[--i] = tok[x]; /* tokens below the root */
                int32_t key[SO_MAX_ORDER];
                for (int n = h->cfg.order_min; n <= h->cfg.order_max; ++n) {
                    if (base_len + d < n) continue;
                    for (int i = 0; i < n; ++i) {
                        int64_t pos = base_len + d - n + i; /* position in context ++ path */
                        key[i] = pos < base_len ? h->ctx[b][pos] : path_tok[pos - base_len];
                    }
                    table_merge(h, ((int64_t)b * N + u) * NO + (n - h->cfg.order_min), n, key, obs_id, obs_p);
                }
            }
        }
    } else
    for (int b = 0; b < h->B; ++b) {
        int64_t base_len = h->ctx_len[b];
        for (int j = 0; j < commit_len[b]; ++j) {
            so_row_obs(row_ptr(h, logits, b, commit_row[(int64_t)b * W + j]), h->cfg.logits_dtype, V,
                       h->cfg.temperature, K, obs_id, obs_p, NULL, NULL);
            /* context before token j: committed context + commit_tok[b][0..j) */
            int32_t key[SO_MAX_ORDER];
            for (int n = h->cfg.order_min; n <= h->cfg.order_max; ++n) {
                if (base_len + j < n) continue;
                for (int i = 0; i < n; ++i) {
                    int64_t pos = base_len + j - n + i; /* position in context ++ commit */
                    key[i] = pos < base_len ? h->ctx[b][pos] : commit_tok[(int64_t)b * W + (pos - base_len)];
                }
                table_merge(h, ((int64_t)b * W + j) * NO + (n - h->cfg.order_min), n, key, obs_id, obs_p);
            }
        }
    }
    for (int b = 0; b < h->B; ++b)
        for (int j = 0; j < commit_len[b]; ++j) ctx_push(h, b, commit_tok[(int64_t)b * W + j]);
}

/* Update with the dropped records named from outside.  Which updates a full table drops depends on the order
 * in which the keys of one step claim the last free slots (a reading of this build: the paper's table is an
 * unbounded dictionary, Sec. 4.1), so a second implementation that claims in another order drops other
 * records, validly.  Here drop[r] != 0 says that record r -- numbered (b * R + position) * orders + (n -
 * order_min), R = depth + 1, or the number of tree nodes when every node's row is merged -- is dropped and
 * counted; every other record is applied whatever the capacity model says.  What is stored afterwards is
 * the recount of the applied updates, which a second implementation must reproduce. */
void so_update_drops(so_handle *h, uint64_t step, const void *logits, const int32_t *commit_tok,
                     const int32_t *commit_row, const int32_t *commit_len, const uint8_t *drop)
{
    h->ext_drop = drop;
    so_update(h, step, logits, commit_tok, commit_row, commit_len);
    h->ext_drop = NULL;
}

/* One speculation step: verify the pending tree, merge the accepted path, draft the next tree. */
void so_step(so_handle *h, uint64_t step, const void *logits, int32_t *out_tok, int32_t *out_node,
             int32_t *out_len, int32_t *next_draft_tok)
{
    so_verify(h, step, logits, out_tok, out_node, out_len);
    so_update(h, step, logits, out_tok, out_node, out_len);
    so_draft(h, step + 1, next_draft_tok);
}

/* Export: entries sorted by fingerprint; each = u64 fp, u32 count, u32 order, i32 ids[K], f32 mu[K]. */
static int ent_cmp(const void *a, const void *b)
{
    const so_entry *x = (const so_entry *)a, *y = (const so_entry *)b;
    return (x->fp > y->fp) - (x->fp < y->fp);
}

int64_t so_table_size(const so_handle *h) { return h->n_ent; }

int64_t so_table_export(const so_handle *h, void *buf, uint64_t cap_bytes)
{
    size_t es = 16 + 8 * (size_t)h->K;
    if ((uint64_t)h->n_ent * es > cap_bytes) return -1;
    so_entry *tmp = (so_entry *)malloc(sizeof(so_entry) * (size_t)(h->n_ent ? h->n_ent : 1));
    memcpy(tmp, h->ent, sizeof(so_entry) * (size_t)h->n_ent);
    qsort(tmp, (size_t)h->n_ent, sizeof(so_entry), ent_cmp);
    char *o = (char *)buf;
    for (int64_t i = 0; i < h->n_ent; ++i) {
        uint32_t order = (uint32_t)tmp[i].n;
        memcpy(o, &tmp[i].fp, 8);
        memcpy(o + 8, &tmp[i].count, 4);
        memcpy(o + 12, &order, 4);
        memcpy(o + 16, tmp[i].ids, 4 * (size_t)h->K);
        memcpy(o + 16 + 4 * (size_t)h->K, tmp[i].mu, 4 * (size_t)h->K);
        o += es;
    }
    free(tmp);
    return h->n_ent;
}

void so_get_stats(const so_handle *h, so_stats *out) { *out = h->st; }

/* Per-node acceptance counters for the data-driven tree (Sec. 4.3: "track which nodes are
 * frequently part of successful speculation paths"): counts[u] = number of verifications in
 * which node u lay on the accepted path (the root lies on every path). */
void so_get_node_counts(const so_handle *h, uint64_t *out) { memcpy(out, h->node_count, sizeof(uint64_t) * (size_t)h->N); }
void so_reset_node_counts(so_handle *h) { memset(h->node_count, 0, sizeof(uint64_t) * (size_t)h->N); }

/* ==========================================================================================
 * Monte-Carlo drivers used by the statistical pins (they run the functions above in a loop).
 * ======================================================================================== */

/* the children of node 0 of trial t, drawn the way so_draft draws them */
static int mc_draft(const int32_t *ids, const float *mu, int K, int c, uint64_t seed, uint64_t t, int mode,
                    int32_t *drawn)
{
    float U[SO_MAX_K];
    if (mode == SO_DRAFT_DETERMINISTIC) return so_top_c(ids, mu, K, c, drawn);
    if (mode == SO_DRAFT_MULTINOMIAL) {
        for (int j = 0; j < c; ++j) U[j] = so_uniform(seed, 0, t, 0, (uint32_t)j, SO_STREAM_DRAFT);
        return so_multinomial_wor(ids, mu, K, c, U, drawn);
    }
    for (int i = 0; i < K; ++i) U[i] = so_uniform(seed, 0, t, 0, (uint32_t)ids[i], SO_STREAM_DRAFT);
    return so_gumbel_topk(ids, mu, K, c, U, drawn);
}

/* counts[t0 * K^(c-1) + ...]: frequency of each ordered c-tuple of entry positions. */
void so_mc_draft(const int32_t *ids, const float *mu, int K, int c, uint64_t trials,
                 uint64_t seed, int mode, uint64_t *counts)
{
    int32_t drawn[SO_MAX_K];
    for (uint64_t t = 0; t < trials; ++t) {
        int nd = mc_draft(ids, mu, K, c, seed, t, mode, drawn);
        uint64_t code = 0;
        for (int j = 0; j < nd; ++j) {
            int pos = 0;
            for (int i = 0; i < K; ++i) if (ids[i] == drawn[j]) pos = i;
            code = code * (uint64_t)K + (uint64_t)pos;
        }
        if (nd == c) counts[code]++;
    }
}

/* One node, fan-out c: draft c children from (ids, mu), verify against dense p, resample on
 * total rejection.  counts[v] = how often token v was emitted; *accepted = trials in which
 * some child was accepted; resid_err = max over trials of |sum(residual) - 1|. */
void so_mc_node(const float *p, int V, int K, const int32_t *ids, const float *mu, int c,
                uint64_t trials, uint64_t seed, int mode, uint64_t *counts, uint64_t *accepted,
                uint64_t *near, double *resid_err, double *resid_min)
{
    float om[SO_MAX_K];
    int32_t drawn[SO_MAX_K];
    float *r = (float *)malloc(sizeof(float) * (size_t)V);
    /* masses of the given dense p on the grid the row masses live on: F(v) = floor(p(v) 2^40) */
    uint64_t *F = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
    uint64_t S = 0;
    for (int v = 0; v < V; ++v) { F[v] = (uint64_t)floor(ldexp((double)p[v], 40)); S += F[v]; }
    *accepted = 0; *near = 0; *resid_err = 0.0; *resid_min = 0.0;
    for (uint64_t t = 0; t < trials; ++t) {
        int nd = mc_draft(ids, mu, K, c, seed, t, mode, drawn);
        for (int j = 0; j < nd; ++j) om[j] = so_uniform(seed, 0, t, (uint32_t)(1 + j), 0, SO_STREAM_ACCEPT);
        so_node_state st;
        int acc = nd > 0 ? so_verify_node(p, K, ids, mu, nd, drawn, om, &st, mode == SO_DRAFT_DETERMINISTIC) : -1;
        if (nd > 0) *near += (uint64_t)st.near_threshold;
        if (acc >= 0) { counts[drawn[acc]]++; (*accepted)++; continue; }
        so_residual_dense(p, V, K, ids, nd > 0 ? &st : NULL, r);
        double sum = 0.0;
        for (int v = 0; v < V; ++v) { sum += (double)r[v]; if ((double)r[v] < *resid_min) *resid_min = (double)r[v]; }
        if (fabs(sum - 1.0) > *resid_err) *resid_err = fabs(sum - 1.0);
        counts[so_residual_draw(F, V, S, K, ids, nd > 0 ? &st : NULL, so_uniform_u64(seed, 0, t, 0, SO_STREAM_BONUS))]++;
    }
    free(r);
    free(F);
}

/* Frequencies of so_residual_draw: masses F, optional support (ids, r, rho) when K > 0. */
void so_mc_draw(const uint64_t *F, int V, uint64_t S, int K, const int32_t *ids, const float *r, float rho,
                uint64_t trials, uint64_t seed, uint64_t *counts)
{
    so_node_state st;
    memset(&st, 0, sizeof st);
    for (int i = 0; i < K; ++i) st.r[i] = r[i];
    st.rho = rho;
    for (uint64_t t = 0; t < trials; ++t)
        counts[so_residual_draw(F, V, S, K, ids, K > 0 ? &st : NULL, so_uniform_u64(seed, 0, t, 0, SO_STREAM_BONUS))]++;
}
