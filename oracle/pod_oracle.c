/*
 * CPU oracle for PoD attention over a split KV cache.  TEST INFRASTRUCTURE ONLY:
 * tests, the smoke check and the bench's cpu_baseline leg call it; the product
 * (the HIP library) never does, and the two share no code.
 *
 * It is written to be read against the paper, not to be fast: double precision
 * arithmetic on bf16 inputs (passed as raw 16-bit patterns), one scalar loop per
 * (query row, head), no blocking, no fusion.  OpenMP only spreads independent
 * (row, head) pairs over cores.
 *
 * What is what (paper: arXiv 2412.02252):
 *   - proximal / distant split and which query and key produce a logit:
 *     Methodology, "Attention Sharing within Each Block", Eq. 3;
 *   - joint softmax over both regions: appendix "Derivation of Integrating
 *     Attention to Proximal and Distant Tokens" (first line of its equation);
 *   - the gate form (two softmaxes + gate g): Eq. 3 and Eq. 4;
 *   - cache regions and their update: derived from Eq. 3's index ranges (the
 *     paper's cache-update drawing, Fig. 2 right, is not available);
 *   - memory accounting: keys of distant tokens stored once per block of layers
 *     (abstract; Eq. 3 line 3), values per layer (Eq. 3 line 4).
 *
 * Readings taken where the paper is silent (0-based positions here):
 *   - Eq. 3 writes the recent window with the sequence length n; for a query at
 *     position i attending j <= i the window is [i-W+1, i] (n replaced by i+1);
 *   - sink and window may overlap for short contexts: a token is proximal if it
 *     is in either, counted once;
 *   - GQA: query head h reads KV head h / (Hq/Hkv), for own and shared keys alike.
 *
 * Parity pins live in tests/ (reduction to textbook attention, closed forms,
 * gate == joint, brute force on tiny inputs, memory formula).  Absolute attention
 * values have no worked example in the paper: "parity unpinned" beyond those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_CAPACITY (-2)
#define ORACLE_ERR_STATE (-3)

static inline double bf16_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double dot_bf16(const uint16_t *a, const uint16_t *b, int d)
{
    double s = 0.0;
    for (int x = 0; x < d; ++x)
        s += bf16_to_double(a[x]) * bf16_to_double(b[x]);
    return s;
}

/* Is key position j proximal for the query at position i?  (Eq. 3: sink tokens
 * [0,S) and the W most recent tokens ending at i.) */
static int is_proximal(long j, long i, int S, int W)
{
    return (j < S) || (j > i - W);
}

/* ------------------------------------------------------------------------- */
/* Attention by definition on full tensors (joint-softmax form).             */
/* ------------------------------------------------------------------------- */

/*
 * q, q_shared : [nrows][Hq][d]   query rows of this layer / of the block's lowest layer
 * k, v        : [n][Hkv][d]      this layer's keys and values for positions 0..n-1
 * k_shared    : [n][Hkv][d]      the lowest layer's keys
 * rows        : [nrows]          position i of each query row (0 <= i < n)
 * out         : [nrows][Hq][d]   double
 * q_shared == NULL or k_shared == NULL means "this layer is the lowest of its
 * block": its own q and k serve the distant tokens too.
 */
int oracle_pod_attention(long n, int Hq, int Hkv, int d, int S, int W, double scale,
                         const uint16_t *q, const uint16_t *k, const uint16_t *v,
                         const uint16_t *q_shared, const uint16_t *k_shared,
                         const long *rows, long nrows, double *out)
{
    if (n < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || S < 0 || W < 1) return ORACLE_ERR_ARG;
    for (long r = 0; r < nrows; ++r)
        if (rows[r] < 0 || rows[r] >= n) return ORACLE_ERR_ARG;
    if (!q_shared || !k_shared) { q_shared = q; k_shared = k; }
    const int rep = Hq / Hkv;
    const long work = nrows * Hq;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long w = 0; w < work; ++w) {
        const long r = w / Hq;
        const int h = (int)(w % Hq);
        const int kv = h / rep;
        const long i = rows[r];
        double *a = (double *)malloc((size_t)(i + 1) * sizeof(double));
        if (!a) { bad = 1; continue; }
        const uint16_t *qi = q + ((size_t)r * Hq + h) * d;
        const uint16_t *qsi = q_shared + ((size_t)r * Hq + h) * d;
        double amax = -INFINITY;
        for (long j = 0; j <= i; ++j) {
            const size_t off = ((size_t)j * Hkv + kv) * d;
            if (is_proximal(j, i, S, W))
                a[j] = scale * dot_bf16(qi, k + off, d);         /* Eq. 3, line 1 */
            else
                a[j] = scale * dot_bf16(qsi, k_shared + off, d); /* Eq. 3, line 3 */
            if (a[j] > amax) amax = a[j];
        }
        double denom = 0.0;
        for (long j = 0; j <= i; ++j) { a[j] = exp(a[j] - amax); denom += a[j]; }
        double *o = out + ((size_t)r * Hq + h) * d;
        for (int x = 0; x < d; ++x) o[x] = 0.0;
        for (long j = 0; j <= i; ++j) {
            const double p = a[j] / denom;
            const uint16_t *vj = v + ((size_t)j * Hkv + kv) * d;  /* values: always this layer */
            for (int x = 0; x < d; ++x) o[x] += p * bf16_to_double(vj[x]);
        }
        free(a);
    }
    return bad ? ORACLE_ERR_CAPACITY : ORACLE_OK;
}

/*
 * The same result through the paper's gate form: separate softmax-weighted
 * outputs o^P and o^D (Eq. 3) mixed by g (Eq. 4).  gate_out[nrows][Hq] receives
 * g (1 when there are no distant tokens: that term is omitted).
 */
int oracle_pod_attention_gate(long n, int Hq, int Hkv, int d, int S, int W, double scale,
                              const uint16_t *q, const uint16_t *k, const uint16_t *v,
                              const uint16_t *q_shared, const uint16_t *k_shared,
                              const long *rows, long nrows, double *out, double *gate_out)
{
    if (n < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || S < 0 || W < 1) return ORACLE_ERR_ARG;
    for (long r = 0; r < nrows; ++r)
        if (rows[r] < 0 || rows[r] >= n) return ORACLE_ERR_ARG;
    if (!q_shared || !k_shared) { q_shared = q; k_shared = k; }
    const int rep = Hq / Hkv;
    for (long r = 0; r < nrows; ++r) {
        const long i = rows[r];
        for (int h = 0; h < Hq; ++h) {
            const int kv = h / rep;
            const uint16_t *qi = q + ((size_t)r * Hq + h) * d;
            const uint16_t *qsi = q_shared + ((size_t)r * Hq + h) * d;
            double *oP = (double *)calloc((size_t)d, sizeof(double));
            double *oD = (double *)calloc((size_t)d, sizeof(double));
            /* a^P and a^D, each with its own reference point for exp() */
            double maxP = -INFINITY, maxD = -INFINITY;
            long nD = 0;
            for (long j = 0; j <= i; ++j) {
                const size_t off = ((size_t)j * Hkv + kv) * d;
                if (is_proximal(j, i, S, W)) {
                    double a = scale * dot_bf16(qi, k + off, d);
                    if (a > maxP) maxP = a;
                } else {
                    double a = scale * dot_bf16(qsi, k_shared + off, d);
                    if (a > maxD) maxD = a;
                    ++nD;
                }
            }
            double sumP = 0.0, sumD = 0.0;
            for (long j = 0; j <= i; ++j) {
                const size_t off = ((size_t)j * Hkv + kv) * d;
                const uint16_t *vj = v + off;
                if (is_proximal(j, i, S, W)) {
                    double e = exp(scale * dot_bf16(qi, k + off, d) - maxP);
                    sumP += e;
                    for (int x = 0; x < d; ++x) oP[x] += e * bf16_to_double(vj[x]);
                } else {
                    double e = exp(scale * dot_bf16(qsi, k_shared + off, d) - maxD);
                    sumD += e;
                    for (int x = 0; x < d; ++x) oD[x] += e * bf16_to_double(vj[x]);
                }
            }
            for (int x = 0; x < d; ++x) oP[x] /= sumP;           /* Eq. 3, line 2 */
            double g = 1.0;
            if (nD > 0) {
                for (int x = 0; x < d; ++x) oD[x] /= sumD;       /* Eq. 3, line 4 */
                /* Eq. 4: g = sum exp(a^P) / (sum exp(a^P) + sum exp(a^D)) */
                g = 1.0 / (1.0 + (sumD / sumP) * exp(maxD - maxP));
            }
            double *o = out + ((size_t)r * Hq + h) * d;
            for (int x = 0; x < d; ++x) o[x] = g * oP[x] + (1.0 - g) * oD[x];
            if (gate_out) gate_out[(size_t)r * Hq + h] = g;
            free(oP);
            free(oD);
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Logical model of the split cache.                                         */
/* ------------------------------------------------------------------------- */

/*
 * Per (layer, sequence) the model keeps four plain lists, token-major
 * [tokens][Hkv][d], in position order:
 *   sink   : K,V of positions [0, S)
 *   recent : K,V of the last min(W, n-S) positions >= S, oldest first
 *   distV  : V of positions [S, n-W)  (every layer)
 *   distK  : K of the same positions, kept only at the lowest layer of a block
 * A position leaving the recent list moves to the distant lists: its value
 * always, its key only if the layer is the lowest of its block.
 *
 * Blocks are per kv head (the paper groups layers head by head, Alg. 1): lowest[l][h]
 * is the lowest layer of the block that layer l belongs to for kv head h.  The
 * uniform case (blocks of G consecutive layers for every head) is lowest = l - l % G.
 * distK of a layer holds the slices of the heads for which it is a lowest layer;
 * the other heads' slices are never written and never read.
 */
typedef struct {
    long n;             /* tokens seen */
    long n_recent;      /* entries in the recent list */
    long n_dist;        /* entries in the distant lists */
    uint16_t *sinkK, *sinkV, *recK, *recV, *distK, *distV;
} seq_state;

typedef struct pod_oracle_cache {
    int L, Hkv, d, S, W, B;
    long max_ctx;
    int *lowest;   /* [L][Hkv] */
    seq_state *st; /* [L][B], storage allocated on first use */
} pod_oracle_cache;

static size_t row_elems(const pod_oracle_cache *c) { return (size_t)c->Hkv * c->d; }
static int lowest_of(const pod_oracle_cache *c, int layer, int h) { return c->lowest[(size_t)layer * c->Hkv + h]; }
static int is_lowest(const pod_oracle_cache *c, int layer, int h) { return lowest_of(c, layer, h) == layer; }
static int is_lowest_any(const pod_oracle_cache *c, int layer)
{
    for (int h = 0; h < c->Hkv; ++h) if (is_lowest(c, layer, h)) return 1;
    return 0;
}

/*
 * lowest: [L][Hkv] table as described above, or NULL for uniform blocks of G layers.
 * A table must describe consecutive blocks: lowest[0][h] = 0 and lowest[l][h] is either
 * lowest[l-1][h] (same block) or l (a new block starts).
 */
pod_oracle_cache *oracle_cache_create_map(int L, int G, int Hkv, int d, int S, int W, int B, long max_ctx,
                                          const int32_t *lowest)
{
    if (L < 1 || Hkv < 1 || d < 1 || S < 0 || W < 1 || B < 1 || max_ctx < 1) return NULL;
    if (!lowest && (G < 1 || L % G)) return NULL;
    pod_oracle_cache *c = (pod_oracle_cache *)calloc(1, sizeof *c);
    if (!c) return NULL;
    c->L = L; c->Hkv = Hkv; c->d = d; c->S = S; c->W = W; c->B = B; c->max_ctx = max_ctx;
    c->st = (seq_state *)calloc((size_t)L * B, sizeof(seq_state));
    c->lowest = (int *)calloc((size_t)L * Hkv, sizeof(int));
    if (!c->st || !c->lowest) { free(c->st); free(c->lowest); free(c); return NULL; }
    for (int l = 0; l < L; ++l)
        for (int h = 0; h < Hkv; ++h) {
            const int lo = lowest ? lowest[(size_t)l * Hkv + h] : l - l % G;
            const int prev = l > 0 ? c->lowest[(size_t)(l - 1) * Hkv + h] : 0;
            if ((l == 0 && lo != 0) || (l > 0 && lo != prev && lo != l)) { free(c->st); free(c->lowest); free(c); return NULL; }
            c->lowest[(size_t)l * Hkv + h] = lo;
        }
    return c;
}

pod_oracle_cache *oracle_cache_create(int L, int G, int Hkv, int d, int S, int W, int B, long max_ctx)
{
    return oracle_cache_create_map(L, G, Hkv, d, S, W, B, max_ctx, NULL);
}

static void seq_free(seq_state *s)
{
    free(s->sinkK); free(s->sinkV); free(s->recK); free(s->recV); free(s->distK); free(s->distV);
    memset(s, 0, sizeof *s);
}

void oracle_cache_destroy(pod_oracle_cache *c)
{
    if (!c) return;
    for (long x = 0; x < (long)c->L * c->B; ++x) seq_free(&c->st[x]);
    free(c->st);
    free(c->lowest);
    free(c);
}

/* Forget one sequence slot (seq >= 0) or all of them (seq < 0), at every layer. */
int oracle_cache_reset(pod_oracle_cache *c, int seq)
{
    if (!c || seq >= c->B) return ORACLE_ERR_ARG;
    for (int l = 0; l < c->L; ++l)
        for (int b = 0; b < c->B; ++b)
            if (seq < 0 || b == seq) seq_free(&c->st[(size_t)l * c->B + b]);
    return ORACLE_OK;
}

static int seq_alloc(const pod_oracle_cache *c, seq_state *s, int lowest)
{
    if (s->sinkV) return ORACLE_OK;
    const size_t re = row_elems(c) * sizeof(uint16_t);
    long cap_dist = c->max_ctx - c->S - c->W;
    if (cap_dist < 0) cap_dist = 0;
    s->sinkK = (uint16_t *)malloc(re * (size_t)(c->S + 1));
    s->sinkV = (uint16_t *)malloc(re * (size_t)(c->S + 1));
    s->recK = (uint16_t *)malloc(re * (size_t)c->W);
    s->recV = (uint16_t *)malloc(re * (size_t)c->W);
    s->distV = (uint16_t *)malloc(re * (size_t)(cap_dist + 1));
    s->distK = lowest ? (uint16_t *)calloc((size_t)(cap_dist + 1), re) : NULL; /* slices of non-lowest heads stay zero */
    if (!s->sinkK || !s->sinkV || !s->recK || !s->recV || !s->distV || (lowest && !s->distK))
        return ORACLE_ERR_CAPACITY;
    return ORACLE_OK;
}

static seq_state *seq_of(pod_oracle_cache *c, int layer, int seq)
{
    return &c->st[(size_t)layer * c->B + seq];
}

long oracle_cache_len(pod_oracle_cache *c, int layer, int seq)
{
    if (!c || layer < 0 || layer >= c->L || seq < 0 || seq >= c->B) return ORACLE_ERR_ARG;
    return seq_of(c, layer, seq)->n;
}

/* rows of distant keys: only the slices of the heads for which `layer` is a lowest layer */
static void copy_lowest_heads(const pod_oracle_cache *c, int layer, uint16_t *dst, const uint16_t *src, long rows)
{
    const size_t re = row_elems(c);
    for (long r = 0; r < rows; ++r)
        for (int h = 0; h < c->Hkv; ++h)
            if (is_lowest(c, layer, h))
                memcpy(dst + (size_t)r * re + (size_t)h * c->d, src + (size_t)r * re + (size_t)h * c->d, (size_t)c->d * sizeof(uint16_t));
}

/* One token (position p = number of tokens already stored) enters the cache. */
static int seq_push(pod_oracle_cache *c, int layer, seq_state *s, const uint16_t *krow, const uint16_t *vrow)
{
    const size_t re = row_elems(c), rb = re * sizeof(uint16_t);
    int rc = seq_alloc(c, s, is_lowest_any(c, layer));
    if (rc) return rc;
    if (s->n >= c->max_ctx) return ORACLE_ERR_CAPACITY;
    const long p = s->n;
    if (p < c->S) {
        memcpy(s->sinkK + (size_t)p * re, krow, rb);
        memcpy(s->sinkV + (size_t)p * re, vrow, rb);
    } else {
        if (s->n_recent == c->W) {
            /* the oldest recent token stops being proximal: demote it */
            memcpy(s->distV + (size_t)s->n_dist * re, s->recV, rb);
            if (is_lowest_any(c, layer))
                copy_lowest_heads(c, layer, s->distK + (size_t)s->n_dist * re, s->recK, 1);
            s->n_dist += 1;
            memmove(s->recK, s->recK + re, rb * (size_t)(c->W - 1));
            memmove(s->recV, s->recV + re, rb * (size_t)(c->W - 1));
            s->n_recent -= 1;
        }
        memcpy(s->recK + (size_t)s->n_recent * re, krow, rb);
        memcpy(s->recV + (size_t)s->n_recent * re, vrow, rb);
        s->n_recent += 1;
    }
    s->n = p + 1;
    return ORACLE_OK;
}

/*
 * Decode-time update: sequence b (0 <= b < Bcur) receives one token at
 * positions[b], which must be its current length.  k_new, v_new: [Bcur][Hkv][d].
 */
int oracle_cache_append(pod_oracle_cache *c, int layer, const uint16_t *k_new, const uint16_t *v_new,
                        const int32_t *positions, int Bcur)
{
    if (!c || layer < 0 || layer >= c->L || Bcur < 1 || Bcur > c->B) return ORACLE_ERR_ARG;
    const size_t re = row_elems(c);
    for (int b = 0; b < Bcur; ++b) {
        seq_state *s = seq_of(c, layer, b);
        if (positions[b] != s->n) return ORACLE_ERR_STATE;
        if (s->n >= c->max_ctx) return ORACLE_ERR_CAPACITY;
    }
    for (int b = 0; b < Bcur; ++b) {
        int rc = seq_push(c, layer, seq_of(c, layer, b), k_new + (size_t)b * re, v_new + (size_t)b * re);
        if (rc) return rc;
    }
    return ORACLE_OK;
}

/*
 * Several tokens per sequence in one call (a chunk of a prompt, or tokens accepted
 * together).  By definition the same as appending them one at a time in position
 * order.  k_new, v_new: [Bcur][T][Hkv][d]; sequence b takes its first counts[b]
 * rows (counts == NULL: all T), the first of them at positions[b], which must be
 * its current length.  Nothing is stored if any sequence fails the checks.
 */
int oracle_cache_append_many(pod_oracle_cache *c, int layer, const uint16_t *k_new, const uint16_t *v_new,
                             const int32_t *positions, const int32_t *counts, int T, int Bcur)
{
    if (!c || layer < 0 || layer >= c->L || Bcur < 1 || Bcur > c->B || T < 1) return ORACLE_ERR_ARG;
    const size_t re = row_elems(c);
    for (int b = 0; b < Bcur; ++b) {
        seq_state *s = seq_of(c, layer, b);
        const int cnt = counts ? counts[b] : T;
        if (cnt < 0 || cnt > T) return ORACLE_ERR_ARG;
        if (cnt > 0 && positions[b] != s->n) return ORACLE_ERR_STATE;
        if (s->n + cnt > c->max_ctx) return ORACLE_ERR_CAPACITY;
    }
    for (int b = 0; b < Bcur; ++b) {
        const int cnt = counts ? counts[b] : T;
        for (int t = 0; t < cnt; ++t) {
            const size_t row = ((size_t)b * T + t) * re;
            int rc = seq_push(c, layer, seq_of(c, layer, b), k_new + row, v_new + row);
            if (rc) return rc;
        }
    }
    return ORACLE_OK;
}

/*
 * Prompt-time construction, stated directly as slices of the prompt's K/V
 * [n][Hkv][d] (not as n appends; the tests check that the two agree):
 *   sink = [0, min(n,S)),  recent = [max(S, n-W), n),  distant = [S, n-W).
 */
int oracle_cache_fill(pod_oracle_cache *c, int layer, int seq, long n, const uint16_t *k, const uint16_t *v)
{
    if (!c || layer < 0 || layer >= c->L || seq < 0 || seq >= c->B || n < 1) return ORACLE_ERR_ARG;
    if (n > c->max_ctx) return ORACLE_ERR_CAPACITY;
    seq_state *s = seq_of(c, layer, seq);
    if (s->n != 0) return ORACLE_ERR_STATE;
    int rc = seq_alloc(c, s, is_lowest_any(c, layer));
    if (rc) return rc;
    const size_t re = row_elems(c), rb = re * sizeof(uint16_t);
    const long n_sink = n < c->S ? n : c->S;
    const long rec_lo = (n - c->W > c->S) ? n - c->W : c->S;
    const long n_rec = n > rec_lo ? n - rec_lo : 0;
    const long n_dist = (n - c->W > c->S) ? n - c->W - c->S : 0;
    memcpy(s->sinkK, k, rb * (size_t)n_sink);
    memcpy(s->sinkV, v, rb * (size_t)n_sink);
    memcpy(s->recK, k + (size_t)rec_lo * re, rb * (size_t)n_rec);
    memcpy(s->recV, v + (size_t)rec_lo * re, rb * (size_t)n_rec);
    memcpy(s->distV, v + (size_t)c->S * re, rb * (size_t)n_dist);
    if (is_lowest_any(c, layer)) copy_lowest_heads(c, layer, s->distK, k + (size_t)c->S * re, n_dist);
    s->n = n; s->n_recent = n_rec; s->n_dist = n_dist;
    return ORACLE_OK;
}

/* counts[3] = {sink, recent, distant} entries.  Any output pointer may be NULL. */
int oracle_cache_export(pod_oracle_cache *c, int layer, int seq, long *counts,
                        uint16_t *sinkK, uint16_t *sinkV, uint16_t *recK, uint16_t *recV,
                        uint16_t *distK, uint16_t *distV)
{
    if (!c || layer < 0 || layer >= c->L || seq < 0 || seq >= c->B) return ORACLE_ERR_ARG;
    seq_state *s = seq_of(c, layer, seq);
    const size_t rb = row_elems(c) * sizeof(uint16_t);
    const long n_sink = s->n < c->S ? s->n : c->S;
    if (counts) { counts[0] = n_sink; counts[1] = s->n_recent; counts[2] = s->n_dist; }
    if (s->n == 0) return ORACLE_OK;
    if (sinkK) memcpy(sinkK, s->sinkK, rb * (size_t)n_sink);
    if (sinkV) memcpy(sinkV, s->sinkV, rb * (size_t)n_sink);
    if (recK) memcpy(recK, s->recK, rb * (size_t)s->n_recent);
    if (recV) memcpy(recV, s->recV, rb * (size_t)s->n_recent);
    if (distV) memcpy(distV, s->distV, rb * (size_t)s->n_dist);
    if (distK) {
        if (!is_lowest_any(c, layer)) return ORACLE_ERR_ARG; /* that layer keeps no distant keys */
        memcpy(distK, s->distK, rb * (size_t)s->n_dist);   /* heads that are not lowest here: zeros */
    }
    return ORACLE_OK;
}

/* bf16 elements the cache holds right now, counted entry by entry. */
long oracle_cache_stored_elems(pod_oracle_cache *c)
{
    long total = 0;
    for (int l = 0; l < c->L; ++l)
        for (int b = 0; b < c->B; ++b) {
            seq_state *s = seq_of(c, l, b);
            const long n_sink = s->n < c->S ? s->n : c->S;
            for (int h = 0; h < c->Hkv; ++h) {
                long rows = 2 * n_sink + 2 * s->n_recent + s->n_dist + (is_lowest(c, l, h) ? s->n_dist : 0);
                total += rows * (long)c->d;
            }
        }
    return total;
}

/*
 * Memory accounting in closed form for one sequence of n tokens, uniform blocks
 * of G layers: every layer keeps K and V of the proximal tokens and V of the
 * distant ones; distant K is kept once per block.  Dense keeps K and V of every
 * token at every layer.  Sizes in bytes for elem_bytes-wide elements.
 */
void oracle_cache_bytes_formula(int L, int G, int Hkv, int d, int S, int W, long n, int elem_bytes,
                                double *pod_bytes, double *dense_bytes)
{
    const double row = (double)Hkv * d * elem_bytes;
    const double n_prox = (double)(n < (long)S + W ? n : (long)S + W);
    const double n_dist = (double)(n - S - W > 0 ? n - S - W : 0);
    *pod_bytes = row * ((double)L * (2.0 * n_prox + n_dist) + ((double)L / G) * n_dist);
    *dense_bytes = 2.0 * row * (double)L * (double)n;
}

/* The same for head-wise blocks: kv head h keeps distant keys once per block of ITS partition. */
void oracle_cache_bytes_formula_map(int L, int Hkv, int d, int S, int W, long n, int elem_bytes,
                                    const int32_t *lowest, double *pod_bytes, double *dense_bytes)
{
    const double row = (double)d * elem_bytes; /* one head */
    const double n_prox = (double)(n < (long)S + W ? n : (long)S + W);
    const double n_dist = (double)(n - S - W > 0 ? n - S - W : 0);
    double total = 0.0;
    for (int h = 0; h < Hkv; ++h) {
        int blocks = 0;
        for (int l = 0; l < L; ++l) blocks += lowest[(size_t)l * Hkv + h] == l;
        total += row * ((double)L * (2.0 * n_prox + n_dist) + (double)blocks * n_dist);
    }
    *pod_bytes = total;
    *dense_bytes = 2.0 * row * Hkv * (double)L * (double)n;
}

/*
 * Decode attention from the cache model: one query token per sequence, at
 * position n-1 where n = ctx_lens[b] must equal the stored length.
 *   q, q_shared : [Bcur][Hq][d];  q_shared may be NULL at a block's lowest layer
 *   out         : [Bcur][Hq][d] double
 * Proximal logits use this layer's q and K (sink + recent lists); distant
 * logits use the lowest layer's q and that layer's stored distant keys; one
 * softmax over all of them; values from this layer's lists.
 */
int oracle_decode_attention(pod_oracle_cache *c, int layer, int Hq, double scale,
                            const uint16_t *q, const uint16_t *q_shared, const int32_t *ctx_lens,
                            int Bcur, double *out)
{
    if (!c || layer < 0 || layer >= c->L || Bcur < 1 || Bcur > c->B || Hq < 1 || Hq % c->Hkv) return ORACLE_ERR_ARG;
    const int rep = Hq / c->Hkv, d = c->d;
    const size_t re = row_elems(c);
    for (int b = 0; b < Bcur; ++b) {
        seq_state *s = seq_of(c, layer, b);
        if (ctx_lens[b] < 1 || ctx_lens[b] != s->n) return ORACLE_ERR_STATE;
        for (int h = 0; h < c->Hkv; ++h) {
            seq_state *sa = seq_of(c, lowest_of(c, layer, h), b);
            if (s->n_dist > 0 && sa->n_dist != s->n_dist) return ORACLE_ERR_STATE;
            if (s->n_dist > 0 && !is_lowest(c, layer, h) && !q_shared) return ORACLE_ERR_ARG;
        }
    }
    const long work = (long)Bcur * Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (long w = 0; w < work; ++w) {
        const int b = (int)(w / Hq), h = (int)(w % Hq), kv = h / rep;
        seq_state *s = seq_of(c, layer, b);
        const int lowest_layer = lowest_of(c, layer, kv);   /* of this head's block */
        seq_state *sa = seq_of(c, lowest_layer, b);
        const long n_sink = s->n < c->S ? s->n : c->S;
        const long total = n_sink + s->n_recent + s->n_dist;
        double *a = (double *)malloc((size_t)total * sizeof(double));
        const uint16_t **vp = (const uint16_t **)malloc((size_t)total * sizeof(*vp));
        const uint16_t *qi = q + ((size_t)b * Hq + h) * d;
        const uint16_t *qs = (layer == lowest_layer || !q_shared) ? qi : q_shared + ((size_t)b * Hq + h) * d;
        long m = 0;
        for (long t = 0; t < n_sink; ++t, ++m) {
            a[m] = scale * dot_bf16(qi, s->sinkK + (size_t)t * re + (size_t)kv * d, d);
            vp[m] = s->sinkV + (size_t)t * re + (size_t)kv * d;
        }
        for (long t = 0; t < s->n_recent; ++t, ++m) {
            a[m] = scale * dot_bf16(qi, s->recK + (size_t)t * re + (size_t)kv * d, d);
            vp[m] = s->recV + (size_t)t * re + (size_t)kv * d;
        }
        for (long t = 0; t < s->n_dist; ++t, ++m) {
            a[m] = scale * dot_bf16(qs, sa->distK + (size_t)t * re + (size_t)kv * d, d);
            vp[m] = s->distV + (size_t)t * re + (size_t)kv * d;
        }
        double amax = -INFINITY, denom = 0.0;
        for (long t = 0; t < total; ++t) if (a[t] > amax) amax = a[t];
        for (long t = 0; t < total; ++t) { a[t] = exp(a[t] - amax); denom += a[t]; }
        double *o = out + ((size_t)b * Hq + h) * d;
        for (int x = 0; x < d; ++x) o[x] = 0.0;
        for (long t = 0; t < total; ++t) {
            const double p = a[t] / denom;
            for (int x = 0; x < d; ++x) o[x] += p * bf16_to_double(vp[t][x]);
        }
        free(a);
        free(vp);
    }
    return ORACLE_OK;
}

/*
 * Decode attention with the gated skip of distant tokens (appendix "Computation
 * Optimization for Distant Tokens").  At a layer that is not the lowest of its
 * block the gate of Eq. 4 is evaluated first,
 *     g = sum exp(a^P) / (sum exp(a^P) + sum exp(a^D)),
 * and if g >= tau the attention over distant tokens is left out: the output is
 * o^P, the softmax over the proximal tokens alone (Eq. 3 lines 1-2).  Otherwise,
 * and always at the lowest layer or without distant tokens, the output is the
 * exact one, g o^P + (1 - g) o^D.  gate_out[Bcur][Hq] receives g (1 without
 * distant tokens), skipped_out[Bcur][Hq] 1 where the distant part was left out.
 * Same arguments and checks as oracle_decode_attention.
 */
int oracle_decode_attention_gated(pod_oracle_cache *c, int layer, int Hq, double scale,
                                  const uint16_t *q, const uint16_t *q_shared, const int32_t *ctx_lens,
                                  int Bcur, double tau, double *out, double *gate_out, int32_t *skipped_out)
{
    if (!c || layer < 0 || layer >= c->L || Bcur < 1 || Bcur > c->B || Hq < 1 || Hq % c->Hkv) return ORACLE_ERR_ARG;
    if (!(tau >= 0.0 && tau <= 1.0)) return ORACLE_ERR_ARG;
    const int rep = Hq / c->Hkv, d = c->d;
    const size_t re = row_elems(c);
    for (int b = 0; b < Bcur; ++b) {
        seq_state *s = seq_of(c, layer, b);
        if (ctx_lens[b] < 1 || ctx_lens[b] != s->n) return ORACLE_ERR_STATE;
        for (int h = 0; h < c->Hkv; ++h) {
            seq_state *sa = seq_of(c, lowest_of(c, layer, h), b);
            if (s->n_dist > 0 && sa->n_dist != s->n_dist) return ORACLE_ERR_STATE;
            if (s->n_dist > 0 && !is_lowest(c, layer, h) && !q_shared) return ORACLE_ERR_ARG;
        }
    }
    const long work = (long)Bcur * Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (long w = 0; w < work; ++w) {
        const int b = (int)(w / Hq), h = (int)(w % Hq), kv = h / rep;
        seq_state *s = seq_of(c, layer, b);
        const int lowest_layer = lowest_of(c, layer, kv);   /* of this head's block */
        seq_state *sa = seq_of(c, lowest_layer, b);
        const long n_sink = s->n < c->S ? s->n : c->S;
        const long nP = n_sink + s->n_recent, nD = s->n_dist;
        double *aP = (double *)malloc((size_t)(nP > 0 ? nP : 1) * sizeof(double));
        double *aD = (double *)malloc((size_t)(nD > 0 ? nD : 1) * sizeof(double));
        const uint16_t *qi = q + ((size_t)b * Hq + h) * d;
        const uint16_t *qs = (layer == lowest_layer || !q_shared) ? qi : q_shared + ((size_t)b * Hq + h) * d;
        double *oP = (double *)calloc((size_t)d, sizeof(double));
        double *oD = (double *)calloc((size_t)d, sizeof(double));
        /* a^P: this layer's query against its own sink and recent keys */
        double maxP = -INFINITY, maxD = -INFINITY;
        for (long t = 0; t < nP; ++t) {
            const uint16_t *krow = t < n_sink ? s->sinkK + (size_t)t * re : s->recK + (size_t)(t - n_sink) * re;
            aP[t] = scale * dot_bf16(qi, krow + (size_t)kv * d, d);
            if (aP[t] > maxP) maxP = aP[t];
        }
        /* a^D: the lowest layer's query against the block's stored distant keys */
        for (long t = 0; t < nD; ++t) {
            aD[t] = scale * dot_bf16(qs, sa->distK + (size_t)t * re + (size_t)kv * d, d);
            if (aD[t] > maxD) maxD = aD[t];
        }
        double sumP = 0.0, sumD = 0.0;
        for (long t = 0; t < nP; ++t) {
            const uint16_t *vrow = t < n_sink ? s->sinkV + (size_t)t * re : s->recV + (size_t)(t - n_sink) * re;
            const double e = exp(aP[t] - maxP);
            sumP += e;
            for (int x = 0; x < d; ++x) oP[x] += e * bf16_to_double(vrow[(size_t)kv * d + x]);
        }
        for (int x = 0; x < d; ++x) oP[x] /= sumP;
        double g = 1.0;
        if (nD > 0) {
            for (long t = 0; t < nD; ++t) sumD += exp(aD[t] - maxD);
            g = 1.0 / (1.0 + (sumD / sumP) * exp(maxD - maxP));
        }
        const int skip = nD > 0 && layer != lowest_layer && g >= tau;
        double *o = out + ((size_t)b * Hq + h) * d;
        if (nD == 0 || skip) {
            for (int x = 0; x < d; ++x) o[x] = oP[x];
        } else {
            for (long t = 0; t < nD; ++t) {
                const double e = exp(aD[t] - maxD);
                const uint16_t *vrow = s->distV + (size_t)t * re + (size_t)kv * d;
                for (int x = 0; x < d; ++x) oD[x] += e * bf16_to_double(vrow[x]);
            }
            for (int x = 0; x < d; ++x) o[x] = g * oP[x] + (1.0 - g) * (oD[x] / sumD);
        }
        if (gate_out) gate_out[(size_t)b * Hq + h] = g;
        if (skipped_out) skipped_out[(size_t)b * Hq + h] = skip;
        free(aP); free(aD); free(oP); free(oD);
    }
    return ORACLE_OK;
}

/*
 * Where the cache model keeps position j of a sequence: key and value rows of kv
 * head kv, or NULL for what it does not keep (the key of a distant position at a
 * layer that is not the lowest of that head's block).
 */
static const uint16_t *stored_key(const pod_oracle_cache *c, int layer, const seq_state *s, long j, int kv)
{
    const size_t re = row_elems(c);
    if (j < 0 || j >= s->n) return NULL;
    if (j < c->S) return s->sinkK + (size_t)j * re + (size_t)kv * c->d;
    const long rec_lo = s->n - s->n_recent;
    if (j >= rec_lo) return s->recK + (size_t)(j - rec_lo) * re + (size_t)kv * c->d;
    if (!is_lowest(c, layer, kv)) return NULL;
    return s->distK + (size_t)(j - c->S) * re + (size_t)kv * c->d;
}
static const uint16_t *stored_value(const pod_oracle_cache *c, const seq_state *s, long j, int kv)
{
    const size_t re = row_elems(c);
    if (j < 0 || j >= s->n) return NULL;
    if (j < c->S) return s->sinkV + (size_t)j * re + (size_t)kv * c->d;
    const long rec_lo = s->n - s->n_recent;
    if (j >= rec_lo) return s->recV + (size_t)(j - rec_lo) * re + (size_t)kv * c->d;
    return s->distV + (size_t)(j - c->S) * re + (size_t)kv * c->d;
}

/*
 * Attention of a chunk of T new tokens of one sequence against the cache model
 * and the chunk itself (a prompt processed in pieces).  The chunk is not stored
 * yet at `layer`: with p0 its stored length, chunk token t has position p0 + t
 * and sees positions j <= p0 + t, each by Eq. 3 taken at the query's own
 * position i (proximal: j < S or j > i - W):
 *   proximal j : this layer's q and key    (stored lists for j < p0, else k row j - p0)
 *   distant j  : q_shared row and the key of the lowest layer of the head's block
 *                (that layer's stored lists for j < p0, else k_shared row j - p0)
 *   value      : always this layer's       (stored lists for j < p0, else v row j - p0)
 * The lowest layer's lists may hold p0 tokens or may have taken the chunk already
 * (p0 + T).  q, q_shared: [T][Hq][d]; k, v, k_shared: [T][Hkv][d]; q_shared and
 * k_shared may be NULL when this layer is the lowest for every kv head.
 * out: [T][Hq][d] double.  One joint softmax per row (Eq. 4 / appendix).
 */
int oracle_chunk_attention(pod_oracle_cache *c, int layer, int seq, int Hq, double scale, int T,
                           const uint16_t *q, const uint16_t *k, const uint16_t *v,
                           const uint16_t *q_shared, const uint16_t *k_shared, double *out)
{
    if (!c || layer < 0 || layer >= c->L || seq < 0 || seq >= c->B || Hq < 1 || Hq % c->Hkv || T < 1) return ORACLE_ERR_ARG;
    const int rep = Hq / c->Hkv, d = c->d, Hkv = c->Hkv;
    seq_state *s = seq_of(c, layer, seq);
    const long p0 = s->n;
    if (p0 + T > c->max_ctx) return ORACLE_ERR_CAPACITY;
    for (int h = 0; h < Hkv; ++h) {
        if (is_lowest(c, layer, h)) continue;
        if (!q_shared || !k_shared) return ORACLE_ERR_ARG;
        const long nl = seq_of(c, lowest_of(c, layer, h), seq)->n;
        if (nl != p0 && nl != p0 + T) return ORACLE_ERR_STATE;
    }
    const long work = (long)T * Hq;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long w = 0; w < work; ++w) {
        const int t = (int)(w / Hq), h = (int)(w % Hq), kv = h / rep;
        const long i = p0 + t;
        const int la = lowest_of(c, layer, kv);
        const seq_state *sa = seq_of(c, la, seq);
        const uint16_t *qi = q + ((size_t)t * Hq + h) * d;
        const uint16_t *qs = la == layer ? qi : q_shared + ((size_t)t * Hq + h) * d;
        double *a = (double *)malloc((size_t)(i + 1) * sizeof(double));
        if (!a) { bad = 1; continue; }
        double amax = -INFINITY;
        for (long j = 0; j <= i; ++j) {
            const uint16_t *key;
            if (is_proximal(j, i, c->S, c->W)) {
                key = j < p0 ? stored_key(c, layer, s, j, kv) : k + ((size_t)(j - p0) * Hkv + kv) * d;
                a[j] = key ? scale * dot_bf16(qi, key, d) : NAN;      /* Eq. 3, line 1 */
            } else {
                if (la == layer) key = j < p0 ? stored_key(c, layer, s, j, kv) : k + ((size_t)(j - p0) * Hkv + kv) * d;
                else key = j < p0 ? stored_key(c, la, sa, j, kv) : k_shared + ((size_t)(j - p0) * Hkv + kv) * d;
                a[j] = key ? scale * dot_bf16(qs, key, d) : NAN;      /* Eq. 3, line 3 */
            }
            if (!key) bad = 2;   /* the model does not hold what Eq. 3 asks for: cannot happen if the cache rule is right */
            if (a[j] > amax) amax = a[j];
        }
        double denom = 0.0;
        for (long j = 0; j <= i; ++j) { a[j] = exp(a[j] - amax); denom += a[j]; }
        double *o = out + ((size_t)t * Hq + h) * d;
        for (int x = 0; x < d; ++x) o[x] = 0.0;
        for (long j = 0; j <= i; ++j) {
            const double p = a[j] / denom;
            const uint16_t *vj = j < p0 ? stored_value(c, s, j, kv) : v + ((size_t)(j - p0) * Hkv + kv) * d;
            for (int x = 0; x < d; ++x) o[x] += p * bf16_to_double(vj[x]);
        }
        free(a);
    }
    return bad == 1 ? ORACLE_ERR_CAPACITY : (bad == 2 ? ORACLE_ERR_STATE : ORACLE_OK);
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
