/*
 * CPU oracle for the HashAttention decode path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar implementation of what the path computes, written
 * from the paper's definitions (arxiv 2412.14468):
 *   - mapping  phi(x) = relu(sign(F(x))), bits packed into an integer (section 4.1, eq. 2)
 *   - SCORE    Hamming distance as bitcount(xor) (section 4.1, eq. 1 and the
 *              "Implementation" paragraph); used as the similarity 32 - H,
 *              which orders tokens exactly as -H does
 *   - TOPK     the k best scores, by an ordinary top-k (section 4); optionally with the first and most
 *              recent tokens always kept and the budget counting only retrieved tokens (section 5)
 *   - GATHER-ATT  softmax attention restricted to the index set (section 4)
 *   - SDPA     single-query dense attention (section 3.1)
 *   - recall   of a selected set against the true pivotal tokens, ranked by a_i ||v_i|| (sections 4, 4.2)
 * All floating point is fp64.  No blocking, no fusion, no vectorisation.
 * It shares no code with the HIP library; only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  The product never does.
 *
 * Readings where the paper is silent (kept identical on the device side):
 *   - sign(0) gives bit 0 (relu(sign(0)) = 0): bit_j = (a_j > 0)
 *   - output unit j of F goes to bit j of the code (LSB = unit 0)
 *   - hidden activation of F is SiLU; no activation before the sign
 *   - ties in TOPK go to the lower token index; the set is returned ascending
 *   - k_eff = min(k, N); softmax is max-subtracted; the scale is an argument
 *   - phi_kv sees the key vector only (section 4.1, last paragraph)
 *
 * Pins: every function below is pinned by tests/test_oracle_*.py to brute
 * force, closed forms or a library routine; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define HA_BITS 32

typedef struct {
    int32_t n_heads;
    int32_t n_layers;            /* number of weight matrices */
    int32_t dims[5];             /* dims[0] = input dim, dims[n_layers] = 32 */
    const float* W[4];           /* [n_heads][dims[l]][dims[l+1]], y = x W */
    const float* bias[4];        /* [n_heads][dims[l+1]] or NULL */
} ha_mlp;

typedef struct {
    uint16_t* k;                 /* bf16 bits; contiguous [B][Hkv][n_max][d] or paged [P][Hkv][page][d] */
    uint16_t* v;
    uint32_t* codes;             /* same layout without the d axis */
    const int32_t* page_table;   /* [B][max_pages_per_seq], paged only */
    int32_t* seq_lens;           /* [B] */
    int64_t n_max;
    int32_t max_pages_per_seq;
    int32_t page_size;           /* 0 = contiguous */
    int32_t n_kv_heads;
    int32_t head_dim;
} ha_cache;

/* ---------------------------------------------------------------- helpers */

static double bf16_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* index of token t's row (in rows, not bytes) for sequence b, KV head h */
static int64_t row_of(const ha_cache* c, int b, int h, int64_t t)
{
    if (c->page_size == 0)
        return ((int64_t)b * c->n_kv_heads + h) * c->n_max + t;
    int64_t page = c->page_table[(int64_t)b * c->max_pages_per_seq + t / c->page_size];
    return (page * c->n_kv_heads + h) * c->page_size + t % c->page_size;
}

/* Threads the (sequence, head) loops may use from now on (timing only: results do not depend on it). */
void ha_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int ha_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------ mapping (section 4.1, eq. 2) */

/* F(x) for one vector and one head, then sign -> bit, packed LSB-first.
 * act (optional, 32 doubles) receives the pre-sign activations. */
uint32_t ha_oracle_encode_vec(const ha_mlp* m, int head, const uint16_t* x_bf16, double* act)
{
    double cur[512], nxt[512];
    int n_in = m->dims[0];
    for (int i = 0; i < n_in; ++i) cur[i] = bf16_to_double(x_bf16[i]);
    for (int l = 0; l < m->n_layers; ++l) {
        int di = m->dims[l], dout = m->dims[l + 1];
        const float* W = m->W[l] + (int64_t)head * di * dout;
        for (int j = 0; j < dout; ++j) {
            double z = 0.0;
            for (int i = 0; i < di; ++i) z += cur[i] * (double)W[(int64_t)i * dout + j];
            if (m->bias[l]) z += (double)m->bias[l][(int64_t)head * dout + j];
            if (l + 1 < m->n_layers) z = z / (1.0 + exp(-z));   /* SiLU between layers */
            nxt[j] = z;
        }
        memcpy(cur, nxt, sizeof(double) * dout);
    }
    uint32_t code = 0;
    for (int j = 0; j < HA_BITS; ++j) {
        if (act) act[j] = cur[j];
        if (cur[j] > 0.0) code |= (uint32_t)1 << j;
    }
    return code;
}

/* q [B][Hq][d] bf16 -> q_codes [B][Hq], act [B][Hq][32] (optional) */
void ha_oracle_encode_query(const ha_mlp* phi_q, const uint16_t* q, int batch, int d,
                            uint32_t* q_codes, double* act)
{
    int H = phi_q->n_heads;
    for (int b = 0; b < batch; ++b)
        for (int h = 0; h < H; ++h) {
            int64_t o = (int64_t)b * H + h;
            q_codes[o] = ha_oracle_encode_vec(phi_q, h, q + o * d, act ? act + o * HA_BITS : NULL);
        }
}

/* Key-code store update.
 * k_new != NULL: append n_new tokens per sequence: rows k_new/v_new [B][Hkv][n_new][d] are
 *   written at positions seq_lens[b] .. seq_lens[b]+n_new-1 together with their codes, then
 *   seq_lens[b] += n_new.
 * k_new == NULL: the rows are already in the cache; codes of the last min(n_new, seq_lens[b])
 *   tokens of every sequence are (re)computed from the cached keys; seq_lens is unchanged.
 * act (optional) receives pre-sign activations [B][Hkv][n_new][32] (slot j = j-th processed token). */
void ha_oracle_encode_keys(const ha_mlp* phi_kv, ha_cache* c, const uint16_t* k_new,
                           const uint16_t* v_new, int batch, int64_t n_new, double* act)
{
    int H = c->n_kv_heads, d = c->head_dim;
    for (int b = 0; b < batch; ++b) {
        int64_t len = c->seq_lens[b];
        int64_t start = k_new ? len : (len > n_new ? len - n_new : 0);
        int64_t cnt = k_new ? n_new : len - start;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < cnt; ++j) {
            for (int h = 0; h < H; ++h) {
                int64_t r = row_of(c, b, h, start + j);
                if (k_new) {
                    int64_t s = (((int64_t)b * H + h) * n_new + j) * d;
                    memcpy(c->k + r * d, k_new + s, sizeof(uint16_t) * d);
                    memcpy(c->v + r * d, v_new + s, sizeof(uint16_t) * d);
                }
                double* a = act ? act + (((int64_t)b * H + h) * n_new + j) * HA_BITS : NULL;
                c->codes[r] = ha_oracle_encode_vec(phi_kv, h, c->k + r * d, a);
            }
        }
        if (k_new) c->seq_lens[b] = (int32_t)(len + n_new);
    }
}

/* ------------------------------------------------ SCORE (section 4.1, eq. 1) */

/* similarity 32 - H(q, k), H = bitcount(xor) */
int32_t ha_oracle_score(uint32_t q_code, uint32_t k_code)
{
    uint32_t x = q_code ^ k_code;
    int32_t h = 0;
    while (x) { h += (int32_t)(x & 1u); x >>= 1; }
    return HA_BITS - h;
}

void ha_oracle_scores(uint32_t q_code, const uint32_t* k_codes, int64_t n, int32_t* scores)
{
    for (int64_t i = 0; i < n; ++i) scores[i] = ha_oracle_score(q_code, k_codes[i]);
}

/* ------------------------------------------------ TOPK (section 4) */

typedef struct { int32_t score; int32_t id; } ha_pair;

static int cmp_score_desc_id_asc(const void* a, const void* b)
{
    const ha_pair* x = (const ha_pair*)a;
    const ha_pair* y = (const ha_pair*)b;
    if (x->score != y->score) return (x->score > y->score) ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

static int cmp_i32(const void* a, const void* b)
{
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

/* Definition: order all tokens by (score descending, index ascending), keep the first
 * min(k, n), return them ascending by index.  Returns the count; *threshold (optional)
 * gets the smallest selected score. */
int64_t ha_oracle_topk_sort(const int32_t* scores, int64_t n, int64_t k, int32_t* idx, int32_t* threshold)
{
    int64_t ke = k < n ? k : n;
    if (ke <= 0) return 0;
    ha_pair* p = (ha_pair*)malloc(sizeof(ha_pair) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) { p[i].score = scores[i]; p[i].id = (int32_t)i; }
    qsort(p, (size_t)n, sizeof(ha_pair), cmp_score_desc_id_asc);
    if (threshold) *threshold = p[ke - 1].score;
    for (int64_t i = 0; i < ke; ++i) idx[i] = p[i].id;
    free(p);
    qsort(idx, (size_t)ke, sizeof(int32_t), cmp_i32);
    return ke;
}

/* Second, independent route to the same set: count tokens per score value, find the
 * largest T with #{score >= T} >= k, take every token above T and the first
 * k - #{score > T} tokens (in index order) that score exactly T. */
int64_t ha_oracle_topk_hist(const int32_t* scores, int64_t n, int64_t k, int32_t* idx, int32_t* threshold)
{
    int64_t ke = k < n ? k : n;
    if (ke <= 0) return 0;
    int64_t hist[HA_BITS + 1];
    memset(hist, 0, sizeof hist);
    for (int64_t i = 0; i < n; ++i) hist[scores[i]]++;
    int T = HA_BITS;
    int64_t at_least = hist[HA_BITS];        /* #{score >= T} */
    while (at_least < ke) { --T; at_least += hist[T]; }
    int64_t above = at_least - hist[T];      /* #{score > T} */
    int64_t quota = ke - above;              /* tokens taken from the tie bucket */
    int64_t out = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (scores[i] > T) idx[out++] = (int32_t)i;
        else if (scores[i] == T && quota > 0) { idx[out++] = (int32_t)i; --quota; }
    }
    if (threshold) *threshold = T;
    return out;
}

/* TOPK with the always-kept tokens of the evaluation protocol (section 5, "Baselines and setup"):
 * the first n_sink and the most recent n_local tokens are in the index set whatever they score, and
 * the budget k counts only the tokens retrieved besides them.  Written out:
 *   I = {0 .. lo-1}  u  lo + topk(scores[lo .. hi-1], k)  u  {hi .. n-1},
 *   lo = min(n_sink, n),  hi = max(lo, n - n_local),
 * ascending by index.  Returns |I|; *threshold gets the smallest retrieved score (0 when nothing is
 * retrieved), *n_retrieved the number of retrieved tokens. */
int64_t ha_oracle_topk_window(const int32_t* scores, int64_t n, int64_t k, int64_t n_sink, int64_t n_local,
                              int32_t* idx, int32_t* threshold, int64_t* n_retrieved)
{
    if (n < 0) n = 0;
    int64_t lo = n_sink < n ? n_sink : n;
    if (lo < 0) lo = 0;
    int64_t hi = n - (n_local > 0 ? n_local : 0);
    if (hi < lo) hi = lo;
    int64_t out = 0;
    for (int64_t t = 0; t < lo; ++t) idx[out++] = (int32_t)t;
    int32_t T = 0;
    int64_t got = ha_oracle_topk_sort(scores + lo, hi - lo, k, idx + out, &T);
    for (int64_t i = 0; i < got; ++i) idx[out + i] += (int32_t)lo;      /* back to token ids of the sequence */
    out += got;
    for (int64_t t = hi; t < n; ++t) idx[out++] = (int32_t)t;
    if (threshold) *threshold = got > 0 ? T : 0;
    if (n_retrieved) *n_retrieved = got;
    return out;
}

/* ------------------------------------------------ GATHER-ATT and SDPA (sections 3.1, 4) */

/* o = sum_{i in I} softmax_i(scale <q, k_i>) v_i over the rows listed in idx (logical token ids
 * of sequence b, KV head h).  out: d doubles.  cnt == 0 gives zeros. */
void ha_oracle_gather_attend(const ha_cache* c, int b, int h, const uint16_t* q_bf16,
                             const int32_t* idx, int64_t cnt, double scale, double* out)
{
    int d = c->head_dim;
    for (int j = 0; j < d; ++j) out[j] = 0.0;
    if (cnt <= 0) return;
    double* logit = (double*)malloc(sizeof(double) * (size_t)cnt);
    double m = -INFINITY;
    for (int64_t i = 0; i < cnt; ++i) {
        const uint16_t* kr = c->k + row_of(c, b, h, idx[i]) * d;
        double s = 0.0;
        for (int j = 0; j < d; ++j) s += bf16_to_double(q_bf16[j]) * bf16_to_double(kr[j]);
        logit[i] = s * scale;
        if (logit[i] > m) m = logit[i];
    }
    double denom = 0.0;
    for (int64_t i = 0; i < cnt; ++i) {
        double w = exp(logit[i] - m);
        const uint16_t* vr = c->v + row_of(c, b, h, idx[i]) * d;
        denom += w;
        for (int j = 0; j < d; ++j) out[j] += w * bf16_to_double(vr[j]);
    }
    for (int j = 0; j < d; ++j) out[j] /= denom;
    free(logit);
}

/* single-query SDPA over all n tokens: the index set is {0..n-1} */
void ha_oracle_dense_attend(const ha_cache* c, int b, int h, const uint16_t* q_bf16,
                            int64_t n, double scale, double* out)
{
    int32_t* all = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) all[i] = (int32_t)i;
    ha_oracle_gather_attend(c, b, h, q_bf16, all, n, scale, out);
    free(all);
}

/* ------------------------------------------------ quality of a SCORE function (sections 4 and 4.2) */

/* Contribution of every token of (b, h) to the dense attention output: a_i * ||v_i||_2, with a the
 * softmax of scale <q, k_i> over all n tokens (the lemma on the best ordering for SDPA, section 4.2).
 * contrib: n doubles. */
void ha_oracle_token_contributions(const ha_cache* c, int b, int h, const uint16_t* q_bf16,
                                   int64_t n, double scale, double* contrib)
{
    int d = c->head_dim;
    if (n <= 0) return;
    double m = -INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        const uint16_t* kr = c->k + row_of(c, b, h, i) * d;
        double s = 0.0;
        for (int j = 0; j < d; ++j) s += bf16_to_double(q_bf16[j]) * bf16_to_double(kr[j]);
        contrib[i] = s * scale;
        if (contrib[i] > m) m = contrib[i];
    }
    double denom = 0.0;
    for (int64_t i = 0; i < n; ++i) { contrib[i] = exp(contrib[i] - m); denom += contrib[i]; }
    for (int64_t i = 0; i < n; ++i) {
        const uint16_t* vr = c->v + row_of(c, b, h, i) * d;
        double nv = 0.0;
        for (int j = 0; j < d; ++j) nv += bf16_to_double(vr[j]) * bf16_to_double(vr[j]);
        contrib[i] = contrib[i] / denom * sqrt(nv);
    }
}

typedef struct { double key; int32_t id; } ha_dpair;

static int cmp_key_desc_id_asc(const void* a, const void* b)
{
    const ha_dpair* x = (const ha_dpair*)a;
    const ha_dpair* y = (const ha_dpair*)b;
    if (x->key != y->key) return (x->key > y->key) ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

/* I_true,k: the min(k, n) tokens with the largest contribution (ties to the lower index), ascending.
 * Returns the count. */
int64_t ha_oracle_true_topk(const ha_cache* c, int b, int h, const uint16_t* q_bf16, int64_t n,
                            int64_t k, double scale, int32_t* idx)
{
    int64_t ke = k < n ? k : n;
    if (ke <= 0) return 0;
    double* contrib = (double*)malloc(sizeof(double) * (size_t)n);
    ha_oracle_token_contributions(c, b, h, q_bf16, n, scale, contrib);
    ha_dpair* p = (ha_dpair*)malloc(sizeof(ha_dpair) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) { p[i].key = contrib[i]; p[i].id = (int32_t)i; }
    qsort(p, (size_t)n, sizeof(ha_dpair), cmp_key_desc_id_asc);
    for (int64_t i = 0; i < ke; ++i) idx[i] = p[i].id;
    qsort(idx, (size_t)ke, sizeof(int32_t), cmp_i32);
    free(p);
    free(contrib);
    return ke;
}

/* recall(I_n, I_true,k) = |I_n intersect I_true,k| / |I_true,k| (section 4); both lists hold distinct
 * token ids in any order.  An empty I_true gives 1. */
double ha_oracle_recall(const int32_t* chosen, int64_t n_chosen, const int32_t* truth, int64_t n_truth)
{
    if (n_truth <= 0) return 1.0;
    int64_t hit = 0;
    for (int64_t i = 0; i < n_truth; ++i)
        for (int64_t j = 0; j < n_chosen; ++j)
            if (chosen[j] == truth[i]) { ++hit; break; }
    return (double)hit / (double)n_truth;
}

/* ------------------------------------------------ one decode layer-step */

/* [append] -> encode query -> SCORE -> TOPK (full sort) -> GATHER-ATT for every
 * (sequence, query head); KV head of query head h is h / (Hq / Hkv).
 * k_new/v_new: [B][Hkv][d] or NULL (no append).  k_per_seq [B].
 * phi_q == NULL: q_codes [B][Hq] is an input (codes drawn directly, no mapping).
 * Outputs: q_codes [B][Hq]; idx [B][Hq][k_max]; count [B][Hq]; threshold [B][Hq];
 * out [B][Hq][d] doubles.  Heads are independent, so the (b, h) loop may run on
 * several threads; each iteration is the plain single-head computation. */
void ha_oracle_decode_step(const ha_mlp* phi_q, const ha_mlp* phi_kv, ha_cache* c,
                           const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new,
                           int batch, int n_q_heads, const int32_t* k_per_seq, int64_t k_max,
                           double scale, uint32_t* q_codes, int32_t* idx, int32_t* count,
                           int32_t* threshold, double* out)
{
    int d = c->head_dim, Hq = n_q_heads, g = Hq / c->n_kv_heads;
    if (k_new) ha_oracle_encode_keys(phi_kv, c, k_new, v_new, batch, 1, NULL);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < (int64_t)batch * Hq; ++bh) {
        int b = (int)(bh / Hq), h = (int)(bh % Hq), hk = h / g;
        int64_t n = c->seq_lens[b];
        const uint16_t* qv = q + bh * d;
        if (phi_q) q_codes[bh] = ha_oracle_encode_vec(phi_q, h, qv, NULL);   /* else: given */
        int32_t* scores = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        for (int64_t t = 0; t < n; ++t)
            scores[t] = ha_oracle_score(q_codes[bh], c->codes[row_of(c, b, hk, t)]);
        int32_t T = 0;
        int64_t cnt = ha_oracle_topk_sort(scores, n, k_per_seq[b], idx + bh * k_max, &T);
        count[bh] = (int32_t)cnt;
        threshold[bh] = T;
        ha_oracle_gather_attend(c, b, hk, qv, idx + bh * k_max, cnt, scale, out + bh * d);
        free(scores);
    }
}

/* The same step with the always-kept window of ha_oracle_topk_window.  idx rows have
 * pitch = k_max + n_sink + n_local entries; count is the size of the whole index set. */
void ha_oracle_decode_step_window(const ha_mlp* phi_q, const ha_mlp* phi_kv, ha_cache* c,
                                  const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new,
                                  int batch, int n_q_heads, const int32_t* k_per_seq, int64_t k_max,
                                  int64_t n_sink, int64_t n_local,
                                  double scale, uint32_t* q_codes, int32_t* idx, int32_t* count,
                                  int32_t* threshold, double* out)
{
    int d = c->head_dim, Hq = n_q_heads, g = Hq / c->n_kv_heads;
    int64_t pitch = k_max + n_sink + n_local;
    if (k_new) ha_oracle_encode_keys(phi_kv, c, k_new, v_new, batch, 1, NULL);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < (int64_t)batch * Hq; ++bh) {
        int b = (int)(bh / Hq), h = (int)(bh % Hq), hk = h / g;
        int64_t n = c->seq_lens[b];
        const uint16_t* qv = q + bh * d;
        if (phi_q) q_codes[bh] = ha_oracle_encode_vec(phi_q, h, qv, NULL);   /* else: given */
        int32_t* scores = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        for (int64_t t = 0; t < n; ++t)
            scores[t] = ha_oracle_score(q_codes[bh], c->codes[row_of(c, b, hk, t)]);
        int32_t T = 0;
        int64_t cnt = ha_oracle_topk_window(scores, n, k_per_seq[b], n_sink, n_local, idx + bh * pitch, &T, NULL);
        count[bh] = (int32_t)cnt;
        threshold[bh] = T;
        ha_oracle_gather_attend(c, b, hk, qv, idx + bh * pitch, cnt, scale, out + bh * d);
        free(scores);
    }
}

/* ------------------------------------------------ wider signatures (section 5.3 ablation on bit width;
 * the SCORE latency table of the appendix lists 64 to 512 bits)
 *
 * A code of b = 32 * words bits is `words` consecutive uint32; output unit j of F goes to bit j % 32
 * of word j / 32.  The similarity is b - bitcount(xor) summed over the words, an integer in 0..b.
 * Code stores have the layout of the key cache without the d axis and with a trailing axis of
 * `words`; they are passed separately from the ha_cache (whose `codes` member is not used here). */

void ha_oracle_encode_vec_wide(const ha_mlp* m, int head, const uint16_t* x_bf16, int words,
                               uint32_t* code, double* act)
{
    double cur[512], nxt[512];
    int n_in = m->dims[0];
    for (int i = 0; i < n_in; ++i) cur[i] = bf16_to_double(x_bf16[i]);
    for (int l = 0; l < m->n_layers; ++l) {
        int di = m->dims[l], dout = m->dims[l + 1];
        const float* W = m->W[l] + (int64_t)head * di * dout;
        for (int j = 0; j < dout; ++j) {
            double z = 0.0;
            for (int i = 0; i < di; ++i) z += cur[i] * (double)W[(int64_t)i * dout + j];
            if (m->bias[l]) z += (double)m->bias[l][(int64_t)head * dout + j];
            if (l + 1 < m->n_layers) z = z / (1.0 + exp(-z));
            nxt[j] = z;
        }
        memcpy(cur, nxt, sizeof(double) * dout);
    }
    for (int w = 0; w < words; ++w) code[w] = 0;
    for (int j = 0; j < HA_BITS * words; ++j) {
        if (act) act[j] = cur[j];
        if (cur[j] > 0.0) code[j / 32] |= (uint32_t)1 << (j % 32);
    }
}

int32_t ha_oracle_score_wide(const uint32_t* q_code, const uint32_t* k_code, int words)
{
    int32_t h = 0;
    for (int w = 0; w < words; ++w) {
        uint32_t x = q_code[w] ^ k_code[w];
        while (x) { h += (int32_t)(x & 1u); x >>= 1; }
    }
    return HA_BITS * words - h;
}

void ha_oracle_scores_wide(const uint32_t* q_code, const uint32_t* k_codes, int64_t n, int words, int32_t* scores)
{
    for (int64_t i = 0; i < n; ++i) scores[i] = ha_oracle_score_wide(q_code, k_codes + i * words, words);
}

/* q [B][Hq][d] -> q_codes [B][Hq][words], act [B][Hq][32 words] (optional) */
void ha_oracle_encode_query_wide(const ha_mlp* phi_q, const uint16_t* q, int batch, int d, int words,
                                 uint32_t* q_codes, double* act)
{
    int H = phi_q->n_heads;
    for (int b = 0; b < batch; ++b)
        for (int h = 0; h < H; ++h) {
            int64_t o = (int64_t)b * H + h;
            ha_oracle_encode_vec_wide(phi_q, h, q + o * d, words, q_codes + o * words,
                                      act ? act + o * HA_BITS * words : NULL);
        }
}

/* as ha_oracle_encode_keys, codes [rows][words] */
void ha_oracle_encode_keys_wide(const ha_mlp* phi_kv, ha_cache* c, uint32_t* codes, int words,
                                const uint16_t* k_new, const uint16_t* v_new, int batch, int64_t n_new, double* act)
{
    int H = c->n_kv_heads, d = c->head_dim;
    for (int b = 0; b < batch; ++b) {
        int64_t len = c->seq_lens[b];
        int64_t start = k_new ? len : (len > n_new ? len - n_new : 0);
        int64_t cnt = k_new ? n_new : len - start;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < cnt; ++j) {
            for (int h = 0; h < H; ++h) {
                int64_t r = row_of(c, b, h, start + j);
                if (k_new) {
                    int64_t s = (((int64_t)b * H + h) * n_new + j) * d;
                    memcpy(c->k + r * d, k_new + s, sizeof(uint16_t) * d);
                    memcpy(c->v + r * d, v_new + s, sizeof(uint16_t) * d);
                }
                double* a = act ? act + (((int64_t)b * H + h) * n_new + j) * HA_BITS * words : NULL;
                ha_oracle_encode_vec_wide(phi_kv, h, c->k + r * d, words, codes + r * words, a);
            }
        }
        if (k_new) c->seq_lens[b] = (int32_t)(len + n_new);
    }
}

/* The decode step with wide codes and the always-kept window (n_sink = n_local = 0: none).
 * q_codes [B][Hq][words]; idx rows of k_max + n_sink + n_local entries. */
void ha_oracle_decode_step_wide(const ha_mlp* phi_q, const ha_mlp* phi_kv, ha_cache* c, uint32_t* codes, int words,
                                const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new,
                                int batch, int n_q_heads, const int32_t* k_per_seq, int64_t k_max,
                                int64_t n_sink, int64_t n_local,
                                double scale, uint32_t* q_codes, int32_t* idx, int32_t* count,
                                int32_t* threshold, double* out)
{
    int d = c->head_dim, Hq = n_q_heads, g = Hq / c->n_kv_heads;
    int64_t pitch = k_max + n_sink + n_local;
    if (k_new) ha_oracle_encode_keys_wide(phi_kv, c, codes, words, k_new, v_new, batch, 1, NULL);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < (int64_t)batch * Hq; ++bh) {
        int b = (int)(bh / Hq), h = (int)(bh % Hq), hk = h / g;
        int64_t n = c->seq_lens[b];
        const uint16_t* qv = q + bh * d;
        if (phi_q) ha_oracle_encode_vec_wide(phi_q, h, qv, words, q_codes + bh * words, NULL);   /* else: given */
        int32_t* scores = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        for (int64_t t = 0; t < n; ++t)
            scores[t] = ha_oracle_score_wide(q_codes + bh * words, codes + row_of(c, b, hk, t) * words, words);
        int32_t T = 0;
        int64_t cnt = ha_oracle_topk_window(scores, n, k_per_seq[b], n_sink, n_local, idx + bh * pitch, &T, NULL);
        count[bh] = (int32_t)cnt;
        threshold[bh] = T;
        ha_oracle_gather_attend(c, b, hk, qv, idx + bh * pitch, cnt, scale, out + bh * d);
        free(scores);
    }
}
