/* Host-side sanitizer run of the CPU oracle: compiled together with oracle/hashattn_oracle.c under
 * -fsanitize=address,undefined by tests/test_oracle_sanitized.py.  Every exported function is called on
 * small inputs that sit on the edges of its buffers (empty and one-token sequences, k > N, a kept window
 * wider than the sequence, the last row of a cache, a paged cache with a ragged last page, a 512-wide
 * last layer), with every buffer allocated at exactly the size the Python wrapper would pass, so an
 * access one element past an end is reported by the sanitizer.  A few invariants are checked as well;
 * the exit status is the number of failed checks. */
#include "../oracle/hashattn_oracle.c"

#include <stdio.h>

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { ++failures; fprintf(stderr, "check failed, line %d: %s\n", __LINE__, #cond); } } while (0)

static uint32_t rng_state = 241214468u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state; }
static uint16_t rnd_bf16(void) { return (uint16_t)(((rnd() >> 16) & 0x807f) | 0x3f00 | ((rnd() >> 20) & 0x0080)); }   /* |x| in [0.5, 2) */
static float rnd_w(void) { return ((float)(rnd() >> 8) / 8388608.0f - 1.0f) * 0.1f; }

static float* weights(int heads, int din, int dout)
{
    float* w = (float*)malloc(sizeof(float) * (size_t)heads * din * dout);
    for (long i = 0; i < (long)heads * din * dout; ++i) w[i] = rnd_w();
    return w;
}

int main(void)
{
    enum { B = 3, HKV = 2, HQ = 4, D = 128, NMAX = 40, PAGE = 16 };
    /* ---- mapping networks: 128 -> 64 -> 32 per head, and a wide one 128 -> 512 */
    ha_mlp phi_q = {HQ, 2, {D, 64, 32, 0, 0}, {weights(HQ, D, 64), weights(HQ, 64, 32), NULL, NULL}, {NULL, NULL, NULL, NULL}};
    ha_mlp phi_kv = {HKV, 2, {D, 64, 32, 0, 0}, {weights(HKV, D, 64), weights(HKV, 64, 32), NULL, NULL}, {NULL, NULL, NULL, NULL}};
    float* bias512 = (float*)malloc(sizeof(float) * HKV * 512);
    for (int i = 0; i < HKV * 512; ++i) bias512[i] = rnd_w();
    ha_mlp phi_wide = {HKV, 1, {D, 512, 0, 0, 0}, {weights(HKV, D, 512), NULL, NULL, NULL}, {bias512, NULL, NULL, NULL}};

    /* ---- contiguous cache: lengths 39 (one free row), 1 and 0 */
    uint16_t* k = (uint16_t*)malloc(sizeof(uint16_t) * B * HKV * NMAX * D);
    uint16_t* v = (uint16_t*)malloc(sizeof(uint16_t) * B * HKV * NMAX * D);
    for (long i = 0; i < (long)B * HKV * NMAX * D; ++i) { k[i] = rnd_bf16(); v[i] = rnd_bf16(); }
    uint32_t* codes = (uint32_t*)calloc((size_t)B * HKV * NMAX, sizeof(uint32_t));
    int32_t lens[B] = {NMAX - 1, 1, 0};
    ha_cache c = {k, v, codes, NULL, lens, NMAX, 0, 0, HKV, D};
    double* act = (double*)malloc(sizeof(double) * B * HKV * NMAX * 32);
    ha_oracle_encode_keys(&phi_kv, &c, NULL, NULL, B, NMAX, act);          /* in place, n_new > every length */
    CHECK(lens[0] == NMAX - 1 && lens[1] == 1 && lens[2] == 0);

    uint16_t* q = (uint16_t*)malloc(sizeof(uint16_t) * B * HQ * D);
    for (int i = 0; i < B * HQ * D; ++i) q[i] = rnd_bf16();
    uint32_t q_codes[B * HQ];
    double q_act[B * HQ * 32];
    ha_oracle_encode_query(&phi_q, q, B, D, q_codes, q_act);
    for (int i = 0; i < B * HQ; ++i)
        for (int j = 0; j < 32; ++j) CHECK(((q_codes[i] >> j) & 1u) == (q_act[i * 32 + j] > 0.0 ? 1u : 0u));

    /* ---- whole step with an append into the last free row; k larger than every sequence */
    uint16_t k_new[B * HKV * D], v_new[B * HKV * D];
    for (int i = 0; i < B * HKV * D; ++i) { k_new[i] = rnd_bf16(); v_new[i] = rnd_bf16(); }
    int32_t k_per_seq[B] = {7, 50, 3};
    enum { KMAX = 50 };
    int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * B * HQ * KMAX);
    int32_t count[B * HQ], thr[B * HQ];
    double* out = (double*)malloc(sizeof(double) * B * HQ * D);
    ha_oracle_decode_step(&phi_q, &phi_kv, &c, q, k_new, v_new, B, HQ, k_per_seq, KMAX, 0.088, q_codes, idx, count, thr, out);
    CHECK(lens[0] == NMAX && lens[1] == 2 && lens[2] == 1);
    CHECK(count[0] == 7 && count[HQ] == 2 && count[2 * HQ] == 1);
    for (int j = 0; j < D; ++j) CHECK(out[2 * HQ * D + j] == bf16_to_double(v_new[2 * HKV * D + j]));   /* one token: its V row */

    /* ---- kept window wider than the sequences; window + budget exactly filling the row */
    enum { SINK = 3, LOCAL = 40 };
    int32_t* idx_w = (int32_t*)malloc(sizeof(int32_t) * B * HQ * (KMAX + SINK + LOCAL));
    lens[0] = NMAX; lens[1] = 2; lens[2] = 0;
    ha_oracle_decode_step_window(&phi_q, NULL, &c, q, NULL, NULL, B, HQ, k_per_seq, KMAX, SINK, LOCAL, 0.088, q_codes,
                                 idx_w, count, thr, out);
    CHECK(count[0] == NMAX && count[HQ] == 2 && count[2 * HQ] == 0);

    /* ---- SCORE / TOPK on the edges */
    int32_t sc[NMAX], sel[NMAX], T = -1;
    ha_oracle_scores(q_codes[0], codes, NMAX, sc);
    for (int i = 0; i < NMAX; ++i) CHECK(sc[i] == 32 - ha_oracle_score(q_codes[0], codes[i]) || sc[i] == ha_oracle_score(q_codes[0], codes[i]));
    CHECK(ha_oracle_score(0xffffffffu, 0u) + ha_oracle_score(0u, 0u) == 32);
    CHECK(ha_oracle_topk_sort(sc, NMAX, NMAX + 5, sel, &T) == NMAX);
    CHECK(ha_oracle_topk_hist(sc, NMAX, NMAX, sel, &T) == NMAX && sel[NMAX - 1] == NMAX - 1);
    CHECK(ha_oracle_topk_sort(sc, 0, 4, sel, &T) == 0 && ha_oracle_topk_hist(sc, 1, 1, sel, &T) == 1);
    int64_t got = -1;
    CHECK(ha_oracle_topk_window(sc, NMAX, 5, 0, 0, sel, &T, &got) == 5 && got == 5);
    CHECK(ha_oracle_topk_window(sc, NMAX, 100, 10, 10, sel, &T, &got) == NMAX && got == NMAX - 20);
    CHECK(ha_oracle_topk_window(sc, 0, 3, 2, 2, sel, &T, &got) == 0);

    /* ---- attention helpers on the last row of the cache */
    int32_t last_row[1] = {NMAX - 1};
    double o1[D], contrib[NMAX];
    ha_oracle_gather_attend(&c, 0, HKV - 1, q, last_row, 1, 0.5, o1);
    for (int j = 0; j < D; ++j) CHECK(o1[j] == bf16_to_double(v[((0 * HKV + HKV - 1) * (long)NMAX + NMAX - 1) * D + j]));
    ha_oracle_dense_attend(&c, 0, 1, q, NMAX, 0.088, o1);
    ha_oracle_gather_attend(&c, 0, 1, q, last_row, 0, 0.5, o1);              /* empty set */
    ha_oracle_token_contributions(&c, 0, 1, q, NMAX, 0.088, contrib);
    int32_t truth[NMAX];
    CHECK(ha_oracle_true_topk(&c, 0, 1, q, NMAX, NMAX + 3, 0.088, truth) == NMAX);
    CHECK(ha_oracle_recall(truth, NMAX, truth, NMAX) == 1.0 && ha_oracle_recall(truth, 0, truth, 4) == 0.0);

    /* ---- paged cache: 3 pages of 16 tokens, sequence of 35 tokens with a ragged last page, append into it */
    enum { NPAGES = 4 };
    uint16_t* pk = (uint16_t*)malloc(sizeof(uint16_t) * NPAGES * HKV * PAGE * D);
    uint16_t* pv = (uint16_t*)malloc(sizeof(uint16_t) * NPAGES * HKV * PAGE * D);
    for (long i = 0; i < (long)NPAGES * HKV * PAGE * D; ++i) { pk[i] = rnd_bf16(); pv[i] = rnd_bf16(); }
    uint32_t* pcodes = (uint32_t*)calloc((size_t)NPAGES * HKV * PAGE, sizeof(uint32_t));
    int32_t table[3] = {3, 0, 2}, plen[1] = {35};
    ha_cache pc = {pk, pv, pcodes, table, plen, 3 * PAGE, 3, PAGE, HKV, D};
    ha_oracle_encode_keys(&phi_kv, &pc, NULL, NULL, 1, 35, NULL);
    int32_t pk_per_seq[1] = {9};
    ha_oracle_decode_step(&phi_q, &phi_kv, &pc, q, k_new, v_new, 1, HQ, pk_per_seq, 9, 0.088, q_codes, idx, count, thr, out);
    CHECK(plen[0] == 36 && count[0] == 9);
    for (int i = 0; i < 9; ++i) CHECK(idx[i] >= 0 && idx[i] < 36 && (i == 0 || idx[i] > idx[i - 1]));

    /* ---- wide signatures: 512 bits = 16 words per code */
    enum { WORDS = 16 };
    uint32_t* wcodes = (uint32_t*)calloc((size_t)B * HKV * NMAX * WORDS, sizeof(uint32_t));
    lens[0] = NMAX - 1; lens[1] = 1; lens[2] = 0;
    ha_oracle_encode_keys_wide(&phi_wide, &c, wcodes, WORDS, NULL, NULL, B, NMAX, NULL);
    ha_oracle_encode_keys_wide(&phi_wide, &c, wcodes, WORDS, k_new, v_new, B, 1, NULL);      /* append into the last row */
    CHECK(lens[0] == NMAX);
    uint32_t wq[WORDS];
    double wact[512];
    ha_oracle_encode_vec_wide(&phi_wide, 1, q, WORDS, wq, wact);
    ha_oracle_scores_wide(wq, wcodes, NMAX, WORDS, sc);
    for (int i = 0; i < NMAX; ++i) CHECK(sc[i] >= 0 && sc[i] <= 512);
    CHECK(ha_oracle_score_wide(wq, wq, WORDS) == 512);

    ha_oracle_set_threads(2);
    CHECK(ha_oracle_num_threads() >= 1);
    if (failures) fprintf(stderr, "%d checks failed\n", failures);
    else printf("oracle sanitizer run: all checks passed\n");
    return failures;
}
