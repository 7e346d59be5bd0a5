/* Driver that walks the oracle's entry points over small, ragged cases; built together with
 * oracle/fss_oracle.c under -fsanitize=address,undefined by tests/test_oracle_sanitized.py.
 * Exit status 0 = every reconstruction held and the sanitizers stayed silent. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

size_t oracle_cmp_key_bytes(int n, size_t batch);
size_t oracle_eq_key_bytes(int n, size_t batch);
int oracle_cmp_gen(int n, size_t batch, const uint32_t *alpha, const uint32_t *alpha_r, const uint8_t *seed0, const uint8_t *seed1, void *key0, void *key1);
int oracle_eq_gen(int n, size_t batch, const uint32_t *alpha, const uint32_t *alpha_r, const uint8_t *seed0, const uint8_t *seed1, void *key0, void *key1);
int oracle_cmp_eval(int party, int n, size_t batch, const void *key, const uint32_t *x, uint32_t *out);
int oracle_eq_eval(int party, int n, size_t batch, const void *key, const uint32_t *x, uint32_t *out);
int oracle_cmp_eval_all_x(int party, int n, size_t batch, const void *key, size_t e, uint32_t *out);
int oracle_sign_mask(int n, size_t batch, const void *key, const uint32_t *y_share, uint32_t *masked);
int oracle_relu_open(int party, int n, size_t batch, const void *key, const uint32_t *masked0, const uint32_t *masked1, const uint32_t *y_share,
                     const uint32_t *tri_a, const uint32_t *tri_b, uint32_t *delta, uint32_t *eps);
int oracle_relu_finish(int party, int n, size_t batch, const uint32_t *delta0, const uint32_t *delta1, const uint32_t *eps0, const uint32_t *eps1,
                       const uint32_t *tri_a, const uint32_t *tri_b, const uint32_t *tri_c, uint32_t *out);
int oracle_maxpool_unroll(size_t channels, int h, int w, int k, int s, const uint32_t *x_share, uint32_t *rows);

static uint64_t state = 0x2006045932006ULL;
static uint32_t rnd(void) { state = state * 6364136223846793005ULL + 1442695040888963407ULL; return (uint32_t)(state >> 32); }
static uint32_t ring(int n) { return n == 32 ? 0xffffffffu : ((1u << n) - 1u); }

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "failed: %s (line %d, n=%d batch=%zu)\n", #c, __LINE__, n, batch); return 1; } } while (0)

/* every buffer is malloc'ed at its exact size, so that an access one element past its end is caught */
static int one_case(int n, size_t batch)
{
    const uint32_t m = ring(n);
    uint32_t *alpha = malloc(4 * batch), *r = malloc(4 * batch), *x = malloc(4 * batch);
    uint8_t *s0 = malloc(16 * batch), *s1 = malloc(16 * batch);
    for (size_t e = 0; e < batch; e++) {
        alpha[e] = rnd() & m; r[e] = rnd() & m;
        x[e] = (e % 3 == 0) ? alpha[e] : (rnd() & m);
        for (int b = 0; b < 16; b++) { s0[16 * e + b] = (uint8_t)rnd(); s1[16 * e + b] = (uint8_t)rnd(); }
    }
    uint32_t *o0 = malloc(4 * batch), *o1 = malloc(4 * batch);
    for (int cmp = 0; cmp < 2; cmp++) {
        size_t nb = cmp ? oracle_cmp_key_bytes(n, batch) : oracle_eq_key_bytes(n, batch);
        void *k0 = malloc(nb), *k1 = malloc(nb);
        CHECK((cmp ? oracle_cmp_gen : oracle_eq_gen)(n, batch, alpha, r, s0, s1, k0, k1) == 0);
        CHECK((cmp ? oracle_cmp_eval : oracle_eq_eval)(0, n, batch, k0, x, o0) == 0);
        CHECK((cmp ? oracle_cmp_eval : oracle_eq_eval)(1, n, batch, k1, x, o1) == 0);
        for (size_t e = 0; e < batch; e++)
            CHECK(((o0[e] + o1[e]) & m) == (uint32_t)(cmp ? x[e] <= alpha[e] : x[e] == alpha[e]));
        if (cmp && n <= 8) {
            uint32_t *a0 = malloc(4u << n), *a1 = malloc(4u << n);
            CHECK(oracle_cmp_eval_all_x(0, n, batch, k0, batch - 1, a0) == 0 && oracle_cmp_eval_all_x(1, n, batch, k1, batch - 1, a1) == 0);
            for (uint32_t v = 0; v <= m; v++) CHECK(((a0[v] + a1[v]) & m) == (uint32_t)(v <= alpha[batch - 1]));
            free(a0); free(a1);
        }
        if (cmp) {   /* the ReLU round on top of the same keys */
            uint32_t *y[2], *ta[2], *tb[2], *tc[2], *mk[2], *dl[2], *ep[2], *z[2];
            for (int j = 0; j < 2; j++) {
                y[j] = malloc(4 * batch); ta[j] = malloc(4 * batch); tb[j] = malloc(4 * batch); tc[j] = malloc(4 * batch);
                mk[j] = malloc(4 * batch); dl[j] = malloc(4 * batch); ep[j] = malloc(4 * batch); z[j] = malloc(4 * batch);
            }
            int32_t *plain = malloc(4 * batch);
            for (size_t e = 0; e < batch; e++) {
                plain[e] = (int32_t)(rnd() % 7) - 3;
                uint32_t a = rnd() & m, b = rnd() & m, c = (a * b) & m;
                y[0][e] = rnd() & m; y[1][e] = ((uint32_t)plain[e] - y[0][e]) & m;
                ta[0][e] = rnd() & m; ta[1][e] = (a - ta[0][e]) & m;
                tb[0][e] = rnd() & m; tb[1][e] = (b - tb[0][e]) & m;
                tc[0][e] = rnd() & m; tc[1][e] = (c - tc[0][e]) & m;
            }
            CHECK(oracle_sign_mask(n, batch, k0, y[0], mk[0]) == 0 && oracle_sign_mask(n, batch, k1, y[1], mk[1]) == 0);
            for (int j = 0; j < 2; j++)
                CHECK(oracle_relu_open(j, n, batch, j ? k1 : k0, mk[0], mk[1], y[j], ta[j], tb[j], dl[j], ep[j]) == 0);
            for (int j = 0; j < 2; j++)
                CHECK(oracle_relu_finish(j, n, batch, dl[0], dl[1], ep[0], ep[1], ta[j], tb[j], tc[j], z[j]) == 0);
            /* what the protocol computes exactly: y . (1 - 1{y + alpha <= alpha}) over the ring */
            for (size_t e = 0; e < batch; e++) {
                const uint32_t masked = ((uint32_t)plain[e] + alpha[e]) & m;
                CHECK(((z[0][e] + z[1][e]) & m) == (masked <= alpha[e] ? 0u : ((uint32_t)plain[e] & m)));
            }
            for (int j = 0; j < 2; j++) { free(y[j]); free(ta[j]); free(tb[j]); free(tc[j]); free(mk[j]); free(dl[j]); free(ep[j]); free(z[j]); }
            free(plain);
        }
        free(k0); free(k1);
    }
    free(alpha); free(r); free(x); free(s0); free(s1); free(o0); free(o1);
    return 0;
}

int main(void)
{
    const int ns[] = { 1, 2, 7, 8, 16, 31, 32 };
    const size_t batches[] = { 1, 63, 64, 65, 130 };
    for (size_t i = 0; i < sizeof(ns) / sizeof(ns[0]); i++)
        for (size_t j = 0; j < sizeof(batches) / sizeof(batches[0]); j++)
            if (one_case(ns[i], batches[j])) return 1;
    /* window unrolling: 3 channels of 7 x 5, 3 x 3 windows at stride 2 -> 3 x 2 windows of 9 */
    {
        int n = 32; size_t batch = 3;
        uint32_t *img = malloc(4 * 3 * 7 * 5), *rows = malloc(4 * 3 * 3 * 2 * 9);
        for (int i = 0; i < 3 * 7 * 5; i++) img[i] = (uint32_t)i;
        CHECK(oracle_maxpool_unroll(3, 7, 5, 3, 2, img, rows) == 0);
        CHECK(rows[0] == 0 && rows[8] == 12 && rows[3 * 3 * 2 * 9 - 1] == 3 * 7 * 5 - 1);
        free(img); free(rows);
    }
    puts("oracle sanitizer walk: ok");
    return 0;
}
