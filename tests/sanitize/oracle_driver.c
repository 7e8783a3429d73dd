/* Drives every entry point of the CPU oracle once over small, ragged problems, for a build with
 * -fsanitize=address,undefined: exact-size heap buffers, so that any read or write past an end, any
 * misaligned access or signed overflow in the oracle is reported.  Values are checked elsewhere
 * (tests/test_oracle_*.py); this program only has to run clean and return 0. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint8_t *k_codes, *v_codes;
    uint16_t *k_meta, *v_meta;
    int32_t num_pages, page_size, num_kv_heads, head_dim, bits, group_size;
} oracle_cache;

uint16_t oracle_f2h_rne(float f);
int oracle_kv_quant_write(const oracle_cache *c, const uint16_t *k, const uint16_t *v, const int64_t *slot_mapping, int32_t T);
int oracle_paged_decode_attn(const oracle_cache *c, const uint16_t *q, double *out, const int32_t *block_tables,
                             int32_t max_blocks_per_seq, const int32_t *context_lens, int32_t B, int32_t H,
                             double softmax_scale, int32_t num_threads);
int oracle_paged_prefill_attn(const oracle_cache *c, const uint16_t *q, double *out, const int32_t *q_start,
                              const int32_t *block_tables, int32_t max_blocks_per_seq, const int32_t *context_lens,
                              int32_t B, int32_t H, double softmax_scale, int32_t num_threads);
int oracle_kv_dequant_page(const oracle_cache *c, int32_t page, uint16_t *k_out, uint16_t *v_out);
size_t oracle_kv_swap_bytes(const oracle_cache *c, int32_t num_tokens);
int oracle_kv_swap_out(const oracle_cache *c, const int32_t *block_table, int32_t num_tokens, uint8_t *packed);
int oracle_kv_swap_in(oracle_cache *c, const int32_t *block_table, int32_t num_tokens, const uint8_t *packed);
int oracle_add_layernorm(const uint16_t *x, const uint16_t *residual, const uint16_t *gamma, const uint16_t *beta,
                         double eps, int64_t rows, int32_t hidden, uint16_t *h_out, double *y_out);
int oracle_bias_relu(const uint16_t *x, const uint16_t *bias, int64_t rows, int32_t cols, uint16_t *y_out);

static uint32_t rng_state = 12345u;
static float rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((float)(rng_state >> 8) / 8388608.0f - 1.0f) * 3.0f;
}
static uint16_t *random_halves(size_t n)
{
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t) + (n == 0));
    for (size_t i = 0; i < n; ++i) p[i] = oracle_f2h_rne(rnd());
    return p;
}
#define CHECK(x) do { if ((x) != 0) { fprintf(stderr, "%s failed at line %d\n", #x, __LINE__); return 1; } } while (0)

static int run(int bits, int G, int D, int P, int Hkv, int H)
{
    enum { B = 3 };
    const int32_t lens[B] = {2 * P + 3, 1, P};            /* ragged, one token, exactly one page */
    const int32_t max_blocks = 3;
    int32_t bt[B * 3];
    oracle_cache c;
    c.num_pages = 7; c.page_size = P; c.num_kv_heads = Hkv; c.head_dim = D; c.bits = bits; c.group_size = G;
    const size_t rows = (size_t)c.num_pages * Hkv * P;
    const size_t code_bytes = rows * (size_t)D * bits / 8, meta_halves = rows * (size_t)(D / G) * 2;
    c.k_codes = (uint8_t *)malloc(code_bytes); c.v_codes = (uint8_t *)malloc(code_bytes);
    c.k_meta = (uint16_t *)malloc(meta_halves * 2); c.v_meta = (uint16_t *)malloc(meta_halves * 2);
    memset(c.k_codes, 0xFF, code_bytes); memset(c.v_codes, 0xFF, code_bytes);
    memset(c.k_meta, 0x7E, meta_halves * 2); memset(c.v_meta, 0x7E, meta_halves * 2);
    /* pages dealt out backwards, the last page of the cache included */
    int next = c.num_pages - 1;
    for (int i = 0; i < B; ++i)
        for (int b = 0; b < max_blocks; ++b) bt[i * max_blocks + b] = b < (lens[i] + P - 1) / P ? next-- : 0;
    for (int i = 0; i < B; ++i) {
        const int32_t L = lens[i];
        uint16_t *k = random_halves((size_t)L * Hkv * D), *v = random_halves((size_t)L * Hkv * D);
        int64_t *slots = (int64_t *)malloc(sizeof(int64_t) * (size_t)L);
        for (int t = 0; t < L; ++t) slots[t] = (int64_t)bt[i * max_blocks + t / P] * P + t % P;
        if (L > 1) slots[0] = -1;                         /* a skipped token */
        CHECK(oracle_kv_quant_write(&c, k, v, slots, L));
        slots[0] = (int64_t)bt[i * max_blocks] * P;
        CHECK(oracle_kv_quant_write(&c, k, v, slots, 1));
        free(k); free(v); free(slots);
    }
    uint16_t *q = random_halves((size_t)B * H * D);
    double *out = (double *)malloc(sizeof(double) * (size_t)B * H * D);
    CHECK(oracle_paged_decode_attn(&c, q, out, bt, max_blocks, lens, B, H, 1.0 / sqrt((double)D), 2));
    const int32_t zero_lens[B] = {0, 0, 0};
    CHECK(oracle_paged_decode_attn(&c, q, out, bt, max_blocks, zero_lens, B, H, 1.0 / sqrt((double)D), 1));
    free(q); free(out);
    const int32_t q_start[B + 1] = {0, P + 2, P + 2, P + 2 + P};      /* chunks of P + 2, 0 and P tokens */
    const int32_t total = q_start[B];
    q = random_halves((size_t)total * H * D);
    out = (double *)malloc(sizeof(double) * (size_t)total * H * D);
    CHECK(oracle_paged_prefill_attn(&c, q, out, q_start, bt, max_blocks, lens, B, H, 1.0 / sqrt((double)D), 3));
    free(q); free(out);
    uint16_t *ko = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)P * Hkv * D), *vo = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)P * Hkv * D);
    CHECK(oracle_kv_dequant_page(&c, c.num_pages - 1, ko, vo));
    CHECK(oracle_kv_dequant_page(&c, 0, ko, vo));
    free(ko); free(vo);
    const size_t nb = oracle_kv_swap_bytes(&c, lens[0]);
    uint8_t *packed = (uint8_t *)malloc(nb);
    CHECK(oracle_kv_swap_out(&c, bt, lens[0], packed));
    const int32_t other[3] = {0, 1, 2};
    CHECK(oracle_kv_swap_in(&c, other, lens[0], packed));
    free(packed);
    free(c.k_codes); free(c.v_codes); free(c.k_meta); free(c.v_meta);
    return 0;
}

int main(void)
{
    CHECK(run(8, 64, 64, 16, 2, 2));
    CHECK(run(8, 16, 128, 8, 3, 3));
    CHECK(run(8, 128, 128, 32, 2, 8));
    CHECK(run(4, 32, 128, 16, 2, 4));
    CHECK(run(4, 64, 64, 8, 1, 3));
    for (int hidden = 8; hidden <= 264; hidden += 128) {
        const int64_t rows = 5;
        uint16_t *x = random_halves((size_t)rows * hidden), *r = random_halves((size_t)rows * hidden);
        uint16_t *g = random_halves((size_t)hidden), *b = random_halves((size_t)hidden);
        uint16_t *h = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)rows * hidden);
        double *y = (double *)malloc(sizeof(double) * (size_t)rows * hidden);
        CHECK(oracle_add_layernorm(x, r, g, b, 1e-5, rows, hidden, h, y));
        CHECK(oracle_add_layernorm(x, NULL, g, b, 0.0, rows, hidden, h, y));
        CHECK(oracle_bias_relu(x, b, rows, hidden, h));
        CHECK(oracle_bias_relu(x, NULL, rows, hidden, h));
        free(x); free(r); free(g); free(b); free(h); free(y);
    }
    puts("oracle sanitizer driver: ok");
    return 0;
}
