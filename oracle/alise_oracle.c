/*
 * CPU oracle for the quantized, paged KV-cache decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  Nothing in the product path may call it; it shares
 * no code, header, table or helper with the HIP sources.
 *
 * What it follows (ALISE, arXiv 2410.23537):
 *   - Sec. 3.2 "KV Compression": x_q = round(x / lambda + z), x = lambda (x_q - z),
 *     lambda = (max - min) / (2^b - 1), b-bit codes, INT8 by default.
 *   - Sec. 2, Eq. 1-2: per-head Attn = softmax(Q K^T / sqrt(d/h)) V, heads concatenated.
 *   - Sec. 2 "LLM Inference": each decode step appends the new token's K/V to the
 *     cache and attends over everything cached.
 *   - Sec. 3.3: the cache is block-level (paged), inherited from PagedAttention.
 *   - Sec. 3.2 "Dynamic Swapping", Alg. 2: a preempted job's whole KV cache is offloaded
 *     to CPU memory and uploaded again later, at the request level.  The oracle states
 *     the data movement (pack a request's pages into one buffer, unpack them into any
 *     pages); which job moves when is the scheduler's business and is not here.
 *
 * Readings where the paper is silent or garbled (all listed in the design notes):
 *   R1  the printed zero-point does not depend on min; taken as z = nint(-min / lambda).
 *   R2  codes and z are clamped to [0, 2^b - 1].
 *   R3  "round" is round-to-nearest, ties to even.
 *   R4  z is inside the rounding, and x * (1/lambda) + z is ONE fused multiply-add.
 *   R5  min/max run over the G values of a group and are widened to include 0.
 *   R6  the scale is floored at 2^-14 (smallest normal fp16).
 *   R7  the scale is stored as fp16, rounded UP, and quantization uses the stored value.
 *   R8  1/lambda is one correctly rounded fp32 division per group.
 *   R9  attention consumes the exact fp32 product lambda * (x_q - z); the page
 *       dequantizer returns its fp16 round-to-nearest-even.
 *   R10 a group is G contiguous channels of one token's one head vector; K and V alike.
 *   R12 the new token is written first and attended to from its quantized form.
 *   R13 the softmax scale is passed in (1/sqrt(head_dim) for Eq. 1).
 *   R14 INT4: channel 2i in the low nibble, 2i+1 in the high nibble of byte i.
 *   R15 query head h reads KV head h / (H / Hkv).
 *   R16 no mask beyond t < L_i; L_i = 0 gives a zero row.
 *   R18 prefill in chunks: the chunk's own K/V are written first (quantized, R12), then
 *       query j of an n-token chunk of a request with L cached tokens sits at position
 *       L - n + j and attends to positions 0 .. L - n + j (causal), all from the cache.
 *   R19 the fused LayerNorm (Sec. 3.3 "Implementation") takes the residual connection with it
 *       (Sec. 2 "Transformer Architecture": LayerNorm and residual connection surround the
 *       attention and FFN modules): h = fp16(x + residual), the exact sum rounded once;
 *       y = gamma (h - mean) / sqrt(var + eps) + beta over the hidden dimension of the
 *       fp16 h, var the biased variance (divide by N); the definition of layer normalization.
 *       The oracle returns y in fp64; the product rounds it to fp16.
 *   R20 the fused ReLU takes the bias of the FFN's first linear layer with it:
 *       y = fp16(max(x + bias, 0)), the exact sum rounded once, -0 becomes +0.
 *   R17 the offloaded form of a request is its pages in logical order, whole pages
 *       (every slot of the last page too), each as [K codes | V codes | K meta | V meta]
 *       per KV head: compressed bytes move as they are, nothing is requantized.
 *
 * Every fp32 step of the quantizer is a single IEEE-754 binary32 operation; build
 * with -ffp-contract=off so the compiler fuses nothing on its own.
 * Attention is evaluated in fp64 with a plain two-pass softmax.
 *
 * Parity pins: see tests/test_oracle_*.py (worked examples under tests/golden/,
 * half-step error bound, structural invariants, dense-attention cross-checks).
 * Layout strides, the INT4 nibble order (R14) and the GQA head mapping (R15) are
 * this build's conventions, not the paper's: parity unpinned by the paper for those.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- fp16 <-> fp32 */

/* Exact widening of an IEEE binary16 bit pattern. */
float oracle_h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int32_t exp = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ffu;
    double v;
    if (exp == 0x1f) {
        v = man ? NAN : INFINITY;
    } else if (exp == 0) {
        v = ldexp((double)man, -24);
    } else {
        v = ldexp((double)(man | 0x400u), exp - 25);
    }
    return (float)(sign ? -v : v);
}

/* binary32 -> binary16, round to nearest, ties to even. */
uint16_t oracle_f2h_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    double a = fabs((double)f);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);   /* rounds to infinity */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);            /* a = m * 2^e, m in [0.5, 1) */
    int ulp_exp = e - 11;          /* 11 significant bits */
    if (ulp_exp < -24) ulp_exp = -24;   /* subnormal spacing */
    double scaled = ldexp(a, -ulp_exp); /* exact */
    double r = nearbyint(scaled);       /* ties to even under the default mode */
    double val = ldexp(r, ulp_exp);     /* a representable binary16 value */
    /* encode */
    if (val == 0.0) return sign;
    int e2;
    double m2 = frexp(val, &e2);        /* val = m2 * 2^e2 */
    if (e2 - 1 < -14) {
        uint32_t man = (uint32_t)ldexp(val, 24);
        return (uint16_t)(sign | man);
    }
    uint32_t man = (uint32_t)ldexp(m2, 11) - 0x400u;
    uint32_t ex = (uint32_t)(e2 - 1 + 15);
    return (uint16_t)(sign | (ex << 10) | man);
}

/* ---------------------------------------------------------------- quantizer */

/*
 * Quantize one group of G fp16 values to b-bit codes (Sec. 3.2, readings R1-R8).
 * codes: one byte per element (unpacked).  scale_h, zero_h: fp16 bit patterns.
 */
void oracle_quant_group(const uint16_t *x, int G, int bits,
                        uint8_t *codes, uint16_t *scale_h, uint16_t *zero_h)
{
    const float qmax = (float)((1 << bits) - 1);
    float mn = 0.0f, mx = 0.0f;                       /* R5: range includes 0 */
    for (int i = 0; i < G; ++i) {
        float v = oracle_h2f(x[i]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    float r = mx - mn;
    float l32 = r / qmax;                             /* lambda = (max-min)/(2^b-1) */
    uint16_t h = oracle_f2h_rne(l32);
    if (oracle_h2f(h) < l32) h = (uint16_t)(h + 1);   /* R7: next fp16 above */
    if (h < 0x0400u) h = 0x0400u;                     /* R6: floor 2^-14 */
    float lam = oracle_h2f(h);
    float inv = 1.0f / lam;                           /* R8 */
    float zf = nearbyintf((-mn) * inv);               /* R1, R3 */
    if (zf < 0.0f) zf = 0.0f;
    if (zf > qmax) zf = qmax;                         /* R2 */
    zf = (float)(int)zf;                              /* an integer; -0 becomes +0 */
    for (int i = 0; i < G; ++i) {
        float u = fmaf(oracle_h2f(x[i]), inv, zf);    /* R4: one rounding */
        float q = nearbyintf(u);                      /* R3 */
        if (q < 0.0f) q = 0.0f;
        if (q > qmax) q = qmax;                       /* R2 */
        codes[i] = (uint8_t)q;
    }
    *scale_h = h;
    *zero_h = oracle_f2h_rne(zf);                     /* integers <= 255 are exact */
}

/* Exact fp32 dequantized value lambda * (x_q - z) (R9). */
static float dequant_f32(uint8_t code, uint16_t scale_h, uint16_t zero_h)
{
    float lam = oracle_h2f(scale_h);
    float z = oracle_h2f(zero_h);
    /* code and every stored zero-point are integers of at most 8 bits: the fp32 difference is exact.
     * (Taken in fp32 rather than in int so that the meta of a slot nobody wrote -- any bit pattern,
     * NaN included -- gives garbage without a float-to-int conversion that C leaves undefined.) */
    return lam * ((float)code - z);
}

/* ---------------------------------------------------------------- cache layout
 * codes: uint8 [num_pages][Hkv][P][D*bits/8]
 * meta : fp16  [num_pages][Hkv][P][D/G][2] = (scale, zero)
 */
typedef struct {
    uint8_t *k_codes, *v_codes;
    uint16_t *k_meta, *v_meta;
    int32_t num_pages, page_size, num_kv_heads, head_dim, bits, group_size;
} oracle_cache;

static size_t row_index(const oracle_cache *c, int64_t page, int head, int off)
{
    return ((size_t)page * c->num_kv_heads + head) * c->page_size + off;
}

static uint8_t get_code(const oracle_cache *c, const uint8_t *codes, size_t row, int d)
{
    size_t rb = (size_t)c->head_dim * c->bits / 8;
    if (c->bits == 8) return codes[row * rb + d];
    uint8_t byte = codes[row * rb + d / 2];           /* R14 */
    return (d & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xf);
}

static void put_code(const oracle_cache *c, uint8_t *codes, size_t row, int d, uint8_t q)
{
    size_t rb = (size_t)c->head_dim * c->bits / 8;
    if (c->bits == 8) { codes[row * rb + d] = q; return; }
    uint8_t *p = &codes[row * rb + d / 2];
    if (d & 1) *p = (uint8_t)((*p & 0x0f) | (q << 4));
    else       *p = (uint8_t)((*p & 0xf0) | (q & 0xf));
}

/* Step 1: quantize-and-write T tokens (k, v: fp16 [T][Hkv][D]) at slot_mapping[t]. */
int oracle_kv_quant_write(const oracle_cache *c, const uint16_t *k, const uint16_t *v,
                          const int64_t *slot_mapping, int32_t T)
{
    const int D = c->head_dim, G = c->group_size, ng = D / G;
    uint8_t *tmp = (uint8_t *)malloc((size_t)G);
    if (!tmp) return 1;
    for (int32_t t = 0; t < T; ++t) {
        int64_t s = slot_mapping[t];
        if (s < 0) continue;
        int64_t page = s / c->page_size;
        int off = (int)(s % c->page_size);
        for (int h = 0; h < c->num_kv_heads; ++h) {
            size_t row = row_index(c, page, h, off);
            for (int which = 0; which < 2; ++which) {
                const uint16_t *src = (which ? v : k) + ((size_t)t * c->num_kv_heads + h) * D;
                uint8_t *codes = which ? c->v_codes : c->k_codes;
                uint16_t *meta = which ? c->v_meta : c->k_meta;
                for (int g = 0; g < ng; ++g) {
                    uint16_t sh, zh;
                    oracle_quant_group(src + g * G, G, c->bits, tmp, &sh, &zh);
                    for (int i = 0; i < G; ++i) put_code(c, codes, row, g * G + i, tmp[i]);
                    meta[(row * ng + g) * 2 + 0] = sh;
                    meta[(row * ng + g) * 2 + 1] = zh;
                }
            }
        }
    }
    free(tmp);
    return 0;
}

/*
 * Step 2: single-query attention per request and query head over the cached,
 * quantized tokens (Eq. 1-2; R9, R12, R13, R15, R16).  out: fp64 [B][H][D].
 * (request, head) pairs are independent; num_threads only splits that loop.
 */
int oracle_paged_decode_attn(const oracle_cache *c, const uint16_t *q, double *out,
                             const int32_t *block_tables, int32_t max_blocks_per_seq,
                             const int32_t *context_lens, int32_t B, int32_t H,
                             double softmax_scale, int32_t num_threads)
{
    const int D = c->head_dim, G = c->group_size, ng = D / G, P = c->page_size;
    const int qper = H / c->num_kv_heads;
    int fail = 0;
    if (num_threads < 1) num_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(num_threads)
    for (int64_t ih = 0; ih < (int64_t)B * H; ++ih) {
        int i = (int)(ih / H), h = (int)(ih % H);
        int hk = h / qper;                                        /* R15 */
        int L = context_lens[i];
        double *o = out + (size_t)ih * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (L <= 0) continue;                                     /* R16 */
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        if (!s) { fail = 1; continue; }
        const uint16_t *qv = q + (size_t)ih * D;
        double m = -INFINITY;
        for (int t = 0; t < L; ++t) {
            int64_t page = block_tables[(size_t)i * max_blocks_per_seq + t / P];
            size_t row = row_index(c, page, hk, t % P);
            double acc = 0.0;
            for (int d = 0; d < D; ++d) {
                int g = d / G;
                float kd = dequant_f32(get_code(c, c->k_codes, row, d),
                                       c->k_meta[(row * ng + g) * 2], c->k_meta[(row * ng + g) * 2 + 1]);
                acc += (double)oracle_h2f(qv[d]) * (double)kd;
            }
            s[t] = acc * softmax_scale;
            if (s[t] > m) m = s[t];
        }
        double denom = 0.0;
        for (int t = 0; t < L; ++t) { s[t] = exp(s[t] - m); denom += s[t]; }
        for (int t = 0; t < L; ++t) {
            int64_t page = block_tables[(size_t)i * max_blocks_per_seq + t / P];
            size_t row = row_index(c, page, hk, t % P);
            double p = s[t] / denom;
            for (int d = 0; d < D; ++d) {
                int g = d / G;
                float vd = dequant_f32(get_code(c, c->v_codes, row, d),
                                       c->v_meta[(row * ng + g) * 2], c->v_meta[(row * ng + g) * 2 + 1]);
                o[d] += p * (double)vd;
            }
        }
        free(s);
    }
    return fail;
}

/* Step 3: one page back to fp16 K and V [P][Hkv][D], every slot (R9). */
int oracle_kv_dequant_page(const oracle_cache *c, int32_t page, uint16_t *k_out, uint16_t *v_out)
{
    const int D = c->head_dim, G = c->group_size, ng = D / G;
    for (int off = 0; off < c->page_size; ++off)
        for (int h = 0; h < c->num_kv_heads; ++h) {
            size_t row = row_index(c, page, h, off);
            for (int d = 0; d < D; ++d) {
                int g = d / G;
                size_t o = ((size_t)off * c->num_kv_heads + h) * D + d;
                k_out[o] = oracle_f2h_rne(dequant_f32(get_code(c, c->k_codes, row, d),
                              c->k_meta[(row * ng + g) * 2], c->k_meta[(row * ng + g) * 2 + 1]));
                v_out[o] = oracle_f2h_rne(dequant_f32(get_code(c, c->v_codes, row, d),
                              c->v_meta[(row * ng + g) * 2], c->v_meta[(row * ng + g) * 2 + 1]));
            }
        }
    return 0;
}

/*
 * Unquantized single-query attention on dense fp64 K, V [L][D] for one head
 * (Eq. 1): the plain definition, used to measure what quantization costs.
 */
void oracle_dense_attn(const double *q, const double *K, const double *V, int L, int D,
                       double softmax_scale, double *out)
{
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    if (L <= 0) return;
    double *s = (double *)malloc(sizeof(double) * (size_t)L);
    double m = -INFINITY, denom = 0.0;
    for (int t = 0; t < L; ++t) {
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += q[d] * K[(size_t)t * D + d];
        s[t] = acc * softmax_scale;
        if (s[t] > m) m = s[t];
    }
    for (int t = 0; t < L; ++t) { s[t] = exp(s[t] - m); denom += s[t]; }
    for (int t = 0; t < L; ++t)
        for (int d = 0; d < D; ++d) out[d] += s[t] / denom * V[(size_t)t * D + d];
    free(s);
}

/*
 * Chunked prefill (Sec. 2 "LLM Inference": the prompt's tokens are processed in one pass;
 * Eq. 1-2 with the causal order of an autoregressive model; R18).  q, out: [total_q][H][D],
 * the chunks of the requests back to back; q_start[i] .. q_start[i+1] - 1 are request i's
 * rows.  Every (query token, head) is the single-query definition over its own prefix.
 * out: fp64.  Returns nonzero if a chunk is longer than its request or memory runs out.
 */
int oracle_paged_prefill_attn(const oracle_cache *c, const uint16_t *q, double *out, const int32_t *q_start,
                              const int32_t *block_tables, int32_t max_blocks_per_seq,
                              const int32_t *context_lens, int32_t B, int32_t H,
                              double softmax_scale, int32_t num_threads)
{
    const int D = c->head_dim, G = c->group_size, ng = D / G, P = c->page_size;
    const int qper = H / c->num_kv_heads;
    int fail = 0;
    if (num_threads < 1) num_threads = 1;
    for (int i = 0; i < B; ++i)
        if (q_start[i + 1] - q_start[i] > context_lens[i] || q_start[i + 1] < q_start[i]) return 2;
#pragma omp parallel for schedule(dynamic, 1) num_threads(num_threads)
    for (int64_t row = 0; row < (int64_t)q_start[B] * H; ++row) {
        int tq = (int)(row / H), h = (int)(row % H);
        int i = 0;
        while (q_start[i + 1] <= tq) ++i;                         /* the request this query token belongs to */
        int n = q_start[i + 1] - q_start[i], j = tq - q_start[i];
        int L = context_lens[i] - n + j + 1;                      /* the query's own position is the last one it sees */
        int hk = h / qper;
        double *o = out + (size_t)row * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        if (!s) { fail = 1; continue; }
        const uint16_t *qv = q + (size_t)row * D;
        double m = -INFINITY;
        for (int t = 0; t < L; ++t) {
            int64_t page = block_tables[(size_t)i * max_blocks_per_seq + t / P];
            size_t r = row_index(c, page, hk, t % P);
            double acc = 0.0;
            for (int d = 0; d < D; ++d) {
                int g = d / G;
                float kd = dequant_f32(get_code(c, c->k_codes, r, d),
                                       c->k_meta[(r * ng + g) * 2], c->k_meta[(r * ng + g) * 2 + 1]);
                acc += (double)oracle_h2f(qv[d]) * (double)kd;
            }
            s[t] = acc * softmax_scale;
            if (s[t] > m) m = s[t];
        }
        double denom = 0.0;
        for (int t = 0; t < L; ++t) { s[t] = exp(s[t] - m); denom += s[t]; }
        for (int t = 0; t < L; ++t) {
            int64_t page = block_tables[(size_t)i * max_blocks_per_seq + t / P];
            size_t r = row_index(c, page, hk, t % P);
            double p = s[t] / denom;
            for (int d = 0; d < D; ++d) {
                int g = d / G;
                float vd = dequant_f32(get_code(c, c->v_codes, r, d),
                                       c->v_meta[(r * ng + g) * 2], c->v_meta[(r * ng + g) * 2 + 1]);
                o[d] += p * (double)vd;
            }
        }
        free(s);
    }
    return fail;
}

/* ---------------------------------------------------------------- dynamic swapping (data movement) */

/* Bytes of one (page, head) block in the offloaded form (R17). */
static size_t swap_block_bytes(const oracle_cache *c)
{
    size_t rowb = (size_t)c->head_dim * c->bits / 8, ng = (size_t)(c->head_dim / c->group_size);
    return 2 * (size_t)c->page_size * rowb + 2 * (size_t)c->page_size * ng * 4;
}

/* Size of the offloaded form of a request of num_tokens tokens. */
size_t oracle_kv_swap_bytes(const oracle_cache *c, int32_t num_tokens)
{
    size_t nblk = num_tokens > 0 ? ((size_t)num_tokens + c->page_size - 1) / c->page_size : 0;
    return nblk * (size_t)c->num_kv_heads * swap_block_bytes(c);
}

/*
 * Offload (Alg. 2 "offload"): copy the request's pages, found through its block table, into
 * `packed`, byte by byte.  Upload ("upload") is the same walk in the other direction, into
 * whatever pages the block table names at that time.  dir = 0: cache -> packed, 1: packed -> cache.
 */
static int swap_walk(oracle_cache *c, const int32_t *block_table, int32_t num_tokens, uint8_t *packed, int dir)
{
    const int P = c->page_size, H = c->num_kv_heads;
    const size_t rowb = (size_t)c->head_dim * c->bits / 8, ng = (size_t)(c->head_dim / c->group_size);
    const int nblk = num_tokens > 0 ? (num_tokens + P - 1) / P : 0;
    size_t pos = 0;
    for (int j = 0; j < nblk; ++j) {
        int64_t page = block_table[j];
        if (page < 0 || page >= c->num_pages) return 1;
        for (int h = 0; h < H; ++h) {
            for (int which = 0; which < 2; ++which) {           /* K codes, then V codes */
                uint8_t *codes = which ? c->v_codes : c->k_codes;
                for (int off = 0; off < P; ++off)
                    for (size_t b = 0; b < rowb; ++b) {
                        uint8_t *cell = &codes[row_index(c, page, h, off) * rowb + b];
                        if (dir == 0) packed[pos] = *cell; else *cell = packed[pos];
                        ++pos;
                    }
            }
            for (int which = 0; which < 2; ++which) {           /* K meta, then V meta: (scale, zero) pairs of fp16 */
                uint16_t *meta = which ? c->v_meta : c->k_meta;
                for (int off = 0; off < P; ++off)
                    for (size_t e = 0; e < ng * 2; ++e) {
                        uint16_t *cell = &meta[row_index(c, page, h, off) * ng * 2 + e];
                        if (dir == 0) { packed[pos] = (uint8_t)(*cell & 0xff); packed[pos + 1] = (uint8_t)(*cell >> 8); }
                        else *cell = (uint16_t)(packed[pos] | ((uint16_t)packed[pos + 1] << 8));
                        pos += 2;
                    }
            }
        }
    }
    return 0;
}

int oracle_kv_swap_out(const oracle_cache *c, const int32_t *block_table, int32_t num_tokens, uint8_t *packed)
{
    return swap_walk((oracle_cache *)c, block_table, num_tokens, packed, 0);
}

int oracle_kv_swap_in(oracle_cache *c, const int32_t *block_table, int32_t num_tokens, const uint8_t *packed)
{
    return swap_walk(c, block_table, num_tokens, (uint8_t *)packed, 1);
}

/* ---------------------------------------------------------------- fused LayerNorm and ReLU (R19, R20) */

/* binary64 -> binary16, round to nearest, ties to even, in one rounding. */
uint16_t oracle_d2h_rne(double d)
{
    uint16_t sign = (uint16_t)(signbit(d) ? 0x8000u : 0u);
    if (isnan(d)) return (uint16_t)(sign | 0x7e00u);
    double a = fabs(d);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);
    int ulp_exp = e - 11;
    if (ulp_exp < -24) ulp_exp = -24;
    double r = nearbyint(ldexp(a, -ulp_exp));       /* the scaling is exact; ties to even */
    double val = ldexp(r, ulp_exp);
    if (val == 0.0) return sign;
    if (val < ldexp(1.0, -14)) return (uint16_t)(sign | (uint32_t)ldexp(val, 24));
    int e2;
    double m2 = frexp(val, &e2);
    return (uint16_t)(sign | ((uint32_t)(e2 - 1 + 15) << 10) | ((uint32_t)ldexp(m2, 11) - 0x400u));
}

/*
 * Residual add + LayerNorm over the rows of a [rows, hidden] matrix (R19).
 * residual may be NULL (h = x).  h_out: fp16 bit patterns [rows, hidden]; y_out: fp64.
 */
int oracle_add_layernorm(const uint16_t *x, const uint16_t *residual, const uint16_t *gamma, const uint16_t *beta,
                         double eps, int64_t rows, int32_t hidden, uint16_t *h_out, double *y_out)
{
    if (rows < 0 || hidden <= 0) return -1;
    for (int64_t i = 0; i < rows; ++i) {
        const uint16_t *xr = x + i * hidden;
        uint16_t *hr = h_out + i * hidden;
        double *yr = y_out + i * hidden;
        for (int j = 0; j < hidden; ++j) {
            double sum = (double)oracle_h2f(xr[j]);
            if (residual) sum += (double)oracle_h2f(residual[i * hidden + j]);    /* exact in binary64 */
            hr[j] = oracle_d2h_rne(sum);
        }
        double mean = 0.0;
        for (int j = 0; j < hidden; ++j) mean += (double)oracle_h2f(hr[j]);
        mean /= hidden;
        double var = 0.0;
        for (int j = 0; j < hidden; ++j) {
            const double dlt = (double)oracle_h2f(hr[j]) - mean;
            var += dlt * dlt;
        }
        var /= hidden;
        const double denom = sqrt(var + eps);
        for (int j = 0; j < hidden; ++j)
            yr[j] = (double)oracle_h2f(gamma[j]) * (((double)oracle_h2f(hr[j]) - mean) / denom) + (double)oracle_h2f(beta[j]);
    }
    return 0;
}

/* Bias + ReLU over a [rows, cols] matrix (R20).  bias may be NULL. */
int oracle_bias_relu(const uint16_t *x, const uint16_t *bias, int64_t rows, int32_t cols, uint16_t *y_out)
{
    if (rows < 0 || cols <= 0) return -1;
    for (int64_t i = 0; i < rows; ++i)
        for (int j = 0; j < cols; ++j) {
            double v = (double)oracle_h2f(x[i * cols + j]);
            if (bias) v += (double)oracle_h2f(bias[j]);
            y_out[i * cols + j] = v > 0.0 ? oracle_d2h_rne(v) : (uint16_t)0;
        }
    return 0;
}
