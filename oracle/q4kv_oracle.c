/*
 * q4kv_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, scalar CPU statement of what the Q4 KV-cache hot path computes.
 * It exists so that the GPU library can be checked against something written
 * independently from the paper.  Only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg may call it.  It shares no code, header, table
 * or helper with the GPU library.
 *
 * What it follows:
 *   - Sec. 3.2 "Q4 Quantization Pipeline": 4-bit codes packed into uint32 words
 *     plus one 16-bit scale and one 16-bit bias per group of g = 64 elements;
 *     K+V bytes per layer = h*d*n*(1 + 8/g).
 *   - Sec. 3.4 "Batched Quantized Inference": append new K/V to each agent's
 *     cache, then attention over every agent of the batch (update_and_fetch);
 *     the left padding of merge/extract is replaced by ragged lengths, so no
 *     padded key exists.
 *   - Sec. 3.6 "Architectural Coverage": GQA, query head h reads KV head
 *     floor(h / n_rep); causal masks for chunked prefill; sliding windows;
 *     asymmetric K/V widths (v_head_dim).
 *   - Sec. 3.1 "Block Pool": fixed blocks of 256 tokens, one list per agent.
 *
 * The paper delegates the quantizer's arithmetic to its framework; the reading
 * used here (fixed by the project brief) is, per group of 64 along head_dim:
 *   bias = min, scale = (max - min)/15 computed in binary32, both stored as
 *   binary16 (round to nearest even); code = clamp(rint((x - min)/scale_stored),
 *   0, 15) with a true binary32 division and ties-to-even; element d of a row
 *   sits in word d/8, bits 4*(d%8) .. 4*(d%8)+3.
 * Sec. 3.1, Sec. 3.2 and the appendix "safetensors Q4 Format" name bfloat16 as the
 * type of scale and bias for one model family and binary16 for another.  The
 * bfloat16 form (param_format 1) is read as the same formula with both parameters
 * rounded to bfloat16 (nearest even) and the codes taken against the STORED
 * parameters: code = clamp(rint((x - bias_stored)/scale_stored), 0, 15).  The
 * stored bias is then no longer exactly the minimum, so x - bias_stored may be
 * slightly negative (code 0) and the top of the range may clamp at 15.
 *
 * Attention reaches exactly (up to rounding order) softmax(sm * q K^T) V on the
 * dequantized values, so it is written as that definition in binary64.
 *
 * Parity pins: tests/test_oracle_pins.py (closed forms, golden byte counts from
 * the paper, round-trip bound, library softmax-attention, brute force, paging
 * and batching invariants).  Every function below is covered by at least one.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC
 * (no -ffast-math: binary32 division and rounding must stay IEEE).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_GROUP 64

/* ---------------------------------------------------------------- binary16 */

/* binary16 bits -> binary32 value, exact. */
float oracle_h2f(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    float v;
    if (e == 0)
        v = ldexpf((float)m, -24);                 /* zero / subnormal */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexpf((float)(m + 1024), e - 25);     /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* binary64 value -> binary16 bits, round to nearest, ties to even.
 * Works on the exact value, so it also serves binary32 inputs. */
uint16_t oracle_d2h(double d)
{
    uint16_t sign = signbit(d) ? 0x8000u : 0;
    double a = fabs(d);
    if (isnan(d)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);      /* rounds to inf */
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);                   /* a = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;                        /* a in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;                  /* subnormal range shares 2^-24 spacing */
    /* spacing of binary16 numbers around a is 2^(e-10) */
    double scaled = ldexp(a, 10 - e);      /* exact */
    double r = nearbyint(scaled);          /* default mode: ties to even */
    /* r in [0, 2048]; r == 2048 means carry into the next binade */
    int biased;
    int mant;
    if (r >= 2048.0) { e += 1; r = 1024.0; }
    if (r < 1024.0) { biased = 0; mant = (int)r; }          /* subnormal or zero */
    else { biased = e + 15; mant = (int)r - 1024; }
    if (biased >= 31) return (uint16_t)(sign | 0x7c00u);
    return (uint16_t)(sign | (biased << 10) | mant);
}

uint16_t oracle_f2h(float f) { return oracle_d2h((double)f); }

/* ---------------------------------------------------------------- bfloat16 */

/* bfloat16 = sign, 8 exponent bits (bias 127), 7 fraction bits: the value of the bits. */
float oracle_bf2f(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xff;
    int m = h & 0x7f;
    float v;
    if (e == 0)
        v = ldexpf((float)m, -133);                /* zero / subnormal: m * 2^-7 * 2^-126 */
    else if (e == 255)
        v = m ? NAN : INFINITY;
    else
        v = ldexpf((float)(m + 128), e - 134);     /* (1 + m/128) * 2^(e-127) */
    return sign ? -v : v;
}

/* binary32 value -> bfloat16 bits, round to nearest, ties to even (arithmetic on the
 * value, not on the bit pattern). */
uint16_t oracle_f2bf(float f)
{
    uint16_t sign = signbit(f) ? 0x8000u : 0;
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7fc0u);
    if (isinf(f)) return (uint16_t)(sign | 0x7f80u);
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);
    int e = ex - 1;                        /* a in [2^e, 2^(e+1)) */
    if (e < -126) e = -126;                /* subnormals share the spacing 2^-133 */
    double scaled = ldexp(a, 7 - e);       /* exact; spacing of bfloat16 around a is 2^(e-7) */
    double r = nearbyint(scaled);          /* ties to even */
    if (r >= 256.0) { e += 1; r = 128.0; }
    int biased, mant;
    if (r < 128.0) { biased = 0; mant = (int)r; }
    else { biased = e + 127; mant = (int)r - 128; }
    if (biased >= 255) return (uint16_t)(sign | 0x7f80u);
    return (uint16_t)(sign | (biased << 7) | mant);
}

/* stored parameter bits -> value, by format (0: binary16, 1: bfloat16) */
static float param_value(uint16_t bits, int fmt) { return fmt ? oracle_bf2f(bits) : oracle_h2f(bits); }

/* ---------------------------------------------------------------- byte counts */

/* Sec. 3.2: FP16 K+V bytes of one layer = 4*h*d*n when K and V are d wide; written
 * here for separate widths: 2 bytes * h * (dk + dv) * n. */
int64_t oracle_fp16_layer_bytes(int64_t kv_heads, int64_t k_dim, int64_t v_dim, int64_t tokens)
{
    return 2 * kv_heads * (k_dim + v_dim) * tokens;
}

/* Sec. 3.2: Q4 K+V bytes of one layer = h*d*n*(1 + 8/g) for dk = dv = d: half a byte
 * per element plus a 2-byte scale and a 2-byte bias per group of g. */
int64_t oracle_q4_layer_bytes(int64_t kv_heads, int64_t k_dim, int64_t v_dim, int64_t tokens)
{
    int64_t elems = kv_heads * (k_dim + v_dim) * tokens;
    return elems / 2 + 4 * (elems / ORACLE_GROUP);
}

/* ---------------------------------------------------------------- quantize */

/* One row of `dim` binary16 values -> dim/8 words, dim/64 scales, dim/64 biases.
 * fmt 0: parameters stored as binary16 (the bias is then exactly the minimum);
 * fmt 1: stored as bfloat16, codes taken against the stored values. */
static void quantize_row(const uint16_t *x, int dim, int fmt, uint32_t *codes, uint16_t *scale, uint16_t *bias)
{
    for (int g = 0; g < dim / ORACLE_GROUP; ++g) {
        const uint16_t *xg = x + g * ORACLE_GROUP;
        float mn = oracle_h2f(xg[0]), mx = mn;
        uint16_t mn_bits = xg[0];
        for (int i = 1; i < ORACLE_GROUP; ++i) {
            float v = oracle_h2f(xg[i]);
            if (v < mn) { mn = v; mn_bits = xg[i]; }   /* first minimal element keeps its bits */
            if (v > mx) mx = v;
        }
        volatile float range = mx - mn;                /* binary32 */
        volatile float scale32 = range / 15.0f;        /* binary32 division */
        uint16_t sh = fmt ? oracle_f2bf(scale32) : oracle_f2h(scale32);
        float s = param_value(sh, fmt);
        scale[g] = sh;
        bias[g] = fmt ? oracle_f2bf(mn) : mn_bits;
        float b = fmt ? oracle_bf2f(bias[g]) : mn;      /* what the decoder will add back */
        for (int w = 0; w < ORACLE_GROUP / 8; ++w) {
            uint32_t word = 0;
            for (int j = 0; j < 8; ++j) {
                uint32_t c = 0;
                if (s != 0.0f) {
                    volatile float diff = oracle_h2f(xg[8 * w + j]) - b;
                    volatile float ratio = diff / s;   /* binary32 division */
                    float r = nearbyintf(ratio);       /* ties to even */
                    if (r < 0.0f) r = 0.0f;
                    if (r > 15.0f) r = 15.0f;
                    c = (uint32_t)r;
                }
                word |= c << (4 * j);
            }
            codes[g * (ORACLE_GROUP / 8) + w] = word;
        }
    }
}

/* x: [rows][dim] binary16 bits.  codes: [rows][dim/8], scale/bias: [rows][dim/64].
 * Returns 0, or -1 on a bad argument. */
int oracle_q4_quantize_fmt(const uint16_t *x, int64_t rows, int dim, int fmt, uint32_t *codes, uint16_t *scale,
                           uint16_t *bias)
{
    if (dim <= 0 || dim % ORACLE_GROUP || rows < 0 || (fmt != 0 && fmt != 1)) return -1;
    int G = dim / ORACLE_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        quantize_row(x + r * dim, dim, fmt, codes + r * (dim / 8), scale + r * G, bias + r * G);
    return 0;
}

int oracle_q4_quantize(const uint16_t *x, int64_t rows, int dim, uint32_t *codes, uint16_t *scale,
                       uint16_t *bias)
{
    return oracle_q4_quantize_fmt(x, rows, dim, 0, codes, scale, bias);
}

/* ---------------------------------------------------------------- dequantize */

static inline uint32_t code_at(const uint32_t *codes, int d) { return (codes[d >> 3] >> (4 * (d & 7))) & 0xfu; }

/* x_hat = code * scale + bias in binary32 (the product is exact), rounded to binary16. */
int oracle_q4_dequantize_fmt(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows,
                             int dim, int fmt, uint16_t *x)
{
    if (dim <= 0 || dim % ORACLE_GROUP || rows < 0 || (fmt != 0 && fmt != 1)) return -1;
    int G = dim / ORACLE_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int d = 0; d < dim; ++d) {
            float s = param_value(scale[r * G + d / ORACLE_GROUP], fmt);
            float b = param_value(bias[r * G + d / ORACLE_GROUP], fmt);
            volatile float prod = (float)code_at(codes + r * (dim / 8), d) * s;
            volatile float v = prod + b;
            x[r * dim + d] = oracle_f2h(v);
        }
    return 0;
}

int oracle_q4_dequantize(const uint32_t *codes, const uint16_t *scale, const uint16_t *bias, int64_t rows,
                         int dim, uint16_t *x)
{
    return oracle_q4_dequantize_fmt(codes, scale, bias, rows, dim, 0, x);
}

/* ---------------------------------------------------------------- paged cache */

typedef struct {
    int32_t num_layers, num_q_heads, num_kv_heads;
    int32_t k_dim, v_dim;
    int32_t v_aliases_k;   /* 1: V row = first v_dim elements of the K row (shared latent) */
    int32_t block_tokens;  /* 256 */
    int32_t group_size;    /* 64 */
    int32_t param_format;  /* type of the stored scale and bias: 0 binary16, 1 bfloat16 */
} oracle_spec;

typedef struct {           /* [num_layers][num_blocks][kv_heads][block_tokens][dim/8 | dim/64] */
    uint32_t *codes;
    uint16_t *scale;
    uint16_t *bias;
    int32_t num_blocks;
} oracle_pool;

/* index of the row (layer, block, head, slot) in a pool */
static int64_t pool_row(const oracle_spec *sp, const oracle_pool *p, int layer, int block, int head, int slot)
{
    return (((int64_t)layer * p->num_blocks + block) * sp->num_kv_heads + head) * sp->block_tokens + slot;
}

/* unrounded dequantized element d of a pool row, exact in binary64 */
static double pool_value(const oracle_pool *p, int fmt, int64_t row, int dim, int d)
{
    int G = dim / ORACLE_GROUP;
    double s = (double)param_value(p->scale[row * G + d / ORACLE_GROUP], fmt);
    double b = (double)param_value(p->bias[row * G + d / ORACLE_GROUP], fmt);
    return (double)code_at(p->codes + row * (dim / 8), d) * s + b;
}

static int spec_ok(const oracle_spec *sp)
{
    return sp && sp->num_layers > 0 && sp->num_kv_heads > 0 && sp->num_q_heads > 0 &&
           sp->num_q_heads % sp->num_kv_heads == 0 && sp->group_size == ORACLE_GROUP && sp->k_dim > 0 &&
           sp->v_dim > 0 && sp->k_dim % ORACLE_GROUP == 0 && sp->v_dim % ORACLE_GROUP == 0 &&
           sp->block_tokens > 0 && (!sp->v_aliases_k || sp->v_dim <= sp->k_dim) &&
           (sp->param_format == 0 || sp->param_format == 1);
}

/* Sec. 3.4 update_and_fetch, first half: quantize each new token's K and V rows and
 * store them at tokens seq_len_before[a] .. +chunk_len-1 of agent a.
 * k_new / v_new: [layer_end-layer_begin][A][chunk_len][kv_heads][dim] binary16 bits.
 * v pool / v_new are ignored when v_aliases_k. */
int oracle_append(const oracle_spec *sp, oracle_pool *k, oracle_pool *v, const uint16_t *k_new,
                  const uint16_t *v_new, const int32_t *block_table, int max_blocks,
                  const int32_t *seq_len_before, int num_agents, int chunk_len, int layer_begin, int layer_end)
{
    if (!spec_ok(sp) || layer_begin < 0 || layer_end > sp->num_layers || layer_begin > layer_end) return -1;
    int H = sp->num_kv_heads, B = sp->block_tokens;
    for (int l = layer_begin; l < layer_end; ++l)
        for (int a = 0; a < num_agents; ++a)
            for (int c = 0; c < chunk_len; ++c) {
                int t = seq_len_before[a] + c;
                if (t / B >= max_blocks) return -2;
                int blk = block_table[a * max_blocks + t / B];
                if (blk < 0 || blk >= k->num_blocks) return -3;
                for (int h = 0; h < H; ++h) {
                    int64_t src = ((((int64_t)(l - layer_begin) * num_agents + a) * chunk_len + c) * H + h);
                    int64_t row = pool_row(sp, k, l, blk, h, t % B);
                    quantize_row(k_new + src * sp->k_dim, sp->k_dim, sp->param_format, k->codes + row * (sp->k_dim / 8),
                                 k->scale + row * (sp->k_dim / ORACLE_GROUP),
                                 k->bias + row * (sp->k_dim / ORACLE_GROUP));
                    if (!sp->v_aliases_k) {
                        row = pool_row(sp, v, l, blk, h, t % B);
                        quantize_row(v_new + src * sp->v_dim, sp->v_dim, sp->param_format, v->codes + row * (sp->v_dim / 8),
                                     v->scale + row * (sp->v_dim / ORACLE_GROUP),
                                     v->bias + row * (sp->v_dim / ORACLE_GROUP));
                    }
                }
            }
    return 0;
}

/* One (layer, agent, query row, query head) unit of attention, binary64 throughout.
 * q_row: k_dim binary16 bits.  out_d: v_dim doubles.  vis = number of visible keys
 * (tokens 0..vis-1); window > 0 additionally hides tokens t <= (vis-1) - window. */
static int attention_unit(const oracle_spec *sp, const oracle_pool *k, const oracle_pool *v, int layer,
                          const int32_t *table_row, int kv_head, const uint16_t *q_row, int vis, int window,
                          double sm_scale, double *out_d, double *z /* scratch, >= vis */)
{
    int B = sp->block_tokens;
    const oracle_pool *vp = sp->v_aliases_k ? k : v;
    int v_row_dim = sp->v_aliases_k ? sp->k_dim : sp->v_dim;
    for (int e = 0; e < sp->v_dim; ++e) out_d[e] = 0.0;
    int first = 0;
    if (window > 0 && vis - window > 0) first = vis - window;
    for (int t = 0; t < first; ++t) z[t] = 0.0;         /* outside the window: weight 0 */
    if (vis <= first) return 0;                         /* no visible key: zeros */
    double zmax = -INFINITY;
    for (int t = first; t < vis; ++t) {
        int blk = table_row[t / B];
        if (blk < 0 || blk >= k->num_blocks) return -3;
        int64_t row = pool_row(sp, k, layer, blk, kv_head, t % B);
        double acc = 0.0;
        for (int d = 0; d < sp->k_dim; ++d) acc += (double)oracle_h2f(q_row[d]) * pool_value(k, sp->param_format, row, sp->k_dim, d);
        z[t] = sm_scale * acc;
        if (z[t] > zmax) zmax = z[t];
    }
    double denom = 0.0;
    for (int t = first; t < vis; ++t) {
        z[t] = exp(z[t] - zmax);
        denom += z[t];
    }
    for (int t = first; t < vis; ++t) {
        z[t] /= denom;                                  /* softmax weight p_t, left in z for the caller */
        int blk = table_row[t / B];
        int64_t row = pool_row(sp, vp, layer, blk, kv_head, t % B);
        for (int e = 0; e < sp->v_dim; ++e) out_d[e] += z[t] * pool_value(vp, sp->param_format, row, v_row_dim, e);
    }
    return 0;
}

/* Sec. 3.4 update_and_fetch, second half, and Sec. 3.6 (GQA grouping, causal chunk mask).
 * q:   [layer_end-layer_begin][A][q_len][q_heads][k_dim] binary16 bits
 * out: same leading shape with v_dim, binary16 bits; out_d (may be NULL) the same in binary64.
 * seq_len[a] = keys visible to the LAST query row of agent a; row r sees
 * seq_len[a] - (q_len-1-r) keys.  window <= 0: global.  window_per_layer (may be NULL)
 * overrides `window` per absolute layer index.
 * Returns 0 or a negative code; *threads_used (may be NULL) gets the OpenMP team size. */
int oracle_attention(const oracle_spec *sp, const oracle_pool *k, const oracle_pool *v, const uint16_t *q,
                     uint16_t *out, double *out_d, const int32_t *block_table, int max_blocks,
                     const int32_t *seq_len, int num_agents, int q_len, float sm_scale, int window,
                     const int32_t *window_per_layer, int layer_begin, int layer_end, int *threads_used)
{
    if (!spec_ok(sp) || layer_begin < 0 || layer_end > sp->num_layers || layer_begin > layer_end || q_len < 1)
        return -1;
    int Hq = sp->num_q_heads, n_rep = sp->num_q_heads / sp->num_kv_heads;
    int max_len = 0;
    for (int a = 0; a < num_agents; ++a) {
        if (seq_len[a] < 0 || seq_len[a] > max_blocks * sp->block_tokens) return -2;
        if (seq_len[a] > max_len) max_len = seq_len[a];
    }
    int64_t units = (int64_t)(layer_end - layer_begin) * num_agents * q_len * Hq;
    int status = 0, team = 1;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        team = omp_get_num_threads();
#endif
        double *z = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        double *o = (double *)malloc(sizeof(double) * (size_t)sp->v_dim);
#pragma omp for schedule(dynamic, 1)
        for (int64_t u = 0; u < units; ++u) {
            int h = (int)(u % Hq);
            int r = (int)((u / Hq) % q_len);
            int a = (int)((u / ((int64_t)Hq * q_len)) % num_agents);
            int li = (int)(u / ((int64_t)Hq * q_len * num_agents));
            int layer = layer_begin + li;
            int vis = seq_len[a] - (q_len - 1 - r);
            if (vis < 0) vis = 0;
            int w = window_per_layer ? window_per_layer[layer] : window;
            int rc = attention_unit(sp, k, v, layer, block_table + (int64_t)a * max_blocks, h / n_rep,
                                    q + u * sp->k_dim, vis, w, (double)sm_scale, o, z);
            if (rc) {
#pragma omp atomic write
                status = rc;
            }
            for (int e = 0; e < sp->v_dim; ++e) {
                out[u * sp->v_dim + e] = oracle_d2h(o[e]);
                if (out_d) out_d[u * sp->v_dim + e] = o[e];
            }
        }
        free(z);
        free(o);
    }
    if (threads_used) *threads_used = team;
    return status;
}

/* Softmax weights of one unit and its binary64 output, for the "rows sum to one" pin:
 * p[t] for t < vis (zero outside the window), out_d[v_dim]. */
int oracle_attention_probs(const oracle_spec *sp, const oracle_pool *k, const oracle_pool *v, int layer,
                           const int32_t *table_row, int kv_head, const uint16_t *q_row, int vis, int window,
                           float sm_scale, double *p, double *out_d)
{
    if (!spec_ok(sp)) return -1;
    return attention_unit(sp, k, v, layer, table_row, kv_head, q_row, vis, window, (double)sm_scale, out_d, p);
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
