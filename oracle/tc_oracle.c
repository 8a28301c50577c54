/*
 * CPU oracle for the mixed-batch paged-attention path.  TEST INFRASTRUCTURE ONLY:
 * the tests, the smoke check and the bench's cpu_baseline leg may call it; the
 * product path never does.  It shares no code with the GPU library.
 *
 * What it computes is the plain definition, in fp64, with nothing tiled, fused,
 * split or re-ordered:
 *   - the KV cache keeps the key and value vectors of every token already
 *     processed (paper Sec. 2.1, "Transformer Architecture"), here in a paged
 *     pool addressed through per-sequence block tables (Sec. 3.5, paged memory);
 *   - a query token at absolute position p attends over tokens 0..p of its own
 *     sequence with scaled dot-product attention (Sec. 2.1); a prefill chunk at
 *     chunk offset ctx holds positions ctx..ctx+q_len-1 (Sec. 2.2, chunked
 *     prefill), a decode is the one-token case (Sec. 2.1, "Two-Phase Inference");
 *   - query head h reads KV head h / (Hq/Hkv) (grouped-query attention, cited in
 *     Sec. 2.2).
 *
 * Tensors are bf16 (or, with dtype = 2, IEEE half) bit patterns (uint16_t) widened exactly to double.
 *
 * Pool layout (an interface shared with the GPU library by specification only;
 * B = block_size tokens per block, D = head_dim):
 *   K pool  [num_blocks][Hkv][D/8][B][8]   element (blk,h,tok,d) ->
 *           (((blk*Hkv + h)*(D/8) + d/8)*B + tok)*8 + d%8
 *   V pool  [num_blocks][Hkv][D][B]        element (blk,h,tok,d) ->
 *           ((blk*Hkv + h)*D + d)*B + slot(tok),  slot(tok) = tok with bits 2 and 3
 *           exchanged (a row holds tokens 0-3, 8-11, 4-7, 12-15 in that order)
 * Token j of sequence s lives in block table[s][j / B] at token index j % B.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (brute force, closed forms, a library routine, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int Hq, Hkv, D, B;
    int64_t num_blocks;
} shape_t;

#define TCO_BF16 1
#define TCO_FP16 2

/* bf16: the upper half of an IEEE single */
static double widen_bf16(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* IEEE half: 1 sign, 5 exponent (bias 15), 10 fraction bits; the precision the paper's runs used (Sec. 4.1) */
static double widen_fp16(uint16_t bits)
{
    int sign = bits >> 15, e = (bits >> 10) & 31, m = bits & 1023;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* zero and subnormals */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

static double widen_as(uint16_t bits, int dtype) { return dtype == TCO_FP16 ? widen_fp16(bits) : widen_bf16(bits); }

double tco_widen(uint16_t bits, int dtype) { return widen_as(bits, dtype); }

static int64_t k_index(const shape_t *sh, int64_t blk, int h, int tok, int d)
{
    return (((blk * sh->Hkv + h) * (sh->D / 8) + d / 8) * sh->B + tok) * 8 + d % 8;
}

static int64_t v_index(const shape_t *sh, int64_t blk, int h, int tok, int d)
{
    int slot = (tok & ~12) | ((tok & 4) << 1) | ((tok & 8) >> 1);
    return ((blk * sh->Hkv + h) * sh->D + d) * sh->B + slot;
}

int tco_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void tco_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* 0 if every page the batch touches has a block id inside the pool, else -1. */
static int check_tables(const shape_t *sh, int S, const int32_t *q_start, const int32_t *ctx_len,
                        const int32_t *table, int max_blocks)
{
    for (int s = 0; s < S; s++) {
        int64_t kv = (int64_t)ctx_len[s] + (q_start[s + 1] - q_start[s]);
        int64_t pages = (kv + sh->B - 1) / sh->B;
        if (ctx_len[s] < 0 || q_start[s + 1] < q_start[s] || pages > max_blocks) return -1;
        for (int64_t b = 0; b < pages; b++) {
            int32_t id = table[(int64_t)s * max_blocks + b];
            if (id < 0 || id >= sh->num_blocks) return -1;
        }
    }
    return 0;
}

/* Store this iteration's K and V rows into the paged pool (Sec. 2.1: K and V are cached). */
int tco_kv_append(int Hkv, int D, int B, int64_t num_blocks, uint16_t *k_pool, uint16_t *v_pool,
                  int S, const int32_t *q_start, const int32_t *ctx_len, const int32_t *table,
                  int max_blocks, const uint16_t *k_new, const uint16_t *v_new)
{
    shape_t sh = {0, Hkv, D, B, num_blocks};
    if (check_tables(&sh, S, q_start, ctx_len, table, max_blocks)) return -1;
    for (int s = 0; s < S; s++) {
        int q_len = q_start[s + 1] - q_start[s];
        for (int i = 0; i < q_len; i++) {
            int64_t pos = (int64_t)ctx_len[s] + i;
            int64_t blk = table[(int64_t)s * max_blocks + pos / B];
            int tok = (int)(pos % B);
            int64_t row = (int64_t)q_start[s] + i;
            for (int h = 0; h < Hkv; h++)
                for (int d = 0; d < D; d++) {
                    k_pool[k_index(&sh, blk, h, tok, d)] = k_new[(row * Hkv + h) * D + d];
                    v_pool[v_index(&sh, blk, h, tok, d)] = v_new[(row * Hkv + h) * D + d];
                }
        }
    }
    return 0;
}

/* Read tokens 0..kv_len-1 of one sequence back out of the pool, un-paged: [kv_len][Hkv][D]. */
int tco_kv_gather(int Hkv, int D, int B, int64_t num_blocks, const uint16_t *k_pool,
                  const uint16_t *v_pool, const int32_t *table_row, int64_t kv_len, uint16_t *k_out,
                  uint16_t *v_out)
{
    shape_t sh = {0, Hkv, D, B, num_blocks};
    for (int64_t j = 0; j < kv_len; j++) {
        int64_t blk = table_row[j / B];
        if (blk < 0 || blk >= num_blocks) return -1;
        int tok = (int)(j % B);
        for (int h = 0; h < Hkv; h++)
            for (int d = 0; d < D; d++) {
                k_out[(j * Hkv + h) * D + d] = k_pool[k_index(&sh, blk, h, tok, d)];
                v_out[(j * Hkv + h) * D + d] = v_pool[v_index(&sh, blk, h, tok, d)];
            }
    }
    return 0;
}

/*
 * KV migration (Sec. 3.5: a request's KV cache moves between instances and is stored into the
 * receiver's paged memory).  The transfer buffer is [L][P][2][Hkv*B*D]: per layer and page the K
 * block, then the V block, each in the pool's block layout.  One call handles one sequence whose
 * pages start at page index page0 of the P pages of the buffer.
 * Export copies tokens 0..kv_len-1 and writes zero into the token slots of the last page that are
 * at or beyond kv_len.
 */
int tco_kv_export(int Hkv, int D, int B, int64_t num_blocks, int L, const uint16_t *const *k_pools,
                  const uint16_t *const *v_pools, const int32_t *table_row, int64_t kv_len, int64_t page0,
                  int64_t P, uint16_t *buf)
{
    shape_t sh = {0, Hkv, D, B, num_blocks};
    int64_t E = (int64_t)Hkv * B * D; /* elements of one block of one pool */
    int64_t pages = (kv_len + B - 1) / B;
    for (int l = 0; l < L; l++)
        for (int64_t j = 0; j < pages * B; j++) {
            int64_t blk = table_row[j / B];
            if (blk < 0 || blk >= num_blocks) return -1;
            int tok = (int)(j % B);
            uint16_t *kdst = buf + ((l * P + page0 + j / B) * 2 + 0) * E;
            uint16_t *vdst = buf + ((l * P + page0 + j / B) * 2 + 1) * E;
            for (int h = 0; h < Hkv; h++)
                for (int d = 0; d < D; d++) {
                    int real = j < kv_len;
                    kdst[k_index(&sh, 0, h, tok, d)] = real ? k_pools[l][k_index(&sh, blk, h, tok, d)] : 0;
                    vdst[v_index(&sh, 0, h, tok, d)] = real ? v_pools[l][v_index(&sh, blk, h, tok, d)] : 0;
                }
        }
    return 0;
}

/* Import stores tokens 0..kv_len-1 of the buffer into the blocks of table_row; nothing else is written. */
int tco_kv_import(int Hkv, int D, int B, int64_t num_blocks, int L, uint16_t *const *k_pools,
                  uint16_t *const *v_pools, const int32_t *table_row, int64_t kv_len, int64_t page0, int64_t P,
                  const uint16_t *buf)
{
    shape_t sh = {0, Hkv, D, B, num_blocks};
    int64_t E = (int64_t)Hkv * B * D;
    for (int l = 0; l < L; l++)
        for (int64_t j = 0; j < kv_len; j++) {
            int64_t blk = table_row[j / B];
            if (blk < 0 || blk >= num_blocks) return -1;
            int tok = (int)(j % B);
            const uint16_t *ksrc = buf + ((l * P + page0 + j / B) * 2 + 0) * E;
            const uint16_t *vsrc = buf + ((l * P + page0 + j / B) * 2 + 1) * E;
            for (int h = 0; h < Hkv; h++)
                for (int d = 0; d < D; d++) {
                    k_pools[l][k_index(&sh, blk, h, tok, d)] = ksrc[k_index(&sh, 0, h, tok, d)];
                    v_pools[l][v_index(&sh, blk, h, tok, d)] = vsrc[v_index(&sh, 0, h, tok, d)];
                }
        }
    return 0;
}

/*
 * Attention for selected packed query rows (rows == NULL: all of them), every head.
 * out is double [n_rows][Hq][D].  Reads the pool as it stands, i.e. after the append.
 *   s_j = scale * sum_d q_d k_{j,d}   (j = 0..p, the token itself included)
 *   m = max_j s_j ; e_j = exp(s_j - m) ; out_d = sum_j e_j v_{j,d} / sum_j e_j
 */
int tco_attention_dtype(int Hq, int Hkv, int D, int B, int64_t num_blocks, const uint16_t *k_pool,
                        const uint16_t *v_pool, int S, const int32_t *q_start, const int32_t *ctx_len,
                        const int32_t *table, int max_blocks, const uint16_t *q, double scale,
                        const int32_t *rows, int64_t n_rows, double *out, int dtype)
{
    shape_t sh = {Hq, Hkv, D, B, num_blocks};
    if (Hkv <= 0 || Hq % Hkv) return -2;
    if (check_tables(&sh, S, q_start, ctx_len, table, max_blocks)) return -1;
    int G = Hq / Hkv;
    int64_t T = q_start[S];
    if (!rows) n_rows = T;
    /* which sequence owns each packed row */
    int32_t *owner = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    if (!owner) return -3;
    for (int s = 0; s < S; s++)
        for (int t = q_start[s]; t < q_start[s + 1]; t++) owner[t] = s;
    int bad = 0;
    int64_t work = n_rows * Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < work; w++) {
        int64_t r = w / Hq;
        int h = (int)(w % Hq);
        int64_t t = rows ? rows[r] : r;
        if (t < 0 || t >= T) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        int s = owner[t];
        int64_t p = (int64_t)ctx_len[s] + (t - q_start[s]); /* absolute position of the query */
        int kvh = h / G;
        const int32_t *trow = table + (int64_t)s * max_blocks;
        double *score = (double *)malloc(sizeof(double) * (size_t)(p + 1));
        double *o = out + (r * Hq + h) * D;
        if (!score) {
#pragma omp atomic write
            bad = 2;
            continue;
        }
        const uint16_t *qv = q + (t * Hq + h) * D;
        double m = -INFINITY;
        for (int64_t j = 0; j <= p; j++) {
            int64_t blk = trow[j / B];
            int tok = (int)(j % B);
            double acc = 0.0;
            for (int d = 0; d < D; d++) acc += widen_as(qv[d], dtype) * widen_as(k_pool[k_index(&sh, blk, kvh, tok, d)], dtype);
            score[j] = scale * acc;
            if (score[j] > m) m = score[j];
        }
        double denom = 0.0;
        for (int d = 0; d < D; d++) o[d] = 0.0;
        for (int64_t j = 0; j <= p; j++) {
            int64_t blk = trow[j / B];
            int tok = (int)(j % B);
            double e = exp(score[j] - m);
            denom += e;
            for (int d = 0; d < D; d++) o[d] += e * widen_as(v_pool[v_index(&sh, blk, kvh, tok, d)], dtype);
        }
        for (int d = 0; d < D; d++) o[d] /= denom;
        free(score);
    }
    free(owner);
    return bad ? -3 : 0;
}

/* The bf16 case under its original name. */
int tco_attention(int Hq, int Hkv, int D, int B, int64_t num_blocks, const uint16_t *k_pool,
                  const uint16_t *v_pool, int S, const int32_t *q_start, const int32_t *ctx_len,
                  const int32_t *table, int max_blocks, const uint16_t *q, double scale,
                  const int32_t *rows, int64_t n_rows, double *out)
{
    return tco_attention_dtype(Hq, Hkv, D, B, num_blocks, k_pool, v_pool, S, q_start, ctx_len, table, max_blocks, q,
                               scale, rows, n_rows, out, TCO_BF16);
}
