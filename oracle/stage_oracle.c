/*
 * CPU ORACLE -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, double-precision statement of what one pipeline stage computes on a hybrid
 * batch of chunked-prefill and decode tokens.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the HIP library.
 *
 * What the paper fixes (arxiv 2504.14775):
 *   - section 2.1: a stage is a run of decoder layers, each a causally masked self-attention,
 *     a normalisation and an MLP;
 *   - section 2.2: prefill processes a prompt's tokens in parallel and fills the KV cache; a
 *     decode step attends the newest token to the stored KV cache; a long prompt may be
 *     computed in chunks over several iterations, mixed with decode tokens in one batch;
 *   - section 3 (opening) / 3.3: prefill and decode tokens are merged into a single batch; the KV cache
 *     is paged, with page tables shared by every stage, pages being assigned before the
 *     micro-batch runs;
 *   - section 4.1: bf16 weights and activations.
 * The paper gives no formula for the layer itself.  The arithmetic below is the public
 * Llama/Qwen decoder layer (pre-norm RMSNorm, rotate-half RoPE, grouped-query attention with
 * scale 1/sqrt(d), SwiGLU MLP, two residual adds), which is what the stage shapes name.
 *
 * Every result here has a plain definition (dense linear algebra and a softmax), so each
 * function is that definition written out.  All arithmetic is IEEE double.  bf16 appears only
 * where the data of the method is bf16: the given weights and input, the contents of the KV
 * pool (a later chunk or decode step can only see earlier K/V through the bf16 pool, so
 * attention always reads K and V back from the pool, including the rows written in this very
 * call), and the stage output.
 *
 * Pins (tests/test_oracle_*.py): brute-force softmax attention in numpy float64, chunked ==
 * unchunked (bitwise), decode row == last row of full causal attention (bitwise), physical
 * page permutation (bitwise), batch-composition independence (bitwise), closed forms for
 * RMSNorm / RoPE / one-key attention / zeroed projections, GQA vs duplicated-head MHA, GEMM
 * entries against numpy, slot placement against the closed form page*16 + offset.
 *
 * KV pool layout (an interface of the library, implemented here independently):
 *   K: [layer][page][kv_head][d/8][slot][8]  bf16   (8-element groups of the head vector)
 *   V: [layer][page][kv_head][d][slot]       bf16   (slot-contiguous)
 * with page_size slots per page.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t num_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, page_size;
    int32_t has_qkv_bias;
    double rms_eps, rope_theta;
    /* 0: the plain definition (the default everywhere).  1: diagnostic reading in which the tensors
     * that feed matrix products -- normalised activations, rotated queries, attention output, SwiGLU
     * output -- are rounded to bf16 where a bf16 model stores them (paper section 4.1: all models use
     * the bfloat16 data type); everything else stays double.  It separates the rounding noise of
     * bf16 operands from errors of any other kind. */
    int32_t round_operands;
    int32_t reserved;
} oracle_config;

/* bf16 matrices are row-major [out_features][in_features]; biases may be NULL */
typedef struct {
    const uint16_t *wq, *wk, *wv, *wo, *wgate, *wup, *wdown, *norm1, *norm2, *bq, *bk, *bv;
} oracle_layer;

/* ---------------------------------------------------------------- bf16 <-> double */
double oracle_bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* round-to-nearest-even straight from double: double -> float with round-to-odd (keeps a
 * sticky bit), then float -> bf16 RNE; the pair is a single correct rounding. */
uint16_t oracle_f64_to_bf16(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if (x != x) return 0x7FC0;
    if ((double)f != x && !isinf(f)) {
        if (fabs((double)f) > fabs(x)) u -= 1; /* truncate towards zero */
        u |= 1;                                /* sticky */
    }
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

void oracle_f64_to_bf16_array(int64_t n, const double *x, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_f64_to_bf16(x[i]);
}

/* x <- the bf16 value nearest to x (ties to even), kept as a double */
static void round_through_bf16(int64_t n, double *x)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) x[i] = oracle_bf16_to_f64(oracle_f64_to_bf16(x[i]));
}

/* ---------------------------------------------------------------- pool addressing */
static inline int64_t k_index(const oracle_config *c, int64_t num_pages, int layer, int64_t page,
                              int kvh, int slot, int dim)
{
    int64_t d = c->head_dim, ps = c->page_size;
    int64_t base = (((int64_t)layer * num_pages + page) * c->n_kv_heads + kvh) * ps * d;
    return base + ((int64_t)(dim / 8) * ps + slot) * 8 + dim % 8;
}

static inline int64_t v_index(const oracle_config *c, int64_t num_pages, int layer, int64_t page,
                              int kvh, int slot, int dim)
{
    int64_t d = c->head_dim, ps = c->page_size;
    int64_t base = (((int64_t)layer * num_pages + page) * c->n_kv_heads + kvh) * ps * d;
    return base + (int64_t)dim * ps + slot;
}

int64_t oracle_k_index(const oracle_config *c, int64_t num_pages, int layer, int64_t page, int kvh,
                       int slot, int dim)
{
    return k_index(c, num_pages, layer, page, kvh, slot, dim);
}

int64_t oracle_v_index(const oracle_config *c, int64_t num_pages, int layer, int64_t page, int kvh,
                       int slot, int dim)
{
    return v_index(c, num_pages, layer, page, kvh, slot, dim);
}

/* ---------------------------------------------------------------- RMSNorm
 * out[t][j] = x[t][j] / sqrt(mean_j x[t][j]^2 + eps) * gamma[j]                      */
void oracle_rmsnorm(int64_t T, int H, const double *x, const uint16_t *gamma, double eps,
                    double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *r = x + t * H;
        double ss = 0.0;
        for (int j = 0; j < H; ++j) ss += r[j] * r[j];
        double inv = 1.0 / sqrt(ss / (double)H + eps);
        for (int j = 0; j < H; ++j) out[t * H + j] = r[j] * inv * oracle_bf16_to_f64(gamma[j]);
    }
}

/* ---------------------------------------------------------------- linear layer
 * y[t][n] = bias[n] + sum_k x[t][k] * W[n][k], the sum taken in ascending k, every product and
 * every addition rounded separately (the file is compiled with -ffp-contract=off), so each
 * y[t][n] is the same sequence of IEEE operations whatever the loop nest around it: no output
 * depends on T or on any other row.  Two loop nests compute exactly that sequence:
 *   - few rows: for every n, walk W[n][:] once and form the dot product of each row with it;
 *   - many rows: the weight is first copied out as doubles with k as the slow index so that the
 *     innermost loop runs over n (which vectorises without reassociating any sum).            */
#define ORACLE_NCHUNK 512
#define ORACLE_FEW_ROWS 64

__attribute__((target_clones("default", "arch=haswell", "arch=skylake-avx512")))
static void axpy_rows(int K, int N, int n0, int n1, const double *xr, const double *wt, double *yr)
{
    for (int k = 0; k < K; ++k) {
        double a = xr[k];
        const double *w = wt + (int64_t)k * N;
        for (int n = n0; n < n1; ++n) yr[n] += a * w[n];
    }
}

void oracle_linear(int64_t T, int K, int N, const double *x, const uint16_t *W,
                   const uint16_t *bias, double *y)
{
    if (T <= ORACLE_FEW_ROWS) {
#pragma omp parallel for schedule(static)
        for (int n = 0; n < N; ++n) {
            const uint16_t *wr = W + (int64_t)n * K;
            for (int64_t t = 0; t < T; ++t) {
                const double *xr = x + t * K;
                double acc = bias ? oracle_bf16_to_f64(bias[n]) : 0.0;
                for (int k = 0; k < K; ++k) acc += xr[k] * oracle_bf16_to_f64(wr[k]);
                y[t * N + n] = acc;
            }
        }
        return;
    }
    double *wt = (double *)malloc((size_t)K * (size_t)N * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) wt[(int64_t)k * N + n] = oracle_bf16_to_f64(W[(int64_t)n * K + k]);
    int nchunks = (N + ORACLE_NCHUNK - 1) / ORACLE_NCHUNK;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t t = 0; t < T; ++t) {
        for (int cb = 0; cb < nchunks; ++cb) {
            int n0 = cb * ORACLE_NCHUNK, n1 = n0 + ORACLE_NCHUNK < N ? n0 + ORACLE_NCHUNK : N;
            double *yr = y + t * N;
            for (int n = n0; n < n1; ++n) yr[n] = bias ? oracle_bf16_to_f64(bias[n]) : 0.0;
            axpy_rows(K, N, n0, n1, x + t * K, wt, yr);
        }
    }
    free(wt);
}

/* ---------------------------------------------------------------- RoPE (rotate-half pairing)
 * For a head vector v of length d at position p, with theta_j = base^(-2j/d), j < d/2:
 *   v'[j]       = v[j] cos(p theta_j) - v[j+d/2] sin(p theta_j)
 *   v'[j+d/2]   = v[j+d/2] cos(p theta_j) + v[j] sin(p theta_j)
 * applied in place to n_heads consecutive head vectors of every row.                      */
void oracle_rope(int64_t T, int n_heads, int d, const int32_t *pos, double base, double *v)
{
    int half = d / 2;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int h = 0; h < n_heads; ++h) {
            double *r = v + ((int64_t)t * n_heads + h) * d;
            for (int j = 0; j < half; ++j) {
                double ang = (double)pos[t] * pow(base, -2.0 * (double)j / (double)d);
                double c = cos(ang), s = sin(ang);
                double a = r[j], b = r[j + half];
                r[j] = a * c - b * s;
                r[j + half] = b * c + a * s;
            }
        }
    }
}

/* ---------------------------------------------------------------- batch bookkeeping
 * Rows are packed in sequence order; token i of sequence s has position cached_len[s] + i.
 * Fills seq_of[t] and pos_of[t]; returns the number of rows.                               */
int64_t oracle_token_map(int S, const int32_t *new_tokens, const int32_t *cached_len,
                         int32_t *seq_of, int32_t *pos_of)
{
    int64_t t = 0;
    for (int s = 0; s < S; ++s)
        for (int i = 0; i < new_tokens[s]; ++i, ++t) {
            if (seq_of) seq_of[t] = s;
            if (pos_of) pos_of[t] = cached_len[s] + i;
        }
    return t;
}

/* ---------------------------------------------------------------- paged KV write
 * Position p of sequence s lives in page block_tables[s][p / page_size], slot p % page_size.
 * k and v are [T][n_kv][d] doubles; they are rounded to bf16 on the way in.                */
void oracle_kv_write(const oracle_config *c, int layer, int64_t T, const int32_t *seq_of,
                     const int32_t *pos_of, const int32_t *block_tables, int max_blocks_per_seq,
                     int64_t num_pages, const double *k, const double *v, uint16_t *k_pool,
                     uint16_t *v_pool)
{
    int d = c->head_dim, ps = c->page_size;
    for (int64_t t = 0; t < T; ++t) {
        int s = seq_of[t], p = pos_of[t];
        int64_t page = block_tables[(int64_t)s * max_blocks_per_seq + p / ps];
        int slot = p % ps;
        for (int h = 0; h < c->n_kv_heads; ++h)
            for (int j = 0; j < d; ++j) {
                int64_t src = ((int64_t)t * c->n_kv_heads + h) * d + j;
                k_pool[k_index(c, num_pages, layer, page, h, slot, j)] = oracle_f64_to_bf16(k[src]);
                v_pool[v_index(c, num_pages, layer, page, h, slot, j)] = oracle_f64_to_bf16(v[src]);
            }
    }
}

/* ---------------------------------------------------------------- ragged paged attention
 * For the row at position p of sequence s and query head hq (kv head hq / (n_q / n_kv)):
 *   score_j = (q . K_j) / sqrt(d)  for j = 0 .. p      (causal: nothing after p)
 *   w = softmax(score)  (subtract the maximum, exponentiate, divide by the sum)
 *   o = sum_j w_j V_j
 * K_j and V_j are read from the bf16 pool through the sequence's page table.
 * q, o: [T][n_q][d] doubles.                                                              */
void oracle_attention(const oracle_config *c, int layer, int64_t T, const int32_t *seq_of,
                      const int32_t *pos_of, const int32_t *block_tables, int max_blocks_per_seq,
                      int64_t num_pages, const double *q, const uint16_t *k_pool,
                      const uint16_t *v_pool, double *o)
{
    int d = c->head_dim, ps = c->page_size, g = c->n_q_heads / c->n_kv_heads;
    double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t t = 0; t < T; ++t) {
        for (int hq = 0; hq < c->n_q_heads; ++hq) {
            int s = seq_of[t], p = pos_of[t], kvh = hq / g;
            const int32_t *bt = block_tables + (int64_t)s * max_blocks_per_seq;
            const double *qr = q + ((int64_t)t * c->n_q_heads + hq) * d;
            double *orow = o + ((int64_t)t * c->n_q_heads + hq) * d;
            int n = p + 1;
            double *w = (double *)malloc((size_t)n * sizeof(double));
            double mx = -INFINITY;
            for (int j = 0; j < n; ++j) {
                double acc = 0.0;
                for (int e = 0; e < d; ++e)
                    acc += qr[e] * oracle_bf16_to_f64(
                                       k_pool[k_index(c, num_pages, layer, bt[j / ps], kvh, j % ps, e)]);
                w[j] = acc * scale;
                if (w[j] > mx) mx = w[j];
            }
            double sum = 0.0;
            for (int j = 0; j < n; ++j) {
                w[j] = exp(w[j] - mx);
                sum += w[j];
            }
            for (int e = 0; e < d; ++e) orow[e] = 0.0;
            for (int j = 0; j < n; ++j) {
                double pj = w[j] / sum;
                for (int e = 0; e < d; ++e)
                    orow[e] += pj * oracle_bf16_to_f64(
                                        v_pool[v_index(c, num_pages, layer, bt[j / ps], kvh, j % ps, e)]);
            }
            free(w);
        }
    }
}

/* ---------------------------------------------------------------- SwiGLU
 * a[t][i] = silu(gate[t][i]) * up[t][i],  silu(z) = z / (1 + exp(-z))                     */
void oracle_swiglu(int64_t count, const double *gate, const double *up, double *a)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) a[i] = gate[i] / (1.0 + exp(-gate[i])) * up[i];
}

/* ---------------------------------------------------------------- one decoder layer
 * x [T][H] is the residual stream (in place).  tap, if not NULL, receives the residual
 * stream after the attention half ([T][H]).
 *
 * need (may be NULL = every row): only the rows t with need[t] != 0 are carried through the
 * layer; the others only contribute what later rows of their sequence can see of them -- their K
 * and V in the pool -- and their x (and tap) rows are left as they were.  A row's result depends
 * on its own x and on the pool alone, and every step function forms each output element by the
 * same sequence of operations whatever other rows are present, so a needed row comes out bit for
 * bit as it does with need = NULL.  This is how a few rows deep inside a long prefill chunk are
 * checked at real shapes without paying for the projections of the whole chunk.            */
static void gather_rows(int64_t n, const int64_t *idx, int64_t width, const double *src, double *dst)
{
    for (int64_t i = 0; i < n; ++i) memcpy(dst + i * width, src + idx[i] * width, (size_t)width * sizeof(double));
}

static void layer_forward_rows(const oracle_config *c, int layer, const oracle_layer *w, int64_t T,
                               const int32_t *seq_of, const int32_t *pos_of, const int32_t *block_tables,
                               int max_blocks_per_seq, int64_t num_pages, uint16_t *k_pool,
                               uint16_t *v_pool, double *x, double *tap, const uint8_t *need)
{
    int H = c->hidden, d = c->head_dim, I = c->intermediate;
    int QD = c->n_q_heads * d, KD = c->n_kv_heads * d;
    int64_t *idx = (int64_t *)malloc((size_t)(T + 1) * sizeof(int64_t));
    int64_t Tn = 0;
    for (int64_t t = 0; t < T; ++t)
        if (!need || need[t]) idx[Tn++] = t;
    int32_t *seq_n = (int32_t *)malloc((size_t)(Tn + 1) * sizeof(int32_t));
    int32_t *pos_n = (int32_t *)malloc((size_t)(Tn + 1) * sizeof(int32_t));
    for (int64_t i = 0; i < Tn; ++i) {
        seq_n[i] = seq_of[idx[i]];
        pos_n[i] = pos_of[idx[i]];
    }
    double *h = (double *)malloc((size_t)(T * H + 1) * sizeof(double));
    double *k = (double *)malloc((size_t)(T * KD + 1) * sizeof(double));
    double *v = (double *)malloc((size_t)(T * KD + 1) * sizeof(double));
    double *xs = (double *)malloc((size_t)(Tn * H + 1) * sizeof(double));
    double *hs = (double *)malloc((size_t)(Tn * H + 1) * sizeof(double));
    double *q = (double *)malloc((size_t)(Tn * QD + 1) * sizeof(double));
    double *o = (double *)malloc((size_t)(Tn * QD + 1) * sizeof(double));
    double *y = (double *)malloc((size_t)(Tn * H + 1) * sizeof(double));
    double *gt = (double *)malloc((size_t)(Tn * I + 1) * sizeof(double));
    double *up = (double *)malloc((size_t)(Tn * I + 1) * sizeof(double));

    /* every row: h = rmsnorm(x), K and V of its position into the pool */
    oracle_rmsnorm(T, H, x, w->norm1, c->rms_eps, h);
    if (c->round_operands) round_through_bf16(T * (int64_t)H, h);
    oracle_linear(T, H, KD, h, w->wk, c->has_qkv_bias ? w->bk : NULL, k);
    oracle_linear(T, H, KD, h, w->wv, c->has_qkv_bias ? w->bv : NULL, v);
    oracle_rope(T, c->n_kv_heads, d, pos_of, c->rope_theta, k);
    oracle_kv_write(c, layer, T, seq_of, pos_of, block_tables, max_blocks_per_seq, num_pages, k, v,
                    k_pool, v_pool);

    /* needed rows, attention half: x += Wo . attention(rope(Wq h), pool) */
    gather_rows(Tn, idx, H, x, xs);
    gather_rows(Tn, idx, H, h, hs);
    oracle_linear(Tn, H, QD, hs, w->wq, c->has_qkv_bias ? w->bq : NULL, q);
    oracle_rope(Tn, c->n_q_heads, d, pos_n, c->rope_theta, q);
    if (c->round_operands) round_through_bf16(Tn * (int64_t)QD, q);
    oracle_attention(c, layer, Tn, seq_n, pos_n, block_tables, max_blocks_per_seq, num_pages, q,
                     k_pool, v_pool, o);
    if (c->round_operands) round_through_bf16(Tn * (int64_t)QD, o);
    oracle_linear(Tn, QD, H, o, w->wo, NULL, y);
    for (int64_t i = 0; i < Tn * H; ++i) xs[i] += y[i];
    if (tap)
        for (int64_t i = 0; i < Tn; ++i) memcpy(tap + idx[i] * H, xs + i * H, (size_t)H * sizeof(double));

    /* needed rows, MLP half: x += Wd . (silu(Wg h2) * (Wu h2)) with h2 = rmsnorm(x) */
    oracle_rmsnorm(Tn, H, xs, w->norm2, c->rms_eps, hs);
    if (c->round_operands) round_through_bf16(Tn * (int64_t)H, hs);
    oracle_linear(Tn, H, I, hs, w->wgate, NULL, gt);
    oracle_linear(Tn, H, I, hs, w->wup, NULL, up);
    oracle_swiglu(Tn * (int64_t)I, gt, up, gt);
    if (c->round_operands) round_through_bf16(Tn * (int64_t)I, gt);
    oracle_linear(Tn, I, H, gt, w->wdown, NULL, y);
    for (int64_t i = 0; i < Tn * H; ++i) xs[i] += y[i];
    for (int64_t i = 0; i < Tn; ++i) memcpy(x + idx[i] * H, xs + i * H, (size_t)H * sizeof(double));

    free(idx); free(seq_n); free(pos_n);
    free(h); free(k); free(v); free(xs); free(hs); free(q); free(o); free(y); free(gt); free(up);
}

void oracle_layer_forward(const oracle_config *c, int layer, const oracle_layer *w, int64_t T,
                          const int32_t *seq_of, const int32_t *pos_of, const int32_t *block_tables,
                          int max_blocks_per_seq, int64_t num_pages, uint16_t *k_pool,
                          uint16_t *v_pool, double *x, double *tap)
{
    layer_forward_rows(c, layer, w, T, seq_of, pos_of, block_tables, max_blocks_per_seq, num_pages,
                       k_pool, v_pool, x, tap, NULL);
}

/* ---------------------------------------------------------------- the stage
 * hidden_in: bf16 [T][H].  out_f64 (may be NULL): residual stream after the last layer.
 * out_bf16 (may be NULL): the same rounded to bf16.  The pools are updated in place.
 * Returns 0, or -1 on a malformed batch (a page id outside the pool, a non-positive
 * new-token count, a negative cached length).                                             */
static int batch_is_valid(const oracle_config *c, int S, const int32_t *new_tokens, const int32_t *cached_len,
                          const int32_t *block_tables, int max_blocks_per_seq, int64_t num_pages)
{
    int ps = c->page_size;
    for (int s = 0; s < S; ++s) {
        if (new_tokens[s] < 1 || cached_len[s] < 0) return 0;
        int nb = (new_tokens[s] + cached_len[s] + ps - 1) / ps;
        if (nb > max_blocks_per_seq) return 0;
        for (int b = 0; b < nb; ++b) {
            int64_t pg = block_tables[(int64_t)s * max_blocks_per_seq + b];
            if (pg < 0 || pg >= num_pages) return 0;
        }
    }
    return 1;
}

int oracle_stage_forward(const oracle_config *c, const oracle_layer *layers, int S,
                         const int32_t *new_tokens, const int32_t *cached_len,
                         const int32_t *block_tables, int max_blocks_per_seq, int64_t num_pages,
                         uint16_t *k_pool, uint16_t *v_pool, const uint16_t *hidden_in,
                         double *out_f64, uint16_t *out_bf16)
{
    int H = c->hidden;
    if (!batch_is_valid(c, S, new_tokens, cached_len, block_tables, max_blocks_per_seq, num_pages)) return -1;
    int64_t T = oracle_token_map(S, new_tokens, cached_len, NULL, NULL);
    int32_t *seq_of = (int32_t *)malloc((size_t)(T + 1) * sizeof(int32_t));
    int32_t *pos_of = (int32_t *)malloc((size_t)(T + 1) * sizeof(int32_t));
    oracle_token_map(S, new_tokens, cached_len, seq_of, pos_of);
    double *x = (double *)malloc((size_t)(T * H + 1) * sizeof(double));
    for (int64_t i = 0; i < T * H; ++i) x[i] = oracle_bf16_to_f64(hidden_in[i]);
    for (int l = 0; l < c->num_layers; ++l)
        oracle_layer_forward(c, l, &layers[l], T, seq_of, pos_of, block_tables, max_blocks_per_seq,
                             num_pages, k_pool, v_pool, x, NULL);
    if (out_f64) memcpy(out_f64, x, (size_t)T * H * sizeof(double));
    if (out_bf16)
        for (int64_t i = 0; i < T * H; ++i) out_bf16[i] = oracle_f64_to_bf16(x[i]);
    free(x); free(seq_of); free(pos_of);
    return 0;
}

/* ---------------------------------------------------------------- one layer of a stage, some rows
 * The stage reduced to its layer `layer` (weights w, that layer's slice of the pools): hidden_in
 * bf16 [T][H] is the residual stream in front of the layer; out_f64 [T][H] receives the stream
 * behind it for the rows with need[t] != 0 (all rows if need is NULL) and the widened input for
 * the others; every row writes its K and V.  Returns 0, or -1 on a malformed batch.          */
int oracle_layer_rows(const oracle_config *c, int layer, const oracle_layer *w, int S,
                      const int32_t *new_tokens, const int32_t *cached_len,
                      const int32_t *block_tables, int max_blocks_per_seq, int64_t num_pages,
                      uint16_t *k_pool, uint16_t *v_pool, const uint16_t *hidden_in,
                      const uint8_t *need, double *out_f64)
{
    int H = c->hidden;
    if (layer < 0 || layer >= c->num_layers) return -1;
    if (!batch_is_valid(c, S, new_tokens, cached_len, block_tables, max_blocks_per_seq, num_pages)) return -1;
    int64_t T = oracle_token_map(S, new_tokens, cached_len, NULL, NULL);
    int32_t *seq_of = (int32_t *)malloc((size_t)(T + 1) * sizeof(int32_t));
    int32_t *pos_of = (int32_t *)malloc((size_t)(T + 1) * sizeof(int32_t));
    oracle_token_map(S, new_tokens, cached_len, seq_of, pos_of);
    for (int64_t i = 0; i < T * H; ++i) out_f64[i] = oracle_bf16_to_f64(hidden_in[i]);
    layer_forward_rows(c, layer, w, T, seq_of, pos_of, block_tables, max_blocks_per_seq, num_pages,
                       k_pool, v_pool, out_f64, NULL, need);
    free(seq_of); free(pos_of);
    return 0;
}
