/*
 * vq_oracle.c -- CPU oracle for matrix products whose weight / KV operand is
 * stored as vector-quantization codes.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the plain definition of what the
 * GPU library must compute, written to be checked against the paper by eye.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * it.  It shares no code with the GPU path and is never tuned.
 *
 * What it follows (VQ-LLM, arXiv 2503.02236):
 *   - Dequantization, Sec. II-A ("Typical VQ Pipeline", last paragraph, and
 *     Fig. 1 lower half): for every residual, look up the entry indexed by
 *     the code in that residual's codebook; combine the residuals of one
 *     sub-space by element-wise accumulation; concatenate the sub-spaces.
 *   - VQ<vector size, log2 #entries, residuals> notation, Sec. II-A / Tbl. I.
 *   - Attention(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V, Sec. II-B, evaluated
 *     for one query per sequence (decode phase) over a cache of T tokens.
 *   - GeMV / GeMM over a weight matrix held as codes, Sec. III-C (VQ-gemv,
 *     VQ-gemm): y = x * dequant(W)^T.
 *
 * Readings where the paper is silent:
 *   - sub-vectors lie along the input-feature (reduction) axis K of W[N][K];
 *   - codes are stored [N][K/v][R], residual index fastest, as uint8/uint16,
 *     or as a packed 12-bit string in the same order (layout at read_code);
 *   - residual entries are summed in fp32, residual 0 first;
 *   - an optional per-output-channel scale multiplies the accumulated sum;
 *   - all T cached tokens come from the VQ cache; seq_lens[b] may shorten T.
 *
 * Precision: fp16 -> fp32 conversion is exact; the dequantized weight is the
 * fp32 sum of its residual entries; every product and every accumulation of
 * the contraction and the whole softmax are done in fp64, natural index
 * order.  Results are returned un-rounded in fp64.
 *
 * Parity pins (tests/test_oracle_pins.py): hand-computed tiny cases, one-hot
 * codebooks (index sums), palette codebooks against a dense fp64 matmul,
 * linearity over residual codebooks and over the scale, GEMM rows against
 * separate GEMVs, entry-permutation invariance, per-tile codebooks against
 * per-tensor results assembled tile by tile, closed-form attention cases
 * (T = 1, q = 0, one dominant key), dense fp64 softmax attention, split
 * invariance, and all 65536 fp16 bit patterns of the half -> float routine.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE-754 binary16 bit pattern -> binary32 value (exact: every half is a float). */
float vq_oracle_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1fu;
    uint32_t frac = (uint32_t)h & 0x3ffu;
    float mag;
    if (expo == 0) {
        mag = ldexpf((float)frac, -24);              /* zero or subnormal: frac * 2^-24 */
    } else if (expo == 31) {
        mag = frac ? NAN : INFINITY;
    } else {
        mag = ldexpf((float)(frac | 0x400u), (int)expo - 25); /* (1024+frac) * 2^(e-15-10) */
    }
    return sign ? -mag : mag;
}

void vq_oracle_half_to_float_array(const uint16_t *h, float *out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = vq_oracle_half_to_float(h[i]);
}

/* Thread count of the following calls (timing harnesses: the single-thread baseline); no effect on results. */
void vq_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int vq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Code number idx of the tensor.  8 and 16 bits: one uint8 / uint16 each.
 * 12 bits (the paper's VQ<8,12,2> configuration has an "unaligned 12-bit
 * storage format", Sec. VII-B; the bit layout is not given, so this is a
 * reading): the codes form one little-endian bit string, code idx occupying
 * bits [12 idx, 12 idx + 12) -- two codes in three bytes:
 *   byte 3p   = low 8 bits of code 2p
 *   byte 3p+1 = high 4 bits of code 2p (low nibble) | low 4 bits of code 2p+1 (high nibble)
 *   byte 3p+2 = high 8 bits of code 2p+1
 */
static inline uint32_t read_code(const void *codes, int code_bits, size_t idx)
{
    if (code_bits == 8) return ((const uint8_t *)codes)[idx];
    if (code_bits == 12) {
        const uint8_t *b = (const uint8_t *)codes + (idx >> 1) * 3;
        if ((idx & 1) == 0) return (uint32_t)b[0] | (((uint32_t)b[1] & 0x0Fu) << 8);
        return ((uint32_t)b[1] >> 4) | ((uint32_t)b[2] << 4);
    }
    return ((const uint16_t *)codes)[idx];
}

/* The first n codes of a packed 12-bit string (test access to the reader above). */
void vq_oracle_unpack12(const uint8_t *packed, size_t n, uint32_t *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = read_code(packed, 12, i);
}

/*
 * Dequantize one row n of W into row[K] (fp32).
 * Sec. II-A: entry lookup per residual, element-wise accumulation over the
 * residuals (fp32, residual 0 first), concatenation over the K/v sub-spaces.
 * codes: [N][K/v][R]; codebooks: fp16 bits [R][E][v].
 * Codebook scope (Sec. III-B and Tbl. III: some algorithms keep one set of
 * codebooks per tensor, others one per tile of the weight, e.g. per (256, 256)
 * tile): with tile_n, tile_k > 0 the codebooks are
 * [ceil(N/tile_n)][K/tile_k][R][E][v] and element (n, k) uses the set of tile
 * (n / tile_n, k / tile_k); tile_n = tile_k = 0 means one set for the tensor.
 */
static void dequant_row(int n, int K, int v, int code_bits, int R, int E, int tile_n, int tile_k,
                        const void *codes, const uint16_t *codebooks_all, float *row)
{
    int J = K / v;
    int tiles_k = tile_k > 0 ? K / tile_k : 1;
    for (int j = 0; j < J; ++j) {
        const uint16_t *codebooks = codebooks_all;
        if (tile_n > 0)
            codebooks += ((size_t)(n / tile_n) * tiles_k + (size_t)(j * v) / tile_k) * ((size_t)R * E * v);
        for (int i = 0; i < v; ++i) {
            float acc = 0.0f;
            for (int r = 0; r < R; ++r) {
                uint32_t c = read_code(codes, code_bits, ((size_t)n * J + j) * R + r);
                float e = vq_oracle_half_to_float(codebooks[((size_t)r * E + c) * v + i]);
                acc = (r == 0) ? e : acc + e;
            }
            row[(size_t)j * v + i] = acc;
        }
    }
}

/* Dense fp32 weight Wd[N][K] (the bit-exact tile reference). */
void vq_oracle_dequant(int N, int K, int v, int code_bits, int R, int E, int tile_n, int tile_k,
                       const void *codes, const uint16_t *codebooks, float *Wd)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        dequant_row(n, K, v, code_bits, R, E, tile_n, tile_k, codes, codebooks, Wd + (size_t)n * K);
}

/*
 * Y[m][n] = scale[n] * sum_k Wd[n][k] * x[m][k]   (fp64, k ascending).
 * GeMV is M = bs (1..16); GeMM is M = number of prefill tokens.
 * rows: optional list of n_rows output channels to evaluate (NULL = all N);
 * Y is [M][n_rows] in that case, column order following `rows`.
 * scale: fp16 bits [N] or NULL.
 */
void vq_oracle_gemm(int N, int K, int v, int code_bits, int R, int E, int tile_n, int tile_k,
                    const void *codes, const uint16_t *codebooks, const uint16_t *scale,
                    const uint16_t *x, int M, const int *rows, int n_rows, double *Y)
{
    int NR = rows ? n_rows : N;
#pragma omp parallel
    {
        float *row = (float *)malloc(sizeof(float) * (size_t)K);
#pragma omp for schedule(static)
        for (int r = 0; r < NR; ++r) {
            int n = rows ? rows[r] : r;
            dequant_row(n, K, v, code_bits, R, E, tile_n, tile_k, codes, codebooks, row);
            double s = scale ? (double)vq_oracle_half_to_float(scale[n]) : 1.0;
            for (int m = 0; m < M; ++m) {
                const uint16_t *xm = x + (size_t)m * K;
                double acc = 0.0;
                for (int k = 0; k < K; ++k)
                    acc += (double)row[k] * (double)vq_oracle_half_to_float(xm[k]);
                Y[(size_t)m * NR + r] = s * acc;
            }
        }
        free(row);
    }
}

/*
 * Dequantize one token's K or V vector of head h: out[D] fp32.
 * codes: uint8 [B][H][T][D/v]; codebooks: fp16 bits [H][G][E][v]; group g of
 * the D/v sub-vectors uses codebook (g * G) / (D/v)  (G = 1: one codebook per
 * head and side; G = D/v: one codebook per sub-space).
 */
static void kv_dequant_token(const uint8_t *codes, const uint16_t *codebooks,
                             int H, int T, int D, int v, int E, int G,
                             int b, int h, int t, float *out)
{
    int P = D / v;
    const uint8_t *c = codes + (((size_t)b * H + h) * T + t) * P;
    for (int p = 0; p < P; ++p) {
        int g = (int)(((long)p * G) / P);
        const uint16_t *entry = codebooks + ((((size_t)h * G + g) * E) + c[p]) * v;
        for (int i = 0; i < v; ++i) out[p * v + i] = vq_oracle_half_to_float(entry[i]);
    }
}

/*
 * Quantization of new K or V vectors (the assignment step of Sec. II-A: a
 * sub-vector is replaced by the index of its closest codebook entry; this is
 * what the on-the-fly KV quantization of Sec. VII "Quantization Overhead" runs
 * for every new token).  x: fp16 bits [B][H][n_new][D]; codebooks as above;
 * out: uint8 [B][H][n_new][D/v].
 * A floating-point comparison decides an integer here, so the precision and
 * the order are part of the definition (the paper gives none; this is the
 * reading the GPU kernel follows too): squared Euclidean distance in fp32,
 *   d = ((x0-c0)^2 + (x1-c1)^2) + ... , elements in ascending order, every
 * subtraction, multiplication and addition rounded separately (no fused
 * multiply-add); the smallest distance wins, ties go to the smallest index.
 */
void vq_oracle_kv_quantize(int B, int H, int D, int n_new, int v, int E, int G,
                           const uint16_t *x, const uint16_t *codebooks, uint8_t *out)
{
    int P = D / v;
#pragma omp parallel for schedule(static)
    for (long bh = 0; bh < (long)B * H; ++bh) {
        int h = (int)(bh % H);
        for (int t = 0; t < n_new; ++t) {
            const uint16_t *xv = x + ((size_t)bh * n_new + t) * D;
            for (int p = 0; p < P; ++p) {
                int g = (int)(((long)p * G) / P);
                const uint16_t *cb = codebooks + (((size_t)h * G + g) * E) * v;
                int best = 0;
                float best_d = 0.0f;
                for (int e = 0; e < E; ++e) {
                    volatile float d = 0.0f;   /* volatile: each step is rounded to fp32, nothing is fused */
                    for (int i = 0; i < v; ++i) {
                        volatile float diff = vq_oracle_half_to_float(xv[p * v + i])
                                            - vq_oracle_half_to_float(cb[(size_t)e * v + i]);
                        volatile float sq = diff * diff;
                        d = d + sq;
                    }
                    if (e == 0 || d < best_d) { best = e; best_d = d; }
                }
                out[((size_t)bh * n_new + t) * P + p] = (uint8_t)best;
            }
        }
    }
}

/* Dense fp32 cache out[B][H][T][D] of one side. */
void vq_oracle_kv_dequant(int B, int H, int D, int T, int v, int E, int G,
                          const uint8_t *codes, const uint16_t *codebooks, float *out)
{
#pragma omp parallel for schedule(static)
    for (long bh = 0; bh < (long)B * H; ++bh) {
        int b = (int)(bh / H), h = (int)(bh % H);
        for (int t = 0; t < T; ++t)
            kv_dequant_token(codes, codebooks, H, T, D, v, E, G, b, h, t,
                             out + (((size_t)b * H + h) * T + t) * D);
    }
}

/*
 * Decode attention over a VQ cache, Sec. II-B formula, one query per (b, h):
 *   s_t = sm_scale * sum_d q[d] * Kd[t][d]
 *   p   = softmax_t(s)          (subtract max_t s_t, fp64)
 *   o[d] = sum_t p_t * Vd[t][d]
 * Tokens t in [t0, t1) clipped to the sequence length; (t0,t1) = (0,T) is the
 * whole cache.  Besides out[B][H][D] the routine can return the softmax
 * statistics m[B][H] (max score) and l[B][H] (sum of exp(s - m)) so that a
 * test can merge two token ranges by log-sum-exp; pass NULL to skip.
 * A (b,h) with no valid token yields o = 0, m = -inf, l = 0.
 */
void vq_oracle_attn_decode(int B, int H, int D, int T, int v, int E, int G,
                           const uint8_t *k_codes, const uint8_t *v_codes,
                           const uint16_t *k_codebooks, const uint16_t *v_codebooks,
                           const int *seq_lens, const uint16_t *q, double sm_scale,
                           int t0, int t1, double *out, double *m_out, double *l_out)
{
#pragma omp parallel
    {
        float *kd = (float *)malloc(sizeof(float) * (size_t)D);
        double *s = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
#pragma omp for schedule(static)
        for (long bh = 0; bh < (long)B * H; ++bh) {
            int b = (int)(bh / H), h = (int)(bh % H);
            int len = seq_lens ? seq_lens[b] : T;
            int lo = t0 < 0 ? 0 : t0;
            int hi = t1 < len ? t1 : len;
            const uint16_t *qv = q + ((size_t)b * H + h) * D;
            double *o = out + ((size_t)b * H + h) * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            double m = -INFINITY, l = 0.0;
            for (int t = lo; t < hi; ++t) {
                kv_dequant_token(k_codes, k_codebooks, H, T, D, v, E, G, b, h, t, kd);
                double acc = 0.0;
                for (int d = 0; d < D; ++d)
                    acc += (double)vq_oracle_half_to_float(qv[d]) * (double)kd[d];
                s[t] = sm_scale * acc;
                if (s[t] > m) m = s[t];
            }
            for (int t = lo; t < hi; ++t) l += exp(s[t] - m);
            for (int t = lo; t < hi; ++t) {
                double p = exp(s[t] - m) / l;
                kv_dequant_token(v_codes, v_codebooks, H, T, D, v, E, G, b, h, t, kd);
                for (int d = 0; d < D; ++d) o[d] += p * (double)kd[d];
            }
            if (m_out) m_out[bh] = m;
            if (l_out) l_out[bh] = l;
        }
        free(kd);
        free(s);
    }
}
