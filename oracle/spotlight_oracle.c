/*
 * CPU oracle for the Spotlight Attention decode hot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may build, load or call it.  It shares no code, header, table or
 * constant generator with the HIP library and neither side includes the other.
 *
 * It is a plain, slow, scalar statement of what the path computes, step by step in the paper's
 * order and notation:
 *
 *   hash      H(x) = sign(W2 SiLU(W1 x + b1))           Sec. 3.2, Eq. 5 and Eq. 6
 *             H(x) = sign(x R)  (hidden == 0)            Sec. 3.2, Eq. 4
 *   pack      32 sign bits -> one uint32                 Appendix "Bit-Packing CUDA Kernel"
 *   score     f~(Q,K) = H(Q) (x) H(K), NXOR + popcount   Sec. 3.2, Eq. 3
 *   select    indices I of the top-k scores              Sec. 3.2 (text after Eq. 3)
 *   attend    gather(K,V,I) then softmax attention       Sec. 3.1, Eq. 2 and Eq. 1
 *
 * Precision.  The sign bit of the MLP output is an integer decision taken from floating point, so
 * both this oracle and the GPU take it in the same arithmetic: IEEE binary32, one accumulator per
 * output, fused multiply-add in increasing index order, and the exponential of SiLU given by the
 * fixed routine ref_exp() below (a specification, not an approximation choice left to a library).
 * The routine is pinned against libm's exp and the whole chain against an fp64 evaluation
 * (ref_hash_margin_f64) by the CPU tests.  Attention is evaluated in fp64 from the stored values.
 *
 * Parity pins (tests/test_oracle_*.py): hand-worked packing examples, bit-by-bit vs popcount
 * Hamming, full sort vs numpy's stable sort, dense softmax attention by numpy for k = N, closed
 * forms (identity MLP, equal keys, single row).  End-to-end retrieval quality (IoU, perplexity)
 * needs trained hash weights and the paper's datasets: parity unpinned for that, no claim made.
 *
 * Every function takes host pointers and returns 0, or a negative number for bad arguments.
 * dtype codes: 0 = float32, 1 = bfloat16 (raw uint16 bit patterns).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_EINVAL (-1)
#define REF_ENOMEM (-2)

static float ref_load(const void *p, int dtype, int64_t i)
{
    if (dtype == 0)
        return ((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16; /* bfloat16 is the top half of a binary32 */
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static size_t ref_elt(int dtype) { return dtype == 0 ? 4 : 2; }

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------
 * SiLU in binary32.  exp(t) for t clamped to [-87, 88]:
 *   n = round-to-nearest-even(t * log2(e));  r = t - n*ln2 in two fused steps (high, low part);
 *   e^r by the degree-7 Taylor polynomial in Horner form with fused multiply-adds;
 *   result = poly * 2^n (exact power of two built from the exponent field).
 * SiLU(a) = a / (1 + exp(-a))   (Eq. 5 uses SiLU; a * sigmoid(a) written as one division).
 * ------------------------------------------------------------------------------------------ */
float ref_exp(float t)
{
    t = (t > -87.0f) ? t : -87.0f; /* also maps NaN to -87 */
    t = (t < 88.0f) ? t : 88.0f;
    float n = rintf(t * 0x1.715476p+0f);
    float r = fmaf(n, -0x1.62e400p-1f, t);
    r = fmaf(n, -0x1.7f7d1cp-20f, r);
    float p = 0x1.a01a02p-13f;          /* 1/5040 */
    p = fmaf(p, r, 0x1.6c16c2p-10f);    /* 1/720  */
    p = fmaf(p, r, 0x1.111112p-7f);     /* 1/120  */
    p = fmaf(p, r, 0x1.555556p-5f);     /* 1/24   */
    p = fmaf(p, r, 0x1.555556p-3f);     /* 1/6    */
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    uint32_t bits = (uint32_t)((int32_t)n + 127) << 23;
    float s;
    memcpy(&s, &bits, 4);
    return p * s;
}

float ref_silu(float a)
{
    float e = ref_exp(-a);
    float den = 1.0f + e;
    return a / den;
}

/* ------------------------------------------------------------------------------------------
 * Hash one vector: L sign bits (0/1 bytes) of MLP(x), hash output j at bits[j].
 *   a_i = b1_i + sum_k W1[i][k] x[k]     (k increasing, fused multiply-add, binary32)
 *   h_i = SiLU(a_i)
 *   y_j = sum_i W2[j][i] h_i             (i increasing, from 0)
 *   bit_j = (y_j > 0)                    sign(0), sign(-0), sign(NaN) give bit 0
 * hidden == 0: y_j = sum_k R[j][k] x[k] with R passed as w1 [L, d] (Eq. 4, R stored row = output).
 * ------------------------------------------------------------------------------------------ */
static void ref_hash_one(const void *x, int x_dtype, int64_t x_off, int d,
                         const void *w1, const void *b1, const void *w2, int w_dtype,
                         int hidden, int L, float *hbuf, uint8_t *bits, float *y_out)
{
    if (hidden == 0) {
        for (int j = 0; j < L; ++j) {
            float y = 0.0f;
            for (int k = 0; k < d; ++k)
                y = fmaf(ref_load(w1, w_dtype, (int64_t)j * d + k), ref_load(x, x_dtype, x_off + k), y);
            bits[j] = (y > 0.0f) ? 1 : 0;
            if (y_out) y_out[j] = y;
        }
        return;
    }
    for (int i = 0; i < hidden; ++i) {
        float a = ref_load(b1, w_dtype, i);
        for (int k = 0; k < d; ++k)
            a = fmaf(ref_load(w1, w_dtype, (int64_t)i * d + k), ref_load(x, x_dtype, x_off + k), a);
        hbuf[i] = ref_silu(a);
    }
    for (int j = 0; j < L; ++j) {
        float y = 0.0f;
        for (int i = 0; i < hidden; ++i)
            y = fmaf(ref_load(w2, w_dtype, (int64_t)j * hidden + i), hbuf[i], y);
        bits[j] = (y > 0.0f) ? 1 : 0;
        if (y_out) y_out[j] = y;
    }
}

/* Bit-packing (Appendix "Bit-Packing CUDA Kernel").  The L bits of one row are cut into 32
 * consecutive chunks of W = L/32 columns; chunk after chunk the W output words shift left by one
 * and take that chunk's W bits in their lowest position.  So chunk 0 ends in bit 31 and chunk 31
 * in bit 0:  word j, bit (31 - c)  holds hash output  c*W + j. */
int ref_pack_bits(const uint8_t *bits, int64_t n_rows, int L, uint32_t *codes)
{
    if (!bits || !codes || n_rows < 0 || L <= 0 || L % 32) return REF_EINVAL;
    int W = L / 32;
    for (int64_t r = 0; r < n_rows; ++r) {
        uint32_t *out = codes + r * W;
        for (int j = 0; j < W; ++j) out[j] = 0;
        for (int c = 0; c < 32; ++c)
            for (int j = 0; j < W; ++j) {
                out[j] <<= 1;
                out[j] |= (uint32_t)(bits[r * L + (int64_t)c * W + j] & 1);
            }
    }
    return REF_OK;
}

/* Hash n_rows vectors x[r] (row stride d) with ONE head's weights.  Any of bits [n_rows, L],
 * codes [n_rows, L/32], y [n_rows, L] (the pre-sign outputs, binary32) may be NULL. */
int ref_hash_rows(const void *x, int x_dtype, int64_t n_rows, int d,
                  const void *w1, const void *b1, const void *w2, int w_dtype,
                  int hidden, int L, uint8_t *bits, uint32_t *codes, float *y)
{
    if (!x || !w1 || n_rows < 0 || d <= 0 || L <= 0 || L % 32 || hidden < 0) return REF_EINVAL;
    if (hidden > 0 && (!b1 || !w2)) return REF_EINVAL;
    if ((x_dtype | w_dtype) & ~1) return REF_EINVAL;
    int fail = 0;
#pragma omp parallel
    {
        float *hbuf = (float *)malloc(sizeof(float) * (size_t)(hidden > 0 ? hidden : 1));
        uint8_t *rb = (uint8_t *)malloc((size_t)L);
        if (!hbuf || !rb) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(static)
            for (int64_t r = 0; r < n_rows; ++r) {
                ref_hash_one(x, x_dtype, r * d, d, w1, b1, w2, w_dtype, hidden, L, hbuf, rb,
                             y ? y + r * L : NULL);
                if (bits) memcpy(bits + r * L, rb, (size_t)L);
                if (codes) ref_pack_bits(rb, 1, L, codes + r * (L / 32));
            }
        }
        free(hbuf);
        free(rb);
    }
    return fail ? REF_ENOMEM : REF_OK;
}

/* The same MLP in fp64 with libm's exp, no fused operations asked for: y64 [n_rows, L] and
 * mag [n_rows, L] = sum_i |W2[j][i] h_i| (the scale against which |y| is "far from zero").
 * Exists only so that a test can check ref_hash_rows' signs wherever the margin is clear. */
int ref_hash_margin_f64(const void *x, int x_dtype, int64_t n_rows, int d,
                        const void *w1, const void *b1, const void *w2, int w_dtype,
                        int hidden, int L, double *y64, double *mag)
{
    if (!x || !w1 || !b1 || !w2 || !y64 || !mag || hidden <= 0 || L <= 0) return REF_EINVAL;
    double *h = (double *)malloc(sizeof(double) * (size_t)hidden);
    if (!h) return REF_ENOMEM;
    for (int64_t r = 0; r < n_rows; ++r) {
        for (int i = 0; i < hidden; ++i) {
            double a = ref_load(b1, w_dtype, i);
            for (int k = 0; k < d; ++k)
                a += (double)ref_load(w1, w_dtype, (int64_t)i * d + k) * (double)ref_load(x, x_dtype, r * d + k);
            h[i] = a / (1.0 + exp(-a));
        }
        for (int j = 0; j < L; ++j) {
            double y = 0.0, m = 0.0;
            for (int i = 0; i < hidden; ++i) {
                double t = (double)ref_load(w2, w_dtype, (int64_t)j * hidden + i) * h[i];
                y += t;
                m += fabs(t);
            }
            y64[r * L + j] = y;
            mag[r * L + j] = m;
        }
    }
    free(h);
    return REF_OK;
}

/* Hamming distance of two packed codes, bit by bit (no popcount instruction, no table):
 * the number of positions where the two codes differ.  The paper's score (Eq. 3, NXOR then
 * popcount) is the number of positions where they agree: score = L - distance. */
static int ref_hamming_one(const uint32_t *a, const uint32_t *b, int W)
{
    int dist = 0;
    for (int w = 0; w < W; ++w)
        for (int bit = 0; bit < 32; ++bit) {
            uint32_t x = (a[w] >> bit) & 1u, y = (b[w] >> bit) & 1u;
            if (x != y) ++dist;
        }
    return dist;
}

int ref_hamming(const uint32_t *qcode, const uint32_t *codes, int64_t n, int L, uint16_t *dist)
{
    if (!qcode || !codes || !dist || n < 0 || L <= 0 || L % 32) return REF_EINVAL;
    int W = L / 32;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t)
        dist[t] = (uint16_t)ref_hamming_one(qcode, codes + t * W, W);
    return REF_OK;
}

/* NXOR score of Eq. 3 for one pair: number of agreeing bit positions. */
int ref_nxor_score(const uint32_t *a, const uint32_t *b, int L)
{
    int W = L / 32, s = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t nx = ~(a[w] ^ b[w]);
        for (int bit = 0; bit < 32; ++bit) s += (nx >> bit) & 1u;
    }
    return s;
}

/* Top-k: sort every (distance, token) pair by distance, then by token index; keep the first k;
 * return their token indices in increasing order. */
typedef struct { uint16_t d; int32_t t; } ref_pair;

static int ref_cmp_pair(const void *pa, const void *pb)
{
    const ref_pair *a = (const ref_pair *)pa, *b = (const ref_pair *)pb;
    if (a->d != b->d) return a->d < b->d ? -1 : 1;
    if (a->t != b->t) return a->t < b->t ? -1 : 1;
    return 0;
}

static int ref_cmp_i32(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

int ref_topk(const uint16_t *dist, int64_t n, int k, int32_t *idx)
{
    if (!dist || !idx || n <= 0 || k <= 0 || k > n || n > INT32_MAX) return REF_EINVAL;
    ref_pair *p = (ref_pair *)malloc(sizeof(ref_pair) * (size_t)n);
    if (!p) return REF_ENOMEM;
    for (int64_t t = 0; t < n; ++t) { p[t].d = dist[t]; p[t].t = (int32_t)t; }
    qsort(p, (size_t)n, sizeof(ref_pair), ref_cmp_pair);
    for (int i = 0; i < k; ++i) idx[i] = p[i].t;
    qsort(idx, (size_t)k, sizeof(int32_t), ref_cmp_i32);
    free(p);
    return REF_OK;
}

/* Top-k with forced tokens: the configuration columns "Sink" and "Local" of the perplexity
 * comparison with MagicPIG (first n_sink tokens, last n_local tokens always kept); the current
 * token that Eq. 1 concatenates is the local window of one.  With
 *   F = { t < n_sink }  U  { t >= n - n_local },
 * the result is F together with the k - |F| nearest of the OTHER tokens (distance, then token
 * index), in increasing token order: k indices in all.  Needs |F| <= k. */
int ref_topk_forced(const uint16_t *dist, int64_t n, int k, int n_sink, int n_local, int32_t *idx)
{
    if (!dist || !idx || n <= 0 || k <= 0 || k > n || n > INT32_MAX || n_sink < 0 || n_local < 0) return REF_EINVAL;
    int64_t n_forced = 0;
    for (int64_t t = 0; t < n; ++t) n_forced += (t < n_sink || t >= n - n_local);
    if (n_forced > k) return REF_EINVAL;
    ref_pair *p = (ref_pair *)malloc(sizeof(ref_pair) * (size_t)n);
    if (!p) return REF_ENOMEM;
    int kept = 0;
    int64_t others = 0;
    for (int64_t t = 0; t < n; ++t) {
        if (t < n_sink || t >= n - n_local) idx[kept++] = (int32_t)t;
        else { p[others].d = dist[t]; p[others].t = (int32_t)t; ++others; }
    }
    qsort(p, (size_t)others, sizeof(ref_pair), ref_cmp_pair);
    for (int i = 0; kept < k; ++i) idx[kept++] = p[i].t;
    qsort(idx, (size_t)k, sizeof(int32_t), ref_cmp_i32);
    free(p);
    return REF_OK;
}

/* Attention over exactly the rows listed in idx (Eq. 2 then Eq. 1 without the current-token
 * concatenation): s_i = scale * <q, K[idx_i]>, p = softmax(s), out = sum_i p_i V[idx_i].
 * K and V point at one head's [*, d] rows; all sums in fp64; out rounded to binary32. */
int ref_sparse_attention(const void *q, const void *K, const void *V, int dtype, int d,
                         const int32_t *idx, int k, double scale, float *out)
{
    if (!q || !K || !V || !idx || !out || d <= 0 || k <= 0 || (dtype & ~1)) return REF_EINVAL;
    double *s = (double *)malloc(sizeof(double) * (size_t)k);
    double *acc = (double *)calloc((size_t)d, sizeof(double));
    if (!s || !acc) { free(s); free(acc); return REF_ENOMEM; }
    double m = -INFINITY;
    for (int i = 0; i < k; ++i) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
            dot += (double)ref_load(q, dtype, c) * (double)ref_load(K, dtype, (int64_t)idx[i] * d + c);
        s[i] = dot * scale;
        if (s[i] > m) m = s[i];
    }
    double z = 0.0;
    for (int i = 0; i < k; ++i) { s[i] = exp(s[i] - m); z += s[i]; }
    for (int i = 0; i < k; ++i) {
        double p = s[i] / z;
        for (int c = 0; c < d; ++c)
            acc[c] += p * (double)ref_load(V, dtype, (int64_t)idx[i] * d + c);
    }
    for (int c = 0; c < d; ++c) out[c] = (float)acc[c];
    free(s);
    free(acc);
    return REF_OK;
}

/* ==========================================================================================
 * Layer-level calls with the data layout of the decode step (all host memory):
 *   q [B, Hq, d]; K, V [B, Hkv, Nmax, d]; codes [B, Hkv, Nmax, W]; weights per kv head
 *   W1 [Hkv, h, d], b1 [Hkv, h], W2 [Hkv, L, h]; query head hq uses kv head hq / (Hq/Hkv).
 * ========================================================================================== */
int ref_hash_keys(int B, int Hkv, int d, int L, int hidden, int64_t Nmax, int kv_dtype, int w_dtype,
                  const void *K, const void *w1, const void *b1, const void *w2,
                  int64_t t0, int64_t n_new, uint32_t *codes)
{
    if (B <= 0 || Hkv <= 0 || !K || !codes || t0 < 0 || n_new < 0 || t0 + n_new > Nmax) return REF_EINVAL;
    int W = L / 32;
    int64_t w1_rows = hidden > 0 ? hidden : L;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int64_t row0 = ((int64_t)b * Hkv + h) * Nmax + t0;
            const char *x = (const char *)K + (size_t)row0 * d * ref_elt(kv_dtype);
            const char *pw1 = (const char *)w1 + (size_t)h * w1_rows * d * ref_elt(w_dtype);
            const char *pb1 = b1 ? (const char *)b1 + (size_t)h * hidden * ref_elt(w_dtype) : NULL;
            const char *pw2 = w2 ? (const char *)w2 + (size_t)h * L * hidden * ref_elt(w_dtype) : NULL;
            int rc = ref_hash_rows(x, kv_dtype, n_new, d, pw1, pb1, pw2, w_dtype, hidden, L,
                                   NULL, codes + row0 * W, NULL);
            if (rc) return rc;
        }
    return REF_OK;
}

static int ref_retrieve(int B, int Hq, int Hkv, int d, int L, int hidden, int64_t Nmax,
                        int kv_dtype, int w_dtype, const void *q,
                        const void *w1, const void *b1, const void *w2,
                        const uint32_t *codes, int64_t n_tokens, int k, int forced, int n_sink, int n_local,
                        int32_t *out_idx, uint32_t *out_qcode, uint16_t *out_dist)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || !q || !codes || !out_idx) return REF_EINVAL;
    if (n_tokens <= 0 || n_tokens > Nmax || k <= 0 || k > n_tokens || L <= 0 || L % 32) return REF_EINVAL;
    int W = L / 32, G = Hq / Hkv;
    int64_t w1_rows = hidden > 0 ? hidden : L;
    uint16_t *dist = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n_tokens);
    if (!dist) return REF_ENOMEM;
    int rc = REF_OK;
    for (int b = 0; b < B && !rc; ++b)
        for (int hq = 0; hq < Hq && !rc; ++hq) {
            int hk = hq / G;
            int64_t bh = (int64_t)b * Hq + hq;
            uint32_t qcode[64];
            const char *x = (const char *)q + (size_t)bh * d * ref_elt(kv_dtype);
            const char *pw1 = (const char *)w1 + (size_t)hk * w1_rows * d * ref_elt(w_dtype);
            const char *pb1 = b1 ? (const char *)b1 + (size_t)hk * hidden * ref_elt(w_dtype) : NULL;
            const char *pw2 = w2 ? (const char *)w2 + (size_t)hk * L * hidden * ref_elt(w_dtype) : NULL;
            if (W > 64) { rc = REF_EINVAL; break; }
            rc = ref_hash_rows(x, kv_dtype, 1, d, pw1, pb1, pw2, w_dtype, hidden, L, NULL, qcode, NULL);
            if (rc) break;
            if (out_qcode) memcpy(out_qcode + bh * W, qcode, sizeof(uint32_t) * (size_t)W);
            rc = ref_hamming(qcode, codes + ((int64_t)b * Hkv + hk) * Nmax * W, n_tokens, L, dist);
            if (rc) break;
            if (out_dist) memcpy(out_dist + bh * n_tokens, dist, sizeof(uint16_t) * (size_t)n_tokens);
            rc = forced ? ref_topk_forced(dist, n_tokens, k, n_sink, n_local, out_idx + bh * k)
                        : ref_topk(dist, n_tokens, k, out_idx + bh * k);
        }
    free(dist);
    return rc;
}

int ref_retrieve_topk(int B, int Hq, int Hkv, int d, int L, int hidden, int64_t Nmax,
                      int kv_dtype, int w_dtype, const void *q,
                      const void *w1, const void *b1, const void *w2,
                      const uint32_t *codes, int64_t n_tokens, int k,
                      int32_t *out_idx, uint32_t *out_qcode, uint16_t *out_dist)
{
    return ref_retrieve(B, Hq, Hkv, d, L, hidden, Nmax, kv_dtype, w_dtype, q, w1, b1, w2, codes, n_tokens, k,
                        0, 0, 0, out_idx, out_qcode, out_dist);
}

int ref_sparse_decode(int B, int Hq, int Hkv, int d, int64_t Nmax, int kv_dtype,
                      const void *q, const void *K, const void *V,
                      const int32_t *idx, int k, double scale, float *out)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || !q || !K || !V || !idx || !out || k <= 0) return REF_EINVAL;
    int G = Hq / Hkv;
    int rc_all = REF_OK;
#pragma omp parallel for schedule(dynamic)
    for (int64_t bh = 0; bh < (int64_t)B * Hq; ++bh) {
        int b = (int)(bh / Hq), hq = (int)(bh % Hq), hk = hq / G;
        size_t head_off = (size_t)(((int64_t)b * Hkv + hk) * Nmax) * d * ref_elt(kv_dtype);
        int rc = ref_sparse_attention((const char *)q + (size_t)bh * d * ref_elt(kv_dtype),
                                      (const char *)K + head_off, (const char *)V + head_off,
                                      kv_dtype, d, idx + bh * k, k, scale, out + bh * d);
        if (rc) {
#pragma omp atomic write
            rc_all = rc;
        }
    }
    return rc_all;
}

/* One decode step of a layer, in the order the method runs it: the key of the token just appended
 * (row n_tokens - 1 of K) is hashed into the code cache, the query is hashed and scored against
 * the n_tokens cached codes, the top-k (with the forced sink / local tokens, see ref_topk_forced)
 * is taken per query head, and attention runs over exactly those rows.  codes is updated in place. */
int ref_decode_step(int B, int Hq, int Hkv, int d, int L, int hidden, int64_t Nmax, int kv_dtype, int w_dtype,
                    const void *q, const void *K, const void *V,
                    const void *w1, const void *b1, const void *w2,
                    uint32_t *codes, int64_t n_tokens, int k, int n_sink, int n_local, double scale,
                    int32_t *out_idx, float *out)
{
    if (n_tokens <= 0 || n_tokens > Nmax) return REF_EINVAL;
    int rc = ref_hash_keys(B, Hkv, d, L, hidden, Nmax, kv_dtype, w_dtype, K, w1, b1, w2, n_tokens - 1, 1, codes);
    if (rc) return rc;
    rc = ref_retrieve(B, Hq, Hkv, d, L, hidden, Nmax, kv_dtype, w_dtype, q, w1, b1, w2, codes, n_tokens, k,
                      1, n_sink, n_local, out_idx, NULL, NULL);
    if (rc) return rc;
    return ref_sparse_decode(B, Hq, Hkv, d, Nmax, kv_dtype, q, K, V, out_idx, k, scale, out);
}
