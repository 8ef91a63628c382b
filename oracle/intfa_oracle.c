/*
 * CPU oracle for the INT-FlashAttention forward pass -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar restatement of what the method computes, written from the
 * paper (arXiv 2409.16997) and sharing no code with the HIP path.  Only tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the product never does.
 *
 * Floating point follows the paper's statement that the scores S, the running max m,
 * the running sum l and the on-chip output O are FP32 (Section 3.2, Figure 1 caption);
 * integer products are exact int32.  Compile WITHOUT fast-math and with
 * -ffp-contract=off so that every fp32 operation below rounds once, as written.
 *
 * Pins (tests/test_oracle_*.py): quantizer identity on the int8 grid, half-step error
 * bound, sign symmetry; int32 GEMMs against int64 numpy; p_quant=0 against fp64
 * brute-force attention; single-block closed form; uniform-score and one-hot closed
 * forms; causal prefix properties; scale linearity; the P-rounding error bound; the fp16
 * rounding helper against numpy's float16 cast; the half-INT8 variant against fp64 attention of
 * the dequantized operands within the fp16 rounding bound, and its closed forms.
 * Unpinned: nothing in this file (the MRE magnitudes of Tables 1-2 are context only).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define R_INT8 127 /* Algorithm 1, Require: INT8 maximum R = 127 */

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Section 3.2 (symmetric quantization without a zero point, S = rowmax|X| / R).
 * One scale per row of a [rows, cols] matrix: cols = d gives the token-level scheme of
 * Q and K; rows = heads, cols = N*d gives the tensor-level scheme of V.
 *   a = max|x|, s = a / 127, q = clamp(rint(x * (127 / a)), -127, 127); a == 0 -> s = 1, q = 0.
 * All in fp32, round-half-to-even. */
void orc_quantize_rows(const float *X, int64_t rows, int64_t cols, int8_t *q, float *s)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *x = X + r * cols;
        int8_t *qr = q + r * cols;
        float a = 0.0f;
        for (int64_t k = 0; k < cols; ++k) {
            float v = fabsf(x[k]);
            if (v > a) a = v;
        }
        if (a == 0.0f) {
            s[r] = 1.0f;
            memset(qr, 0, (size_t)cols);
            continue;
        }
        s[r] = a / 127.0f;
        const float inv = 127.0f / a;
        for (int64_t k = 0; k < cols; ++k) {
            float t = rintf(x[k] * inv);
            if (t > 127.0f) t = 127.0f;
            if (t < -127.0f) t = -127.0f;
            qr[k] = (int8_t)t;
        }
    }
}

/* Walsh-Hadamard transform of every row (Sylvester order, unnormalized: H_d H_d = d I), the rotation the paper
 * names as future work (Section 5, the combination with Hadamard transformations).  Applied to the rows of both
 * Q and K it leaves Q K^T unchanged up to the factor d, and spreads outlier channels over all channels before
 * the token-level quantization.  The butterflies run in fp32 in the textbook order h = 1, 2, 4, ...:
 * (x[i], x[i+h]) <- (x[i] + x[i+h], x[i] - x[i+h]) for every i with bit h clear.  cols must be a power of two. */
void orc_hadamard_rows(const float *X, int64_t rows, int64_t cols, float *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        float *y = Y + r * cols;
        memcpy(y, X + r * cols, sizeof(float) * (size_t)cols);
        for (int64_t h = 1; h < cols; h <<= 1)
            for (int64_t i = 0; i < cols; ++i)
                if ((i & h) == 0) {
                    const float a = y[i], b = y[i + h];
                    y[i] = a + b;
                    y[i + h] = a - b;
                }
    }
}

/* Algorithm 1 line 9, integer part: S_int[i][j] = sum_k Q[i][k] * K[j][k], one head. */
void orc_qk_i32(const int8_t *Q, const int8_t *K, int64_t N, int d, int32_t *S)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int32_t acc = 0;
            for (int k = 0; k < d; ++k) acc += (int32_t)Q[i * d + k] * (int32_t)K[j * d + k];
            S[i * N + j] = acc;
        }
}

/* Algorithm 1 line 13, integer part: PV[i][c] = sum_j P[i][j] * V[j][c], one head. */
void orc_pv_i32(const int8_t *P, const int8_t *V, int64_t N, int d, int32_t *PV)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i)
        for (int c = 0; c < d; ++c) {
            int32_t acc = 0;
            for (int64_t j = 0; j < N; ++j) acc += (int32_t)P[i * N + j] * (int32_t)V[j * d + c];
            PV[i * d + c] = acc;
        }
}

/*
 * Algorithm 1, one query row at a time (rows are independent, so B_r plays no role).
 *
 *   Q         int8 [B*H, Nq, d], sQ fp32 [B*H, Nq];  K, V int8 [B*H, N, d], sK fp32 [B*H, N];  sV fp32 [B*H]
 *             Nq = N is the paper's setting.  Nq != N (a chunk of queries against a longer key sequence) is an
 *             extension: rows are independent, so nothing else changes.
 *   sv_per_block  0: sV is the tensor-level scalar of Section 3.2, one per head, applied on line 16.
 *             1: the per-block scheme the paper names as future work (Section 3.2 footnote, Section 5):
 *             sV is fp32 [B*H, ceil(N/Bc)], one scale per key block V_j, applied where P V_j enters O
 *             (line 13 becomes O = alpha O + s_V,j (P V_j)) and line 16 divides by l only.
 *   Bc        key-block size: the result depends on it, because block j is rounded on
 *             the grid of the running max after block j, not of the final max.
 *   causal    extension (not in the paper): key index > query index + (N - Nq) gets S = -inf, P = 0
 *             (the queries are the LAST Nq positions of the key sequence; needs N >= Nq).
 *   p_quant   1: Algorithm 1 (P rounded to int8, l sums the rounded P)
 *             0: the FlashAttention-2 recurrence of Section 3.1 (P~ kept real), in fp64
 *   row_idx   global row ids head*Nq + i to evaluate (NULL: all B*H*N rows in order)
 *   O         fp32 [n_rows, d]
 *   l_out, m_out   optional fp32 [n_rows]: final l and m
 *   n_tie     optional int32 [n_rows]: number of P entries whose rounding would change if
 *             the exponent argument moved by tie_rel * (|S| + |m|) + tie_abs; a different
 *             fp32 evaluation order may legitimately round those the other way.
 *   P_out     optional int8 [n_rows, N]: the rounded P of every key (p_quant = 1 only)
 *   tie_flip  optional uint64 [n_rows]: bit k set = the k-th flagged near-tie entry of that row (in key order, k < 64)
 *             takes the OTHER of its two neighbouring integers.  Line 11's round() is decided on an fp32 argument;
 *             for a flagged entry a second, equally valid fp32 evaluation of that argument lands on the other side
 *             of the half-integer, so both integers are results of Algorithm 1.  Used by the parity tests to check
 *             that an output which differs from the default resolution is the output of another valid one.
 */
void orc_int_flash_attn_fwd(const int8_t *Q, const int8_t *K, const int8_t *V,
                            const float *sQ, const float *sK, const float *sV,
                            int B, int H, int64_t Nq, int64_t N, int d, int causal, int Bc, int p_quant, int sv_per_block,
                            const int64_t *row_idx, int64_t n_rows,
                            float *O, float *l_out, float *m_out,
                            double tie_rel, double tie_abs, int32_t *n_tie, int8_t *P_out, const uint64_t *tie_flip)
{
    const int64_t total = (int64_t)B * H * Nq;
    const int64_t shift = N - Nq;   /* causal: query i sees keys j <= i + shift (the last query sees every key) */
    const int64_t Tc = (N + Bc - 1) / Bc;
    if (row_idx == NULL) n_rows = total;

#pragma omp parallel
    {
        float *S = (float *)malloc(sizeof(float) * (size_t)Bc);
        int32_t *P = (int32_t *)malloc(sizeof(int32_t) * (size_t)Bc);
        double *Pr = (double *)malloc(sizeof(double) * (size_t)Bc);
        float *o = (float *)malloc(sizeof(float) * (size_t)d);
        double *od = (double *)malloc(sizeof(double) * (size_t)d);

#pragma omp for schedule(dynamic, 16)
        for (int64_t r = 0; r < n_rows; ++r) {
            const int64_t g = row_idx ? row_idx[r] : r;
            const int64_t head = g / Nq, i = g % Nq + (causal ? shift : 0);   /* i: last visible key if causal */
            const int8_t *q = Q + g * d;
            const int8_t *Kh = K + head * N * d;
            const int8_t *Vh = V + head * N * d;
            const float sq = sQ[g];
            const float *skh = sK + head * N;

            float m = -INFINITY, l = 0.0f;   /* line 6 */
            double ld = 0.0;
            int32_t ties = 0;
            for (int c = 0; c < d; ++c) { o[c] = 0.0f; od[c] = 0.0; }
            if (P_out) memset(P_out + r * N, 0, (size_t)N);

            for (int64_t j0 = 0; j0 < N; j0 += Bc) {              /* line 7 */
                if (causal && j0 > i) break;
                const int nb = (int)((N - j0 < Bc) ? (N - j0) : Bc);
                float bmax = -INFINITY;
                for (int jj = 0; jj < nb; ++jj) {                  /* line 9 */
                    const int64_t j = j0 + jj;
                    if (causal && j > i) { S[jj] = -INFINITY; continue; }
                    const int8_t *k = Kh + j * d;
                    int32_t acc = 0;
                    for (int t = 0; t < d; ++t) acc += (int32_t)q[t] * (int32_t)k[t];
                    S[jj] = ((float)acc * sq) * skh[j];
                    if (S[jj] > bmax) bmax = S[jj];
                }
                const float svj = sv_per_block ? sV[head * Tc + j0 / Bc] : 1.0f;
                const float m_new = (bmax > m) ? bmax : m;         /* line 10 */
                const double alpha = (m == -INFINITY) ? 0.0 : exp((double)(m - m_new));

                if (p_quant) {
                    int32_t psum = 0;
                    for (int jj = 0; jj < nb; ++jj) {              /* line 11 */
                        if (S[jj] == -INFINITY) { P[jj] = 0; continue; }
                        const float t = S[jj] - m_new;
                        const double u = (double)R_INT8 * exp((double)t);
                        P[jj] = (int32_t)nearbyint(u);
                        if (n_tie || tie_flip) {
                            const double half = floor(u) + 0.5;
                            const double dt = tie_rel * (fabs((double)S[jj]) + fabs((double)m_new)) + tie_abs;
                            if (fabs(u - half) <= u * dt) {
                                if (tie_flip && ties < 64 && ((tie_flip[r] >> ties) & 1u))
                                    P[jj] = (P[jj] == (int32_t)floor(u)) ? (int32_t)floor(u) + 1 : (int32_t)floor(u);
                                ++ties;
                            }
                        }
                        psum += P[jj];
                        if (P_out) P_out[r * N + j0 + jj] = (int8_t)P[jj];
                    }
                    l = l * (float)alpha + (float)psum;            /* line 12 */
                    for (int c = 0; c < d; ++c) {                  /* line 13 */
                        int32_t pv = 0;
                        for (int jj = 0; jj < nb; ++jj) pv += P[jj] * (int32_t)Vh[(j0 + jj) * d + c];
                        o[c] = sv_per_block ? o[c] * (float)alpha + (float)pv * svj
                                            : o[c] * (float)alpha + (float)pv;
                    }
                } else {
                    double psum = 0.0;
                    for (int jj = 0; jj < nb; ++jj) {
                        Pr[jj] = (S[jj] == -INFINITY) ? 0.0 : exp((double)S[jj] - (double)m_new);
                        psum += Pr[jj];
                    }
                    ld = ld * alpha + psum;
                    for (int c = 0; c < d; ++c) {
                        double pv = 0.0;
                        for (int jj = 0; jj < nb; ++jj) pv += Pr[jj] * (double)Vh[(j0 + jj) * d + c];
                        od[c] = od[c] * alpha + pv * (double)svj;
                    }
                }
                m = m_new;
            }

            const float sv = sv_per_block ? 1.0f : sV[head];
            if (p_quant) {
                for (int c = 0; c < d; ++c) O[r * d + c] = (o[c] / l) * sv;   /* line 16 */
                if (l_out) l_out[r] = l;
            } else {
                for (int c = 0; c < d; ++c) O[r * d + c] = (float)((od[c] / ld) * (double)sv);
                if (l_out) l_out[r] = (float)ld;
            }
            if (m_out) m_out[r] = m;
            if (n_tie) n_tie[r] = ties;
        }
        free(S); free(P); free(Pr); free(o); free(od);
    }
}

/* Nearest fp16 value of x (round half to even, gradual underflow, overflow to infinity), returned as a float.
 * Written out on the bit pattern: fp16 has 10 fraction bits, exponents 2^-14 .. 2^15, subnormal step 2^-24. */
float orc_round_to_half(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    const uint32_t sign = u & 0x80000000u;
    uint32_t a = u & 0x7fffffffu;
    float r;
    if (a >= 0x7f800000u) return x;                               /* inf, nan */
    if (a >= 0x477ff000u) { a = 0x7f800000u; }                    /* >= 65520 rounds to infinity */
    else if (a >= 0x38800000u) {                                  /* normal half: drop 13 fraction bits */
        const uint32_t rem = a & 0x1fffu, lsb = (a >> 13) & 1u;
        a &= ~0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && lsb)) a += 0x2000u;
    } else {                                                      /* subnormal half: multiples of 2^-24 */
        float m;
        memcpy(&m, &a, 4);
        m = (float)nearbyint((double)m * 16777216.0) * (1.0f / 16777216.0f);   /* exact: at most 2^10 steps */
        memcpy(&a, &m, 4);
    }
    a |= sign;
    memcpy(&r, &a, 4);
    return r;
}

/*
 * The half-INT8 variant of Section 4 (INT8 Q and K with token-level scales, FP16 V): Algorithm 1 with the
 * second GEMM in half precision.  The paper gives one sentence; the reading taken, by analogy with lines 11-13:
 *   S as in line 9 (int32 product, fp32 scales);  m as in line 10;
 *   P~ = fp16(exp(S - m))            no factor R, rounded to the nearest fp16 value
 *   l  = alpha l + rowsum(P~)        the ROUNDED weights, summed in fp32 (as line 12 sums the rounded P)
 *   O  = alpha O + P~ V_j            fp16 x fp16 products are exact in fp32; fp32 accumulation in key order
 *   O  = O / l                       no s_V: V is not quantized
 * Vf holds the caller's fp16 V widened to fp32 [B*H, N, d]; Q is [B*H, Nq, d].  Other arguments as
 * orc_int_flash_attn_fwd.
 */
void orc_int_flash_attn_fwd_half(const int8_t *Q, const int8_t *K, const float *Vf,
                                 const float *sQ, const float *sK,
                                 int B, int H, int64_t Nq, int64_t N, int d, int causal, int Bc,
                                 const int64_t *row_idx, int64_t n_rows,
                                 float *O, float *l_out, float *m_out)
{
    const int64_t total = (int64_t)B * H * Nq;
    const int64_t shift = N - Nq;   /* causal: query i sees keys j <= i + shift, as in orc_int_flash_attn_fwd */
    if (row_idx == NULL) n_rows = total;

#pragma omp parallel
    {
        float *S = (float *)malloc(sizeof(float) * (size_t)Bc);
        float *P = (float *)malloc(sizeof(float) * (size_t)Bc);
        float *o = (float *)malloc(sizeof(float) * (size_t)d);

#pragma omp for schedule(dynamic, 16)
        for (int64_t r = 0; r < n_rows; ++r) {
            const int64_t g = row_idx ? row_idx[r] : r;
            const int64_t head = g / Nq, i = g % Nq + (causal ? shift : 0);   /* i: last visible key if causal */
            const int8_t *q = Q + g * d;
            const int8_t *Kh = K + head * N * d;
            const float *Vh = Vf + head * N * d;
            const float sq = sQ[g];
            const float *skh = sK + head * N;

            float m = -INFINITY, l = 0.0f;
            for (int c = 0; c < d; ++c) o[c] = 0.0f;

            for (int64_t j0 = 0; j0 < N; j0 += Bc) {
                if (causal && j0 > i) break;
                const int nb = (int)((N - j0 < Bc) ? (N - j0) : Bc);
                float bmax = -INFINITY;
                for (int jj = 0; jj < nb; ++jj) {
                    const int64_t j = j0 + jj;
                    if (causal && j > i) { S[jj] = -INFINITY; continue; }
                    const int8_t *k = Kh + j * d;
                    int32_t acc = 0;
                    for (int t = 0; t < d; ++t) acc += (int32_t)q[t] * (int32_t)k[t];
                    S[jj] = ((float)acc * sq) * skh[j];
                    if (S[jj] > bmax) bmax = S[jj];
                }
                const float m_new = (bmax > m) ? bmax : m;
                const float alpha = (m == -INFINITY) ? 0.0f : (float)exp((double)(m - m_new));
                float psum = 0.0f;
                for (int jj = 0; jj < nb; ++jj) {
                    P[jj] = (S[jj] == -INFINITY) ? 0.0f : orc_round_to_half((float)exp((double)(S[jj] - m_new)));
                    psum += P[jj];
                }
                l = l * alpha + psum;
                for (int c = 0; c < d; ++c) {
                    float pv = 0.0f;
                    for (int jj = 0; jj < nb; ++jj) pv += P[jj] * Vh[(j0 + jj) * d + c];
                    o[c] = o[c] * alpha + pv;
                }
                m = m_new;
            }
            for (int c = 0; c < d; ++c) O[r * d + c] = o[c] / l;
            if (l_out) l_out[r] = l;
            if (m_out) m_out[r] = m;
        }
        free(S); free(P); free(o);
    }
}

/*
 * Standard attention, Section 2.1: O = softmax(scale * Q K^T) V, row-wise softmax,
 * fp64 throughout, written out as the definition (max, exponentials, sum, divide).
 * Q, K, V are real [heads, N, d] in fp64.  `scale` is 1 for the paper's literal S = QK^T.
 */
void orc_attention_fp64(const double *Q, const double *K, const double *V,
                        int64_t heads, int64_t N, int d, int causal, double scale,
                        const int64_t *row_idx, int64_t n_rows, double *O)
{
    if (row_idx == NULL) n_rows = heads * N;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 16)
        for (int64_t r = 0; r < n_rows; ++r) {
            const int64_t g = row_idx ? row_idx[r] : r;
            const int64_t head = g / N, i = g % N;
            const double *q = Q + g * d;
            const double *Kh = K + head * N * d;
            const double *Vh = V + head * N * d;
            const int64_t nk = causal ? i + 1 : N;
            double mx = -INFINITY;
            for (int64_t j = 0; j < nk; ++j) {
                double acc = 0.0;
                for (int t = 0; t < d; ++t) acc += q[t] * Kh[j * d + t];
                s[j] = acc * scale;
                if (s[j] > mx) mx = s[j];
            }
            double sum = 0.0;
            for (int64_t j = 0; j < nk; ++j) { s[j] = exp(s[j] - mx); sum += s[j]; }
            for (int c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int64_t j = 0; j < nk; ++j) acc += s[j] * Vh[j * d + c];
                O[r * d + c] = acc / sum;
            }
        }
        free(s);
    }
}
