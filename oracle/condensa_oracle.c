/*
 * CPU oracle for the compression (C) step of the L-C algorithm.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, scalar statement of
 * what the compression step computes; the GPU library is checked against it.
 * It shares no code with the GPU library and must never be called from it.
 *
 * What is written out here (paper passages in brackets):
 *   - unstructured magnitude pruning to an exact kept count: the weights of
 *     lower magnitude are set to zero [Background, magnitude-based
 *     thresholding; Section 3.3, pruning as D(Theta) = Theta with fewer non-zeros;
 *     Section 3.1, the magnitude threshold that realises a given sparsity];
 *     sparsity is the proportion of zero-valued parameters [Introduction];
 *   - low-precision approximation, binary32 -> binary16 and back [Background;
 *     Section 3.1 quantize/dequantize; Section 3.3 w_i = theta_i];
 *   - aggregation of filters (3-D blocks) and 2-D blocks followed by
 *     selection [Table 1, FilterPrune / BlockPrune; Section 3.1];
 *   - the C step as C(w) = argmin ||w - D(Theta)||^2 inside one augmented
 *     Lagrangian iteration with multipliers lambda and penalty mu
 *     [Section 3.3; constants in L-C Optimizer Settings].
 *
 * Readings where the paper is silent (identical on the GPU side by
 * specification, not by shared code):
 *   - kept count k = llround(density * N) (half away from zero), clamped;
 *   - order is by the bit pattern of |x| (so -0 == +0, inf above finite, NaN
 *     patterns above inf); ties go to the lowest flat index;
 *   - pruned positions hold +0.0; kept values are copied bit for bit;
 *   - structure keys are sums of squares accumulated in binary64 in memory
 *     order inside the structure (row-major inside a 2-D block);
 *   - L-C arithmetic is binary32, one rounding per operation, in the order
 *     t = lambda/mu; v = w - t; theta = prune(v); e = w - theta; p = mu*e;
 *     lambda' = lambda - p; g = p - lambda'.
 *
 * Selection is sort based: the k-th largest key of a fully sorted copy.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint64_t n;             /* population size                                   */
    uint64_t k;             /* kept count                                        */
    uint64_t n_gt;          /* keys strictly above the threshold key             */
    uint64_t n_tie_kept;    /* keys equal to the threshold that are kept         */
    uint64_t n_tie;         /* keys equal to the threshold                       */
    uint64_t threshold_key; /* k-th largest key; all ones when k == 0            */
    uint64_t tie_end;       /* ties with index < tie_end are the kept ones; n    */
                            /* when every tie is kept, 0 when k == 0             */
} oracle_select;

/* ---- kept count -------------------------------------------------------- */

uint64_t oracle_kept_count(double density, uint64_t n)
{
    double x = density * (double)n;
    long long r = llround(x);
    if (r < 0) return 0;
    if ((uint64_t)r > n) return n;
    return (uint64_t)r;
}

/* ---- keys -------------------------------------------------------------- */

static uint32_t f32_bits(float x) { uint32_t b; memcpy(&b, &x, 4); return b; }
static float bits_f32(uint32_t b) { float x; memcpy(&x, &b, 4); return x; }
static uint64_t f64_bits(double x) { uint64_t b; memcpy(&b, &x, 8); return b; }

/* magnitude key of a binary32 value: its bit pattern without the sign */
void oracle_magnitude_keys(const float* x, uint64_t n, uint64_t* keys)
{
    for (uint64_t i = 0; i < n; ++i) keys[i] = (uint64_t)(f32_bits(x[i]) & 0x7FFFFFFFu);
}

/* key of a non-negative binary64 aggregate: its bit pattern without the sign */
void oracle_aggregate_keys(const double* s, uint64_t n, uint64_t* keys)
{
    for (uint64_t i = 0; i < n; ++i) keys[i] = f64_bits(s[i]) & 0x7FFFFFFFFFFFFFFFull;
}

static int cmp_desc_u64(const void* a, const void* b)
{
    uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
    return (x < y) - (x > y);
}

void oracle_sort_desc(uint64_t* keys, uint64_t n)
{
    qsort(keys, (size_t)n, sizeof(uint64_t), cmp_desc_u64);
}

/* ---- selection --------------------------------------------------------- */

/*
 * keys        : the population in flat-index order
 * sorted_desc : the same keys sorted in descending order
 * keep[i]     : 1 for the k elements of largest key, ties to the lowest index
 */
void oracle_select_keep(const uint64_t* keys, const uint64_t* sorted_desc, uint64_t n,
                        uint64_t k, oracle_select* sel, uint8_t* keep)
{
    sel->n = n;
    sel->k = k;
    if (k == 0) {
        sel->n_gt = 0; sel->n_tie_kept = 0; sel->n_tie = 0;
        sel->threshold_key = UINT64_MAX; sel->tie_end = 0;
        for (uint64_t i = 0; i < n; ++i) keep[i] = 0;
        return;
    }
    const uint64_t T = sorted_desc[k - 1];
    uint64_t n_gt = 0, n_tie = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (keys[i] > T) ++n_gt;
        else if (keys[i] == T) ++n_tie;
    }
    const uint64_t r = k - n_gt;
    uint64_t seen = 0, last_kept_tie = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (keys[i] > T) keep[i] = 1;
        else if (keys[i] == T && seen < r) { keep[i] = 1; ++seen; last_kept_tie = i; }
        else keep[i] = 0;
    }
    sel->n_gt = n_gt;
    sel->n_tie_kept = r;
    sel->n_tie = n_tie;
    sel->threshold_key = T;
    sel->tie_end = (r == n_tie) ? n : last_kept_tie + 1;
}

/* theta[i] = keep ? x[i] : +0.0  (values copied bit for bit) */
void oracle_apply_keep(const float* x, const uint8_t* keep, uint64_t n, float* theta)
{
    for (uint64_t i = 0; i < n; ++i) theta[i] = keep[i] ? x[i] : bits_f32(0u);
}

/* ---- binary32 <-> binary16 -------------------------------------------- */

/* round to nearest, ties to even; overflow to infinity; gradual underflow */
static uint16_t f32_to_f16_bits(uint32_t b)
{
    const uint16_t sign = (uint16_t)((b >> 16) & 0x8000u);
    const uint32_t a = b & 0x7FFFFFFFu;
    if (a > 0x7F800000u)                         /* NaN: quiet, top payload bits */
        return (uint16_t)(sign | 0x7E00u | ((a >> 13) & 0x03FFu));
    if (a == 0x7F800000u) return (uint16_t)(sign | 0x7C00u);
    const uint32_t e = a >> 23;                  /* biased binary32 exponent     */
    const uint32_t m = a & 0x007FFFFFu;
    if (e >= 143u) return (uint16_t)(sign | 0x7C00u);          /* |x| >= 2^16    */
    if (e >= 113u) {                             /* normal binary16 (before rounding) */
        uint32_t h = ((e - 112u) << 10) | (m >> 13);
        const uint32_t rem = m & 0x1FFFu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h; /* carry may reach inf */
        return (uint16_t)(sign | h);
    }
    if (e < 102u) return sign;                   /* |x| < 2^-25 -> zero          */
    /* subnormal binary16: value = M * 2^(e-150), unit 2^-24, shift = 126 - e in [14,24] */
    const uint32_t M = m | 0x00800000u;
    const uint32_t s = 126u - e;
    uint32_t h = M >> s;
    const uint32_t rem = M & ((1u << s) - 1u);
    const uint32_t half = 1u << (s - 1u);
    if (rem > half || (rem == half && (h & 1u))) ++h;
    return (uint16_t)(sign | h);
}

/* exact widening */
static uint32_t f16_to_f32_bits(uint16_t h)
{
    const uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    const uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t m = h & 0x03FFu;
    if (e == 31u) return sign | 0x7F800000u | (m << 13);
    if (e == 0u) {
        if (m == 0u) return sign;
        int shift = 0;                           /* normalise the subnormal      */
        while (!(m & 0x0400u)) { m <<= 1; ++shift; }
        m &= 0x03FFu;
        return sign | ((uint32_t)(113 - shift) << 23) | (m << 13);
    }
    return sign | ((e + 112u) << 23) | (m << 13);
}

void oracle_quantize_f16(const float* x, uint64_t n, uint16_t* q, float* dq /* nullable */)
{
    for (uint64_t i = 0; i < n; ++i) {
        const uint16_t h = f32_to_f16_bits(f32_bits(x[i]));
        q[i] = h;
        if (dq) dq[i] = bits_f32(f16_to_f32_bits(h));
    }
}

void oracle_dequantize_f16(const uint16_t* q, uint64_t n, float* dq)
{
    for (uint64_t i = 0; i < n; ++i) dq[i] = bits_f32(f16_to_f32_bits(q[i]));
}

/* ---- bfloat16: Quantize(dtype) with the other common 16-bit floating-point type (Table 1; the Conclusions
 * name further quantization data types as an extension).  bfloat16 is the upper half of binary32:
 * 1 sign, 8 exponent, 7 fraction bits.  Round to nearest, ties to even, decided on the 16 dropped bits;
 * a carry out of the fraction moves into the exponent (the largest finite values round to infinity);
 * NaN stays NaN: sign and upper payload bits kept, quiet bit set. */
static uint16_t f32_to_bf16_bits(uint32_t u)
{
    const uint32_t upper = u >> 16, dropped = u & 0xFFFFu;
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)(upper | 0x0040u);
    if (dropped > 0x8000u) return (uint16_t)(upper + 1u);
    if (dropped == 0x8000u) return (uint16_t)(upper + (upper & 1u));
    return (uint16_t)upper;
}

void oracle_quantize_bf16(const float* x, uint64_t n, uint16_t* q, float* dq /* nullable */)
{
    for (uint64_t i = 0; i < n; ++i) {
        const uint16_t h = f32_to_bf16_bits(f32_bits(x[i]));
        q[i] = h;
        if (dq) dq[i] = bits_f32((uint32_t)h << 16);
    }
}

void oracle_dequantize_bf16(const uint16_t* q, uint64_t n, float* dq)
{
    for (uint64_t i = 0; i < n; ++i) dq[i] = bits_f32((uint32_t)q[i] << 16);
}

/* ---- 8-bit floating point: Quantize(dtype) with the two 8-bit formats of the OCP 8-bit floating point
 * specification (Table 1; low-precision approximation = a fixed codebook, Background).
 *   format 0, E4M3: 1 sign, 4 exponent (bias 7), 3 fraction bits; no infinity; S.1111.111 is NaN;
 *                   largest finite value 448, smallest subnormal 2^-9.
 *   format 1, E5M2: 1 sign, 5 exponent (bias 15), 2 fraction bits; IEEE-like infinities and NaNs;
 *                   largest finite value 57344, smallest subnormal 2^-16.
 * A code's value is written out from the definition; quantization is the definition too: the nearest
 * finite value of the format, found by search over all of them, ties to the code with the even fraction.
 * Reading where the paper says nothing: finite inputs beyond the largest finite value saturate to it
 * (the usual choice for weights); E5M2 keeps infinite inputs infinite, E4M3 (no infinity) saturates them;
 * NaN gives the format's NaN with the sign kept (E5M2: quiet NaN S.11111.10) and widens to the
 * binary32 quiet NaN S.0x7FC00000. */
static int fp8_geometry(int format, int* mant_bits, int* bias, int* max_code, int* has_inf)
{
    if (format == 0) { *mant_bits = 3; *bias = 7;  *max_code = 0x7E; *has_inf = 0; return 1; }
    if (format == 1) { *mant_bits = 2; *bias = 15; *max_code = 0x7B; *has_inf = 1; return 1; }
    return 0;
}

/* value of the non-negative finite code c (0 <= c <= max_code) */
static double fp8_code_value(int c, int mant_bits, int bias)
{
    const int e = c >> mant_bits, m = c & ((1 << mant_bits) - 1);
    if (e == 0) return ldexp((double)m, 1 - bias - mant_bits);
    return ldexp(1.0 + ldexp((double)m, -mant_bits), e - bias);
}

static uint8_t f32_to_fp8(float x, int mant_bits, int bias, int max_code, int has_inf)
{
    const uint32_t u = f32_bits(x);
    const uint8_t sign = (uint8_t)((u >> 31) << 7);
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint8_t)(sign | (has_inf ? 0x7E : 0x7F));
    if (a == 0x7F800000u) return (uint8_t)(sign | (has_inf ? 0x7C : max_code));
    const double v = fabs((double)x);
    if (v >= fp8_code_value(max_code, mant_bits, bias)) return (uint8_t)(sign | max_code);   /* saturation */
    int best = 0;
    double best_err = v;                                   /* distance to code 0 */
    for (int c = 1; c <= max_code; ++c) {
        const double err = fabs(v - fp8_code_value(c, mant_bits, bias));
        if (err < best_err || (err == best_err && (c & 1) == 0)) { best = c; best_err = err; }
    }
    return (uint8_t)(sign | best);
}

static float fp8_to_f32(uint8_t c, int mant_bits, int bias, int max_code, int has_inf)
{
    const uint32_t sign = (uint32_t)(c & 0x80u) << 24;
    const int mag = c & 0x7F;
    if (mag > max_code) {
        if (has_inf && mag == 0x7C) return bits_f32(sign | 0x7F800000u);
        return bits_f32(sign | 0x7FC00000u);
    }
    const float v = (float)fp8_code_value(mag, mant_bits, bias);   /* exact: at most 4 significant bits */
    return bits_f32(sign | f32_bits(v));
}

int oracle_quantize_fp8(const float* x, uint64_t n, int format, uint8_t* q, float* dq /* nullable */)
{
    int mb, bias, mc, inf;
    if (!fp8_geometry(format, &mb, &bias, &mc, &inf)) return -1;
    for (uint64_t i = 0; i < n; ++i) {
        const uint8_t c = f32_to_fp8(x[i], mb, bias, mc, inf);
        q[i] = c;
        if (dq) dq[i] = fp8_to_f32(c, mb, bias, mc, inf);
    }
    return 0;
}

int oracle_dequantize_fp8(const uint8_t* q, uint64_t n, int format, float* dq)
{
    int mb, bias, mc, inf;
    if (!fp8_geometry(format, &mb, &bias, &mc, &inf)) return -1;
    for (uint64_t i = 0; i < n; ++i) dq[i] = fp8_to_f32(q[i], mb, bias, mc, inf);
    return 0;
}

/* ---- structure aggregates --------------------------------------------- */

/* filters of one tensor [n_filters, len]: S_f = sum of squares, binary64, memory order */
void oracle_filter_sumsq(const float* w, uint64_t n_filters, uint64_t len, double* s)
{
    for (uint64_t f = 0; f < n_filters; ++f) {
        double acc = 0.0;
        for (uint64_t e = 0; e < len; ++e) {
            const double x = (double)w[f * len + e];
            acc = acc + x * x;
        }
        s[f] = acc;
    }
}

/* 2-D blocks of one matrix [rows, cols]; block id row-major over the block grid;
 * inside a block the elements are added in row-major order */
void oracle_block_sumsq(const float* w, uint64_t rows, uint64_t cols, uint64_t bh, uint64_t bw, double* s)
{
    const uint64_t gr = rows / bh, gc = cols / bw;
    for (uint64_t br = 0; br < gr; ++br)
        for (uint64_t bc = 0; bc < gc; ++bc) {
            double acc = 0.0;
            for (uint64_t y = 0; y < bh; ++y)
                for (uint64_t x = 0; x < bw; ++x) {
                    const double v = (double)w[(br * bh + y) * cols + bc * bw + x];
                    acc = acc + v * v;
                }
            s[br * gc + bc] = acc;
        }
}

void oracle_norms(const double* s, uint64_t n, float* norms)
{
    for (uint64_t i = 0; i < n; ++i) norms[i] = (float)sqrt(s[i]);
}

/* theta/mask of one tensor given the keep flag of each of its structures */
void oracle_filter_apply(const float* w, uint64_t n_filters, uint64_t len, const uint8_t* keep,
                         float* theta, uint8_t* mask)
{
    for (uint64_t f = 0; f < n_filters; ++f)
        for (uint64_t e = 0; e < len; ++e) {
            const uint64_t i = f * len + e;
            theta[i] = keep[f] ? w[i] : bits_f32(0u);
            mask[i] = keep[f] ? 1 : 0;
        }
}

void oracle_block_apply(const float* w, uint64_t rows, uint64_t cols, uint64_t bh, uint64_t bw,
                        const uint8_t* keep, float* theta, uint8_t* mask)
{
    const uint64_t gc = cols / bw;
    for (uint64_t r = 0; r < rows; ++r)
        for (uint64_t c = 0; c < cols; ++c) {
            const uint64_t b = (r / bh) * gc + (c / bw);
            const uint64_t i = r * cols + c;
            theta[i] = keep[b] ? w[i] : bits_f32(0u);
            mask[i] = keep[b] ? 1 : 0;
        }
}

/* ---- L-C step ---------------------------------------------------------- */

/* v = w - lambda/mu, binary32, one rounding per operation */
void oracle_lc_shifted(const float* w, const float* lambda, uint64_t n, float mu, float* v)
{
    for (uint64_t i = 0; i < n; ++i) {
        volatile float t = lambda[i] / mu;
        volatile float d = w[i] - t;
        v[i] = d;
    }
}

/* theta = keep ? v : +0; e = w - theta; p = mu*e; lambda' = lambda - p; g = p - lambda' */
void oracle_lc_update(const float* w, const float* lambda, const float* v, const uint8_t* keep,
                      uint64_t n, float mu, float* theta, float* lambda_out, float* grad)
{
    for (uint64_t i = 0; i < n; ++i) {
        const float th = keep[i] ? v[i] : bits_f32(0u);
        volatile float e = w[i] - th;
        volatile float p = mu * e;
        volatile float l = lambda[i] - p;
        volatile float g = p - l;
        theta[i] = th;
        lambda_out[i] = l;
        grad[i] = g;
    }
}

/* ---- n-D blocks with ragged edges (BlockPrune over blocks of any dimensionality, Table 1) ------------------
 * The tensor is viewed as 4-D [d0,d1,d2,d3] (leading dims 1 for lower ranks), the block as
 * [b0,b1,b2,b3].  The block grid has ceil(d/b) cells per dim; cells at the far edges are smaller.
 * Block id is row-major over the grid; inside a block the squares are added in row-major order. */
static uint64_t ceil_div_u64(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

void oracle_block_sumsq_nd(const float* w, const uint64_t* d, const uint64_t* b, double* s)
{
    const uint64_t G0 = ceil_div_u64(d[0], b[0]), G1 = ceil_div_u64(d[1], b[1]),
                   G2 = ceil_div_u64(d[2], b[2]), G3 = ceil_div_u64(d[3], b[3]);
    for (uint64_t g0 = 0; g0 < G0; ++g0)
    for (uint64_t g1 = 0; g1 < G1; ++g1)
    for (uint64_t g2 = 0; g2 < G2; ++g2)
    for (uint64_t g3 = 0; g3 < G3; ++g3) {
        double acc = 0.0;
        for (uint64_t x0 = g0 * b[0]; x0 < (g0 + 1) * b[0] && x0 < d[0]; ++x0)
        for (uint64_t x1 = g1 * b[1]; x1 < (g1 + 1) * b[1] && x1 < d[1]; ++x1)
        for (uint64_t x2 = g2 * b[2]; x2 < (g2 + 1) * b[2] && x2 < d[2]; ++x2)
        for (uint64_t x3 = g3 * b[3]; x3 < (g3 + 1) * b[3] && x3 < d[3]; ++x3) {
            const double v = (double)w[((x0 * d[1] + x1) * d[2] + x2) * d[3] + x3];
            acc = acc + v * v;
        }
        s[((g0 * G1 + g1) * G2 + g2) * G3 + g3] = acc;
    }
}

void oracle_block_apply_nd(const float* w, const uint64_t* d, const uint64_t* b, const uint8_t* keep,
                           float* theta, uint8_t* mask)
{
    const uint64_t G1 = ceil_div_u64(d[1], b[1]), G2 = ceil_div_u64(d[2], b[2]), G3 = ceil_div_u64(d[3], b[3]);
    for (uint64_t x0 = 0; x0 < d[0]; ++x0)
    for (uint64_t x1 = 0; x1 < d[1]; ++x1)
    for (uint64_t x2 = 0; x2 < d[2]; ++x2)
    for (uint64_t x3 = 0; x3 < d[3]; ++x3) {
        const uint64_t i = ((x0 * d[1] + x1) * d[2] + x2) * d[3] + x3;
        const uint64_t u = (((x0 / b[0]) * G1 + x1 / b[1]) * G2 + x2 / b[2]) * G3 + x3 / b[3];
        theta[i] = keep[u] ? w[i] : bits_f32(0u);
        mask[i] = keep[u] ? 1 : 0;
    }
}

/* ---- L-C step with the composed scheme Compose([Prune(), Quantize(float16)]) (Evaluation, Objective 1) ----
 * Theta = binary16(prune(v)); D(Theta) = exact widening; the multiplier update uses D(Theta):
 * e = w - D(Theta); p = mu*e; lambda' = lambda - p; g = p - lambda'. */
void oracle_lc_update_pq(const float* w, const float* lambda, const float* v, const uint8_t* keep,
                         uint64_t n, float mu, uint16_t* theta16, float* theta, float* lambda_out, float* grad)
{
    for (uint64_t i = 0; i < n; ++i) {
        const float pruned = keep[i] ? v[i] : bits_f32(0u);
        const uint16_t h = f32_to_f16_bits(f32_bits(pruned));
        const float th = bits_f32(f16_to_f32_bits(h));
        volatile float e = w[i] - th;
        volatile float p = mu * e;
        volatile float l = lambda[i] - p;
        volatile float g = p - l;
        theta16[i] = h;
        theta[i] = th;
        lambda_out[i] = l;
        grad[i] = g;
    }
}

/* Memory footprint objective (Evaluation, Objective 1): the number of non-zero parameters; the
 * footprint in bytes is that count times the size of the stored type.  -0 counts as zero. */
uint64_t oracle_count_nonzero_f32(const float* x, uint64_t n)
{
    uint64_t c = 0;
    for (uint64_t i = 0; i < n; ++i) c += (f32_bits(x[i]) & 0x7FFFFFFFu) != 0u;
    return c;
}

uint64_t oracle_count_nonzero_f16(const uint16_t* x, uint64_t n)
{
    uint64_t c = 0;
    for (uint64_t i = 0; i < n; ++i) c += (x[i] & 0x7FFFu) != 0u;
    return c;
}

uint64_t oracle_count_nonzero_u8(const uint8_t* x, uint64_t n)
{
    uint64_t c = 0;
    for (uint64_t i = 0; i < n; ++i) c += (x[i] & 0x7Fu) != 0u;
    return c;
}

/* ---- thinning: physically remove zero structures (Section 3.4, Network Thinning, final phase) ----
 * out[o', i', r] = w[keep_out[o'], keep_in[i'], r] for a tensor viewed as [Cout, Cin, kh*kw];
 * a NULL list keeps every index of that dimension. */
void oracle_thin(const float* w, uint64_t c_out, uint64_t c_in, uint64_t ksize,
                 const int32_t* keep_out, uint64_t n_out, const int32_t* keep_in, uint64_t n_in, float* out)
{
    (void)c_out;
    for (uint64_t o = 0; o < n_out; ++o)
        for (uint64_t i = 0; i < n_in; ++i)
            for (uint64_t r = 0; r < ksize; ++r) {
                const uint64_t so = keep_out ? (uint64_t)keep_out[o] : o;
                const uint64_t si = keep_in ? (uint64_t)keep_in[i] : i;
                out[(o * n_in + i) * ksize + r] = w[(so * c_in + si) * ksize + r];
            }
}

/* ---- learning-step update with the L-C penalty folded in (Section 3.3: the L step trains w with a
 * quadratic regularisation term; L-C Optimizer Settings: SGD with momentum 0.9) ------------------
 * gradient of  L(w) + mu/2 ||w - theta - lambda/mu||^2  is  grad L + mu (w - theta) - lambda;
 * momentum update  buf' = m buf + g;  w' = w - lr buf'.  binary32, one rounding per operation. */
void oracle_lc_sgd_step(const float* w, const float* grad_loss, const float* theta, const float* lambda,
                        const float* buf, uint64_t n, float mu, float lr, float momentum,
                        float* w_out, float* buf_out)
{
    for (uint64_t i = 0; i < n; ++i) {
        volatile float t1 = w[i] - theta[i];
        volatile float t2 = mu * t1;
        volatile float t3 = grad_loss[i] + t2;
        volatile float t4 = t3 - lambda[i];
        volatile float t5 = momentum * buf[i];
        volatile float b = t5 + t4;
        volatile float t6 = lr * b;
        volatile float wn = w[i] - t6;
        buf_out[i] = b;
        w_out[i] = wn;
    }
}
