/*
 * ogq_oracle.c -- plain CPU oracle for per-bucket optimal gradient quantization.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * GPU library must compute.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may build, load or call it.  It shares no code, header, table or helper
 * with the HIP implementation and neither side includes the other.
 *
 * Source: "Optimal Gradient Quantization Condition for Communication-Efficient Distributed
 * Training" (Xu, Huo, Huang; arXiv 2002.11082).  Each function names the passage it follows.
 * Arithmetic is double precision over the fp32 inputs, except (a) the stochastic-rounding test,
 * which decides an integer code and is therefore taken in fp32 exactly as the device takes it, and
 * (b) the floor of the right-hand side of the discrete optimal condition, which decides which
 * bucket element becomes a level and is taken in exact (multi-word integer) arithmetic.
 *
 * Pins (see tests/test_oracle_*.py): Philox known-answer vectors; the exact sums against Python's
 * rationals; Q* against exhaustive minimisation of the discrete rounding error in exact rationals
 * and, at bucket sizes of 2048 .. 32768 elements, against floor(T) taken in exact rationals; s=3 global optimum; sweeps
 * never increase the error and end coordinate-wise optimal; uniform data gives the midpoint
 * (Remark after Theorem 1); endpoints are min/max (Corollary 1); BinGrad-b levels are the
 * conditional means, reduce to Scaled SignSGD on +-paired data and converge to 1-D 2-means;
 * random rounding is unbiased with variance (v-b_k)(b_{k+1}-v) by Monte Carlo; pack/unpack
 * round trip and hand-placed bits; decode-average special cases; clipping against a hand example,
 * the library standard deviation and its limiting cases; the comparison rules against their
 * closed forms (mean magnitude, TernGrad's {-max, 0, +max}, numpy's lower quantiles) and the
 * ordering of the quantization errors the paper reports.
 * No function here is "parity unpinned".
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC ogq_oracle.c -o libogq_oracle.so -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BINGRAD_B = 0, ORACLE_ORQ = 1, ORACLE_BINGRAD_PB = 2, ORACLE_ORQ_PAPER = 3,
       ORACLE_SCALED_SIGN = 4, ORACLE_EVEN = 5, ORACLE_LINEAR = 6 };

/* Levels per bucket: BinGrad-b, BinGrad-pb and Scaled SignSGD 2; ORQ 2^bits; ORQ with the paper's
 * level counts s = 2^K + 1 (Algorithm 1: 3, 5, 9 levels), whose indices need bits = K + 1 bits, and
 * the same counts for the evenly spaced (QSGD-s, TernGrad) and Linear-s comparison rules.
 * 0 = bad combination. */
uint32_t ogq_oracle_levels_per_bucket(uint32_t scheme, uint32_t bits)
{
    if (scheme == ORACLE_BINGRAD_B || scheme == ORACLE_BINGRAD_PB || scheme == ORACLE_SCALED_SIGN)
        return bits == 1 ? 2u : 0u;
    if (scheme == ORACLE_ORQ) return (bits >= 1 && bits <= 8) ? 1u << bits : 0u;
    if (scheme == ORACLE_ORQ_PAPER || scheme == ORACLE_EVEN || scheme == ORACLE_LINEAR)
        return (bits >= 2 && bits <= 8) ? (1u << (bits - 1)) + 1u : 0u;
    return 0u;
}

/* ------------------------------------------------------------------------------------------
 * Counter-based random numbers: Philox4x32 with 10 rounds, as published by Salmon, Moraes,
 * Dror and Shaw ("Parallel random numbers: as easy as 1, 2, 3", SC'11).  The paper does not
 * name a generator; the build's problem statement fixes this one.
 * ---------------------------------------------------------------------------------------- */
void ogq_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod_a = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod_b = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod_b;
        uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod_a;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform draw that belongs to the element with global index `index`:
 * four consecutive elements share one Philox block; the block counter is index/4 (64-bit,
 * split over the first two counter words), the key is the 64-bit seed, the element takes
 * word index%4, and the top 24 bits of that word give u in [0,1) on a 2^-24 grid. */
float ogq_oracle_uniform(uint64_t seed, uint64_t index)
{
    uint64_t block = index >> 2;
    uint32_t ctr[4] = { (uint32_t)block, (uint32_t)(block >> 32), 0u, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    ogq_oracle_philox4x32_10(ctr, key, r);
    return (float)(r[index & 3u] >> 8) * 0x1p-24f;
}

/* ------------------------------------------------------------------------------------------
 * BinGrad-b (Section 3.2, the deterministic two-level scheme and its optimal condition).
 * The threshold b0 starts at the bucket mean (the paper's stated implementation shortcut);
 * b_{-1} and b_1 are the means of the elements below / not below b0; each further iteration
 * moves b0 to the midpoint of the two levels (first relation of the optimal condition) and
 * recomputes the conditional means.  An empty lower side (constant bucket) takes b_{-1}=b_1.
 * Outputs: levels[0]=b_{-1}, levels[1]=b_1 rounded to fp32, *b0_out = the threshold of the
 * partition that produced them (code = v >= b0).
 * ---------------------------------------------------------------------------------------- */
void ogq_oracle_bingrad_bucket(const float* g, size_t n, uint32_t iters, float levels[2], float* b0_out)
{
    double total = 0.0;
    for (size_t i = 0; i < n; ++i) total += (double)g[i];
    float b0 = (float)(total / (double)n);
    double b_lo = 0.0, b_hi = 0.0;
    for (uint32_t it = 0;; ++it) {
        double sum_lo = 0.0, sum_hi = 0.0;
        size_t n_lo = 0, n_hi = 0;
        for (size_t i = 0; i < n; ++i) {
            if (g[i] < b0) { sum_lo += (double)g[i]; ++n_lo; }
            else           { sum_hi += (double)g[i]; ++n_hi; }
        }
        if (n_hi > 0) b_hi = sum_hi / (double)n_hi;
        if (n_lo > 0) b_lo = sum_lo / (double)n_lo;
        if (n_lo == 0) b_lo = b_hi;
        if (n_hi == 0) b_hi = b_lo;
        if (it == iters) break;
        b0 = (float)((b_lo + b_hi) * 0.5);
    }
    levels[0] = (float)b_lo;
    levels[1] = (float)b_hi;
    *b0_out = b0;
}

/* ------------------------------------------------------------------------------------------
 * BinGrad-pb (Section 3.2, the partially biased two-level scheme): levels -b_1 and +b_1; elements
 * outside [-b_1, b_1) are clamped to the nearer level, elements inside are rounded at random, which
 * is the random-rounding rule of Section 3.1 applied to the two levels (see the encode routine).
 * b_1 follows the scheme's optimal condition  b_1 * P(v > 0) = integral_{b_1}^inf v p(v) dv, which for
 * a bucket reads  b_1 * #{v > 0} = sum_{v >= b_1} v;  as the paper prescribes for discrete values, the
 * absolute difference of the two sides is minimised, here over the bucket's positive values (the
 * smaller value on a tie).  A bucket without positive values gets b_1 = 0.
 * ---------------------------------------------------------------------------------------- */
float ogq_oracle_bingrad_pb_level(const float* g, size_t n)
{
    size_t positives = 0;
    for (size_t i = 0; i < n; ++i) if (g[i] > 0.0f) ++positives;
    float best = 0.0f;
    double best_gap = -1.0;
    for (size_t i = 0; i < n; ++i) {
        float b = g[i];
        if (!(b > 0.0f)) continue;
        double tail = 0.0;
        for (size_t j = 0; j < n; ++j) if (g[j] >= b) tail += (double)g[j];
        double gap = fabs((double)b * (double)positives - tail);
        if (best_gap < 0.0 || gap < best_gap || (gap == best_gap && b < best)) {
            best_gap = gap;
            best = b;
        }
    }
    return best;
}

/* ------------------------------------------------------------------------------------------
 * Exact sums of fp32 values with small integer coefficients.  The floor of T = S / (R - L) below
 * decides which bucket element becomes a level, so it is taken in exact arithmetic: every fp32
 * value is an integer multiple of 2^-149, and a sum  c_1 v_1 + c_2 v_2 + ...  with |c_i| < 2^20 is
 * held as a signed fixed-point number in limbs of 32 bits (each limb an int64, so that tens of
 * thousands of partial products can be added before carries are propagated).
 *     value = sum_i limb[i] * 2^(32 i - 149)
 * ---------------------------------------------------------------------------------------- */
enum { EXACT_LIMBS = 12 };  /* 278 bits for |v| < 2^129 as multiples of 2^-149, 20 bits for the coefficient */
typedef struct { int64_t limb[EXACT_LIMBS]; } exact_sum_t;

static void exact_clear(exact_sum_t* a) { memset(a->limb, 0, sizeof a->limb); }

/* a += c * v */
static void exact_add(exact_sum_t* a, float v, int64_t c)
{
    uint32_t bits;
    memcpy(&bits, &v, sizeof bits);
    uint32_t biased = (bits >> 23) & 0xFFu, fraction = bits & 0x7FFFFFu;
    /* |v| = mantissa * 2^(position - 149): subnormals have position 0 and no hidden bit */
    uint64_t mantissa = biased ? (fraction | 0x800000u) : fraction;
    uint32_t position = biased ? biased - 1u : 0u;
    int negative = ((bits >> 31) != 0) != (c < 0);
    uint64_t magnitude = mantissa * (uint64_t)(c < 0 ? -c : c);         /* < 2^44 */
    unsigned __int128 shifted = (unsigned __int128)magnitude << (position % 32u);  /* < 2^76 */
    uint32_t first = position / 32u;                                   /* <= 7, so first + 2 < EXACT_LIMBS */
    for (int k = 0; k < 3; ++k) {
        int64_t piece = (int64_t)(uint32_t)(shifted >> (32 * k));
        a->limb[first + k] += negative ? -piece : piece;
    }
}

/* sign of the value: -1, 0 or +1 (carries are propagated on a copy) */
static int exact_sign(const exact_sum_t* a)
{
    int64_t limb[EXACT_LIMBS];
    int64_t carry = 0;
    for (int i = 0; i < EXACT_LIMBS; ++i) {
        int64_t t = a->limb[i] + carry;
        carry = t >> 32;                  /* floor division by 2^32 (arithmetic shift) */
        limb[i] = t - carry * 4294967296; /* in [0, 2^32) */
    }
    if (carry < 0) return -1;             /* what is left above the top limb carries the sign */
    if (carry > 0) return 1;
    for (int i = 0; i < EXACT_LIMBS; ++i) if (limb[i] != 0) return 1;
    return 0;
}

/* Test hook for the pins: sign of sum_i coefficient[i] * value[i], exactly. */
int ogq_oracle_exact_sign(const float* value, const int64_t* coefficient, size_t count)
{
    exact_sum_t a;
    exact_clear(&a);
    for (size_t i = 0; i < count; ++i) exact_add(&a, value[i], coefficient[i]);
    return exact_sign(&a);
}

/* ------------------------------------------------------------------------------------------
 * ORQ: one solve of the optimal condition for the middle level of three (Theorem 1, in the
 * simplified form of the second remark and its discrete version).
 *
 * With outer levels L < R fixed, the expected random-rounding error of the elements in [L,R],
 *     D(b) = sum_{L<=v<=b} (v-L)(b-v) + sum_{b<v<=R} (v-b)(R-v),
 * is continuous and piecewise linear in b with right-slope  S - (R-L) * #{b < v <= R},
 * where S = sum_{L<=v<=R} (v-L) is the numerator of the remark's right-hand side.  The slope
 * is non-decreasing in b, so D is minimal at the smallest data value b whose count
 * #{b < v <= R} does not exceed T = S/(R-L): the discrete optimal condition read as
 * "count above b_k equals the right-hand side", resolved to the exact minimiser.  When the
 * slope is exactly zero on an interval every point of it is optimal; the lower end is taken.
 *
 * T is a ratio of two sums of fp32 values, i.e. a rational number, and floor(T) = the largest
 * integer m with S - m (R-L) >= 0 is found in exact arithmetic (the expression is
 * sum_{L<=v<=R} v - (c - m) L - m R with c the number of elements in [L,R], and does not grow
 * with m), so that the level does not depend on the order or precision of a floating-point sum.
 *
 * x[0..n) must be sorted ascending.  Returns the level value.
 * ---------------------------------------------------------------------------------------- */
float ogq_oracle_qstar(const float* x, size_t n, float L, float R)
{
    if (!(L < R)) return L;
    exact_sum_t inside_sum;
    exact_clear(&inside_sum);
    size_t count_le_R = 0, inside = 0;
    for (size_t t = 0; t < n; ++t) {
        if (x[t] <= R) {
            ++count_le_R;
            if (x[t] >= L) { exact_add(&inside_sum, x[t], 1); ++inside; }
        }
    }
    /* floor(T): m = 0 gives S >= 0, m = inside gives sum_{[L,R]} (v - R) <= 0 */
    size_t lo = 0, hi = inside;
    while (lo < hi) {
        size_t mid = lo + (hi - lo + 1) / 2;
        exact_sum_t excess = inside_sum;                          /* S - mid (R - L) */
        exact_add(&excess, L, -(int64_t)(inside - mid));
        exact_add(&excess, R, -(int64_t)mid);
        if (exact_sign(&excess) >= 0) lo = mid;
        else hi = mid - 1;
    }
    size_t m = lo;                             /* how many elements may lie above b */
    size_t rank;                               /* 1-based rank of b among the sorted bucket */
    if (m >= count_le_R) rank = 1;
    else rank = count_le_R - m;
    if (rank < 1) rank = 1;
    float b = x[rank - 1];
    if (b < L) b = L;
    return b;
}

static int cmp_float_asc(const void* pa, const void* pb)
{
    float a = *(const float*)pa, b = *(const float*)pb;
    return (a > b) - (a < b);
}

/* Greedy recursive placement (Algorithm 1): the level in the middle of [l, r] is the solve
 * between the two outer levels, then both halves are treated the same way.  The paper states
 * it for s = 2^K + 1 levels, where (l+r)/2 is always an integer; for other s the middle index
 * is rounded down.  The recursion ends when no index lies strictly between l and r. */
static void orq_place(const float* x, size_t n, float* b, int l, int r)
{
    if (r - l < 2) return;
    int mid = (l + r) / 2;
    b[mid] = ogq_oracle_qstar(x, n, b[l], b[r]);
    orq_place(x, n, b, l, mid);
    orq_place(x, n, b, mid, r);
}

/* ORQ levels of one bucket: endpoints are the bucket minimum and maximum (Corollary 1), the
 * interior comes from the greedy placement, and `sweeps` rounds of re-solving every interior
 * level between its current neighbours (k ascending) move the greedy result towards a
 * solution of the coupled condition of Theorem 1.  `s` levels are written, non-decreasing. */
void ogq_oracle_orq_levels_bucket(const float* g, size_t n, uint32_t s, uint32_t sweeps, float* levels)
{
    float* x = (float*)malloc(n * sizeof(float));
    memcpy(x, g, n * sizeof(float));
    qsort(x, n, sizeof(float), cmp_float_asc);
    levels[0] = x[0];
    levels[s - 1] = x[n - 1];
    for (uint32_t k = 1; k + 1 < s; ++k) levels[k] = x[0];
    orq_place(x, n, levels, 0, (int)s - 1);
    for (uint32_t sw = 0; sw < sweeps; ++sw)
        for (uint32_t k = 1; k + 1 < s; ++k)
            levels[k] = ogq_oracle_qstar(x, n, levels[k - 1], levels[k + 1]);
    free(x);
}

/* ------------------------------------------------------------------------------------------
 * The level rules the paper compares against (Section 5, list of methods), per bucket.  They
 * feed the same random rounding, packing and decoding as ORQ.
 * ------------------------------------------------------------------------------------------ */

/* Scaled SignSGD (first equation of Section 3.2): Q(G) = (||G||_1 / dim G) * sign(G).  As a
 * two-level code: levels {-m, +m} with m = mean |v| (fp64 sum in index order, rounded to fp32
 * once); the code of an element is 1 when v >= 0 (reading: a zero, whose sign the formula leaves
 * at 0, goes to +m, since two levels have no zero). */
void ogq_oracle_scaled_sign_bucket(const float* g, size_t n, float levels[2])
{
    double sum = 0.0;
    for (size_t i = 0; i < n; ++i) sum += fabs((double)g[i]);
    float m = (float)(sum / (double)n);
    levels[0] = -m;
    levels[1] = m;
}

/* QSGD-s and TernGrad (Section 3.1, the paragraph after the random-rounding equation): s levels
 * evenly spaced from -||G|| to +||G||.  Reading: ||G|| is the largest magnitude M of the bucket
 * (TernGrad's scaler; any larger norm would only widen every interval), s is odd so that 0 is a
 * level, and b_k = M * (2k - (s-1)) / (s-1), k = 0..s-1, in fp64 rounded to fp32 once. */
void ogq_oracle_even_levels_bucket(const float* g, size_t n, uint32_t s, float* levels)
{
    double M = 0.0;
    for (size_t i = 0; i < n; ++i) if (fabs((double)g[i]) > M) M = fabs((double)g[i]);
    for (uint32_t k = 0; k < s; ++k)
        levels[k] = (float)(M * ((double)(2 * (long long)k) - (double)(s - 1)) / (double)(s - 1));
}

/* Linear-s (Section 5): s levels that divide the bucket's cumulative distribution linearly.
 * Reading: level k is the order statistic at the fraction k/(s-1) of the sorted bucket,
 * x_(floor(k (n-1) / (s-1))) with 0-based ranks, so that level 0 is the minimum and level s-1
 * the maximum and random rounding is defined for every element. */
void ogq_oracle_linear_levels_bucket(const float* g, size_t n, uint32_t s, float* levels)
{
    float* x = (float*)malloc(n * sizeof(float));
    memcpy(x, g, n * sizeof(float));
    qsort(x, n, sizeof(float), cmp_float_asc);
    for (uint32_t k = 0; k < s; ++k) levels[k] = x[(size_t)(((unsigned long long)k * (n - 1)) / (s - 1))];
    free(x);
}

/* Random rounding of one element (Section 3.1): v in [b_k, b_{k+1}] goes up to b_{k+1} with
 * probability (v-b_k)/(b_{k+1}-b_k).  k is the last level not above v (at most s-2); the
 * probability test is the division-free u*w < delta, in fp32, one rounding per operation. */
uint32_t ogq_oracle_orq_encode_element(float v, const float* levels, uint32_t s, float u)
{
    uint32_t not_above = 0;
    for (uint32_t k = 0; k < s; ++k) if (levels[k] <= v) ++not_above;
    uint32_t k = not_above > 0 ? not_above - 1 : 0;
    if (k > s - 2) k = s - 2;
    float w = levels[k + 1] - levels[k];
    float delta = v - levels[k];
    float scaled = u * w;
    return k + (scaled < delta ? 1u : 0u);
}

/* Bit-plane packing: element i sits in group i/64 at lane i%64; bit `lane` of 64-bit word
 * group*bits + p is bit p of the element's code. */
void ogq_oracle_pack(const uint8_t* codes, size_t n, uint32_t bits, uint64_t* words)
{
    size_t groups = (n + 63) / 64;
    memset(words, 0, groups * bits * sizeof(uint64_t));
    for (size_t i = 0; i < n; ++i)
        for (uint32_t p = 0; p < bits; ++p)
            if ((codes[i] >> p) & 1u) words[(i / 64) * bits + p] |= (uint64_t)1 << (i % 64);
}

void ogq_oracle_unpack(const uint64_t* words, size_t n, uint32_t bits, uint8_t* codes)
{
    for (size_t i = 0; i < n; ++i) {
        uint32_t c = 0;
        for (uint32_t p = 0; p < bits; ++p)
            c |= (uint32_t)((words[(i / 64) * bits + p] >> (i % 64)) & 1u) << p;
        codes[i] = (uint8_t)c;
    }
}

/* Gradient clipping before quantization (Section 5, the technique taken over from TernGrad):
 * clip(v) = sign(v) * min(|v|, c * sigma), sigma^2 = variance of the bucket's elements about their
 * mean (population variance, fp64), threshold rounded to fp32.  Applied per bucket, because every
 * bucket is quantized on its own.  c <= 0 leaves the bucket unchanged. */
void ogq_oracle_clip_bucket(const float* g, size_t n, float c, float* out)
{
    if (!(c > 0.0f)) {
        for (size_t i = 0; i < n; ++i) out[i] = g[i];
        return;
    }
    double sum = 0.0;
    for (size_t i = 0; i < n; ++i) sum += (double)g[i];
    double mean = sum / (double)n;
    double ss = 0.0;
    for (size_t i = 0; i < n; ++i) {
        double dv = (double)g[i] - mean;
        ss += dv * dv;
    }
    double sigma = sqrt(ss / (double)n);
    float limit = (float)((double)c * sigma);
    for (size_t i = 0; i < n; ++i) {
        float v = g[i];
        if (v > limit) v = limit;
        if (v < -limit) v = -limit;
        out[i] = v;
    }
}

/* Quantize a whole gradient bucket by bucket (bucket-based quantization, Section 5; the last
 * bucket is shorter when bucket_size does not divide n).  Writes (n/bucket_size rounded up)
 * * 2^bits level floats, one unpacked code per element, and, when thresholds != NULL and the
 * scheme is BinGrad-b, one b0 per bucket.  Returns 0, or -1 on bad arguments. */
int ogq_oracle_quantize_codes(const float* g, size_t n, uint32_t bucket_size, uint32_t bits,
                              uint32_t scheme, uint32_t level_iters, uint64_t seed,
                              uint64_t index_offset, float clip_factor, float* levels, uint8_t* codes,
                              float* thresholds)
{
    if (!g || !levels || !codes || bucket_size == 0 || bits == 0 || bits > 8) return -1;
    uint32_t s = ogq_oracle_levels_per_bucket(scheme, bits);
    if (s == 0) return -1;
    long long num_buckets = (long long)((n + bucket_size - 1) / bucket_size);
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (long long b = 0; b < num_buckets; ++b) {
        size_t begin = (size_t)b * bucket_size;
        size_t len = n - begin < bucket_size ? n - begin : bucket_size;
        float* gb = (float*)malloc(len * sizeof(float));
        ogq_oracle_clip_bucket(g + begin, len, clip_factor, gb);
        float* lv = levels + (size_t)b * s;
        if (scheme == ORACLE_BINGRAD_B) {
            float b0;
            ogq_oracle_bingrad_bucket(gb, len, level_iters, lv, &b0);
            if (thresholds) thresholds[b] = b0;
            for (size_t i = 0; i < len; ++i) codes[begin + i] = gb[i] >= b0 ? 1 : 0;
        } else if (scheme == ORACLE_SCALED_SIGN) {
            ogq_oracle_scaled_sign_bucket(gb, len, lv);
            if (thresholds) thresholds[b] = 0.0f;
            for (size_t i = 0; i < len; ++i) codes[begin + i] = gb[i] >= 0.0f ? 1 : 0;
        } else {
            if (scheme == ORACLE_BINGRAD_PB) {
                float b1 = ogq_oracle_bingrad_pb_level(gb, len);
                lv[0] = -b1;
                lv[1] = b1;
                if (thresholds) thresholds[b] = b1;
            } else if (scheme == ORACLE_EVEN) {
                ogq_oracle_even_levels_bucket(gb, len, s, lv);
            } else if (scheme == ORACLE_LINEAR) {
                ogq_oracle_linear_levels_bucket(gb, len, s, lv);
            } else {
                ogq_oracle_orq_levels_bucket(gb, len, s, level_iters, lv);
            }
            for (size_t i = 0; i < len; ++i) {
                float u = ogq_oracle_uniform(seed, index_offset + begin + i);
                codes[begin + i] = (uint8_t)ogq_oracle_orq_encode_element(gb[i], lv, s, u);
            }
        }
        free(gb);
    }
    return 0;
}

/* Quantize + pack: what one worker sends (Algorithm 2, "compute levels / quantize / encode"). */
int ogq_oracle_quantize(const float* g, size_t n, uint32_t bucket_size, uint32_t bits,
                        uint32_t scheme, uint32_t level_iters, uint64_t seed,
                        uint64_t index_offset, float clip_factor, float* levels, uint64_t* words)
{
    if (!words) return -1;
    uint8_t* codes = (uint8_t*)malloc(n ? n : 1);
    int rc = ogq_oracle_quantize_codes(g, n, bucket_size, bits, scheme, level_iters, seed,
                                       index_offset, clip_factor, levels, codes, NULL);
    if (rc == 0) ogq_oracle_pack(codes, n, bits, words);
    free(codes);
    return rc;
}

/* Server side of Algorithm 2: decode every worker's stream with that worker's levels and
 * average: out_i = (1/W) * sum_w levels_w[bucket(i)][code_{w,i}], summed in double. */
int ogq_oracle_dequantize_average(const uint64_t* const* words, const float* const* levels,
                                  uint32_t num_workers, size_t n, uint32_t bucket_size,
                                  uint32_t bits, uint32_t levels_per_bucket, float* out)
{
    if (!words || !levels || !out || num_workers == 0 || bucket_size == 0 || bits == 0 || bits > 8)
        return -1;
    if (levels_per_bucket == 0 || levels_per_bucket > (1u << bits)) return -1;
    uint32_t s = levels_per_bucket;
    long long nn = (long long)n;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (long long i = 0; i < nn; ++i) {
        size_t bucket = (size_t)i / bucket_size;
        double acc = 0.0;
        for (uint32_t w = 0; w < num_workers; ++w) {
            uint32_t c = 0;
            for (uint32_t p = 0; p < bits; ++p)
                c |= (uint32_t)((words[w][((size_t)i / 64) * bits + p] >> ((size_t)i % 64)) & 1u) << p;
            acc += (double)levels[w][bucket * s + c];
        }
        out[i] = (float)(acc / (double)num_workers);
    }
    return 0;
}

int ogq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void ogq_oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}
