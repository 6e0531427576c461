/*
 * CPU oracle for the local share of FlexLink's collectives.
 *
 * THIS FILE IS TEST INFRASTRUCTURE, NOT THE PRODUCT. It is called only by the
 * test-suite, by the smoke check and by the benchmark's CPU-baseline leg. The
 * HIP library never links, includes or calls anything in here, and nothing in
 * here includes or calls the HIP library.
 *
 * What is computed follows the paper's statement of the two collectives it
 * supports (Evaluation, "System and Workload Configuration": AllReduce and
 * AllGather; "End-to-End Performance": ring AllReduce = reduce-scatter with a
 * reduce-sum followed by an all-gather; "Limitations and Future Work": the
 * reduction is a sum).  The paper is silent on element type, accumulation
 * precision and summation order; the reading taken here is: contributions are
 * added strictly in rank order 0..N-1, starting from rank 0's value, in IEEE
 * binary32 with round-to-nearest-even, and the accumulator is rounded once to
 * the element type at the end.  The abstract's "lossless" claim is read as:
 * the result does not depend on how the message is split over paths, so the
 * oracle has no notion of paths at all.
 *
 * Parity pins: library routines on special cases, exact rational brute force,
 * hand-derived values (see the test-suite).  The paper prints no numerical
 * example of a collective, so nothing here is pinned to a value from the paper.
 *
 * Plain loops, one element at a time, no blocking or reordering.  The OpenMP
 * pragma only partitions the independent element index over threads.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bfloat16 -> binary32: bfloat16 is the upper 16 bits of a binary32, so the
 * widening is exact. */
static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary32 -> bfloat16, round to nearest, ties to even.  Dropping 16 mantissa
 * bits: add half an output ulp minus one, plus the lowest kept bit, then
 * truncate.  A carry out of the mantissa moves into the exponent, which is the
 * correct rounding up to the next binade or to infinity.  NaN keeps its sign
 * and upper payload and has its quiet bit forced so that it stays a NaN. */
static uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lowest_kept = (u >> 16) & 1u;
    u += 0x7fffu + lowest_kept;
    return (uint16_t)(u >> 16);
}

/* IEEE binary16 -> binary32 (exact).  1 sign, 5 exponent (bias 15), 10 mantissa
 * bits.  Normal numbers re-bias the exponent (127 - 15 = 112) and left-align
 * the mantissa; subnormals are m * 2^-24; exponent 31 is infinity or NaN. */
static float f16_bits_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t m = h & 0x3ffu;
    uint32_t u;
    if (e == 0) {
        float mag = (float)m * 0x1p-24f;            /* exact: m < 1024 */
        memcpy(&u, &mag, sizeof u);
        u |= sign;
    } else if (e == 31) {
        u = sign | 0x7f800000u | (m << 13);
    } else {
        u = sign | ((e + 112u) << 23) | (m << 13);
    }
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary32 -> IEEE binary16, round to nearest, ties to even.  Magnitudes of
 * 2^16 and above (and anything that rounds up to 2^16) become infinity; below
 * the smallest normal 2^-14 the result is a multiple of 2^-24 (subnormal),
 * obtained by shifting the 24-bit significand right and rounding what falls
 * off.  NaN stays NaN (quiet bit set, upper payload kept). */
static uint16_t f32_to_f16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t mag = u & 0x7fffffffu;
    uint32_t e32 = mag >> 23;
    uint32_t mant = mag & 0x7fffffu;
    if (mag > 0x7f800000u)
        return (uint16_t)(sign | 0x7e00u | (mant >> 13));
    if (mag >= 0x47800000u)                         /* |f| >= 2^16, or infinity */
        return (uint16_t)(sign | 0x7c00u);
    if (e32 >= 113) {                               /* normal binary16 range */
        uint32_t h = ((e32 - 112u) << 10) | (mant >> 13);
        uint32_t rem = mant & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u)))
            h += 1;                                 /* may carry up to 0x7c00 = infinity */
        return (uint16_t)(sign | h);
    }
    /* subnormal or zero result: value = sig * 2^(e32 - 150), quantum 2^-24 */
    uint32_t shift = 126u - e32;
    if (e32 == 0 || shift > 25)
        return sign;                                /* below 2^-26: rounds to zero */
    uint32_t sig = mant | 0x800000u;
    uint32_t h = sig >> shift;
    uint32_t rem = sig & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (h & 1u)))
        h += 1;                                     /* may carry up to 0x0400 = smallest normal */
    return (uint16_t)(sign | h);
}

/* AllReduce(sum), binary32 elements.
 * b: n pointers to `count` floats each (rank r's contribution is b[r]).
 * out[i] = ((b[0][i] + b[1][i]) + b[2][i]) + ... + b[n-1][i]. */
void oracle_allreduce_f32(const float *const *b, int n, size_t count, float *out)
{
    long long i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < (long long)count; ++i) {
        float acc = b[0][i];
        for (int r = 1; r < n; ++r)
            acc = acc + b[r][i];
        out[i] = acc;
    }
}

/* AllReduce(sum), bfloat16 elements given as raw 16-bit patterns.
 * Accumulate in binary32 in rank order, round once at the end. */
void oracle_allreduce_bf16(const uint16_t *const *b, int n, size_t count, uint16_t *out)
{
    long long i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < (long long)count; ++i) {
        float acc = bf16_bits_to_f32(b[0][i]);
        for (int r = 1; r < n; ++r)
            acc = acc + bf16_bits_to_f32(b[r][i]);
        out[i] = f32_to_bf16_bits(acc);
    }
}

/* AllReduce(sum), IEEE binary16 elements given as raw 16-bit patterns.
 * Accumulate in binary32 in rank order, round once at the end. */
void oracle_allreduce_f16(const uint16_t *const *b, int n, size_t count, uint16_t *out)
{
    long long i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < (long long)count; ++i) {
        float acc = f16_bits_to_f32(b[0][i]);
        for (int r = 1; r < n; ++r)
            acc = acc + f16_bits_to_f32(b[r][i]);
        out[i] = f32_to_f16_bits(acc);
    }
}

/* AllGather: out is the concatenation, in rank order, of n slices of
 * slice_bytes bytes each.  Bytes are moved untouched. */
void oracle_allgather(const void *const *in, int n, size_t slice_bytes, void *out)
{
    unsigned char *o = (unsigned char *)out;
    for (int r = 0; r < n; ++r) {
        const unsigned char *s = (const unsigned char *)in[r];
        long long j;
#pragma omp parallel for schedule(static)
        for (j = 0; j < (long long)slice_bytes; ++j)
            o[(size_t)r * slice_bytes + (size_t)j] = s[j];
    }
}

/* AllToAll, the receive buffer of rank `rank`: piece r of out is what rank r
 * addresses to `rank`, i.e. piece number `rank` of rank r's buffer.  Pieces are
 * piece_bytes long; bytes are moved untouched. */
void oracle_alltoall(const void *const *in, int n, int rank, size_t piece_bytes, void *out)
{
    unsigned char *o = (unsigned char *)out;
    for (int r = 0; r < n; ++r) {
        const unsigned char *s = (const unsigned char *)in[r] + (size_t)rank * piece_bytes;
        for (size_t j = 0; j < piece_bytes; ++j)
            o[(size_t)r * piece_bytes + j] = s[j];
    }
}

/* Scalar conversions exported so that the tests can pin them on their own. */
float oracle_bf16_to_f32(uint16_t h) { return bf16_bits_to_f32(h); }
uint16_t oracle_f32_to_bf16(float f) { return f32_to_bf16_bits(f); }

/* The same rounding over an array of binary32 bit patterns, so that NaN
 * payloads and every other pattern reach it unchanged. */
void oracle_f32_bits_to_bf16(const uint32_t *bits, size_t n, uint16_t *out)
{
    for (size_t i = 0; i < n; ++i) {
        float f;
        memcpy(&f, &bits[i], sizeof f);
        out[i] = f32_to_bf16_bits(f);
    }
}

float oracle_f16_to_f32(uint16_t h) { return f16_bits_to_f32(h); }

void oracle_f32_bits_to_f16(const uint32_t *bits, size_t n, uint16_t *out)
{
    for (size_t i = 0; i < n; ++i) {
        float f;
        memcpy(&f, &bits[i], sizeof f);
        out[i] = f32_to_f16_bits(f);
    }
}

/* Thread control for the timed baseline: how many threads the loops above
 * will use, and a setter. */
int oracle_get_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}
