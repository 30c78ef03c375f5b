/*
 * Plain CPU executor of a collective schedule.  TEST INFRASTRUCTURE: this is
 * the oracle the GPU library is compared with; it shares nothing with it.
 *
 * What it computes (sections 3.3 and 3.5 and the first paragraph of section 4
 * of the paper: a schedule says which chunk is sent, from where to where, in
 * which synchronous step, and with which chunk it is reduced):
 *
 *   every rank n owns one buffer of G chunks, chunk c at element offset
 *   c * elems_per_chunk in every buffer (global chunk numbering, section
 *   3.2.2); optionally a slot map says instead that chunk c sits in slot
 *   slot[c*P + n] of rank n's buffer (the paper numbers chunks globally but
 *   does not prescribe where a node stores them: a node only needs room for
 *   the chunks it ever holds);
 *
 *   for s = 0 .. S-1, for the sends of step s in array order
 *     COPY   (c, n -> n'):  buf[n'][c] = buf[n][c]
 *     REDUCE (c, n -> n'):  all REDUCE sends of this step into the same
 *                           (c, n') form one group, sources n_1..n_k in array
 *                           order, and per element
 *                               acc = widen(buf[n'][c][e])
 *                               acc = acc + widen(buf[n_j][c][e])   j = 1..k
 *                               buf[n'][c][e] = narrow(acc)
 *
 *   widen/narrow: identity for int32 (the sum wraps modulo 2^32) and fp32
 *   (IEEE binary32 add, round to nearest even); fp16 is widened exactly to
 *   fp32, summed in fp32, and narrowed ONCE per group with round to nearest
 *   even.  Between steps the buffers hold fp16.
 *
 * The schedule must have passed the validator: no (c, n) is both read and
 * written within a step, so processing sends one after the other equals the
 * "all reads see the start of the step" semantics without a snapshot.
 *
 * The only parallelism is OpenMP across the element index e, which never
 * changes the order of operations applied to any one element.
 *
 * Build: gcc -O2 -fno-fast-math -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { DT_I32 = 0, DT_F32 = 1, DT_F16 = 2 };
enum { OP_COPY = 0, OP_REDUCE = 1 };

/* IEEE binary16 -> binary32, exact. */
static float half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t exp = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ff;
    uint32_t bits;
    float f;
    if (exp == 0) {
        /* zero or subnormal: man * 2^-24, exact in binary32 */
        f = (float)man * 5.9604644775390625e-08f;
        memcpy(&bits, &f, 4);
        bits |= sign;
    } else if (exp == 0x1f) {
        bits = sign | 0x7f800000u | (man << 13);
    } else {
        bits = sign | ((exp + 112u) << 23) | (man << 13);
    }
    memcpy(&f, &bits, 4);
    return f;
}

/* IEEE binary32 -> binary16, round to nearest, ties to even. */
static uint16_t float_to_half(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t a = x & 0x7fffffffu;
    if (a > 0x7f800000u)                         /* NaN: quiet, keep top payload bits */
        return (uint16_t)(sign | 0x7e00u | ((a >> 13) & 0x3ffu));
    if (a >= 0x477ff000u)                        /* >= 65520: rounds to infinity (also inf itself) */
        return (uint16_t)(sign | 0x7c00u);
    if (a >= 0x38800000u) {                      /* >= 2^-14: normal binary16 */
        uint32_t e = (a >> 23) - 112u;
        uint32_t m = a & 0x7fffffu;
        uint32_t h = (e << 10) | (m >> 13);
        uint32_t rem = m & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u)))
            h++;                                  /* a carry runs into the exponent, as it should */
        return (uint16_t)(sign | h);
    }
    /* below 2^-14: result is q * 2^-24 with q = RNE(value * 2^24) */
    uint32_t e = a >> 23;
    if (e < 102u)                                 /* value < 2^-25 (or a binary32 subnormal): rounds to zero */
        return sign;
    uint32_t m = (a & 0x7fffffu) | 0x800000u;     /* 24-bit significand, value = m * 2^(e-150) */
    uint32_t shift = 126u - e;                    /* 14 .. 24 */
    uint32_t q = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t halfway = 1u << (shift - 1u);
    if (rem > halfway || (rem == halfway && (q & 1u)))
        q++;
    return (uint16_t)(sign | q);
}

/* exported for the conversion pins */
void oracle_f16_to_f32(const uint16_t *in, float *out, int64_t n)
{
    for (int64_t i = 0; i < n; i++) out[i] = half_to_float(in[i]);
}

void oracle_f32_to_f16(const float *in, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; i++) out[i] = float_to_half(in[i]);
}

int32_t oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static void copy_chunk(void *dst, const void *src, int64_t n, int elem_bytes, int nthreads)
{
    if (elem_bytes == 4) {
        uint32_t *d = (uint32_t *)dst;
        const uint32_t *s = (const uint32_t *)src;
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; e++) d[e] = s[e];
    } else {
        uint16_t *d = (uint16_t *)dst;
        const uint16_t *s = (const uint16_t *)src;
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; e++) d[e] = s[e];
    }
}

static void reduce_group(int dtype, void *dst, const void **srcs, int k, int64_t n, int nthreads)
{
    if (dtype == DT_I32) {
        uint32_t *d = (uint32_t *)dst;
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; e++) {
            uint32_t acc = d[e];
            for (int j = 0; j < k; j++) acc += ((const uint32_t *)srcs[j])[e];
            d[e] = acc;
        }
    } else if (dtype == DT_F32) {
        float *d = (float *)dst;
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; e++) {
            float acc = d[e];
            for (int j = 0; j < k; j++) acc = acc + ((const float *)srcs[j])[e];
            d[e] = acc;
        }
    } else {
        uint16_t *d = (uint16_t *)dst;
#pragma omp parallel for num_threads(nthreads) schedule(static)
        for (int64_t e = 0; e < n; e++) {
            float acc = half_to_float(d[e]);
            for (int j = 0; j < k; j++) acc = acc + half_to_float(((const uint16_t *)srcs[j])[e]);
            d[e] = float_to_half(acc);
        }
    }
}

/*
 * sends: num_sends rows of 5 int32 (chunk, src, dst, step, op), array order
 * significant.  bufs: P host pointers, each G * elems_per_chunk elements, or
 * slots_per_rank * elems_per_chunk when a slot map (G x P int32, -1 = rank
 * never holds the chunk) is given; slot == NULL means slot c for every rank.
 * first_elem / num_elems: the element range WITHIN every chunk to process
 * (0, elems_per_chunk for the whole thing); elements are independent, so a
 * sub-range is the same computation on a sample.
 * Returns 0, or -1 on a bad argument.
 */
int32_t oracle_execute(int32_t P, int32_t G, int64_t elems_per_chunk, int32_t dtype, int32_t S,
                       int64_t num_sends, const int32_t *sends, void *const *bufs,
                       int64_t first_elem, int64_t num_elems, int32_t nthreads,
                       const int32_t *slot, int32_t slots_per_rank)
{
    if (P < 1 || G < 1 || elems_per_chunk < 0 || S < 0 || num_sends < 0) return -1;
    if (dtype != DT_I32 && dtype != DT_F32 && dtype != DT_F16) return -1;
    if (first_elem < 0 || num_elems < 0 || first_elem + num_elems > elems_per_chunk) return -1;
    if (nthreads < 1) nthreads = 1;
    int eb = (dtype == DT_F16) ? 2 : 4;
    uint8_t *done = (uint8_t *)calloc((size_t)(num_sends ? num_sends : 1), 1);
    const void **srcs = (const void **)malloc(sizeof(void *) * (size_t)(num_sends ? num_sends : 1));
    if (!done || !srcs) { free(done); free(srcs); return -1; }
    for (int64_t i = 0; i < num_sends; i++) {
        const int32_t *t = sends + 5 * i;
        if (t[0] < 0 || t[0] >= G || t[1] < 0 || t[1] >= P || t[2] < 0 || t[2] >= P ||
            t[3] < 0 || t[3] >= S || (t[4] != OP_COPY && t[4] != OP_REDUCE)) {
            free(done); free(srcs); return -1;
        }
        if (slot) {
            int32_t a = slot[(int64_t)t[0] * P + t[1]], b = slot[(int64_t)t[0] * P + t[2]];
            if (a < 0 || a >= slots_per_rank || b < 0 || b >= slots_per_rank) { free(done); free(srcs); return -1; }
        }
    }
    for (int32_t s = 0; s < S; s++) {
        for (int64_t i = 0; i < num_sends; i++) {
            const int32_t *t = sends + 5 * i;
            if (t[3] != s || done[i]) continue;
            int32_t c = t[0], n = t[1], m = t[2];
#define CHUNK_AT(rank) (((int64_t)(slot ? slot[(int64_t)c * P + (rank)] : c) * elems_per_chunk + first_elem) * eb)
            if (t[4] == OP_COPY) {
                copy_chunk((uint8_t *)bufs[m] + CHUNK_AT(m), (const uint8_t *)bufs[n] + CHUNK_AT(n), num_elems, eb, nthreads);
                done[i] = 1;
            } else {
                int k = 0;
                for (int64_t j = i; j < num_sends; j++) {
                    const int32_t *u = sends + 5 * j;
                    if (u[3] == s && u[4] == OP_REDUCE && u[0] == c && u[2] == m && !done[j]) {
                        srcs[k++] = (const uint8_t *)bufs[u[1]] + CHUNK_AT(u[1]);
                        done[j] = 1;
                    }
                }
                reduce_group(dtype, (uint8_t *)bufs[m] + CHUNK_AT(m), srcs, k, num_elems, nthreads);
            }
        }
    }
    free(done);
    free(srcs);
    return 0;
}
