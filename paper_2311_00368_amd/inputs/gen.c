/*
 * Seeded synthetic inputs for the CSR SPMM / SDDMM / FusedMM kernels.
 *
 * Test and benchmark infrastructure only: this file draws random patterns and
 * random dense values and holds none of the arithmetic of the three
 * operations.  Both the HIP path and the CPU oracle are fed from here, so the
 * two see bit-identical operands.
 *
 * The paper (section "Sparse Matrix Collection") only says that its inputs are
 * randomized matrices at 70-90 % sparsity; the distributions below are this
 * repository's synthetic stand-ins: an i.i.d. Bernoulli pattern, and a pattern
 * with log-normally distributed row lengths.
 *
 * Random numbers come from a stateless counter-based generator,
 * u64 = mix(key(seed, stream) + (index+1)*golden), i.e. one splitmix64 step
 * from a stream-dependent start state.  Every value depends only on
 * (seed, stream, index), so generation is order-independent and can be
 * parallelised over rows.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GOLDEN 0x9E3779B97F4A7C15ull

static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

static inline uint64_t stream_key(uint64_t seed, uint64_t stream) {
    return mix64(mix64(seed + GOLDEN) ^ mix64(stream * GOLDEN + 0x632BE59BD9B4E019ull));
}

static inline uint64_t draw_u64(uint64_t key, uint64_t index) {
    return mix64(key + (index + 1) * GOLDEN);
}

/* uniform in [0,1) with 53 random bits */
static inline double draw_u01(uint64_t key, uint64_t index) {
    return (double)(draw_u64(key, index) >> 11) * 0x1.0p-53;
}

/* uniform in (0,1] (safe argument for log) */
static inline double draw_u01_open0(uint64_t key, uint64_t index) {
    return (double)((draw_u64(key, index) >> 11) + 1) * 0x1.0p-53;
}

/* standard normal by Box-Muller from draws 2*index and 2*index+1 */
static inline double draw_normal(uint64_t key, uint64_t index) {
    const double u1 = draw_u01_open0(key, 2 * index);
    const double u2 = draw_u01(key, 2 * index + 1);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

/* raw generator output, exposed so tests can check determinism and statistics */
void gen_raw_u64(uint64_t seed, uint64_t stream, uint64_t first, uint64_t n, uint64_t *out) {
    const uint64_t key = stream_key(seed, stream);
    for (uint64_t t = 0; t < n; ++t) out[t] = draw_u64(key, first + t);
}

/* out[t] = lo + (hi-lo)*u01, rounded to FP32 */
void gen_uniform_f32(uint64_t seed, uint64_t stream, uint64_t n, float lo, float hi, float *out) {
    const uint64_t key = stream_key(seed, stream);
    const double a = lo, w = (double)hi - (double)lo;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < (int64_t)n; ++t)
        out[t] = (float)(a + w * draw_u01(key, (uint64_t)t));
}

/* out[t] ~ N(0,1), rounded to FP32 */
void gen_normal_f32(uint64_t seed, uint64_t stream, uint64_t n, float *out) {
    const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < (int64_t)n; ++t)
        out[t] = (float)draw_normal(key, (uint64_t)t);
}

/*
 * Bernoulli pattern: entry (i,j) is stored iff u01(seed, stream, i*K+j) < p.
 * Two passes: count (fills rowptr), then fill (colidx, ascending in each row).
 * Call with colidx == NULL to get rowptr only (rowptr[M] = nnz), then allocate
 * and call again.
 */
void gen_bernoulli_csr(uint64_t seed, uint64_t stream, int32_t M, int32_t K, double p,
                       int32_t *rowptr, int32_t *colidx) {
    const uint64_t key = stream_key(seed, stream);
    if (!colidx) {
        rowptr[0] = 0;
#pragma omp parallel for schedule(static)
        for (int32_t i = 0; i < M; ++i) {
            int32_t c = 0;
            const uint64_t base = (uint64_t)i * (uint64_t)K;
            for (int32_t j = 0; j < K; ++j) c += draw_u01(key, base + (uint64_t)j) < p;
            rowptr[i + 1] = c;
        }
        for (int32_t i = 0; i < M; ++i) rowptr[i + 1] += rowptr[i];
        return;
    }
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < M; ++i) {
        int32_t w = rowptr[i];
        const uint64_t base = (uint64_t)i * (uint64_t)K;
        for (int32_t j = 0; j < K; ++j)
            if (draw_u01(key, base + (uint64_t)j) < p) colidx[w++] = j;
    }
}

/*
 * Skewed pattern: row length = clip(rint(exp(mu + sigma*z_i)), 1, K) with z_i
 * standard normal from `len_stream`; the columns of a row are a uniform sample
 * without replacement, taken by sequential selection sampling over 0..K-1
 * (column j is taken with probability (still needed)/(columns left)), which
 * yields them in ascending order.  Same two-call protocol as above.
 */
void gen_lognormal_csr(uint64_t seed, uint64_t stream, uint64_t len_stream, int32_t M, int32_t K,
                       double mu, double sigma, int32_t *rowptr, int32_t *colidx) {
    const uint64_t key = stream_key(seed, stream);
    const uint64_t lkey = stream_key(seed, len_stream);
    if (!colidx) {
        rowptr[0] = 0;
        for (int32_t i = 0; i < M; ++i) {
            double len = rint(exp(mu + sigma * draw_normal(lkey, (uint64_t)i)));
            if (len < 1.0) len = 1.0;
            if (len > (double)K) len = (double)K;
            rowptr[i + 1] = rowptr[i] + (int32_t)len;
        }
        return;
    }
#pragma omp parallel for schedule(dynamic, 16)
    for (int32_t i = 0; i < M; ++i) {
        int32_t need = rowptr[i + 1] - rowptr[i];
        int32_t w = rowptr[i];
        const uint64_t base = (uint64_t)i * (uint64_t)K;
        for (int32_t j = 0; j < K && need > 0; ++j) {
            if (draw_u01(key, base + (uint64_t)j) * (double)(K - j) < (double)need) {
                colidx[w++] = j;
                --need;
            }
        }
    }
}
