/*
 * ROBE-Z CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, sequential-by-default C implementation of what the ROBE-Z
 * embedding path computes (Desai, Chou, Shrivastava, "Random Offset Block
 * Embedding Array", arXiv 2108.02191, Section 3).  It exists to check the GPU
 * library and to be timed beside it as a CPU baseline.  Nothing in the product
 * package may import, link or execute it; only tests/, the smoke check and
 * the benchmark's cpu_baseline leg do.  It shares no code, header, table or
 * helper with the HIP path.
 *
 * Conventions (all 0-based):
 *   e  table id  = feature column index                     (Section 3.1, "Multiple embedding tables")
 *   x  token id  = the int64 index read as an unsigned 64-bit integer
 *   c  chunk id  = floor(i / Z),  i = element position in [0, d)
 *   coef[8] = { A_h, B_h, C_h, D_h, A_g, B_g, C_g, D_g }     (Section 3.2, text under the idx equation)
 *
 * Every integer formula is evaluated over the integers with a 128-bit
 * accumulator, so no intermediate can wrap.  Floating-point sums are carried
 * in double and rounded to float once.
 *
 * Parity pins live in tests/test_oracle_*.py: arbitrary-precision brute force
 * for h, g and idx; the explicit sketching matrix (Section 4) for forward and
 * backward; the published SplitMix64 vectors for the coefficient stream;
 * torch.optim.Adagrad and torch.optim.SGD (CPU, float64) for the optimizer
 * steps.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef unsigned __int128 u128;

/* ------------------------------------------------------------------ */
/* Coefficient stream.  The paper says only that the coefficients are  */
/* "randomly chosen" (Section 3.2).  The library documents how they    */
/* come from a seed: a SplitMix64 stream (Steele, Lea, Flood, OOPSLA   */
/* 2014) started at `seed`; multipliers are 1 + r mod (P-1), additive  */
/* constants are r mod P, drawn in the order A_h B_h C_h D_h A_g B_g   */
/* C_g D_g.  This is that recipe written out again, independently.     */
/* ------------------------------------------------------------------ */
uint64_t oracle_splitmix64_next(uint64_t *state)
{
    *state += 0x9E3779B97F4A7C15ULL;
    uint64_t z = *state;
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

void oracle_init_hash(uint64_t seed, uint64_t P, uint64_t coef[8])
{
    uint64_t st = seed;
    for (int k = 0; k < 8; ++k) {
        uint64_t r = oracle_splitmix64_next(&st);
        int additive = (k == 3 || k == 7);
        coef[k] = additive ? (r % P) : (1 + r % (P - 1));
    }
}

/* h(e,x,c) = ((A_h e + B_h x + C_h c + D_h) mod P) mod m   (Section 3.2, idx equation, line for h) */
uint64_t oracle_h(const uint64_t coef[8], uint64_t P, uint64_t m,
                  uint64_t e, uint64_t x, uint64_t c)
{
    u128 t = (u128)coef[0] * e + (u128)coef[1] * x + (u128)coef[2] * c + (u128)coef[3];
    return (uint64_t)((t % P) % m);
}

/* g(e,x,i) = 2 * (((A_g e + B_g x + C_g i + D_g) mod P) mod 2) - 1   (Section 3.1, hash equation, line for g) */
int oracle_g(const uint64_t coef[8], uint64_t P, int use_sign,
             uint64_t e, uint64_t x, uint64_t i)
{
    if (!use_sign) return 1;
    u128 t = (u128)coef[4] * e + (u128)coef[5] * x + (u128)coef[6] * i + (u128)coef[7];
    return 2 * (int)((t % P) % 2) - 1;
}

/*
 * idx(e,x,i) = (h(e,x,floor(i/Z)) + i mod Z) mod m   (Section 3.2, idx equation), for Z <= d.
 *
 * Z > d (Section 3.3; Appendix, "ROBE-Z": the table is flattened row by row and cut into chunks of
 * Z, each chunk hashed to its place): element i of token x is entry n = x*d + i of table e's
 * flattened rows, in chunk floor(n / Z) at place n mod Z.  With d | Z a chunk holds r = Z/d whole
 * embeddings, so the chunk is floor(x / r) and the place is (x mod r)*d + i; the chunk id takes the
 * token's seat in h and the chunk number c is 0.
 */
uint64_t oracle_idx(const uint64_t coef[8], uint64_t P, uint64_t m, uint32_t d, uint32_t Z,
                    uint64_t e, uint64_t x, uint64_t i)
{
    if (Z <= d) {
        uint64_t c = i / Z, j = i % Z;
        return (oracle_h(coef, P, m, e, x, c) + j) % m;
    }
    uint64_t r = Z / d;
    uint64_t chunk = x / r, place = (x % r) * d + i;
    return (oracle_h(coef, P, m, e, chunk, 0) + place) % m;
}

/* Chunk offsets of n lookups; lookup k belongs to feature k mod F.  out[k*C + c], C = d/Z (Z <= d). */
void oracle_offsets(const uint64_t coef[8], uint64_t P, uint64_t m, uint32_t d, uint32_t Z,
                    const int64_t *indices, int64_t n, int32_t F, int64_t *out)
{
    if (Z > d) { /* one entry per lookup: where element 0 of the embedding sits */
        for (int64_t k = 0; k < n; ++k)
            out[k] = (int64_t)oracle_idx(coef, P, m, d, Z, (uint64_t)(k % F), (uint64_t)indices[k], 0);
        return;
    }
    uint32_t C = d / Z;
    for (int64_t k = 0; k < n; ++k)
        for (uint32_t c = 0; c < C; ++c)
            out[k * C + c] = (int64_t)oracle_h(coef, P, m, (uint64_t)(k % F), (uint64_t)indices[k], c);
}

/* Element signs of n lookups; out[k*d + i] in {-1,+1}. */
void oracle_signs(const uint64_t coef[8], uint64_t P, uint32_t d, int use_sign,
                  const int64_t *indices, int64_t n, int32_t F, int8_t *out)
{
    for (int64_t k = 0; k < n; ++k)
        for (uint32_t i = 0; i < d; ++i)
            out[k * d + i] = (int8_t)oracle_g(coef, P, use_sign, (uint64_t)(k % F), (uint64_t)indices[k], i);
}

/*
 * Forward (Section 3.2, forward equation; E = G o P).
 *   offsets == NULL : single-hot, indices[batch*F], out[k,:] = E_f(indices[k]), k = b*F + f.
 *   offsets != NULL : bag-sum, bag k = b*F + f holds indices[offsets[k] .. offsets[k+1]);
 *                     out[k,:] = sum over the bag of E_f(x_t), duplicates counted, empty bag -> 0.
 * Sums are taken in index order in double and rounded once.
 */
void oracle_forward(const uint64_t coef[8], uint64_t P, uint64_t m, uint32_t d, uint32_t Z, int use_sign,
                    const float *array, const int64_t *indices, const int64_t *offsets,
                    int64_t batch, int32_t F, float *out, int threads)
{
    int64_t rows = batch * (int64_t)F;
    (void)threads;
#pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
    for (int64_t k = 0; k < rows; ++k) {
        uint64_t e = (uint64_t)(k % F);
        int64_t t0 = offsets ? offsets[k] : k;
        int64_t t1 = offsets ? offsets[k + 1] : k + 1;
        for (uint32_t i = 0; i < d; ++i) {
            if (offsets == NULL) {
                /* single-hot: one term, a copy with an exact sign flip */
                uint64_t x = (uint64_t)indices[k];
                float v = array[oracle_idx(coef, P, m, d, Z, e, x, i)];
                out[k * (int64_t)d + i] = oracle_g(coef, P, use_sign, e, x, i) < 0 ? -v : v;
                continue;
            }
            double acc = 0.0;
            for (int64_t t = t0; t < t1; ++t) {
                uint64_t x = (uint64_t)indices[t];
                uint64_t j = oracle_idx(coef, P, m, d, Z, e, x, i);
                acc += (double)oracle_g(coef, P, use_sign, e, x, i) * (double)array[j];
            }
            out[k * (int64_t)d + i] = (float)acc;
        }
    }
}

/*
 * Backward (Section 3.1, backward-pass equation):
 *   grad_array[j] += sum over (k, t, i) with idx(f, x_t, i) == j of g(f, x_t, i) * grad_out[k, i];
 * every token of a bag receives its bag's gradient row.  Accumulates into the
 * caller's double buffers; abs_sum (may be NULL) receives the sum of |term|
 * per slot, which tests use as the scale of the rounding-error bound.
 * With threads > 1 the same loops run under OpenMP with atomic double adds
 * (timing leg of the benchmark); threads <= 1 is the sequential reference.
 */
void oracle_backward(const uint64_t coef[8], uint64_t P, uint64_t m, uint32_t d, uint32_t Z, int use_sign,
                     const float *grad_out, const int64_t *indices, const int64_t *offsets,
                     int64_t batch, int32_t F, double *grad_array, double *abs_sum, int threads)
{
    int64_t rows = batch * (int64_t)F;
    (void)threads;
#pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
    for (int64_t k = 0; k < rows; ++k) {
        uint64_t e = (uint64_t)(k % F);
        int64_t t0 = offsets ? offsets[k] : k;
        int64_t t1 = offsets ? offsets[k + 1] : k + 1;
        for (int64_t t = t0; t < t1; ++t) {
            uint64_t x = (uint64_t)indices[t];
            for (uint32_t i = 0; i < d; ++i) {
                uint64_t j = oracle_idx(coef, P, m, d, Z, e, x, i);
                double term = (double)oracle_g(coef, P, use_sign, e, x, i) * (double)grad_out[k * (int64_t)d + i];
#pragma omp atomic
                grad_array[j] += term;
                if (abs_sum) {
#pragma omp atomic
                    abs_sum[j] += fabs(term);
                }
            }
        }
    }
}

/*
 * Low-precision array (Section 2 notes that quantisation composes with the method; no format is
 * fixed there).  The array is stored as bfloat16: the upper 16 bits of the float32 pattern.
 * float32 -> bfloat16 rounds to nearest, ties to even, on the 16 dropped bits; NaN stays NaN (quiet
 * bit set, payload truncated); bfloat16 -> float32 appends 16 zero bits and is exact.
 */
uint16_t oracle_bf16_from_f32(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16, drop = u & 0xFFFFu;
    if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) keep += 1u;   /* may carry into the exponent: correct */
    return (uint16_t)keep;
}

float oracle_f32_from_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float v;
    memcpy(&v, &u, 4);
    return v;
}

void oracle_array_to_bf16(const float *src, uint16_t *dst, uint64_t n)
{
    for (uint64_t j = 0; j < n; ++j) dst[j] = oracle_bf16_from_f32(src[j]);
}

/* Forward (ROBE-Z forward equation) on a bfloat16 array: every element read is widened exactly,
 * then the definition is that of oracle_forward (single-hot: a copy with an exact sign flip; bags:
 * sums in double, rounded once to float32). */
void oracle_forward_bf16(const uint64_t coef[8], uint64_t P, uint64_t m, uint32_t d, uint32_t Z, int use_sign,
                         const uint16_t *array, const int64_t *indices, const int64_t *offsets,
                         int64_t batch, int32_t F, float *out)
{
    int64_t rows = batch * (int64_t)F;
    for (int64_t k = 0; k < rows; ++k) {
        uint64_t e = (uint64_t)(k % F);
        int64_t t0 = offsets ? offsets[k] : k;
        int64_t t1 = offsets ? offsets[k + 1] : k + 1;
        for (uint32_t i = 0; i < d; ++i) {
            if (offsets == NULL) {
                uint64_t x = (uint64_t)indices[k];
                float v = oracle_f32_from_bf16(array[oracle_idx(coef, P, m, d, Z, e, x, i)]);
                out[k * (int64_t)d + i] = oracle_g(coef, P, use_sign, e, x, i) < 0 ? -v : v;
                continue;
            }
            double acc = 0.0;
            for (int64_t t = t0; t < t1; ++t) {
                uint64_t x = (uint64_t)indices[t];
                acc += (double)oracle_g(coef, P, use_sign, e, x, i) *
                       (double)oracle_f32_from_bf16(array[oracle_idx(coef, P, m, d, Z, e, x, i)]);
            }
            out[k * (int64_t)d + i] = (float)acc;
        }
    }
}

/*
 * Tables of different embedding dimensions sharing the one array (Section 3.2,
 * "Multiple embedding tables": all tables, even with varying dimensions, share
 * the array; the table id is an argument of h and g).  Table f has dimension
 * dims[f]; its embedding is the same construction with d = dims[f].  A sample's
 * output is the concatenation of its F embeddings: row b of out holds
 * D = sum(dims) floats, table f at column col[f] = dims[0] + ... + dims[f-1].
 * Single-hot (offsets == NULL) copies with an exact sign flip; bags sum in double.
 */
void oracle_forward_mixed(const uint64_t coef[8], uint64_t P, uint64_t m, const uint32_t *dims, uint32_t Z,
                          int use_sign, const float *array, const int64_t *indices, const int64_t *offsets,
                          int64_t batch, int32_t F, float *out)
{
    int64_t D = 0;
    for (int32_t f = 0; f < F; ++f) D += dims[f];
    for (int64_t b = 0; b < batch; ++b) {
        int64_t col = 0;
        for (int32_t f = 0; f < F; ++f) {
            int64_t k = b * (int64_t)F + f;
            uint32_t d = dims[f];
            int64_t t0 = offsets ? offsets[k] : k;
            int64_t t1 = offsets ? offsets[k + 1] : k + 1;
            for (uint32_t i = 0; i < d; ++i) {
                float *dst = &out[b * D + col + i];
                if (offsets == NULL) {
                    uint64_t x = (uint64_t)indices[k];
                    float v = array[oracle_idx(coef, P, m, d, Z, (uint64_t)f, x, i)];
                    *dst = oracle_g(coef, P, use_sign, (uint64_t)f, x, i) < 0 ? -v : v;
                    continue;
                }
                double acc = 0.0;
                for (int64_t t = t0; t < t1; ++t) {
                    uint64_t x = (uint64_t)indices[t];
                    acc += (double)oracle_g(coef, P, use_sign, (uint64_t)f, x, i) *
                           (double)array[oracle_idx(coef, P, m, d, Z, (uint64_t)f, x, i)];
                }
                *dst = (float)acc;
            }
            col += d;
        }
    }
}

/* Backward of the above (backward-pass equation of Section 3.1 with d = dims[f] per table);
 * grad_out has the layout of out.  Accumulates into double buffers; abs_sum may be NULL. */
void oracle_backward_mixed(const uint64_t coef[8], uint64_t P, uint64_t m, const uint32_t *dims, uint32_t Z,
                           int use_sign, const float *grad_out, const int64_t *indices, const int64_t *offsets,
                           int64_t batch, int32_t F, double *grad_array, double *abs_sum)
{
    int64_t D = 0;
    for (int32_t f = 0; f < F; ++f) D += dims[f];
    for (int64_t b = 0; b < batch; ++b) {
        int64_t col = 0;
        for (int32_t f = 0; f < F; ++f) {
            int64_t k = b * (int64_t)F + f;
            uint32_t d = dims[f];
            int64_t t0 = offsets ? offsets[k] : k;
            int64_t t1 = offsets ? offsets[k + 1] : k + 1;
            for (int64_t t = t0; t < t1; ++t) {
                uint64_t x = (uint64_t)indices[t];
                for (uint32_t i = 0; i < d; ++i) {
                    uint64_t j = oracle_idx(coef, P, m, d, Z, (uint64_t)f, x, i);
                    double term = (double)oracle_g(coef, P, use_sign, (uint64_t)f, x, i) * (double)grad_out[b * D + col + i];
                    grad_array[j] += term;
                    if (abs_sum) abs_sum[j] += fabs(term);
                }
            }
            col += d;
        }
    }
}

/*
 * Adagrad step (Duchi, Hazan, Singer 2011; not part of the paper, named by the
 * workload): for every slot j, in double on float-stored operands,
 *   s'[j] = s[j] + g[j]^2 ;  M'[j] = M[j] - lr * g[j] / (sqrt(s'[j]) + eps) ;  g[j] = 0.
 * A slot with g == 0 is left exactly unchanged, so the dense sweep equals an
 * update of the touched slots only.
 */
void oracle_adagrad(float *array, float *state, float *grad, uint64_t m, double lr, double eps, int threads)
{
    (void)threads;
#pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
    for (int64_t j = 0; j < (int64_t)m; ++j) {
        double g = (double)grad[j];
        double s = (double)state[j] + g * g;
        double w = (double)array[j] - lr * g / (sqrt(s) + eps);
        state[j] = (float)s;
        array[j] = (float)w;
        grad[j] = 0.0f;
    }
}

/*
 * Plain SGD step, the optimizer the paper trains DLRM with (Appendix, hyper-parameter table:
 * SGD, learning rate 1.0):  M'[j] = M[j] - lr * g[j] ;  g[j] = 0.  Double arithmetic on
 * float-stored operands, one rounding.  A slot with g == 0 is left exactly unchanged.
 */
void oracle_sgd(float *array, float *grad, uint64_t m, double lr, int threads)
{
    (void)threads;
#pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
    for (int64_t j = 0; j < (int64_t)m; ++j) {
        array[j] = (float)((double)array[j] - lr * (double)grad[j]);
        grad[j] = 0.0f;
    }
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
