// C ABI of the ROBE-Z library (see include/robe.h): argument validation,
// launch geometry and kernel selection.  All device work is in robe_kernels.h
// and robe_backward_dedup.h.
//
// Tuning knobs, read from the environment at call time (for experiments and for
// tests that must reach every kernel variant; the defaults are the measured
// best choices):
//   ROBE_TUNE_FWD, ROBE_TUNE_BWD = "V,consec"   lane layout: V in {1,2,4} elements per lane,
//                                               consec 1 = consecutive elements of one chunk,
//                                               0 = strided; "0,0" = shape-generic kernel
//   ROBE_TUNE_TL                                 lookups per wavefront tile (single-hot kernels)
//   ROBE_TUNE_XCD = 0 | 1 | 2                    row order: memory order / table by table per XCD /
//                                               the latter even for tiny launches
//   ROBE_TUNE_BWD_MODE = direct | dedup          backward scatter strategy
//   ROBE_TUNE_KEY_BITS = 8..31                   key bits the backward sort looks at
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/robe.h"
#include "robe_kernels.h"
#include <rocprim/device/device_radix_sort.hpp>

#include "robe_backward_dedup.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char *what)
{
    hipError_t st = hipGetLastError();
    if (st != hipSuccess) return fail(ROBE_EHIP, "%s: %s", what, hipGetErrorString(st));
    return ROBE_OK;
}

// SplitMix64 (Steele, Lea, Flood 2014): the documented coefficient stream.
uint64_t splitmix64(uint64_t &state)
{
    state += 0x9E3779B97F4A7C15ull;
    uint64_t z = state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int check_shape(uint64_t m, uint32_t d, uint32_t Z)
{
    if (m < 1 || m > (uint64_t)ROBE_PRIME) return fail(ROBE_EINVAL, "m = %llu outside [1, 2^31 - 1]", (unsigned long long)m);
    if (d < 1 || Z < 1) return fail(ROBE_EINVAL, "d = %u and Z = %u must be >= 1", d, Z);
    if (Z <= d ? d % Z != 0 : Z % d != 0)
        return fail(ROBE_EINVAL, "Z = %u must divide d = %u or be a multiple of it", Z, d);
    if ((uint64_t)Z > m) return fail(ROBE_EINVAL, "Z = %u exceeds m = %llu", Z, (unsigned long long)m);
    return ROBE_OK;
}

int check_hash(const robe_hash_t *h)
{
    if (h == nullptr) return fail(ROBE_EINVAL, "hash is NULL");
    if (int rc = check_shape(h->m, h->d, h->Z)) return rc;
    if (h->P != ROBE_PRIME) return fail(ROBE_EINVAL, "P = %u, only 2^31 - 1 is supported", h->P);
    const uint32_t mult[6] = {h->Ah, h->Bh, h->Ch, h->Ag, h->Bg, h->Cg};
    for (uint32_t v : mult)
        if (v < 1 || v > ROBE_PRIME - 1) return fail(ROBE_EINVAL, "hash multiplier %u outside [1, P-1]", v);
    if (h->Dh > ROBE_PRIME - 1 || h->Dg > ROBE_PRIME - 1) return fail(ROBE_EINVAL, "hash constant outside [0, P-1]");
    return ROBE_OK;
}

robe::Params to_params(const robe_hash_t *h)
{
    robe::Params p;
    p.m = (uint32_t)h->m;
    const uint64_t recip = (1ull << 32) / h->m;
    p.m_recip = recip > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)recip;
    p.d = h->d;
    p.Z = h->Z;
    p.C = h->Z <= h->d ? h->d / h->Z : 1u;
    p.r = h->Z <= h->d ? 0u : h->Z / h->d;
    p.Ah = h->Ah; p.Bh = h->Bh; p.Ch = h->Ch; p.Dh = h->Dh;
    p.Ag = h->Ag; p.Bg = h->Bg; p.Cg = h->Cg; p.Dg = h->Dg;
    return p;
}

bool is_pow2(uint32_t v) { return v && !(v & (v - 1)); }
uint32_t log2u(uint32_t v) { uint32_t s = 0; while ((1u << s) < v) ++s; return s; }
bool aligned(const void *ptr, size_t a) { return ((uintptr_t)ptr % a) == 0; }

// Which elements a lane owns.  V == 0 means "use the shape-generic kernel".
struct Layout {
    int V;
    bool consec;
    uint32_t G;
};

// Optional override for experiments: ROBE_TUNE_FWD / ROBE_TUNE_BWD = "V,consec" (e.g. "4,1").
bool tuned_layout(const char *var, const robe_hash_t *h, Layout *out)
{
    const char *s = getenv(var);
    if (!s) return false;
    int V = 0, consec = 0;
    if (sscanf(s, "%d,%d", &V, &consec) != 2) return false;
    if (V == 0 || h->Z > h->d) { *out = {0, false, 0}; return true; }
    if (V != 1 && V != 2 && V != 4) return false;
    if (h->d % V) return false;
    const uint32_t G = h->d / V;
    if (!is_pow2(G) || G > 64) return false;
    if (consec && h->Z % V) return false;
    *out = {V, consec != 0, G};
    return true;
}

Layout pick_layout(const robe_hash_t *h, bool bwd, const void *rows_ptr)
{
    Layout t;
    if (tuned_layout(bwd ? "ROBE_TUNE_BWD" : "ROBE_TUNE_FWD", h, &t)) {
        if (!t.consec || aligned(rows_ptr, 4 * (size_t)t.V)) return t;
    }
    if (h->Z > h->d) return {0, false, 0};   // embeddings sharing a chunk: shape-generic kernel
    const int vs[3] = {4, 2, 1};
    if (!bwd) {
        // forward: widest per-lane load that stays inside one chunk
        for (int V : vs) {
            if (h->Z % V || h->d % V) continue;
            const uint32_t G = h->d / V;
            if (is_pow2(G) && G <= 64 && aligned(rows_ptr, 4 * (size_t)V)) return {V, true, G};
        }
    }
    // backward (and forward when Z is too small): lanes of a group on consecutive addresses
    for (int V : {1, 2, 4}) {
        if (h->d % V) continue;
        const uint32_t G = h->d / V;
        if (is_pow2(G) && G <= 64) return {V, false, G};
    }
    return {0, false, 0};
}

int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return v ? atoi(v) : dflt;
}

template <bool BWD>
int launch_rows(const robe_hash_t *h, const float *src, const int64_t *indices, const int64_t *offsets,
                int64_t n_indices, int64_t rows, uint32_t F, float *dst, const void *rows_ptr, hipStream_t stream)
{
    const robe::Params p = to_params(h);
    const Layout lay = pick_layout(h, BWD, rows_ptr);
    const bool sign = h->use_sign != 0;
    const bool bags = offsets != nullptr;

    if (lay.V == 0) {
        uint32_t rpb = robe::kBlock / h->d;
        if (rpb < 1) rpb = 1;
        const int64_t blocks = (rows + rpb - 1) / rpb;
        if (blocks > 0x7FFFFFFFll) return fail(ROBE_EINVAL, "too many rows for one launch");
        if (sign)
            robe::generic_kernel<true, BWD><<<dim3((uint32_t)blocks), dim3(robe::kBlock), 0, stream>>>(p, F, rpb, src, indices, offsets, rows, n_indices, dst);
        else
            robe::generic_kernel<false, BWD><<<dim3((uint32_t)blocks), dim3(robe::kBlock), 0, stream>>>(p, F, rpb, src, indices, offsets, rows, n_indices, dst);
        return check_launch(BWD ? "backward (generic)" : "forward (generic)");
    }

    robe::Geom q;
    q.F = F;
    q.G = lay.G;
    q.g_shift = log2u(lay.G);
    const uint32_t step = 64u / lay.G;
    // one pass of the gather loop per wavefront tile measured best (more, shorter wavefronts)
    q.TL = step * robe::kUnroll >= 64u ? 64u : step * robe::kUnroll;
    if (const char *s = getenv("ROBE_TUNE_TL")) {
        const int tl = atoi(s);
        if (tl >= (int)step && tl <= 64 && tl % (int)step == 0) q.TL = (uint32_t)tl;
    }
    const int64_t rows_per_wave = bags ? (int64_t)step : (int64_t)q.TL;
    const int64_t waves = (rows + rows_per_wave - 1) / rows_per_wave;
    int64_t blocks = (waves + robe::kWavesPerBlock - 1) / robe::kWavesPerBlock;
    // Walk the rows table by table, one eighth of that order per XCD (see RowWalk), unless the launch
    // is too small to matter.  ROBE_TUNE_XCD=0 keeps the memory order.
    q.batch = rows / (int64_t)F;
    q.bpx = 0;
    // It pays where array reads dominate the traffic: bags (many blocks read per row written) and
    // blocks of at most one 64-byte sector (several sectors fetched per sector used).  For single-hot
    // lookups with larger blocks the row writes dominate and the memory order is slightly faster.
    // The direct backward scatter keeps the memory order too: table by table, the copies of a frequent
    // token arrive close together in time and their same-address atomics serialise (measured 30 % slower).
    const int xcd_mode = env_int("ROBE_TUNE_XCD", (!BWD && (bags || h->Z * 4 <= 64)) ? 1 : 0);   // 2: even for tiny launches
    if (F >= 2 && ((xcd_mode == 1 && blocks >= 64) || xcd_mode == 2)) {
        q.bpx = (uint32_t)((blocks + robe::kXcds - 1) / robe::kXcds);
        blocks = (int64_t)q.bpx * robe::kXcds;
    }
    if (blocks > 0x7FFFFFFFll) return fail(ROBE_EINVAL, "too many rows for one launch");
    const dim3 grid((uint32_t)blocks), block(robe::kBlock);

#define ROBE_LAUNCH(V_, C_, S_)                                                                                       \
    do {                                                                                                              \
        if (bags)                                                                                                     \
            robe::bag_kernel<V_, C_, S_, BWD><<<grid, block, 0, stream>>>(p, q, src, indices, offsets, rows, n_indices, dst); \
        else                                                                                                          \
            robe::single_hot_kernel<V_, C_, S_, BWD><<<grid, block, 0, stream>>>(p, q, src, indices, rows, dst);     \
    } while (0)
#define ROBE_LAUNCH_CS(V_)                                           \
    do {                                                             \
        if (lay.consec) {                                            \
            if (sign) ROBE_LAUNCH(V_, true, true);                   \
            else ROBE_LAUNCH(V_, true, false);                       \
        } else {                                                     \
            if (sign) ROBE_LAUNCH(V_, false, true);                  \
            else ROBE_LAUNCH(V_, false, false);                      \
        }                                                            \
    } while (0)

    switch (lay.V) {
        case 1: ROBE_LAUNCH_CS(1); break;
        case 2: ROBE_LAUNCH_CS(2); break;
        default: ROBE_LAUNCH_CS(4); break;
    }
#undef ROBE_LAUNCH_CS
#undef ROBE_LAUNCH
    return check_launch(BWD ? "backward" : "forward");
}


// ---------------------------------------------------------------------------
// Backward with duplicate tokens combined: plan (shared by robe_workspace_bytes
// and robe_backward) and launch.
// ---------------------------------------------------------------------------
struct BwdPlan {
    bool dedup;
    Layout lay;
    uint32_t key_bits;   // most significant key bits the sort looks at
    size_t off_keys_in, off_keys_out, off_vals_in, off_vals_out, off_tok_bag, off_temp, temp_bytes, bytes;
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Decide between the direct scatter and the combine-duplicates one, and lay out the workspace.
// ROBE_TUNE_BWD_MODE = direct | dedup overrides the size heuristic (not the hard limits).
BwdPlan plan_backward(const robe_hash_t *h, int64_t rows, int64_t n_indices, bool bags, const void *grad_out)
{
    BwdPlan pl;
    memset(&pl, 0, sizeof(pl));
    const char *mode = getenv("ROBE_TUNE_BWD_MODE");
    if (mode && strcmp(mode, "direct") == 0) return pl;
    const bool forced = mode && strcmp(mode, "dedup") == 0;
    // 32-bit positions and row numbers
    if (rows < 1 || n_indices < 1 || rows >= 0x7FFFFFFFll || n_indices >= 0x7FFFFFFFll) return pl;
    pl.lay = pick_layout(h, true, grad_out);
    if (pl.lay.V == 0 || pl.lay.consec) return pl;   // shapes only the generic kernel handles
    // sorting costs about 0.1 ms plus 45 ns per thousand tokens: not worth it for small scatters
    if (!forced && (uint64_t)n_indices * h->d < (1ull << 25)) return pl;
    // Sorting on the top 24 key bits is one radix pass cheaper; tokens that share those bits merely
    // interleave and are merged less often, which stays rare while there are far fewer tokens than 2^24.
    pl.key_bits = (uint32_t)env_int("ROBE_TUNE_KEY_BITS", n_indices <= (1ll << 24) ? 24 : 31);
    if (pl.key_bits < 8 || pl.key_bits > 31) pl.key_bits = 31;

    const size_t n = (size_t)n_indices;
    size_t temp = 0;
    uint32_t *nul = nullptr;
    if (rocprim::radix_sort_pairs(nullptr, temp, nul, nul, nul, nul, n, 31 - pl.key_bits, 31) != hipSuccess) {
        (void)hipGetLastError();
        return pl;                                    // no device to ask: the caller cannot run the scatter either
    }
    pl.dedup = true;
    size_t off = 0;
    pl.off_keys_in = off;  off = align_up(off + n * 4, 256);
    pl.off_keys_out = off; off = align_up(off + n * 4, 256);
    pl.off_vals_in = off;  off = align_up(off + n * 4, 256);
    pl.off_vals_out = off; off = align_up(off + n * 4, 256);
    pl.off_tok_bag = off;  if (bags) off = align_up(off + n * 4, 256);
    pl.off_temp = off;     off = align_up(off + temp, 256);
    pl.temp_bytes = temp;
    pl.bytes = off;
    return pl;
}

int launch_dedup_backward(const robe_hash_t *h, const BwdPlan &pl, const float *grad_out, const int64_t *indices,
                          const int64_t *offsets, int64_t n_indices, int64_t rows, uint32_t F,
                          float *grad_array, void *workspace, hipStream_t stream)
{
    const robe::Params p = to_params(h);
    char *ws = static_cast<char *>(workspace);
    uint32_t *keys_in = reinterpret_cast<uint32_t *>(ws + pl.off_keys_in);
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(ws + pl.off_keys_out);
    uint32_t *vals_in = reinterpret_cast<uint32_t *>(ws + pl.off_vals_in);
    uint32_t *vals_out = reinterpret_cast<uint32_t *>(ws + pl.off_vals_out);
    uint32_t *tok_bag = reinterpret_cast<uint32_t *>(ws + pl.off_tok_bag);
    const bool bags = offsets != nullptr;
    const bool sign = h->use_sign != 0;
    const uint32_t n = (uint32_t)n_indices, urows = (uint32_t)rows;

    // S1: keys.  With a well-formed CSR every position is written; the fill keeps stray positions harmless.
    if (bags) {
        robe::fill_pairs_kernel<<<dim3(2048), dim3(256), 0, stream>>>(keys_in, vals_in, n);
        if (int rc = check_launch("backward (clear keys)")) return rc;
    }
    uint32_t g_shift = 0;
    if (bags) {
        const uint64_t avg = ((uint64_t)n_indices + rows - 1) / rows;
        while (g_shift < 6 && (1ull << g_shift) < avg) ++g_shift;
    }
    const uint64_t key_threads = (uint64_t)rows << g_shift;
    uint64_t key_blocks = (key_threads + 255) / 256;
    if (key_blocks > 65536) key_blocks = 65536;
    if (bags)
        robe::token_keys_kernel<true><<<dim3((uint32_t)key_blocks), dim3(256), 0, stream>>>(p, F, g_shift, indices, offsets, urows, n, keys_in, vals_in, tok_bag);
    else
        robe::token_keys_kernel<false><<<dim3((uint32_t)key_blocks), dim3(256), 0, stream>>>(p, F, g_shift, indices, offsets, urows, n, keys_in, vals_in, tok_bag);
    if (int rc = check_launch("backward (keys)")) return rc;

    // S2: sort (key, position) pairs by the top key_bits bits of the 31-bit key
    size_t temp = pl.temp_bytes;
    hipError_t st = rocprim::radix_sort_pairs(ws + pl.off_temp, temp, keys_in, keys_out, vals_in, vals_out,
                                              (size_t)n, 31 - pl.key_bits, 31, stream);
    if (st != hipSuccess) return fail(ROBE_EHIP, "backward (sort): %s", hipGetErrorString(st));

    // S3: combine runs and scatter
    robe::Geom q;
    q.F = F;
    q.G = pl.lay.G;
    q.g_shift = log2u(pl.lay.G);
    q.TL = 0;
    q.bpx = 0;
    q.batch = 0;
    const uint64_t blocks = ((uint64_t)n + robe::kBlock - 1) / robe::kBlock;   // one lane per sorted position
    const dim3 grid((uint32_t)blocks), block(robe::kBlock);
#define ROBE_COMBINE(V_)                                                                                              \
    do {                                                                                                              \
        if (sign && bags) robe::combine_scatter_kernel<V_, true, true><<<grid, block, 0, stream>>>(p, q, grad_out, indices, keys_out, vals_out, tok_bag, urows, n, grad_array);   \
        else if (sign) robe::combine_scatter_kernel<V_, true, false><<<grid, block, 0, stream>>>(p, q, grad_out, indices, keys_out, vals_out, tok_bag, urows, n, grad_array);    \
        else if (bags) robe::combine_scatter_kernel<V_, false, true><<<grid, block, 0, stream>>>(p, q, grad_out, indices, keys_out, vals_out, tok_bag, urows, n, grad_array);    \
        else robe::combine_scatter_kernel<V_, false, false><<<grid, block, 0, stream>>>(p, q, grad_out, indices, keys_out, vals_out, tok_bag, urows, n, grad_array);             \
    } while (0)
    switch (pl.lay.V) {
        case 1: ROBE_COMBINE(1); break;
        case 2: ROBE_COMBINE(2); break;
        default: ROBE_COMBINE(4); break;
    }
#undef ROBE_COMBINE
    return check_launch("backward (combine and scatter)");
}

int check_rows(const robe_hash_t *h, const int64_t *indices, const int64_t *offsets, int64_t n_indices,
               int64_t batch, int32_t n_features, int64_t *rows_out)
{
    if (int rc = check_hash(h)) return rc;
    if (batch < 0) return fail(ROBE_EINVAL, "batch = %lld is negative", (long long)batch);
    if (n_features < 1) return fail(ROBE_EINVAL, "n_features = %d must be >= 1", n_features);
    if (n_indices < 0) return fail(ROBE_EINVAL, "n_indices = %lld is negative", (long long)n_indices);
    if (batch > (int64_t)0x7FFFFFFFFFFFll / n_features) return fail(ROBE_EINVAL, "batch * n_features overflows");
    const int64_t rows = batch * (int64_t)n_features;
    if (rows > (int64_t)0x7FFFFFFFFFFFFFll / (int64_t)h->d) return fail(ROBE_EINVAL, "batch * n_features * d overflows");
    if (offsets == nullptr && n_indices != rows)
        return fail(ROBE_EINVAL, "single-hot: n_indices = %lld but batch * n_features = %lld", (long long)n_indices, (long long)rows);
    if (rows > 0 && n_indices > 0 && indices == nullptr) return fail(ROBE_EINVAL, "indices is NULL");
    *rows_out = rows;
    return ROBE_OK;
}

}  // namespace

extern "C" {

const char *robe_last_error(void) { return g_err; }

int robe_init_hash(uint64_t seed, uint64_t m, uint32_t d, uint32_t Z, int use_sign, robe_hash_t *out)
{
    if (out == nullptr) return fail(ROBE_EINVAL, "out is NULL");
    if (int rc = check_shape(m, d, Z)) return rc;
    uint64_t st = seed;
    uint32_t c[8];
    for (int k = 0; k < 8; ++k) {
        const uint64_t r = splitmix64(st);
        c[k] = (k == 3 || k == 7) ? (uint32_t)(r % ROBE_PRIME) : (uint32_t)(1 + r % (ROBE_PRIME - 1));
    }
    out->m = m;
    out->d = d;
    out->Z = Z;
    out->use_sign = use_sign ? 1u : 0u;
    out->P = ROBE_PRIME;
    out->Ah = c[0]; out->Bh = c[1]; out->Ch = c[2]; out->Dh = c[3];
    out->Ag = c[4]; out->Bg = c[5]; out->Cg = c[6]; out->Dg = c[7];
    return ROBE_OK;
}

int robe_offsets(const robe_hash_t *hash, const int64_t *indices, int64_t n, int32_t n_features,
                 int64_t *out_offsets, int8_t *out_signs, void *stream)
{
    if (int rc = check_hash(hash)) return rc;
    if (n < 0) return fail(ROBE_EINVAL, "n = %lld is negative", (long long)n);
    if (n_features < 1) return fail(ROBE_EINVAL, "n_features = %d must be >= 1", n_features);
    if (n > (int64_t)0x7FFFFFFFFFFFFFll / (int64_t)hash->d) return fail(ROBE_EINVAL, "n * d overflows");
    if (n == 0 || (out_offsets == nullptr && out_signs == nullptr)) return ROBE_OK;
    if (indices == nullptr) return fail(ROBE_EINVAL, "indices is NULL");
    const robe::Params p = to_params(hash);
    hipStream_t s = (hipStream_t)stream;
    auto grid_for = [](int64_t total) {
        int64_t b = (total + robe::kBlock - 1) / robe::kBlock;
        return dim3((uint32_t)(b > 65536 ? 65536 : b));
    };
    if (out_offsets) {
        robe::offsets_kernel<<<grid_for(n * (int64_t)p.C), dim3(robe::kBlock), 0, s>>>(p, (uint32_t)n_features, indices, n, out_offsets);
        if (int rc = check_launch("offsets")) return rc;
    }
    if (out_signs) {
        robe::signs_kernel<<<grid_for(n * (int64_t)p.d), dim3(robe::kBlock), 0, s>>>(p, (uint32_t)n_features, hash->use_sign, indices, n, out_signs);
        if (int rc = check_launch("signs")) return rc;
    }
    return ROBE_OK;
}

int robe_forward(const robe_hash_t *hash, const float *array, const int64_t *indices, const int64_t *offsets,
                 int64_t n_indices, int64_t batch, int32_t n_features, float *out, void *stream)
{
    int64_t rows = 0;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    if (rows == 0) return ROBE_OK;
    if (array == nullptr) return fail(ROBE_EINVAL, "array is NULL");
    if (out == nullptr) return fail(ROBE_EINVAL, "out is NULL");
    if (!aligned(array, 4) || !aligned(out, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    return launch_rows<false>(hash, array, indices, offsets, n_indices, rows, (uint32_t)n_features, out, out, (hipStream_t)stream);
}

size_t robe_workspace_bytes(const robe_hash_t *hash, int64_t batch, int32_t n_features, int64_t n_indices)
{
    if (hash == nullptr || check_hash(hash) != ROBE_OK || batch < 0 || n_features < 1 || n_indices < 0) return 0;
    if (batch > (int64_t)0x7FFFFFFFFFFFll / n_features) return 0;
    // sized for bags and for an aligned grad_out; robe_backward never needs more than this
    const BwdPlan pl = plan_backward(hash, batch * (int64_t)n_features, n_indices, true, nullptr);
    return pl.dedup ? pl.bytes : 0;
}

int robe_backward(const robe_hash_t *hash, const float *grad_out, const int64_t *indices, const int64_t *offsets,
                  int64_t n_indices, int64_t batch, int32_t n_features, float *grad_array,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    int64_t rows = 0;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    const BwdPlan pl = plan_backward(hash, rows, n_indices, offsets != nullptr, grad_out);
    if (pl.dedup) {
        if (workspace == nullptr || workspace_bytes < pl.bytes)
            return fail(ROBE_EINVAL, "workspace of %zu bytes needed, %zu given", pl.bytes, workspace_bytes);
        if (!aligned(workspace, 256)) return fail(ROBE_EINVAL, "workspace must be 256-byte aligned");
    }
    if (rows == 0) return ROBE_OK;
    if (grad_out == nullptr) return fail(ROBE_EINVAL, "grad_out is NULL");
    if (grad_array == nullptr) return fail(ROBE_EINVAL, "grad_array is NULL");
    if (!aligned(grad_out, 4) || !aligned(grad_array, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    if (pl.dedup)
        return launch_dedup_backward(hash, pl, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features,
                                      grad_array, workspace, (hipStream_t)stream);
    return launch_rows<true>(hash, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features, grad_array, grad_out, (hipStream_t)stream);
}

static int launch_update(int rule, const robe_hash_t *hash, float *array, float *state, float *grad_array,
                         float lr, float eps, void *stream)
{
    const uint64_t m = hash->m;
    hipStream_t s = (hipStream_t)stream;
    const bool vec = aligned(array, 16) && aligned(grad_array, 16) && (rule != 0 || aligned(state, 16)) && m >= 4;
    uint64_t work = vec ? m / 4 : m;   // one thread per vector
    if (work < 1) work = 1;
    const uint64_t blocks = (work + robe::kBlock - 1) / robe::kBlock;   // <= 2^23 since m < 2^31
    const dim3 grid((uint32_t)blocks), block(robe::kBlock);
    if (rule == 0) {
        if (vec) robe::update_kernel<4, 0><<<grid, block, 0, s>>>(array, state, grad_array, m, lr, eps);
        else robe::update_kernel<1, 0><<<grid, block, 0, s>>>(array, state, grad_array, m, lr, eps);
    } else {
        if (vec) robe::update_kernel<4, 1><<<grid, block, 0, s>>>(array, nullptr, grad_array, m, lr, 0.0f);
        else robe::update_kernel<1, 1><<<grid, block, 0, s>>>(array, nullptr, grad_array, m, lr, 0.0f);
    }
    return check_launch(rule == 0 ? "adagrad" : "sgd");
}

int robe_adagrad_update(const robe_hash_t *hash, float *array, float *state, float *grad_array,
                        float lr, float eps, void *stream)
{
    if (int rc = check_hash(hash)) return rc;
    if (array == nullptr || state == nullptr || grad_array == nullptr) return fail(ROBE_EINVAL, "array, state or grad_array is NULL");
    if (!std::isfinite(lr) || !std::isfinite(eps) || !(eps > 0.0f)) return fail(ROBE_EINVAL, "need finite lr and eps > 0");
    if (!aligned(array, 4) || !aligned(state, 4) || !aligned(grad_array, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    return launch_update(0, hash, array, state, grad_array, lr, eps, stream);
}

int robe_sgd_update(const robe_hash_t *hash, float *array, float *grad_array, float lr, void *stream)
{
    if (int rc = check_hash(hash)) return rc;
    if (array == nullptr || grad_array == nullptr) return fail(ROBE_EINVAL, "array or grad_array is NULL");
    if (!std::isfinite(lr)) return fail(ROBE_EINVAL, "need a finite lr");
    if (!aligned(array, 4) || !aligned(grad_array, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    return launch_update(1, hash, array, nullptr, grad_array, lr, 0.0f, stream);
}

}  // extern "C"
