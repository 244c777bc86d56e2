// C ABI of the ROBE-Z library (see include/robe.h): argument validation,
// launch geometry and kernel selection.  All device work is in robe_kernels.h
// (forward, direct backward, update rules), robe_backward_dedup.h (sorted
// backward with float atomics), robe_backward_regions.h (sorted backward
// without them, fused Adagrad) and robe_radix_sort.h (the token sort).
//
// Nothing here is process-wide state: every choice a call makes follows from
// its arguments and its robe_options_t (NULL = all defaults).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "../../include/robe.h"
#include "robe_kernels.h"
#include "robe_backward_dedup.h"
#include "robe_backward_regions.h"
#include "robe_radix_sort.h"

// Workspace of robe_backward_noalloc: device memory that exists from the moment the library is
// loaded, one copy per GPU, so that the call itself allocates nothing.
#define ROBE_STATIC_SCRATCH_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[ROBE_STATIC_SCRATCH_BYTES];

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

// A call's options, checked and with defaults filled in (see robe_options_t in the header).
struct Opt {
    bool reproducible = false;
    int bwd_route = ROBE_ROUTE_AUTO, fused_route = ROBE_ROUTE_AUTO;
    int fwd_elems = 0, fwd_strided = 0, bwd_elems = 0, bwd_strided = 0;
    int tile_lookups = 0, row_order = ROBE_ROWS_AUTO, tile_combine = 0, region_shift = 0, key_bits = 0;
    int region_records = 0;
    int probe_kernel = ROBE_PROBE_NONE;
    hipEvent_t probe_begin = nullptr, probe_end = nullptr;
};

// Record the caller's probe events around kernel `which` (see robe_options_t).
int probe(const Opt &opt, int which, bool end, hipStream_t stream)
{
    if (opt.probe_kernel != which || opt.probe_begin == nullptr || opt.probe_end == nullptr) return ROBE_OK;
    hipError_t st = hipEventRecord(end ? opt.probe_end : opt.probe_begin, stream);
    if (st != hipSuccess) return fail(ROBE_EHIP, "probe event: %s", hipGetErrorString(st));
    return ROBE_OK;
}

bool elems_ok(int v, int strided)
{
    if (v == 0 || v == -1) return true;
    if (v == 1 || v == 2 || v == 4) return true;
    return strided && (v == 3 || v == 6 || v == 8);
}

int read_options(const robe_options_t *o, Opt *out)
{
    *out = Opt();
    if (o == nullptr) return ROBE_OK;
    if ((o->reproducible | 1) != 1) return fail(ROBE_EINVAL, "options: reproducible = %d is neither 0 nor 1", o->reproducible);
    if (o->backward_route < ROBE_ROUTE_AUTO || o->backward_route > ROBE_ROUTE_REGIONS)
        return fail(ROBE_EINVAL, "options: backward_route = %d is not a scatter strategy", o->backward_route);
    if (o->fused_route != ROBE_ROUTE_AUTO && o->fused_route != ROBE_ROUTE_REGIONS && o->fused_route != ROBE_ROUTE_TWO_STEP)
        return fail(ROBE_EINVAL, "options: fused_route = %d is none of AUTO, REGIONS, TWO_STEP", o->fused_route);
    if ((o->fwd_strided | 1) != 1 || (o->bwd_strided | 1) != 1) return fail(ROBE_EINVAL, "options: fwd_strided / bwd_strided must be 0 or 1");
    if (!elems_ok(o->fwd_elems, o->fwd_strided) || !elems_ok(o->bwd_elems, o->bwd_strided))
        return fail(ROBE_EINVAL, "options: elements per lane must be -1, 0, 1, 2, 4 (or 3, 6, 8 when strided)");
    if (o->tile_lookups < 0 || o->tile_lookups > 64) return fail(ROBE_EINVAL, "options: tile_lookups = %d outside 0..64", o->tile_lookups);
    if (o->row_order < ROBE_ROWS_AUTO || o->row_order > ROBE_ROWS_BY_TABLE_ALWAYS) return fail(ROBE_EINVAL, "options: row_order = %d", o->row_order);
    if (o->tile_combine < 0 || o->tile_combine > 2) return fail(ROBE_EINVAL, "options: tile_combine = %d outside 0..2", o->tile_combine);
    if (o->region_shift != 0 && (o->region_shift < 10 || o->region_shift > 15))
        return fail(ROBE_EINVAL, "options: region_shift = %d outside 10..15", o->region_shift);
    if (o->key_bits != 0 && (o->key_bits < 8 || o->key_bits > 31)) return fail(ROBE_EINVAL, "options: key_bits = %d outside 8..31", o->key_bits);
    if (o->region_records < 0 || o->region_records > 2) return fail(ROBE_EINVAL, "options: region_records = %d outside 0..2", o->region_records);
    if (o->probe_kernel < ROBE_PROBE_NONE || o->probe_kernel > ROBE_PROBE_SORT) return fail(ROBE_EINVAL, "options: probe_kernel = %d", o->probe_kernel);
    if (o->reserved[0] | o->reserved[1]) return fail(ROBE_EINVAL, "options: reserved fields must be zero");
    out->reproducible = o->reproducible != 0;
    out->bwd_route = o->backward_route;
    out->fused_route = o->fused_route;
    out->fwd_elems = o->fwd_elems; out->fwd_strided = o->fwd_strided;
    out->bwd_elems = o->bwd_elems; out->bwd_strided = o->bwd_strided;
    out->tile_lookups = o->tile_lookups;
    out->row_order = o->row_order;
    out->tile_combine = o->tile_combine;
    out->region_shift = o->region_shift;
    out->key_bits = o->key_bits;
    out->region_records = o->region_records;
    out->probe_kernel = o->probe_kernel;
    out->probe_begin = (hipEvent_t)o->probe_begin;
    out->probe_end = (hipEvent_t)o->probe_end;
    return ROBE_OK;
}

// Which elements a lane owns.  V == 0 means "use the shape-generic kernel".
struct Layout {
    int V;
    bool consec;
    uint32_t G;
};

// The layout the options ask for, if they ask for one (elems != 0): ROBE_EINVAL when the shape or
// the alignment of the rows cannot take it.
int requested_layout(int elems, int strided, const robe_hash_t *h, const void *rows_ptr, Layout *out)
{
    if (elems == -1) { *out = {0, false, 0}; return ROBE_OK; }
    const int V = elems;
    const bool consec = strided == 0;
    if (h->d % V) return fail(ROBE_EINVAL, "options: %d elements per lane do not divide d = %u", V, h->d);
    const uint32_t G = h->d / V;
    if (!is_pow2(G) || G > 64) return fail(ROBE_EINVAL, "options: d / elements per lane = %u is not a power of two <= 64", G);
    if (consec && h->Z <= h->d && h->Z % V) return fail(ROBE_EINVAL, "options: %d consecutive elements per lane do not divide Z = %u", V, h->Z);
    if (consec && !aligned(rows_ptr, 4 * (size_t)V)) return fail(ROBE_EINVAL, "options: rows are not aligned for %d-element vectors", V);
    *out = {V, consec, G};
    return ROBE_OK;
}

int pick_layout(const robe_hash_t *h, bool bwd, const void *rows_ptr, const Opt &opt, Layout *out)
{
    const int elems = bwd ? opt.bwd_elems : opt.fwd_elems;
    if (elems != 0) return requested_layout(elems, bwd ? opt.bwd_strided : opt.fwd_strided, h, rows_ptr, out);
    // (blocks larger than embeddings, Z > d: an embedding is one contiguous piece of its chunk, so
    // any V that divides d stays inside it)
    const int vs[3] = {4, 2, 1};
    if (!bwd) {
        // forward: widest per-lane load that stays inside one chunk
        for (int V : vs) {
            if ((h->Z <= h->d && h->Z % V) || h->d % V) continue;
            const uint32_t G = h->d / V;
            if (is_pow2(G) && G <= 64 && aligned(rows_ptr, 4 * (size_t)V)) { *out = {V, true, G}; return ROBE_OK; }
        }
    }
    // backward (and forward when Z is too small): lanes of a group on consecutive addresses.  Three, six
    // or eight elements per lane cover d = 3 * 2^k (24 .. 192), 384 and 512; four-byte accesses only.
    for (int V : {1, 2, 3, 4, 6, 8}) {
        if (h->d % V) continue;
        const uint32_t G = h->d / V;
        if (is_pow2(G) && G <= 64) { *out = {V, false, G}; return ROBE_OK; }
    }
    // Any other d up to 512: the smallest G * V >= d, the lane slots past d idle (d = 100: 2 x 64)
    Layout best = {0, false, 0};
    for (int V : {1, 2, 3, 4, 6, 8}) {
        for (uint32_t G = 1; G <= 64; G <<= 1) {
            if ((uint64_t)G * V < h->d) continue;
            if (best.V == 0 || G * V < best.G * best.V || (G * V == best.G * (uint32_t)best.V && G > best.G)) best = {V, false, G};
            break;
        }
    }
    *out = best;
    return ROBE_OK;
}

// Where a launch's tables sit inside a sample's input row and output row (see robe::Geom).
struct TableView {
    uint32_t F_in, e0;
    int64_t row_floats, col0;
};

template <bool BWD, typename AT = float>
int launch_rows(const robe_hash_t *h, const Opt &opt, const AT *src, const int64_t *indices, const int64_t *offsets,
                int64_t n_indices, int64_t rows, uint32_t F, float *dst, const void *rows_ptr, hipStream_t stream,
                const TableView *view = nullptr)
{
    const robe::Params p = to_params(h);
    Layout lay;
    if (int rc = pick_layout(h, BWD, rows_ptr, opt, &lay)) return rc;
    const bool sign = h->use_sign != 0;
    const bool bags = offsets != nullptr;

    robe::Geom q;
    memset(&q, 0, sizeof(q));
    q.F = F;
    q.d = h->d;
    q.batch = rows / (int64_t)F;
    q.F_in = view ? view->F_in : F;
    q.e0 = view ? view->e0 : 0u;
    q.row_floats = view ? view->row_floats : (int64_t)F * h->d;
    q.col0 = view ? view->col0 : 0;

    if (lay.V == 0) {
        uint32_t rpb = robe::kBlock / h->d;
        if (rpb < 1) rpb = 1;
        const int64_t blocks = (rows + rpb - 1) / rpb;
        if (blocks > 0x7FFFFFFFll) return fail(ROBE_EINVAL, "too many rows for one launch");
        if (sign)
            robe::generic_kernel<true, BWD, AT><<<dim3((uint32_t)blocks), dim3(robe::kBlock), 0, stream>>>(p, q, rpb, src, indices, offsets, rows, n_indices, dst);
        else
            robe::generic_kernel<false, BWD, AT><<<dim3((uint32_t)blocks), dim3(robe::kBlock), 0, stream>>>(p, q, rpb, src, indices, offsets, rows, n_indices, dst);
        return check_launch(BWD ? "backward (generic)" : "forward (generic)");
    }

    q.G = lay.G;
    q.g_shift = log2u(lay.G);
    const uint32_t step = 64u / lay.G;
    // one pass of the gather loop per wavefront tile measured best (more, shorter wavefronts)
    q.TL = step * robe::kUnroll >= 64u ? 64u : step * robe::kUnroll;
    if (opt.tile_lookups) {
        if (opt.tile_lookups < (int)step || opt.tile_lookups % (int)step != 0)
            return fail(ROBE_EINVAL, "options: tile_lookups = %d is not a multiple of %u", opt.tile_lookups, step);
        q.TL = (uint32_t)opt.tile_lookups;
    }
    // single-hot backward: tiles of 64 lookups whose duplicates are combined before the atomics,
    // from 32768 lookups on: below that the 64-lookup tiles leave too few wavefronts (measured at
    // d = 128: 26624 lookups 27 us plain, 32 us tiled; 53248 lookups 56 us plain, 38 us tiled).
    // options->tile_combine: 1 never, 2 always.
    const bool tile = BWD && !bags && !lay.consec && (opt.tile_combine == 2 || (opt.tile_combine == 0 && rows >= 32768));
    const int64_t rows_per_wave = tile ? 64 : (bags ? (int64_t)step : (int64_t)q.TL);
    const int64_t waves = (rows + rows_per_wave - 1) / rows_per_wave;
    int64_t blocks = (waves + robe::kWavesPerBlock - 1) / robe::kWavesPerBlock;
    // Walk the rows table by table, one eighth of that order per XCD (see RowWalk), unless the launch
    // is too small to matter.  options->row_order overrides.
    q.bpx = 0;
    // It pays where array reads dominate the traffic: bags (many blocks read per row written) and
    // blocks of at most one 64-byte sector (several sectors fetched per sector used).  For single-hot
    // lookups with larger blocks the row writes dominate and the memory order is slightly faster.
    // The direct backward scatter keeps the memory order too: table by table, the copies of a frequent
    // token arrive close together in time and their same-address atomics serialise (measured 30 % slower).
    // With tiles that combine their duplicates it is the other way round: a tile of one table holds
    // many copies of that table's frequent tokens.
    int order = opt.row_order;
    if (order == ROBE_ROWS_AUTO) order = ((!BWD && (bags || h->Z * 4 <= 64)) || tile) ? ROBE_ROWS_BY_TABLE : ROBE_ROWS_MEMORY;
    if (F >= 2 && ((order == ROBE_ROWS_BY_TABLE && blocks >= 64) || order == ROBE_ROWS_BY_TABLE_ALWAYS)) {
        q.bpx = (uint32_t)((blocks + robe::kXcds - 1) / robe::kXcds);
        blocks = (int64_t)q.bpx * robe::kXcds;
    }
    if (blocks > 0x7FFFFFFFll) return fail(ROBE_EINVAL, "too many rows for one launch");
    const dim3 grid((uint32_t)blocks), block(robe::kBlock);

#define ROBE_LAUNCH(V_, C_, S_)                                                                                       \
    do {                                                                                                              \
        if (bags)                                                                                                     \
            robe::bag_kernel<V_, C_, S_, BWD, AT><<<grid, block, 0, stream>>>(p, q, src, indices, offsets, rows, n_indices, dst); \
        else                                                                                                          \
            robe::single_hot_kernel<V_, C_, S_, BWD, AT><<<grid, block, 0, stream>>>(p, q, src, indices, rows, dst); \
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

#define ROBE_LAUNCH_TILE(V_)                                                                                          \
    do {                                                                                                              \
        if (sign) robe::single_hot_backward_tile_kernel<V_, true><<<grid, block, 0, stream>>>(p, q, src, indices, rows, dst);  \
        else robe::single_hot_backward_tile_kernel<V_, false><<<grid, block, 0, stream>>>(p, q, src, indices, rows, dst);      \
    } while (0)
    if constexpr (BWD && sizeof(AT) == 4) {
        if (tile) {
            switch (lay.V) {
                case 1: ROBE_LAUNCH_TILE(1); break;
                case 2: ROBE_LAUNCH_TILE(2); break;
                case 3: ROBE_LAUNCH_TILE(3); break;
                case 6: ROBE_LAUNCH_TILE(6); break;
                case 8: ROBE_LAUNCH_TILE(8); break;
                default: ROBE_LAUNCH_TILE(4); break;
            }
            return check_launch("backward (tiles)");
        }
    }
#undef ROBE_LAUNCH_TILE
    // three, six and eight elements per lane exist in the strided layout only
#define ROBE_LAUNCH_S(V_)                                            \
    do {                                                             \
        if (sign) ROBE_LAUNCH(V_, false, true);                      \
        else ROBE_LAUNCH(V_, false, false);                          \
    } while (0)
    switch (lay.V) {
        case 1: ROBE_LAUNCH_CS(1); break;
        case 2: ROBE_LAUNCH_CS(2); break;
        case 3: ROBE_LAUNCH_S(3); break;
        case 6: ROBE_LAUNCH_S(6); break;
        case 8: ROBE_LAUNCH_S(8); break;
        default: ROBE_LAUNCH_CS(4); break;
    }
#undef ROBE_LAUNCH_S
#undef ROBE_LAUNCH_CS
#undef ROBE_LAUNCH
    return check_launch(BWD ? "backward" : "forward");
}


// ---------------------------------------------------------------------------
// Backward with duplicate tokens combined: plan (shared by robe_workspace_bytes
// and robe_backward) and launch.
// ---------------------------------------------------------------------------
// Stable sort of n (key, value) pairs on key bits [lo, hi) with the kernels of robe_radix_sort.h.
// The sorted pairs end in (keys_b, vals_b) after an odd number of passes, else in (keys_a, vals_a):
// *in_b says which.  temp: radix_sort_temp_bytes(n) bytes, 256-byte aligned.
size_t radix_sort_temp_bytes(uint64_t n)
{
    const uint64_t tiles = (n + robe::kSortTile - 1) / robe::kSortTile;
    return (size_t)(robe::kDigits * tiles * 4 + 4 * robe::kDigits * 4);      // tile counts + totals of up to 4 passes
}

int launch_radix_sort(uint32_t *keys_a, uint32_t *vals_a, uint32_t *keys_b, uint32_t *vals_b, uint32_t n,
                      uint32_t lo, uint32_t hi, void *temp, hipStream_t stream, bool *in_b)
{
    *in_b = false;
    if (n == 0 || hi <= lo) return ROBE_OK;
    const uint32_t passes = (hi - lo + 7) / 8;
    if (passes > 4) return fail(ROBE_EINVAL, "internal: more than 32 key bits");
    robe::SortPass sp;
    sp.n = n;
    sp.tiles = (uint32_t)(((uint64_t)n + robe::kSortTile - 1) / robe::kSortTile);
    sp.tile_count = static_cast<uint32_t *>(temp);
    uint32_t *totals = sp.tile_count + (size_t)robe::kDigits * sp.tiles;
    uint32_t *ks = keys_a, *vs = vals_a, *kd = keys_b, *vd = vals_b;
    for (uint32_t pass = 0; pass < passes; ++pass) {
        sp.shift = lo + 8 * pass;
        const uint32_t bits = hi - sp.shift < 8 ? hi - sp.shift : 8;
        sp.mask = (1u << bits) - 1u;
        sp.totals = totals + pass * robe::kDigits;
        if (pass == 0) robe::sort_count_kernel<false><<<dim3(sp.tiles), dim3(robe::kSortBlock), 0, stream>>>(sp, ks);
        else robe::sort_count_kernel<true><<<dim3(sp.tiles), dim3(robe::kSortBlock), 0, stream>>>(sp, ks);
        if (int rc = check_launch("sort (count)")) return rc;
        robe::sort_offsets_kernel<<<dim3(robe::kDigits), dim3(robe::kSortBlock), 0, stream>>>(sp);
        if (int rc = check_launch("sort (offsets)")) return rc;
        robe::sort_scatter_kernel<robe::kScatterBlock><<<dim3(sp.tiles), dim3(robe::kScatterBlock), 0, stream>>>(sp, ks, vs, kd, vd);
        if (int rc = check_launch("sort (scatter)")) return rc;
        uint32_t *t = ks; ks = kd; kd = t;
        t = vs; vs = vd; vd = t;
    }
    *in_b = (passes & 1u) != 0;
    return ROBE_OK;
}

// An array of up to 128 MiB written with the default cache policy is still in the 256 MB last-level
// cache when the next forward pass gathers from it (measured on the 100 MB array: forward 0.29 ->
// 0.24 ms; no gain from 160 MB on, a loss from 400 MB on).  Larger arrays are streamed.
const uint64_t kKeepArrayMax = 1ull << 25;

struct BwdPlan {
    bool dedup;          // sort the tokens and combine identical ones
    bool regions;        // ... and then sort the blocks by destination region instead of using float atomics
    bool spill_rows;     // ... with room in LDS for a row of Z floats per lane group of the reduce kernel
    bool gather;         // ... and the reduce kernel finds its blocks in the sorted token list (no record kernels)
    bool window_sort;    // atomics route after a sort on few key bits: the combine kernel orders each wavefront's positions itself
    Layout lay;
    robe_hash_t eff;     // the instance the kernels after the key kernel run on: the caller's, or (Z > d) its one-chunk form
    uint32_t key_top;    // keys are below 2^key_top
    uint32_t key_bits;   // most significant key bits (below key_top) the sort looks at
    size_t off_keys_in, off_keys_out, off_vals_in, off_vals_out, off_tok_bag, off_temp, temp_bytes, bytes;
    // regions only
    robe::RegionPlan rp;
    size_t off_head, off_src_row, off_run_tg, off_run_c, off_P, off_counts, off_starts, off_wg_first, off_rec, off_rec_tg, off_dir;
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Whether the region-sorted scatter replaces the float atomics when nothing is requested.  Measured:
// 11 % faster on the 1 GB array with 8.5 M tokens, but 80 % slower on the 100 MB array with 1.7 M
// tokens (few regions, a fixed cost per region), and it needs several times the workspace.
bool regions_by_default(const robe_hash_t *h, int64_t n_indices)
{
    return h->m >= (1ull << 26) && n_indices >= (1ll << 21);
}

int fail_not_reproducible()
{
    return fail(ROBE_EINVAL, "reproducible option: this shape or size has no route without float atomics "
                             "(it needs d <= 512, d / Z and the lane group a power of two, at most 2^30 array slots, "
                             "32-bit record counts and a region size that leaves no short last region)");
}

// Region size for the region-sorted scatter with record kernels: 2^shift floats.  A region must hold
// two blocks and the array at most kMaxRegions regions.  0: no size fits.
uint32_t pick_region_shift(const robe_hash_t *h, int requested)
{
    auto fits = [&](uint32_t shift) {
        const uint64_t R = 1ull << shift, NR = (h->m + R - 1) >> shift;
        return NR <= robe::kMaxRegions && R >= 2ull * h->Z;
    };
    if (requested) return fits((uint32_t)requested) ? (uint32_t)requested : 0u;
    for (uint32_t shift = 13; shift <= 15; ++shift)
        if (fits(shift)) return shift;
    return 0;
}

uint32_t ceil_log2(uint64_t v) { uint32_t s = 0; while ((1ull << s) < v) ++s; return s; }

// Decide between the direct scatter, the combine-duplicates one and the region-sorted one, and lay
// out the workspace.  Host arithmetic only, so that the workspace queries and the calls agree.
// need_regions: the caller (the fused step) wants the region-sorted scatter whatever the size.
// mixed_floats: 0, or (tables of different dimensions, all multiples of Z; the hash is the widest
// table's) the floats of grad_out, batch * sum(dims).
BwdPlan plan_backward(const robe_hash_t *caller_hash, const Opt &opt, int64_t rows, int64_t n_indices, bool bags,
                      const void *grad_out, bool need_regions = false, uint64_t mixed_floats = 0)
{
    BwdPlan pl;
    memset(&pl, 0, sizeof(pl));
    // Blocks larger than embeddings (Z > d, Section 3.3): a token writes one piece of d slots, and the
    // sort key is that piece's array offset (sort_key in robe_backward_dedup.h).  From the sort on the
    // problem is an instance with blocks of d slots, one chunk per embedding and keys below m.
    pl.eff = *caller_hash;
    pl.key_top = 31;
    if (caller_hash->Z > caller_hash->d) {
        pl.eff.Z = caller_hash->d;
        pl.key_top = ceil_log2(caller_hash->m) ? ceil_log2(caller_hash->m) : 1u;
    }
    const robe_hash_t *h = &pl.eff;
    int route = opt.bwd_route;
    if (opt.reproducible) {
        need_regions = true;   // the only route without float atomics
        route = ROBE_ROUTE_AUTO;
    }
    if (route == ROBE_ROUTE_DIRECT && !need_regions) return pl;
    const bool forced = need_regions || route == ROBE_ROUTE_COMBINE || route == ROBE_ROUTE_REGIONS;
    // 32-bit positions and row numbers
    if (rows < 1 || n_indices < 1 || rows >= 0x7FFFFFFFll || n_indices >= 0x7FFFFFFFll) return pl;
    if (pick_layout(h, true, grad_out, opt, &pl.lay) != ROBE_OK) return pl;   // the launch reports the bad layout
    if (pl.lay.V == 0 || pl.lay.consec) return pl;   // shapes the sorted routes do not handle
    // sorting costs about 0.1 ms plus 45 ns per thousand tokens: not worth it for small scatters
    if (!forced && (uint64_t)n_indices * h->d < (1ull << 25)) return pl;
    // Sorting on the top 24 key bits is one radix pass cheaper; tokens that share those bits merely
    // interleave and are merged less often, which stays rare while there are far fewer tokens than 2^24.
    // (up to 2^18 tokens 16 bits do: a key bucket then holds four tokens at most on average)
    pl.key_bits = opt.key_bits ? (uint32_t)opt.key_bits : (n_indices <= (1ll << 18) ? 16u : (n_indices <= (1ll << 24) ? 24u : 31u));
    if (pl.key_bits > pl.key_top) pl.key_bits = pl.key_top;

    const size_t n = (size_t)n_indices;
    const size_t temp = radix_sort_temp_bytes(n);
    pl.dedup = true;
    size_t off = 0;
    pl.off_keys_in = off;  off = align_up(off + (n + 8) * 4, 256);
    pl.off_keys_out = off; off = align_up(off + (n + 8) * 4, 256);
    pl.off_vals_in = off;  off = align_up(off + n * 4, 256);
    pl.off_vals_out = off; off = align_up(off + n * 4, 256);
    pl.off_tok_bag = off;  if (bags && h->use_sign) off = align_up(off + n * 4, 256);   // sign off: the sorted value is the row
    pl.off_temp = off;     off = align_up(off + temp, 256);
    pl.temp_bytes = temp;
    pl.bytes = off;

    // Region-sorted scatter on top of the combined runs.
    const bool want_regions = need_regions || (route == ROBE_ROUTE_AUTO ? regions_by_default(h, n_indices) : route == ROBE_ROUTE_REGIONS);
    if (!want_regions) {
        // Atomics after the sort: up to 2^21 tokens, 16 key bits - two radix passes instead of three,
        // each three launches of 5 to 10 us.  The tokens of a key bucket (2^-16 of them) then sit
        // interleaved, and the combine kernel sorts every wavefront's 64 positions by the whole key.
        if (!opt.key_bits && pl.key_bits >= 16 && n_indices <= (1ll << 21)) {
            pl.key_bits = 16;
            pl.window_sort = true;
        }
        return pl;
    }
    const uint64_t C = h->d / h->Z;                       // Z <= d here
    uint32_t lg = 8;  // lanes per record in the reduce kernel: at most 64 groups per workgroup, a group inside one wavefront
    while (lg < robe::kMaxRecordLanes && lg < h->Z) lg <<= 1;
    static_assert(robe::kMaxRecordLanes <= 64 && (robe::kMaxRecordLanes & (robe::kMaxRecordLanes - 1)) == 0,
                  "a lane group of the reduce kernel is a power of two and never spans two wavefronts");
    const uint32_t grp_shift = 9 - log2u(lg);
    // Gather variant: the reduce kernel reads the sorted token list through a range table of
    // C * ((P - 1) / m + 3) entries, which must fit its LDS: large arrays, few chunks per embedding.
    // No record kernels, no record storage, any number of regions.  options->region_records asks for
    // either variant.
    uint32_t shift = 0;
    {
        const uint32_t gshift = opt.region_shift ? (uint32_t)opt.region_shift : 13u;
        const uint64_t R = 1ull << gshift, kmax = ((uint64_t)ROBE_PRIME - 1) / h->m, NE = C * (kmax + 3);
        const uint32_t cap = h->use_sign ? robe::gather_entries_max<true>() : robe::gather_entries_max<false>();
        const bool can = R >= 2ull * h->Z && h->m >= R + h->Z && NE <= cap && gshift >= grp_shift &&
                         (1u << (gshift - grp_shift)) >= h->Z && ((h->m + R - 1) >> gshift) <= 0x7FFFFFFFull;
        // By default on arrays of 2^26 slots or more, from 2^22 tokens on: with fewer tokens the record
        // kernels are quicker (batch 1024 of the benchmark's bags on the 1 GB array: 0.48 against
        // 0.51 ms; most regions then hold a handful of blocks, which a region's workgroup reads in one
        // trip instead of looking them up in two), unless their record counts or region table do not fit.
        // (The reproducible option keeps the lookup: its order of additions needs no bound on a region's records.)
        const bool records_fit = pick_region_shift(h, opt.region_shift) != 0 && 3ull * n * C < 0xFFFFFFFFull;
        const bool want = opt.region_records == 2 ||
                          (opt.region_records == 0 && h->m >= (1ull << 26) && (n >= (1ull << 22) || !records_fit || opt.reproducible));
        if (can && want) {
            pl.gather = true;
            shift = gshift;
        }
    }
    if (!pl.gather) {
        shift = pick_region_shift(h, opt.region_shift);
        if (shift == 0 || shift < grp_shift || (1u << (shift - grp_shift)) < h->Z) return pl;   // a slice of the region must hold one block
    }
    const uint64_t NR = (h->m + (1ull << shift) - 1) >> shift;
    // record kernels: a block leaves at most one more record, two when the array ends in a region
    // shorter than a block (a block can pass through it and go on at slot 0)
    const uint64_t last_len = h->m - ((NR - 1) << shift);
    const uint64_t rec_per_block = (NR > 1 && last_len < h->Z) ? 3 : 2;
    if (!pl.gather && rec_per_block * n * C >= 0xFFFFFFFFull) return pl;
    // The reproducible order of the record kernels splits an overfull region into at most
    // 2^kMaxClassShift classes of at most one round's records each.  Refuse what could come near that:
    // one and a half times the average region (hashed offsets spread evenly; a block in Z / R leaves a
    // second record), plus every run of the most frequent token (one per walk of a lane group) in one
    // region, against six tenths of the room.  (The gather variant stages its records in an order
    // that is fixed by the sorted list and needs no such split.)
    auto within_reproducible_bound = [&](uint64_t walk_positions) {
        if (!opt.reproducible || pl.gather) return true;
        const uint64_t batch = h->use_sign ? robe::rec_batch<true>() : robe::rec_batch<false>();
        const uint64_t room = ((batch << robe::kMaxClassShift) * 6) / 10;
        const uint64_t R = 1ull << shift, span = R < h->m ? R : h->m;
        const uint64_t avg = (n * C * (span + h->Z) / span + NR - 1) / NR;
        const uint64_t worst = avg + avg / 2 + 2ull * C * (n / walk_positions + 1);
        return worst <= room;
    };
    // rows of P: an eighth of the positions a lane group of the combine kernel walks, for every group
    // (a group that meets more runs of repeated tokens than that leaves the rest uncombined; on the
    // Zipf-distributed bags of the benchmark a walk of 512 positions holds 26 such runs on average
    // and 60 at most)
    // (long walks combine more copies of a frequent token per record, but a small problem needs its
    // wavefronts: halve the walk until the combine kernel has a couple of thousand workgroups)
    // (as long as the bound above holds: it counts one run of the most frequent token per walk)
    uint32_t stretch = robe::kStretch;
    while (stretch > 1 && n / ((uint64_t)robe::kBlock * stretch) < 2048) stretch >>= 1;
    while (stretch < (uint32_t)robe::kStretch && !within_reproducible_bound((uint64_t)stretch * pl.lay.G)) stretch <<= 1;
    if (!within_reproducible_bound((uint64_t)stretch * pl.lay.G)) return pl;
    const uint64_t walk = (uint64_t)stretch * pl.lay.G;
    const uint32_t p_quota = walk / 8 ? (uint32_t)(walk / 8) : 1u;
    const uint64_t combine_blocks = (n + (uint64_t)robe::kBlock * stretch - 1) / ((uint64_t)robe::kBlock * stretch);
    const uint64_t p_rows = combine_blocks * (robe::kBlock / pl.lay.G) * p_quota;
    // source blocks (Z floats each): those of grad_out, then those of P
    const uint64_t src_own = mixed_floats ? mixed_floats / h->Z : (uint64_t)rows * C;
    if (src_own + p_rows * C >= 0x7FFFFFFFull) return pl;                // 31-bit source block numbers

    pl.regions = true;
    robe::RegionPlan &r = pl.rp;
    r.r_shift = shift;
    r.NR = (uint32_t)NR;
    r.n = (uint32_t)n;
    r.rows = (uint32_t)rows;
    r.src_own = (uint32_t)src_own;
    r.src_blocks = (uint32_t)(src_own + p_rows * C);
    r.p_quota = p_quota;
    r.stretch = stretch;
    r.key_mask = pl.key_top >= 31 ? (uint32_t)ROBE_PRIME : (1u << pl.key_top) - 1u;
    r.bin_blocks = NR * 4 > 80 * 1024 ? 256u : 512u;      // one or two workgroups per CU by LDS
    if (n < (size_t)r.bin_blocks * 1024) r.bin_blocks = (uint32_t)((n + 1023) / 1024);
    r.pos_per_block = (uint32_t)((n + r.bin_blocks - 1) / r.bin_blocks);
    r.lg_shift = log2u(lg);
    // measured: it pays below about eight regions per workgroup slot (1024 slots), and in the
    // reproducible mode, whose rounds are longer
    r.fullest_first = (NR <= 8192 || opt.reproducible) ? 1u : 0u;
    r.keep_rows = bags ? 1u : 0u;
    // the slots the tokens can reach, against the array: below a quarter, most 64-byte granules stay untouched
    r.sparse_regions = (uint64_t)n * h->d < h->m / 4 ? 1u : 0u;
    pl.spill_rows = (uint64_t)(512u / lg) * h->Z <= robe::kSpillFloats;
    // (the reduce kernel of the gather variant reads keys, src_row and run_tg eight positions at a
    // time: every such array is padded to whole chunks)
    pl.off_head = off;    if (!pl.gather) off = align_up(off + n, 256);
    pl.off_src_row = off; off = align_up(off + (n + 8) * 4, 256);
    pl.off_run_tg = off;  if (h->use_sign) off = align_up(off + (n + 8) * 4, 256);
    pl.off_run_c = off;   if (mixed_floats) off = align_up(off + (n + 8) * 4, 256);
    pl.off_P = off;       off = align_up(off + p_rows * h->d * 4, 256);
    if (pl.gather) {
        // directory buckets: about two sorted positions each, never finer than what the sort looked at
        uint32_t bits = ceil_log2(n) > 1 ? ceil_log2(n) - 1 : 1;
        if (bits > 22) bits = 22;
        if (bits > pl.key_bits) bits = pl.key_bits;
        r.dir_shift = pl.key_top - bits;
        r.dir_buckets = 1u << bits;
        r.epc = (uint32_t)(((uint64_t)ROBE_PRIME - 1) / h->m + 3);
        r.NE = (uint32_t)(C * r.epc);
        r.epc_recip = (65536u + r.epc - 1) / r.epc;
        pl.off_dir = off;  off = align_up(off + ((size_t)r.dir_buckets + 1) * 4, 256);
    } else {
        pl.off_counts = off;  off = align_up(off + NR * 4, 256);
        pl.off_starts = off;  off = align_up(off + (NR + 1) * 4, 256);
        pl.off_wg_first = off; off = align_up(off + (size_t)r.bin_blocks * NR * 4, 256);
        pl.off_rec = off;     off = align_up(off + rec_per_block * n * C * 8, 256);
        pl.off_rec_tg = off;  if (h->use_sign) off = align_up(off + rec_per_block * n * C * 4, 256);
    }
    pl.bytes = off + 256;      // (slack: the padded reads above never leave the workspace)
    return pl;
}

template <typename K>
int allow_lds(K kernel, size_t bytes, const char *what)
{
    if (bytes <= 64 * 1024) return ROBE_OK;
    hipError_t st = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (st != hipSuccess) return fail(ROBE_EHIP, "%s: cannot reserve %zu bytes of LDS: %s", what, bytes, hipGetErrorString(st));
    return ROBE_OK;
}

// rule 0: grad_array += scatter.  Regions only: rule 1, Adagrad on (array = dst, state) with the scatter
// as gradient; rule 2, SGD on array = dst (the scatter rule of the reduce kernel with the scale -lr).
int launch_dedup_backward(const robe_hash_t *h, const Opt &opt, const BwdPlan &pl, const float *grad_out, const int64_t *indices,
                          const int64_t *offsets, int64_t n_indices, int64_t rows, uint32_t F,
                          float *grad_array, void *workspace, hipStream_t stream,
                          int rule = 0, float *state = nullptr, float lr = 0.0f, float eps = 0.0f,
                          uint2 *tables = nullptr, int64_t sample_floats = 0, const uint32_t *dims = nullptr)
{
    const robe::Params p_keys = to_params(h);     // the caller's instance: S1 hashes the ids with it
    h = &pl.eff;                                  // everything after S1 (see plan_backward)
    const robe::Params p = to_params(h);
    char *ws = static_cast<char *>(workspace);
    uint32_t *keys_in = reinterpret_cast<uint32_t *>(ws + pl.off_keys_in);
    uint32_t *keys_out = reinterpret_cast<uint32_t *>(ws + pl.off_keys_out);    // the sorted pairs, after S2
    uint32_t *vals_in = reinterpret_cast<uint32_t *>(ws + pl.off_vals_in);
    uint32_t *vals_out = reinterpret_cast<uint32_t *>(ws + pl.off_vals_out);
    uint32_t *tok_bag = reinterpret_cast<uint32_t *>(ws + pl.off_tok_bag);
    const bool bags = offsets != nullptr;
    const bool sign = h->use_sign != 0;
    const uint32_t n = (uint32_t)n_indices, urows = (uint32_t)rows;

    // S1: keys.  A well-formed CSR writes every position.  Positions a malformed one leaves out keep
    // whatever the workspace held; the combine kernel bounds-checks every position and row it reads,
    // so such entries can only add tokens to bags whose content is unspecified anyway.
    uint32_t g_shift = 0;
    if (bags) {
        const uint64_t avg = ((uint64_t)n_indices + rows - 1) / rows;
        while (g_shift < 6 && (1ull << g_shift) < avg) ++g_shift;
    }
    const uint64_t key_threads = bags ? (((uint64_t)rows + robe::kKeyBags - 1) / robe::kKeyBags) << g_shift : (uint64_t)rows;
    uint64_t key_blocks = (key_threads + 255) / 256;
    if (key_blocks > 65536) key_blocks = 65536;
    const dim3 kgrid((uint32_t)key_blocks), kblock(256);
    // tables of mixed dimensions: the key kernel also writes the per-table map (its first kTableArgs entries)
    robe::TableArgs tab;
    memset(&tab, 0, sizeof(tab));
    uint32_t n_tab = 0;
    if (tables != nullptr && dims != nullptr) {
        uint32_t col = 0;
        n_tab = F < (uint32_t)robe::kTableArgs ? F : (uint32_t)robe::kTableArgs;
        for (uint32_t k = 0; k < n_tab; ++k) {
            tab.col[k] = col;
            tab.dim[k] = dims[k];
            col += dims[k];
        }
    }
    // sign off: the sorted value is the token's row of grad_out and positions are never needed again
    if (bags && sign) robe::token_keys_kernel<true, false><<<kgrid, kblock, 0, stream>>>(p_keys, F, g_shift, indices, offsets, urows, n, keys_in, vals_in, tok_bag, tab, n_tab, tables);
    else if (bags) robe::token_keys_kernel<true, true><<<kgrid, kblock, 0, stream>>>(p_keys, F, g_shift, indices, offsets, urows, n, keys_in, vals_in, tok_bag, tab, n_tab, tables);
    else robe::token_keys_kernel<false, true><<<kgrid, kblock, 0, stream>>>(p_keys, F, g_shift, indices, offsets, urows, n, keys_in, vals_in, tok_bag, tab, n_tab, tables);
    if (int rc = check_launch("backward (keys)")) return rc;

    // S2: sort (key, value) pairs by the top key_bits bits of the key
    {
        bool in_b = false;
        if (int rc = probe(opt, ROBE_PROBE_SORT, false, stream)) return rc;
        // Which key_bits bits: the most significant ones - except for offset keys (blocks larger than
        // embeddings) on the atomics route, where neighbours in that order are pieces a few slots apart
        // whose atomics would meet in the same cache lines (measured 15 % slower): there the least
        // significant bits, which put far-apart pieces next to each other.  (The region route needs
        // the order of the whole key for its directory.)
        const uint32_t lo = (!pl.regions && pl.key_top < 31) ? 0u : pl.key_top - pl.key_bits;
        if (int rc = launch_radix_sort(keys_in, vals_in, keys_out, vals_out, n, lo, lo + pl.key_bits, ws + pl.off_temp,
                                       stream, &in_b))
            return rc;
        if (int rc = probe(opt, ROBE_PROBE_SORT, true, stream)) return rc;
        if (!in_b) {        // an even number of passes leaves the result in the first pair of buffers
            keys_out = keys_in;
            vals_out = vals_in;
        }
    }

    robe::Geom q;
    memset(&q, 0, sizeof(q));
    q.F = F;
    q.d = h->d;
    q.G = pl.lay.G;
    q.g_shift = log2u(pl.lay.G);
    q.tables = tables;              // tables of mixed dimensions
    q.window_sort = pl.window_sort ? 1u : 0u;
    q.row_floats = sample_floats;
    const uint64_t blocks = ((uint64_t)n + robe::kBlock - 1) / robe::kBlock;   // one lane per sorted position
    const dim3 grid((uint32_t)blocks), block(robe::kBlock);

    if (pl.regions) {
        robe::RegionPlan r = pl.rp;
        r.keys = keys_out;
        r.keep_array = (rule != 0 && h->m <= kKeepArrayMax) ? 1u : 0u;
        const float scale = rule == 2 ? -lr : (rule == 0 ? 1.0f : lr);    // what the reduce kernel gets as lr
        r.head = pl.gather ? nullptr : reinterpret_cast<uint8_t *>(ws + pl.off_head);
        r.src_row = reinterpret_cast<uint32_t *>(ws + pl.off_src_row);
        r.run_tg = reinterpret_cast<uint32_t *>(ws + pl.off_run_tg);
        r.run_c = tables != nullptr ? reinterpret_cast<uint32_t *>(ws + pl.off_run_c) : nullptr;
        r.P = reinterpret_cast<float *>(ws + pl.off_P);
        if (pl.gather) {
            r.dir = reinterpret_cast<uint32_t *>(ws + pl.off_dir);
            r.counts = r.starts = r.wg_first = r.rec_tg = nullptr;
            r.rec = nullptr;
        } else {
            r.dir = nullptr;
            r.counts = reinterpret_cast<uint32_t *>(ws + pl.off_counts);
            r.starts = reinterpret_cast<uint32_t *>(ws + pl.off_starts);
            r.wg_first = reinterpret_cast<uint32_t *>(ws + pl.off_wg_first);
            r.rec = reinterpret_cast<uint2 *>(ws + pl.off_rec);
            r.rec_tg = reinterpret_cast<uint32_t *>(ws + pl.off_rec_tg);
        }

        if (int rc = probe(opt, ROBE_PROBE_COMBINE, false, stream)) return rc;
        // R1: combine runs into P, leave one record per run (a lane group walks r.stretch * G positions)
        const dim3 rgrid1((uint32_t)(((uint64_t)n + (uint64_t)robe::kBlock * r.stretch - 1) / ((uint64_t)robe::kBlock * r.stretch)));
#define ROBE_COMBINE_ROWS_M(V_, M_)                                                                                   \
    do {                                                                                                              \
        if (sign && bags) robe::combine_rows_kernel<V_, true, true, M_><<<rgrid1, block, 0, stream>>>(p, q, r, grad_out, indices, vals_out, tok_bag);   \
        else if (sign) robe::combine_rows_kernel<V_, true, false, M_><<<rgrid1, block, 0, stream>>>(p, q, r, grad_out, indices, vals_out, tok_bag);    \
        else if (bags) robe::combine_rows_kernel<V_, false, true, M_><<<rgrid1, block, 0, stream>>>(p, q, r, grad_out, indices, vals_out, tok_bag);    \
        else robe::combine_rows_kernel<V_, false, false, M_><<<rgrid1, block, 0, stream>>>(p, q, r, grad_out, indices, vals_out, tok_bag);             \
    } while (0)
#define ROBE_COMBINE_ROWS(V_)                                                                                         \
    do {                                                                                                              \
        if (tables != nullptr) ROBE_COMBINE_ROWS_M(V_, true);                                                         \
        else ROBE_COMBINE_ROWS_M(V_, false);                                                                          \
    } while (0)
        switch (pl.lay.V) {
            case 1: ROBE_COMBINE_ROWS(1); break;
            case 2: ROBE_COMBINE_ROWS(2); break;
            case 3: ROBE_COMBINE_ROWS(3); break;
            case 6: ROBE_COMBINE_ROWS(6); break;
            case 8: ROBE_COMBINE_ROWS(8); break;
            default: ROBE_COMBINE_ROWS(4); break;
        }
#undef ROBE_COMBINE_ROWS_M
#undef ROBE_COMBINE_ROWS
        if (int rc = check_launch("backward (combine rows)")) return rc;
        if (int rc = probe(opt, ROBE_PROBE_COMBINE, true, stream)) return rc;

        // R2..R4: records sorted by region (the gather variant of R5 does without)
        if (!pl.gather) {
            const size_t lds_bin = (size_t)r.NR * 4;
            if (int rc = allow_lds(robe::region_bin_kernel<false, false>, lds_bin, "backward (count)")) return rc;
            robe::region_bin_kernel<false, false><<<dim3(r.bin_blocks), dim3(robe::kBinBlock), lds_bin, stream>>>(p, r);
            if (int rc = check_launch("backward (count)")) return rc;
            robe::region_scan_kernel<<<dim3(1), dim3(1024), 0, stream>>>(r);
            if (int rc = check_launch("backward (scan)")) return rc;
            if (sign) {
                if (int rc = allow_lds(robe::region_bin_kernel<true, true>, lds_bin, "backward (records)")) return rc;
                robe::region_bin_kernel<true, true><<<dim3(r.bin_blocks), dim3(robe::kBinBlock), lds_bin, stream>>>(p, r);
            } else {
                if (int rc = allow_lds(robe::region_bin_kernel<false, true>, lds_bin, "backward (records)")) return rc;
                robe::region_bin_kernel<false, true><<<dim3(r.bin_blocks), dim3(robe::kBinBlock), lds_bin, stream>>>(p, r);
            }
            if (int rc = check_launch("backward (records)")) return rc;
        }

        // R5: one workgroup per region
        const size_t lds_red = robe::reduce_lds_bytes(r.r_shift, sign, pl.gather, pl.spill_rows);
        const int vec_ok = aligned(grad_array, 16) && (rule != 1 || aligned(state, 16)) ? 1 : 0;
        const dim3 rgrid(r.NR), rblock(robe::kReduceBlock);
        const bool canon = opt.reproducible;
#define ROBE_REDUCE_G(S_, R_, C_, P_, G_)                                                                             \
    do {                                                                                                              \
        if (int rc = allow_lds(robe::region_reduce_kernel<S_, R_, C_, P_, G_>, lds_red, "backward (reduce)")) return rc;  \
        robe::region_reduce_kernel<S_, R_, C_, P_, G_><<<rgrid, rblock, lds_red, stream>>>(p, r, grad_out, grad_array, state, scale, eps, vec_ok); \
    } while (0)
#define ROBE_REDUCE_C(S_, R_, C_, P_)                                                                                 \
    do {                                                                                                              \
        if (pl.gather) ROBE_REDUCE_G(S_, R_, C_, P_, true);                                                           \
        else ROBE_REDUCE_G(S_, R_, C_, P_, false);                                                                    \
    } while (0)
#define ROBE_REDUCE(S_, R_)                                                                                           \
    do {                                                                                                              \
        if (canon && pl.spill_rows) ROBE_REDUCE_C(S_, R_, true, true);                                                \
        else if (canon) ROBE_REDUCE_C(S_, R_, true, false);                                                           \
        else if (pl.spill_rows) ROBE_REDUCE_C(S_, R_, false, true);                                                   \
        else ROBE_REDUCE_C(S_, R_, false, false);                                                                     \
    } while (0)
        if (int rc = probe(opt, ROBE_PROBE_REDUCE, false, stream)) return rc;
        if (sign) { if (rule == 1) ROBE_REDUCE(true, 1); else ROBE_REDUCE(true, 0); }
        else      { if (rule == 1) ROBE_REDUCE(false, 1); else ROBE_REDUCE(false, 0); }
#undef ROBE_REDUCE
#undef ROBE_REDUCE_C
#undef ROBE_REDUCE_G
        if (int rc = check_launch("backward (reduce)")) return rc;
        return probe(opt, ROBE_PROBE_REDUCE, true, stream);
    }
    if (rule != 0) return fail(ROBE_EINVAL, "internal: fused update needs the region-sorted scatter");

    if (int rc = probe(opt, ROBE_PROBE_COMBINE, false, stream)) return rc;
    // S3: combine runs and scatter with float atomics (a lane group walks kWalk * G positions)
    const dim3 sgrid((uint32_t)(((uint64_t)n + (uint64_t)robe::kBlock * robe::kWalk - 1) / ((uint64_t)robe::kBlock * robe::kWalk)));
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
        case 3: ROBE_COMBINE(3); break;
        case 6: ROBE_COMBINE(6); break;
        case 8: ROBE_COMBINE(8); break;
        default: ROBE_COMBINE(4); break;
    }
#undef ROBE_COMBINE
    if (int rc = check_launch("backward (combine and scatter)")) return rc;
    return probe(opt, ROBE_PROBE_COMBINE, true, stream);
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

// Tables of mixed dimensions: one launch per run of consecutive tables of one dimension, each a view
// into the [batch][n_features] inputs and the [batch][sum(dims)] rows.
template <bool BWD>
int launch_mixed(const robe_hash_t *hash, const Opt &opt, const uint32_t *dims, const float *src, const int64_t *indices,
                        const int64_t *offsets, int64_t n_indices, int64_t batch, int32_t n_features, float *dst,
                        const float *rows_ptr, void *stream)
{
    int64_t rows = 0;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    if (dims == nullptr) return fail(ROBE_EINVAL, "dims is NULL");
    int64_t D = 0;
    for (int32_t f = 0; f < n_features; ++f) {
        if (dims[f] < 1 || (dims[f] % hash->Z != 0 && hash->Z % dims[f] != 0))
            return fail(ROBE_EINVAL, "dims[%d] = %u is neither a multiple nor a divisor of Z = %u", f, dims[f], hash->Z);
        D += dims[f];
        if (D > 0x7FFFFFFFll) return fail(ROBE_EINVAL, "sum of dims exceeds 2^31 - 1");
    }
    if (batch > (int64_t)0x7FFFFFFFFFFFFFll / D) return fail(ROBE_EINVAL, "batch * sum(dims) overflows");
    if (rows == 0) return ROBE_OK;
    if (src == nullptr || dst == nullptr) return fail(ROBE_EINVAL, BWD ? "grad_out or grad_array is NULL" : "array or out is NULL");
    if (!aligned(src, 4) || !aligned(dst, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    int64_t col = 0;
    for (int32_t f0 = 0; f0 < n_features;) {
        int32_t f1 = f0 + 1;
        while (f1 < n_features && dims[f1] == dims[f0]) ++f1;
        robe_hash_t h = *hash;
        h.d = dims[f0];
        const TableView view = {(uint32_t)n_features, (uint32_t)f0, D, col};
        // the vector layouts need every row start of this view on a vector boundary
        const uintptr_t probe = (uintptr_t)rows_ptr | (uintptr_t)(D * 4) | (uintptr_t)(col * 4);
        const uint32_t Fv = (uint32_t)(f1 - f0);
        if (int rc = launch_rows<BWD>(&h, opt, src, indices, offsets, n_indices, batch * (int64_t)Fv, Fv, dst,
                                      reinterpret_cast<const void *>(probe), (hipStream_t)stream, &view))
            return rc;
        col += (int64_t)Fv * dims[f0];
        f0 = f1;
    }
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
                 int64_t n_indices, int64_t batch, int32_t n_features, float *out,
                 const robe_options_t *options, void *stream)
{
    int64_t rows = 0;
    Opt opt;
    if (int rc = read_options(options, &opt)) return rc;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    if (rows == 0) return ROBE_OK;
    if (array == nullptr) return fail(ROBE_EINVAL, "array is NULL");
    if (out == nullptr) return fail(ROBE_EINVAL, "out is NULL");
    if (!aligned(array, 4) || !aligned(out, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    return launch_rows<false>(hash, opt, array, indices, offsets, n_indices, rows, (uint32_t)n_features, out, out, (hipStream_t)stream);
}

int robe_forward_bf16(const robe_hash_t *hash, const uint16_t *array, const int64_t *indices, const int64_t *offsets,
                      int64_t n_indices, int64_t batch, int32_t n_features, float *out,
                      const robe_options_t *options, void *stream)
{
    int64_t rows = 0;
    Opt opt;
    if (int rc = read_options(options, &opt)) return rc;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    if (rows == 0) return ROBE_OK;
    if (array == nullptr) return fail(ROBE_EINVAL, "array is NULL");
    if (out == nullptr) return fail(ROBE_EINVAL, "out is NULL");
    if (!aligned(array, 2) || !aligned(out, 4)) return fail(ROBE_EINVAL, "array must be 2-byte and out 4-byte aligned");
    return launch_rows<false, uint16_t>(hash, opt, array, indices, offsets, n_indices, rows, (uint32_t)n_features, out, out,
                                        (hipStream_t)stream);
}

int robe_array_to_bf16(const float *src, uint16_t *dst, uint64_t n, void *stream)
{
    if (n == 0) return ROBE_OK;
    if (src == nullptr || dst == nullptr) return fail(ROBE_EINVAL, "src or dst is NULL");
    if (!aligned(src, 4) || !aligned(dst, 2)) return fail(ROBE_EINVAL, "src must be 4-byte and dst 2-byte aligned");
    const int vec_ok = aligned(src, 16) && aligned(dst, 8) ? 1 : 0;
    uint64_t blocks = (n / 4 + robe::kBlock - 1) / robe::kBlock;
    blocks = blocks < 1 ? 1 : (blocks > 65536 ? 65536 : blocks);
    robe::to_bf16_kernel<<<dim3((uint32_t)blocks), dim3(robe::kBlock), 0, (hipStream_t)stream>>>(src, dst, n, vec_ok);
    return check_launch("array to bfloat16");
}

// Shared argument checks of the two workspace queries.
static int check_query(const robe_hash_t *hash, int64_t batch, int32_t n_features, int64_t n_indices,
                       const robe_options_t *options, size_t *bytes, Opt *opt)
{
    if (bytes == nullptr) return fail(ROBE_EINVAL, "bytes is NULL");
    *bytes = 0;
    if (int rc = read_options(options, opt)) return rc;
    if (int rc = check_hash(hash)) return rc;
    if (batch < 0 || n_features < 1 || n_indices < 0) return fail(ROBE_EINVAL, "batch and n_indices must be >= 0 and n_features >= 1");
    if (batch > (int64_t)0x7FFFFFFFFFFFll / n_features) return fail(ROBE_EINVAL, "batch * n_features overflows");
    return ROBE_OK;
}

int robe_workspace_bytes(const robe_hash_t *hash, int64_t batch, int32_t n_features, int64_t n_indices,
                         const robe_options_t *options, size_t *bytes)
{
    Opt opt;
    if (int rc = check_query(hash, batch, n_features, n_indices, options, bytes, &opt)) return rc;
    // sized for bags and for an aligned grad_out; robe_backward never needs more than this
    const int64_t rows = batch * (int64_t)n_features;
    const BwdPlan pl = plan_backward(hash, opt, rows, n_indices, true, nullptr);
    if (opt.reproducible && !pl.regions && rows > 0 && n_indices > 0) return fail_not_reproducible();
    *bytes = pl.dedup ? pl.bytes : 0;
    return ROBE_OK;
}

int robe_backward(const robe_hash_t *hash, const float *grad_out, const int64_t *indices, const int64_t *offsets,
                  int64_t n_indices, int64_t batch, int32_t n_features, float *grad_array,
                  void *workspace, size_t workspace_bytes, const robe_options_t *options, void *stream)
{
    int64_t rows = 0;
    Opt opt;
    if (int rc = read_options(options, &opt)) return rc;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    const BwdPlan pl = plan_backward(hash, opt, rows, n_indices, offsets != nullptr, grad_out);
    if (pl.dedup) {
        if (workspace == nullptr || workspace_bytes < pl.bytes)
            return fail(ROBE_EINVAL, "workspace of %zu bytes needed, %zu given", pl.bytes, workspace_bytes);
        if (!aligned(workspace, 256)) return fail(ROBE_EINVAL, "workspace must be 256-byte aligned");
    }
    if (rows == 0 || n_indices == 0) return ROBE_OK;      // nothing to scatter
    if (grad_out == nullptr) return fail(ROBE_EINVAL, "grad_out is NULL");
    if (grad_array == nullptr) return fail(ROBE_EINVAL, "grad_array is NULL");
    if (!aligned(grad_out, 4) || !aligned(grad_array, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    if (opt.reproducible && !pl.regions) return fail_not_reproducible();
    if (pl.dedup)
        return launch_dedup_backward(hash, opt, pl, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features,
                                      grad_array, workspace, (hipStream_t)stream);
    return launch_rows<true>(hash, opt, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features, grad_array, grad_out, (hipStream_t)stream);
}

int robe_forward_mixed(const robe_hash_t *hash, const uint32_t *dims, const float *array, const int64_t *indices,
                       const int64_t *offsets, int64_t n_indices, int64_t batch, int32_t n_features, float *out,
                       const robe_options_t *options, void *stream)
{
    Opt opt;
    if (int rc = read_options(options, &opt)) return rc;
    return launch_mixed<false>(hash, opt, dims, array, indices, offsets, n_indices, batch, n_features, out, out, stream);
}

// Backward over tables of mixed dimensions: one token sort for all tables when the scatter is large
// enough (or a route is asked for), every dimension is a multiple of Z and the largest has a lane
// layout - then either the combine kernel with float atomics, or the region route (no float atomics;
// the reproducible option and the fused step need it); else one direct scatter per run of equal
// dimensions.  The plan is host arithmetic shared by the queries and the calls.
struct MixedPlan {
    bool sorted;            // one sort over all tables; pl says which route follows it
    BwdPlan pl;
    robe_hash_t widest;     // the hash with d = the largest dimension: lane constants and the sort's plan
    size_t off_tables, bytes;
    int64_t D;
};

// need_regions: the caller (the fused step) wants the region route whatever the size.
static int plan_mixed(const robe_hash_t *hash, const Opt &opt, const uint32_t *dims, int64_t batch, int32_t n_features,
                      int64_t n_indices, bool bags, const void *grad_out, bool need_regions, MixedPlan *mp)
{
    memset(mp, 0, sizeof(*mp));
    if (dims == nullptr) return fail(ROBE_EINVAL, "dims is NULL");
    uint32_t dmax = 0;
    bool narrow = false;
    int64_t D = 0;
    for (int32_t f = 0; f < n_features; ++f) {
        if (dims[f] < 1 || (dims[f] % hash->Z != 0 && hash->Z % dims[f] != 0))
            return fail(ROBE_EINVAL, "dims[%d] = %u is neither a multiple nor a divisor of Z = %u", f, dims[f], hash->Z);
        narrow = narrow || dims[f] < hash->Z;
        dmax = dims[f] > dmax ? dims[f] : dmax;
        D += dims[f];
        if (D > 0x7FFFFFFFll) return fail(ROBE_EINVAL, "sum of dims exceeds 2^31 - 1");
    }
    mp->D = D;
    mp->widest = *hash;
    mp->widest.d = dmax;
    const bool regions = need_regions || opt.reproducible || opt.bwd_route == ROBE_ROUTE_REGIONS;
    if ((opt.bwd_route == ROBE_ROUTE_DIRECT && !regions) || narrow || batch < 1 || n_indices < 1) return ROBE_OK;
    if ((uint64_t)batch * (uint64_t)D >= 0xFFFFFFFFull) return ROBE_OK;           // 32-bit row starts in the combine kernels
    const bool forced = regions || opt.bwd_route == ROBE_ROUTE_COMBINE;
    // the same size rule as robe_backward, on the average dimension
    if (!forced && (uint64_t)n_indices * (uint64_t)(D / n_features) < (1ull << 25)) return ROBE_OK;
    const int64_t rows = batch * (int64_t)n_features;
    Opt sorted = opt;
    sorted.bwd_route = regions ? ROBE_ROUTE_REGIONS : ROBE_ROUTE_COMBINE;
    mp->pl = plan_backward(&mp->widest, sorted, rows, n_indices, bags, grad_out, need_regions, (uint64_t)batch * (uint64_t)D);
    if (regions && !mp->pl.regions) {
        if (need_regions || opt.reproducible) return ROBE_OK;     // the caller falls back, or refuses
        sorted.bwd_route = ROBE_ROUTE_COMBINE;                    // a route was merely asked for: the next best
        mp->pl = plan_backward(&mp->widest, sorted, rows, n_indices, bags, grad_out, false, (uint64_t)batch * (uint64_t)D);
    }
    if (!mp->pl.dedup) return ROBE_OK;
    mp->sorted = true;
    mp->off_tables = mp->pl.bytes;
    mp->bytes = align_up(mp->pl.bytes + (size_t)n_features * sizeof(uint2), 256);
    return ROBE_OK;
}

// The sorted scatter of a MixedPlan into dst (rule 0: a gradient array; rule 1, region route only:
// Adagrad on dst = array and state).
static int launch_mixed_sorted(const MixedPlan &mp, const Opt &opt, const uint32_t *dims, const float *grad_out,
                               const int64_t *indices, const int64_t *offsets, int64_t n_indices, int64_t rows,
                               int32_t n_features, float *dst, void *workspace, hipStream_t s,
                               int rule = 0, float *state = nullptr, float lr = 0.0f, float eps = 0.0f)
{
    uint2 *tables = reinterpret_cast<uint2 *>(static_cast<char *>(workspace) + mp.off_tables);
    // the per-table map: its first kTableArgs entries travel with the key kernel, the rest go here
    uint32_t col = 0;
    for (int32_t f = 0; f < n_features && f < robe::kTableArgs; ++f) col += dims[f];
    for (int32_t f0 = robe::kTableArgs; f0 < n_features; f0 += robe::kTableArgs) {
        robe::TableArgs a;
        memset(&a, 0, sizeof(a));
        const int32_t cnt = n_features - f0 < robe::kTableArgs ? n_features - f0 : robe::kTableArgs;
        for (int32_t k = 0; k < cnt; ++k) {
            a.col[k] = col;
            a.dim[k] = dims[f0 + k];
            col += dims[f0 + k];
        }
        robe::table_map_kernel<<<dim3(1), dim3(64), 0, s>>>(a, (uint32_t)f0, (uint32_t)cnt, tables);
        if (int rc = check_launch("backward (table map)")) return rc;
    }
    return launch_dedup_backward(&mp.widest, opt, mp.pl, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features,
                                 dst, workspace, s, rule, state, lr, eps, tables, mp.D, dims);
}

int robe_mixed_workspace_bytes(const robe_hash_t *hash, const uint32_t *dims, int64_t batch, int32_t n_features,
                               int64_t n_indices, const robe_options_t *options, size_t *bytes)
{
    Opt opt;
    if (int rc = check_query(hash, batch, n_features, n_indices, options, bytes, &opt)) return rc;
    MixedPlan mp;
    if (int rc = plan_mixed(hash, opt, dims, batch, n_features, n_indices, true, nullptr, false, &mp)) return rc;
    if (opt.reproducible && !(mp.sorted && mp.pl.regions) && batch > 0 && n_indices > 0) return fail_not_reproducible();
    *bytes = mp.sorted ? mp.bytes : 0;
    return ROBE_OK;
}

int robe_backward_mixed(const robe_hash_t *hash, const uint32_t *dims, const float *grad_out, const int64_t *indices,
                        const int64_t *offsets, int64_t n_indices, int64_t batch, int32_t n_features,
                        float *grad_array, void *workspace, size_t workspace_bytes,
                        const robe_options_t *options, void *stream)
{
    Opt opt;
    if (int rc = read_options(options, &opt)) return rc;
    int64_t rows = 0;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    MixedPlan mp;
    if (int rc = plan_mixed(hash, opt, dims, batch, n_features, n_indices, offsets != nullptr, grad_out, false, &mp)) return rc;
    if (opt.reproducible && rows > 0 && n_indices > 0 && !(mp.sorted && mp.pl.regions)) return fail_not_reproducible();
    if (!mp.sorted)
        return launch_mixed<true>(hash, opt, dims, grad_out, indices, offsets, n_indices, batch, n_features, grad_array,
                                  grad_out, stream);
    if (workspace == nullptr || workspace_bytes < mp.bytes)
        return fail(ROBE_EINVAL, "workspace of %zu bytes needed, %zu given", mp.bytes, workspace_bytes);
    if (!aligned(workspace, 256)) return fail(ROBE_EINVAL, "workspace must be 256-byte aligned");
    if (grad_out == nullptr || grad_array == nullptr) return fail(ROBE_EINVAL, "grad_out or grad_array is NULL");
    if (!aligned(grad_out, 4) || !aligned(grad_array, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    return launch_mixed_sorted(mp, opt, dims, grad_out, indices, offsets, n_indices, rows, n_features, grad_array, workspace,
                               (hipStream_t)stream);
}

// The address of `scratch` on the current device.  In host code the array's name is only a handle
// for the symbol: the device address comes from hipGetSymbolAddress, once per device, and every
// later use goes through the pointer kept here.
static int static_scratch(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void *ptr_of_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t st = hipGetDevice(&dev);
    if (st != hipSuccess) return fail(ROBE_EHIP, "hipGetDevice: %s", hipGetErrorString(st));
    if (dev < 0 || dev >= kMaxDevices) return fail(ROBE_EINVAL, "device %d: at most %d devices are supported", dev, kMaxDevices);
    std::lock_guard<std::mutex> hold(lock);
    if (ptr_of_device[dev] == nullptr) {
        void *ptr = nullptr;
        st = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (st != hipSuccess || ptr == nullptr)
            return fail(ROBE_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(st));
        ptr_of_device[dev] = ptr;
    }
    *out = ptr_of_device[dev];
    return ROBE_OK;
}

size_t robe_noalloc_max_workspace_bytes(void) { return (size_t)ROBE_STATIC_SCRATCH_BYTES; }

int robe_backward_noalloc(const robe_hash_t *hash, const float *grad_out, const int64_t *indices, const int64_t *offsets,
                          int64_t n_indices, int64_t batch, int32_t n_features, float *grad_array,
                          const robe_options_t *options, void *stream)
{
    size_t need = 0;
    if (int rc = robe_workspace_bytes(hash, batch, n_features, n_indices, options, &need)) return rc;
    if (need > (size_t)ROBE_STATIC_SCRATCH_BYTES)
        return fail(ROBE_EINVAL, "robe_backward_noalloc: this problem needs a workspace of %zu bytes, the built-in one holds %zu; "
                                 "use robe_backward with a workspace of your own, or ROBE_ROUTE_DIRECT",
                    need, (size_t)ROBE_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (need > 0)
        if (int rc = static_scratch(&ws)) return rc;
    return robe_backward(hash, grad_out, indices, offsets, n_indices, batch, n_features, grad_array,
                         ws, need > 0 ? (size_t)ROBE_STATIC_SCRATCH_BYTES : 0, options, stream);
}

size_t robe_sort_workspace_bytes(uint64_t n)
{
    return align_up(radix_sort_temp_bytes(n), 256);
}

int robe_sort_pairs(uint32_t *keys_a, uint32_t *vals_a, uint32_t *keys_b, uint32_t *vals_b, uint64_t n,
                    uint32_t lo_bit, uint32_t hi_bit, void *workspace, size_t workspace_bytes, int *result_in_b,
                    void *stream)
{
    if (result_in_b == nullptr) return fail(ROBE_EINVAL, "result_in_b is NULL");
    *result_in_b = 0;
    if (lo_bit > hi_bit || hi_bit > 32) return fail(ROBE_EINVAL, "need lo_bit <= hi_bit <= 32");
    if (n >= 0xFFFFFFFFull) return fail(ROBE_EINVAL, "at most 2^32 - 2 pairs");
    if (n == 0 || lo_bit == hi_bit) return ROBE_OK;
    if (keys_a == nullptr || vals_a == nullptr || keys_b == nullptr || vals_b == nullptr)
        return fail(ROBE_EINVAL, "a key or value buffer is NULL");
    if (workspace == nullptr || workspace_bytes < radix_sort_temp_bytes(n))
        return fail(ROBE_EINVAL, "workspace of %zu bytes needed, %zu given", radix_sort_temp_bytes(n), workspace_bytes);
    if (!aligned(workspace, 256)) return fail(ROBE_EINVAL, "workspace must be 256-byte aligned");
    bool in_b = false;
    if (int rc = launch_radix_sort(keys_a, vals_a, keys_b, vals_b, (uint32_t)n, lo_bit, hi_bit, workspace,
                                   (hipStream_t)stream, &in_b))
        return rc;
    *result_in_b = in_b ? 1 : 0;
    return ROBE_OK;
}

// clear_grad: leave grad_array zeroed (the entry points' contract); false for a gradient array that
// lives in a workspace and is cleared before every use anyway.
static int launch_update(int rule, const robe_hash_t *hash, float *array, float *state, float *grad_array,
                         float lr, float eps, void *stream, bool clear_grad = true)
{
    const uint64_t m = hash->m;
    hipStream_t s = (hipStream_t)stream;
    const bool vec = aligned(array, 16) && aligned(grad_array, 16) && (rule != 0 || aligned(state, 16)) && m >= 4;
    uint64_t work = vec ? m / 4 : m;   // one thread per vector
    if (work < 1) work = 1;
    const uint64_t blocks = (work + robe::kBlock - 1) / robe::kBlock;   // <= 2^23 since m < 2^31
    const dim3 grid((uint32_t)blocks), block(robe::kBlock);
    const bool keep = m <= kKeepArrayMax;
    if (rule == 0) {
        if (vec) robe::update_kernel<4, 0><<<grid, block, 0, s>>>(array, state, grad_array, m, lr, eps, keep, clear_grad);
        else robe::update_kernel<1, 0><<<grid, block, 0, s>>>(array, state, grad_array, m, lr, eps, keep, clear_grad);
    } else {
        if (vec) robe::update_kernel<4, 1><<<grid, block, 0, s>>>(array, nullptr, grad_array, m, lr, 0.0f, keep, clear_grad);
        else robe::update_kernel<1, 1><<<grid, block, 0, s>>>(array, nullptr, grad_array, m, lr, 0.0f, keep, clear_grad);
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

// The fused step uses the region-sorted scatter when it applies and is worth its launches;
// otherwise a gradient array in the workspace and the two separate steps.  On arrays of 2^26 slots
// or more the two-step route would fill and sweep all m slots, which alone costs more than the
// region route's fixed part, so there the region route is taken whatever the batch size.
static bool fused_plan(const robe_hash_t *hash, const Opt &opt, int64_t rows, int64_t n_indices, bool bags,
                       const void *grad_out, BwdPlan *pl, size_t *scratch_bytes)
{
    *scratch_bytes = 0;
    const bool want = opt.fused_route == ROBE_ROUTE_AUTO ? hash->m >= (1ull << 26) : opt.fused_route == ROBE_ROUTE_REGIONS;
    if (opt.reproducible || want) {
        *pl = plan_backward(hash, opt, rows, n_indices, bags, grad_out, true);
        if (pl->regions) return true;
    }
    *pl = plan_backward(hash, opt, rows, n_indices, bags, grad_out);
    if (pl->regions) { pl->regions = false; }            // the two-step fallback adds onto a gradient array
    *scratch_bytes = align_up((size_t)hash->m * 4, 256);
    return false;
}

int robe_fused_workspace_bytes(const robe_hash_t *hash, int64_t batch, int32_t n_features, int64_t n_indices,
                               const robe_options_t *options, size_t *bytes)
{
    Opt opt;
    if (int rc = check_query(hash, batch, n_features, n_indices, options, bytes, &opt)) return rc;
    BwdPlan pl;
    size_t scratch = 0;
    const int64_t rows = batch * (int64_t)n_features;
    const bool fused = fused_plan(hash, opt, rows, n_indices, true, nullptr, &pl, &scratch);
    if (opt.reproducible && !fused && rows > 0 && n_indices > 0) return fail_not_reproducible();
    *bytes = scratch + ((pl.dedup || pl.regions) ? pl.bytes : 0);
    return ROBE_OK;
}

// Backward and update rule in one call (rule 1: Adagrad, rule 2: SGD): the fused region route when
// the plan has one, else two steps through a gradient array at the front of the workspace.
static int fused_step(int rule, const robe_hash_t *hash, const float *grad_out, const int64_t *indices, const int64_t *offsets,
                      int64_t n_indices, int64_t batch, int32_t n_features, float *array, float *state,
                      float lr, float eps, void *workspace, size_t workspace_bytes,
                      const robe_options_t *options, void *stream)
{
    int64_t rows = 0;
    Opt opt;
    if (int rc = read_options(options, &opt)) return rc;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    if (array == nullptr || (rule == 1 && state == nullptr)) return fail(ROBE_EINVAL, rule == 1 ? "array or state is NULL" : "array is NULL");
    if (!std::isfinite(lr)) return fail(ROBE_EINVAL, "need a finite lr");
    if (rule == 1 && (!std::isfinite(eps) || !(eps > 0.0f))) return fail(ROBE_EINVAL, "need finite lr and eps > 0");
    if (!aligned(array, 4) || (rule == 1 && !aligned(state, 4))) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    if (rows == 0 || n_indices == 0) return ROBE_OK;      // no gradient anywhere: nothing is touched
    if (grad_out == nullptr) return fail(ROBE_EINVAL, "grad_out is NULL");
    if (!aligned(grad_out, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    BwdPlan pl;
    size_t scratch = 0;
    const bool fused = fused_plan(hash, opt, rows, n_indices, offsets != nullptr, grad_out, &pl, &scratch);
    if (opt.reproducible && !fused) return fail_not_reproducible();
    const size_t need = scratch + ((pl.dedup || pl.regions) ? pl.bytes : 0);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need))
        return fail(ROBE_EINVAL, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    if (need > 0 && !aligned(workspace, 256)) return fail(ROBE_EINVAL, "workspace must be 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    if (fused)
        return launch_dedup_backward(hash, opt, pl, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features,
                                     array, workspace, s, rule, state, lr, eps);
    // two steps through a gradient array at the front of the workspace
    float *grad = static_cast<float *>(workspace);
    const uint64_t m = hash->m;
    uint64_t fill_blocks = (m + 255) / 256;
    if (fill_blocks > 65536) fill_blocks = 65536;
    robe::fill_u32_kernel<<<dim3((uint32_t)fill_blocks), dim3(256), 0, s>>>(reinterpret_cast<uint32_t *>(grad), (uint32_t)m, 0u);
    if (int rc = check_launch("fused step (clear gradient)")) return rc;
    char *rest = static_cast<char *>(workspace) + scratch;
    int rc;
    if (pl.dedup)
        rc = launch_dedup_backward(hash, opt, pl, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features, grad, rest, s);
    else
        rc = launch_rows<true>(hash, opt, grad_out, indices, offsets, n_indices, rows, (uint32_t)n_features, grad, grad_out, s);
    if (rc) return rc;
    return launch_update(rule == 1 ? 0 : 1, hash, array, state, grad, lr, eps, stream, false);
}

int robe_backward_adagrad(const robe_hash_t *hash, const float *grad_out, const int64_t *indices, const int64_t *offsets,
                          int64_t n_indices, int64_t batch, int32_t n_features, float *array, float *state,
                          float lr, float eps, void *workspace, size_t workspace_bytes,
                          const robe_options_t *options, void *stream)
{
    return fused_step(1, hash, grad_out, indices, offsets, n_indices, batch, n_features, array, state, lr, eps, workspace,
                      workspace_bytes, options, stream);
}

int robe_backward_sgd(const robe_hash_t *hash, const float *grad_out, const int64_t *indices, const int64_t *offsets,
                      int64_t n_indices, int64_t batch, int32_t n_features, float *array, float lr,
                      void *workspace, size_t workspace_bytes, const robe_options_t *options, void *stream)
{
    return fused_step(2, hash, grad_out, indices, offsets, n_indices, batch, n_features, array, nullptr, lr, 0.0f, workspace,
                      workspace_bytes, options, stream);
}

// The fused step over tables of mixed dimensions: the region route when the plan has one (and the
// array is large, or it is asked for), else two steps through a gradient array at the front of the
// workspace, like robe_backward_adagrad.
static int fused_mixed_plan(const robe_hash_t *hash, const Opt &opt, const uint32_t *dims, int64_t batch, int32_t n_features,
                            int64_t n_indices, bool bags, const void *grad_out, MixedPlan *mp, bool *fused, size_t *scratch_bytes)
{
    *scratch_bytes = 0;
    *fused = false;
    const bool want = opt.fused_route == ROBE_ROUTE_AUTO ? hash->m >= (1ull << 26) : opt.fused_route == ROBE_ROUTE_REGIONS;
    if (opt.reproducible || want) {
        if (int rc = plan_mixed(hash, opt, dims, batch, n_features, n_indices, bags, grad_out, true, mp)) return rc;
        if (mp->sorted && mp->pl.regions) {
            *fused = true;
            return ROBE_OK;
        }
    }
    Opt two = opt;
    if (two.bwd_route == ROBE_ROUTE_REGIONS) two.bwd_route = ROBE_ROUTE_COMBINE;   // the two steps add onto a gradient array
    if (int rc = plan_mixed(hash, two, dims, batch, n_features, n_indices, bags, grad_out, false, mp)) return rc;
    *scratch_bytes = align_up((size_t)hash->m * 4, 256);
    return ROBE_OK;
}

int robe_fused_mixed_workspace_bytes(const robe_hash_t *hash, const uint32_t *dims, int64_t batch, int32_t n_features,
                                     int64_t n_indices, const robe_options_t *options, size_t *bytes)
{
    Opt opt;
    if (int rc = check_query(hash, batch, n_features, n_indices, options, bytes, &opt)) return rc;
    MixedPlan mp;
    bool fused = false;
    size_t scratch = 0;
    if (int rc = fused_mixed_plan(hash, opt, dims, batch, n_features, n_indices, true, nullptr, &mp, &fused, &scratch)) return rc;
    if (opt.reproducible && !fused && batch > 0 && n_indices > 0) return fail_not_reproducible();
    *bytes = scratch + (mp.sorted ? mp.bytes : 0);
    return ROBE_OK;
}

int robe_backward_adagrad_mixed(const robe_hash_t *hash, const uint32_t *dims, const float *grad_out, const int64_t *indices,
                                const int64_t *offsets, int64_t n_indices, int64_t batch, int32_t n_features,
                                float *array, float *state, float lr, float eps, void *workspace, size_t workspace_bytes,
                                const robe_options_t *options, void *stream)
{
    int64_t rows = 0;
    Opt opt;
    if (int rc = read_options(options, &opt)) return rc;
    if (int rc = check_rows(hash, indices, offsets, n_indices, batch, n_features, &rows)) return rc;
    if (array == nullptr || state == nullptr) return fail(ROBE_EINVAL, "array or state is NULL");
    if (!std::isfinite(lr) || !std::isfinite(eps) || !(eps > 0.0f)) return fail(ROBE_EINVAL, "need finite lr and eps > 0");
    if (!aligned(array, 4) || !aligned(state, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    MixedPlan mp;
    bool fused = false;
    size_t scratch = 0;
    if (int rc = fused_mixed_plan(hash, opt, dims, batch, n_features, n_indices, offsets != nullptr, grad_out, &mp, &fused, &scratch))
        return rc;
    if (rows == 0 || n_indices == 0) return ROBE_OK;      // no gradient anywhere: nothing is touched
    if (grad_out == nullptr) return fail(ROBE_EINVAL, "grad_out is NULL");
    if (!aligned(grad_out, 4)) return fail(ROBE_EINVAL, "float buffers must be 4-byte aligned");
    if (opt.reproducible && !fused) return fail_not_reproducible();
    const size_t need = scratch + (mp.sorted ? mp.bytes : 0);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need))
        return fail(ROBE_EINVAL, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    if (need > 0 && !aligned(workspace, 256)) return fail(ROBE_EINVAL, "workspace must be 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    if (fused)
        return launch_mixed_sorted(mp, opt, dims, grad_out, indices, offsets, n_indices, rows, n_features, array, workspace, s,
                                   1, state, lr, eps);
    // two steps through a gradient array at the front of the workspace
    float *grad = static_cast<float *>(workspace);
    const uint64_t m = hash->m;
    uint64_t fill_blocks = (m + 255) / 256;
    if (fill_blocks > 65536) fill_blocks = 65536;
    robe::fill_u32_kernel<<<dim3((uint32_t)fill_blocks), dim3(256), 0, s>>>(reinterpret_cast<uint32_t *>(grad), (uint32_t)m, 0u);
    if (int rc = check_launch("fused step (clear gradient)")) return rc;
    char *rest = static_cast<char *>(workspace) + scratch;
    int rc;
    if (mp.sorted)
        rc = launch_mixed_sorted(mp, opt, dims, grad_out, indices, offsets, n_indices, rows, n_features, grad, rest, s);
    else
        rc = launch_mixed<true>(hash, opt, dims, grad_out, indices, offsets, n_indices, batch, n_features, grad, grad_out, stream);
    if (rc) return rc;
    return launch_update(0, hash, array, state, grad, lr, eps, stream, false);
}

}  // extern "C"
