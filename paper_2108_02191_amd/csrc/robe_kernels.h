// HIP kernels of the ROBE-Z path for gfx950 (wave64).
//
// Work decomposition shared by the forward gather and the backward scatter:
//
//   * A wavefront owns a tile of rows (single-hot: TL consecutive lookups;
//     bags: 64/G consecutive bags).  In a first pass every lane hashes ONE
//     token of the tile - the part of h and g that depends on the token and on
//     the table id, (B*x + A*e + D) mod P - so the 64-bit modular work is done
//     once per token instead of once per lane that touches the token.
//   * In a second pass a group of G = d/V lanes walks the tile's tokens.  A
//     lane fetches the staged token term from the lane that hashed it
//     (wavefront shuffle), adds its own chunk term (C*c) mod P, which is a
//     per-lane constant, and finishes with one reciprocal-multiply `mod m`.
//   * A lane owns V elements of a row.  CONSEC layout: V consecutive elements
//     of one chunk (one hash, one unaligned 4V-byte load).  STRIDED layout:
//     elements grp + k*G, k < V (lanes of a group touch consecutive addresses,
//     which is what coalesces float atomics, and what Z < V needs).
//
// The integer maps are those of Eq. 5 (h, idx) and Eq. 2 (g) of the paper; the
// gather is Eq. 4, the scatter Eq. 3.
#pragma once
#include "robe_device.h"

namespace robe {

constexpr int kBlock = 256;           // 4 wavefronts
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kUnroll = 4;            // tokens in flight per lane group

// Launch geometry, filled on the host.
struct Geom {
    uint32_t F;        // number of tables (features)
    uint32_t G;        // lanes per row, power of two, <= 64; G * V >= d
    uint32_t d;        // elements per row; in the strided layout lane slots grp + k * G past it stay idle
    uint32_t g_shift;  // log2(G)
    uint32_t TL;       // rows per wavefront tile (single-hot kernels), multiple of 64/G, <= 64 (0: unused)
    uint32_t bpx;      // workgroups per XCD when rows are walked table by table (0: walk rows in memory order)
    int64_t batch;     // rows = batch * F
    // Where the F tables of this launch sit in the caller's buffers.  A plain call covers all of a
    // sample's tables (F_in = F, e0 = 0, row_floats = F * d, col0 = 0); a call for tables of mixed
    // dimensions launches once per run of consecutive tables of one dimension.
    uint32_t F_in;       // tables per sample in indices / offsets
    uint32_t e0;         // table id of this launch's first table = its place in a sample's input row
    int64_t row_floats;  // floats per sample in out / grad_out
    int64_t col0;        // first float of this launch's first table inside a sample
    // Sorted backward over tables of different dimensions (one launch for all of them): per table its
    // first float inside a sample (.x) and its dimension (.y); d above is then the largest dimension.
    // NULL: every table has dimension d and row k starts at float k * d.
    const uint2 *tables;
    // Sorted backward with float atomics: 1 when the sort looked at few key bits, so that tokens whose
    // keys agree in those bits sit interleaved; the combine kernel then sorts every wavefront's 64
    // positions by the whole key before it looks for runs.
    uint32_t window_sort;
};

// One row of a launch: where its id (or bag bounds) and its d floats live, and its table id.
struct RowRef {
    int64_t in_row;    // index into indices (single-hot) or offsets (bags)
    int64_t out_off;   // first float in out / grad_out
    uint32_t e;
};

// Which rows a wavefront works on.
//
// Row k = b*F + f of the [batch][F] layout belongs to table f.  Workgroups are handed to the 8 XCDs
// round-robin, and every XCD has its own L2.  Walking the rows in memory order shows every L2 the
// frequent tokens of all F tables; walking them table by table (position q = f*batch + b) and giving
// XCD x the x-th eighth of that order shows each L2 the frequent tokens of about F/8 tables only, so
// far more of them stay resident.  With bpx == 0 the order is the memory order.
constexpr uint32_t kXcds = 8;

struct RowWalk {
    int64_t q0;    // first position of this wavefront in walk order
    int64_t b0;    // its sample
    uint32_t f0;   // its table
};

__device__ __forceinline__ bool start_walk(const Geom &q, int64_t rows, int64_t rows_per_wave, RowWalk &w)
{
    uint32_t block = blockIdx.x;
    if (q.bpx) {
        const uint32_t x = block % kXcds, j = block / kXcds;
        block = x * q.bpx + j;
    }
    w.q0 = ((int64_t)block * kWavesPerBlock + (threadIdx.x >> 6)) * rows_per_wave;
    if (w.q0 >= rows) return false;
    if (q.bpx) {
        w.f0 = (uint32_t)(w.q0 / q.batch);
        w.b0 = w.q0 - (int64_t)w.f0 * q.batch;
    } else {
        w.b0 = w.q0 / (int64_t)q.F;
        w.f0 = (uint32_t)(w.q0 - w.b0 * (int64_t)q.F);
    }
    return true;
}

// The row `ahead` steps after the wavefront's first one (ahead < 64).
__device__ __forceinline__ RowRef walk_row(const Geom &q, const RowWalk &w, uint32_t ahead, uint32_t d)
{
    int64_t b;
    uint32_t f;
    if (q.bpx) {
        b = w.b0 + ahead;
        f = w.f0;
        while (b >= q.batch) {   // crosses into the next table(s); at most `ahead` rounds
            b -= q.batch;
            ++f;
        }
    } else {
        const uint32_t t = w.f0 + ahead;  // < F + 64
        const uint32_t over = t / q.F;
        f = t - over * q.F;
        b = w.b0 + over;
    }
    RowRef r;
    r.in_row = b * (int64_t)q.F_in + q.e0 + f;
    r.out_off = b * q.row_floats + q.col0 + (int64_t)f * d;
    r.e = q.e0 + f;
    return r;
}

template <int V>
struct Vec {
    typedef float A __attribute__((ext_vector_type(V)));  // V floats at natural vector alignment
    typedef A U __attribute__((aligned(4)));              // the same at 4-byte alignment
    typedef uint16_t HA __attribute__((ext_vector_type(V)));  // V bfloat16 bit patterns
    typedef HA HU __attribute__((aligned(2)));                 // ... at 2-byte alignment
};

// An array element as float32.  The array is float32, or bfloat16 bit patterns (uint16_t): the upper
// half of the float32 pattern, widened exactly by appending 16 zero bits.
__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// float32 -> bfloat16 bit pattern: round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ uint16_t narrow_bf16(float v)
{
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0u) return (uint16_t)((u >> 16) | 0x0040u);
    const uint32_t keep = u >> 16, drop = u & 0xFFFFu;
    return (uint16_t)(keep + ((drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) ? 1u : 0u));
}

// Per-lane constants: which elements this lane owns and their chunk terms.
template <int V, bool CONSEC, bool SIGN>
struct Lane {
    static constexpr int NH = CONSEC ? 1 : V;   // distinct (chunk, position) pairs
    uint32_t cc[NH];                             // (Ch * c) mod P
    uint32_t jj[NH];                             // position inside the chunk
    uint32_t cg[SIGN ? V : 1];                   // (Cg * i) mod P per owned element
    uint32_t live;                               // bit k: owned element k exists (strided layout with G * V > d)

    __device__ __forceinline__ bool has(int k) const { return CONSEC || ((live >> k) & 1u) != 0u; }

    __device__ __forceinline__ void init(const Params &p, const Geom &q, uint32_t grp)
    {
        live = 0;
#pragma unroll
        for (int k = 0; k < NH; ++k) {
            uint32_t i = CONSEC ? grp * V : grp + (uint32_t)k * q.G;
            if (!CONSEC) {
                if (i < q.d) live |= 1u << k;
                else i = 0;       // an idle slot: it reads element 0's array slot (in bounds) and writes nothing
            }
            const uint32_t c = i / p.Z;
            jj[k] = i - c * p.Z;
            cc[k] = mod_p((uint64_t)p.Ch * c);
        }
        if constexpr (SIGN) {
#pragma unroll
            for (int k = 0; k < V; ++k) {
                const uint32_t i = CONSEC ? grp * V + k : grp + (uint32_t)k * q.G;
                cg[k] = mod_p((uint64_t)p.Cg * i);
            }
        }
    }

    // Array position of pair k for a token whose staged term is th.  `place` is 0 unless blocks are
    // larger than embeddings (Z > d): then it is where the token's embedding starts inside its chunk,
    // place + jj < Z <= m, so one wrap still does.
    __device__ __forceinline__ uint32_t position(const Params &p, uint32_t th, int k, uint32_t place = 0) const
    {
        return wrap(offset_of(p, th, cc[k]) + jj[k] + place, p.m);
    }

    __device__ __forceinline__ uint32_t mask(uint32_t tg, int k) const
    {
        return SIGN ? sign_mask(add_p(tg, cg[k])) : 0u;
    }

    // v[k] = g * M[idx] for the V owned elements of one token.
    template <typename AT>
    __device__ __forceinline__ void gather(const Params &p, const AT *__restrict__ array,
                                           uint32_t th, uint32_t tg, float (&v)[V], uint32_t place = 0) const
    {
        if constexpr (CONSEC) {
            const uint32_t pos = position(p, th, 0, place);
            if (V == 1 || pos + V <= p.m) {
                if constexpr (sizeof(AT) == 4) {
                    const typename Vec<V>::A u = *reinterpret_cast<const typename Vec<V>::U *>(array + pos);
#pragma unroll
                    for (int k = 0; k < V; ++k) v[k] = u[k];
                } else {
                    const typename Vec<V>::HA u = *reinterpret_cast<const typename Vec<V>::HU *>(array + pos);
#pragma unroll
                    for (int k = 0; k < V; ++k) v[k] = widen((uint16_t)u[k]);
                }
            } else {  // the lane's own span crosses the end of the circular array
#pragma unroll
                for (int k = 0; k < V; ++k) v[k] = widen(array[wrap(pos + k, p.m)]);
            }
        } else {
#pragma unroll
            for (int k = 0; k < V; ++k) v[k] = widen(array[position(p, th, k, place)]);   // idle slots read some valid slot
        }
        if constexpr (SIGN) {
#pragma unroll
            for (int k = 0; k < V; ++k) v[k] = apply_sign(v[k], mask(tg, k));
        }
    }

    // grad_array[idx] += g * v[k] for the V owned elements of one token.
    // own: the lane's first element (grp in the strided layout); dlim: elements at or past it do not
    // exist in this row (tables of mixed dimensions; the lane constants are those of the largest).
    __device__ __forceinline__ void scatter(const Params &p, float *__restrict__ grad_array,
                                            uint32_t th, uint32_t tg, const float (&v)[V], uint32_t place = 0,
                                            uint32_t own = 0, uint32_t stride = 0, uint32_t dlim = 0xFFFFFFFFu) const
    {
        const uint32_t pos0 = CONSEC ? position(p, th, 0, place) : 0u;
#pragma unroll
        for (int k = 0; k < V; ++k) {
            // CONSEC: every element wraps on its own
            if (!has(k) || own + (uint32_t)k * stride >= dlim) continue;
            const uint32_t pos = CONSEC ? wrap(pos0 + (uint32_t)k, p.m) : position(p, th, k, place);
            const float val = SIGN ? apply_sign(v[k], mask(tg, k)) : v[k];
            __hip_atomic_fetch_add(grad_array + pos, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
};

// Load / store the V owned elements of one output row.
template <int V, bool CONSEC>
__device__ __forceinline__ void store_row(float *__restrict__ row, const Geom &q, uint32_t grp, const float (&v)[V])
{
    if constexpr (CONSEC) {
        typename Vec<V>::A a;
#pragma unroll
        for (int k = 0; k < V; ++k) a[k] = v[k];
        __builtin_nontemporal_store(a, reinterpret_cast<typename Vec<V>::A *>(row + grp * V));
    } else {
#pragma unroll
        for (int k = 0; k < V; ++k)
            if (grp + (uint32_t)k * q.G < q.d) __builtin_nontemporal_store(v[k], row + grp + (uint32_t)k * q.G);
    }
}

// KEEP: the row will be read again soon (the tokens of a bag all read the bag's row), so it is loaded
// with the default cache policy; otherwise it is streamed past the caches' resident lines.
// (strided layout) the same for a row of d elements, d <= q.d
template <int V, bool KEEP>
__device__ __forceinline__ void load_row_of(const float *__restrict__ row, uint32_t G, uint32_t d, uint32_t grp, float (&v)[V])
{
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const uint32_t i = grp + (uint32_t)k * G;
        const float *at = row + (i < d ? i : 0u);           // idle slots read element 0; nobody stores their value
        v[k] = KEEP ? *at : __builtin_nontemporal_load(at);
    }
}

template <int V, bool CONSEC, bool KEEP = false>
__device__ __forceinline__ void load_row(const float *__restrict__ row, const Geom &q, uint32_t grp, float (&v)[V])
{
    if constexpr (CONSEC) {
        const typename Vec<V>::A *at = reinterpret_cast<const typename Vec<V>::A *>(row + grp * V);
        const typename Vec<V>::A a = KEEP ? *at : __builtin_nontemporal_load(at);
#pragma unroll
        for (int k = 0; k < V; ++k) v[k] = a[k];
    } else {
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const uint32_t i = grp + (uint32_t)k * q.G;
            const float *at = row + (i < q.d ? i : 0u);       // idle slots read element 0; nobody stores their value
            v[k] = KEEP ? *at : __builtin_nontemporal_load(at);
        }
    }
}

// Blocks larger than embeddings (Z > d, Section 3.3): r = Z / d consecutive tokens of a table share
// a chunk.  The chunk id x div r takes the token's seat in h, and the embedding starts
// (x mod r) * d places into the chunk.  Otherwise the key is the token and the place is 0.
__device__ __forceinline__ int64_t block_key(const Params &p, int64_t x, uint32_t &place)
{
    place = 0;
    if (p.r == 0) return x;
    place = (uint32_t)((uint64_t)x % p.r) * p.d;
    return (int64_t)((uint64_t)x / p.r);
}

// Token-and-table part of h (and of g) for one token.
__device__ __forceinline__ uint32_t staged_h(const Params &p, int64_t x, uint32_t e)
{
    return add_p(token_term(p.Bh, x), mod_p((uint64_t)p.Ah * e + p.Dh));
}
__device__ __forceinline__ uint32_t staged_g(const Params &p, int64_t x, uint32_t e)
{
    return add_p(token_term(p.Bg, x), mod_p((uint64_t)p.Ag * e + p.Dg));
}

// ---------------------------------------------------------------------------
// Single-hot forward / backward: one wavefront per tile of TL lookups.
// ---------------------------------------------------------------------------
template <int V, bool CONSEC, bool SIGN, bool BWD, typename AT = float>
__global__ __launch_bounds__(kBlock) void single_hot_kernel(Params p, Geom q,
                                                            const AT *__restrict__ src,      // fwd: array; bwd: grad_out
                                                            const int64_t *__restrict__ indices,
                                                            int64_t rows,
                                                            float *__restrict__ dst)         // fwd: out; bwd: grad_array
{
    const uint32_t lane = threadIdx.x & 63u;
    RowWalk w;
    if (!start_walk(q, rows, (int64_t)q.TL, w)) return;  // uniform over the wavefront
    const uint32_t n = (uint32_t)((rows - w.q0) < (int64_t)q.TL ? (rows - w.q0) : (int64_t)q.TL);

    // pass 1: lane l hashes the l-th lookup of the tile
    uint32_t th = 0, tg = 0, pl = 0;
    if (lane < n) {
        const RowRef k = walk_row(q, w, lane, p.d);
        const int64_t x = indices[k.in_row];
        th = staged_h(p, block_key(p, x, pl), k.e);
        if constexpr (SIGN) tg = staged_g(p, x, k.e);
    }

    // pass 2: groups of G lanes walk the tile, 64/G rows per step
    const uint32_t grp = lane & (q.G - 1u);
    const uint32_t sub = lane >> q.g_shift;
    const uint32_t step = 64u >> q.g_shift;
    Lane<V, CONSEC, SIGN> L;
    L.init(p, q, grp);

    for (uint32_t r = 0; r < n; r += step * kUnroll) {  // trip count uniform over the wavefront
        uint32_t rl[kUnroll], thr[kUnroll], tgr[kUnroll], plr[kUnroll];
        bool live[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            rl[u] = r + (uint32_t)u * step + sub;
            live[u] = rl[u] < n;
            const uint32_t srcl = live[u] ? rl[u] : 0u;
            thr[u] = __shfl(th, (int)srcl);
            tgr[u] = SIGN ? __shfl(tg, (int)srcl) : 0u;
            plr[u] = p.r ? __shfl(pl, (int)srcl) : 0u;
        }
        if constexpr (!BWD) {
            float v[kUnroll][V];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) L.gather(p, src, thr[u], tgr[u], v[u], plr[u]);  // lookup 0 stands in for dead slots
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (live[u]) store_row<V, CONSEC>(dst + walk_row(q, w, rl[u], p.d).out_off, q, grp, v[u]);
        } else {
            float v[kUnroll][V];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint32_t safe = live[u] ? rl[u] : 0u;
                load_row<V, CONSEC>(src + walk_row(q, w, safe, p.d).out_off, q, grp, v[u]);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (live[u]) L.scatter(p, dst, thr[u], tgr[u], v[u], plr[u]);
        }
    }
}

// ---------------------------------------------------------------------------
// Single-hot backward for the direct scatter, with the duplicates of a tile combined first.
//
// Float atomics on one address serialise (tens of nanoseconds each), and a table with a handful of
// distinct tokens sends thousands of lookups of a batch to the same d addresses.  A wavefront takes
// a tile of 64 lookups - with the table-by-table row walk, 64 consecutive samples of one table -
// finds the distinct tokens among them (ballots over the staged hash terms), and every lane group
// sums the gradient rows of one distinct token at a time and scatters the sum once.  Strided lane
// layout (lanes of a group on consecutive addresses), as in the plain scatter.
// ---------------------------------------------------------------------------
template <int V, bool SIGN>
__global__ __launch_bounds__(kBlock) void single_hot_backward_tile_kernel(Params p, Geom q,
                                                                          const float *__restrict__ grad_out,
                                                                          const int64_t *__restrict__ indices,
                                                                          int64_t rows,
                                                                          float *__restrict__ grad_array)
{
    const uint32_t lane = threadIdx.x & 63u;
    RowWalk w;
    if (!start_walk(q, rows, 64, w)) return;             // uniform over the wavefront
    const uint32_t n = (uint32_t)((rows - w.q0) < 64 ? (rows - w.q0) : 64);

    // lane l hashes the l-th lookup of the tile
    uint32_t th = 0, tg = 0, pl = 0;
    const bool have = lane < n;
    if (have) {
        const RowRef k = walk_row(q, w, lane, p.d);
        const int64_t x = indices[k.in_row];
        th = staged_h(p, block_key(p, x, pl), k.e);
        if constexpr (SIGN) tg = staged_g(p, x, k.e);
    }
    // Distinct tokens: the lowest lane of every set of equal (th, place, tg) leads it and keeps the
    // set.  (Equal th and place mean equal offsets; with the sign on, equal tg as well means equal signs.)
    uint64_t remaining = __ballot(have), members = 0;
    while (remaining) {                                   // one round per distinct token; uniform
        const int lead = __ffsll((unsigned long long)remaining) - 1;
        const uint32_t lth = __shfl(th, lead), ltg = SIGN ? __shfl(tg, lead) : 0u, lpl = __shfl(pl, lead);
        const uint64_t same = __ballot(have && th == lth && pl == lpl && (!SIGN || tg == ltg));
        if ((int)lane == lead) members = same;
        remaining &= ~same;
    }
    const uint32_t mem_lo = (uint32_t)members, mem_hi = (uint32_t)(members >> 32);

    const uint32_t grp = lane & (q.G - 1u);
    const uint32_t sub = lane >> q.g_shift;
    const uint32_t step = 64u >> q.g_shift;               // lane groups per wavefront
    Lane<V, false, SIGN> L;
    L.init(p, q, grp);

    // Group `sub` takes the leaders among lanes sub, sub + step, ..., kUnroll of them at a time: the
    // first row of each is requested at once (distinct tokens keep kUnroll rows in flight, as in the
    // plain scatter), the further rows of a set follow, and every set is scattered once.
    for (uint32_t l0 = 0; l0 < 64u; l0 += step * kUnroll) {        // same trip count for every lane
        uint64_t todo[kUnroll];
        uint32_t lth[kUnroll], ltg[kUnroll], lpl[kUnroll];
        bool any_rows[kUnroll];
        float acc[kUnroll][V];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t lead = l0 + (uint32_t)u * step + sub;
            const bool in = lead < 64u;
            const int from = (int)(in ? lead : 0u);
            todo[u] = ((uint64_t)__shfl(mem_hi, from) << 32) | __shfl(mem_lo, from);
            if (!in) todo[u] = 0;
            lth[u] = __shfl(th, from);
            ltg[u] = SIGN ? __shfl(tg, from) : 0u;
            lpl[u] = p.r ? __shfl(pl, from) : 0u;
            any_rows[u] = todo[u] != 0;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {                         // first row of every set
            const uint32_t j = any_rows[u] ? (uint32_t)(__ffsll((unsigned long long)todo[u]) - 1) : 0u;
            todo[u] &= todo[u] - 1u;                               // (0 stays 0)
            load_row<V, false>(grad_out + walk_row(q, w, j, p.d).out_off, q, grp, acc[u]);   // lookup 0 stands in
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {                         // the other rows of the set
            while (__any(todo[u] != 0)) {
                float v[kUnroll][V];
                bool live[kUnroll];
#pragma unroll
                for (int t = 0; t < kUnroll; ++t) {
                    live[t] = todo[u] != 0;
                    const uint32_t j = live[t] ? (uint32_t)(__ffsll((unsigned long long)todo[u]) - 1) : 0u;
                    todo[u] &= todo[u] - 1u;
                    load_row<V, false>(grad_out + walk_row(q, w, j, p.d).out_off, q, grp, v[t]);
                }
#pragma unroll
                for (int t = 0; t < kUnroll; ++t) {
                    if (live[t]) {
#pragma unroll
                        for (int k = 0; k < V; ++k) acc[u][k] += v[t][k];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            if (any_rows[u]) L.scatter(p, grad_array, lth[u], ltg[u], acc[u], lpl[u]);
    }
}

// ---------------------------------------------------------------------------
// Bag-sum forward / bag backward: one group of G lanes per bag, 64/G bags per
// wavefront.  A group stages up to G of its bag's tokens at a time.
// ---------------------------------------------------------------------------
template <int V, bool CONSEC, bool SIGN, bool BWD, typename AT = float>
__global__ __launch_bounds__(kBlock) void bag_kernel(Params p, Geom q,
                                                     const AT *__restrict__ src,         // fwd: array; bwd: grad_out
                                                     const int64_t *__restrict__ indices,
                                                     const int64_t *__restrict__ offsets,
                                                     int64_t rows, int64_t n_indices,
                                                     float *__restrict__ dst)            // fwd: out; bwd: grad_array
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t step = 64u >> q.g_shift;                 // bags per wavefront
    RowWalk w;
    if (!start_walk(q, rows, (int64_t)step, w)) return;     // uniform over the wavefront
    const uint32_t grp = lane & (q.G - 1u);
    const uint32_t sub = lane >> q.g_shift;
    const uint32_t base_lane = lane - grp;                  // first lane of this group
    const bool have_bag = w.q0 + sub < rows;
    const RowRef bag = walk_row(q, w, have_bag ? sub : 0u, p.d);
    const uint32_t e = bag.e;

    int64_t t0 = 0, t1 = 0;
    if (have_bag) {
        t0 = offsets[bag.in_row];
        t1 = offsets[bag.in_row + 1];
        t0 = t0 < 0 ? 0 : (t0 > n_indices ? n_indices : t0);
        t1 = t1 < t0 ? t0 : (t1 > n_indices ? n_indices : t1);
    }

    Lane<V, CONSEC, SIGN> L;
    L.init(p, q, grp);

    float acc[V];
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = 0.0f;
    if constexpr (BWD) {
        if (have_bag) load_row<V, CONSEC>(src + bag.out_off, q, grp, acc);
    }

    for (int64_t tb = t0; __any(tb < t1); tb += q.G) {
        // stage: lane `grp` of the group hashes token tb + grp
        const int64_t left = t1 - tb;                       // <= 0 once this group is done
        const uint32_t cnt = left <= 0 ? 0u : (left < (int64_t)q.G ? (uint32_t)left : q.G);
        uint32_t th = 0, tg = 0, pl = 0;
        if (grp < cnt) {
            const int64_t x = indices[tb + grp];
            th = staged_h(p, block_key(p, x, pl), e);
            if constexpr (SIGN) tg = staged_g(p, x, e);
        }
        for (uint32_t u0 = 0; __any(u0 < cnt); u0 += kUnroll) {
            uint32_t thr[kUnroll], tgr[kUnroll], plr[kUnroll];
            bool live[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                live[u] = u0 + u < cnt;
                const uint32_t srcl = base_lane + (live[u] ? u0 + u : 0u);
                thr[u] = __shfl(th, (int)srcl);
                tgr[u] = SIGN ? __shfl(tg, (int)srcl) : 0u;
                plr[u] = p.r ? __shfl(pl, (int)srcl) : 0u;
            }
            if constexpr (!BWD) {
                float v[kUnroll][V];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) L.gather(p, src, thr[u], tgr[u], v[u], plr[u]);
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    if (live[u]) {
#pragma unroll
                        for (int k = 0; k < V; ++k) acc[k] += v[u][k];
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u)
                    if (live[u]) L.scatter(p, dst, thr[u], tgr[u], acc, plr[u]);
            }
        }
    }
    if constexpr (!BWD) {
        if (have_bag) store_row<V, CONSEC>(dst + bag.out_off, q, grp, acc);
    }
}

// ---------------------------------------------------------------------------
// Shape-generic fallback (any d, Z with Z | d): one thread per (row, element),
// every hash evaluated in full by the thread that needs it.
// ---------------------------------------------------------------------------
template <bool SIGN, bool BWD, typename AT = float>
__global__ __launch_bounds__(kBlock) void generic_kernel(Params p, Geom q, uint32_t rows_per_block,
                                                         const AT *__restrict__ src,
                                                         const int64_t *__restrict__ indices,
                                                         const int64_t *__restrict__ offsets,  // NULL: single-hot
                                                         int64_t rows, int64_t n_indices,
                                                         float *__restrict__ dst)
{
    const int64_t row_base = (int64_t)blockIdx.x * rows_per_block;
    const uint64_t items = (uint64_t)rows_per_block * p.d;
    for (uint64_t local = threadIdx.x; local < items; local += kBlock) {
        const uint32_t rl = (uint32_t)(local / p.d);
        const uint32_t i = (uint32_t)(local - (uint64_t)rl * p.d);
        const int64_t row = row_base + rl;
        if (row >= rows) break;
        const int64_t b = row / (int64_t)q.F;
        const uint32_t f = (uint32_t)(row - b * (int64_t)q.F);
        const uint32_t e = q.e0 + f;
        const int64_t in_row = b * (int64_t)q.F_in + e;
        const int64_t at = b * q.row_floats + q.col0 + (int64_t)f * p.d + i;   // this element in out / grad_out
        const uint32_t c = i / p.Z, j = i - c * p.Z;
        const uint32_t cc = mod_p((uint64_t)p.Ch * c);
        const uint32_t cg = SIGN ? mod_p((uint64_t)p.Cg * i) : 0u;
        int64_t t0 = in_row, t1 = in_row + 1;
        if (offsets != nullptr) {
            t0 = offsets[in_row];
            t1 = offsets[in_row + 1];
            t0 = t0 < 0 ? 0 : (t0 > n_indices ? n_indices : t0);
            t1 = t1 < t0 ? t0 : (t1 > n_indices ? n_indices : t1);
        }
        float acc = 0.0f;
        if constexpr (BWD) acc = src[at];
        for (int64_t t = t0; t < t1; ++t) {
            const int64_t x = indices[t];
            // Z > d (Section 3.3): r = Z/d embeddings share a chunk; the chunk id x / r takes the
            // token's seat in h and the embedding starts (x mod r) * d places into the chunk
            const int64_t key = p.r ? (int64_t)((uint64_t)x / p.r) : x;
            const uint32_t place = p.r ? (uint32_t)((uint64_t)x % p.r) * p.d : 0u;
            const uint32_t pos = wrap(offset_of(p, staged_h(p, key, e), cc) + j + place, p.m);
            const uint32_t msk = SIGN ? sign_mask(add_p(staged_g(p, x, e), cg)) : 0u;
            if constexpr (BWD) {
                __hip_atomic_fetch_add(dst + pos, apply_sign(acc, msk), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                const float v = apply_sign(widen(src[pos]), msk);
                acc = (offsets == nullptr) ? v : acc + v;   // single-hot keeps the sign of zero
            }
        }
        if constexpr (!BWD) dst[at] = acc;
    }
}

// ---------------------------------------------------------------------------
// float32 array -> bfloat16 array (post-hoc quantisation of a trained array).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void to_bf16_kernel(const float *__restrict__ src, uint16_t *__restrict__ dst,
                                                         uint64_t n, int vec_ok)
{
    const uint64_t tid = (uint64_t)blockIdx.x * kBlock + threadIdx.x, stride = (uint64_t)gridDim.x * kBlock;
    const uint64_t nvec = vec_ok ? n / 4u : 0u;
    for (uint64_t i = tid; i < nvec; i += stride) {
        const Vec<4>::A a = __builtin_nontemporal_load(reinterpret_cast<const Vec<4>::A *>(src) + i);
        Vec<4>::HA h;
#pragma unroll
        for (int k = 0; k < 4; ++k) h[k] = narrow_bf16(a[k]);
        __builtin_nontemporal_store(h, reinterpret_cast<Vec<4>::HA *>(dst) + i);
    }
    for (uint64_t i = 4u * nvec + tid; i < n; i += stride) dst[i] = narrow_bf16(src[i]);
}

// ---------------------------------------------------------------------------
// Integer maps alone (testing aid): one thread per (lookup, chunk) / (lookup, element).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void offsets_kernel(Params p, uint32_t F, const int64_t *__restrict__ indices,
                                                         int64_t n, int64_t *__restrict__ out)
{
    const int64_t total = n * (int64_t)p.C;
    for (int64_t it = (int64_t)blockIdx.x * kBlock + threadIdx.x; it < total; it += (int64_t)gridDim.x * kBlock) {
        const int64_t k = it / p.C;
        const uint32_t c = (uint32_t)(it - k * p.C);
        const uint32_t e = (uint32_t)(k % (int64_t)F);
        const int64_t x = indices[k];
        if (p.r) {  // Z > d: one entry per lookup, the place of element 0
            const uint32_t place = (uint32_t)((uint64_t)x % p.r) * p.d;
            out[it] = (int64_t)wrap(offset_of(p, staged_h(p, (int64_t)((uint64_t)x / p.r), e), 0u) + place, p.m);
        } else {
            out[it] = (int64_t)offset_of(p, staged_h(p, x, e), mod_p((uint64_t)p.Ch * c));
        }
    }
}

__global__ __launch_bounds__(kBlock) void signs_kernel(Params p, uint32_t F, uint32_t use_sign,
                                                       const int64_t *__restrict__ indices, int64_t n,
                                                       int8_t *__restrict__ out)
{
    const int64_t total = n * (int64_t)p.d;
    for (int64_t it = (int64_t)blockIdx.x * kBlock + threadIdx.x; it < total; it += (int64_t)gridDim.x * kBlock) {
        const int64_t k = it / p.d;
        const uint32_t i = (uint32_t)(it - k * p.d);
        const uint32_t e = (uint32_t)(k % (int64_t)F);
        const uint32_t res = add_p(staged_g(p, indices[k], e), mod_p((uint64_t)p.Cg * i));
        out[it] = (!use_sign || (res & 1u)) ? (int8_t)1 : (int8_t)-1;
    }
}

// ---------------------------------------------------------------------------
// Optimizer steps on touched slots (Adagrad, SGD).  Explicitly rounded float32 steps (no contraction).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void adagrad_one(float &w, float &s, float g, float lr, float eps)
{
    s = __fadd_rn(s, __fmul_rn(g, g));
    w = __fsub_rn(w, __fdiv_rn(__fmul_rn(lr, g), __fadd_rn(__fsqrt_rn(s), eps)));
}

// One thread per vector of V slots, no loop: measured fastest on MI355X (deeper per-thread
// unrolling lost to register pressure); streaming loads and stores keep the three arrays from
// displacing each other in the caches.  keep_array: the array is small enough to stay in the
// last-level cache until the next forward pass reads it, so it alone is read and written with
// the default cache policy.  The skip decision is taken per aligned group of kLineLanes
// lanes (64 bytes when V = 4, the granule that measured best among 16..256 bytes): a granule is
// either rewritten whole or not touched at all, because partially written granules cost the
// memory system far more than the bytes they save.
constexpr uint32_t kLineLanes = 4;

// RULE 0: Adagrad (array, state, grad).  RULE 1: SGD (array, grad; `state` and `eps` unused).
template <int V, int RULE>
__global__ __launch_bounds__(kBlock) void update_kernel(float *__restrict__ array, float *__restrict__ state,
                                                        float *__restrict__ grad, uint64_t m, float lr, float eps,
                                                        bool keep_array, bool clear_grad)
{
    typedef typename Vec<V>::A VT;
    const uint64_t nvec = m / V;
    const uint64_t it = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool in_range = it < nvec;
    VT g;
#pragma unroll
    for (int k = 0; k < V; ++k) g[k] = 0.0f;
    if (in_range) g = __builtin_nontemporal_load(reinterpret_cast<const VT *>(grad + it * V));
    bool any = false;
#pragma unroll
    for (int k = 0; k < V; ++k) any |= (g[k] != 0.0f);
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t line_any = (__ballot(any) >> (lane & ~(kLineLanes - 1u))) & ((1ull << kLineLanes) - 1ull);
    if (in_range && line_any != 0) {  // an untouched granule: nothing read beyond the gradient, nothing written
        VT w;
        if (keep_array) w = *reinterpret_cast<const VT *>(array + it * V);
        else w = __builtin_nontemporal_load(reinterpret_cast<const VT *>(array + it * V));
        VT s;
        if constexpr (RULE == 0) s = __builtin_nontemporal_load(reinterpret_cast<const VT *>(state + it * V));
#pragma unroll
        for (int k = 0; k < V; ++k) {
            if (g[k] != 0.0f) {      // slots with a zero gradient are rewritten with the bits they had
                if constexpr (RULE == 0) {
                    float wk = w[k], sk = s[k];
                    adagrad_one(wk, sk, g[k], lr, eps);
                    w[k] = wk;
                    s[k] = sk;
                } else {
                    w[k] = __fsub_rn(w[k], __fmul_rn(lr, g[k]));
                }
            }
            g[k] = 0.0f;
        }
        if (keep_array) *reinterpret_cast<VT *>(array + it * V) = w;
        else __builtin_nontemporal_store(w, reinterpret_cast<VT *>(array + it * V));
        if constexpr (RULE == 0) __builtin_nontemporal_store(s, reinterpret_cast<VT *>(state + it * V));
        if (clear_grad) __builtin_nontemporal_store(g, reinterpret_cast<VT *>(grad + it * V));
    }
    // tail (m not a multiple of V): first threads of block 0
    if (V > 1 && blockIdx.x == 0) {
        const uint64_t j = nvec * V + threadIdx.x;
        if (threadIdx.x < V && j < m) {
            const float gj = grad[j];
            if (gj != 0.0f) {
                if constexpr (RULE == 0) {
                    float wj = array[j], sj = state[j];
                    adagrad_one(wj, sj, gj, lr, eps);
                    array[j] = wj;
                    state[j] = sj;
                } else {
                    array[j] = __fsub_rn(array[j], __fmul_rn(lr, gj));
                }
                grad[j] = 0.0f;
            }
        }
    }
}

}  // namespace robe
