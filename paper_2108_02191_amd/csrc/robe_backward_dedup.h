// Backward scatter-add (Eq. 3 of the paper) with duplicate tokens combined first.
//
// Float atomics on device memory run at a fixed, low rate on this GPU (about one
// element per clock per memory channel, whatever the footprint; LDS float
// atomics are no faster), and every token costs d of them.  Recommendation
// batches repeat their frequent tokens many times, and all copies of a token
// (same table, same id) hit the same d slots with the same signs.  So:
//
//   S1 keys     every token gets the key th = (Bh*x + Ah*e + Dh) mod P - the token
//               part of its offset hash, equal for equal (e, x) - and a value: its
//               row of grad_out when the sign is off, its position when it is on.
//               (Blocks larger than embeddings: the key is the array offset itself, see sort_key.)
//   S2 sort     stable radix sort of (key, value) pairs (robe_radix_sort.h).
//   S3 combine  a group of G lanes walks G consecutive sorted tokens, adds the
//               gradient rows of runs of identical tokens in registers, and issues
//               the d atomics once per run.  A run longer than a group's walk (kWalk
//               stretches of G positions) is flushed once per walk, which also spreads
//               very frequent tokens over many groups.
//
// When are two tokens "identical"?  Every offset of a token is a function of th
// alone (h(e,x,c) = ((th + Ch*c) mod P) mod m), so with the sign off two tokens
// with the same th write the same slots whatever their table and id are: th is
// the identity, and S3 needs neither the ids nor the positions again (no random
// reads besides the gradient rows).  With the sign on, g depends on (e, x)
// through a second hash; identity is then checked on (th, table, id), which
// takes the position to fetch the id; distinct tokens that share th are merely
// not merged.
//
// The order of the float additions is not fixed, so results agree with an exact
// sum to rounding only.
#pragma once
#include "robe_kernels.h"

namespace robe {

constexpr int kRowsInFlight = 8;   // gradient rows a lane group loads before it adds them
constexpr int kWalk = 1;           // stretches of G sorted positions a lane group walks before it flushes its open run
                                   // (longer walks measured slower here: fewer, longer-lived groups)

// S1.  Bags: a group of G lanes takes kKeyBags consecutive bags at a time (their bounds, then their
// first G tokens each, are loaded together: a wavefront that did one bag and left spent its life in
// two dependent trips to memory), grid-stride over such sets; single-hot: one lane per lookup.
constexpr int kKeyBags = 4;        // eight measured the same, sixteen slower

// The sort key of a token.  Z <= d: the token part of the offset hash.  Z > d (Section 3.3): the token
// has one piece of d slots, at its place inside the chunk it shares with r - 1 neighbours; the array
// offset of that piece, below m, says all there is to say about where the token writes, so it is the
// key, and every kernel after the sort runs on the instance (Z' = d, one chunk, key = offset).
__device__ __forceinline__ uint32_t sort_key(const Params &p, int64_t x, uint32_t e)
{
    if (p.r == 0) return staged_h(p, x, e);
    uint32_t place;
    const int64_t chunk = block_key(p, x, place);
    return wrap(offset_of(p, staged_h(p, chunk, e), 0u) + place, p.m);
}

// Tables of mixed dimensions: the per-table map (first float inside a sample, dimension) that the
// combine kernels look rows up in, written from kernel arguments: the first kTableArgs tables by the
// key kernel (which runs before anything reads the map), further ones kTableArgs per launch of
// table_map_kernel.
constexpr int kTableArgs = 64;
struct TableArgs {
    uint32_t col[kTableArgs], dim[kTableArgs];
};

__global__ __launch_bounds__(64) void table_map_kernel(TableArgs a, uint32_t first, uint32_t count, uint2 *__restrict__ tables)
{
    if (threadIdx.x < count) tables[first + threadIdx.x] = make_uint2(a.col[threadIdx.x], a.dim[threadIdx.x]);
}

template <bool BAGS, bool ROWVAL>
__global__ __launch_bounds__(256) void token_keys_kernel(Params p, uint32_t F, uint32_t g_shift,
                                                         const int64_t *__restrict__ indices,
                                                         const int64_t *__restrict__ offsets,
                                                         uint32_t rows, uint32_t n_indices,
                                                         uint32_t *__restrict__ keys, uint32_t *__restrict__ vals,
                                                         uint32_t *__restrict__ tok_bag,
                                                         TableArgs tab, uint32_t n_tab, uint2 *__restrict__ tables)
{
    if (blockIdx.x == 0 && threadIdx.x < n_tab) tables[threadIdx.x] = make_uint2(tab.col[threadIdx.x], tab.dim[threadIdx.x]);
    const uint32_t G = 1u << g_shift;
    const uint32_t lane = threadIdx.x & (G - 1u);
    const uint64_t groups = ((uint64_t)gridDim.x * 256u) >> g_shift;
    const uint64_t group = ((uint64_t)blockIdx.x * 256u + threadIdx.x) >> g_shift;
    if constexpr (!BAGS) {
        for (uint64_t k = group; k < rows; k += groups) {      // G = 1: one lookup per lane
            keys[k] = sort_key(p, indices[k], (uint32_t)k % F);
            vals[k] = (uint32_t)k;
        }
    } else {
        for (uint64_t bag0 = group * kKeyBags; bag0 < rows; bag0 += groups * kKeyBags) {
            int64_t t0[kKeyBags], t1[kKeyBags];
#pragma unroll
            for (int j = 0; j < kKeyBags; ++j) {
                const uint64_t bag = bag0 + j < rows ? bag0 + j : rows - 1u;
                t0[j] = offsets[bag];
                t1[j] = offsets[bag + 1];
            }
            int64_t x[kKeyBags];
#pragma unroll
            for (int j = 0; j < kKeyBags; ++j) {
                t0[j] = t0[j] < 0 ? 0 : (t0[j] > (int64_t)n_indices ? (int64_t)n_indices : t0[j]);
                t1[j] = t1[j] < t0[j] ? t0[j] : (t1[j] > (int64_t)n_indices ? (int64_t)n_indices : t1[j]);
                if (bag0 + j >= rows) t1[j] = t0[j];           // past the last bag: nothing to do
                x[j] = t0[j] + lane < t1[j] ? indices[t0[j] + lane] : 0;
            }
#pragma unroll
            for (int j = 0; j < kKeyBags; ++j) {
                const uint32_t bag = (uint32_t)(bag0 + j);
                const uint32_t e = bag % F;
                int64_t t = t0[j] + lane;
                if (t < t1[j]) {
                    keys[t] = sort_key(p, x[j], e);
                    vals[t] = ROWVAL ? bag : (uint32_t)t;
                    if constexpr (!ROWVAL) tok_bag[t] = bag;
                }
                for (t += G; t < t1[j]; t += G) {              // bags longer than the lane group
                    keys[t] = sort_key(p, indices[t], e);
                    vals[t] = ROWVAL ? bag : (uint32_t)t;
                    if constexpr (!ROWVAL) tok_bag[t] = bag;
                }
            }
        }
    }
}

// S3.  Lane layout as in the direct scatter: G lanes per row, lane `grp` owns elements grp + k*G.
template <int V, bool SIGN, bool BAGS>
__global__ __launch_bounds__(kBlock) void combine_scatter_kernel(Params p, Geom q,
                                                                 const float *__restrict__ grad_out,
                                                                 const int64_t *__restrict__ indices,
                                                                 const uint32_t *__restrict__ keys,     // sorted
                                                                 const uint32_t *__restrict__ vals,     // sorted with the keys
                                                                 const uint32_t *__restrict__ tok_bag,
                                                                 uint32_t rows, uint32_t n_indices,
                                                                 float *__restrict__ grad_array)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t grp = lane & (q.G - 1u);
    const uint32_t base_lane = lane - grp;
    const uint64_t thread_id = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if ((thread_id - lane) * kWalk >= n_indices) return;     // the whole wavefront is past the end
    const uint64_t i_first = (thread_id - grp) * kWalk;       // first sorted position of this group's walk

    Lane<V, false, SIGN> L;
    L.init(p, q, grp);

    float acc[V];
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = 0.0f;
    uint32_t run_th = 0, run_tg = 0, run_d = q.d;
    bool open = false;
    // the last token of the stretch before (none before the first stretch)
    uint32_t c_th = 0, c_e = 0, c_xlo = 0, c_xhi = 0;
    bool c_ok = false;

    for (uint32_t st = 0; st < (uint32_t)kWalk; ++st) {
        const uint64_t i0 = i_first + (uint64_t)st * q.G;
        if (__all(i0 >= n_indices)) break;                   // every group of the wavefront is past the end

        // lane l of the group looks at sorted position i0 + l
        uint32_t my_th = 0, my_tg = 0, my_at = 0, my_d = q.d, my_e = 0;   // my_at: the token's gradient row (mixed dimensions: its first float)
        int64_t my_x = 0;
        bool my_ok = false;
        if (i0 + grp < n_indices) {
            const uint32_t t = vals[i0 + grp];                 // sign off: the row itself
            const uint32_t row = !SIGN ? t : (t < n_indices ? (BAGS ? tok_bag[t] : t) : rows);
            if (row < rows) {
                my_ok = true;
                my_at = row;
                my_th = keys[i0 + grp];
                if (SIGN || q.tables != nullptr) my_e = row % q.F;
                if (q.tables != nullptr) {                      // tables of mixed dimensions
                    const uint2 tab = q.tables[my_e];
                    my_at = (row / q.F) * (uint32_t)q.row_floats + tab.x;
                    my_d = tab.y;
                }
                if constexpr (SIGN) {
                    my_x = indices[t];
                    my_tg = staged_g(p, my_x, my_e);
                }
            }
        }
        // A coarse sort (few key bits) leaves the tokens of one key bucket interleaved.  A lane group's
        // run never outlives its walk anyway, so putting the wavefront's 64 positions in key order
        // here (bitonic network over the lanes; the key is made unique by the lane it came from, which
        // also says where to fetch the rest of the token) finds the same runs a full sort would.
        if (q.window_sort) {
            uint64_t sk = my_ok ? (((uint64_t)my_th << 6) | lane) : ((1ull << 40) | lane);
#pragma unroll
            for (uint32_t kk = 2; kk <= 64u; kk <<= 1) {
#pragma unroll
                for (uint32_t j = kk >> 1; j > 0; j >>= 1) {
                    const uint32_t lo = __shfl_xor((uint32_t)sk, (int)j), hi = __shfl_xor((uint32_t)(sk >> 32), (int)j);
                    const uint64_t other = ((uint64_t)hi << 32) | lo;
                    const bool take_min = ((lane & j) == 0) == ((lane & kk) == 0);
                    sk = take_min ? (other < sk ? other : sk) : (other > sk ? other : sk);
                }
            }
            const int from = (int)(sk & 63u);
            my_ok = (sk >> 40) == 0;
            my_th = my_ok ? (uint32_t)(sk >> 6) : 0u;
            my_at = __shfl(my_at, from);
            if (q.tables != nullptr) my_d = __shfl(my_d, from);
            if (SIGN || q.tables != nullptr) my_e = __shfl(my_e, from);
            if constexpr (SIGN) {
                my_tg = __shfl(my_tg, from);
                const uint32_t xlo = __shfl((uint32_t)my_x, from), xhi = __shfl((uint32_t)((uint64_t)my_x >> 32), from);
                my_x = (int64_t)(((uint64_t)xhi << 32) | xlo);
            }
        }
        // does this position start a new run?  (a different token than the one before, or the walk begins)
        const int prev = (int)(base_lane + (grp ? grp - 1u : 0u));
        uint32_t p_th = __shfl(my_th, prev);
        bool p_ok = __shfl((int)my_ok, prev) != 0;
        if (grp == 0) {
            p_th = c_th;
            p_ok = c_ok;
        }
        bool my_head = !p_ok || p_th != my_th;
        if (!SIGN && q.tables != nullptr) {     // equal keys of two tables (a hash collision) may differ in dimension: not one run
            uint32_t p_e = __shfl(my_e, prev);
            if (grp == 0) p_e = c_e;
            my_head = my_head || p_e != my_e;
        }
        if constexpr (SIGN) {
            uint32_t p_e = __shfl(my_e, prev);
            uint32_t p_xlo = __shfl((uint32_t)my_x, prev), p_xhi = __shfl((uint32_t)((uint64_t)my_x >> 32), prev);
            if (grp == 0) {
                p_e = c_e;
                p_xlo = c_xlo;
                p_xhi = c_xhi;
            }
            my_head = my_head || p_e != my_e || p_xlo != (uint32_t)my_x || p_xhi != (uint32_t)((uint64_t)my_x >> 32);
        }

        for (uint32_t k0 = 0; k0 < q.G; k0 += kRowsInFlight) {     // same trip count for every lane of the wavefront
            uint32_t at[kRowsInFlight], dd[kRowsInFlight], th[kRowsInFlight], tg[kRowsInFlight];
            bool ok[kRowsInFlight], head[kRowsInFlight];
#pragma unroll
            for (int u = 0; u < kRowsInFlight; ++u) {
                const int from = (int)(base_lane + ((k0 + u) & (q.G - 1u)));
                ok[u] = (k0 + u < q.G) && __shfl((int)my_ok, from) != 0;
                at[u] = __shfl(my_at, from);
                dd[u] = q.tables != nullptr ? __shfl(my_d, from) : q.d;
                th[u] = __shfl(my_th, from);
                tg[u] = SIGN ? __shfl(my_tg, from) : 0u;
                head[u] = __shfl((int)my_head, from) != 0;
                if (!ok[u]) at[u] = 0;                         // any valid row: its values are discarded
            }
            float v[kRowsInFlight][V];
#pragma unroll
            for (int u = 0; u < kRowsInFlight; ++u)
                load_row_of<V, BAGS>(grad_out + (q.tables != nullptr ? (uint64_t)at[u] : (uint64_t)at[u] * p.d), q.G, dd[u], grp, v[u]);
#pragma unroll
            for (int u = 0; u < kRowsInFlight; ++u) {
                if (!ok[u]) continue;
                if (head[u] && open) {
                    L.scatter(p, grad_array, run_th, run_tg, acc, 0, grp, q.G, run_d);
#pragma unroll
                    for (int k = 0; k < V; ++k) acc[k] = 0.0f;
                }
#pragma unroll
                for (int k = 0; k < V; ++k) acc[k] += v[u][k];
                run_th = th[u];
                run_tg = tg[u];
                run_d = dd[u];
                open = true;
            }
        }
        const int last = (int)(base_lane + q.G - 1u);
        c_th = __shfl(my_th, last);
        c_ok = __shfl((int)my_ok, last) != 0;
        if (!SIGN && q.tables != nullptr) c_e = __shfl(my_e, last);
        if constexpr (SIGN) {
            c_e = __shfl(my_e, last);
            c_xlo = __shfl((uint32_t)my_x, last);
            c_xhi = __shfl((uint32_t)((uint64_t)my_x >> 32), last);
        }
    }
    if (open) L.scatter(p, grad_array, run_th, run_tg, acc, 0, grp, q.G, run_d);
}

}  // namespace robe
