// Backward scatter-add (Eq. 3 of the paper) with no float atomics at all, and the fused
// backward + Adagrad step built on it.
//
// After the tokens are sorted by key (robe_backward_dedup.h, S1 and S2):
//
//   R1 combine   a group of G lanes walks G consecutive sorted tokens.  A run of identical tokens
//                that is longer than one gets its gradient rows summed into a row of the scratch
//                matrix P; a run of one just points at its row of grad_out.  Every run leaves a
//                record at its first sorted position: a head flag, the key, the source row.
//   R2 count     every run's d/Z blocks are hashed to their array offsets; the array is cut into
//                regions of 2^r_shift floats; each workgroup histograms its share of the blocks per
//                region in LDS and adds the counts to a global table.  A block that runs past the
//                end of its region (or of the array) counts in both regions it touches.
//   R3 scan      exclusive prefix sum: first record slot of every region.
//   R4 scatter   same walk as R2; a workgroup reserves its slots of every region with one integer
//                atomic per region and writes (offset, source block [, sign term]) records.
//   R5 reduce    one workgroup per region: the region's records are applied to an LDS copy of the
//                region with plain read-modify-writes - float atomics in LDS are as slow as those
//                in memory - made race-free by ownership: the region is cut into one slice per lane
//                group, a batch of records is counting-sorted by slice with integer atomics, every
//                group applies the records that start in its slice, and the elements that reach past
//                a slice's end are applied after a barrier.  The finished region is then added to
//                grad_array with coalesced plain read-modify-writes - or, fused, fed straight into
//                the Adagrad update of array and state, so that the gradient never exists in HBM.
//
// Every array slot is owned by exactly one workgroup, so nothing here is atomic on floats.  The order
// of the additions inside a region follows the order of its records, which is not fixed.
#pragma once
#include "robe_kernels.h"

namespace robe {

constexpr int kRowsAhead = 8;          // gradient rows a lane group requests before adding them (R1)
constexpr int kStretch = 8;            // stretches of G sorted positions a lane group walks in R1, at most (RegionPlan::stretch)
constexpr int kBinBlock = 1024;        // R2 / R4
constexpr int kReduceBlock = 512;      // R5 (the slice arithmetic assumes 2^9)
constexpr uint32_t kMaxRecordLanes = 64;   // lanes per record in R5: a lane group must stay inside one wavefront
static_assert(kReduceBlock == 512 && kReduceBlock % 64 == 0, "R5: 2^9 threads, whole wavefronts");
// Records sorted and applied per round in R5 (at most 2 per thread).  32 KB region + batch (8 bytes
// a record, 12 with the sign term) + counters + spill-over rows stay under 40 KB: four workgroups per CU.
template <bool SIGN>
constexpr int rec_batch() { return SIGN ? 448 : 640; }
constexpr uint32_t kSpillFloats = 512; // LDS floats for the spill-over rows of R5 (used when groups * Z fits)
constexpr int kRecAhead = 8;           // gradient blocks a lane group requests before adding them (R5)
constexpr int kWb = 1;                 // vectors per thread and pass in the dense write-back of R5 (more did not pay: registers)
constexpr int kCanonAhead = 4;         // records of a slice compared per step when R5 puts them in canonical order
constexpr uint32_t kMaxRegions = 32768;
constexpr uint32_t kMaxClassShift = 10;  // R5 splits an overfull region into at most 2^10 classes (the table lives in the batch area)
constexpr uint32_t kPartBit = 0x80000000u;   // record flag: the elements past the end of the block's own region
constexpr uint32_t kDeadRecord = 0xFFFFFFFFu;
constexpr uint32_t kNoRun = 0xFFFFFFFFu;     // src_row of a sorted position where no run starts

struct RegionPlan {
    uint32_t r_shift;        // log2 of the region size in floats
    uint32_t NR;             // regions = ceil(m / 2^r_shift)
    uint32_t n;              // sorted token positions
    uint32_t rows;           // rows of grad_out
    uint32_t src_own;        // blocks of Z floats in grad_out: source blocks below this live there, the rest in P
    uint32_t src_blocks;     // src_own + P rows * C: exclusive bound of a record's source block
    uint32_t bin_blocks;     // grid of R2 / R4
    uint32_t pos_per_block;  // sorted positions per workgroup in R2 / R4
    uint32_t lg_shift;       // log2 of the lanes per record in R5
    uint32_t fullest_first;  // 1: R5 takes the regions by descending size class instead of by address
    uint32_t keep_rows;      // 1: gradient rows are read more than once (bags): R5 loads them with the default cache policy
    uint32_t sparse_regions; // 1: the tokens reach a small part of the array: R5 writes back by a list of touched granules
    uint32_t keep_array;     // 1: R5 updates the array (Adagrad, SGD) and leaves it in the caches for the next forward pass (small arrays)
    // gather variant of R5 (no R2..R4): the range table has NE = C * epc entries, epc = kmax + 3 with
    // kmax = (P - 1) / m; dir[b] is the first sorted position whose key >> dir_shift is >= b
    // (dir[buckets] = n), written by R1; NULL when R2..R4 run instead
    uint32_t NE, epc, epc_recip, dir_shift, dir_buckets;   // epc_recip = ceil(2^16 / epc)
    uint32_t key_mask;       // the key bits: 2^31 - 1, or fewer when the keys are array offsets (blocks larger than embeddings)
    uint32_t *dir;
    const uint32_t *keys;    // sorted keys
    uint8_t *head;           // [n]  1: a run starts here
    uint32_t *src_row;       // [n]  at run starts: the first source block of the run's row (in grad_out, or src_own + row of P * C); else kNoRun
    uint32_t *run_c;         // [n]  at run starts: chunks of the run's embedding; NULL unless tables differ in dimension (then C is the most any has)
    uint32_t *run_tg;        // [n]  at run starts: token part of the sign hash (sign on only)
    uint32_t stretch;        // stretches of G sorted positions a lane group of R1 walks (1 .. kStretch)
    uint32_t p_quota;        // rows of P per lane group of R1
    float *P;                // [lane groups of R1 * p_quota][d] summed rows of the runs longer than one (d: the widest table's)
    uint32_t *counts, *starts;   // [NR], [NR + 1]; after R3 counts holds the order of the regions for R5
    uint32_t *wg_first;      // [bin_blocks][NR]: R2 -> R4, see region_bin_kernel
    uint2 *rec;              // [<= 2 * n * C] (offset, source block | part flag)
    uint32_t *rec_tg;        // sign on only
};

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *dst, uint32_t n, uint32_t v)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) dst[i] = v;
}

// ---------------------------------------------------------------------------------------------
// R1.  Lane layout as in the direct scatter: G lanes per row, lane `grp` owns elements grp + k*G.
// A group walks s.stretch * G consecutive sorted positions, G at a time; a run is cut only where the
// group's walk begins and ends, so a token that fills whole stretches leaves one record per
// s.stretch * G copies.
// ---------------------------------------------------------------------------------------------
struct SortedToken {
    uint32_t th, sb, dd, e, xlo, xhi, tg;    // sb: first block of Z floats of its gradient row; dd: its dimension
    bool ok;
};

// Equal keys write equal slots; with the sign on the token itself must agree (g hashes it again), and
// among tables of different dimensions the table must (two tables may share a key by collision).
template <bool SIGN>
__device__ __forceinline__ bool same_token(const SortedToken &a, const SortedToken &b, bool mixed)
{
    bool same = a.th == b.th;
    if (mixed) same = same && a.e == b.e;
    if constexpr (SIGN) same = same && a.e == b.e && a.xlo == b.xlo && a.xhi == b.xhi;
    return same;
}

template <bool SIGN>
__device__ __forceinline__ SortedToken shfl_token(const SortedToken &t, int from, bool mixed)
{
    SortedToken r;
    r.th = __shfl(t.th, from);
    r.ok = __shfl((int)t.ok, from) != 0;
    r.sb = 0;
    r.dd = 0;
    r.tg = 0;
    r.e = (SIGN || mixed) ? __shfl(t.e, from) : 0u;
    r.xlo = SIGN ? __shfl(t.xlo, from) : 0u;
    r.xhi = SIGN ? __shfl(t.xhi, from) : 0u;
    return r;
}

template <int V, bool SIGN, bool BAGS, bool MIXED>
__global__ __launch_bounds__(kBlock) void combine_rows_kernel(Params p, Geom q, RegionPlan s,
                                                              const float *__restrict__ grad_out,
                                                              const int64_t *__restrict__ indices,
                                                              const uint32_t *__restrict__ vals,     // sorted with the keys
                                                              const uint32_t *__restrict__ tok_bag)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t grp = lane & (q.G - 1u);
    const uint32_t base_lane = lane - grp;
    const uint32_t n = s.n;
    const uint64_t thread_id = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    // the record counts of R2 start at zero (this kernel is the last one before it)
    if (s.counts != nullptr)
        for (uint64_t i = thread_id; i < s.NR; i += (uint64_t)gridDim.x * kBlock) s.counts[i] = 0;
    if ((thread_id - lane) * s.stretch >= n) return;    // the whole wavefront is past the end
    const uint64_t i_first = (thread_id - grp) * s.stretch;  // first sorted position of this group's walk

    // the token at a sorted position (lane l of the group looks at position i0 + l)
    constexpr bool mixed = MIXED;                       // tables of different dimensions (every one a multiple of Z): q.tables
    auto fetch = [&](uint64_t pos) -> SortedToken {
        SortedToken t;
        t.th = t.sb = t.e = t.xlo = t.xhi = t.tg = 0;
        t.dd = q.d;
        t.ok = false;
        if (pos < n) {
            const uint32_t v = vals[pos];                  // sign off: the row itself (see robe_backward_dedup.h)
            const uint32_t row = !SIGN ? v : (v < n ? (BAGS ? tok_bag[v] : v) : s.rows);
            t.th = s.keys[pos];                            // also for a token that is not ok: the directory covers every position
            if (row < s.rows && t.th < kP) {               // (a key that is no residue: a position no bag of a malformed CSR wrote)
                t.ok = true;
                t.sb = row * p.C;
                if (SIGN || mixed) t.e = row % q.F;
                if (mixed) {
                    const uint2 tab = q.tables[t.e];
                    t.sb = (uint32_t)(((uint64_t)(row / q.F) * (uint64_t)q.row_floats + tab.x) / p.Z);
                    t.dd = tab.y;
                }
                if constexpr (SIGN) {
                    const int64_t x = indices[v];
                    t.xlo = (uint32_t)x;
                    t.xhi = (uint32_t)((uint64_t)x >> 32);
                    t.tg = staged_g(p, x, t.e);
                }
            }
        }
        return t;
    };

    float acc[V];
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = 0.0f;
    uint32_t head_pos = 0;
    // Rows of P: every lane group owns p_quota of them, at row (group number) * p_quota, and hands
    // them to the runs longer than one that start in its walk, in order.  A group that meets more
    // such runs leaves the rest uncombined: each of their tokens becomes a run of its own.
    const uint32_t p_first = (uint32_t)((thread_id - grp) >> q.g_shift) * s.p_quota;
    uint32_t n_multi = 0, run_slot = 0;        // multi-token runs started so far; slot of the run being summed
    uint32_t open_slot = 0;                    // slot of the run that the stretch before left open, if it has one
    bool open_over = false;                    // ... or whether that run found the quota used up

    SortedToken cur = fetch(i_first + grp);
    SortedToken carry;          // the last token of the stretch before; none before the first
    carry.th = carry.sb = carry.dd = carry.e = carry.xlo = carry.xhi = carry.tg = 0;
    carry.ok = false;
    if (s.dir != nullptr && i_first > 0 && i_first <= n) carry.th = s.keys[i_first - 1];   // its key only: the directory needs it
    for (uint32_t st = 0; st < s.stretch; ++st) {
        const uint64_t i0 = i_first + (uint64_t)st * q.G;
        if (__all(i0 >= n)) break;                          // every group of the wavefront is past the end
        SortedToken nxt;
        if (st + 1u < s.stretch) {
            nxt = fetch(i0 + q.G + grp);
        } else {
            nxt = carry;
            nxt.ok = false;
        }
        // does a run start here (a different token than the one before, or the walk begins), and
        // does it end here (a different token after, or the walk ends)?
        SortedToken before = shfl_token<SIGN>(cur, (int)(base_lane + (grp ? grp - 1u : 0u)), mixed);
        if (grp == 0) before = carry;
        const bool my_head = cur.ok && (!before.ok || !same_token<SIGN>(before, cur, mixed));
        SortedToken after = shfl_token<SIGN>(cur, (int)(base_lane + (grp + 1u < q.G ? grp + 1u : grp)), mixed);
        const SortedToken first_of_next = shfl_token<SIGN>(nxt, (int)base_lane, mixed);
        if (grp + 1u >= q.G) after = first_of_next;
        const bool my_end = cur.ok && (!after.ok || !same_token<SIGN>(after, cur, mixed));
        bool my_single = my_head && my_end;
        // the slot of the run every position belongs to: the run of the last head at or before it (none:
        // the run left open by the stretch before), counted among this walk's multi-token runs
        uint32_t my_slot = open_slot;
        bool my_over = open_over;
        {
            const uint64_t gmask = q.G >= 64u ? ~0ull : ((1ull << q.G) - 1ull);
            const uint64_t heads = (__ballot(my_head) >> base_lane) & gmask;
            const uint64_t multi = (__ballot(my_head && !my_end) >> base_lane) & gmask;
            const uint64_t upto = heads & ((2ull << grp) - 1ull);
            if (upto) {
                const uint32_t hl = 63u - (uint32_t)__builtin_clzll(upto);
                my_slot = n_multi + (uint32_t)__popcll(multi & ((1ull << hl) - 1ull));
                my_over = my_slot >= s.p_quota;
            }
            n_multi += (uint32_t)__popcll(multi);
        }
        if (cur.ok && !my_single && my_over) my_single = true;     // no row of P left: this token alone
        const bool my_lead = my_head || (cur.ok && my_over);      // a record starts at this position

        // Directory for the gather variant of R5: the first sorted position of every key bucket.  The
        // position whose bucket differs from the one before it writes the entries in between (a long gap
        // is shared out over the wavefront), the last position writes the rest.
        if (s.dir != nullptr) {
            const uint64_t pos = i0 + grp;
            uint32_t blo = 1, bhi = 0;                           // empty
            if (pos < n) {
                // (bits above the key bits: the sort ignores them, so they are masked to keep the buckets in order)
                blo = pos == 0 ? 0u : ((before.th & s.key_mask) >> s.dir_shift) + 1u;
                bhi = (cur.th & s.key_mask) >> s.dir_shift;
            }
            const bool any = blo <= bhi, wide = any && bhi - blo >= 16u;
            if (any && !wide)
                for (uint32_t b = blo; b <= bhi; ++b) s.dir[b] = (uint32_t)pos;
            uint32_t clo = bhi + 1u;                            // what the last position closes: (its bucket, buckets]
            uint64_t todo = __ballot(wide), closer = __ballot(pos + 1u == n);
            while (todo) {
                const int l = __builtin_ctzll(todo);
                todo &= todo - 1ull;
                const uint32_t lo = __shfl(blo, l), hi = __shfl(bhi, l), v = __shfl((uint32_t)pos, l);
                for (uint32_t b = lo + lane; b <= hi; b += 64u) s.dir[b] = v;
            }
            if (closer) {
                const uint32_t lo = __shfl(clo, __builtin_ctzll(closer));
                for (uint32_t b = lo + lane; b <= s.dir_buckets; b += 64u) s.dir[b] = n;
            }
        }

        if (i0 + grp < n) {
            if (s.head != nullptr) s.head[i0 + grp] = my_lead ? 1 : 0;
            // a run of one reads grad_out in place; the head of a longer run gets its row of P when the run
            // ends; every other position says that no run starts there (the gather variant of R5 reads
            // this array alone to find the runs)
            if (my_single) s.src_row[i0 + grp] = cur.sb;
            else if (!my_head) s.src_row[i0 + grp] = kNoRun;
            if constexpr (SIGN) {
                if (my_lead) s.run_tg[i0 + grp] = cur.tg;
            }
            if (mixed && my_lead) s.run_c[i0 + grp] = cur.dd / p.Z;
        }

        // runs longer than one: sum their rows into P (a run may have begun in an earlier stretch)
        for (uint32_t k0 = 0; k0 < q.G; k0 += kRowsAhead) {     // same trip count for every lane of the wavefront
            uint32_t sb[kRowsAhead], dd[kRowsAhead], slot[kRowsAhead];
            bool use[kRowsAhead], head[kRowsAhead], end[kRowsAhead];
            // what the loop below needs of a position, in one word: its run's slot, whether the position
            // takes part, starts a run, ends one
            const uint32_t mine = (my_slot << 3) | ((cur.ok && !my_single) ? 4u : 0u) | (my_head ? 2u : 0u) | (my_end ? 1u : 0u);
#pragma unroll
            for (int u = 0; u < kRowsAhead; ++u) {
                const int from = (int)(base_lane + ((k0 + u) & (q.G - 1u)));
                const bool in = k0 + u < q.G;
                const uint32_t theirs = __shfl(mine, from);
                sb[u] = __shfl(cur.sb, from);
                dd[u] = mixed ? __shfl(cur.dd, from) : q.d;
                use[u] = in && (theirs & 4u) != 0;
                head[u] = (theirs & 2u) != 0;
                end[u] = (theirs & 1u) != 0;
                slot[u] = theirs >> 3;
            }
            float v[kRowsAhead][V];
#pragma unroll
            for (int u = 0; u < kRowsAhead; ++u) {
                if (use[u]) load_row_of<V, BAGS>(grad_out + (uint64_t)sb[u] * p.Z, q.G, dd[u], grp, v[u]);
            }
#pragma unroll
            for (int u = 0; u < kRowsAhead; ++u) {
                if (!use[u]) continue;
                if (head[u]) {
                    head_pos = (uint32_t)i0 + k0 + u;
                    run_slot = slot[u];
#pragma unroll
                    for (int k = 0; k < V; ++k) acc[k] = 0.0f;
                }
#pragma unroll
                for (int k = 0; k < V; ++k) acc[k] += v[u][k];
                if (end[u]) {
                    const uint32_t prow = p_first + run_slot;
                    store_row<V, false>(s.P + (uint64_t)prow * p.d, q, grp, acc);
                    if (grp == 0) s.src_row[head_pos] = s.src_own + prow * p.C;
                }
            }
        }
        carry = shfl_token<SIGN>(cur, (int)(base_lane + q.G - 1u), mixed);
        open_slot = __shfl(my_slot, (int)(base_lane + q.G - 1u));
        open_over = __shfl((int)my_over, (int)(base_lane + q.G - 1u)) != 0;
        cur = nxt;
    }
}

// ---------------------------------------------------------------------------------------------
// R2 / R4.  Walk this workgroup's sorted positions; call f(offset, source block, region, part flag,
// sign term) for every block of every run, twice when the block leaves its region.
// ---------------------------------------------------------------------------------------------
constexpr int kBinAhead = 4;

template <bool SIGN, typename F>
__device__ __forceinline__ void for_each_block(const Params &p, const RegionPlan &s, F f)
{
    const uint64_t b = (uint64_t)blockIdx.x * s.pos_per_block;
    uint64_t e = b + s.pos_per_block;
    if (e > s.n) e = s.n;
    // kBinAhead positions per thread and trip, their flag, key and source row all requested at once
    // (for positions that head no run the last two are read for nothing: a thread that asked for the
    // flag first and the rest after spent the sweep in two dependent trips to memory per position)
    for (uint64_t i0 = b + threadIdx.x; i0 < e; i0 += (uint64_t)kBinBlock * kBinAhead) {
        uint32_t hd[kBinAhead], th[kBinAhead], sr[kBinAhead], tgv[kBinAhead], nc[kBinAhead];
#pragma unroll
        for (int u = 0; u < kBinAhead; ++u) {
            const uint64_t i = i0 + (uint64_t)u * kBinBlock;
            const uint64_t at = i < e ? i : i0;               // i0 < e: a position of this workgroup
            hd[u] = i < e ? s.head[at] : 0u;
            th[u] = s.keys[at];
            sr[u] = s.src_row[at];
            tgv[u] = SIGN ? s.run_tg[at] : 0u;
            nc[u] = s.run_c != nullptr ? s.run_c[at] : p.C;
        }
#pragma unroll
        for (int u = 0; u < kBinAhead; ++u) {
            if (!hd[u]) continue;
            const uint32_t src0 = sr[u];
            const uint32_t chunks = nc[u] < p.C ? nc[u] : p.C;
            uint32_t cc = 0;  // (Ch * c) mod P, built up by addition
            uint32_t tgc = tgv[u];   // sign term of the chunk's element 0: the token's plus (Cg * c * Z) mod P
            const uint32_t tg_step = SIGN ? mod_p((uint64_t)p.Cg * p.Z) : 0u;
            for (uint32_t c = 0; c < chunks; ++c) {
                const uint32_t o = offset_of(p, th[u], cc);
                uint32_t r = o >> s.r_shift;
                f(o, src0 + c, r, 0u, tgc);
                // the regions the block enters after its own: normally at most one; two when the array
                // ends in a region shorter than the block and the block passes through it to slot 0
                uint64_t r_end = ((uint64_t)(r + 1u) << s.r_shift) < p.m ? ((uint64_t)(r + 1u) << s.r_shift) : p.m;
                uint64_t left = (uint64_t)o + p.Z > r_end ? (uint64_t)o + p.Z - r_end : 0u;
                for (int hop = 0; hop < 2 && left > 0; ++hop) {
                    r = r_end == p.m ? 0u : r + 1u;
                    f(o, src0 + c, r, kPartBit, tgc);
                    const uint64_t r_begin = (uint64_t)r << s.r_shift;
                    r_end = ((uint64_t)(r + 1u) << s.r_shift) < p.m ? ((uint64_t)(r + 1u) << s.r_shift) : p.m;
                    left = left > r_end - r_begin ? left - (r_end - r_begin) : 0u;
                }
                cc = add_p(cc, p.Ch);
                if constexpr (SIGN) tgc = add_p(tgc, tg_step);
            }
        }
    }
}

// R2 counts this workgroup's records per region in LDS and adds the counts to the regions' totals;
// what each addition returns - how many records of the region the workgroups before it (in arrival
// order) hold - is kept in wg_first[workgroup][region].  R4, launched with the same grid after the
// prefix sums of R3, starts its LDS cursors at starts[region] + wg_first and writes every record in
// one sweep, with no further global atomics.
template <bool SIGN, bool SCATTER>
__global__ __launch_bounds__(kBinBlock) void region_bin_kernel(Params p, RegionPlan s)
{
    extern __shared__ uint32_t hist[];  // NR counters (R2) or cursors (R4)
    uint32_t *mine = s.wg_first + (uint64_t)blockIdx.x * s.NR;
    if constexpr (!SCATTER) {
        for (uint32_t r = threadIdx.x; r < s.NR; r += kBinBlock) hist[r] = 0;
        __syncthreads();
        for_each_block<false>(p, s, [&](uint32_t, uint32_t, uint32_t r, uint32_t, uint32_t) { atomicAdd(&hist[r], 1u); });
        __syncthreads();
        for (uint32_t r = threadIdx.x; r < s.NR; r += kBinBlock) {
            const uint32_t c = hist[r];
            if (c) mine[r] = atomicAdd(&s.counts[r], c);     // regions without records of this workgroup: never read
        }
    } else {
        for (uint32_t r = threadIdx.x; r < s.NR; r += kBinBlock) hist[r] = s.starts[r] + mine[r];
        __syncthreads();
        const uint32_t cap = s.starts[s.NR];                 // all records counted by R2
        for_each_block<SIGN>(p, s, [&](uint32_t o, uint32_t src, uint32_t r, uint32_t part, uint32_t tg) {
            const uint32_t slot = atomicAdd(&hist[r], 1u);
            if (slot < cap) {  // always true unless the inputs changed between R2 and R4
                s.rec[slot] = make_uint2(o, src | part);
                if constexpr (SIGN) s.rec_tg[slot] = tg;
            }
        });
    }
}

// R3: one workgroup.  starts: exclusive prefix of counts, grand total in starts[NR];
// then the order in which R5 takes the regions.
constexpr uint32_t kScanPer = kMaxRegions / 1024u;

// Exclusive prefix sums over kMaxRegions values in index order, by one workgroup of 1024 threads.
// Thread t holds elements t, t + 1024, ... (coalesced loads, all requested at once); every chunk of
// 1024 is scanned inside the wavefronts by shuffles, and the 32 x 16 (chunk, wavefront) totals are
// scanned once more to give every wavefront its base in every chunk.  Returns the grand total.
__device__ __forceinline__ uint32_t block_scan(const uint32_t (&c)[kScanPer], uint32_t (&excl)[kScanPer],
                                               uint32_t *base /* [kScanPer * 16] */, uint32_t *upper /* [8] */)
{
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
#pragma unroll
    for (uint32_t k = 0; k < kScanPer; ++k) {
        uint32_t v = c[k];
#pragma unroll
        for (uint32_t off = 1; off < 64u; off <<= 1) {
            const uint32_t up = __shfl_up(v, off);
            if (lane >= off) v += up;
        }
        excl[k] = v - c[k];
        if (lane == 63u) base[k * 16u + wave] = v;
    }
    __syncthreads();
    // exclusive scan of the 512 totals in (chunk, wavefront) order, by the first 512 threads
    uint32_t x = 0, xi = 0;
    if (t < kScanPer * 16u) {
        x = base[t];
        xi = x;
#pragma unroll
        for (uint32_t off = 1; off < 64u; off <<= 1) {
            const uint32_t up = __shfl_up(xi, off);
            if (lane >= off) xi += up;
        }
        if (lane == 63u) upper[wave] = xi;
    }
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (uint32_t w = 0; w < 8u; ++w) {
        const uint32_t u = upper[w];
        before += w < wave ? u : 0u;
        total += u;
    }
    if (t < kScanPer * 16u) base[t] = before + xi - x;
    __syncthreads();
#pragma unroll
    for (uint32_t k = 0; k < kScanPer; ++k) excl[k] += base[k * 16u + wave];
    __syncthreads();    // base and upper may be reused
    return total;
}

__global__ __launch_bounds__(1024) void region_scan_kernel(RegionPlan s)
{
    __shared__ uint32_t base[kScanPer * 16u];
    __shared__ uint32_t upper[8];
    const uint32_t t = threadIdx.x;
    uint32_t c[kScanPer], at[kScanPer];
#pragma unroll
    for (uint32_t k = 0; k < kScanPer; ++k) c[k] = k * 1024u + t < s.NR ? s.counts[k * 1024u + t] : 0u;
    const uint32_t total = block_scan(c, at, base, upper);
#pragma unroll
    for (uint32_t k = 0; k < kScanPer; ++k) {
        const uint32_t i = k * 1024u + t;
        if (i < s.NR) {
            s.starts[i] = at[k];
        }
    }
    if (t == 0) s.starts[s.NR] = total;

    // Order in which R5 takes the regions (it overwrites counts, which nothing reads after this
    // kernel; every thread has its counts in registers by now).  With few regions per workgroup
    // slot the ones the frequent tokens hit, which take several times the average, must not end up
    // as the tail of the launch: fullest first, by power-of-two size class.  With many regions per
    // slot the tails even out and the address order is as good or better.
    if (!s.fullest_first) {
#pragma unroll
        for (uint32_t k = 0; k < kScanPer; ++k) {
            if (k * 1024u + t < s.NR) s.counts[k * 1024u + t] = k * 1024u + t;
        }
        return;
    }
    __shared__ uint32_t cls_n[32], cls_at[32];
    if (t < 32u) cls_n[t] = 0;
    __syncthreads();
#pragma unroll
    for (uint32_t k = 0; k < kScanPer; ++k) {
        if (k * 1024u + t < s.NR) atomicAdd(&cls_n[31 - __clz((int)(c[k] | 1u))], 1u);
    }
    __syncthreads();
    if (t == 0) {
        uint32_t a = 0;
        for (int cls = 31; cls >= 0; --cls) {
            cls_at[cls] = a;
            a += cls_n[cls];
        }
    }
    __syncthreads();
#pragma unroll
    for (uint32_t k = 0; k < kScanPer; ++k) {
        const uint32_t i = k * 1024u + t;
        if (i < s.NR) s.counts[atomicAdd(&cls_at[31 - __clz((int)(c[k] | 1u))], 1u)] = i;
    }
}

// ---------------------------------------------------------------------------------------------
// R5.  RULE 0: dst += lr * region, each operation rounded on its own (lr = 1: the scatter onto a
// gradient array; lr = minus the learning rate: SGD on the array, the gradient never in memory).
// RULE 1: Adagrad on array / state with the region as gradient.
//
// Where a region's records come from:
//   GATHER = false   from the region-sorted copy that R2..R4 wrote (s.rec).
//   GATHER = true    straight from the sorted token list, with no R2..R4 at all.  Block c of a token
//                    with key th starts at ((th + (Ch c mod P)) mod P) mod m, so the tokens whose
//                    block c meets a given region are those with th in a few contiguous ranges - one
//                    per multiple of m below P - and a range of keys is a stretch of the sorted list.
//                    The workgroup works those ranges out (R5-a), finds the stretches through a
//                    directory that R1 left (first sorted position of every key bucket), and walks
//                    them eight positions per thread, picking up the runs that start there.  The
//                    order in which records are staged is a function of the sorted list alone, so
//                    the reproducible variant needs no class split here.
// ---------------------------------------------------------------------------------------------
// tg: the sign term of the block's element 0 (the token's term plus (Cg * c * Z) mod P for chunk c)
template <bool SIGN>
__device__ __forceinline__ float signed_block_value(const Params &p, float v, uint32_t tg, uint32_t j)
{
    if constexpr (SIGN) {
        return apply_sign(v, sign_mask(add_p(tg, mod_p((uint64_t)p.Cg * j))));
    } else {
        return v;
    }
}

// Class of a record among 2^shift classes: a fixed hash of its offset and source word.  (Two records
// that agree in both come from copies of one token in one bag and are interchangeable.)
__device__ __forceinline__ uint32_t record_class(uint2 rec, uint32_t shift)
{
    return ((rec.y * 0x9E3779B1u) ^ (rec.x * 0x85EBCA6Bu + 0xC2B2AE35u) * 0x27D4EB2Fu) >> (32u - shift);
}

// Which elements of a record a region holds.  Element j of a block at offset o sits at array position
// (o + j) mod m.  A record without the part flag starts inside the region (r0 <= o < r0 + len) and
// keeps the elements before the region's end; one with the flag belongs to a block that starts before
// the region and enters it at its first slot, with element js = (r0 - o) mod m, 0 < js < Z.  Element j
// lands in region slot abase + j (unsigned wrap-around arithmetic) for jlo <= j < jhi.
struct RecordSpan {
    uint32_t abase, jlo, jhi;
    bool ok;
};

__device__ __forceinline__ RecordSpan span_of(uint32_t o, bool part, uint32_t r0, uint32_t region_len, uint32_t m, uint32_t Z)
{
    RecordSpan sp;
    if (!part) {
        sp.ok = o >= r0 && o - r0 < region_len;
        const uint32_t keep = r0 + region_len - o;
        sp.abase = o - r0;
        sp.jlo = 0;
        sp.jhi = keep < Z ? keep : Z;
    } else {
        const uint32_t js = r0 >= o ? r0 - o : r0 + (m - o);
        sp.ok = js > 0 && js < Z;
        sp.abase = 0u - js;
        sp.jlo = js;
        sp.jhi = js + region_len < Z ? js + region_len : Z;
    }
    return sp;
}

// Inclusive prefix sums of one value per thread over the first WAVES wavefronts of the workgroup
// (the values of the other threads are not looked at and their result is meaningless); `total` is
// valid in every thread.  One barrier; wave_tot is LDS for one word per wavefront, free again after
// the workgroup's next barrier.
template <uint32_t WAVES>
__device__ __forceinline__ uint32_t reduce_block_scan(uint32_t v, uint32_t *wave_tot, uint32_t &total)
{
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint32_t incl = v;
    if (wave < WAVES) {                       // uniform over a wavefront
#pragma unroll
        for (uint32_t off = 1; off < 64u; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane == 63u) wave_tot[wave] = incl;
    }
    __syncthreads();
    uint32_t before = 0;
    total = 0;
#pragma unroll
    for (uint32_t w = 0; w < WAVES; ++w) {
        const uint32_t x = wave_tot[w];
        before += w < wave ? x : 0u;
        total += x;
    }
    return before + incl;
}

// R5-a.  Entry e of a region's range table: chunk c = e / epc of the embedding, and within the chunk
// either the k-th multiple of m (k = e % epc <= kmax + 1) or, for the last entry, the lower part of
// the one range that the wrap-around of (th + cc) mod P cuts in two.  Gives the keys [ta, tb) (empty
// when ta >= tb) whose block c meets [r0 - Z + 1, r0 + len) modulo m.
struct KeyRange {
    uint32_t ta, tb, cc, c;
};

__device__ __forceinline__ KeyRange key_range(const Params &p, const RegionPlan &s, uint32_t e, uint32_t r0, uint32_t region_len)
{
    KeyRange kr;
    kr.c = (e * s.epc_recip) >> 16;              // e / epc for e < 2^8 (the host checks the reciprocal)
    const uint32_t j = e - kr.c * s.epc;
    kr.cc = mod_p((uint64_t)p.Ch * kr.c);
    kr.ta = kr.tb = 0;
    const int64_t lo = (int64_t)r0 - (int64_t)p.Z + 1, hi = (int64_t)r0 + region_len, cc = kr.cc, P = kP;
    int64_t k = j;
    if (j + 1u == s.epc) {                       // the split entry: which multiple of m holds cc?
        if (cc < lo) return kr;
        const uint32_t x = (uint32_t)(cc - lo);  // <= P + Z: 32 bits; x / m by the reciprocal, low by at most one
        uint32_t q = __umulhi(x, p.m_recip);
        if (x - q * p.m >= p.m) ++q;
        k = q;
        if (k > (int64_t)s.epc - 2) return kr;
    }
    int64_t a = k * p.m + lo, b = k * p.m + hi;
    if (a < 0) a = 0;
    if (b > P) b = P;
    if (a >= b) return kr;
    if (j + 1u == s.epc) {
        if (a < cc && cc < b) { kr.ta = (uint32_t)(a + P - cc); kr.tb = (uint32_t)P; }
    } else if (a >= cc) {
        kr.ta = (uint32_t)(a - cc); kr.tb = (uint32_t)(b - cc);
    } else if (b <= cc) {
        kr.ta = (uint32_t)(a + P - cc); kr.tb = (uint32_t)(b + P - cc);
    } else {
        kr.ta = 0; kr.tb = (uint32_t)(b - cc);
    }
    return kr;
}

// Records staged and applied per round.  32 KB region + batch (8 bytes a record, 12 with the sign
// term) + counters + spill-over rows (+ the range table) stay under 40 KB: four workgroups per CU.
template <bool SIGN, bool GATHER>
constexpr int reduce_batch() { return GATHER ? (SIGN ? 384 : 512) : rec_batch<SIGN>(); }
// Range-table entries that fit beside that (8 bytes each).
template <bool SIGN>
constexpr uint32_t gather_entries_max() { return SIGN ? 56u : 120u; }
constexpr uint32_t kGatherChunk = 4;     // sorted positions a thread of the gather variant looks at per round
static_assert(kGatherChunk == 4, "one uint4 of keys per thread");
constexpr uint32_t kReduceWords = 64 + 65 + 1 + 8 + 2;   // slice counters, slice starts, stage counter, scan totals, round totals

__host__ __device__ constexpr size_t reduce_lds_bytes(uint32_t r_shift, bool sign, bool gather, bool spill)
{
    const size_t batch = gather ? (sign ? 384u : 512u) : (sign ? 448u : 640u);
    return ((size_t)1 << r_shift) * 4 + batch * (sign ? 12u : 8u) + kReduceWords * 4 + (spill ? (size_t)kSpillFloats * 4 : 0)
           + (gather ? ((size_t)(sign ? 56u : 120u) * 2 + 1) * 4 + 512u : 0);   // range table, and the entry of each of the first 512 chunks
}
static_assert(reduce_lds_bytes(13, false, false, true) <= 40960 && reduce_lds_bytes(13, true, false, true) <= 40960 &&
              reduce_lds_bytes(13, false, true, true) <= 40960 && reduce_lds_bytes(13, true, true, true) <= 40960,
              "R5 with 32 KB regions: four workgroups per CU");

template <bool SIGN, int RULE, bool CANON, bool SPILL, bool GATHER>
__global__ __launch_bounds__(kReduceBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void region_reduce_kernel(Params p, RegionPlan s,
                                                                     const float *__restrict__ grad_out,
                                                                     float *__restrict__ dst,      // RULE 0: grad_array, or the array (SGD); RULE 1: array
                                                                     float *__restrict__ state,    // RULE 1 only
                                                                     float lr, float eps, int vec_ok)
{
    constexpr int kRecBatch = reduce_batch<SIGN, GATHER>();
    constexpr int kPer = (kRecBatch + kReduceBlock - 1) / kReduceBlock;     // records per thread and round
    extern __shared__ float acc[];  // 2^r_shift floats, then the batch staging area
    const uint32_t r = GATHER ? blockIdx.x : s.counts[blockIdx.x];     // records path, after R3: the regions, fullest first
    if (r >= s.NR) return;
    uint32_t rb = 0, re = 0;
    if constexpr (!GATHER) {
        rb = s.starts[r];
        re = s.starts[r + 1];
        if (rb >= re) return;           // nothing lands in this region: it is not touched at all
    }

    const uint32_t R = 1u << s.r_shift;
    const uint32_t r0 = r << s.r_shift;
    const uint32_t region_len = (p.m - r0) < R ? (p.m - r0) : R;
    const uint32_t src_own = s.src_own;      // source blocks below this live in grad_out, the rest in P

    uint2 *srt = reinterpret_cast<uint2 *>(acc + R);
    uint32_t *srt_tg = reinterpret_cast<uint32_t *>(srt + kRecBatch);
    uint32_t *cnt = srt_tg + (SIGN ? kRecBatch : 0);   // 64 slice counters
    uint32_t *pre = cnt + 64;                          // 65 slice starts
    uint32_t *sel = pre + 65;                          // records staged for this round
    uint32_t *wave_tot = sel + 1;                      // 8 words for the block scans
    uint32_t *round_tot = wave_tot + 8;                // 2 words: chunks taken, records staged (gather)
    float *spill_base = reinterpret_cast<float *>(round_tot + 2);
    // this group's spill-over row, as an index into acc
    const uint32_t spill_at = (uint32_t)(spill_base - acc) + (threadIdx.x >> s.lg_shift) * p.Z;
    uint32_t *tab_pa = reinterpret_cast<uint32_t *>(spill_base + (SPILL ? kSpillFloats : 0u));   // gather: first position (a multiple of 8) of every range
    uint32_t *tab_cum = tab_pa + gather_entries_max<SIGN>();                                    // gather: chunks before every range, total last
    uint8_t *chunk_entry = reinterpret_cast<uint8_t *>(tab_cum + gather_entries_max<SIGN>() + 1);   // gather: the range of each of the first kReduceBlock chunks

    // R5-a: the ranges of this region and where they sit in the sorted list
    uint32_t total_chunks = 0;
    if constexpr (GATHER) {
        uint32_t pa = 0, pb = 0;
        if (threadIdx.x < s.NE) {
            const KeyRange kr = key_range(p, s, threadIdx.x, r0, region_len);
            const uint32_t tb = kr.tb <= s.key_mask ? kr.tb : s.key_mask + 1u;      // no key has a bit above the mask
            if (kr.ta < kr.tb && kr.ta < tb) {
                pa = s.dir[kr.ta >> s.dir_shift];
                pb = s.dir[((tb - 1u) >> s.dir_shift) + 1u];
            }
        }
        // (the region is cleared while the directory entries are on their way)
        for (uint32_t i = threadIdx.x; i < region_len; i += kReduceBlock) acc[i] = 0.0f;
        uint32_t my_chunks = 0, my_pa = 0;
        pb = pb < s.n ? pb : s.n;                            // (whatever the directory holds, nothing past the list is read)
        if (pb > pa) {
            my_pa = pa & ~(kGatherChunk - 1u);
            my_chunks = (pb - my_pa + kGatherChunk - 1u) / kGatherChunk;
        }
        static_assert(gather_entries_max<SIGN>() <= 128u, "the range table is scanned by the first two wavefronts");
        const uint32_t incl = reduce_block_scan<2>(my_chunks, wave_tot, total_chunks);
        if (total_chunks == 0) return;  // no token's block comes near this region: it is not touched at all
        if (threadIdx.x < s.NE) {
            tab_pa[threadIdx.x] = my_pa;
            tab_cum[threadIdx.x] = incl - my_chunks;
            for (uint32_t g = incl - my_chunks; g < incl && g < (uint32_t)kReduceBlock; ++g) chunk_entry[g] = (uint8_t)threadIdx.x;
        }
        if (threadIdx.x == 0) tab_cum[s.NE] = total_chunks;
    } else {
        for (uint32_t i = threadIdx.x; i < region_len; i += kReduceBlock) acc[i] = 0.0f;
    }

    typedef Vec<4>::A V4;
    const uint32_t nvec = vec_ok ? region_len / 4u : 0u;

    const uint32_t LG = 1u << s.lg_shift;
    const uint32_t j0 = threadIdx.x & (LG - 1u);
    const uint32_t grp = threadIdx.x >> s.lg_shift;
    const uint32_t grp_shift = 9u - s.lg_shift;               // log2(groups) for 512 threads
    const uint32_t groups = 1u << grp_shift;
    const uint32_t slice_shift = s.r_shift - grp_shift;       // the host guarantees 2^slice_shift >= Z
    const uint32_t slice_end = (grp + 1u) << slice_shift;

    // Records path: which records go into which round must not depend on the order in which the
    // records were written (that order comes from integer atomics and changes from run to run): a
    // region with more than one round's worth of records is split into classes by a hash of the
    // record, with as many classes as it takes for every class to fit one round.  The host refuses
    // reproducible calls whose regions could need more than 2^kMaxClassShift classes; should one turn
    // up all the same (ids chosen against the hash), its slots receive NaN instead of a sum whose bits
    // could change from run to run.
    const uint32_t count = re - rb;
    uint32_t cls_shift = 0;
    bool by_class = false;
    if (!GATHER && CANON && count > (uint32_t)kRecBatch) {
        uint32_t *hist = reinterpret_cast<uint32_t *>(srt);
        cls_shift = 1;
        while (((count + (1u << cls_shift) - 1u) >> cls_shift) > (uint32_t)kRecBatch / 2u) ++cls_shift;
        for (; cls_shift <= kMaxClassShift; ++cls_shift) {
            const uint32_t ncls = 1u << cls_shift;
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < ncls; i += kReduceBlock) hist[i] = 0;
            if (threadIdx.x == 0) *sel = 0;
            __syncthreads();
            for (uint32_t k = threadIdx.x; k < count; k += kReduceBlock)
                atomicAdd(&hist[record_class(s.rec[rb + k], cls_shift)], 1u);
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < ncls; i += kReduceBlock)
                if (hist[i] > (uint32_t)kRecBatch) *sel = 1;      // a class that does not fit one round
            __syncthreads();
            if (*sel == 0) {
                by_class = true;
                break;
            }
        }
    }
    const bool poison = !GATHER && CANON && count > (uint32_t)kRecBatch && !by_class;
    const uint32_t rounds = GATHER ? 0u : (poison ? 0u : (by_class ? (1u << cls_shift) : (count + kRecBatch - 1u) / kRecBatch));
    if (poison) {
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < region_len; i += kReduceBlock) acc[i] = __uint_as_float(0x7FC00000u);
    }

    uint32_t chunk_base = 0, window = kReduceBlock;           // gather: chunks taken by the rounds before; chunks this round tries
    for (uint32_t round = 0; GATHER ? chunk_base < total_chunks : round < rounds; ++round) {
        if (threadIdx.x < groups) cnt[threadIdx.x] = 0;
        if (threadIdx.x == 0) *sel = 0;
        __syncthreads();   // also orders the previous round's last pass before this round's writes
        uint32_t bb = rb + round * kRecBatch;
        uint32_t nb = re - bb < (uint32_t)kRecBatch ? re - bb : (uint32_t)kRecBatch;
        if constexpr (GATHER) {
            // R5-b: thread t looks at the t-th of the next `window` chunks of four sorted positions: their
            // keys and source rows in one vector load each (the arrays are padded to whole chunks).  A run
            // starts where the source row says so; it belongs to this range when its key does (a bucket
            // of the directory is wider than the range's ends).  Every run found is staged at once, its
            // slot taken from a counter; should the window hold more runs than the batch has room for,
            // the round is done again with half the window (a window of a quarter of the batch always
            // fits).  Which runs a round takes is thus a function of the sorted list alone; the order of
            // the slots is not, and does not matter.
            const uint32_t g = chunk_base + threadIdx.x;
            if (threadIdx.x < window && g < total_chunks) {
                uint32_t lo_e = 0;                             // the range of chunk g: tab_cum[lo_e] <= g < tab_cum[lo_e + 1]
                if (g < (uint32_t)kReduceBlock) {
                    lo_e = chunk_entry[g];
                } else {
                    uint32_t hi_e = s.NE;
                    while (hi_e - lo_e > 1u) {
                        const uint32_t mid = (lo_e + hi_e) >> 1;
                        if (tab_cum[mid] <= g) lo_e = mid; else hi_e = mid;
                    }
                }
                const uint32_t q = tab_pa[lo_e] + kGatherChunk * (g - tab_cum[lo_e]);
                if (q < s.n) {
                    const uint4 k4 = *reinterpret_cast<const uint4 *>(s.keys + q);
                    const uint4 s4 = *reinterpret_cast<const uint4 *>(s.src_row + q);
                    const KeyRange kr = key_range(p, s, lo_e, r0, region_len);
                    const uint32_t th4[4] = {k4.x, k4.y, k4.z, k4.w}, sr4[4] = {s4.x, s4.y, s4.z, s4.w};
                    const uint32_t live = s.n - q < 4u ? s.n - q : 4u;          // positions past the end hold nothing
                    uint32_t hits = 0;
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if ((uint32_t)k < live && sr4[k] != kNoRun && th4[k] >= kr.ta && th4[k] < kr.tb) hits |= 1u << k;
                    if (hits && s.run_c != nullptr) {          // tables of different dimensions: has the run a chunk kr.c at all?
                        const uint4 c4 = *reinterpret_cast<const uint4 *>(s.run_c + q);
                        const uint32_t nc4[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (((hits >> k) & 1u) && nc4[k] <= kr.c) hits &= ~(1u << k);
                    }
                    if (hits) {
                        uint32_t tg4[4] = {0, 0, 0, 0};
                        if constexpr (SIGN) {
                            const uint4 g4 = *reinterpret_cast<const uint4 *>(s.run_tg + q);
                            tg4[0] = g4.x; tg4[1] = g4.y; tg4[2] = g4.z; tg4[3] = g4.w;
                        }
                        uint32_t slot = atomicAdd(sel, (uint32_t)__popc(hits));
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            if (!((hits >> k) & 1u)) continue;
                            if (slot < (uint32_t)kRecBatch) {
                                const uint32_t o = offset_of(p, th4[k], kr.cc);
                                const bool inside = o >= r0 && o - r0 < region_len;
                                srt[slot] = make_uint2(o, (sr4[k] + kr.c) | (inside ? 0u : kPartBit));
                                if constexpr (SIGN) srt_tg[slot] = add_p(tg4[k], mod_p((uint64_t)p.Cg * (kr.c * p.Z)));
                            }
                            ++slot;
                        }
                    }
                }
            }
            __syncthreads();
            nb = *sel;
            if (nb > (uint32_t)kRecBatch) {     // too many runs in this window (uniform over the workgroup)
                __syncthreads();                // everyone has read the counter before the next attempt clears it
                window >>= 1;
                --round;
                continue;
            }
            chunk_base += window;
            window = kReduceBlock;
        }
        if (!GATHER && CANON && by_class) {
            // stage this round's class in the batch area, in any order
            for (uint32_t k = threadIdx.x; k < count; k += kReduceBlock) {
                const uint2 x = s.rec[rb + k];
                if (record_class(x, cls_shift) != round) continue;
                const uint32_t at = atomicAdd(sel, 1u);
                if (at < (uint32_t)kRecBatch) {
                    srt[at] = x;
                    if constexpr (SIGN) srt_tg[at] = s.rec_tg[rb + k];
                }
            }
            __syncthreads();
            nb = *sel < (uint32_t)kRecBatch ? *sel : (uint32_t)kRecBatch;
        }

        // 1. each thread takes its records, finds their slice and their rank inside it
        uint2 rc[kPer];
        uint32_t tgv[kPer], sl[kPer], rk[kPer];
        if (GATHER || (CANON && by_class)) {   // two branches: one reads LDS, the other global memory
#pragma unroll
            for (int t = 0; t < kPer; ++t) {
                const uint32_t k = threadIdx.x + (uint32_t)t * kReduceBlock;
                rc[t] = make_uint2(0u, kDeadRecord);
                tgv[t] = 0;
                if (k < nb) {
                    rc[t] = srt[k];
                    if constexpr (SIGN) tgv[t] = srt_tg[k];
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < kPer; ++t) {
                const uint32_t k = threadIdx.x + (uint32_t)t * kReduceBlock;
                rc[t] = make_uint2(0u, kDeadRecord);
                tgv[t] = 0;
                if (k < nb) {
                    rc[t] = s.rec[bb + k];
                    if constexpr (SIGN) tgv[t] = s.rec_tg[bb + k];
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kPer; ++t) {
            sl[t] = 0;
            rk[t] = 0;
            if (rc[t].y != kDeadRecord) {
                const uint32_t o = rc[t].x, src = rc[t].y & ~kPartBit;
                const bool part1 = (rc[t].y & kPartBit) != 0;
                // anything that does not belong here cannot occur with consistent inputs and is dropped
                const RecordSpan sp = span_of(o, part1, r0, region_len, p.m, p.Z);
                if (o < p.m && src < s.src_blocks && sp.ok) {
                    // From here on the record carries, instead of its offset, the region slot of its
                    // element 0 (negative when the block enters the region at slot 0 with a later
                    // element): element j then lands in slot x + j whenever that is a slot of the region.
                    rc[t].x = sp.abase;
                    sl[t] = part1 ? 0u : sp.abase >> slice_shift;
                    rk[t] = atomicAdd(&cnt[sl[t]], 1u);
                } else {
                    rc[t].y = kDeadRecord;
                }
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t a = 0;
            for (uint32_t g = 0; g < groups; ++g) {
                pre[g] = a;
                a += cnt[g];
            }
            pre[groups] = a;
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < kPer; ++t) {
            if (rc[t].y != kDeadRecord) {
                const uint32_t at = pre[sl[t]] + rk[t];
                srt[at] = rc[t];
                if constexpr (SIGN) srt_tg[at] = tgv[t];
            }
        }
        __syncthreads();
        if constexpr (CANON) {
            // The rank above came from an atomic and is arbitrary.  The order in which a slice's records
            // are added decides the rounding, so it is made canonical: by source word, then offset, then
            // sign term.  Records that agree in all three are interchangeable; their arbitrary places only
            // keep them apart.  (Tokens of one bag share their source blocks, so the source word alone
            // does not identify a record.)
            auto goes_before = [&](const uint2 &x, uint32_t tk, uint32_t k, const uint2 &mine, uint32_t mine_tg,
                                   uint32_t mine_at) -> bool {
                if (x.y != mine.y) return x.y < mine.y;
                if (x.x != mine.x) return x.x < mine.x;
                return tk < mine_tg || (tk == mine_tg && k < mine_at);
            };
#pragma unroll
            for (int t = 0; t < kPer; ++t) {
                if (rc[t].y != kDeadRecord) {
                    const uint32_t a = pre[sl[t]], b = pre[sl[t] + 1u], me = a + rk[t];
                    uint32_t c = 0;
                    for (uint32_t k0 = a; k0 < b; k0 += kCanonAhead) {     // kCanonAhead independent LDS reads per step
                        uint2 x[kCanonAhead];
                        uint32_t tk[kCanonAhead];
#pragma unroll
                        for (int u = 0; u < kCanonAhead; ++u) {
                            const uint32_t k = k0 + u < b ? k0 + u : me;   // past the end: compare with itself, never "before"
                            x[u] = srt[k];
                            tk[u] = SIGN ? srt_tg[k] : 0u;
                        }
#pragma unroll
                        for (int u = 0; u < kCanonAhead; ++u) {
                            const uint32_t k = k0 + u < b ? k0 + u : me;
                            c += goes_before(x[u], tk[u], k, rc[t], tgv[t], me);
                        }
                    }
                    rk[t] = c;
                }
            }
            __syncthreads();
#pragma unroll
            for (int t = 0; t < kPer; ++t) {
                if (rc[t].y != kDeadRecord) {
                    const uint32_t at = pre[sl[t]] + rk[t];
                    srt[at] = rc[t];
                    if constexpr (SIGN) srt_tg[at] = tgv[t];
                }
            }
            __syncthreads();
        }

        // 2. every group applies the records that start in its slice, kRecAhead loads in flight.
        //    Elements at or past the slice end belong to the next group's slice: they are summed in the
        //    group's own spill-over row (first element past the end first) and added in pass 3, or,
        //    when there is no room for such rows, read again in pass 3.
        //    The read-modify-writes below are plain LDS accesses, and a group's next record may hit a
        //    slot that another lane of the group wrote for the record before.  That is ordered because a
        //    lane group never spans two wavefronts (LG <= 64, groups aligned to LG) and a wavefront's LDS
        //    accesses are performed in program order for all of its lanes; the wave_barrier between
        //    records keeps the compiler from moving one record's accesses across another's.
        const uint32_t lb = pre[grp], le = pre[grp + 1];
        if constexpr (SPILL) {
            for (uint32_t j = j0; j < p.Z; j += LG) acc[spill_at + j] = 0.0f;
        }
        for (uint32_t k0 = lb; k0 < le; k0 += kRecAhead) {
            // per record: element j lands at region slot abase + j if that is one (unsigned compare)
            uint32_t abase[kRecAhead], src[kRecAhead], tg[kRecAhead];
#pragma unroll
            for (int u = 0; u < kRecAhead; ++u) {
                const bool live = k0 + u < le;
                const uint2 x = srt[live ? k0 + u : lb];
                src[u] = x.y & ~kPartBit;
                tg[u] = SIGN ? srt_tg[live ? k0 + u : lb] : 0u;
                abase[u] = live ? x.x : region_len;            // (a record past the end lands nowhere)
            }
            for (uint32_t j = j0; j < p.Z; j += LG) {
                float v[kRecAhead];
#pragma unroll
                for (int u = 0; u < kRecAhead; ++u) {
                    const float *base = src[u] < src_own ? grad_out + (uint64_t)src[u] * p.Z
                                                         : s.P + (uint64_t)(src[u] - src_own) * p.Z;
                    v[u] = s.keep_rows ? base[j] : __builtin_nontemporal_load(base + j);
                }
#pragma unroll
                for (int u = 0; u < kRecAhead; ++u) {
                    const uint32_t a = abase[u] + j;
                    if (a < region_len) {
                        const float val = signed_block_value<SIGN>(p, v[u], tg[u], j);
                        if constexpr (SPILL) {
                            // one read-modify-write, in the slice or in the group's spill-over row
                            // (which follows acc at spill_at; a - slice_end < Z - 1)
                            acc[a < slice_end ? a : spill_at + (a - slice_end)] += val;
                        } else {
                            if (a < slice_end) acc[a] += val;
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
        __syncthreads();

        // 3. elements past the slice end: the next slice's first Z-1 floats, which nobody else writes now
        if constexpr (SPILL) {
            for (uint32_t j = j0; j + 1u < p.Z; j += LG) {
                const uint32_t a = slice_end + j;
                if (a < region_len) acc[a] += acc[spill_at + j];
            }
        } else {
            for (uint32_t k = lb; k < le; ++k) {
                const uint2 x = srt[k];
                if (x.y & kPartBit) continue;                       // such a record starts slice 0 at its first slot: never past a slice end
                const uint32_t abase = x.x, src = x.y;
                if (abase + p.Z <= slice_end) continue;
                const uint32_t tgk = SIGN ? srt_tg[k] : 0u;
                const float *base = src < src_own ? grad_out + (uint64_t)src * p.Z : s.P + (uint64_t)(src - src_own) * p.Z;
                for (uint32_t j = j0; j < p.Z; j += LG) {
                    const uint32_t a = abase + j;
                    if (a >= slice_end && a < region_len)
                        acc[a] += signed_block_value<SIGN>(p, base[j], tgk, j);
                }
            }
        }
    }
    __syncthreads();

    // The region is complete and this workgroup is the only one that holds any of its slots.
    // Write-back per 64-byte granule (4 vectors, 4 lanes): partially written granules cost more than
    // they save, untouched ones are neither read nor written.
    const uint32_t lane = threadIdx.x & 63u;
    if (!s.sparse_regions) {
        // most granules are touched: sweep the region, one vector per thread and pass
        for (uint32_t it0 = 0; it0 < nvec; it0 += kWb * kReduceBlock) {   // same trip count for the whole workgroup
            V4 g[kWb], w[kWb], st[kWb];
            bool touch[kWb];
#pragma unroll
            for (int u = 0; u < kWb; ++u) {
                const uint32_t it = it0 + (uint32_t)u * kReduceBlock + threadIdx.x;
#pragma unroll
                for (int k = 0; k < 4; ++k) g[u][k] = 0.0f;
                if (it < nvec) g[u] = *reinterpret_cast<const V4 *>(&acc[4u * it]);
                const bool any = g[u][0] != 0.0f || g[u][1] != 0.0f || g[u][2] != 0.0f || g[u][3] != 0.0f;
                // decide per 64-byte granule (4 lanes): partially written granules cost more than they save
                const uint64_t gran_any = (__ballot(any) >> (lane & ~3u)) & 0xFull;
                touch[u] = it < nvec && gran_any != 0;
            }
#pragma unroll
            for (int u = 0; u < kWb; ++u) {
                if (touch[u]) {
                    const uint32_t it = it0 + (uint32_t)u * kReduceBlock + threadIdx.x;
                    if (s.keep_array) w[u] = *reinterpret_cast<const V4 *>(dst + r0 + 4u * it);
                    else w[u] = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(dst + r0 + 4u * it));
                    if constexpr (RULE == 1) st[u] = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(state + r0 + 4u * it));
                }
            }
#pragma unroll
            for (int u = 0; u < kWb; ++u) {
                if (!touch[u]) continue;
                const uint32_t it = it0 + (uint32_t)u * kReduceBlock + threadIdx.x;
                if constexpr (RULE == 0) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) w[u][k] = __fadd_rn(w[u][k], __fmul_rn(g[u][k], lr));
                    if (s.keep_array) *reinterpret_cast<V4 *>(dst + r0 + 4u * it) = w[u];
                    else __builtin_nontemporal_store(w[u], reinterpret_cast<V4 *>(dst + r0 + 4u * it));
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if (g[u][k] != 0.0f) {
                            float wk = w[u][k], sk = st[u][k];
                            adagrad_one(wk, sk, g[u][k], lr, eps);
                            w[u][k] = wk;
                            st[u][k] = sk;
                        }
                    }
                    if (s.keep_array) *reinterpret_cast<V4 *>(dst + r0 + 4u * it) = w[u];
                    else __builtin_nontemporal_store(w[u], reinterpret_cast<V4 *>(dst + r0 + 4u * it));
                    __builtin_nontemporal_store(st[u], reinterpret_cast<V4 *>(state + r0 + 4u * it));
                }
            }
        }
    } else {
        // few granules are touched: list them first (in the batch area, which is free now), then take
        // 128 of them per pass - one pass of loads for the whole region instead of one per 2 KB of it
        uint16_t *gran = reinterpret_cast<uint16_t *>(srt);
        static_assert(kRecBatch * (SIGN ? 12 : 8) >= (1 << (15 - 3)), "the batch area holds one 16-bit entry per granule of the largest region (2^15 floats)");
        if (threadIdx.x == 0) *sel = 0;
        __syncthreads();
        for (uint32_t it0 = 0; it0 < nvec; it0 += kReduceBlock) {            // same trip count for the whole workgroup
            const uint32_t it = it0 + threadIdx.x;
            bool any = false;
            if (it < nvec) {
                const V4 g = *reinterpret_cast<const V4 *>(&acc[4u * it]);
                any = g[0] != 0.0f || g[1] != 0.0f || g[2] != 0.0f || g[3] != 0.0f;
            }
            const uint64_t b = __ballot(any);
            const uint64_t touched = (b | (b >> 1) | (b >> 2) | (b >> 3)) & 0x1111111111111111ull;   // bit 4k: granule k of this wavefront
            uint32_t at = 0;
            if (lane == 0 && touched) at = atomicAdd(sel, (uint32_t)__popcll(touched));
            at = __shfl(at, 0);
            if ((touched >> lane) & 1ull) gran[at + (uint32_t)__popcll(touched & ((1ull << lane) - 1ull))] = (uint16_t)(it >> 2);
        }
        __syncthreads();
        const uint32_t n_gran = *sel;
        for (uint32_t k0 = 0; k0 < n_gran; k0 += kReduceBlock / 4u) {
            const uint32_t k = k0 + (threadIdx.x >> 2);
            if (k >= n_gran) continue;
            const uint32_t it = (uint32_t)gran[k] * 4u + (threadIdx.x & 3u);
            if (it >= nvec) continue;
            const V4 g = *reinterpret_cast<const V4 *>(&acc[4u * it]);
            V4 w, st;
            if (s.keep_array) w = *reinterpret_cast<const V4 *>(dst + r0 + 4u * it);
            else w = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(dst + r0 + 4u * it));
            if constexpr (RULE == 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = __fadd_rn(w[e], __fmul_rn(g[e], lr));
                if (s.keep_array) *reinterpret_cast<V4 *>(dst + r0 + 4u * it) = w;
                else __builtin_nontemporal_store(w, reinterpret_cast<V4 *>(dst + r0 + 4u * it));
            } else {
                st = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(state + r0 + 4u * it));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (g[e] != 0.0f) {
                        float wk = w[e], sk = st[e];
                        adagrad_one(wk, sk, g[e], lr, eps);
                        w[e] = wk;
                        st[e] = sk;
                    }
                }
                if (s.keep_array) *reinterpret_cast<V4 *>(dst + r0 + 4u * it) = w;
                else __builtin_nontemporal_store(w, reinterpret_cast<V4 *>(dst + r0 + 4u * it));
                __builtin_nontemporal_store(st, reinterpret_cast<V4 *>(state + r0 + 4u * it));
            }
        }
    }
    for (uint32_t i = 4u * nvec + threadIdx.x; i < region_len; i += kReduceBlock) {   // tail, or unaligned buffers
        const float g = acc[i];
        if (g == 0.0f) continue;
        if constexpr (RULE == 0) {
            dst[r0 + i] = __fadd_rn(dst[r0 + i], __fmul_rn(g, lr));
        } else {
            float wk = dst[r0 + i], sk = state[r0 + i];
            adagrad_one(wk, sk, g, lr, eps);
            dst[r0 + i] = wk;
            state[r0 + i] = sk;
        }
    }
}

}  // namespace robe
