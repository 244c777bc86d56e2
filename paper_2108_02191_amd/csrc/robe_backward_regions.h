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
constexpr int kStretch = 8;            // stretches of G sorted positions a lane group walks in R1
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
constexpr int kCanonAhead = 4;         // records of a slice compared per step when R5 puts them in canonical order
constexpr int kWb = 1;                 // vectors per thread and pass in the write-back of R5 (more did not pay: registers)
constexpr uint32_t kMaxRegions = 32768;
constexpr uint32_t kMaxClassShift = 10;  // R5 splits an overfull region into at most 2^10 classes (the table lives in the batch area)
constexpr uint32_t kPartBit = 0x80000000u;   // record flag: the elements past the end of the block's own region
constexpr uint32_t kDeadRecord = 0xFFFFFFFFu;

struct RegionPlan {
    uint32_t r_shift;        // log2 of the region size in floats
    uint32_t NR;             // regions = ceil(m / 2^r_shift)
    uint32_t n;              // sorted token positions
    uint32_t rows;           // rows of grad_out
    uint32_t src_blocks;     // (rows + P rows) * C: exclusive bound of a record's source block
    uint32_t bin_blocks;     // grid of R2 / R4
    uint32_t pos_per_block;  // sorted positions per workgroup in R2 / R4
    uint32_t lg_shift;       // log2 of the lanes per record in R5
    uint32_t fullest_first;  // 1: R5 takes the regions by descending size class instead of by address
    uint32_t keep_rows;      // 1: gradient rows are read more than once (bags): R5 loads them with the default cache policy
    uint32_t keep_array;     // 1: R5 with the Adagrad rule leaves the array in the caches for the next forward pass (small arrays)
    const uint32_t *keys;    // sorted keys
    uint8_t *head;           // [n]  1: a run starts here
    uint32_t *src_row;       // [n]  at run starts: row of grad_out, or rows + row of P
    uint32_t *run_tg;        // [n]  at run starts: token part of the sign hash (sign on only)
    float *P;                // [(n + 1) / 2][d] summed rows of the runs longer than one
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
// A group walks kStretch * G consecutive sorted positions, G at a time; a run is cut only where the
// group's walk begins and ends, so a token that fills whole stretches leaves one record per
// kStretch * G copies.
// ---------------------------------------------------------------------------------------------
struct SortedToken {
    uint32_t th, row, e, xlo, xhi, tg;
    bool ok;
};

template <bool SIGN>
__device__ __forceinline__ bool same_token(const SortedToken &a, const SortedToken &b)
{
    bool same = a.th == b.th;
    if constexpr (SIGN) same = same && a.e == b.e && a.xlo == b.xlo && a.xhi == b.xhi;
    return same;
}

template <bool SIGN>
__device__ __forceinline__ SortedToken shfl_token(const SortedToken &t, int from)
{
    SortedToken r;
    r.th = __shfl(t.th, from);
    r.ok = __shfl((int)t.ok, from) != 0;
    r.row = 0;
    r.tg = 0;
    r.e = SIGN ? __shfl(t.e, from) : 0u;
    r.xlo = SIGN ? __shfl(t.xlo, from) : 0u;
    r.xhi = SIGN ? __shfl(t.xhi, from) : 0u;
    return r;
}

template <int V, bool SIGN, bool BAGS>
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
    for (uint64_t i = thread_id; i < s.NR; i += (uint64_t)gridDim.x * kBlock) s.counts[i] = 0;
    if ((thread_id - lane) * kStretch >= n) return;     // the whole wavefront is past the end
    const uint64_t i_first = (thread_id - grp) * kStretch;   // first sorted position of this group's walk

    // the token at a sorted position (lane l of the group looks at position i0 + l)
    auto fetch = [&](uint64_t pos) -> SortedToken {
        SortedToken t;
        t.th = t.row = t.e = t.xlo = t.xhi = t.tg = 0;
        t.ok = false;
        if (pos < n) {
            const uint32_t v = vals[pos];                  // sign off: the row itself (see robe_backward_dedup.h)
            const uint32_t row = !SIGN ? v : (v < n ? (BAGS ? tok_bag[v] : v) : s.rows);
            if (row < s.rows) {
                t.ok = true;
                t.row = row;
                t.th = s.keys[pos];
                if constexpr (SIGN) {
                    const int64_t x = indices[v];
                    t.e = row % q.F;
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

    SortedToken cur = fetch(i_first + grp);
    SortedToken carry;          // the last token of the stretch before; none before the first
    carry.th = carry.row = carry.e = carry.xlo = carry.xhi = carry.tg = 0;
    carry.ok = false;
    for (uint32_t st = 0; st < (uint32_t)kStretch; ++st) {
        const uint64_t i0 = i_first + (uint64_t)st * q.G;
        if (__all(i0 >= n)) break;                          // every group of the wavefront is past the end
        SortedToken nxt;
        if (st + 1u < (uint32_t)kStretch) {
            nxt = fetch(i0 + q.G + grp);
        } else {
            nxt = carry;
            nxt.ok = false;
        }
        // does a run start here (a different token than the one before, or the walk begins), and
        // does it end here (a different token after, or the walk ends)?
        SortedToken before = shfl_token<SIGN>(cur, (int)(base_lane + (grp ? grp - 1u : 0u)));
        if (grp == 0) before = carry;
        const bool my_head = cur.ok && (!before.ok || !same_token<SIGN>(before, cur));
        SortedToken after = shfl_token<SIGN>(cur, (int)(base_lane + (grp + 1u < q.G ? grp + 1u : grp)));
        const SortedToken first_of_next = shfl_token<SIGN>(nxt, (int)base_lane);
        if (grp + 1u >= q.G) after = first_of_next;
        const bool my_end = cur.ok && (!after.ok || !same_token<SIGN>(after, cur));
        const bool my_single = my_head && my_end;

        if (i0 + grp < n) {
            s.head[i0 + grp] = my_head ? 1 : 0;
            if (my_single) s.src_row[i0 + grp] = cur.row;            // a run of one: read grad_out in place
            if constexpr (SIGN) {
                if (my_head) s.run_tg[i0 + grp] = cur.tg;
            }
        }

        // runs longer than one: sum their rows into P (a run may have begun in an earlier stretch)
        for (uint32_t k0 = 0; k0 < q.G; k0 += kRowsAhead) {     // same trip count for every lane of the wavefront
            uint32_t row[kRowsAhead];
            bool use[kRowsAhead], head[kRowsAhead], end[kRowsAhead];
#pragma unroll
            for (int u = 0; u < kRowsAhead; ++u) {
                const int from = (int)(base_lane + ((k0 + u) & (q.G - 1u)));
                const bool in = k0 + u < q.G;
                use[u] = in && __shfl((int)(cur.ok && !my_single), from) != 0;
                row[u] = __shfl(cur.row, from);
                head[u] = __shfl((int)my_head, from) != 0;
                end[u] = __shfl((int)my_end, from) != 0;
            }
            float v[kRowsAhead][V];
#pragma unroll
            for (int u = 0; u < kRowsAhead; ++u) {
                if (use[u]) load_row<V, false, BAGS>(grad_out + (uint64_t)row[u] * p.d, q, grp, v[u]);
            }
#pragma unroll
            for (int u = 0; u < kRowsAhead; ++u) {
                if (!use[u]) continue;
                if (head[u]) {
                    head_pos = (uint32_t)i0 + k0 + u;
#pragma unroll
                    for (int k = 0; k < V; ++k) acc[k] = 0.0f;
                }
#pragma unroll
                for (int k = 0; k < V; ++k) acc[k] += v[u][k];
                if (end[u]) {
                    // two runs longer than one start at least two positions apart: head_pos / 2 is unique
                    const uint32_t prow = head_pos >> 1;
                    store_row<V, false>(s.P + (uint64_t)prow * p.d, q, grp, acc);
                    if (grp == 0) s.src_row[head_pos] = s.rows + prow;
                }
            }
        }
        carry = shfl_token<SIGN>(cur, (int)(base_lane + q.G - 1u));
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
        uint32_t hd[kBinAhead], th[kBinAhead], sr[kBinAhead], tgv[kBinAhead];
#pragma unroll
        for (int u = 0; u < kBinAhead; ++u) {
            const uint64_t i = i0 + (uint64_t)u * kBinBlock;
            const uint64_t at = i < e ? i : i0;               // i0 < e: a position of this workgroup
            hd[u] = i < e ? s.head[at] : 0u;
            th[u] = s.keys[at];
            sr[u] = s.src_row[at];
            tgv[u] = SIGN ? s.run_tg[at] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kBinAhead; ++u) {
            if (!hd[u]) continue;
            const uint32_t src0 = sr[u] * p.C;
            uint32_t cc = 0;  // (Ch * c) mod P, built up by addition
            for (uint32_t c = 0; c < p.C; ++c) {
                const uint32_t o = offset_of(p, th[u], cc);
                const uint32_t r = o >> s.r_shift;
                f(o, src0 + c, r, 0u, tgv[u]);
                const uint64_t r_end = ((uint64_t)(r + 1u) << s.r_shift) < p.m ? ((uint64_t)(r + 1u) << s.r_shift) : p.m;
                if ((uint64_t)o + p.Z > r_end) f(o, src0 + c, r_end == p.m ? 0u : r + 1u, kPartBit, tgv[u]);
                cc = add_p(cc, p.Ch);
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
// R5.  RULE 0: grad_array += region.  RULE 1: Adagrad on array / state with the region as gradient.
// ---------------------------------------------------------------------------------------------
template <bool SIGN>
__device__ __forceinline__ float signed_block_value(const Params &p, float v, uint32_t tg, uint32_t src, uint32_t j)
{
    if constexpr (SIGN) {
        const uint32_t el = (src % p.C) * p.Z + j;
        return apply_sign(v, sign_mask(add_p(tg, mod_p((uint64_t)p.Cg * el))));
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

template <bool SIGN, int RULE, bool CANON, bool SPILL>
__global__ __launch_bounds__(kReduceBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void region_reduce_kernel(Params p, RegionPlan s,
                                                                     const float *__restrict__ grad_out,
                                                                     float *__restrict__ dst,      // RULE 0: grad_array; RULE 1: array
                                                                     float *__restrict__ state,    // RULE 1 only
                                                                     float lr, float eps, int vec_ok)
{
    constexpr int kRecBatch = rec_batch<SIGN>();
    extern __shared__ float acc[];  // 2^r_shift floats, then the batch staging area
    const uint32_t r = s.counts[blockIdx.x];     // after R3: the regions, fullest first
    if (r >= s.NR) return;
    const uint32_t rb = s.starts[r], re = s.starts[r + 1];
    if (rb >= re) return;           // nothing lands in this region: it is not touched at all

    const uint32_t R = 1u << s.r_shift;
    const uint32_t r0 = r << s.r_shift;
    const uint32_t region_len = (p.m - r0) < R ? (p.m - r0) : R;
    const uint32_t src_own = s.rows * p.C;   // source blocks below this live in grad_out, the rest in P

    uint2 *srt = reinterpret_cast<uint2 *>(acc + R);
    uint32_t *srt_tg = reinterpret_cast<uint32_t *>(srt + kRecBatch);
    uint32_t *cnt = srt_tg + (SIGN ? kRecBatch : 0);   // 64 slice counters
    uint32_t *pre = cnt + 64;                          // 65 slice starts
    uint32_t *sel = pre + 65;                          // records staged for this round
    // this group's spill-over row, as an index into acc
    const uint32_t spill_at = (uint32_t)(reinterpret_cast<float *>(sel + 1) - acc) + (threadIdx.x >> s.lg_shift) * p.Z;

    for (uint32_t i = threadIdx.x; i < region_len; i += kReduceBlock) acc[i] = 0.0f;

    typedef Vec<4>::A V4;
    const uint32_t nvec = vec_ok ? region_len / 4u : 0u;

    const uint32_t LG = 1u << s.lg_shift;
    const uint32_t j0 = threadIdx.x & (LG - 1u);
    const uint32_t grp = threadIdx.x >> s.lg_shift;
    const uint32_t grp_shift = 9u - s.lg_shift;               // log2(groups) for 512 threads
    const uint32_t groups = 1u << grp_shift;
    const uint32_t slice_shift = s.r_shift - grp_shift;       // the host guarantees 2^slice_shift >= Z
    const uint32_t slice_end = (grp + 1u) << slice_shift;

    // Elements of a record that this region (and this record's part) holds: element j sits at array
    // position (o + j) mod m; part 0 keeps the elements before the end of o's own region, part 1 the
    // rest, which continue at the start of the next region (or of the array).
    auto own_end = [&](uint32_t o) -> uint32_t {              // end of the region that holds offset o
        const uint64_t e = ((uint64_t)((o >> s.r_shift) + 1u)) << s.r_shift;
        return e < p.m ? (uint32_t)e : p.m;
    };

    // Which records go into which round must not depend on the order in which the records were
    // written (that order comes from integer atomics and changes from run to run): a region with more
    // than one round's worth of records is split into classes by a hash of the record, with as many
    // classes as it takes for every class to fit one round.  The host refuses reproducible calls whose
    // regions could need more than 2^kMaxClassShift classes; should one turn up all the same (ids
    // chosen against the hash), its slots receive NaN instead of a sum whose bits could change from
    // run to run.
    const uint32_t count = re - rb;
    uint32_t cls_shift = 0;
    bool by_class = false;
    if (CANON && count > (uint32_t)kRecBatch) {
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
    const bool poison = CANON && count > (uint32_t)kRecBatch && !by_class;
    const uint32_t rounds = poison ? 0u : (by_class ? (1u << cls_shift) : (count + kRecBatch - 1u) / kRecBatch);
    if (poison) {
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < region_len; i += kReduceBlock) acc[i] = __uint_as_float(0x7FC00000u);
    }

    for (uint32_t round = 0; round < rounds; ++round) {
        if (threadIdx.x < groups) cnt[threadIdx.x] = 0;
        if (threadIdx.x == 0) *sel = 0;
        __syncthreads();   // also orders the previous round's last pass before this round's writes
        uint32_t bb = rb + round * kRecBatch;
        uint32_t nb = re - bb < (uint32_t)kRecBatch ? re - bb : (uint32_t)kRecBatch;
        if (CANON && by_class) {
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

        // 1. each thread takes two records, finds their slice and their rank inside it
        uint2 rc[2];
        uint32_t tgv[2], sl[2], rk[2];
        if (CANON && by_class) {   // two branches: one reads LDS, the other global memory
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t k = threadIdx.x + (uint32_t)t * kReduceBlock;
                rc[t] = make_uint2(kDeadRecord, 0u);
                tgv[t] = 0;
                if (k < nb) {
                    rc[t] = srt[k];
                    if constexpr (SIGN) tgv[t] = srt_tg[k];
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t k = threadIdx.x + (uint32_t)t * kReduceBlock;
                rc[t] = make_uint2(kDeadRecord, 0u);
                tgv[t] = 0;
                if (k < nb) {
                    rc[t] = s.rec[bb + k];
                    if constexpr (SIGN) tgv[t] = s.rec_tg[bb + k];
                }
            }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            sl[t] = 0;
            rk[t] = 0;
            if (rc[t].x != kDeadRecord) {
                const uint32_t o = rc[t].x, src = rc[t].y & ~kPartBit;
                const bool part1 = (rc[t].y & kPartBit) != 0;
                // where the record's first element of this part lands; anything else cannot occur
                // with consistent inputs and is dropped
                const uint32_t first = part1 ? own_end(o) % p.m : o;
                if (o < p.m && src < s.src_blocks && (first >> s.r_shift) == r) {
                    sl[t] = (first - r0) >> slice_shift;
                    rk[t] = atomicAdd(&cnt[sl[t]], 1u);
                } else {
                    rc[t].x = kDeadRecord;
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
        for (int t = 0; t < 2; ++t) {
            if (rc[t].x != kDeadRecord) {
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
            for (int t = 0; t < 2; ++t) {
                if (rc[t].x != kDeadRecord) {
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
            for (int t = 0; t < 2; ++t) {
                if (rc[t].x != kDeadRecord) {
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
            // per record: element j lands at region slot abase + j, for j in [jlo, jhi) (packed; Z <= 2^15)
            uint32_t abase[kRecAhead], win[kRecAhead], src[kRecAhead], tg[kRecAhead];
#pragma unroll
            for (int u = 0; u < kRecAhead; ++u) {
                const bool live = k0 + u < le;
                const uint2 x = srt[live ? k0 + u : lb];
                src[u] = x.y & ~kPartBit;
                tg[u] = SIGN ? srt_tg[live ? k0 + u : lb] : 0u;
                const uint32_t keep = own_end(x.x) - x.x;                 // elements before the end of o's own region
                const uint32_t cut = keep < p.Z ? keep : p.Z;
                if (x.y & kPartBit) {
                    abase[u] = 0u - cut;                                  // element `cut` is the first of this region
                    win[u] = cut | (p.Z << 16);
                } else {
                    abase[u] = x.x - r0;
                    win[u] = cut << 16;
                }
                if (!live) win[u] = 0;
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
                    if (j >= (win[u] & 0xFFFFu) && j < (win[u] >> 16) && a < region_len) {
                        const float val = signed_block_value<SIGN>(p, v[u], tg[u], src[u], j);
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
                if (x.y & kPartBit) continue;                       // a part-1 record starts its slice: never past its end
                const uint32_t o = x.x, src = x.y;
                if (o - r0 + p.Z <= slice_end) continue;
                const uint32_t oend = own_end(o);
                const uint32_t tgk = SIGN ? srt_tg[k] : 0u;
                const float *base = src < src_own ? grad_out + (uint64_t)src * p.Z : s.P + (uint64_t)(src - src_own) * p.Z;
                for (uint32_t j = j0; j < p.Z; j += LG) {
                    const uint32_t a = o + j - r0;
                    if (o + j < oend && a >= slice_end && a < region_len)
                        acc[a] += signed_block_value<SIGN>(p, base[j], tgk, src, j);
                }
            }
        }
    }
    __syncthreads();

    // The region is complete and this workgroup is the only one that holds any of its slots.
    // kWb vectors per thread and pass: all their loads are requested before the first is used.
    const uint32_t lane = threadIdx.x & 63u;
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
                if (RULE == 1 && s.keep_array) w[u] = *reinterpret_cast<const V4 *>(dst + r0 + 4u * it);
                else w[u] = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(dst + r0 + 4u * it));
                if constexpr (RULE == 1) st[u] = __builtin_nontemporal_load(reinterpret_cast<const V4 *>(state + r0 + 4u * it));
            }
        }
#pragma unroll
        for (int u = 0; u < kWb; ++u) {
            if (!touch[u]) continue;
            const uint32_t it = it0 + (uint32_t)u * kReduceBlock + threadIdx.x;
            if constexpr (RULE == 0) {
                w[u] += g[u];
                __builtin_nontemporal_store(w[u], reinterpret_cast<V4 *>(dst + r0 + 4u * it));
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
    for (uint32_t i = 4u * nvec + threadIdx.x; i < region_len; i += kReduceBlock) {   // tail, or unaligned buffers
        const float g = acc[i];
        if (g == 0.0f) continue;
        if constexpr (RULE == 0) {
            dst[r0 + i] += g;
        } else {
            float wk = dst[r0 + i], sk = state[r0 + i];
            adagrad_one(wk, sk, g, lr, eps);
            dst[r0 + i] = wk;
            state[r0 + i] = sk;
        }
    }
}

}  // namespace robe
