// Stable LSD radix sort of (key, value) pairs of 32-bit words on a range of key bits, for the token
// sort of the backward pass (S2 in robe_backward_dedup.h).
//
// Eight bits per pass, three kernels per pass, no kernel ever waits for another workgroup:
//
//   count    a workgroup takes a tile of kSortTile pairs, counts the digits of its keys in LDS and
//            writes the counts to tile_count[digit][tile].
//   offsets  one workgroup per digit: an exclusive prefix over that digit's row of tile counts -
//            how many pairs of the digit the tiles before hold - and the digit's total.
//   scatter  a workgroup takes its tile again, finds where every digit starts (an exclusive scan of
//            the 256 totals), ranks every pair among the tile's pairs of the same digit in input
//            order (so the sort is stable), puts the tile into LDS in digit order and writes it out
//            from there, a digit's pairs to consecutive slots.
//
// Inside a tile, wavefront w of the scatter kernel owns pairs [w * 512, (w + 1) * 512) and walks
// them 64 at a time, so the input order is (wavefront, round, lane): a pair's rank is what earlier rounds of its wavefront
// counted for the digit, plus the lanes below it in its own round with the same digit (found with one
// ballot per digit bit), plus what the wavefronts before it hold.
//
// It records nothing but kernels on the stream (no fill operations), and for the sizes met here
// (10^5 .. 10^7 pairs) it is shorter on launches than the device library's sort.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace robe {

constexpr int kSortBlock = 256;                       // count and offsets kernels: 4 wavefronts
constexpr int kSortRounds = 16;                       // count kernel: keys per thread
constexpr uint32_t kSortTile = kSortBlock * kSortRounds;   // 4096 pairs
constexpr uint32_t kDigits = 256;
static_assert(kSortBlock == (int)kDigits, "one thread per digit in the per-digit steps");

struct SortPass {
    uint32_t shift;      // first key bit of this pass's digit
    uint32_t mask;       // (1 << bits) - 1, bits <= 8
    uint32_t n;          // pairs
    uint32_t tiles;      // ceil(n / kSortTile)
    uint32_t *tile_count;   // [kDigits][tiles]: counts, then the digit's pairs in the tiles before
    uint32_t *totals;       // [kDigits]: pairs of each digit
};

// RUNS: equal keys sit side by side (every pass after the first: the pairs are sorted by the lower
// digits), and the copies of a frequent token would put dozens of LDS atomics of a wavefront on one
// word.  Then each run of equal digits among the 64 consecutive keys of a wavefront adds once, its
// length (31 -> 12 us on 8.5 M keys in runs of 37; 10 -> 12 us on keys without runs, hence not in
// the first pass).
template <bool RUNS>
__global__ __launch_bounds__(kSortBlock) void sort_count_kernel(SortPass s, const uint32_t *__restrict__ keys)
{
    __shared__ uint32_t h[kDigits];
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t tile = blockIdx.x;
    const uint64_t base = (uint64_t)tile * kSortTile;
    uint32_t k[kSortRounds];
#pragma unroll
    for (int i = 0; i < kSortRounds; ++i) {
        const uint64_t at = base + (uint32_t)i * kSortBlock + threadIdx.x;
        k[i] = at < s.n ? keys[at] : 0u;
    }
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int i = 0; i < kSortRounds; ++i) {
        const uint64_t at = base + (uint32_t)i * kSortBlock + threadIdx.x;
        const bool have = at < s.n;
        const uint32_t digit = have ? ((k[i] >> s.shift) & s.mask) : 0xFFFFFFFFu;   // no key: a run of its own, never added
        if constexpr (RUNS) {
            const uint32_t prev = __shfl_up(digit, 1);
            const bool head = lane == 0 || digit != prev;
            const uint64_t heads = __ballot(head);
            if (head && have) {
                const uint64_t above = heads & ~((2ull << lane) - 1ull);            // heads in the lanes after this one
                const uint32_t next = above ? (uint32_t)__builtin_ctzll(above) : 64u;
                atomicAdd(&h[digit], next - lane);
            }
        } else {
            if (have) atomicAdd(&h[digit], 1u);
        }
    }
    __syncthreads();
    s.tile_count[(uint64_t)threadIdx.x * s.tiles + tile] = h[threadIdx.x];
}

// Exclusive prefix of one value per thread over the workgroup's BLOCK threads.  `wave_total` is LDS
// for BLOCK / 64 words; the call ends with a barrier, so it may be reused right after.
template <int BLOCK>
__device__ __forceinline__ uint32_t exclusive_scan_block(uint32_t v, uint32_t *wave_total, uint32_t &total)
{
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (uint32_t off = 1; off < 64u; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (lane == 63u) wave_total[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    total = 0;
#pragma unroll
    for (uint32_t w = 0; w < (uint32_t)BLOCK / 64u; ++w) {
        const uint32_t x = wave_total[w];
        before += w < wave ? x : 0u;
        total += x;
    }
    __syncthreads();
    return before + incl - v;
}

// One workgroup per digit.
constexpr int kOffsetItems = 8;   // tile counts per thread and step

__global__ __launch_bounds__(kSortBlock) void sort_offsets_kernel(SortPass s)
{
    __shared__ uint32_t wave_total[4];
    const uint32_t digit = blockIdx.x, t = threadIdx.x;
    uint32_t carry = 0;           // the same in every thread
    uint32_t *row = s.tile_count + (uint64_t)digit * s.tiles;
    for (uint32_t t0 = 0; t0 < s.tiles; t0 += kSortBlock * kOffsetItems) {     // same trip count for the whole workgroup
        uint32_t c[kOffsetItems], sum = 0;
#pragma unroll
        for (int k = 0; k < kOffsetItems; ++k) {
            const uint32_t i = t0 + t * kOffsetItems + (uint32_t)k;
            c[k] = i < s.tiles ? row[i] : 0u;
            sum += c[k];
        }
        uint32_t total;
        uint32_t a = carry + exclusive_scan_block<kSortBlock>(sum, wave_total, total);
#pragma unroll
        for (int k = 0; k < kOffsetItems; ++k) {
            const uint32_t i = t0 + t * kOffsetItems + (uint32_t)k;
            if (i < s.tiles) row[i] = a;
            a += c[k];
        }
        carry += total;
    }
    if (t == 0) s.totals[digit] = carry;
}

// BLOCK threads take a tile of kSortTile pairs, kSortTile / BLOCK rounds of 64 per wavefront.
// Measured on 8.5 M pairs: 512 threads (74 registers, six wavefronts per SIMD) 2 us per pass faster
// than 256 (128 registers, four per SIMD); 1024 slower again.
constexpr int kScatterBlock = 512;

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void sort_scatter_kernel(SortPass s, const uint32_t *__restrict__ keys_in,
                                                             const uint32_t *__restrict__ vals_in,
                                                             uint32_t *__restrict__ keys_out,
                                                             uint32_t *__restrict__ vals_out)
{
    constexpr int ROUNDS = (int)kSortTile / BLOCK, WAVES = BLOCK / 64;
    static_assert(BLOCK >= (int)kDigits && BLOCK * ROUNDS == (int)kSortTile, "a thread per digit, whole rounds");
    __shared__ uint32_t wave_count[WAVES][kDigits];   // per wavefront: pairs of each digit so far; later: its base in the tile
    __shared__ uint32_t digit_slot[kDigits];          // first output slot of this tile's pairs of each digit; later: minus the digit's first tile-local slot
    __shared__ uint2 staged[kSortTile];               // the tile in digit order
    __shared__ uint32_t wave_total[WAVES];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x;
    const uint64_t base = (uint64_t)tile * kSortTile + (uint64_t)wave * (ROUNDS * 64u);
    for (uint32_t d = t; d < (uint32_t)WAVES * kDigits; d += BLOCK) (&wave_count[0][0])[d] = 0;
    {   // a digit's pairs start after all pairs of the smaller digits, then after the digit's pairs in the tiles before
        uint32_t all;
        const uint32_t before_tiles = t < kDigits ? s.tile_count[(uint64_t)t * s.tiles + tile] : 0u;
        const uint32_t before_digits = exclusive_scan_block<BLOCK>(t < kDigits ? s.totals[t] : 0u, wave_total, all);
        if (t < kDigits) digit_slot[t] = before_digits + before_tiles;
    }
    __syncthreads();

    uint32_t key[ROUNDS], val[ROUNDS], rank[ROUNDS];
#pragma unroll
    for (int i = 0; i < ROUNDS; ++i) {
        const uint64_t at = base + (uint32_t)i * 64u + lane;
        key[i] = at < s.n ? keys_in[at] : 0xFFFFFFFFu;
        val[i] = at < s.n ? vals_in[at] : 0u;
    }
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < ROUNDS; ++i) {
        const uint64_t at = base + (uint32_t)i * 64u + lane;
        const bool have = at < s.n;
        const uint32_t digit = (key[i] >> s.shift) & s.mask;
        // the lanes of this round that hold the same digit
        uint64_t same = __ballot(have);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t bit = __ballot((digit >> b) & 1u);
            same &= ((digit >> b) & 1u) ? bit : ~bit;
        }
        const uint32_t so_far = wave_count[wave][digit];        // every lane reads before the first lane of a set adds
        rank[i] = so_far + (uint32_t)__popcll(same & below);
        __builtin_amdgcn_wave_barrier();
        if (have && (same & below) == 0) wave_count[wave][digit] = so_far + (uint32_t)__popcll(same);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // per digit: the tile's count, every wavefront's base inside the digit, the digit's first slot
    uint32_t in_digit = 0;
    if (t < kDigits) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const uint32_t c = wave_count[w][t];
            wave_count[w][t] = in_digit;
            in_digit += c;
        }
    }
    {   // exclusive scan of the 256 digit counts: where each digit starts in the tile.  Folded into the
        // two tables the loops below look up once per pair: a wavefront's first tile-local slot of a
        // digit, and the distance from a digit's tile-local slots to its output slots.
        uint32_t all;
        const uint32_t start = exclusive_scan_block<BLOCK>(in_digit, wave_total, all);
        if (t < kDigits) {
#pragma unroll
            for (int w = 0; w < WAVES; ++w) wave_count[w][t] += start;
            digit_slot[t] -= start;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ROUNDS; ++i) {
        const uint64_t at = base + (uint32_t)i * 64u + lane;
        if (at < s.n) {
            const uint32_t digit = (key[i] >> s.shift) & s.mask;
            staged[wave_count[wave][digit] + rank[i]] = make_uint2(key[i], val[i]);
        }
    }
    __syncthreads();
    const uint64_t tile_base = (uint64_t)tile * kSortTile;
    const uint32_t in_tile = s.n - tile_base < kSortTile ? (uint32_t)(s.n - tile_base) : kSortTile;
#pragma unroll
    for (int i = 0; i < ROUNDS; ++i) {
        const uint32_t j = (uint32_t)i * BLOCK + t;
        if (j < in_tile) {
            const uint2 kv = staged[j];
            const uint32_t digit = (kv.x >> s.shift) & s.mask;
            const uint32_t slot = digit_slot[digit] + j;      // wraps like the subtraction above: the sum is the slot
            keys_out[slot] = kv.x;
            vals_out[slot] = kv.y;
        }
    }
}

}  // namespace robe
