// Device-side integer maps of ROBE-Z for gfx950: h (Eq. 5), g (Eq. 2), idx (Eq. 5)
// of arXiv 2108.02191, evaluated in registers with 32/64-bit arithmetic only.
//
// Every shortcut below is exact over the integers:
//   * P = 2^31 - 1 is a Mersenne prime, so t mod P folds: 2^31 == 1 (mod P).
//   * a sum of residues is reduced again before it can reach 2^64.
//   * r mod m for r < 2^31 uses a 32-bit reciprocal estimate that is low by at
//     most one, corrected by a single conditional subtraction.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace robe {

constexpr uint32_t kP = 2147483647u;

// Kernel-argument form of a ROBE-Z instance (host fills it from robe_hash_t).
struct Params {
    uint32_t m;        // array length, 1 <= m <= 2^31 - 1
    uint32_t m_recip;  // min(floor(2^32 / m), 2^32 - 1)
    uint32_t d, Z, C;  // C = d / Z chunks per embedding (1 when Z > d)
    uint32_t r;        // Z / d embeddings per chunk when Z > d, else 0
    uint32_t Ah, Bh, Ch, Dh;
    uint32_t Ag, Bg, Cg, Dg;
};

// t mod P for any 64-bit t, result in [0, P).
__device__ __forceinline__ uint32_t mod_p(uint64_t t)
{
    uint64_t s = (t & kP) + (t >> 31);              // < 2^33 + 2^31, congruent to t
    uint32_t r = (uint32_t)(s & kP) + (uint32_t)(s >> 31);  // < 2^31 + 5
    return r >= kP ? r - kP : r;
}

// (a + b) mod P for a, b in [0, P).
__device__ __forceinline__ uint32_t add_p(uint32_t a, uint32_t b)
{
    uint32_t s = a + b;                              // < 2^32 - 2
    return s >= kP ? s - kP : s;
}

// (a * b) mod P for a, b < 2^31 (product < 2^62).
__device__ __forceinline__ uint32_t mul_p(uint32_t a, uint32_t b)
{
    return mod_p((uint64_t)a * (uint64_t)b);
}

// r mod m for r < 2^31.  q = floor(r * recip / 2^32) is floor(r/m) or one less.
__device__ __forceinline__ uint32_t mod_m(uint32_t r, uint32_t m, uint32_t recip)
{
    uint32_t q = __umulhi(r, recip);
    uint32_t rem = r - q * m;                        // in [0, 2m), fits since m < 2^31
    return rem >= m ? rem - m : rem;
}

// Token part of a hash: (B * x) mod P with x read as an unsigned 64-bit integer.
__device__ __forceinline__ uint32_t token_term(uint32_t B, int64_t x)
{
    return mul_p(B, mod_p((uint64_t)x));
}

// Table-and-position part: (A*e + C*k + D) mod P for e < 2^31, k < 2^32.
__device__ __forceinline__ uint32_t static_term(uint32_t A, uint32_t C, uint32_t D, uint32_t e, uint32_t k)
{
    uint32_t te = mod_p((uint64_t)A * e + D);        // < 2^62 + 2^31
    uint32_t tk = mod_p((uint64_t)C * k);            // < 2^63
    return add_p(te, tk);
}

// h(e,x,c) from the two parts.
__device__ __forceinline__ uint32_t offset_of(const Params &p, uint32_t tok_h, uint32_t stat_h)
{
    return mod_m(add_p(tok_h, stat_h), p.m, p.m_recip);
}

// (o + j) mod m for o < m, j < Z <= m.
__device__ __forceinline__ uint32_t wrap(uint32_t pos, uint32_t m)
{
    return pos >= m ? pos - m : pos;
}

// Sign bit mask of g: 0x80000000 when g == -1 (hash residue even), else 0.
__device__ __forceinline__ uint32_t sign_mask(uint32_t residue)
{
    return ((residue & 1u) ^ 1u) << 31;
}

__device__ __forceinline__ float apply_sign(float v, uint32_t mask)
{
    return __uint_as_float(__float_as_uint(v) ^ mask);
}

}  // namespace robe
