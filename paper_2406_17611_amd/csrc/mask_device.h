// Device side of the keyed choice of kept positions (see MaskRule in varco_internal.h).
#pragma once

#include "varco_internal.h"

// Bijective 32-bit xorshift-multiply mixer; multipliers floor(2^32 frac(sqrt 2)) and floor(2^32 frac(sqrt 3)).
__device__ __forceinline__ uint32_t varco_mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x6A09E667u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

// x mod width for x < 2^32 using the precomputed floor(2^32 / width): the estimated quotient is short
// by at most one, so a single conditional subtraction finishes the reduction.
__device__ __forceinline__ uint32_t varco_mod_width(uint32_t x, uint32_t width, uint32_t magic) {
    uint32_t r = x - __umulhi(x, magic) * width;
    return r >= width ? r - width : r;
}

// The two key words of the rule's step, layer and hop: kernel arguments, or the device-resident step table.
__device__ __forceinline__ uint32_t varco_key0(const MaskRule& rule) { return rule.words ? rule.words[0] : rule.s0; }
__device__ __forceinline__ uint32_t varco_key1(const MaskRule& rule) { return rule.words ? rule.words[1] : rule.s1; }

struct MaskAffine {
    uint32_t a, b, a_inv;
};

__device__ __forceinline__ MaskAffine varco_affine(const MaskRule& rule, uint32_t gid) {
    const uint32_t h1 = varco_mix32(gid ^ varco_key0(rule));
    const uint32_t h2 = varco_mix32(h1 ^ varco_key1(rule));
    const uint32_t u = __umulhi(h2, rule.n_units);
    MaskAffine m;
    m.b = __umulhi(h1, rule.width);
    m.a = rule.units[u];
    m.a_inv = rule.units_inv[u];
    return m;
}

// pi_v(j); the caller handles k == width (identity) itself.
__device__ __forceinline__ uint32_t varco_position(const MaskRule& rule, const MaskAffine& m, uint32_t j) {
    return varco_mod_width(m.a * j + m.b, rule.width, rule.width_magic);
}

// j with pi_v(j) == c (in [0, width)); c is kept iff the result is < k.
__device__ __forceinline__ uint32_t varco_inverse_position(const MaskRule& rule, const MaskAffine& m, uint32_t c) {
    const uint32_t d = c >= m.b ? c - m.b : c + rule.width - m.b;
    return varco_mod_width(m.a_inv * d, rule.width, rule.width_magic);
}
