// Bit geometry of the sign-only carry chain (the circuit of Sec. 4.2 evaluated only
// where bit 63 of the sum depends on it), shared by the two- and three-party chains.
//
// Prefix level l (shift d = 2^l, group s = 2d) needs G', P' only at the positions
// S_l = { p : p = s-2 (mod s), p <= 62 }.  pack_l puts s consecutive elements in
// one word: element k contributes rotl(word & msb_mask(l), k).  A level reads its
// operands from two words of pack_(l-1) (elements 0..d-1 and d..2d-1 of the
// group; pack_(-1) is the plain word) where S_(l-1) splits into the positions
// p (kept: sel_mask) and p - d (shifted in: low_mask).
#pragma once
#include "common.h"

constexpr u64 rotl_c(u64 x, int k) { k &= 63; return k ? (x << k) | (x >> (64 - k)) : x; }
constexpr u64 msb_mask(int level)
{
    const int s = 2 << level; u64 m = 0;
    for (int p = s - 2; p < 63; p += s) m |= (u64)1 << p;
    return m;
}
constexpr u64 sel_mask(int level)
{
    u64 a = 0;
    for (int k = 0; k < (1 << level); ++k) a |= rotl_c(msb_mask(level), k);
    return a;
}
constexpr u64 low_mask(int level)
{
    u64 b = 0;
    for (int k = 0; k < (1 << level); ++k) b |= rotl_c(msb_mask(level) >> (1 << level), k);
    return b;
}
template <int K> __device__ __forceinline__ u64 rotl(u64 x)
{
    constexpr int k = K & 63;
    if constexpr (k == 0) return x; else return (x << k) | (x >> (64 - k));
}

// words of level l's packed arrays for n elements: ceil64(n) / 2^(l+1), rounded up to 4
inline size_t msb_level_words(size_t n, int l)
{
    const size_t n64 = (n + 63) / 64 * 64;
    return ((n64 >> (l + 1)) + 3) / 4 * 4;
}
