// Exact rational numbers on 128-bit integers with overflow detection (host only).
// Used to generate the Cook-Toom matrices without any rounding; every operation reports
// overflow through the `ok` flag of the arithmetic context instead of wrapping.
#pragma once
#include <cstdint>
#include <cmath>

namespace nova {

typedef __int128 i128;
typedef unsigned __int128 u128;

struct Rat {
    i128 num = 0;
    i128 den = 1;   // always > 0, gcd(|num|, den) == 1
};

struct RatCtx {
    bool ok = true;   // cleared on the first overflow; results after that are meaningless

    static i128 iabs(i128 v) { return v < 0 ? -v : v; }
    static i128 gcd(i128 a, i128 b)
    {
        a = iabs(a); b = iabs(b);
        while (b != 0) { i128 r = a % b; a = b; b = r; }
        return a;
    }
    i128 mul(i128 a, i128 b)
    {
        i128 r;
        if (__builtin_mul_overflow(a, b, &r)) { ok = false; return 0; }
        return r;
    }
    i128 add(i128 a, i128 b)
    {
        i128 r;
        if (__builtin_add_overflow(a, b, &r)) { ok = false; return 0; }
        return r;
    }
    Rat make(i128 num, i128 den)
    {
        Rat r;
        if (den == 0) { ok = false; return r; }
        if (den < 0) { num = -num; den = -den; }
        i128 g = gcd(num, den);
        if (g > 1) { num /= g; den /= g; }
        r.num = num; r.den = den;
        return r;
    }
    Rat mul(const Rat &a, const Rat &b)
    {
        // cross-reduce first to keep the factors small
        i128 g1 = gcd(a.num, b.den), g2 = gcd(b.num, a.den);
        if (g1 == 0) g1 = 1;
        if (g2 == 0) g2 = 1;
        return make(mul(a.num / g1, b.num / g2), mul(a.den / g2, b.den / g1));
    }
    Rat add(const Rat &a, const Rat &b)
    {
        i128 g = gcd(a.den, b.den);
        i128 bd = b.den / g, ad = a.den / g;
        return make(add(mul(a.num, bd), mul(b.num, ad)), mul(a.den, bd));
    }
    Rat neg(const Rat &a) { Rat r = a; r.num = -r.num; return r; }
    Rat sub(const Rat &a, const Rat &b) { return add(a, neg(b)); }
    Rat inv(const Rat &a) { return make(a.den, a.num); }
    static bool eq(const Rat &a, const Rat &b) { return a.num == b.num && a.den == b.den; }
    static bool is_zero(const Rat &a) { return a.num == 0; }
    static bool fits64(const Rat &a)
    {
        return a.num >= INT64_MIN + 1 && a.num <= INT64_MAX && a.den <= INT64_MAX;
    }
};

// Nearest binary floating-point value with `P` significand bits (ties to even), computed
// from the exact quotient by integer division.  Requires |num|, den < 2^63 and a result in
// the normal range of the target format (transform entries always are).
template <int P>
inline double round_rat_to_bits(const Rat &a)
{
    if (a.num == 0) return 0.0;
    bool negative = a.num < 0;
    u128 num = (u128)(negative ? -a.num : a.num);
    u128 den = (u128)a.den;
    int bl_num = 0, bl_den = 0;
    for (u128 v = num; v != 0; v >>= 1) ++bl_num;
    for (u128 v = den; v != 0; v >>= 1) ++bl_den;
    // choose s so that q = floor(num * 2^s / den) has P+2 or P+3 bits
    int s = (P + 2) - (bl_num - bl_den);
    u128 q, rem;
    if (s >= 0) { q = (num << s) / den; rem = (num << s) % den; }
    else        { q = num / (den << -s); rem = num % (den << -s); }
    int bl_q = 0;
    for (u128 v = q; v != 0; v >>= 1) ++bl_q;
    int drop = bl_q - P;                       // 2 or 3 low bits to round away
    u128 kept = q >> drop;
    u128 low = q & (((u128)1 << drop) - 1);
    u128 half = (u128)1 << (drop - 1);
    bool sticky = rem != 0;
    if (low > half || (low == half && (sticky || (kept & 1)))) ++kept;
    double v = std::ldexp((double)(uint64_t)kept, drop - s);   // kept <= 2^P <= 2^53: exact
    return negative ? -v : v;
}

// Nearest binary16 value (ties to even) as a double: sub-normals below 2^-14 (multiples of
// 2^-24) and overflow to infinity above the largest finite value included.
// Requires |num|, den < 2^63.
inline double rat_to_f16_value(const Rat &a)
{
    if (a.num == 0) return 0.0;
    const bool negative = a.num < 0;
    const u128 num = (u128)(negative ? -a.num : a.num), den = (u128)a.den;
    double v;
    if ((num << 14) < den) {                                 // |a| < 2^-14: fixed quantum 2^-24
        const u128 q = (num << 24) / den, rem = (num << 24) % den;
        u128 kept = q;
        if (2 * rem > den || (2 * rem == den && (kept & 1))) ++kept;
        v = std::ldexp((double)(uint64_t)kept, -24);
    } else {
        Rat mag = a;
        mag.num = (i128)num;
        v = round_rat_to_bits<11>(mag);
        if (v > 65504.0) v = INFINITY;
    }
    return negative ? -v : v;
}

inline double rat_to_f64(const Rat &a) { return round_rat_to_bits<53>(a); }
inline float rat_to_f32(const Rat &a) { return (float)round_rat_to_bits<24>(a); }

}  // namespace nova
