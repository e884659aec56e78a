// CPU stand-in for the half-precision conversions libprep uses (test infrastructure).
#pragma once
#include <cstdint>
#include <cstring>

struct __half { uint16_t x; };
struct __half2 { __half lo, hi; };

// IEEE 754 binary32 -> binary16, round to nearest even
inline __half __float2half_rn(float f)
{
    uint32_t b;
    memcpy(&b, &f, 4);
    const uint32_t sign = (b >> 16) & 0x8000u;
    const int32_t exp = (int32_t)((b >> 23) & 0xFF) - 127 + 15;
    uint32_t man = b & 0x7FFFFFu;
    uint16_t h;
    if (((b >> 23) & 0xFF) == 0xFF) {
        h = (uint16_t)(sign | 0x7C00u | (man ? 0x200u : 0u));
    } else if (exp >= 31) {
        h = (uint16_t)(sign | 0x7C00u);
    } else if (exp <= 0) {
        if (exp < -10) {
            h = (uint16_t)sign;
        } else {
            man |= 0x800000u;
            const int shift = 14 - exp;  // 14..24
            uint32_t v = man >> shift;
            const uint32_t rem = man & ((1u << shift) - 1u), half = 1u << (shift - 1);
            if (rem > half || (rem == half && (v & 1u))) v++;
            h = (uint16_t)(sign | v);
        }
    } else {
        uint32_t v = ((uint32_t)exp << 10) | (man >> 13);
        const uint32_t rem = man & 0x1FFFu;
        if (rem > 0x1000u || (rem == 0x1000u && (v & 1u))) v++;
        h = (uint16_t)(sign | v);
    }
    return __half{h};
}
inline __half2 __floats2half2_rn(float a, float b) { return __half2{__float2half_rn(a), __float2half_rn(b)}; }
