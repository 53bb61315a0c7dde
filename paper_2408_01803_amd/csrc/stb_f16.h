// IEEE binary16 <-> binary32 conversions in integer arithmetic, shared by the host packer and the packer kernels so
// that both round a scale to the same bits whatever the conversion instructions of the machine do.
#ifndef STB_F16_H
#define STB_F16_H
#include <stdint.h>
#include <string.h>

#if defined(__HIPCC__)
#define STB_HD __host__ __device__
#else
#define STB_HD
#endif

// float -> IEEE binary16 bits, round-to-nearest-even, subnormals kept, overflow to infinity.
STB_HD inline uint16_t stb_f32_to_f16_bits(float f) {
    uint32_t x;
    memcpy(&x, &f, 4);
    const uint32_t sign = (x >> 16) & 0x8000u;
    x &= 0x7fffffffu;
    if (x >= 0x7f800000u) return (uint16_t)(sign | 0x7c00u | ((x > 0x7f800000u) ? 0x200u : 0u));
    if (x >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);             // rounds to >= 65520 -> inf
    if (x < 0x33000001u) return (uint16_t)sign;                         // <= 2^-25 rounds to zero
    int32_t e = (int32_t)(x >> 23) - 127;
    uint32_t m = (x & 0x7fffffu) | 0x800000u;                           // 24-bit significand
    int shift = (e < -14) ? (13 + (-14 - e)) : 13;                       // bits dropped
    uint32_t half = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t halfway = 1u << (shift - 1);
    if (rem > halfway || (rem == halfway && (half & 1u))) half++;
    uint32_t out;
    if (e < -14) out = half;                                            // subnormal (may carry into normal)
    else out = ((uint32_t)(e + 15) << 10) + (half - 0x400u);            // carry propagates into exponent
    return (uint16_t)(sign | out);
}

STB_HD inline float stb_f16_bits_to_f32(uint16_t h) {
    const uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu, x;
    if (e == 0) {
        if (m == 0) x = sign;
        else {
            int s = 0;
            while (!(m & 0x400u)) { m <<= 1; s++; }
            x = sign | ((uint32_t)(127 - 15 - s + 1) << 23) | ((m & 0x3ffu) << 13);
        }
    } else if (e == 31) x = sign | 0x7f800000u | (m << 13);
    else x = sign | ((e + 112u) << 23) | (m << 13);
    float f;
    memcpy(&f, &x, 4);
    return f;
}

// fp64 -> fp32 -> fp16, each step round-to-nearest-even: the storage rule of every scale.
STB_HD inline uint16_t stb_f64_to_f16_bits(double v) { return stb_f32_to_f16_bits((float)v); }

#endif
