// Compile-time AES-128 constants for the device PRG: the combined SubBytes+MixColumns
// table and the expanded round keys of the three fixed PRG keys.
//
// Everything here is derived at compile time from the definitions in FIPS-197 (field
// GF(2^8) mod x^8+x^4+x^3+x+1, S-box = affine map of the inverse, key expansion of
// section 5.2); no table is typed in.  The inverse is taken through discrete logarithms
// to the generator 0x03.
//
// PRG keys (paper, appendix C.1: "fixed and hard-coded"; the values are this library's
// choice): k_m = 00 01 02 .. 0e (0f + m - 1), m = 1, 2, 3.
#pragma once
#include <stdint.h>

namespace fss {

struct AesConsts {
    uint8_t sbox[256];
    // te0[v] = column (2,1,1,3) * S(v): bytes b0..b3 = 2s, s, s, 3s, little-endian in a u32.
    // The contributions of rows 1..3 are byte rotations of it: te_r[v] = rotl32(te0[v], 8 r).
    uint32_t te0[256];
    // rk[m][4 r + c] = little-endian word of bytes 4c..4c+3 of round key r of PRG key m+1
    uint32_t rk[3][44];
};

constexpr uint8_t gf_double(uint8_t a) { return (uint8_t)((a << 1) ^ ((a & 0x80) ? 0x1b : 0)); }

constexpr uint8_t rotl8(uint8_t v, int k) { return (uint8_t)((v << k) | (v >> (8 - k))); }

constexpr AesConsts make_aes_consts()
{
    AesConsts c{};
    uint8_t pow3[256] = {};
    uint8_t log3[256] = {};
    uint8_t p = 1;
    for (int i = 0; i < 255; i++) {
        pow3[i] = p;
        log3[p] = (uint8_t)i;
        p = (uint8_t)(p ^ gf_double(p));   // multiply by the generator 0x03
    }
    for (int v = 0; v < 256; v++) {
        uint8_t inv = 0;
        if (v != 0) inv = pow3[(255 - log3[v]) % 255];
        uint8_t s = (uint8_t)(inv ^ rotl8(inv, 1) ^ rotl8(inv, 2) ^ rotl8(inv, 3) ^ rotl8(inv, 4) ^ 0x63);
        c.sbox[v] = s;
        uint8_t s2 = gf_double(s);
        uint8_t s3 = (uint8_t)(s2 ^ s);
        c.te0[v] = (uint32_t)s2 | ((uint32_t)s << 8) | ((uint32_t)s << 16) | ((uint32_t)s3 << 24);
    }
    for (int m = 0; m < 3; m++) {
        uint8_t w[176] = {};
        for (int i = 0; i < 16; i++) w[i] = (uint8_t)i;
        w[15] = (uint8_t)(0x0f + m);
        uint8_t rcon = 1;
        for (int i = 4; i < 44; i++) {
            uint8_t t0 = w[4 * i - 4], t1 = w[4 * i - 3], t2 = w[4 * i - 2], t3 = w[4 * i - 1];
            if (i % 4 == 0) {
                uint8_t u0 = (uint8_t)(c.sbox[t1] ^ rcon), u1 = c.sbox[t2], u2 = c.sbox[t3], u3 = c.sbox[t0];
                t0 = u0; t1 = u1; t2 = u2; t3 = u3;
                rcon = gf_double(rcon);
            }
            w[4 * i + 0] = (uint8_t)(w[4 * i - 16] ^ t0);
            w[4 * i + 1] = (uint8_t)(w[4 * i - 15] ^ t1);
            w[4 * i + 2] = (uint8_t)(w[4 * i - 14] ^ t2);
            w[4 * i + 3] = (uint8_t)(w[4 * i - 13] ^ t3);
        }
        for (int i = 0; i < 44; i++)
            c.rk[m][i] = (uint32_t)w[4 * i] | ((uint32_t)w[4 * i + 1] << 8) | ((uint32_t)w[4 * i + 2] << 16) |
                         ((uint32_t)w[4 * i + 3] << 24);
    }
    return c;
}

inline constexpr AesConsts kAes = make_aes_consts();

// spot checks against values printed in FIPS-197 (figure 7 and appendix A.1)
static_assert(kAes.sbox[0x00] == 0x63 && kAes.sbox[0x53] == 0xed && kAes.sbox[0xff] == 0x16, "S-box");
static_assert(kAes.rk[0][4] == 0xfd74aad6u, "key expansion of 000102..0f, word 4 = d6aa74fd");

}  // namespace fss
