// Bit-plane ("bitsliced") AES-128 for the PRG, eight blocks per lane, ALU only.
//
// The table-driven AES of fss_kernels.hip is bound by the LDS (160 lookups per block);
// the vector ALU idles most of the time.  This engine computes the same function with
// no memory access at all: the S-box is a Boolean circuit (aes_sbox_circuit.inc, 109
// three-input operations, generated and exhaustively checked by gen_sbox_circuit.py) and
// the linear layers are XORs and byte rotations of registers.
//
// Layout: eight blocks j = 0..7 are processed together.  Register P[i][r] (i = bit 0..7 of
// a state byte, r = row 0..3) holds, in byte c (column) and bit j of that byte, bit i of
// state byte (r, c) of block j.  32 registers carry 8 blocks; one S-box circuit evaluation
// on (P[0..7][r]) substitutes 32 bytes; ShiftRows rotates P[i][r] by r bytes; MixColumns
// works across r inside each byte lane, so it needs no data movement at all.
//
// The code is plain C++ on uint32_t so that the same source is exercised on the host
// (tests build it with g++ and check it against FIPS-197) and compiled for gfx950, where
// FSS_B3 maps to v_bitop3_b32.
#pragma once
#include <stdint.h>

#include "aes_consts.h"

#if defined(__HIPCC__)
#define FSS_BP_FN __host__ __device__ __forceinline__
#else
#define FSS_BP_FN inline
#endif

namespace fss {
namespace bp {
// host stand-ins with the semantics of v_bitop3_b32, v_perm_b32 and v_alignbit_b32
FSS_BP_FN uint32_t host_b3(uint32_t tt, uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r = 0;
    for (int idx = 0; idx < 8; idx++)
        if ((tt >> idx) & 1u)
            r |= ((idx & 4) ? a : ~a) & ((idx & 2) ? b : ~b) & ((idx & 1) ? c : ~c);
    return r;
}
// selector byte 0..3 picks a byte of `lo`, 4..7 a byte of `hi`, 0x0c gives 0x00
FSS_BP_FN uint32_t host_perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    uint32_t r = 0;
    for (int k = 0; k < 4; k++) {
        uint32_t s = (sel >> (8 * k)) & 0xffu, v;
        if (s < 4) v = (lo >> (8 * s)) & 0xffu;
        else if (s < 8) v = (hi >> (8 * (s - 4))) & 0xffu;
        else v = (s == 0x0c) ? 0u : 0xffu;
        r |= v << (8 * k);
    }
    return r;
}
}  // namespace bp
}  // namespace fss

#if defined(__HIP_DEVICE_COMPILE__)
#define FSS_B3(tt, a, b, c) __builtin_amdgcn_bitop3_b32((a), (b), (c), (tt))
#define FSS_PERM(hi, lo, sel) __builtin_amdgcn_perm((hi), (lo), (sel))
#define FSS_ROTR(v, k) __builtin_amdgcn_alignbit((v), (v), (k))
#else
#define FSS_B3(tt, a, b, c) ::fss::bp::host_b3((tt), (a), (b), (c))
#define FSS_PERM(hi, lo, sel) ::fss::bp::host_perm((hi), (lo), (sel))
#define FSS_ROTR(v, k) ((k) == 0 ? (v) : (((v) >> (k)) | ((v) << (32 - (k)))))
#endif

namespace fss {
namespace bp {

typedef uint32_t W;

constexpr uint32_t kTtXor3 = 0xF0 ^ 0xCC ^ 0xAA;              // a ^ b ^ c
constexpr uint32_t kTtXorAnd = 0xF0 ^ (0xCC & 0xAA);          // a ^ (b & c)
constexpr uint32_t kTtSel = (0xF0 & 0xCC) | (0x0F & 0xAA);    // a ? b : c

struct Planes {
    W p[8][4];   // [bit][row]
};

// ---------------------------------------------------------------------------------------
// round keys as planes.  A key plane register has, in byte c, 0xff where bit i of round-key
// byte (r, c) is set: the same key for all eight blocks.  Block-dependent keys are formed
// from these by masking the bits (blocks) they apply to.
// ---------------------------------------------------------------------------------------

struct KeyPlanes {
    uint32_t k[3][11][8][4];   // [PRG key][round][bit][row]
};

constexpr KeyPlanes make_key_planes()
{
    KeyPlanes kp{};
    for (int m = 0; m < 3; m++)
        for (int rd = 0; rd < 11; rd++)
            for (int i = 0; i < 8; i++)
                for (int r = 0; r < 4; r++) {
                    uint32_t v = 0;
                    for (int c = 0; c < 4; c++) {
                        uint32_t byte = (kAes.rk[m][4 * rd + c] >> (8 * r)) & 0xffu;
                        if ((byte >> i) & 1u) v |= 0xffu << (8 * c);
                    }
                    kp.k[m][rd][i][r] = v;
                }
    return kp;
}

inline constexpr KeyPlanes kKeyPlanes = make_key_planes();

// Which PRG key each of the eight blocks uses.
//   kUniform<M>: all blocks key M (0..2).
//   kPickLowK3High: blocks 0..3 use key 0 or 1 per block (bit j of `pick` set -> key 1),
//                   blocks 4..7 use key 2.
//   kPickAll:       blocks 0..7 use key 0 or 1 per block.
enum KeyMode { kUniform0 = 0, kUniform1 = 1, kUniform2 = 2, kPickLowK3High = 3, kPickAll = 4 };

// state ^= round key `rd`.  pick: byte-replicated mask (same 8 bits in all four bytes), bit j
// set = block j takes PRG key 1 instead of key 0.
template <int MODE>
FSS_BP_FN void add_round_key(Planes &s, int rd, W pick)
{
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
            if (MODE <= 2) {
                const uint32_t k = kKeyPlanes.k[MODE][rd][i][r];
                if (k != 0) s.p[i][r] ^= k;
            } else {
                const uint32_t lowmask = (MODE == kPickLowK3High) ? 0x0f0f0f0fu : 0xffffffffu;
                const uint32_t base = (kKeyPlanes.k[0][rd][i][r] & lowmask) | (kKeyPlanes.k[2][rd][i][r] & ~lowmask);
                const uint32_t diff = (kKeyPlanes.k[0][rd][i][r] ^ kKeyPlanes.k[1][rd][i][r]) & lowmask;
                W v = s.p[i][r];
                if (base != 0) v ^= base;
                if (diff != 0) v = FSS_B3(kTtXorAnd, v, pick, diff);
                s.p[i][r] = v;
            }
        }
}

// ---------------------------------------------------------------------------------------
// SubBytes: the generated circuit on each row's eight planes
// ---------------------------------------------------------------------------------------

FSS_BP_FN void sbox8(W &y0, W &y1, W &y2, W &y3, W &y4, W &y5, W &y6, W &y7,
                     W x0, W x1, W x2, W x3, W x4, W x5, W x6, W x7)
{
#include "aes_sbox_circuit.inc"
}

FSS_BP_FN void sub_bytes(Planes &s)
{
#pragma unroll
    for (int r = 0; r < 4; r++)
        sbox8(s.p[0][r], s.p[1][r], s.p[2][r], s.p[3][r], s.p[4][r], s.p[5][r], s.p[6][r], s.p[7][r],
              s.p[0][r], s.p[1][r], s.p[2][r], s.p[3][r], s.p[4][r], s.p[5][r], s.p[6][r], s.p[7][r]);
}

// ShiftRows: row r moves left by r columns; new byte c = old byte (c + r) mod 4
FSS_BP_FN void shift_rows(Planes &s)
{
#pragma unroll
    for (int i = 0; i < 8; i++) {
        s.p[i][1] = FSS_ROTR(s.p[i][1], 8);
        s.p[i][2] = FSS_ROTR(s.p[i][2], 16);
        s.p[i][3] = FSS_ROTR(s.p[i][3], 24);
    }
}

// MixColumns: y_r = 2 (a_r ^ a_{r+1}) ^ a_{r+1} ^ a_{r+2} ^ a_{r+3}, all inside one byte lane.
// With b_r = a_r ^ a_{r+1}: y_r = xtime(b_r) ^ a_{r+1} ^ b_{r+2}, and xtime on planes is a
// renaming of planes plus b_7 folded into planes 0, 1, 3, 4 (polynomial 0x1b).
FSS_BP_FN void mix_columns(Planes &s)
{
    W b[8][4];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int r = 0; r < 4; r++) b[i][r] = s.p[i][r] ^ s.p[i][(r + 1) & 3];
    Planes y;
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const int r1 = (r + 1) & 3, r2 = (r + 2) & 3;
        y.p[0][r] = FSS_B3(kTtXor3, b[7][r], s.p[0][r1], b[0][r2]);
        y.p[1][r] = FSS_B3(kTtXor3, b[0][r], b[7][r], s.p[1][r1]) ^ b[1][r2];
        y.p[2][r] = FSS_B3(kTtXor3, b[1][r], s.p[2][r1], b[2][r2]);
        y.p[3][r] = FSS_B3(kTtXor3, b[2][r], b[7][r], s.p[3][r1]) ^ b[3][r2];
        y.p[4][r] = FSS_B3(kTtXor3, b[3][r], b[7][r], s.p[4][r1]) ^ b[4][r2];
        y.p[5][r] = FSS_B3(kTtXor3, b[4][r], s.p[5][r1], b[5][r2]);
        y.p[6][r] = FSS_B3(kTtXor3, b[5][r], s.p[6][r1], b[6][r2]);
        y.p[7][r] = FSS_B3(kTtXor3, b[6][r], s.p[7][r1], b[7][r2]);
    }
    s = y;
}

// ---------------------------------------------------------------------------------------
// conversion between eight ordinary blocks and the plane form
// blk[j][c] = little-endian word of column c of block j (byte r of the word = row r)
// ---------------------------------------------------------------------------------------

// exchange the bits selected by `m` in b with the bits `sh` higher in a
FSS_BP_FN void swap_bits(W &a, W &b, uint32_t m, int sh)
{
    const W na = FSS_B3(kTtSel, m << sh, b << sh, a);
    const W nb = FSS_B3(kTtSel, m, a >> sh, b);
    a = na;
    b = nb;
}

// 8x8 bit transpose inside every byte lane of v[0..7]: afterwards bit j of a byte of v[i]
// is what bit i of the same byte of v[j] was
FSS_BP_FN void transpose_bits8(W (&v)[8])
{
    swap_bits(v[0], v[4], 0x0f0f0f0fu, 4); swap_bits(v[1], v[5], 0x0f0f0f0fu, 4);
    swap_bits(v[2], v[6], 0x0f0f0f0fu, 4); swap_bits(v[3], v[7], 0x0f0f0f0fu, 4);
    swap_bits(v[0], v[2], 0x33333333u, 2); swap_bits(v[1], v[3], 0x33333333u, 2);
    swap_bits(v[4], v[6], 0x33333333u, 2); swap_bits(v[5], v[7], 0x33333333u, 2);
    swap_bits(v[0], v[1], 0x55555555u, 1); swap_bits(v[2], v[3], 0x55555555u, 1);
    swap_bits(v[4], v[5], 0x55555555u, 1); swap_bits(v[6], v[7], 0x55555555u, 1);
}

// 4x4 byte transpose: out[r] byte c = in[c] byte r
FSS_BP_FN void transpose_bytes4(W (&out)[4], const W (&in)[4])
{
    const W t0 = FSS_PERM(in[1], in[0], 0x05010400u);   // in0.b0 in1.b0 in0.b1 in1.b1
    const W t1 = FSS_PERM(in[1], in[0], 0x07030602u);   // in0.b2 in1.b2 in0.b3 in1.b3
    const W u0 = FSS_PERM(in[3], in[2], 0x05010400u);
    const W u1 = FSS_PERM(in[3], in[2], 0x07030602u);
    out[0] = FSS_PERM(u0, t0, 0x05040100u);
    out[1] = FSS_PERM(u0, t0, 0x07060302u);
    out[2] = FSS_PERM(u1, t1, 0x05040100u);
    out[3] = FSS_PERM(u1, t1, 0x07060302u);
}

FSS_BP_FN void pack(Planes &s, const W (&blk)[8][4])
{
    W rows[8][4];   // rows[j][r]: byte c = state byte (r, c) of block j
#pragma unroll
    for (int j = 0; j < 8; j++) transpose_bytes4(rows[j], blk[j]);
#pragma unroll
    for (int r = 0; r < 4; r++) {
        W v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = rows[j][r];
        transpose_bits8(v);
#pragma unroll
        for (int i = 0; i < 8; i++) s.p[i][r] = v[i];
    }
}

FSS_BP_FN void unpack(W (&blk)[8][4], const Planes &s)
{
    W rows[8][4];
#pragma unroll
    for (int r = 0; r < 4; r++) {
        W v[8];
#pragma unroll
        for (int i = 0; i < 8; i++) v[i] = s.p[i][r];
        transpose_bits8(v);
#pragma unroll
        for (int j = 0; j < 8; j++) rows[j][r] = v[j];
    }
#pragma unroll
    for (int j = 0; j < 8; j++) transpose_bytes4(blk[j], rows[j]);   // the byte transpose is an involution
}

// ---------------------------------------------------------------------------------------
// AES-128 encryption of eight blocks, then the Matyas-Meyer-Oseas feed-forward
// ---------------------------------------------------------------------------------------

template <int MODE>
FSS_BP_FN void encrypt8(Planes &s, W pick)
{
    add_round_key<MODE>(s, 0, pick);
#pragma unroll
    for (int rd = 1; rd <= 9; rd++) {
        sub_bytes(s);
        shift_rows(s);
        mix_columns(s);
        add_round_key<MODE>(s, rd, pick);
    }
    sub_bytes(s);
    shift_rows(s);
    add_round_key<MODE>(s, 10, pick);
}

// out[j] = E_{key of block j}(in[j]) ^ in[j]
template <int MODE>
FSS_BP_FN void mmo8(W (&out)[8][4], const W (&in)[8][4], W pick)
{
    Planes s;
    pack(s, in);
    encrypt8<MODE>(s, pick);
    unpack(out, s);
#pragma unroll
    for (int j = 0; j < 8; j++)
#pragma unroll
        for (int c = 0; c < 4; c++) out[j][c] ^= in[j][c];
}

}  // namespace bp
}  // namespace fss
