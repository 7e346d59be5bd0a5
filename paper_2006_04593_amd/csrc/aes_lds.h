// AES-128 (Matyas-Meyer-Oseas PRG blocks) on bank-replicated tables in LDS -- the engine
// the FSS kernels use.  Device-only header.
//
// gfx950 has no AES instruction.  AES runs on combined SubBytes+MixColumns tables:
//   - four tables (one per state row) x 256 entries, each entry replicated 32 times so
//     that lane l always reads bank (l mod 32): lookups with data-dependent indices never
//     collide inside a half-wavefront, whatever the data;
//   - an entry owns 256 bytes: [T_even copy 0..31 | T_odd copy 0..31], tables 0/1 in the
//     first 64 KiB and tables 2/3 in the second.  The byte address of a lookup is then
//     (index << 8) | lane_base, which ONE v_perm_b32 forms straight from a state word
//     (byte k of the word dropped into byte 1 of a per-lane constant);
//   - 128 KiB of the CU's 160 KiB LDS, one workgroup per CU.
// Round keys are compile-time constants (scalar operands).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aes_consts.h"

namespace fss {

// ------------------------------------------------------------------------------------
// LDS tables
// ------------------------------------------------------------------------------------

constexpr uint32_t kLdsBytes = 128u * 1024u;
constexpr uint32_t kRegionB = 64u * 1024u;   // tables 2 and 3
constexpr uint32_t kOddTable = 128u;         // tables 1 and 3 inside an entry
constexpr int kThreads = 1024;

__constant__ AesConsts c_aes = make_aes_consts();

typedef __attribute__((address_space(3))) uint32_t lds_u32;

__device__ __forceinline__ uint32_t lds_load(uint32_t byte_addr)
{
    return *reinterpret_cast<const lds_u32 *>(byte_addr);
}

__device__ __forceinline__ uint32_t rotl32(uint32_t v, int k) { return k == 0 ? v : __builtin_amdgcn_alignbit(v, v, 32 - k); }

// Every thread of the workgroup writes its share of the 32768 table words.
__device__ __forceinline__ void fill_tables(uint32_t *lds)
{
    for (uint32_t j = threadIdx.x; j < kLdsBytes / 4; j += blockDim.x) {
        uint32_t region = j >> 14;          // 0: tables 0/1, 1: tables 2/3
        uint32_t v = (j >> 6) & 255u;       // table index
        uint32_t odd = (j >> 5) & 1u;
        uint32_t t = c_aes.te0[v];
        lds[j] = rotl32(t, 8 * (int)(2 * region + odd));   // te_r = te_0 rotated by r bytes
    }
}

struct LaneBase {
    uint32_t a;   // byte address of this lane's copy inside an entry, region of tables 0/1
    uint32_t b;   // same for tables 2/3
};

__device__ __forceinline__ LaneBase lane_base(const uint32_t *lds)
{
    // LDS pointers are 32-bit offsets; the dynamic segment may not start at 0.
    uint32_t base = (uint32_t)(uintptr_t)((const lds_u32 *)lds);
    LaneBase l;
    l.a = base + ((threadIdx.x & 31u) << 2);
    l.b = l.a + kRegionB;
    return l;
}

// byte address (index << 8) | lane_base with index = byte K of w
template <int K>
__device__ __forceinline__ uint32_t entry_addr(uint32_t w, uint32_t base)
{
    // v_perm_b32: selector values 0..3 pick bytes of the second operand, 4..7 of the first
    return __builtin_amdgcn_perm(w, base, 0x03020000u | ((4u + K) << 8));
}

// ------------------------------------------------------------------------------------
// AES-128 on NB independent blocks per lane (interleaved for latency hiding).
// st[b][c] = little-endian word of state column c of block b.
// Key selection: block b uses PRG key `key[b]` (0..2) if key[b] >= 0; key[b] == -1 means
// "per lane: PRG key 2 where `pick` is set, else PRG key 1".
// ------------------------------------------------------------------------------------

// v_bitop3_b32: any three-input bitwise function; truth table built from a=0xF0, b=0xCC, c=0xAA
constexpr uint32_t kXor3 = 0xF0 ^ 0xCC ^ 0xAA;            // a ^ b ^ c
constexpr uint32_t kXorAnd = 0xF0 ^ (0xCC & 0xAA);        // a ^ (b & c)
constexpr uint32_t kOrXor = (0xF0 | 0xCC) ^ 0xAA;         // (a | b) ^ c
constexpr uint32_t kSelect = (0xF0 & 0xCC) | (0x0F & 0xAA);   // a ? b : c, bit by bit

template <uint32_t TT>
__device__ __forceinline__ uint32_t bitop3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, TT);
}

// m must be 0 or ~0: all bits of x1 where m is set, else of x0
__device__ __forceinline__ uint32_t pick32(uint32_t m, uint32_t x1, uint32_t x0) { return bitop3<kSelect>(m, x1, x0); }

// acc ^ extra ^ round-key word `idx` of PRG key `m`.  m = 0..2: that key for every lane.
// m = -1: PRG key 1 for lanes with pick = 0 and PRG key 2 for lanes with pick = ~0, formed as
// key_1 ^ (pick & (key_1 ^ key_2)) so that both constants stay in scalar registers.
// (m is a compile-time constant after unrolling; the branches fold away.)
__device__ __forceinline__ uint32_t add_round_key(int m, uint32_t acc, uint32_t extra, int idx, uint32_t pick)
{
    if (m >= 0) return bitop3<kXor3>(acc, extra, kAes.rk[m][idx]);
    uint32_t v = bitop3<kXor3>(acc, extra, kAes.rk[0][idx]);
    return bitop3<kXorAnd>(v, pick, kAes.rk[0][idx] ^ kAes.rk[1][idx]);
}

// The four table lookups that feed output column c of the next round.  lk[r] is the
// contribution of the row-r byte (ShiftRows: it comes from state column c + r).  Rounds
// 1..9 read table r; the last round reads table r + 2, whose byte r is S(v).
template <bool LAST>
__device__ __forceinline__ void issue_column(uint32_t *lk, const uint32_t (&st)[4], int c, LaneBase L)
{
    const uint32_t b01 = LAST ? L.b : L.a;   // rows 0,1: tables 0,1 (2,3 in the last round)
    const uint32_t b23 = LAST ? L.a : L.b;   // rows 2,3: tables 2,3 (0,1 in the last round)
    lk[0] = lds_load(entry_addr<0>(st[c], b01));
    lk[1] = lds_load(entry_addr<1>(st[(c + 1) & 3], b01) + kOddTable);
    lk[2] = lds_load(entry_addr<2>(st[(c + 2) & 3], b23));
    lk[3] = lds_load(entry_addr<3>(st[(c + 3) & 3], b23) + kOddTable);
}

// NB independent AES-128 encryptions per lane, each followed by the Matyas-Meyer-Oseas
// feed-forward: out[b] = E_{key M_b}(seed[b]) ^ seed[b].  pick[b] (0 or ~0 per lane) is only
// read by blocks whose key is -1.
//
// A wavefront can keep 16 LDS instructions in flight and a round of one block is exactly 16
// lookups, so the unit of work is a block-round: issue its 16 lookups, then combine.  The
// combine starts with the LAST column, so one wait covers the whole round (fewer
// instructions on the wave's in-order issue path than a wait per column).
template <int... M>
__device__ __forceinline__ void aes_mmo(uint32_t (&out)[sizeof...(M)][4], const uint32_t (&seed)[sizeof...(M)][4],
                                        const uint32_t (&pick)[sizeof...(M)], LaneBase L)
{
    constexpr int NB = sizeof...(M);
    constexpr int keys[NB] = { M... };
    uint32_t st[NB][4];
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int c = 0; c < 4; c++) st[b][c] = add_round_key(keys[b], seed[b][c], 0u, c, pick[b]);
#pragma clang loop unroll(full)
    for (int r = 1; r <= 10; r++) {
#pragma clang loop unroll(full)
        for (int b = 0; b < NB; b++) {
            uint32_t lk[16];
#pragma unroll
            for (int c = 0; c < 4; c++) {
                if (r < 10) issue_column<false>(&lk[4 * c], st[b], c, L);
                else issue_column<true>(&lk[4 * c], st[b], c, L);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cc = 0; cc < 4; cc++) {
                const int c = 3 - cc;
                if (r < 10) {
                    st[b][c] = add_round_key(keys[b], bitop3<kXor3>(lk[4 * c], lk[4 * c + 1], lk[4 * c + 2]),
                                             lk[4 * c + 3], 4 * r + c, pick[b]);
                } else {
                    // last round: SubBytes + ShiftRows only, S(v) = byte r of the row-r lookup
                    uint32_t lo = __builtin_amdgcn_perm(lk[4 * c + 1], lk[4 * c + 0], 0x0c0c0500u);   // l0.b0, l1.b1, 0, 0
                    uint32_t hi = __builtin_amdgcn_perm(lk[4 * c + 3], lk[4 * c + 2], 0x07020c0cu);   // 0, 0, l2.b2, l3.b3
                    out[b][c] = add_round_key(keys[b], bitop3<kOrXor>(lo, hi, seed[b][c]), 0u, 40 + c, pick[b]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

}  // namespace fss
