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

__device__ __forceinline__ uint32_t rotl32_var(uint32_t v, uint32_t k) { return __builtin_amdgcn_alignbit(v, v, (32u - k) & 31u); }

// The 128 KiB are 8192 chunks of 16 bytes, four copies of one table entry each; chunk c belongs to
// entry (c >> 4) & 255 of table 2 (c >> 12) + ((c >> 3) & 1) (te_r = te_0 rotated by r bytes).
// Thread t writes chunks t, t + blockDim.x, ...: consecutive lanes write consecutive chunks.
__device__ __forceinline__ void fill_tables(uint32_t *lds)
{
    uint4 *dst = reinterpret_cast<uint4 *>(lds);
    for (uint32_t c = threadIdx.x; c < kLdsBytes / 16; c += blockDim.x) {
        const uint32_t table = ((c >> 12) << 1) | ((c >> 3) & 1u);
        const uint32_t t = rotl32_var(c_aes.te0[(c >> 4) & 255u], 8 * table);
        dst[c] = make_uint4(t, t, t, t);
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

// Blocks that encrypt the SAME input under keys that differ in few bytes walk through equal
// state bytes for a while, and equal bytes mean equal lookups.  The three PRG keys differ only
// in their last byte, so after the first AddRoundKey 15 of 16 state bytes coincide, and after
// the second (round key 1 differs in 5 bytes, column 0 has diffused) still 8 of 16.
// shared_lookups(rd, ka, kb): bit 4c + r is set iff, in round rd (1 or 2), the row-r lookup for
// output column c is the same for a block under PRG key ka and one under PRG key kb.
// Derived from the round keys at compile time; no property of the keys is assumed.
constexpr uint32_t rk_byte(int key, int rd, int col, int row) { return (kAes.rk[key][4 * rd + col] >> (8 * row)) & 0xffu; }

constexpr uint32_t shared_lookups(int rd, int ka, int kb)
{
    bool eq[4][4] = {};                       // [col][row]: state bytes equal entering round 1
    for (int col = 0; col < 4; col++)
        for (int row = 0; row < 4; row++) eq[col][row] = rk_byte(ka, 0, col, row) == rk_byte(kb, 0, col, row);
    uint32_t mask = 0;
    for (int step = 1; step <= rd; step++) {
        mask = 0;
        for (int c = 0; c < 4; c++)
            for (int r = 0; r < 4; r++)
                if (eq[(c + r) & 3][r]) mask |= 1u << (4 * c + r);
        // state entering the next round: a column is equal where all four of its lookups were
        // and the next round key agrees
        bool nxt[4][4] = {};
        for (int c = 0; c < 4; c++)
            for (int row = 0; row < 4; row++)
                nxt[c][row] = ((mask >> (4 * c)) & 0xfu) == 0xfu && rk_byte(ka, step, c, row) == rk_byte(kb, step, c, row);
        for (int c = 0; c < 4; c++)
            for (int row = 0; row < 4; row++) eq[c][row] = nxt[c][row];
    }
    return mask;
}

// key id -1 stands for "PRG key 1 or 2, chosen per lane": shared only where both agree
constexpr uint32_t shared_lookups_any(int rd, int ka, int kb)
{
    uint32_t m = 0xffffu;
    for (int a = (ka < 0 ? 0 : ka); a <= (ka < 0 ? 1 : ka); a++)
        for (int b = (kb < 0 ? 0 : kb); b <= (kb < 0 ? 1 : kb); b++) m &= shared_lookups(rd, a, b);
    return m;
}

// What the tree walk reads of G_3(s): words 0 and 1 (sigma^L, sigma^R) and the two low bits of
// byte 8 (tau^L, tau^R), i.e. final-round columns 0 and 1 and the row-0 byte of column 2.
constexpr uint32_t kNeedSigmaTau = 0x01ffu;
constexpr uint32_t kNeedAll = 0xffffu;

static_assert(shared_lookups(1, 0, 2) == 0xfff7u && shared_lookups(1, 1, 2) == 0xfff7u, "round 1: all but the (column 0, row 3) lookup");
static_assert(__builtin_popcount(shared_lookups(2, 0, 2)) == 8 && shared_lookups(3, 0, 2) == 0, "round 2: half; round 3: none");

// Byte addresses of the 16 lookups of one block-round (table immediates not included).  Lookup
// 4c + r is the contribution of the row-r byte to output column c (ShiftRows: it comes from state
// column c + r).  Rounds 1..9 read table r; the last round reads table r + 2, whose byte r is S(v).
// Entries whose bit is set in `skip` are not needed and left untouched.
template <bool LAST>
__device__ __forceinline__ void lookup_addresses(uint32_t (&ad)[16], const uint32_t (&st)[4], uint32_t skip, LaneBase L)
{
    const uint32_t b01 = LAST ? L.b : L.a;   // rows 0,1: tables 0,1 (2,3 in the last round)
    const uint32_t b23 = LAST ? L.a : L.b;   // rows 2,3: tables 2,3 (0,1 in the last round)
#pragma unroll
    for (int c = 0; c < 4; c++) {
        if (!((skip >> (4 * c + 0)) & 1u)) ad[4 * c + 0] = entry_addr<0>(st[c], b01);
        if (!((skip >> (4 * c + 1)) & 1u)) ad[4 * c + 1] = entry_addr<1>(st[(c + 1) & 3], b01);
        if (!((skip >> (4 * c + 2)) & 1u)) ad[4 * c + 2] = entry_addr<2>(st[(c + 2) & 3], b23);
        if (!((skip >> (4 * c + 3)) & 1u)) ad[4 * c + 3] = entry_addr<3>(st[(c + 3) & 3], b23);
    }
}

// s_waitcnt lgkmcnt(0) alone (vmcnt and expcnt fields at their maximum)
__device__ __forceinline__ void wait_lds() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// NB AES-128 encryptions per lane, each followed by the Matyas-Meyer-Oseas feed-forward:
// out[b] = E_{key M_b}(seed[b]) ^ seed[b].  pick[b] (0 or ~0 per lane) is only read by blocks
// whose key is -1.  With SAME_INPUT the caller guarantees seed[b] == seed[0] for every b, and
// blocks b > 0 take the lookups of rounds 1 and 2 that provably equal block 0's from block 0.
// LAST_NEED: which lookups of the final round the caller needs from the LAST block (bit 4c + r);
// output bytes whose lookup is skipped are unspecified.
//
// Schedule.  A wavefront can keep 16 LDS instructions in flight and a round of one block is
// exactly 16 lookups, each round needing the whole previous one, so the unit of work is a
// block-round.  The block-rounds (block 0 round 1, block 1 round 1, ..., block 0 round 2, ...) run
// as a two-stage pipeline: while the lookups of step k are in flight, the wavefront does the
// vector-ALU work of its neighbours -- combining step k-1 into the next state and forming the
// addresses of step k+1 -- and the moment step k's data is back, step k+1's 16 lookups are
// issued from addresses that are already waiting.  The LDS queue of the wavefront is refilled
// immediately after every wait instead of after a combine and 16 address computations.
// (A single block cannot overlap its own rounds; it runs issue / wait / combine.)
template <bool SAME_INPUT, uint32_t LAST_NEED, int... M>
__device__ __forceinline__ void aes_mmo_impl(uint32_t (&out)[sizeof...(M)][4], const uint32_t (&seed)[sizeof...(M)][4],
                                             const uint32_t (&pick)[sizeof...(M)], LaneBase L)
{
    constexpr int NB = sizeof...(M);
    constexpr int keys[NB] = { M... };
    constexpr int STEPS = 10 * NB;
    uint32_t st[NB][4];
    uint32_t lk[2][16];                       // lookups of step k live in lk[k & 1]
    uint32_t ad[16];                          // addresses of the next step to issue
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int c = 0; c < 4; c++) st[b][c] = add_round_key(keys[b], seed[b][c], 0u, c, pick[b]);

    // which lookups of step k are NOT loaded: shared with block 0 (rounds 1, 2) or not needed (last round)
    auto skip_of = [&](int k) constexpr -> uint32_t {
        const int b = k % NB, r = k / NB + 1;
        if (SAME_INPUT && b > 0 && r <= 2) return shared_lookups_any(r, keys[0], keys[b]);
        if (r == 10 && b == NB - 1) return ~LAST_NEED & 0xffffu;
        return 0u;
    };
    auto addresses = [&](int k) {
        const int b = k % NB, r = k / NB + 1;
        if (r == 10) lookup_addresses<true>(ad, st[b], skip_of(k), L);
        else lookup_addresses<false>(ad, st[b], skip_of(k), L);
    };
    auto issue = [&](int k) {
        const int b = k % NB, r = k / NB + 1;
        const uint32_t skip = skip_of(k);
        uint32_t *dst = lk[k & 1];
        const uint32_t *blk0 = lk[(k - b) & 1];   // block 0's lookups of the same round (complete by now)
#pragma unroll
        for (int q = 0; q < 16; q++) {
            if (!((skip >> q) & 1u)) dst[q] = lds_load(ad[q] + ((q & 1) ? kOddTable : 0u));
            else if (r == 10) dst[q] = 0u;
            else dst[q] = blk0[q];
        }
    };
    auto combine = [&](int k) {
        const int b = k % NB, r = k / NB + 1;
        const uint32_t *v = lk[k & 1];
#pragma unroll
        for (int cc = 0; cc < 4; cc++) {
            const int c = 3 - cc;
            if (r < 10) {
                st[b][c] = add_round_key(keys[b], bitop3<kXor3>(v[4 * c], v[4 * c + 1], v[4 * c + 2]), v[4 * c + 3], 4 * r + c, pick[b]);
            } else {
                // last round: SubBytes + ShiftRows only, S(v) = byte r of the row-r lookup
                uint32_t lo = __builtin_amdgcn_perm(v[4 * c + 1], v[4 * c + 0], 0x0c0c0500u);   // l0.b0, l1.b1, 0, 0
                uint32_t hi = __builtin_amdgcn_perm(v[4 * c + 3], v[4 * c + 2], 0x07020c0cu);   // 0, 0, l2.b2, l3.b3
                out[b][c] = add_round_key(keys[b], bitop3<kOrXor>(lo, hi, seed[b][c]), 0u, 40 + c, pick[b]);
            }
        }
    };

    addresses(0);
    issue(0);
    if (NB > 1) addresses(1);
    __builtin_amdgcn_sched_barrier(0);
#pragma clang loop unroll(full)
    for (int k = 0; k < STEPS; k++) {
        wait_lds();                               // step k's lookups are back
        __builtin_amdgcn_sched_barrier(0);
        if (NB > 1 && k + 1 < STEPS) issue(k + 1);
        __builtin_amdgcn_sched_barrier(0);
        combine(k);
        if (NB > 1) {
            if (k + 2 < STEPS) addresses(k + 2);
        } else if (k + 1 < STEPS) {
            addresses(k + 1);
            issue(k + 1);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// independent inputs per block
template <int... M>
__device__ __forceinline__ void aes_mmo(uint32_t (&out)[sizeof...(M)][4], const uint32_t (&seed)[sizeof...(M)][4],
                                        const uint32_t (&pick)[sizeof...(M)], LaneBase L)
{
    aes_mmo_impl<false, 0xffffu, M...>(out, seed, pick, L);
}

// every block expands the same seed (one node of the tree under several PRG keys)
template <uint32_t LAST_NEED, int... M>
__device__ __forceinline__ void aes_mmo_same_input(uint32_t (&out)[sizeof...(M)][4], const uint32_t (&seed)[4],
                                                   const uint32_t (&pick)[sizeof...(M)], LaneBase L)
{
    constexpr int NB = sizeof...(M);
    uint32_t in[NB][4];
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int c = 0; c < 4; c++) in[b][c] = seed[c];
    aes_mmo_impl<true, LAST_NEED, M...>(out, in, pick, L);
}

}  // namespace fss
