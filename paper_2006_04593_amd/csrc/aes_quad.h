// The same LDS-table AES as aes_lds.h in a second register layout, for batches too small to fill
// the chip with one element per lane.  Device-only header.
//
// Quad layout: four adjacent lanes share one AES block, lane 4q + c holding state column c (one
// 32-bit word).  A round is then FOUR lookups per lane instead of sixteen -- the row-r byte of the
// lane's own column in table r -- and ShiftRows becomes a rotation inside the quad: output column
// c takes the row-r lookup of lane (c + r) mod 4, which a DPP quad_perm operand delivers for free
// on the XOR that combines it.  A wavefront covers 16 elements instead of 64, so a batch spreads
// over four times as many wavefronts and each wavefront's dependent chain (10 rounds x blocks x
// levels) is four times shorter per step.  The price: round keys differ per lane (one VGPR per
// key and round instead of scalar constants), lookups shared between blocks of one seed can only
// be skipped a whole row at a time, and the tree walk around the PRG is repeated in the four
// lanes.  Throughput on large batches is therefore lower than the lane layout's; latency on small
// ones is much better.
#pragma once
#include "aes_lds.h"

namespace fss {

// DPP quad_perm controls: lane c reads lane (c + k) mod 4 of its quad; lane c reads lane k
constexpr int kQuadRot1 = 1 | (2 << 2) | (3 << 4) | (0 << 6);
constexpr int kQuadRot2 = 2 | (3 << 2) | (0 << 4) | (1 << 6);
constexpr int kQuadRot3 = 3 | (0 << 2) | (1 << 4) | (2 << 6);

template <int CTRL>
__device__ __forceinline__ uint32_t quad_perm(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xf, 0xf, true);
}

template <int K>
__device__ __forceinline__ uint32_t quad_broadcast(uint32_t v) { return quad_perm<K * 0x55>(v); }

// Column (lane & 3) of all eleven round keys of the three PRG keys.
struct QuadKeys {
    uint32_t k[3][11];
};

__device__ __forceinline__ QuadKeys load_quad_keys()
{
    QuadKeys q;
    const uint32_t col = threadIdx.x & 3u;
#pragma unroll
    for (int m = 0; m < 3; m++)
#pragma unroll
        for (int r = 0; r < 11; r++) q.k[m][r] = c_aes.rk[m][4 * r + col];
    return q;
}

// rows (0..3) whose lookup in round rd is the same in EVERY column for blocks under keys ka, kb
constexpr uint32_t shared_rows(int rd, int ka, int kb)
{
    const uint32_t m = shared_lookups_any(rd, ka, kb);
    uint32_t rows = 0;
    for (int r = 0; r < 4; r++) {
        bool all = true;
        for (int c = 0; c < 4; c++) all = all && ((m >> (4 * c + r)) & 1u);
        if (all) rows |= 1u << r;
    }
    return rows;
}

static_assert(shared_rows(1, 0, 2) == 0x7u && shared_rows(1, -1, 2) == 0x7u && shared_rows(3, 0, 2) == 0u,
              "round 1: the three PRG keys differ only in a row-3 byte");

// NB Matyas-Meyer-Oseas blocks per quad: out[b] = column of E_{key M_b}(seed[b]) ^ seed[b].
// Key ids as in aes_mmo_impl: 0..2, or -1 for "PRG key 2 where pick is all ones, else PRG key 1".
// GROUP > 0: blocks come in runs of GROUP that expand the same seed (seed[b] equals the seed of the
// first block of its run); later blocks of a run take the shared rows of rounds 1 and 2 from the
// first.  GROUP = 0: unrelated inputs.
//
// Schedule: the blocks take turns, and a block's turn is "combine my previous round, form the four
// addresses of my next round, issue its lookups".  Between two turns of one block all other
// blocks have theirs, so NB block-rounds (4 NB lookups) are in flight per wavefront.
template <int GROUP, int... M>
__device__ __forceinline__ void aes_mmo_quad(uint32_t (&out)[sizeof...(M)], const uint32_t (&seed)[sizeof...(M)], uint32_t pick,
                                             const QuadKeys &K, LaneBase L)
{
    constexpr int NB = sizeof...(M);
    constexpr int keys[NB] = { M... };
    uint32_t st[NB];
    uint32_t lk[NB][4];
    uint32_t first[GROUP > 0 ? NB / GROUP : 1][4];   // lookups of the first block of each run, kept for the others

    auto round_key = [&](int b, int r) -> uint32_t {
        return keys[b] >= 0 ? K.k[keys[b]][r] : pick32(pick, K.k[1][r], K.k[0][r]);
    };
    auto skip_of = [&](int b, int r) constexpr -> uint32_t {
        if (GROUP > 0 && b % (GROUP > 0 ? GROUP : 1) != 0 && r <= 2) return shared_rows(r, keys[b - b % (GROUP > 0 ? GROUP : 1)], keys[b]);
        return 0u;
    };
    auto issue = [&](int b, int r) {
        const uint32_t skip = skip_of(b, r);
        const uint32_t b01 = r == 10 ? L.b : L.a;     // rows 0,1: tables 0,1 (2,3 in the last round)
        const uint32_t b23 = r == 10 ? L.a : L.b;
        if (!(skip & 1u)) lk[b][0] = lds_load(entry_addr<0>(st[b], b01));
        if (!(skip & 2u)) lk[b][1] = lds_load(entry_addr<1>(st[b], b01) + kOddTable);
        if (!(skip & 4u)) lk[b][2] = lds_load(entry_addr<2>(st[b], b23));
        if (!(skip & 8u)) lk[b][3] = lds_load(entry_addr<3>(st[b], b23) + kOddTable);
    };
    auto combine = [&](int b, int r) {
        uint32_t v[4];
#pragma unroll
        for (int q = 0; q < 4; q++) {
            if ((skip_of(b, r) >> q) & 1u) v[q] = first[GROUP > 0 ? b / (GROUP > 0 ? GROUP : 1) : 0][q];
            else v[q] = lk[b][q];
            if (GROUP > 0 && b % (GROUP > 0 ? GROUP : 1) == 0 && r <= 2) first[b / (GROUP > 0 ? GROUP : 1)][q] = v[q];
        }
        const uint32_t v1 = quad_perm<kQuadRot1>(v[1]), v2 = quad_perm<kQuadRot2>(v[2]), v3 = quad_perm<kQuadRot3>(v[3]);
        if (r < 10) {
            // two independent pairs, then one three-way XOR: no DPP operand waits for a result that a
            // vector instruction has just written (the chain v0 ^ v1 ^ v2 ^ v3 costs two idle cycles per link)
            st[b] = bitop3<kXor3>(v[0] ^ v1, v2 ^ v3, round_key(b, r));
        } else {
            // last round: SubBytes + ShiftRows only, S(x) = byte r of the row-r lookup
            const uint32_t lo = __builtin_amdgcn_perm(v1, v[0], 0x0c0c0500u);
            const uint32_t hi = __builtin_amdgcn_perm(v3, v2, 0x07020c0cu);
            out[b] = bitop3<kOrXor>(lo, hi, seed[b]) ^ round_key(b, 10);
        }
    };

#pragma unroll
    for (int b = 0; b < NB; b++) {
        st[b] = seed[b] ^ round_key(b, 0);
        issue(b, 1);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma clang loop unroll(full)
    for (int r = 1; r <= 10; r++) {
#pragma clang loop unroll(full)
        for (int b = 0; b < NB; b++) {
            combine(b, r);
            if (r < 10) issue(b, r + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

}  // namespace fss
