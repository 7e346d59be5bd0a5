// HIP kernels (gfx950) for batched FSS key generation and evaluation, and the C ABI of
// include/fss.h on top of them.
//
// One lane walks one element's GGM tree (paper: Algorithms 1-4).  The cost is the PRG:
// AES-128 in Matyas-Meyer-Oseas mode under three fixed keys (section 3.1 "Implementation",
// appendix C.1).  gfx950 has no AES instruction, so AES runs on combined
// SubBytes+MixColumns tables held in LDS:
//   - four tables (one per state row) x 256 entries, each entry replicated 32 times so
//     that lane l always reads bank (l mod 32): lookups with data-dependent indices never
//     collide inside a half-wavefront, whatever the data;
//   - an entry owns 256 bytes: [T_even copy 0..31 | T_odd copy 0..31], tables 0/1 in the
//     first 64 KiB and tables 2/3 in the second.  The byte address of a lookup is then
//     (index << 8) | lane_base, which ONE v_perm_b32 forms straight from a state word
//     (byte k of the word dropped into byte 1 of a per-lane constant);
//   - 128 KiB of the CU's 160 KiB LDS, one 1024-thread workgroup per CU.
// Round keys are compile-time constants.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fss.h"
#include "aes_consts.h"
#include "key_layout.h"

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

// ------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------

__device__ __forceinline__ uint32_t ring_mask(int n) { return n == 32 ? 0xffffffffu : ((1u << n) - 1u); }

struct EvalArgs {
    const uint8_t *key;
    const uint32_t *x;
    uint32_t *out;
    size_t batch;
    int n;
    int party;
};

struct GenArgs {
    const uint32_t *alpha;
    const uint32_t *alpha_r;
    const uint4 *seed0;
    const uint4 *seed1;
    uint8_t *key0;
    uint8_t *key1;
    size_t batch;
    int n;
};

// ------------------------------------------------------------------------------------
// Eval: Algorithm 2 (CMP = false) and Algorithm 4 (CMP = true)
// ------------------------------------------------------------------------------------

template <bool CMP>
__global__ __launch_bounds__(kThreads) void eval_kernel(EvalArgs a)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const KeyLayout k = key_layout(CMP, a.n, a.batch);
    const int n = a.n;
    const uint32_t mask = ring_mask(n);
    const uint4 *seed_p = reinterpret_cast<const uint4 *>(a.key + k.seed);
    const uint4 *scw_p = reinterpret_cast<const uint4 *>(a.key + k.s_cw);
    const uint32_t *sig_p = reinterpret_cast<const uint32_t *>(a.key + k.sigma_cw);
    const uint32_t *leaf_p = reinterpret_cast<const uint32_t *>(a.key + k.leaf);
    const uint32_t *last_p = reinterpret_cast<const uint32_t *>(a.key + k.last);

    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < a.batch; e += stride) {
        uint4 sv = seed_p[e];
        uint32_t s[4] = { sv.x & ~1u, sv.y, sv.z, sv.w };
        uint32_t t = (uint32_t)a.party;                 // t^(1) = j
        uint32_t tcw[2], taucw[2] = { 0, 0 };
        if constexpr (CMP) {
            uint4 c = reinterpret_cast<const uint4 *>(a.key + k.ctrl)[e];
            tcw[0] = c.x; tcw[1] = c.y; taucw[0] = c.z; taucw[1] = c.w;
        } else {
            uint2 c = reinterpret_cast<const uint2 *>(a.key + k.ctrl)[e];
            tcw[0] = c.x; tcw[1] = c.y;
        }
        const uint32_t x = a.x[e] & mask;
        uint32_t acc = 0;

        // correction words are fetched one level ahead of their use
        uint4 scw_next = scw_p[e];
        uint32_t sig_next = 0, leaf_next = 0;
        if constexpr (CMP) { sig_next = sig_p[e]; leaf_next = leaf_p[e]; }
        for (int i = 0; i < n; i++) {                   // level i + 1
            const uint4 scw = scw_next;
            const uint32_t sigcw = sig_next, leaf = leaf_next;
            if (i + 1 < n) {
                const size_t pe = (size_t)(i + 1) * k.bp + e;
                scw_next = scw_p[pe];
                if constexpr (CMP) { sig_next = sig_p[pe]; leaf_next = leaf_p[pe]; }
            }
            const uint32_t b = (x >> (n - 1 - i)) & 1u;  // x[i], most significant first
            const bool right = b != 0;
            const uint32_t pick = 0u - b;                // all ones iff x[i] = 1
            const uint32_t tm = 0u - t;                  // all ones iff t = 1

            uint32_t child[4];
            if constexpr (CMP) {
                uint32_t g[2][4];
                const uint32_t in[2][4] = { { s[0], s[1], s[2], s[3] }, { s[0], s[1], s[2], s[3] } };
                const uint32_t pk[2] = { pick, 0u };
                aes_mmo<-1, 2>(g, in, pk, L);            // G_{1+x[i]}(s) and G_3(s)
                const uint32_t sigma = ((right ? g[1][1] : g[1][0]) ^ (sigcw & tm)) & mask;
                const uint32_t tau = ((g[1][2] >> b) ^ (t & ((right ? taucw[1] : taucw[0]) >> i))) & 1u;
                acc += (tau ? leaf : 0u) + sigma;        // out_i, sign applied at the end
#pragma unroll
                for (int c = 0; c < 4; c++) child[c] = g[0][c];
            } else {
                uint32_t g[1][4];
                const uint32_t in[1][4] = { { s[0], s[1], s[2], s[3] } };
                const uint32_t pk[1] = { pick };
                aes_mmo<-1>(g, in, pk, L);
#pragma unroll
                for (int c = 0; c < 4; c++) child[c] = g[0][c];
            }
            // (s, t) <- state_{x[i]} = G(s) xor t . CW, all gated by the t entering the level
            const uint32_t t_child = child[0] & 1u;
            s[0] = (child[0] & ~1u) ^ (scw.x & tm);
            s[1] = child[1] ^ (scw.y & tm);
            s[2] = child[2] ^ (scw.z & tm);
            s[3] = child[3] ^ (scw.w & tm);
            t = t_child ^ (t & ((right ? tcw[1] : tcw[0]) >> i) & 1u);
        }
        acc += (t ? last_p[e] : 0u) + (s[3] & mask);     // out_{n+1}
        if (a.party) acc = 0u - acc;
        a.out[e] = acc & mask;
    }
}

// ------------------------------------------------------------------------------------
// KeyGen: Algorithm 1 (CMP = false) and Algorithm 3 (CMP = true), shortened correction words
// ------------------------------------------------------------------------------------

template <bool CMP>
__global__ __launch_bounds__(kThreads) void gen_kernel(GenArgs a)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const KeyLayout k = key_layout(CMP, a.n, a.batch);
    const int n = a.n;
    const uint32_t mask = ring_mask(n);

    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < k.bp; e += stride) {
        if (e >= a.batch) {
            // padding elements: defined (zero) contents in every plane
#pragma unroll
            for (int j = 0; j < 2; j++) {
                uint8_t *kb = j == 0 ? a.key0 : a.key1;
                reinterpret_cast<uint32_t *>(kb + k.alpha_share)[e] = 0;
                reinterpret_cast<uint4 *>(kb + k.seed)[e] = make_uint4(0, 0, 0, 0);
                if constexpr (CMP) reinterpret_cast<uint4 *>(kb + k.ctrl)[e] = make_uint4(0, 0, 0, 0);
                else reinterpret_cast<uint2 *>(kb + k.ctrl)[e] = make_uint2(0, 0);
                for (int i = 0; i < n; i++) {
                    const size_t pe = (size_t)i * k.bp + e;
                    reinterpret_cast<uint4 *>(kb + k.s_cw)[pe] = make_uint4(0, 0, 0, 0);
                    if constexpr (CMP) {
                        reinterpret_cast<uint32_t *>(kb + k.sigma_cw)[pe] = 0;
                        reinterpret_cast<uint32_t *>(kb + k.leaf)[pe] = 0;
                    }
                }
                reinterpret_cast<uint32_t *>(kb + k.last)[e] = 0;
            }
            continue;
        }
        const uint32_t alpha = a.alpha[e] & mask;
        const uint32_t r = a.alpha_r[e] & mask;
        uint4 v0 = a.seed0[e], v1 = a.seed1[e];
        uint32_t s[2][4] = { { v0.x & ~1u, v0.y, v0.z, v0.w }, { v1.x & ~1u, v1.y, v1.z, v1.w } };
        uint32_t t[2] = { 0u, 1u };                       // t_j^(1) = j
        uint32_t ctrl[4] = { 0, 0, 0, 0 };

        reinterpret_cast<uint32_t *>(a.key0 + k.alpha_share)[e] = r;
        reinterpret_cast<uint32_t *>(a.key1 + k.alpha_share)[e] = (alpha - r) & mask;
        reinterpret_cast<uint4 *>(a.key0 + k.seed)[e] = make_uint4(s[0][0], s[0][1], s[0][2], s[0][3]);
        reinterpret_cast<uint4 *>(a.key1 + k.seed)[e] = make_uint4(s[1][0], s[1][1], s[1][2], s[1][3]);

        for (int i = 0; i < n; i++) {                     // level i + 1
            const uint32_t abit = (alpha >> (n - 1 - i)) & 1u;   // alpha[i]; Keep = abit, Lose = 1 - abit
            uint32_t g[2][3][4];                          // [party][G_1, G_2, G_3][word]
            if constexpr (CMP) {
                uint32_t h[6][4];
                const uint32_t in[6][4] = { { s[0][0], s[0][1], s[0][2], s[0][3] }, { s[0][0], s[0][1], s[0][2], s[0][3] },
                                            { s[0][0], s[0][1], s[0][2], s[0][3] }, { s[1][0], s[1][1], s[1][2], s[1][3] },
                                            { s[1][0], s[1][1], s[1][2], s[1][3] }, { s[1][0], s[1][1], s[1][2], s[1][3] } };
                const uint32_t pk[6] = { 0, 0, 0, 0, 0, 0 };
                aes_mmo<0, 1, 2, 0, 1, 2>(h, in, pk, L);
#pragma unroll
                for (int j = 0; j < 2; j++)
#pragma unroll
                    for (int m = 0; m < 3; m++)
#pragma unroll
                        for (int c = 0; c < 4; c++) g[j][m][c] = h[3 * j + m][c];
            } else {
                uint32_t h[4][4];
                const uint32_t in[4][4] = { { s[0][0], s[0][1], s[0][2], s[0][3] }, { s[0][0], s[0][1], s[0][2], s[0][3] },
                                            { s[1][0], s[1][1], s[1][2], s[1][3] }, { s[1][0], s[1][1], s[1][2], s[1][3] } };
                const uint32_t pk[4] = { 0, 0, 0, 0 };
                aes_mmo<0, 1, 0, 1>(h, in, pk, L);
#pragma unroll
                for (int j = 0; j < 2; j++)
#pragma unroll
                    for (int c = 0; c < 4; c++) { g[j][0][c] = h[2 * j][c]; g[j][1][c] = h[2 * j + 1][c]; g[j][2][c] = 0; }
            }
            // control bits of the children, and the children with that bit cleared
            uint32_t tL[2], tR[2];
#pragma unroll
            for (int j = 0; j < 2; j++) {
                tL[j] = g[j][0][0] & 1u; g[j][0][0] &= ~1u;
                tR[j] = g[j][1][0] & 1u; g[j][1][0] &= ~1u;
            }
            const uint32_t km = 0u - abit;               // all ones iff Keep = R
            // (s,t) part of CW: the Lose-side string, and bits making t_0^t_1 = 1 on Keep, 0 on Lose
            uint32_t scw[4];
#pragma unroll
            for (int c = 0; c < 4; c++)
                scw[c] = pick32(km, g[0][0][c] ^ g[1][0][c], g[0][1][c] ^ g[1][1][c]);
            const uint32_t tcwL = tL[0] ^ tL[1] ^ abit ^ 1u;
            const uint32_t tcwR = tR[0] ^ tR[1] ^ abit;
            ctrl[0] |= tcwL << i;
            ctrl[1] |= tcwR << i;

            uint32_t sigcw = 0, leaf = 0;
            if constexpr (CMP) {
                // (sigma,tau) part: Keep-side string published, tau_0^tau_1 = 1 on Lose
                const uint32_t sgL0 = g[0][2][0] & mask, sgR0 = g[0][2][1] & mask;
                const uint32_t sgL1 = g[1][2][0] & mask, sgR1 = g[1][2][1] & mask;
                const uint32_t tauL0 = g[0][2][2] & 1u, tauR0 = (g[0][2][2] >> 1) & 1u;
                const uint32_t tauL1 = g[1][2][2] & 1u, tauR1 = (g[1][2][2] >> 1) & 1u;
                sigcw = pick32(km, sgR0 ^ sgR1, sgL0 ^ sgL1);
                const uint32_t taucwL = tauL0 ^ tauL1 ^ abit;
                const uint32_t taucwR = tauR0 ^ tauR1 ^ abit ^ 1u;
                ctrl[2] |= taucwL << i;
                ctrl[3] |= taucwR << i;
                // state'_{j, Lose}
                const uint32_t taucw_lose = pick32(km, taucwL, taucwR);
                const uint32_t sg0 = pick32(km, sgL0, sgR0) ^ (sigcw & (0u - t[0]));
                const uint32_t sg1 = pick32(km, sgL1, sgR1) ^ (sigcw & (0u - t[1]));
                const uint32_t tau1 = pick32(km, tauL1, tauR1) ^ (t[1] & taucw_lose);
                leaf = (abit - sg0 + sg1) & mask;         // (-1)^{tau_1} (alpha[i] - sigma_0 + sigma_1)
                leaf = ((leaf ^ (0u - tau1)) + tau1) & mask;   // negate iff tau_1 = 1
            }
            // both parties move to state_{j, Keep}, corrected with the OLD t_j
            const uint32_t tcw_keep = pick32(km, tcwR, tcwL);
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const uint32_t tm = 0u - t[j];
#pragma unroll
                for (int c = 0; c < 4; c++)
                    s[j][c] = pick32(km, g[j][1][c], g[j][0][c]) ^ (scw[c] & tm);
                t[j] = pick32(km, tR[j], tL[j]) ^ (t[j] & tcw_keep);
            }
            const size_t pe = (size_t)i * k.bp + e;
#pragma unroll
            for (int j = 0; j < 2; j++) {
                reinterpret_cast<uint4 *>((j == 0 ? a.key0 : a.key1) + k.s_cw)[pe] = make_uint4(scw[0], scw[1], scw[2], scw[3]);
                if constexpr (CMP) {
                    reinterpret_cast<uint32_t *>((j == 0 ? a.key0 : a.key1) + k.sigma_cw)[pe] = sigcw;
                    reinterpret_cast<uint32_t *>((j == 0 ? a.key0 : a.key1) + k.leaf)[pe] = leaf;
                }
            }
        }
        // CW^(n+1) = (-1)^{t_1} (1 - conv(s_0) + conv(s_1))
        uint32_t last = (1u - (s[0][3] & mask) + (s[1][3] & mask)) & mask;
        if (t[1]) last = (0u - last) & mask;
#pragma unroll
        for (int j = 0; j < 2; j++) {
            reinterpret_cast<uint32_t *>((j == 0 ? a.key0 : a.key1) + k.last)[e] = last;
            if constexpr (CMP) reinterpret_cast<uint4 *>((j == 0 ? a.key0 : a.key1) + k.ctrl)[e] = make_uint4(ctrl[0], ctrl[1], ctrl[2], ctrl[3]);
            else reinterpret_cast<uint2 *>((j == 0 ? a.key0 : a.key1) + k.ctrl)[e] = make_uint2(ctrl[0], ctrl[1]);
        }
    }
}

// ------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------

static thread_local int g_last_hip_error = 0;

struct DeviceInfo {
    int ok;        // 1 usable, -1 not usable, 0 unknown
    int cus;
};

static int prepare_device(DeviceInfo *info)
{
    // per-device, idempotent: raise the dynamic-LDS limit of the four kernels
    static DeviceInfo cache[64] = {};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) { g_last_hip_error = (int)err; return FSS_ELAUNCH; }
    if (dev < 0 || dev >= 64) return FSS_EDEVICE;
    if (cache[dev].ok == 0) {
        int lds = 0, cus = 0;
        err = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
        if (err == hipSuccess) err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (err != hipSuccess) { g_last_hip_error = (int)err; return FSS_ELAUNCH; }
        if ((uint32_t)lds < kLdsBytes) { cache[dev].ok = -1; g_last_hip_error = 0; return FSS_EDEVICE; }
        const void *fns[4] = { (const void *)eval_kernel<true>, (const void *)eval_kernel<false>,
                               (const void *)gen_kernel<true>, (const void *)gen_kernel<false> };
        for (int i = 0; i < 4; i++) {
            err = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
            if (err != hipSuccess) { g_last_hip_error = (int)err; return FSS_ELAUNCH; }
        }
        cache[dev].cus = cus > 0 ? cus : 256;
        cache[dev].ok = 1;
    }
    if (cache[dev].ok < 0) return FSS_EDEVICE;
    *info = cache[dev];
    return FSS_OK;
}

static bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

static bool bad_n(int n) { return n < 1 || n > 32; }

struct LaunchShape {
    unsigned grid, threads;
};

// One workgroup per CU (its tables take 128 KiB of the CU's LDS).  Large batches: 1024 threads
// per workgroup and a grid-stride loop.  Batches that would leave CUs idle at that size are
// spread over all CUs with fewer wavefronts per workgroup instead.
static LaunchShape shape_for(size_t elems, const DeviceInfo &d)
{
    const size_t cus = (size_t)d.cus;
    size_t threads = (elems + cus - 1) / cus;                  // elements per CU if spread evenly
    threads = (threads + 63) / 64 * 64;
    if (threads < 64) threads = 64;
    if (threads > (size_t)kThreads) threads = kThreads;
    size_t tiles = (elems + threads - 1) / threads;
    LaunchShape s;
    s.threads = (unsigned)threads;
    s.grid = (unsigned)(tiles < cus ? tiles : cus);
    return s;
}

static int check_launch()
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) { g_last_hip_error = (int)err; return FSS_ELAUNCH; }
    return FSS_OK;
}

static int gen_common(bool cmp, int n, size_t batch, const uint32_t *d_alpha, const uint32_t *d_alpha_r,
                      const uint8_t *d_seed0, const uint8_t *d_seed1, void *d_key0, void *d_key1, fss_stream_t stream)
{
    if (bad_n(n)) return FSS_EINVAL;
    if (batch == 0) return FSS_OK;
    if (!d_alpha || !d_alpha_r || !d_seed0 || !d_seed1 || !d_key0 || !d_key1) return FSS_EINVAL;
    if (misaligned(d_alpha, 4) || misaligned(d_alpha_r, 4) || misaligned(d_seed0, 16) || misaligned(d_seed1, 16) ||
        misaligned(d_key0, 256) || misaligned(d_key1, 256))
        return FSS_EINVAL;
    const size_t bytes = key_layout(cmp, n, batch).total;
    const uintptr_t k0 = reinterpret_cast<uintptr_t>(d_key0), k1 = reinterpret_cast<uintptr_t>(d_key1);
    if (k0 < k1 + bytes && k1 < k0 + bytes) return FSS_EINVAL;   // overlapping outputs
    DeviceInfo dev;
    int rc = prepare_device(&dev);
    if (rc != FSS_OK) return rc;
    GenArgs a;
    a.alpha = d_alpha; a.alpha_r = d_alpha_r;
    a.seed0 = reinterpret_cast<const uint4 *>(d_seed0); a.seed1 = reinterpret_cast<const uint4 *>(d_seed1);
    a.key0 = static_cast<uint8_t *>(d_key0); a.key1 = static_cast<uint8_t *>(d_key1);
    a.batch = batch; a.n = n;
    const LaunchShape ls = shape_for(padded_batch(batch), dev);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cmp) hipLaunchKernelGGL(gen_kernel<true>, dim3(ls.grid), dim3(ls.threads), kLdsBytes, st, a);
    else hipLaunchKernelGGL(gen_kernel<false>, dim3(ls.grid), dim3(ls.threads), kLdsBytes, st, a);
    return check_launch();
}

static int eval_common(bool cmp, int party, int n, size_t batch, const void *d_key, const uint32_t *d_x,
                       uint32_t *d_out, fss_stream_t stream)
{
    if (bad_n(n) || (party != 0 && party != 1)) return FSS_EINVAL;
    if (batch == 0) return FSS_OK;
    if (!d_key || !d_x || !d_out) return FSS_EINVAL;
    if (misaligned(d_key, 256) || misaligned(d_x, 4) || misaligned(d_out, 4)) return FSS_EINVAL;
    DeviceInfo dev;
    int rc = prepare_device(&dev);
    if (rc != FSS_OK) return rc;
    EvalArgs a;
    a.key = static_cast<const uint8_t *>(d_key); a.x = d_x; a.out = d_out;
    a.batch = batch; a.n = n; a.party = party;
    const LaunchShape ls = shape_for(batch, dev);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cmp) hipLaunchKernelGGL(eval_kernel<true>, dim3(ls.grid), dim3(ls.threads), kLdsBytes, st, a);
    else hipLaunchKernelGGL(eval_kernel<false>, dim3(ls.grid), dim3(ls.threads), kLdsBytes, st, a);
    return check_launch();
}

}  // namespace fss

extern "C" {

size_t fss_cmp_key_bytes(int n, size_t batch) { return fss::bad_n(n) ? 0 : fss::key_layout(true, n, batch).total; }

size_t fss_eq_key_bytes(int n, size_t batch) { return fss::bad_n(n) ? 0 : fss::key_layout(false, n, batch).total; }

int fss_cmp_gen(int n, size_t batch, const uint32_t *d_alpha, const uint32_t *d_alpha_r, const uint8_t *d_seed0,
                const uint8_t *d_seed1, void *d_key0, void *d_key1, fss_stream_t stream)
{
    return fss::gen_common(true, n, batch, d_alpha, d_alpha_r, d_seed0, d_seed1, d_key0, d_key1, stream);
}

int fss_eq_gen(int n, size_t batch, const uint32_t *d_alpha, const uint32_t *d_alpha_r, const uint8_t *d_seed0,
               const uint8_t *d_seed1, void *d_key0, void *d_key1, fss_stream_t stream)
{
    return fss::gen_common(false, n, batch, d_alpha, d_alpha_r, d_seed0, d_seed1, d_key0, d_key1, stream);
}

int fss_cmp_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_x, uint32_t *d_out,
                 fss_stream_t stream)
{
    return fss::eval_common(true, party, n, batch, d_key, d_x, d_out, stream);
}

int fss_eq_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_x, uint32_t *d_out,
                fss_stream_t stream)
{
    return fss::eval_common(false, party, n, batch, d_key, d_x, d_out, stream);
}

const char *fss_strerror(int code)
{
    switch (code) {
    case FSS_OK: return "success";
    case FSS_EINVAL: return "invalid argument (party, n, NULL/misaligned/overlapping pointer)";
    case FSS_ELAUNCH: return "HIP runtime error while preparing or launching a kernel";
    case FSS_EDEVICE: return "device unsupported: kernels need 128 KiB of LDS per workgroup";
    default: return "unknown fss error code";
    }
}

int fss_last_hip_error(void) { return fss::g_last_hip_error; }

}  // extern "C"
