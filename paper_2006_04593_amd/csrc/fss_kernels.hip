// HIP kernels (gfx950) for batched FSS key generation and evaluation, and the C ABI of
// include/fss.h on top of them.
//
// One lane walks one element's GGM tree (paper: Algorithms 1-4).  The cost is the PRG:
// AES-128 in Matyas-Meyer-Oseas mode under three fixed keys (section 3.1 "Implementation",
// appendix C.1), computed by the LDS-table engine of aes_lds.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <tuple>

#include "../../include/fss.h"
#include "aes_lds.h"
#include "aes_quad.h"
#include "key_layout.h"

namespace fss {

// ------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------

__device__ __forceinline__ uint32_t ring_mask(int n) { return n == 32 ? 0xffffffffu : ((1u << n) - 1u); }

// index of the wavefront inside its workgroup, as a scalar: tile counters derived from it stay in scalar registers
__device__ __forceinline__ uint32_t wave_index() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

// Wavefront priority by progress through the tile.  A SIMD issues from its OLDEST wavefront first,
// so with equal priorities the first wavefront of every SIMD runs at full speed and the youngest
// is starved: they drift a whole tile apart per pass, the old ones finish all their tiles early,
// and the launch ends with a long stretch in which too few wavefronts are left to keep the LDS
// busy (measured: the four wavefronts of a SIMD finish 30 us apart after ONE 64-element tile).
// Lowering a wavefront's priority as it advances (3 in the first half of the walk, then 2, 1, 0
// from n/2, 3n/4 and 7n/8 on) lets the ones behind catch up, so that they finish together.
// Cost: one scalar compare per level (`i == next`), three priority changes per tile.  `balance` is
// false for launches with at most one working wavefront per SIMD, where there is nobody to wait for
// (the level loop of such a launch is pure latency, and even untaken branches count there).
__device__ __forceinline__ int tile_priority_start(int n, bool balance)
{
    if (!balance) return -1;
    __builtin_amdgcn_s_setprio(3);
    return n >> 1;
}

// called when level i has reached the threshold `next`; returns the next threshold
__device__ __forceinline__ int lower_priority(int i, int n)
{
    if (i < n - (n >> 2)) { __builtin_amdgcn_s_setprio(2); return n - (n >> 2); }
    if (i < n - (n >> 3)) { __builtin_amdgcn_s_setprio(1); return n - (n >> 3); }
    __builtin_amdgcn_s_setprio(0);
    return -1;
}

// What the evaluation kernel reads as its public input and writes as its result.
//   kPlain:    x given; out = share of f(x)                                   (Algorithms 2, 4)
//   kSign:     x = x[e] + x2[e] (the two published masked shares)              (Algorithm 5)
//   kReluOpen: as kSign, then the party's messages for the ReLU product: with w the share of
//              1{y <= 0} and v = [party = 0] - w the share of 1{y > 0},
//              out = delta_j = [[y]]_j - [[a]]_j,  out2 = eps_j = v - [[b]]_j   (section 4.2)
enum EvalMode { kPlain = 0, kSign = 1, kReluOpen = 2 };

struct EvalArgs {
    const uint8_t *key;
    const uint32_t *x;
    const uint32_t *x2;        // second masked share (kSign, kReluOpen)
    uint32_t *out;
    uint32_t *out2;            // eps_j (kReluOpen)
    const uint32_t *y_share;   // [[y]]_j (kReluOpen)
    const uint32_t *tri_a;     // [[a]]_j (kReluOpen)
    const uint32_t *tri_b;     // [[b]]_j (kReluOpen)
    size_t batch;
    int n;
    int party;
    size_t lane_tiles;         // eval_kernel: 64-element tiles walked one lane per element, from element 0
    size_t quad_tiles;         // eval_kernel: 16-element tiles walked four lanes per element, after those
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
    size_t lane_tiles;         // gen_kernel: as in EvalArgs; quad_tiles reaches to the end of the padded batch
    size_t quad_tiles;
};

// ------------------------------------------------------------------------------------
// Eval: Algorithm 2 (CMP = false) and Algorithm 4 (CMP = true)
// ------------------------------------------------------------------------------------

struct EvalPlanes {
    const uint4 *seed;
    const uint8_t *ctrl;
    const uint4 *scw;
    const uint32_t *sig, *leaf, *last;
    size_t bp;
};

__device__ __forceinline__ EvalPlanes eval_planes(const EvalArgs &a, const KeyLayout &k)
{
    EvalPlanes p;
    p.seed = reinterpret_cast<const uint4 *>(a.key + k.seed);
    p.ctrl = a.key + k.ctrl;
    p.scw = reinterpret_cast<const uint4 *>(a.key + k.s_cw);
    p.sig = reinterpret_cast<const uint32_t *>(a.key + k.sigma_cw);
    p.leaf = reinterpret_cast<const uint32_t *>(a.key + k.leaf);
    p.last = reinterpret_cast<const uint32_t *>(a.key + k.last);
    p.bp = k.bp;
    return p;
}

// What one lane reads before the first level of its element (one lane per element).
template <bool CMP>
struct LaneInputs {
    uint4 seed;
    uint4 ctrl;                 // t_CW^L, t_CW^R, tau_CW^L, tau_CW^R (equality: the first two)
    uint32_t x;
    uint32_t last;              // CW^(n+1), used after the last level
};

template <bool CMP, int MODE>
__device__ __forceinline__ LaneInputs<CMP> load_lane_inputs(const EvalArgs &a, const EvalPlanes &p, size_t e)
{
    LaneInputs<CMP> in;
    in.seed = p.seed[e];
    if constexpr (CMP) {
        in.ctrl = reinterpret_cast<const uint4 *>(p.ctrl)[e];
    } else {
        const uint2 c = reinterpret_cast<const uint2 *>(p.ctrl)[e];
        in.ctrl = make_uint4(c.x, c.y, 0u, 0u);
    }
    uint32_t xin = a.x[e];
    if constexpr (MODE != kPlain) xin += a.x2[e];        // the reveal: x = alpha + y
    in.x = xin;
    in.last = p.last[e];
    return in;
}

template <int MODE>
__device__ __forceinline__ void store_share(const EvalArgs &a, size_t e, uint32_t acc, uint32_t mask)
{
    if (a.party) acc = 0u - acc;
    acc &= mask;
    if constexpr (MODE == kReluOpen) {
        const uint32_t v = ((a.party ? 0u : 1u) - acc) & mask;     // share of 1{y > 0}
        a.out[e] = (a.y_share[e] - a.tri_a[e]) & mask;
        a.out2[e] = (v - a.tri_b[e]) & mask;
    } else {
        a.out[e] = acc;
    }
}

// The walk of one element by one lane.
template <bool CMP, int MODE>
__device__ __forceinline__ void eval_lane_walk(const EvalArgs &a, const EvalPlanes &p, const LaneBase L, size_t e,
                                               const LaneInputs<CMP> &in)
{
    const int n = a.n;
    const uint32_t mask = ring_mask(n);
    uint32_t s[4] = { in.seed.x & ~1u, in.seed.y, in.seed.z, in.seed.w };
    uint32_t t = (uint32_t)a.party;                 // t^(1) = j
    const uint32_t tcw[2] = { in.ctrl.x, in.ctrl.y }, taucw[2] = { in.ctrl.z, in.ctrl.w };
    const uint32_t x = in.x & mask;
    uint32_t acc = 0;

    int next_drop = tile_priority_start(n, true);
    for (int i = 0; i < n; i++) {                   // level i + 1
        if (i == next_drop) next_drop = lower_priority(i, n);
        // The level's correction words are requested here and used after its AES blocks, which at the
        // occupancy this layout runs at take several HBM round trips (fetching a level ahead instead
        // costs twelve register moves a level to rotate "next" into "current").
        const size_t pe = (size_t)i * p.bp + e;
        const uint4 scw = p.scw[pe];
        uint32_t sigcw = 0, leaf = 0;
        if constexpr (CMP) { sigcw = p.sig[pe]; leaf = p.leaf[pe]; }
        const uint32_t b = (x >> (n - 1 - i)) & 1u;  // x[i], most significant first
        const bool right = b != 0;
        const uint32_t pick = 0u - b;                // all ones iff x[i] = 1
        const uint32_t tm = 0u - t;                  // all ones iff t = 1

        uint32_t child[4];
        if constexpr (CMP) {
            uint32_t g[2][4];
            const uint32_t pk[2] = { pick, 0u };
            aes_mmo_same_input<kNeedSigmaTau, -1, 2>(g, s, pk, L);  // G_{1+x[i]}(s) and G_3(s)
            const uint32_t sigma = ((right ? g[1][1] : g[1][0]) ^ (sigcw & tm)) & mask;
            const uint32_t tau = ((g[1][2] >> b) ^ (t & ((right ? taucw[1] : taucw[0]) >> i))) & 1u;
            acc += (tau ? leaf : 0u) + sigma;        // out_i, sign applied at the end
#pragma unroll
            for (int c = 0; c < 4; c++) child[c] = g[0][c];
        } else {
            uint32_t g[1][4];
            const uint32_t sin[1][4] = { { s[0], s[1], s[2], s[3] } };
            const uint32_t pk[1] = { pick };
            aes_mmo<-1>(g, sin, pk, L);
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
    acc += (t ? in.last : 0u) + (s[3] & mask);       // out_{n+1}
    store_share<MODE>(a, e, acc, mask);
}

// The same walk with four lanes per element (quad layout of aes_quad.h): lane 4q + c owns word c of
// the element's seed and of its seed-sized correction words; the scalar pieces of the walk (t,
// sigma, tau, the accumulator) are kept in all four lanes and lane 4q writes the result.
template <bool CMP, int MODE, bool BALANCE>
__device__ __forceinline__ void eval_quad_walk(const EvalArgs &a, const EvalPlanes &p, const LaneBase L, const QuadKeys &K,
                                               size_t e, uint32_t col)
{
    const int n = a.n;
    const uint32_t mask = ring_mask(n);
    const uint32_t keep = col == 0 ? ~1u : ~0u;           // clears the control bit, which lives in column 0
    const uint32_t *seed_w = reinterpret_cast<const uint32_t *>(p.seed);
    const uint32_t *scw_w = reinterpret_cast<const uint32_t *>(p.scw);
    uint32_t s = seed_w[4 * e + col] & keep;
    uint32_t t = (uint32_t)a.party;
    uint32_t tcw[2], taucw[2] = { 0, 0 };
    if constexpr (CMP) {
        const uint4 c = reinterpret_cast<const uint4 *>(p.ctrl)[e];
        tcw[0] = c.x; tcw[1] = c.y; taucw[0] = c.z; taucw[1] = c.w;
    } else {
        const uint2 c = reinterpret_cast<const uint2 *>(p.ctrl)[e];
        tcw[0] = c.x; tcw[1] = c.y;
    }
    uint32_t xin = a.x[e];
    if constexpr (MODE != kPlain) xin += a.x2[e];
    const uint32_t x = xin & mask;
    uint32_t acc = 0;

    uint32_t scw_next = scw_w[4 * e + col];
    uint32_t sig_next = 0, leaf_next = 0;
    if constexpr (CMP) { sig_next = p.sig[e]; leaf_next = p.leaf[e]; }
    int next_drop = tile_priority_start(n, BALANCE);
    for (int i = 0; i < n; i++) {
        if constexpr (BALANCE) {
            if (i == next_drop) next_drop = lower_priority(i, n);
        }
        const uint32_t scw = scw_next, sigcw = sig_next, leaf = leaf_next;
        if (i + 1 < n) {
            const size_t pe = (size_t)(i + 1) * p.bp + e;
            scw_next = scw_w[4 * pe + col];
            if constexpr (CMP) { sig_next = p.sig[pe]; leaf_next = p.leaf[pe]; }
        }
        const uint32_t b = (x >> (n - 1 - i)) & 1u;
        const bool right = b != 0;
        const uint32_t pick = 0u - b;
        const uint32_t tm = 0u - t;
        uint32_t child;
        if constexpr (CMP) {
            uint32_t g[2];
            const uint32_t sin[2] = { s, s };
            aes_mmo_quad<2, -1, 2>(g, sin, pick, K, L);             // G_{1+x[i]}(s) and G_3(s)
            const uint32_t sigL = quad_broadcast<0>(g[1]), sigR = quad_broadcast<1>(g[1]), w2 = quad_broadcast<2>(g[1]);
            const uint32_t sigma = ((right ? sigR : sigL) ^ (sigcw & tm)) & mask;
            const uint32_t tau = ((w2 >> b) ^ (t & ((right ? taucw[1] : taucw[0]) >> i))) & 1u;
            acc += (tau ? leaf : 0u) + sigma;
            child = g[0];
        } else {
            uint32_t g[1];
            const uint32_t sin[1] = { s };
            aes_mmo_quad<0, -1>(g, sin, pick, K, L);
            child = g[0];
        }
        const uint32_t t_child = quad_broadcast<0>(child) & 1u;
        s = (child & keep) ^ (scw & tm);
        t = t_child ^ (t & ((right ? tcw[1] : tcw[0]) >> i) & 1u);
    }
    acc += (t ? p.last[e] : 0u) + (quad_broadcast<3>(s) & mask);
    if (col == 0) store_share<MODE>(a, e, acc, mask);
}

// Comparison Eval with EIGHT lanes per element, for the smallest batches.  With four lanes per
// element a wavefront issues the lookups, combines and addresses of both blocks of a level (26
// instructions per AES round), and while it is the only wavefront on its SIMD that issue stream,
// not the LDS round trip, is what a round costs (measured: 164 clocks per round for two blocks in
// one wavefront, 124 for one block each in two wavefronts of a SIMD).  Here the two blocks of a
// level sit on two quads of different halves of a 16-lane row -- lanes 0-3 / 4-7 of a row walk the
// x[i] child of elements 2r / 2r + 1, lanes 8-11 / 12-15 their sigma/tau block -- so a wavefront
// covers 8 elements, there are twice as many wavefronts, and each issues half as much per round.
// One DPP row rotation by 8 per level hands each quad the other one's block; from there both
// quads carry the same walk, and lane 0 of the child quad writes the result.
struct OctoKeys {
    QuadKeys q;      // q.k[0], q.k[1]: PRG keys 1 and 2 (child quad) or PRG key 3 twice (sigma/tau quad); q.k[2] unused
};

__device__ __forceinline__ OctoKeys load_octo_keys(uint32_t col, uint32_t half)
{
    OctoKeys o;
#pragma unroll
    for (int r = 0; r < 11; r++) {
        o.q.k[0][r] = c_aes.rk[half ? 2 : 0][4 * r + col];
        o.q.k[1][r] = c_aes.rk[half ? 2 : 1][4 * r + col];
        o.q.k[2][r] = 0;
    }
    return o;
}

// lane i of a 16-lane row reads lane (i + 8) mod 16
__device__ __forceinline__ uint32_t row_swap_halves(uint32_t v) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xf, 0xf, true); }

template <int MODE, bool BALANCE>
__device__ __forceinline__ void eval_octo_walk(const EvalArgs &a, const EvalPlanes &p, const LaneBase L, const OctoKeys &K, size_t e,
                                               uint32_t col, uint32_t half)
{
    const int n = a.n;
    const uint32_t mask = ring_mask(n);
    const uint32_t keep = col == 0 ? ~1u : ~0u;
    const uint32_t hm = 0u - half;                        // all ones in the sigma/tau quad
    const uint32_t *seed_w = reinterpret_cast<const uint32_t *>(p.seed);
    const uint32_t *scw_w = reinterpret_cast<const uint32_t *>(p.scw);
    uint32_t s = seed_w[4 * e + col] & keep;
    uint32_t t = (uint32_t)a.party;
    const uint4 c = reinterpret_cast<const uint4 *>(p.ctrl)[e];
    const uint32_t tcw[2] = { c.x, c.y }, taucw[2] = { c.z, c.w };
    uint32_t xin = a.x[e];
    if constexpr (MODE != kPlain) xin += a.x2[e];
    const uint32_t x = xin & mask;
    uint32_t acc = 0;

    uint32_t scw_next = scw_w[4 * e + col];
    uint32_t sig_next = p.sig[e], leaf_next = p.leaf[e];
    int next_drop = tile_priority_start(n, BALANCE);
    for (int i = 0; i < n; i++) {
        if constexpr (BALANCE) {
            if (i == next_drop) next_drop = lower_priority(i, n);
        }
        const uint32_t scw = scw_next, sigcw = sig_next, leaf = leaf_next;
        if (i + 1 < n) {
            const size_t pe = (size_t)(i + 1) * p.bp + e;
            scw_next = scw_w[4 * pe + col];
            sig_next = p.sig[pe]; leaf_next = p.leaf[pe];
        }
        const uint32_t b = (x >> (n - 1 - i)) & 1u;
        const bool right = b != 0;
        const uint32_t tm = 0u - t;
        uint32_t g[1];
        const uint32_t sin[1] = { s };
        aes_mmo_quad<0, -1>(g, sin, 0u - b, K.q, L);       // child quad: G_{1+x[i]}(s); sigma/tau quad: G_3(s)
        const uint32_t other = row_swap_halves(g[0]);
        const uint32_t child = pick32(hm, other, g[0]);    // both quads now hold both blocks
        const uint32_t w = pick32(hm, g[0], other);
        const uint32_t sigL = quad_broadcast<0>(w), sigR = quad_broadcast<1>(w), w2 = quad_broadcast<2>(w);
        const uint32_t sigma = ((right ? sigR : sigL) ^ (sigcw & tm)) & mask;
        const uint32_t tau = ((w2 >> b) ^ (t & ((right ? taucw[1] : taucw[0]) >> i))) & 1u;
        acc += (tau ? leaf : 0u) + sigma;
        const uint32_t t_child = quad_broadcast<0>(child) & 1u;
        s = (child & keep) ^ (scw & tm);
        t = t_child ^ (t & ((right ? tcw[1] : tcw[0]) >> i) & 1u);
    }
    acc += (t ? p.last[e] : 0u) + (quad_broadcast<3>(s) & mask);
    if (col == 0 && half == 0) store_share<MODE>(a, e, acc, mask);
}

template <int MODE, bool BALANCE>
__global__ __launch_bounds__(kThreads) void eval_octo_kernel(EvalArgs a)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const uint32_t lane = threadIdx.x & 63u, col = lane & 3u, half = (lane >> 3) & 1u;
    const OctoKeys K = load_octo_keys(col, half);
    const KeyLayout k = key_layout(true, a.n, a.batch);
    const EvalPlanes p = eval_planes(a, k);
    const size_t tiles = (a.batch + 7) / 8;
    const size_t stride = (size_t)(blockDim.x >> 6) * gridDim.x;
    for (size_t tile = (size_t)wave_index() * gridDim.x + blockIdx.x; tile < tiles; tile += stride) {
        const size_t e = tile * 8 + (lane >> 4) * 2 + ((lane >> 2) & 1u);
        if (e < a.batch) eval_octo_walk<MODE, BALANCE>(a, p, L, K, e, col, half);     // both quads of an element drop out together
    }
}

// Batches from the layout switch on.  Elements [0, 64 lane_tiles) are walked one lane per element:
// the unit of work is a 64-element tile per wavefront, and tile (p W + w) G + g goes to wavefront w
// of workgroup g in pass p (G workgroups of W wavefronts), so that every workgroup holds the same
// number of tiles.  The elements behind them -- a short rest after the last full pass and the last,
// partial row of tiles, as the host's split_work decides -- come as quad_tiles tiles of 16 elements,
// walked four lanes per element by the same wavefronts (four times the wavefronts, a quarter of
// the dependent chain each).
template <bool CMP, int MODE>
__global__ __launch_bounds__(kThreads) void eval_kernel(EvalArgs a)
{
    extern __shared__ uint32_t lds[];
    const KeyLayout k = key_layout(CMP, a.n, a.batch);
    const EvalPlanes p = eval_planes(a, k);
    const uint32_t lane = threadIdx.x & 63u;
    const size_t stride = (size_t)(blockDim.x >> 6) * gridDim.x;
    const size_t slot = (size_t)wave_index() * gridDim.x + blockIdx.x;

    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);

    for (size_t tile = slot; tile < a.lane_tiles; tile += stride) {
        const size_t e = tile * 64 + lane;
        if (e < a.batch) eval_lane_walk<CMP, MODE>(a, p, L, e, load_lane_inputs<CMP, MODE>(a, p, e));
    }

    if (a.quad_tiles != 0) {
        const QuadKeys K = load_quad_keys();
        const size_t first = a.lane_tiles * 64;
        // dealt from the first wavefront that has no 64-element tile in the last, partial pass
        const size_t used = a.lane_tiles % stride;
        for (size_t q = slot >= used ? slot - used : slot + stride - used; q < a.quad_tiles; q += stride) {
            const size_t qe = first + q * 16 + (lane >> 2);
            if (qe < a.batch) eval_quad_walk<CMP, MODE, true>(a, p, L, K, qe, threadIdx.x & 3u);   // whole quads drop out together
        }
    }
}

// Batches below the layout switch: every element four lanes wide, 16-element tiles dealt to
// wavefronts like the 64-element tiles above.  BALANCE: some SIMD has more than one working wavefront.
template <bool CMP, int MODE, bool BALANCE>
__global__ __launch_bounds__(kThreads) void eval_quad_kernel(EvalArgs a)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const QuadKeys K = load_quad_keys();
    const KeyLayout k = key_layout(CMP, a.n, a.batch);
    const EvalPlanes p = eval_planes(a, k);
    const size_t tiles = (a.batch + 15) / 16;
    const size_t stride = (size_t)(blockDim.x >> 6) * gridDim.x;
    for (size_t tile = (size_t)wave_index() * gridDim.x + blockIdx.x; tile < tiles; tile += stride) {
        const size_t e = tile * 16 + ((threadIdx.x & 63u) >> 2);
        if (e < a.batch) eval_quad_walk<CMP, MODE, BALANCE>(a, p, L, K, e, threadIdx.x & 3u);
    }
}

// [[y]]_j + [[alpha]]_j: the value party j publishes in the Sign protocol (Algorithm 5)
__global__ void sign_mask_kernel(const uint32_t *alpha_share, const uint32_t *y_share, uint32_t *masked, size_t batch, uint32_t mask)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < batch; e += stride)
        masked[e] = (y_share[e] + alpha_share[e]) & mask;
}

// Algorithm 6, first loop before the reveal: masked share of x_i - x_j for every ordered pair
// (j, i), i != j, of every row.  e = (r m + j)(m - 1) + t with i = t for t < j, else t + 1.
__global__ void argmax_diff_mask_kernel(const uint32_t *alpha_share, const uint32_t *x_share, uint32_t *masked, size_t rows,
                                        uint32_t m, uint32_t mask)
{
    const size_t total = rows * m * (m - 1);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const size_t rj = e / (m - 1);
        const uint32_t t = (uint32_t)(e - rj * (m - 1));
        const size_t r = rj / m;
        const uint32_t j = (uint32_t)(rj - r * m);
        const uint32_t i = t < j ? t : t + 1;
        masked[e] = (x_share[r * m + i] - x_share[r * m + j] + alpha_share[e]) & mask;
    }
}

// Algorithm 6 between the loops: [[s_j]] = sum of the m - 1 comparison shares of (r, j), then the
// masked share of s_j - (m - 1) under the equality key of (r, j)
__global__ void argmax_count_mask_kernel(const uint32_t *alpha_share, const uint32_t *w_share, uint32_t *masked, size_t count,
                                         uint32_t m, uint32_t mask, int party)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
        uint32_t sum = party == 0 ? 0u - (m - 1) : 0u;
        for (uint32_t t = 0; t < m - 1; t++) sum += w_share[e * (m - 1) + t];
        masked[e] = (sum + alpha_share[e]) & mask;
    }
}

// Algorithm 7, unrolling: one row of k*k shares per k x k window (stride s, no padding)
__global__ void maxpool_unroll_kernel(const uint32_t *x_share, uint32_t *rows_out, size_t channels, int h, int w, int k, int s,
                                      int oh, int ow)
{
    const size_t total = channels * (size_t)oh * ow * k * k;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        size_t q = e;
        const int dx = (int)(q % k); q /= k;
        const int dy = (int)(q % k); q /= k;
        const int ox = (int)(q % ow); q /= ow;
        const int oy = (int)(q % oh); q /= oh;
        rows_out[e] = x_share[(q * h + (size_t)(oy * s + dy)) * w + (size_t)(ox * s + dx)];
    }
}

// messages of a pointwise product with multiplication triples (section 4.2)
__global__ void mul_open_kernel(const uint32_t *u, const uint32_t *v, const uint32_t *ta, const uint32_t *tb, uint32_t *delta,
                                uint32_t *eps, size_t count, uint32_t mask)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
        delta[e] = (u[e] - ta[e]) & mask;
        eps[e] = (v[e] - tb[e]) & mask;
    }
}

// inner product of Algorithm 7: one output per row of m products
__global__ void dot_finish_kernel(const uint32_t *d0, const uint32_t *d1, const uint32_t *e0, const uint32_t *e1,
                                  const uint32_t *ta, const uint32_t *tb, const uint32_t *tc, uint32_t *out, size_t rows,
                                  uint32_t m, uint32_t mask, int party)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t r = (size_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += stride) {
        uint32_t acc = 0;
        for (uint32_t i = 0; i < m; i++) {
            const size_t e = r * m + i;
            const uint32_t delta = d0[e] + d1[e], eps = e0[e] + e1[e];
            acc += delta * tb[e] + eps * ta[e] + tc[e];
            if (party == 0) acc += delta * eps;
        }
        out[r] = acc & mask;
    }
}

// [[u.v]]_j = delta.[[b]]_j + eps.[[a]]_j + [[c]]_j (+ delta.eps for party 0), section 4.2
__global__ void relu_finish_kernel(const uint32_t *d0, const uint32_t *d1, const uint32_t *e0, const uint32_t *e1,
                                   const uint32_t *ta, const uint32_t *tb, const uint32_t *tc, uint32_t *out,
                                   size_t batch, uint32_t mask, int party)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < batch; e += stride) {
        const uint32_t delta = d0[e] + d1[e], eps = e0[e] + e1[e];
        uint32_t z = delta * tb[e] + eps * ta[e] + tc[e];
        if (party == 0) z += delta * eps;
        out[e] = z & mask;
    }
}

// One wavefront that sleeps for `iterations` x 8128 shader clocks and reports how many shader clocks
// and how many ticks of the constant-rate wall clock went by: their ratio is the clock the chip
// sustains under whatever runs beside it.  (s_sleep keeps the wavefront off the execution units.)
__global__ void clock_probe_kernel(unsigned long long *ticks, uint32_t iterations)
{
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (uint32_t i = 0; i < iterations; i++) __builtin_amdgcn_s_sleep(127);
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0) { ticks[0] = c1 - c0; ticks[1] = w1 - w0; }
}

// ------------------------------------------------------------------------------------
// KeyGen: Algorithm 1 (CMP = false) and Algorithm 3 (CMP = true), shortened correction words
// ------------------------------------------------------------------------------------

// padding elements (batch <= e < padded batch): defined (zero) contents in every plane of both keys
template <bool CMP>
__device__ __forceinline__ void zero_padding_element(uint8_t *key0, uint8_t *key1, const KeyLayout &k, size_t e, int n)
{
#pragma unroll
    for (int j = 0; j < 2; j++) {
        uint8_t *kb = j == 0 ? key0 : key1;
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
}

// KeyGen of one element by one lane.
template <bool CMP>
__device__ __forceinline__ void gen_lane_walk(const GenArgs &a, const KeyLayout &k, const LaneBase L, size_t e)
{
    const int n = a.n;
    const uint32_t mask = ring_mask(n);
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

    int next_drop = tile_priority_start(n, true);
    for (int i = 0; i < n; i++) {                     // level i + 1
        if (i == next_drop) next_drop = lower_priority(i, n);
        const uint32_t abit = (alpha >> (n - 1 - i)) & 1u;   // alpha[i]; Keep = abit, Lose = 1 - abit
        uint32_t g[2][3][4];                          // [party][G_1, G_2, G_3][word]
        if constexpr (CMP) {
#pragma unroll
            for (int j = 0; j < 2; j++) {
                uint32_t h[3][4];
                const uint32_t pk[3] = { 0, 0, 0 };
                aes_mmo_same_input<kNeedSigmaTau, 0, 1, 2>(h, s[j], pk, L);
#pragma unroll
                for (int m = 0; m < 3; m++)
#pragma unroll
                    for (int c = 0; c < 4; c++) g[j][m][c] = h[m][c];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 2; j++) {
                uint32_t h[2][4];
                const uint32_t pk[2] = { 0, 0 };
                aes_mmo_same_input<kNeedAll, 0, 1>(h, s[j], pk, L);
#pragma unroll
                for (int c = 0; c < 4; c++) { g[j][0][c] = h[0][c]; g[j][1][c] = h[1][c]; g[j][2][c] = 0; }
            }
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

// KeyGen with four lanes per key pair (quad layout of aes_quad.h): lane 4q + c owns word c of
// both parties' seeds and of the seed-sized correction word; all six PRG blocks of a level (three
// per party) are in flight together.
template <bool CMP, bool BALANCE>
__device__ __forceinline__ void gen_quad_walk(const GenArgs &a, const KeyLayout &k, const LaneBase L, const QuadKeys &K, size_t e,
                                              uint32_t col)
{
    const int n = a.n;
    const uint32_t mask = ring_mask(n);
    const uint32_t keep = col == 0 ? ~1u : ~0u;
    uint8_t *const my_key = (col & 1u) ? a.key1 : a.key0;   // scalar planes: lanes 0,2 write k_0, lanes 1,3 write k_1
    const uint32_t *seed0_w = reinterpret_cast<const uint32_t *>(a.seed0);
    const uint32_t *seed1_w = reinterpret_cast<const uint32_t *>(a.seed1);
    const uint32_t alpha = a.alpha[e] & mask;
    const uint32_t r = a.alpha_r[e] & mask;
    uint32_t s[2] = { seed0_w[4 * e + col] & keep, seed1_w[4 * e + col] & keep };
    uint32_t t[2] = { 0u, 1u };
    uint32_t ctrl[4] = { 0, 0, 0, 0 };
    reinterpret_cast<uint32_t *>(a.key0 + k.seed)[4 * e + col] = s[0];
    reinterpret_cast<uint32_t *>(a.key1 + k.seed)[4 * e + col] = s[1];

    int next_drop = tile_priority_start(n, BALANCE);
    for (int i = 0; i < n; i++) {
        if constexpr (BALANCE) {
            if (i == next_drop) next_drop = lower_priority(i, n);
        }
        const uint32_t abit = (alpha >> (n - 1 - i)) & 1u;
        uint32_t g[2][3];                             // [party][G_1, G_2, G_3], this lane's column
        if constexpr (CMP) {
            uint32_t h[6];
            const uint32_t in[6] = { s[0], s[0], s[0], s[1], s[1], s[1] };
            aes_mmo_quad<3, 0, 1, 2, 0, 1, 2>(h, in, 0u, K, L);
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int m = 0; m < 3; m++) g[j][m] = h[3 * j + m];
        } else {
            uint32_t h[4];
            const uint32_t in[4] = { s[0], s[0], s[1], s[1] };
            aes_mmo_quad<2, 0, 1, 0, 1>(h, in, 0u, K, L);
#pragma unroll
            for (int j = 0; j < 2; j++) { g[j][0] = h[2 * j]; g[j][1] = h[2 * j + 1]; g[j][2] = 0; }
        }
        uint32_t tL[2], tR[2];
#pragma unroll
        for (int j = 0; j < 2; j++) {
            tL[j] = quad_broadcast<0>(g[j][0]) & 1u; g[j][0] &= keep;
            tR[j] = quad_broadcast<0>(g[j][1]) & 1u; g[j][1] &= keep;
        }
        const uint32_t km = 0u - abit;
        const uint32_t scw = pick32(km, g[0][0] ^ g[1][0], g[0][1] ^ g[1][1]);
        const uint32_t tcwL = tL[0] ^ tL[1] ^ abit ^ 1u;
        const uint32_t tcwR = tR[0] ^ tR[1] ^ abit;
        ctrl[0] |= tcwL << i;
        ctrl[1] |= tcwR << i;

        uint32_t sigcw = 0, leaf = 0;
        if constexpr (CMP) {
            const uint32_t sgL0 = quad_broadcast<0>(g[0][2]) & mask, sgR0 = quad_broadcast<1>(g[0][2]) & mask;
            const uint32_t sgL1 = quad_broadcast<0>(g[1][2]) & mask, sgR1 = quad_broadcast<1>(g[1][2]) & mask;
            const uint32_t w0 = quad_broadcast<2>(g[0][2]), w1 = quad_broadcast<2>(g[1][2]);
            const uint32_t tauL0 = w0 & 1u, tauR0 = (w0 >> 1) & 1u;
            const uint32_t tauL1 = w1 & 1u, tauR1 = (w1 >> 1) & 1u;
            sigcw = pick32(km, sgR0 ^ sgR1, sgL0 ^ sgL1);
            const uint32_t taucwL = tauL0 ^ tauL1 ^ abit;
            const uint32_t taucwR = tauR0 ^ tauR1 ^ abit ^ 1u;
            ctrl[2] |= taucwL << i;
            ctrl[3] |= taucwR << i;
            const uint32_t taucw_lose = pick32(km, taucwL, taucwR);
            const uint32_t sg0 = pick32(km, sgL0, sgR0) ^ (sigcw & (0u - t[0]));
            const uint32_t sg1 = pick32(km, sgL1, sgR1) ^ (sigcw & (0u - t[1]));
            const uint32_t tau1 = pick32(km, tauL1, tauR1) ^ (t[1] & taucw_lose);
            leaf = (abit - sg0 + sg1) & mask;
            leaf = ((leaf ^ (0u - tau1)) + tau1) & mask;
        }
        const uint32_t tcw_keep = pick32(km, tcwR, tcwL);
#pragma unroll
        for (int j = 0; j < 2; j++) {
            s[j] = pick32(km, g[j][1], g[j][0]) ^ (scw & (0u - t[j]));
            t[j] = pick32(km, tR[j], tL[j]) ^ (t[j] & tcw_keep);
        }
        const size_t pe = (size_t)i * k.bp + e;
        reinterpret_cast<uint32_t *>(a.key0 + k.s_cw)[4 * pe + col] = scw;
        reinterpret_cast<uint32_t *>(a.key1 + k.s_cw)[4 * pe + col] = scw;
        if constexpr (CMP) {
            // one store for the four scalar words: lanes 0,1 sigma_CW of k_0, k_1; lanes 2,3 CW_leaf of k_0, k_1
            reinterpret_cast<uint32_t *>(my_key + ((col & 2u) ? k.leaf : k.sigma_cw))[pe] = (col & 2u) ? leaf : sigcw;
        }
    }
    const uint32_t c0 = quad_broadcast<3>(s[0]) & mask, c1 = quad_broadcast<3>(s[1]) & mask;
    uint32_t last = (1u - c0 + c1) & mask;
    if (t[1]) last = (0u - last) & mask;
    // lanes 0,1: [[alpha]]_0, [[alpha]]_1; lanes 2,3: CW^(n+1) of k_0, k_1
    const uint32_t share = (col & 1u) ? ((alpha - r) & mask) : r;
    reinterpret_cast<uint32_t *>(my_key + ((col & 2u) ? k.last : k.alpha_share))[e] = (col & 2u) ? last : share;
    if constexpr (CMP) {
        const uint32_t cw = col == 0 ? ctrl[0] : col == 1 ? ctrl[1] : col == 2 ? ctrl[2] : ctrl[3];
        reinterpret_cast<uint32_t *>(a.key0 + k.ctrl)[4 * e + col] = cw;
        reinterpret_cast<uint32_t *>(a.key1 + k.ctrl)[4 * e + col] = cw;
    } else if (col < 2) {
        const uint32_t cw = col == 0 ? ctrl[0] : ctrl[1];
        reinterpret_cast<uint32_t *>(a.key0 + k.ctrl)[2 * e + col] = cw;
        reinterpret_cast<uint32_t *>(a.key1 + k.ctrl)[2 * e + col] = cw;
    }
}

// KeyGen with EIGHT lanes per key pair, for the smallest batches: one quad per PARTY.  With four
// lanes per pair a wavefront carries all six PRG blocks of a level, 78 instructions per AES round
// which a lone wavefront issues at about 5 clocks apiece; split by party, two wavefronts of a
// SIMD issue 39 each and interleave.  Lanes 0-3 / 4-7 of a 16-lane row are party 0 of pairs
// 2r / 2r + 1, lanes 8-11 / 12-15 party 1 (as in eval_octo_walk); a quad expands its own
// party's seed, one DPP row rotation by 8 per block hands it the other party's three blocks, the
// correction words (symmetric in the parties) are formed in both quads, and each quad writes its own
// party's key.
template <bool CMP, bool BALANCE>
__device__ __forceinline__ void gen_octo_walk(const GenArgs &a, const KeyLayout &k, const LaneBase L, const QuadKeys &K, size_t e,
                                              uint32_t col, uint32_t half)
{
    const int n = a.n;
    const uint32_t mask = ring_mask(n);
    const uint32_t keep = col == 0 ? ~1u : ~0u;
    const uint32_t hm = 0u - half;                           // all ones in party 1's quad
    uint8_t *const key = half ? a.key1 : a.key0;
    const uint32_t alpha = a.alpha[e] & mask;
    const uint32_t r = a.alpha_r[e] & mask;
    uint32_t s = reinterpret_cast<const uint32_t *>(half ? a.seed1 : a.seed0)[4 * e + col] & keep;
    uint32_t t_mine = half, t_other = half ^ 1u;             // t_j^(1) = j
    uint32_t ctrl[4] = { 0, 0, 0, 0 };
    reinterpret_cast<uint32_t *>(key + k.seed)[4 * e + col] = s;

    int next_drop = tile_priority_start(n, BALANCE);
    for (int i = 0; i < n; i++) {
        if constexpr (BALANCE) {
            if (i == next_drop) next_drop = lower_priority(i, n);
        }
        const uint32_t abit = (alpha >> (n - 1 - i)) & 1u;
        uint32_t h[3] = { 0, 0, 0 }, o[3] = { 0, 0, 0 };       // G_1, G_2, G_3 of my party's seed / of the other party's, this lane's column
        if constexpr (CMP) {
            const uint32_t in[3] = { s, s, s };
            aes_mmo_quad<3, 0, 1, 2>(h, in, 0u, K, L);
        } else {
            uint32_t h2[2];
            const uint32_t in[2] = { s, s };
            aes_mmo_quad<2, 0, 1>(h2, in, 0u, K, L);
            h[0] = h2[0]; h[1] = h2[1];
        }
#pragma unroll
        for (int m = 0; m < (CMP ? 3 : 2); m++) o[m] = row_swap_halves(h[m]);
        const uint32_t tL_m = quad_broadcast<0>(h[0]) & 1u, tR_m = quad_broadcast<0>(h[1]) & 1u;
        const uint32_t tL_o = quad_broadcast<0>(o[0]) & 1u, tR_o = quad_broadcast<0>(o[1]) & 1u;
        const uint32_t hL = h[0] & keep, hR = h[1] & keep, oL = o[0] & keep, oR = o[1] & keep;
        const uint32_t km = 0u - abit;                       // all ones iff Keep = R
        const uint32_t scw = pick32(km, hL ^ oL, hR ^ oR);   // the Lose-side strings
        const uint32_t tcwL = tL_m ^ tL_o ^ abit ^ 1u;
        const uint32_t tcwR = tR_m ^ tR_o ^ abit;
        ctrl[0] |= tcwL << i;
        ctrl[1] |= tcwR << i;

        uint32_t sigcw = 0, leaf = 0;
        if constexpr (CMP) {
            const uint32_t sgL_m = quad_broadcast<0>(h[2]) & mask, sgR_m = quad_broadcast<1>(h[2]) & mask, w_m = quad_broadcast<2>(h[2]);
            const uint32_t sgL_o = quad_broadcast<0>(o[2]) & mask, sgR_o = quad_broadcast<1>(o[2]) & mask, w_o = quad_broadcast<2>(o[2]);
            const uint32_t tauL_m = w_m & 1u, tauR_m = (w_m >> 1) & 1u, tauL_o = w_o & 1u, tauR_o = (w_o >> 1) & 1u;
            sigcw = pick32(km, sgR_m ^ sgR_o, sgL_m ^ sgL_o);                // the Keep-side strings
            const uint32_t taucwL = tauL_m ^ tauL_o ^ abit;
            const uint32_t taucwR = tauR_m ^ tauR_o ^ abit ^ 1u;
            ctrl[2] |= taucwL << i;
            ctrl[3] |= taucwR << i;
            // state'_{j, Lose} of either party, then sorted into party 0 / party 1
            const uint32_t taucw_lose = pick32(km, taucwL, taucwR);
            const uint32_t sg_m = pick32(km, sgL_m, sgR_m) ^ (sigcw & (0u - t_mine));
            const uint32_t sg_o = pick32(km, sgL_o, sgR_o) ^ (sigcw & (0u - t_other));
            const uint32_t tau_m = pick32(km, tauL_m, tauR_m) ^ (t_mine & taucw_lose);
            const uint32_t tau_o = pick32(km, tauL_o, tauR_o) ^ (t_other & taucw_lose);
            const uint32_t sg0 = pick32(hm, sg_o, sg_m), sg1 = pick32(hm, sg_m, sg_o), tau1 = pick32(hm, tau_m, tau_o);
            leaf = (abit - sg0 + sg1) & mask;                 // (-1)^{tau_1} (alpha[i] - sigma_0 + sigma_1)
            leaf = ((leaf ^ (0u - tau1)) + tau1) & mask;
        }
        // both parties move to state_{j, Keep}, corrected with the OLD t_j; this quad keeps its own seed and both control bits
        const uint32_t tcw_keep = pick32(km, tcwR, tcwL);
        s = pick32(km, hR, hL) ^ (scw & (0u - t_mine));
        t_mine = pick32(km, tR_m, tL_m) ^ (t_mine & tcw_keep);
        t_other = pick32(km, tR_o, tL_o) ^ (t_other & tcw_keep);
        const size_t pe = (size_t)i * k.bp + e;
        reinterpret_cast<uint32_t *>(key + k.s_cw)[4 * pe + col] = scw;
        if constexpr (CMP) {
            // lane 0 of the quad: sigma_CW, lane 1: CW_leaf, of this party's key
            if (col < 2) reinterpret_cast<uint32_t *>(key + (col ? k.leaf : k.sigma_cw))[pe] = col ? leaf : sigcw;
        }
    }
    const uint32_t c_m = quad_broadcast<3>(s) & mask, c_o = quad_broadcast<3>(row_swap_halves(s)) & mask;
    const uint32_t c0 = pick32(hm, c_o, c_m), c1 = pick32(hm, c_m, c_o), t1 = pick32(hm, t_mine, t_other);
    uint32_t last = (1u - c0 + c1) & mask;                    // CW^(n+1) = (-1)^{t_1} (1 - conv(s_0) + conv(s_1))
    if (t1) last = (0u - last) & mask;
    // lane 0: [[alpha]]_j, lane 1: CW^(n+1), of this party's key
    const uint32_t share = half ? ((alpha - r) & mask) : r;
    if (col < 2) reinterpret_cast<uint32_t *>(key + (col ? k.last : k.alpha_share))[e] = col ? last : share;
    if constexpr (CMP) {
        const uint32_t cw = col == 0 ? ctrl[0] : col == 1 ? ctrl[1] : col == 2 ? ctrl[2] : ctrl[3];
        reinterpret_cast<uint32_t *>(key + k.ctrl)[4 * e + col] = cw;
    } else if (col < 2) {
        reinterpret_cast<uint32_t *>(key + k.ctrl)[2 * e + col] = col == 0 ? ctrl[0] : ctrl[1];
    }
}

template <bool CMP, bool BALANCE>
__global__ __launch_bounds__(kThreads) void gen_octo_kernel(GenArgs a)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const QuadKeys K = load_quad_keys();
    const KeyLayout k = key_layout(CMP, a.n, a.batch);
    const uint32_t lane = threadIdx.x & 63u, col = lane & 3u, half = (lane >> 3) & 1u;
    const size_t tiles = k.bp / 8;
    const size_t stride = (size_t)(blockDim.x >> 6) * gridDim.x;
    for (size_t tile = (size_t)wave_index() * gridDim.x + blockIdx.x; tile < tiles; tile += stride) {
        const size_t e = tile * 8 + (lane >> 4) * 2 + ((lane >> 2) & 1u);
        if (e < a.batch) gen_octo_walk<CMP, BALANCE>(a, k, L, K, e, col, half);     // both quads of a pair drop out together
        else if (col == 0 && half == 0) zero_padding_element<CMP>(a.key0, a.key1, k, e, a.n);
    }
}

// Batches from the layout switch on: the same split of the work as eval_kernel.  The 16-element
// tiles run to the end of the PADDED batch, so that the padding elements are written too.
template <bool CMP>
__global__ __launch_bounds__(kThreads) void gen_kernel(GenArgs a)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const KeyLayout k = key_layout(CMP, a.n, a.batch);
    const uint32_t lane = threadIdx.x & 63u;
    const size_t stride = (size_t)(blockDim.x >> 6) * gridDim.x;
    const size_t slot = (size_t)wave_index() * gridDim.x + blockIdx.x;
    for (size_t tile = slot; tile < a.lane_tiles; tile += stride) {
        const size_t e = tile * 64 + lane;
        if (e < a.batch) gen_lane_walk<CMP>(a, k, L, e);
        else zero_padding_element<CMP>(a.key0, a.key1, k, e, a.n);
    }
    if (a.quad_tiles != 0) {
        const QuadKeys K = load_quad_keys();
        const size_t first = a.lane_tiles * 64;
        const size_t used = a.lane_tiles % stride;
        const uint32_t col = threadIdx.x & 3u;
        for (size_t q = slot >= used ? slot - used : slot + stride - used; q < a.quad_tiles; q += stride) {
            const size_t e = first + q * 16 + (lane >> 2);
            if (e < a.batch) gen_quad_walk<CMP, true>(a, k, L, K, e, col);
            else if (col == 0) zero_padding_element<CMP>(a.key0, a.key1, k, e, a.n);
        }
    }
}

// Batches below the layout switch: every key pair four lanes wide.
template <bool CMP, bool BALANCE>
__global__ __launch_bounds__(kThreads) void gen_quad_kernel(GenArgs a)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const QuadKeys K = load_quad_keys();
    const KeyLayout k = key_layout(CMP, a.n, a.batch);
    const uint32_t col = threadIdx.x & 3u;
    const size_t tiles = k.bp / 16;
    const size_t stride = (size_t)(blockDim.x >> 6) * gridDim.x;
    for (size_t tile = (size_t)wave_index() * gridDim.x + blockIdx.x; tile < tiles; tile += stride) {
        const size_t e = tile * 16 + ((threadIdx.x & 63u) >> 2);
        if (e < a.batch) gen_quad_walk<CMP, BALANCE>(a, k, L, K, e, col);
        else if (col == 0) zero_padding_element<CMP>(a.key0, a.key1, k, e, a.n);
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
    // per-device, idempotent: raise the dynamic-LDS limit of the kernels that hold the tables
    static DeviceInfo cache[64] = {};
    static std::mutex cache_lock;
    std::lock_guard<std::mutex> guard(cache_lock);
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
        const void *fns[] = { (const void *)eval_kernel<true, kPlain>, (const void *)eval_kernel<false, kPlain>,
                              (const void *)eval_kernel<true, kSign>, (const void *)eval_kernel<true, kReluOpen>,
                              (const void *)eval_kernel<false, kSign>,
                              (const void *)eval_quad_kernel<true, kPlain, true>, (const void *)eval_quad_kernel<false, kPlain, true>,
                              (const void *)eval_quad_kernel<true, kSign, true>, (const void *)eval_quad_kernel<true, kReluOpen, true>,
                              (const void *)eval_quad_kernel<false, kSign, true>,
                              (const void *)eval_quad_kernel<true, kPlain, false>, (const void *)eval_quad_kernel<false, kPlain, false>,
                              (const void *)eval_quad_kernel<true, kSign, false>, (const void *)eval_quad_kernel<true, kReluOpen, false>,
                              (const void *)eval_quad_kernel<false, kSign, false>,
                              (const void *)eval_octo_kernel<kPlain, true>, (const void *)eval_octo_kernel<kSign, true>,
                              (const void *)eval_octo_kernel<kReluOpen, true>, (const void *)eval_octo_kernel<kPlain, false>,
                              (const void *)eval_octo_kernel<kSign, false>, (const void *)eval_octo_kernel<kReluOpen, false>,
                              (const void *)gen_octo_kernel<true, true>, (const void *)gen_octo_kernel<false, true>,
                              (const void *)gen_octo_kernel<true, false>, (const void *)gen_octo_kernel<false, false>,
                              (const void *)gen_kernel<true>, (const void *)gen_kernel<false>,
                              (const void *)gen_quad_kernel<true, true>, (const void *)gen_quad_kernel<false, true>,
                              (const void *)gen_quad_kernel<true, false>, (const void *)gen_quad_kernel<false, false> };
        for (size_t i = 0; i < sizeof(fns) / sizeof(fns[0]); i++) {
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

static bool bad_count(size_t count) { return count > kMaxBatch; }

// a * b as an element count, or kMaxBatch + 1 if it does not fit the limit
static size_t checked_product(size_t a, size_t b)
{
    if (a == 0 || b == 0) return 0;
    if (a > kMaxBatch || b > kMaxBatch / a) return kMaxBatch + 1;
    return a * b;
}

struct LaunchShape {
    unsigned grid, threads;
    int balance;      // some SIMD gets more than one working wavefront
};

// One workgroup per CU (its tables take 128 KiB of the CU's LDS), always of 16 wavefronts: the
// kernels loop over tiles of 64 elements (16 in the quad layout), and wavefronts that get no tile
// still help to fill the tables (2-3 us of a small launch).  Every CU gets a workgroup as soon as
// there are that many tiles.
static LaunchShape shape_for(size_t elems, const DeviceInfo &d, size_t tile_elems = 64)
{
    const size_t cus = (size_t)d.cus;
    const size_t tiles = (elems + tile_elems - 1) / tile_elems;
    LaunchShape s;
    s.threads = (unsigned)kThreads;
    s.grid = (unsigned)(tiles < cus ? tiles : cus);
    s.balance = tiles > 4 * (size_t)s.grid;     // wavefront w of a workgroup runs on SIMD w mod 4
    return s;
}

// The quad layout (four lanes per element) serves batches that would leave the CUs short of
// wavefronts with one lane per element.  Measured on MI355X, for KeyGen and Eval, comparison and
// equality alike: the quad layout is faster below about 8 wavefronts of 64 elements per CU (2.4x
// for Eval and 2.3x for KeyGen at 16,384 elements, still 5 % at 114,688), slower above (by 25-30 %
// on large batches).
#ifndef FSS_QUAD_BELOW
#define FSS_QUAD_BELOW 8        // -D override: how the crossover was measured (builds with other values, same box)
#endif
constexpr size_t kQuadBelowWavesPerCu = FSS_QUAD_BELOW;

static size_t quad_layout_below(const DeviceInfo &d) { return (size_t)d.cus * 64 * kQuadBelowWavesPerCu; }

static bool use_quad_layout(size_t batch, const DeviceInfo &d) { return batch < quad_layout_below(d); }

// The eight-lanes-per-element comparison Eval (see eval_octo_walk) pays while the SIMDs hold one or two
// wavefronts of the quad layout.  Measured against it, same box: -11 % up to 8,192 elements, -2 %
// at 12,288, equal at 16,384, -7 % at 20,480, -5 % at 24,576, equal at 32,768, slower beyond.
#ifndef FSS_OCTO_UPTO
#define FSS_OCTO_UPTO 8         // in quad wavefronts (16 elements) per CU; -D override, as for FSS_QUAD_BELOW
#endif
constexpr size_t kOctoUpToWavesPerCu = FSS_OCTO_UPTO;

static bool use_octo_layout(size_t batch, const DeviceInfo &d) { return batch <= (size_t)d.cus * 16 * kOctoUpToWavesPerCu; }

// KeyGen with eight lanes per key pair (gen_octo_walk).  Measured against four lanes per pair, same
// box, comparison / equality: -37 % / -40 % up to 8,192 pairs, -21 % / -25 % at 16,384 and 24,576,
// -8 % / -11 % at 32,768, slower from 40,960 on.
#ifndef FSS_GEN_OCTO_UPTO
#define FSS_GEN_OCTO_UPTO 8     // in quad wavefronts (16 pairs) per CU; -D override, as for FSS_QUAD_BELOW
#endif
constexpr size_t kGenOctoUpToWavesPerCu = FSS_GEN_OCTO_UPTO;

static bool use_gen_octo_layout(size_t batch, const DeviceInfo &d) { return batch <= (size_t)d.cus * 16 * kGenOctoUpToWavesPerCu; }

// Launch through hipLaunchKernel and report ITS return value: the thread's last-error slot (which
// hipGetLastError would read and clear) may hold an unrelated error of the host application.
template <typename... P, typename... A>
static int launch(void (*kernel)(P...), unsigned grid, unsigned threads, size_t lds_bytes, hipStream_t st, A... a)
{
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    std::tuple<P...> vals(static_cast<P>(a)...);
    void *ptrs[sizeof...(P)];
    size_t i = 0;
    std::apply([&](auto &...v) { ((ptrs[i++] = static_cast<void *>(&v)), ...); }, vals);
    const hipError_t err = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(grid), dim3(threads), ptrs, lds_bytes, st);
    if (err != hipSuccess) { g_last_hip_error = (int)err; return FSS_ELAUNCH; }
    return FSS_OK;
}

// How a batch at or above the layout switch is walked.  Tiles of 64 elements, one lane per element,
// are dealt in rows of one tile per workgroup; 16 rows make a full pass.  Whole rows stay in that
// layout, except that a short rest after the last full pass (fewer than kQuadTailBelowWavesPerCu
// rows) is better off four lanes per element, and so is the last, partial row, which would give
// some CUs one wavefront more than the others (a fourth on one SIMD where the others have three
// costs the launch as much as a whole row).  Those elements become 16-element tiles at the end of
// the same launch (see eval_kernel).
struct WorkSplit {
    size_t lane_tiles, quad_tiles;
};

#ifndef FSS_QUAD_TAIL_BELOW
#define FSS_QUAD_TAIL_BELOW 8   // -D override, as for FSS_QUAD_BELOW
#endif
constexpr size_t kQuadTailBelowWavesPerCu = FSS_QUAD_TAIL_BELOW;

static WorkSplit split_work(size_t batch, const LaunchShape &ls)
{
    const size_t tiles = batch / 64;                               // whole tiles; a ragged end joins the rest below
    const size_t row = ls.grid, per_pass = row * (ls.threads / 64);
    const size_t full = tiles / per_pass * per_pass;
    const size_t rows_left = (tiles - full) / row;
    WorkSplit w;
    w.lane_tiles = full + (full > 0 && rows_left < kQuadTailBelowWavesPerCu ? 0 : rows_left * row);
    w.quad_tiles = (batch - w.lane_tiles * 64 + 15) / 16;
    return w;
}

typedef void (*EvalKernel)(EvalArgs);

static EvalKernel pick_eval_kernel(bool cmp, int mode)
{
    if (!cmp) return mode == kPlain ? eval_kernel<false, kPlain> : eval_kernel<false, kSign>;
    return mode == kPlain ? eval_kernel<true, kPlain> : mode == kSign ? eval_kernel<true, kSign> : eval_kernel<true, kReluOpen>;
}

template <bool BALANCE>
static EvalKernel pick_eval_quad_kernel_b(bool cmp, int mode)
{
    if (!cmp) return mode == kPlain ? eval_quad_kernel<false, kPlain, BALANCE> : eval_quad_kernel<false, kSign, BALANCE>;
    return mode == kPlain ? eval_quad_kernel<true, kPlain, BALANCE>
         : mode == kSign  ? eval_quad_kernel<true, kSign, BALANCE>
                          : eval_quad_kernel<true, kReluOpen, BALANCE>;
}

template <bool BALANCE>
static EvalKernel pick_eval_octo_kernel_b(int mode)
{
    return mode == kPlain ? eval_octo_kernel<kPlain, BALANCE> : mode == kSign ? eval_octo_kernel<kSign, BALANCE> : eval_octo_kernel<kReluOpen, BALANCE>;
}

static EvalKernel pick_eval_octo_kernel(int mode, bool balance)
{
    return balance ? pick_eval_octo_kernel_b<true>(mode) : pick_eval_octo_kernel_b<false>(mode);
}

static EvalKernel pick_eval_quad_kernel(bool cmp, int mode, bool balance)
{
    return balance ? pick_eval_quad_kernel_b<true>(cmp, mode) : pick_eval_quad_kernel_b<false>(cmp, mode);
}

static int gen_common(bool cmp, int n, size_t batch, const uint32_t *d_alpha, const uint32_t *d_alpha_r,
                      const uint8_t *d_seed0, const uint8_t *d_seed1, void *d_key0, void *d_key1, fss_stream_t stream)
{
    if (bad_n(n) || bad_count(batch)) return FSS_EINVAL;
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
    hipStream_t st = static_cast<hipStream_t>(stream);
    a.lane_tiles = 0; a.quad_tiles = 0;
    if (use_gen_octo_layout(batch, dev)) {
        const LaunchShape ls = shape_for(padded_batch(batch), dev, 8);
        void (*kernel)(GenArgs) = ls.balance ? (cmp ? gen_octo_kernel<true, true> : gen_octo_kernel<false, true>)
                                             : (cmp ? gen_octo_kernel<true, false> : gen_octo_kernel<false, false>);
        return launch(kernel, ls.grid, ls.threads, kLdsBytes, st, a);
    }
    if (use_quad_layout(batch, dev)) {
        const LaunchShape ls = shape_for(padded_batch(batch), dev, 16);
        void (*kernel)(GenArgs) = ls.balance ? (cmp ? gen_quad_kernel<true, true> : gen_quad_kernel<false, true>)
                                             : (cmp ? gen_quad_kernel<true, false> : gen_quad_kernel<false, false>);
        return launch(kernel, ls.grid, ls.threads, kLdsBytes, st, a);
    }
    const LaunchShape ls = shape_for(batch, dev);
    const WorkSplit w = split_work(batch, ls);
    a.lane_tiles = w.lane_tiles;
    a.quad_tiles = (padded_batch(batch) - w.lane_tiles * 64) / 16;
    return launch(cmp ? gen_kernel<true> : gen_kernel<false>, ls.grid, ls.threads, kLdsBytes, st, a);
}

static int eval_common(bool cmp, int mode, int party, int n, size_t batch, const void *d_key, const uint32_t *d_x,
                       const uint32_t *d_x2, uint32_t *d_out, uint32_t *d_out2, const uint32_t *d_y, const uint32_t *d_ta,
                       const uint32_t *d_tb, fss_stream_t stream)
{
    if (bad_n(n) || (party != 0 && party != 1) || bad_count(batch)) return FSS_EINVAL;
    if (batch == 0) return FSS_OK;
    if (!d_key || !d_x || !d_out) return FSS_EINVAL;
    if (misaligned(d_key, 256) || misaligned(d_x, 4) || misaligned(d_out, 4)) return FSS_EINVAL;
    if (mode != kPlain && (!d_x2 || misaligned(d_x2, 4))) return FSS_EINVAL;
    if (mode == kReluOpen && (!d_out2 || !d_y || !d_ta || !d_tb || misaligned(d_out2, 4) || misaligned(d_y, 4) ||
                              misaligned(d_ta, 4) || misaligned(d_tb, 4)))
        return FSS_EINVAL;
    DeviceInfo dev;
    int rc = prepare_device(&dev);
    if (rc != FSS_OK) return rc;
    EvalArgs a;
    a.key = static_cast<const uint8_t *>(d_key); a.x = d_x; a.x2 = d_x2; a.out = d_out; a.out2 = d_out2;
    a.y_share = d_y; a.tri_a = d_ta; a.tri_b = d_tb;
    a.batch = batch; a.n = n; a.party = party;
    hipStream_t st = static_cast<hipStream_t>(stream);
    a.lane_tiles = 0; a.quad_tiles = 0;
    if (cmp && use_octo_layout(batch, dev)) {
        const LaunchShape ls = shape_for(batch, dev, 8);
        return launch(pick_eval_octo_kernel(mode, ls.balance != 0), ls.grid, ls.threads, kLdsBytes, st, a);
    }
    if (use_quad_layout(batch, dev)) {
        const LaunchShape ls = shape_for(batch, dev, 16);
        return launch(pick_eval_quad_kernel(cmp, mode, ls.balance != 0), ls.grid, ls.threads, kLdsBytes, st, a);
    }
    const LaunchShape ls = shape_for(batch, dev);
    const WorkSplit w = split_work(batch, ls);
    a.lane_tiles = w.lane_tiles; a.quad_tiles = w.quad_tiles;
    return launch(pick_eval_kernel(cmp, mode), ls.grid, ls.threads, kLdsBytes, st, a);
}

static unsigned elementwise_grid(size_t batch)
{
    size_t g = (batch + 255) / 256;
    return (unsigned)(g < 4096 ? g : 4096);
}

static uint32_t host_ring_mask(int n) { return n == 32 ? 0xffffffffu : ((1u << n) - 1u); }

static bool bad_u32_ptr(const void *p) { return p == nullptr || misaligned(p, 4); }

// [[y]]_j + [[alpha]]_j with [[alpha]]_j the first plane of a key buffer (Algorithm 5 / wrapper of Algorithm 2)
static int mask_common(bool cmp, int n, size_t batch, const void *d_key, const uint32_t *d_y_share, uint32_t *d_masked,
                       fss_stream_t stream)
{
    if (bad_n(n) || bad_count(batch)) return FSS_EINVAL;
    if (batch == 0) return FSS_OK;
    if (!d_key || misaligned(d_key, 256) || bad_u32_ptr(d_y_share) || bad_u32_ptr(d_masked)) return FSS_EINVAL;
    const uint32_t *alpha_share = reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(d_key) + key_layout(cmp, n, batch).alpha_share);
    return launch(sign_mask_kernel, elementwise_grid(batch), 256, 0, static_cast<hipStream_t>(stream), alpha_share, d_y_share, d_masked,
                  batch, host_ring_mask(n));
}

struct StreamEvents {
    hipEvent_t copied[2];     // half h holds its chunk
    hipEvent_t consumed[2];   // half h has been evaluated and may be overwritten
};

static int streamed_args_ok(int party, int n, size_t batch, size_t chunk, const void *h_key_chunks, const uint32_t *d_x,
                            uint32_t *d_out, fss_stream_t copy_stream, fss_stream_t stream)
{
    if (bad_n(n) || (party != 0 && party != 1) || bad_count(batch) || bad_count(chunk) || chunk == 0 || chunk % 64 != 0) return FSS_EINVAL;
    if (batch == 0) return FSS_OK;
    if (!h_key_chunks || !d_x || !d_out || misaligned(d_x, 4) || misaligned(d_out, 4)) return FSS_EINVAL;
    if (copy_stream == stream) return FSS_EINVAL;
    return FSS_OK;
}

// Chunk c + 1 is copied host-to-device on the copy stream into one half of `staging` while chunk c
// is evaluated out of the other half; returns after the last chunk has been evaluated (the halves
// and the events must outlive the enqueued work).
static int streamed_walk(int party, int n, size_t batch, size_t chunk, const void *h_key_chunks, const uint32_t *d_x,
                         uint32_t *d_out, uint8_t *staging, const StreamEvents &ev, fss_stream_t copy_stream, fss_stream_t stream)
{
    hipStream_t cs = static_cast<hipStream_t>(copy_stream), es = static_cast<hipStream_t>(stream);
    const size_t chunk_bytes = key_layout(true, n, chunk).total;
    uint8_t *stage[2] = { staging, staging + chunk_bytes };
    int rc = FSS_OK;
    hipError_t err = hipSuccess;
    const uint8_t *src = static_cast<const uint8_t *>(h_key_chunks);
    const size_t nchunks = (batch + chunk - 1) / chunk;
    for (size_t c = 0; c < nchunks && err == hipSuccess && rc == FSS_OK; c++) {
        const int h = (int)(c & 1);
        const size_t first = c * chunk, len = (batch - first < chunk) ? batch - first : chunk;
        const size_t bytes = key_layout(true, n, len).total;
        if (c >= 2) err = hipStreamWaitEvent(cs, ev.consumed[h], 0);          // the half is free again
        if (err == hipSuccess) err = hipMemcpyAsync(stage[h], src, bytes, hipMemcpyHostToDevice, cs);
        if (err == hipSuccess) err = hipEventRecord(ev.copied[h], cs);
        if (err == hipSuccess) err = hipStreamWaitEvent(es, ev.copied[h], 0);
        if (err != hipSuccess) break;
        rc = eval_common(true, kPlain, party, n, len, stage[h], d_x + first, nullptr, d_out + first, nullptr, nullptr, nullptr,
                         nullptr, stream);
        if (rc == FSS_OK) err = hipEventRecord(ev.consumed[h], es);
        src += bytes;
    }
    const hipError_t e2 = hipStreamSynchronize(cs);
    const hipError_t e3 = hipStreamSynchronize(es);
    if (err == hipSuccess) err = e2 != hipSuccess ? e2 : e3;
    if (err != hipSuccess) { g_last_hip_error = (int)err; return FSS_ELAUNCH; }
    return rc;
}

// ------------------------------------------------------------------------------------
// Built-in staging memory for callers that cannot allocate
// ------------------------------------------------------------------------------------

// Two staging halves for fss_cmp_eval_streamed_static.  One copy of the array exists on every GPU
// the library runs on, from the moment its code is loaded there until the process ends.
constexpr size_t kStaticStagingBytes = (size_t)32 << 20;
static __device__ __align__(256) uint8_t scratch[kStaticStagingBytes];

struct StaticStaging {
    int ok;               // 1 ready, 0 not set up yet
    uint8_t *ptr;         // DEVICE address of this device's copy of `scratch` (the array's name is only a host-side handle)
    StreamEvents ev;      // created once, reused by every call on the device
};

// Per device, once, with that device current: the device address of `scratch` and four events.
static int prepare_static_staging(StaticStaging *out)
{
    static StaticStaging cache[64] = {};
    static std::mutex cache_lock;
    std::lock_guard<std::mutex> guard(cache_lock);
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) { g_last_hip_error = (int)err; return FSS_ELAUNCH; }
    if (dev < 0 || dev >= 64) return FSS_EDEVICE;
    StaticStaging &c = cache[dev];
    if (!c.ok) {
        void *p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err == hipSuccess && p == nullptr) err = hipErrorInvalidSymbol;
        StreamEvents ev = {};
        for (int i = 0; i < 2 && err == hipSuccess; i++) {
            err = hipEventCreateWithFlags(&ev.copied[i], hipEventDisableTiming);
            if (err == hipSuccess) err = hipEventCreateWithFlags(&ev.consumed[i], hipEventDisableTiming);
        }
        if (err != hipSuccess) {
            for (int i = 0; i < 2; i++) {
                if (ev.copied[i]) (void)hipEventDestroy(ev.copied[i]);
                if (ev.consumed[i]) (void)hipEventDestroy(ev.consumed[i]);
            }
            g_last_hip_error = (int)err;
            return FSS_ELAUNCH;
        }
        c.ptr = static_cast<uint8_t *>(p);
        c.ev = ev;
        c.ok = 1;
    }
    *out = c;
    return FSS_OK;
}

}  // namespace fss

extern "C" {

size_t fss_cmp_key_bytes(int n, size_t batch) { return fss::bad_n(n) || fss::bad_count(batch) ? 0 : fss::key_layout(true, n, batch).total; }

size_t fss_eq_key_bytes(int n, size_t batch) { return fss::bad_n(n) || fss::bad_count(batch) ? 0 : fss::key_layout(false, n, batch).total; }

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
    return fss::eval_common(true, fss::kPlain, party, n, batch, d_key, d_x, nullptr, d_out, nullptr, nullptr, nullptr, nullptr, stream);
}

int fss_eq_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_x, uint32_t *d_out,
                fss_stream_t stream)
{
    return fss::eval_common(false, fss::kPlain, party, n, batch, d_key, d_x, nullptr, d_out, nullptr, nullptr, nullptr, nullptr, stream);
}

int fss_sign_mask(int n, size_t batch, const void *d_key, const uint32_t *d_y_share, uint32_t *d_masked, fss_stream_t stream)
{
    return fss::mask_common(true, n, batch, d_key, d_y_share, d_masked, stream);
}

int fss_eq_mask(int n, size_t batch, const void *d_key, const uint32_t *d_y_share, uint32_t *d_masked, fss_stream_t stream)
{
    return fss::mask_common(false, n, batch, d_key, d_y_share, d_masked, stream);
}

int fss_eq_masked_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_masked0, const uint32_t *d_masked1,
                       uint32_t *d_out, fss_stream_t stream)
{
    return fss::eval_common(false, fss::kSign, party, n, batch, d_key, d_masked0, d_masked1, d_out, nullptr, nullptr, nullptr, nullptr, stream);
}

int fss_argmax_diff_mask(int n, size_t rows, int m, const void *d_cmp_key, const uint32_t *d_x_share, uint32_t *d_masked,
                         fss_stream_t stream)
{
    using namespace fss;
    if (bad_n(n) || m < 2) return FSS_EINVAL;
    const size_t batch = checked_product(rows, (size_t)m * (size_t)(m - 1));
    if (bad_count(batch)) return FSS_EINVAL;
    if (rows == 0) return FSS_OK;
    if (!d_cmp_key || misaligned(d_cmp_key, 256) || bad_u32_ptr(d_x_share) || bad_u32_ptr(d_masked)) return FSS_EINVAL;
    const uint32_t *alpha_share = reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(d_cmp_key) + key_layout(true, n, batch).alpha_share);
    return launch(argmax_diff_mask_kernel, elementwise_grid(batch), 256, 0, static_cast<hipStream_t>(stream), alpha_share, d_x_share,
                  d_masked, rows, (uint32_t)m, host_ring_mask(n));
}

int fss_argmax_count_mask(int party, int n, size_t rows, int m, const uint32_t *d_w_share, const void *d_eq_key,
                          uint32_t *d_masked, fss_stream_t stream)
{
    using namespace fss;
    if (bad_n(n) || m < 2 || (party != 0 && party != 1)) return FSS_EINVAL;
    const size_t batch = checked_product(rows, (size_t)m);
    if (bad_count(checked_product(batch, (size_t)(m - 1)))) return FSS_EINVAL;    // the comparison shares it sums
    if (rows == 0) return FSS_OK;
    if (!d_eq_key || misaligned(d_eq_key, 256) || bad_u32_ptr(d_w_share) || bad_u32_ptr(d_masked)) return FSS_EINVAL;
    const uint32_t *alpha_share = reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(d_eq_key) + key_layout(false, n, batch).alpha_share);
    return launch(argmax_count_mask_kernel, elementwise_grid(batch), 256, 0, static_cast<hipStream_t>(stream), alpha_share, d_w_share,
                  d_masked, batch, (uint32_t)m, host_ring_mask(n), party);
}

int fss_maxpool_unroll(size_t channels, int h, int w, int k, int s, const uint32_t *d_x_share, uint32_t *d_rows, fss_stream_t stream)
{
    using namespace fss;
    if (k < 1 || s < 1 || h < k || w < k) return FSS_EINVAL;
    const int oh = (h - k) / s + 1, ow = (w - k) / s + 1;
    const size_t total = checked_product(checked_product(channels, checked_product((size_t)oh, (size_t)ow)), checked_product((size_t)k, (size_t)k));
    if (bad_count(total) || bad_count(checked_product(channels, checked_product((size_t)h, (size_t)w)))) return FSS_EINVAL;
    if (channels == 0) return FSS_OK;
    if (bad_u32_ptr(d_x_share) || bad_u32_ptr(d_rows)) return FSS_EINVAL;
    return launch(maxpool_unroll_kernel, elementwise_grid(total), 256, 0, static_cast<hipStream_t>(stream), d_x_share, d_rows, channels,
                  h, w, k, s, oh, ow);
}

int fss_mul_open(int n, size_t count, const uint32_t *d_u_share, const uint32_t *d_v_share, const uint32_t *d_tri_a,
                 const uint32_t *d_tri_b, uint32_t *d_delta, uint32_t *d_eps, fss_stream_t stream)
{
    using namespace fss;
    if (bad_n(n) || bad_count(count)) return FSS_EINVAL;
    if (count == 0) return FSS_OK;
    if (bad_u32_ptr(d_u_share) || bad_u32_ptr(d_v_share) || bad_u32_ptr(d_tri_a) || bad_u32_ptr(d_tri_b) || bad_u32_ptr(d_delta) ||
        bad_u32_ptr(d_eps))
        return FSS_EINVAL;
    return launch(mul_open_kernel, elementwise_grid(count), 256, 0, static_cast<hipStream_t>(stream), d_u_share, d_v_share, d_tri_a,
                  d_tri_b, d_delta, d_eps, count, host_ring_mask(n));
}

int fss_dot_finish(int party, int n, size_t rows, int m, const uint32_t *d_delta0, const uint32_t *d_delta1, const uint32_t *d_eps0,
                   const uint32_t *d_eps1, const uint32_t *d_tri_a, const uint32_t *d_tri_b, const uint32_t *d_tri_c,
                   uint32_t *d_out, fss_stream_t stream)
{
    using namespace fss;
    if (bad_n(n) || m < 1 || (party != 0 && party != 1) || bad_count(checked_product(rows, (size_t)m))) return FSS_EINVAL;
    if (rows == 0) return FSS_OK;
    const void *ptrs[8] = { d_delta0, d_delta1, d_eps0, d_eps1, d_tri_a, d_tri_b, d_tri_c, d_out };
    for (int i = 0; i < 8; i++)
        if (bad_u32_ptr(ptrs[i])) return FSS_EINVAL;
    return launch(dot_finish_kernel, elementwise_grid(rows), 256, 0, static_cast<hipStream_t>(stream), d_delta0, d_delta1, d_eps0,
                  d_eps1, d_tri_a, d_tri_b, d_tri_c, d_out, rows, (uint32_t)m, host_ring_mask(n), party);
}

int fss_sign_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_masked0, const uint32_t *d_masked1,
                  uint32_t *d_out, fss_stream_t stream)
{
    return fss::eval_common(true, fss::kSign, party, n, batch, d_key, d_masked0, d_masked1, d_out, nullptr, nullptr, nullptr, nullptr, stream);
}

int fss_relu_open(int party, int n, size_t batch, const void *d_key, const uint32_t *d_masked0, const uint32_t *d_masked1,
                  const uint32_t *d_y_share, const uint32_t *d_tri_a, const uint32_t *d_tri_b, uint32_t *d_delta,
                  uint32_t *d_eps, fss_stream_t stream)
{
    return fss::eval_common(true, fss::kReluOpen, party, n, batch, d_key, d_masked0, d_masked1, d_delta, d_eps, d_y_share, d_tri_a,
                            d_tri_b, stream);
}

int fss_relu_finish(int party, int n, size_t batch, const uint32_t *d_delta0, const uint32_t *d_delta1, const uint32_t *d_eps0,
                    const uint32_t *d_eps1, const uint32_t *d_tri_a, const uint32_t *d_tri_b, const uint32_t *d_tri_c,
                    uint32_t *d_out, fss_stream_t stream)
{
    using namespace fss;
    if (bad_n(n) || (party != 0 && party != 1) || bad_count(batch)) return FSS_EINVAL;
    if (batch == 0) return FSS_OK;
    const void *ptrs[8] = { d_delta0, d_delta1, d_eps0, d_eps1, d_tri_a, d_tri_b, d_tri_c, d_out };
    for (int i = 0; i < 8; i++)
        if (bad_u32_ptr(ptrs[i])) return FSS_EINVAL;
    const uint32_t mask = host_ring_mask(n);
    return launch(relu_finish_kernel, elementwise_grid(batch), 256, 0, static_cast<hipStream_t>(stream), d_delta0, d_delta1, d_eps0,
                  d_eps1, d_tri_a, d_tri_b, d_tri_c, d_out, batch, mask, party);
}

size_t fss_cmp_chunked_key_bytes(int n, size_t batch, size_t chunk)
{
    if (fss::bad_n(n) || fss::bad_count(batch) || fss::bad_count(chunk) || chunk == 0 || chunk % 64 != 0) return 0;
    const size_t full = batch / chunk, rest = batch % chunk;
    return full * fss::key_layout(true, n, chunk).total + (rest ? fss::key_layout(true, n, rest).total : 0);
}

int fss_cmp_eval_streamed(int party, int n, size_t batch, size_t chunk, const void *h_key_chunks, const uint32_t *d_x,
                          uint32_t *d_out, void *d_staging, fss_stream_t copy_stream, fss_stream_t stream)
{
    using namespace fss;
    const int rc = streamed_args_ok(party, n, batch, chunk, h_key_chunks, d_x, d_out, copy_stream, stream);
    if (rc != FSS_OK || batch == 0) return rc;
    if (!d_staging || misaligned(d_staging, 256)) return FSS_EINVAL;
    StreamEvents ev = {};
    hipError_t err = hipSuccess;
    for (int i = 0; i < 2 && err == hipSuccess; i++) {
        err = hipEventCreateWithFlags(&ev.copied[i], hipEventDisableTiming);
        if (err == hipSuccess) err = hipEventCreateWithFlags(&ev.consumed[i], hipEventDisableTiming);
    }
    int out = FSS_OK;
    if (err != hipSuccess) { g_last_hip_error = (int)err; out = FSS_ELAUNCH; }
    else out = streamed_walk(party, n, batch, chunk, h_key_chunks, d_x, d_out, static_cast<uint8_t *>(d_staging), ev, copy_stream, stream);
    for (int i = 0; i < 2; i++) {
        if (ev.copied[i]) (void)hipEventDestroy(ev.copied[i]);
        if (ev.consumed[i]) (void)hipEventDestroy(ev.consumed[i]);
    }
    return out;
}

size_t fss_static_staging_bytes(void) { return fss::kStaticStagingBytes; }

int fss_cmp_eval_streamed_static(int party, int n, size_t batch, size_t chunk, const void *h_key_chunks, const uint32_t *d_x,
                                 uint32_t *d_out, fss_stream_t copy_stream, fss_stream_t stream)
{
    using namespace fss;
    int rc = streamed_args_ok(party, n, batch, chunk, h_key_chunks, d_x, d_out, copy_stream, stream);
    if (rc != FSS_OK) return rc;
    if (2 * key_layout(true, n, chunk).total > kStaticStagingBytes) return FSS_ELIMIT;   // chunk <= 2^40: no overflow
    if (batch == 0) return FSS_OK;
    StaticStaging st;
    rc = prepare_static_staging(&st);       // after the first call on a device: a table lookup
    if (rc != FSS_OK) return rc;
    return streamed_walk(party, n, batch, chunk, h_key_chunks, d_x, d_out, st.ptr, st.ev, copy_stream, stream);
}

int fss_clock_probe(uint64_t *d_ticks, uint32_t iterations, fss_stream_t stream)
{
    using namespace fss;
    if (!d_ticks || misaligned(d_ticks, 8) || iterations == 0 || iterations > (1u << 20)) return FSS_EINVAL;
    return launch(clock_probe_kernel, 1, 64, 0, static_cast<hipStream_t>(stream), reinterpret_cast<unsigned long long *>(d_ticks), iterations);
}

int fss_wall_clock_khz(void)
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
    return khz;
}

int fss_prepare(void)
{
    fss::DeviceInfo dev;
    int rc = fss::prepare_device(&dev);
    if (rc != FSS_OK) return rc;
    fss::StaticStaging st;
    return fss::prepare_static_staging(&st);
}

size_t fss_quad_layout_below(void)
{
    fss::DeviceInfo dev;
    return fss::prepare_device(&dev) == FSS_OK ? fss::quad_layout_below(dev) : 0;
}

const char *fss_strerror(int code)
{
    switch (code) {
    case FSS_OK: return "success";
    case FSS_EINVAL: return "invalid argument (party, n, element count above 2^40, NULL/misaligned/overlapping pointer)";
    case FSS_ELAUNCH: return "HIP runtime error while preparing or launching a kernel";
    case FSS_EDEVICE: return "device unsupported: kernels need 128 KiB of LDS per workgroup";
    case FSS_ELIMIT: return "size beyond the fixed limit of this entry point (chunk too large for the built-in staging memory)";
    default: return "unknown fss error code";
    }
}

int fss_last_hip_error(void) { return fss::g_last_hip_error; }

}  // extern "C"
