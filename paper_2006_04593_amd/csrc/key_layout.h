// Byte offsets of the planes of one party's key buffer (layout documented in
// include/fss.h).  Plain arithmetic shared by the host entry points and the kernels.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define FSS_HD __host__ __device__
#else
#define FSS_HD
#endif

namespace fss {

constexpr size_t kPadElems = 64;  // plane length granularity = one wavefront
constexpr size_t kMaxBatch = (size_t)1 << 40;   // elements per call; keeps every byte offset far below 2^64

FSS_HD inline size_t padded_batch(size_t batch) { return (batch + kPadElems - 1) / kPadElems * kPadElems; }

struct KeyLayout {
    size_t bp;            // padded batch
    size_t alpha_share;   // u32[bp]
    size_t seed;          // u8[bp][16]
    size_t ctrl;          // u32[bp][4] (comparison) or u32[bp][2] (equality)
    size_t s_cw;          // u8[n][bp][16]
    size_t sigma_cw;      // u32[n][bp]   (comparison only)
    size_t leaf;          // u32[n][bp]   (comparison only)
    size_t last;          // u32[bp]
    size_t total;
};

FSS_HD inline KeyLayout key_layout(bool cmp, int n, size_t batch)
{
    KeyLayout k;
    size_t bp = padded_batch(batch), off = 0;
    k.bp = bp;
    k.alpha_share = off; off += 4 * bp;
    k.seed = off;        off += 16 * bp;
    k.ctrl = off;        off += (cmp ? 16 : 8) * bp;
    k.s_cw = off;        off += (size_t)n * 16 * bp;
    k.sigma_cw = off;    if (cmp) off += (size_t)n * 4 * bp;
    k.leaf = off;        if (cmp) off += (size_t)n * 4 * bp;
    k.last = off;        off += 4 * bp;
    k.total = off;
    return k;
}

}  // namespace fss
