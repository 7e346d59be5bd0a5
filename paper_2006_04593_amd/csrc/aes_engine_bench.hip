// Stand-alone micro-benchmark behind the choice of AES engine (one MI355X, no inputs):
//   1. raw Matyas-Meyer-Oseas blocks/s of the LDS-table engine (aes_lds.h), as the kernels use it;
//   2. the same for the ALU-only bit-plane engine (aes_bitplane.h);
//   3. the machine rates that bound them: conflict-free ds_read_b32 lookups per clock per CU
//      (the kernel's 32-copy access pattern and an unreplicated table for comparison), the LDS
//      read port by access width (b32 / b64 / b128), and the issue rate of the vector-ALU
//      instructions both engines are made of;
//   4. the LDS-table engine in its four-lanes-per-block layout (aes_quad.h);
//   5. whether the vector-memory path could carry some of the lookups beside the LDS (gathers
//      from a 1-KiB table that stays in the L1 cache);
//   6. whether the ALU-only engine, launched on a second stream, finds unused vector-ALU cycles
//      beside the LDS-table engine on the same CUs (its workgroups need no LDS, so they fit).
// All figures come from HIP events around long launches that fill every CU.
//
// usage: aes_engine_bench            (prints a table; exit status 0)
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "aes_bitplane.h"
#include "aes_lds.h"
#include "aes_quad.h"

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            return 1;                                                                \
        }                                                                            \
    } while (0)

using namespace fss;

// ---- engine 1: LDS tables, two chained blocks per lane per iteration (keys 1/2 per lane + key 3)
__global__ __launch_bounds__(kThreads) void lds_engine(uint32_t *out, int iters)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    uint32_t s[4] = { threadIdx.x * 2654435761u, blockIdx.x * 40503u + 1u, threadIdx.x ^ 0x5bd1e995u, 7u };
    for (int it = 0; it < iters; it++) {
        uint32_t g[2][4];
        // two independent inputs: the raw engine rate, without the sharing of lookups that blocks
        // of the same input enjoy in the kernels
        const uint32_t in[2][4] = { { s[0], s[1], s[2], s[3] }, { s[1], s[2], s[3], s[0] } };
        const uint32_t pk[2] = { 0u - (s[3] & 1u), 0u };
        aes_mmo<-1, 2>(g, in, pk, L);
#pragma unroll
        for (int c = 0; c < 4; c++) s[c] = g[0][c] ^ g[1][(c + 1) & 3];
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = s[0] ^ s[1] ^ s[2] ^ s[3];
}

// ---- engine 2 in small workgroups (256 threads, no LDS), to run beside engine 1 on the same CU
__global__ __launch_bounds__(256) void bitplane_engine_small(uint32_t *out, int iters)
{
    bp::W a[8][4];
    for (int j = 0; j < 8; j++)
        for (int c = 0; c < 4; c++) a[j][c] = threadIdx.x * 2654435761u + blockIdx.x * 40503u + j * 97u + c;
    const bp::W pick = ((threadIdx.x * 0x9e3779b9u) >> 24) * 0x01010101u;
    for (int it = 0; it < iters; it++) {
        bp::W o[8][4];
        bp::mmo8<bp::kPickLowK3High>(o, a, pick);
        for (int j = 0; j < 8; j++)
            for (int c = 0; c < 4; c++) a[j][c] = o[j][c];
    }
    uint32_t r = 0;
    for (int j = 0; j < 8; j++)
        for (int c = 0; c < 4; c++) r ^= a[j][c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// ---- engine 1 in the quad layout: two chained blocks per quad per iteration
__global__ __launch_bounds__(kThreads) void quad_engine(uint32_t *out, int iters)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    const QuadKeys K = load_quad_keys();
    uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 1u;
    for (int it = 0; it < iters; it++) {
        uint32_t g[2];
        const uint32_t in[2] = { s, s ^ 0x9e3779b9u };
        aes_mmo_quad<0, -1, 2>(g, in, 0u - (quad_broadcast<3>(s) & 1u), K, L);
        s = g[0] ^ quad_broadcast<1>(g[1]);
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- 16 lookups per lane and iteration from pseudo-random bytes, the first G of them as buffer
// loads from a 1-KiB table in global memory, the others from the LDS tables
template <int G>
__global__ __launch_bounds__(kThreads) void gather_mix(uint32_t *out, const uint32_t *table, int iters)
{
    extern __shared__ uint32_t lds[];
    fill_tables(lds);
    __syncthreads();
    const LaneBase L = lane_base(lds);
    __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)table, 0, 1024, 0x00020000);
    uint32_t r[4];
    for (int c = 0; c < 4; c++) r[c] = threadIdx.x * 747796405u + blockIdx.x * 2891336453u + 12345u * (c + 1);
    for (int it = 0; it < iters; it++) {
        uint32_t v[16];
#pragma unroll
        for (int q = 0; q < 16; q++) {
            const uint32_t w = r[q >> 2];
            if (q < G) {
                const uint32_t index = __builtin_amdgcn_perm(w, 0u, 0x0c0c0c04u + (q & 3));
                v[q] = __builtin_amdgcn_raw_buffer_load_b32(rs, index << 2, 0, 0);
            } else {
                const uint32_t base = (q & 2) ? L.b : L.a;
                const uint32_t addr = __builtin_amdgcn_perm(w, base, 0x03020000u | ((4u + (q & 3)) << 8));
                v[q] = lds_load(addr + ((q & 1) ? kOddTable : 0u));
            }
        }
#pragma unroll
        for (int c = 0; c < 4; c++)
            r[c] = bitop3<kXor3>(bitop3<kXor3>(v[4 * c], v[4 * c + 1], v[4 * c + 2]), v[4 * c + 3], r[(c + 1) & 3]) + 0x9e3779b9u;
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = r[0] ^ r[1] ^ r[2] ^ r[3];
}

// ---- engine 2: bit planes, eight chained blocks per lane per iteration
__global__ __launch_bounds__(kThreads) void bitplane_engine(uint32_t *out, int iters)
{
    bp::W a[8][4];
    for (int j = 0; j < 8; j++)
        for (int c = 0; c < 4; c++) a[j][c] = threadIdx.x * 2654435761u + blockIdx.x * 40503u + j * 97u + c;
    const bp::W pick = ((threadIdx.x * 0x9e3779b9u) >> 24) * 0x01010101u;
    for (int it = 0; it < iters; it++) {
        bp::W o[8][4];
        bp::mmo8<bp::kPickLowK3High>(o, a, pick);
        for (int j = 0; j < 8; j++)
            for (int c = 0; c < 4; c++) a[j][c] = o[j][c];
    }
    uint32_t acc = 0;
    for (int j = 0; j < 8; j++)
        for (int c = 0; c < 4; c++) acc ^= a[j][c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

// ---- machine rate: ds_read_b32 with per-lane addresses and (almost) no ALU work beside it
// REPL = true: the kernels' pattern ((entry << 8) | copy of lane); false: one 1-KiB table for all lanes.
// The 16 addresses of a lane are drawn once; every iteration issues the 16 loads, waits, and
// folds the results with 16 two-operand XORs.
// FAIR: the wavefront lowers its priority as it advances (3, 2, 1, 0 from 0, 1/2, 3/4, 7/8 of its
// iterations), as the FSS kernels do per tile; without it the SIMD serves its oldest wavefront first,
// the old ones finish early and the launch ends with too few wavefronts to keep the LDS busy.
template <bool REPL, bool FAIR>
__global__ __launch_bounds__(kThreads) void lds_rate(uint32_t *out, int iters)
{
    extern __shared__ uint32_t lds[];
    for (uint32_t j = threadIdx.x; j < kLdsBytes / 4; j += blockDim.x) lds[j] = j * 2654435761u;
    __syncthreads();
    const uint32_t lane4 = (threadIdx.x & 31u) << 2;
    uint32_t r = threadIdx.x * 747796405u + blockIdx.x * 2891336453u + 12345u, acc = 0;
    uint32_t a[16];
#pragma unroll
    for (int k = 0; k < 16; k++) {
        r = r * 1664525u + 1013904223u;
        const uint32_t e = (r >> 13) & 255u;
        a[k] = REPL ? ((e << 8) | lane4 | ((k & 1) << 7) | ((k & 2) << 15)) : ((e << 2) | (k << 10));
    }
    if (FAIR) __builtin_amdgcn_s_setprio(3);
    for (int it = 0; it < iters; it++) {
        if (FAIR) {
            if (it == (iters >> 1)) __builtin_amdgcn_s_setprio(2);
            else if (it == iters - (iters >> 2)) __builtin_amdgcn_s_setprio(1);
            else if (it == iters - (iters >> 3)) __builtin_amdgcn_s_setprio(0);
        }
        uint32_t v[16];
#pragma unroll
        for (int k = 0; k < 16; k++) asm volatile("ds_read_b32 %0, %1" : "=v"(v[k]) : "v"(a[k]) : "memory");
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                       "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
                     :
                     : "memory");
#pragma unroll
        for (int k = 0; k < 16; k++) acc ^= v[k];
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

// ---- machine rate of the LDS read port by access width: ds_read_b32 / _b64 / _b128 with
// data-dependent per-lane addresses that are conflict-free by construction.  Every entry owns 256
// bytes (the kernels' stride); a lane reads WIDTH bytes at offset (lane mod COPIES) * WIDTH inside
// a pseudo-random entry, so any COPIES consecutive lanes cover COPIES * WIDTH distinct consecutive
// bytes' worth of banks whatever the entries are:
//   WIDTH 4, COPIES 32: the kernels' pattern (lanes l and l + 32 share a bank);
//   WIDTH 4, COPIES 64: one bank per lane if the LDS had 64 independent banks for 32-bit reads;
//   WIDTH 8, COPIES 32 and WIDTH 16, COPIES 16: 256 bytes per 32 (16) lanes.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int WIDTH, int COPIES>
__global__ __launch_bounds__(kThreads) void lds_width_rate(uint32_t *out, int iters)
{
    static_assert(WIDTH * COPIES <= 256, "a lane's read stays inside its entry");
    extern __shared__ uint32_t lds[];
    for (uint32_t j = threadIdx.x; j < kLdsBytes / 4; j += blockDim.x) lds[j] = j * 2654435761u;
    __syncthreads();
    const uint32_t off = (threadIdx.x % COPIES) * WIDTH;
    uint32_t r = threadIdx.x * 747796405u + blockIdx.x * 2891336453u + 12345u, acc = 0;
    uint32_t a[8];
#pragma unroll
    for (int k = 0; k < 8; k++) {
        r = r * 1664525u + 1013904223u;
        a[k] = (((r >> 13) & 511u) << 8) | off;         // 512 entries x 256 B = the 128 KiB that were filled
    }
    for (int it = 0; it < iters; it++) {
        if constexpr (WIDTH == 4) {
            uint32_t v[8];
#pragma unroll
            for (int k = 0; k < 8; k++) asm volatile("ds_read_b32 %0, %1" : "=v"(v[k]) : "v"(a[k]) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]) : : "memory");
#pragma unroll
            for (int k = 0; k < 8; k++) acc ^= v[k];
        } else if constexpr (WIDTH == 8) {
            u32x2 v[8];
#pragma unroll
            for (int k = 0; k < 8; k++) asm volatile("ds_read_b64 %0, %1" : "=v"(v[k]) : "v"(a[k]) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]) : : "memory");
#pragma unroll
            for (int k = 0; k < 8; k++) acc ^= v[k].x ^ v[k].y;
        } else {
            u32x4 v[8];
#pragma unroll
            for (int k = 0; k < 8; k++) asm volatile("ds_read_b128 %0, %1" : "=v"(v[k]) : "v"(a[k]) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]) : : "memory");
#pragma unroll
            for (int k = 0; k < 8; k++) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
        }
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

// ---- machine rate: vector-ALU instructions, 8 independent chains per wavefront
#define FSS_ALU_LOOP(INSTRS)                                                                                  \
    asm volatile("v_mov_b32 v10, %1\n v_mov_b32 v11, %1\n v_mov_b32 v12, %1\n v_mov_b32 v13, %1\n"            \
                 "v_mov_b32 v14, %1\n v_mov_b32 v15, %1\n v_mov_b32 v16, %1\n v_mov_b32 v17, %1\n"            \
                 "v_mov_b32 v18, %1\n v_mov_b32 v19, %1\n v_mov_b32 v20, %1\n v_mov_b32 v21, %1\n"            \
                 "s_mov_b32 s20, %2\n s_mov_b32 s21, 0x03020500\n"                                            \
                 "1:\n .rept 16\n" INSTRS ".endr\n"                                                           \
                 "s_sub_u32 s20, s20, 1\n s_cmp_lg_u32 s20, 0\n s_cbranch_scc1 1b\n"                          \
                 "v_xor_b32 %0, v10, v11\n v_xor_b32 %0, %0, v12\n v_xor_b32 %0, %0, v13\n"                   \
                 "v_xor_b32 %0, %0, v14\n v_xor_b32 %0, %0, v15\n v_xor_b32 %0, %0, v16\n v_xor_b32 %0, %0, v17\n" \
                 : "=&v"(r)                                                                                   \
                 : "v"(seed), "s"(iters)                                                                      \
                 : "v10", "v11", "v12", "v13", "v14", "v15", "v16", "v17", "v18", "v19", "v20", "v21", "s20", "s21", "scc", "memory")
#define FSS_ALU_8(op, b, c)                                                                       \
    op " v10, v10, " b "18, " c "\n" op " v11, v11, " b "19, " c "\n" op " v12, v12, " b "20, " c "\n" \
    op " v13, v13, " b "21, " c "\n" op " v14, v14, " b "18, " c "\n" op " v15, v15, " b "19, " c "\n" \
    op " v16, v16, " b "20, " c "\n" op " v17, v17, " b "21, " c "\n"

template <int OP>
__global__ __launch_bounds__(kThreads) void alu_rate(uint32_t *out, int iters)
{
    uint32_t seed = threadIdx.x + blockIdx.x, r;
    if (OP == 0) FSS_ALU_LOOP(FSS_ALU_8("v_perm_b32", "v", "s21"));
    if (OP == 1) FSS_ALU_LOOP(FSS_ALU_8("v_bitop3_b32", "v", "v19 bitop3:0x96"));
    if (OP == 2) FSS_ALU_LOOP(FSS_ALU_8("v_bitop3_b32", "v", "s21 bitop3:0x96"));
    if (OP == 3) FSS_ALU_LOOP("v_xor_b32 v10, v10, v18\n v_xor_b32 v11, v11, v19\n v_xor_b32 v12, v12, v20\n v_xor_b32 v13, v13, v21\n"
                              "v_xor_b32 v14, v14, v18\n v_xor_b32 v15, v15, v19\n v_xor_b32 v16, v16, v20\n v_xor_b32 v17, v17, v21\n");
    if (OP == 4) FSS_ALU_LOOP(FSS_ALU_8("v_alignbit_b32", "v", "8"));
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

template <typename F>
static int time_launch(F launch, float *best_ms)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    *best_ms = 1e30f;
    for (int rep = 0; rep < 3; rep++) {
        CK(hipEventRecord(a, 0));
        launch();
        CK(hipEventRecord(b, 0));
        CK(hipEventSynchronize(b));
        CK(hipGetLastError());
        float ms;
        CK(hipEventElapsedTime(&ms, a, b));
        if (ms < *best_ms) *best_ms = ms;
    }
    return 0;
}

int main()
{
    hipDeviceProp_t p;
    CK(hipGetDeviceProperties(&p, 0));
    const int cus = p.multiProcessorCount;
    printf("device %s, %d CUs, nominal clock %.0f MHz, LDS per workgroup %zu B\n", p.gcnArchName, cus, p.clockRate / 1e3,
           (size_t)p.sharedMemPerBlock);
    uint32_t *out;
    CK(hipMalloc(&out, (size_t)cus * 8 * kThreads * 4));
    CK(hipFuncSetAttribute((const void *)lds_engine, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    CK(hipFuncSetAttribute((const void *)lds_rate<true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    CK(hipFuncSetAttribute((const void *)lds_rate<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    CK(hipFuncSetAttribute((const void *)lds_rate<false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    float ms;
    const double ghz = 2.4;

    printf("\nAES engines (Matyas-Meyer-Oseas blocks, every CU busy)\n");
    {
        const int iters = 2000;
        if (time_launch([&] { hipLaunchKernelGGL(lds_engine, dim3(cus), dim3(kThreads), kLdsBytes, 0, out, iters); }, &ms)) return 1;
        const double blocks = (double)cus * kThreads * iters * 2;
        printf("  LDS-table engine   %8.3f ms  %7.1f G blocks/s  %5.2f clk/block/CU at %.1f GHz\n", ms, blocks / ms / 1e6,
               ms * 1e-3 * ghz * 1e9 * cus / blocks, ghz);
    }
    {
        const int iters = 250;
        if (time_launch([&] { hipLaunchKernelGGL(bitplane_engine, dim3(cus), dim3(kThreads), 0, 0, out, iters); }, &ms)) return 1;
        const double blocks = (double)cus * kThreads * iters * 8;
        printf("  bit-plane engine   %8.3f ms  %7.1f G blocks/s  %5.2f clk/block/CU at %.1f GHz\n", ms, blocks / ms / 1e6,
               ms * 1e-3 * ghz * 1e9 * cus / blocks, ghz);
    }

    printf("\nds_read_b32 with data-dependent addresses, 16 wavefronts per CU\n");
    {
        const int iters = 20000;
        const double lanes = (double)cus * kThreads * iters * 16;
        if (time_launch([&] { hipLaunchKernelGGL((lds_rate<true, false>), dim3(cus), dim3(kThreads), kLdsBytes, 0, out, iters); }, &ms)) return 1;
        printf("  32 copies per entry (kernels' layout) %8.3f ms  %6.1f lookups/clk/CU  %6.1f TB/s\n", ms,
               lanes / (ms * 1e-3) / cus / (ghz * 1e9), lanes * 4 / (ms * 1e-3) / 1e12);
        if (time_launch([&] { hipLaunchKernelGGL((lds_rate<true, true>), dim3(cus), dim3(kThreads), kLdsBytes, 0, out, iters); }, &ms)) return 1;
        printf("  the same, priority falling with progress %5.3f ms  %6.1f lookups/clk/CU  %6.1f TB/s\n", ms,
               lanes / (ms * 1e-3) / cus / (ghz * 1e9), lanes * 4 / (ms * 1e-3) / 1e12);
        if (time_launch([&] { hipLaunchKernelGGL((lds_rate<false, false>), dim3(cus), dim3(kThreads), kLdsBytes, 0, out, iters); }, &ms)) return 1;
        printf("  one 1-KiB table, no replication       %8.3f ms  %6.1f lookups/clk/CU  %6.1f TB/s\n", ms,
               lanes / (ms * 1e-3) / cus / (ghz * 1e9), lanes * 4 / (ms * 1e-3) / 1e12);
    }

    printf("\nLDS read port by access width: conflict-free per-lane addresses (random 256-byte entry, own slot inside it), 16 wavefronts per CU\n");
    {
        const int iters = 20000;
        const double reads = (double)cus * kThreads * iters * 8;
        struct { const char *name; int width; const void *fn; } rows[4] = {
            { "ds_read_b32,  32 slots of 4 B  (kernels' pattern)", 4, (const void *)lds_width_rate<4, 32> },
            { "ds_read_b32,  64 slots of 4 B  (one bank per lane)", 4, (const void *)lds_width_rate<4, 64> },
            { "ds_read_b64,  32 slots of 8 B", 8, (const void *)lds_width_rate<8, 32> },
            { "ds_read_b128, 16 slots of 16 B", 16, (const void *)lds_width_rate<16, 16> },
        };
        for (int i = 0; i < 4; i++) {
            CK(hipFuncSetAttribute(rows[i].fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
            uint32_t *o = out;
            int it = iters;
            void *args[2] = { &o, &it };
            const void *fn = rows[i].fn;
            if (time_launch([&] { (void)hipLaunchKernel(fn, dim3(cus), dim3(kThreads), args, kLdsBytes, 0); }, &ms)) return 1;
            printf("  %-52s %8.3f ms  %6.1f reads/clk/CU  %6.1f B/clk/CU  %6.1f TB/s\n", rows[i].name, ms,
                   reads / (ms * 1e-3) / cus / (ghz * 1e9), reads * rows[i].width / (ms * 1e-3) / cus / (ghz * 1e9),
                   reads * rows[i].width / (ms * 1e-3) / 1e12);
        }
    }

    printf("\nvector-ALU issue rate, 4 wavefronts per SIMD, 8 independent chains\n");
    {
        const int iters = 20000;
        const double laneops = (double)cus * kThreads * iters * 128;
        const char *names[5] = { "v_perm_b32 (v,v,s)", "v_bitop3_b32 (v,v,v)", "v_bitop3_b32 (v,v,s)", "v_xor_b32 (v,v)", "v_alignbit_b32 (v,v,imm)" };
        for (int op = 0; op < 5; op++) {
            int rc = 0;
            if (op == 0) rc = time_launch([&] { hipLaunchKernelGGL(alu_rate<0>, dim3(cus), dim3(kThreads), 0, 0, out, iters); }, &ms);
            if (op == 1) rc = time_launch([&] { hipLaunchKernelGGL(alu_rate<1>, dim3(cus), dim3(kThreads), 0, 0, out, iters); }, &ms);
            if (op == 2) rc = time_launch([&] { hipLaunchKernelGGL(alu_rate<2>, dim3(cus), dim3(kThreads), 0, 0, out, iters); }, &ms);
            if (op == 3) rc = time_launch([&] { hipLaunchKernelGGL(alu_rate<3>, dim3(cus), dim3(kThreads), 0, 0, out, iters); }, &ms);
            if (op == 4) rc = time_launch([&] { hipLaunchKernelGGL(alu_rate<4>, dim3(cus), dim3(kThreads), 0, 0, out, iters); }, &ms);
            if (rc) return 1;
            printf("  %-26s %8.3f ms  %6.1f T lane-ops/s  %6.1f lanes/clk/CU at %.1f GHz\n", names[op], ms, laneops / (ms * 1e-3) / 1e12,
                   laneops / (ms * 1e-3) / cus / (ghz * 1e9), ghz);
        }
    }

    printf("\nLDS-table engine, four lanes per block (small-batch layout)\n");
    {
        CK(hipFuncSetAttribute((const void *)quad_engine, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
        const int iters = 2000;
        if (time_launch([&] { hipLaunchKernelGGL(quad_engine, dim3(cus), dim3(kThreads), kLdsBytes, 0, out, iters); }, &ms)) return 1;
        const double blocks = (double)cus * (kThreads / 4) * iters * 2;
        printf("  quad layout        %8.3f ms  %7.1f G blocks/s  %5.2f clk/block/CU at %.1f GHz\n", ms, blocks / ms / 1e6,
               ms * 1e-3 * ghz * 1e9 * cus / blocks, ghz);
    }

    printf("\n16 lookups per lane and step, G of them gathered from a 1-KiB global table (buffer_load_dword), the rest from LDS\n");
    {
        uint32_t *table;
        CK(hipMalloc(&table, 1024));
        CK(hipMemset(table, 0x5a, 1024));
        CK(hipFuncSetAttribute((const void *)gather_mix<0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
        CK(hipFuncSetAttribute((const void *)gather_mix<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
        CK(hipFuncSetAttribute((const void *)gather_mix<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
        CK(hipFuncSetAttribute((const void *)gather_mix<16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
        const int iters = 4000;
        const double lookups = (double)cus * kThreads * iters * 16;
        const int gs[4] = { 0, 1, 2, 16 };
        for (int i = 0; i < 4; i++) {
            int rc = 0;
            if (i == 0) rc = time_launch([&] { hipLaunchKernelGGL(gather_mix<0>, dim3(cus), dim3(kThreads), kLdsBytes, 0, out, table, iters); }, &ms);
            if (i == 1) rc = time_launch([&] { hipLaunchKernelGGL(gather_mix<1>, dim3(cus), dim3(kThreads), kLdsBytes, 0, out, table, iters); }, &ms);
            if (i == 2) rc = time_launch([&] { hipLaunchKernelGGL(gather_mix<2>, dim3(cus), dim3(kThreads), kLdsBytes, 0, out, table, iters); }, &ms);
            if (i == 3) rc = time_launch([&] { hipLaunchKernelGGL(gather_mix<16>, dim3(cus), dim3(kThreads), kLdsBytes, 0, out, table, iters); }, &ms);
            if (rc) return 1;
            printf("  G = %2d  %8.3f ms  %6.2f lookups/clk/CU in all, %5.2f of them gathered\n", gs[i], ms,
                   lookups / (ms * 1e-3) / cus / (ghz * 1e9), lookups * gs[i] / 16 / (ms * 1e-3) / cus / (ghz * 1e9));
        }
        CK(hipFree(table));
    }

    printf("\nboth engines at once: LDS-table engine on one stream, bit-plane engine (4 workgroups of 256 threads per CU) on another\n");
    {
        uint32_t *out2;
        CK(hipMalloc(&out2, (size_t)cus * 4 * 256 * 4));
        hipStream_t sa, sb;
        CK(hipStreamCreate(&sa));
        CK(hipStreamCreate(&sb));
        hipEvent_t a0, a1, b1;
        CK(hipEventCreate(&a0));
        CK(hipEventCreate(&a1));
        CK(hipEventCreate(&b1));
        const int it_lds = 2000;
        const int bp_iters[3] = { 0, 60, 120 };      // none; about half; about all of the other kernel's duration
        for (int i = 0; i < 3; i++) {
            float best = 1e30f;
            for (int rep = 0; rep < 3; rep++) {
                CK(hipDeviceSynchronize());
                CK(hipEventRecord(a0, sa));
                hipLaunchKernelGGL(lds_engine, dim3(cus), dim3(kThreads), kLdsBytes, sa, out, it_lds);
                if (bp_iters[i]) hipLaunchKernelGGL(bitplane_engine_small, dim3(cus * 4), dim3(256), 0, sb, out2, bp_iters[i]);
                CK(hipEventRecord(a1, sa));
                CK(hipEventRecord(b1, sb));
                CK(hipDeviceSynchronize());
                CK(hipGetLastError());
                float ta, tb;
                CK(hipEventElapsedTime(&ta, a0, a1));
                CK(hipEventElapsedTime(&tb, a0, b1));
                const float span = ta > tb ? ta : tb;
                if (span < best) best = span;
            }
            const double b_lds = (double)cus * kThreads * it_lds * 2, b_bp = (double)cus * 4 * 256 * bp_iters[i] * 8;
            printf("  bit-plane iterations %3d  %8.3f ms  %6.1f G + %5.1f G = %6.1f G blocks/s\n", bp_iters[i], best, b_lds / best / 1e6,
                   b_bp / best / 1e6, (b_lds + b_bp) / best / 1e6);
        }
        CK(hipFree(out2));
    }
    CK(hipFree(out));
    return 0;
}
