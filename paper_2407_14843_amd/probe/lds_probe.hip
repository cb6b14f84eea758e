// LDS read-bandwidth and vector-issue probes.  Not part of the solve and not
// part of its library: a small library of its own (libthemis_probe.so) that the
// benchmark loads to measure the figures the kernels' rooflines are priced
// against.  Every lane of every wavefront streams instructions of one kind and
// nothing else; the caller times the launch.
//
//   probe_lds_read(width, misalign, iters, blocks, d_sink, stream)
//     conflict-free LDS reads of `width` bytes (4, 8 or 16) at byte misalignment
//     `misalign` (0, or 2/4/8 where smaller than the width; with width 8, -1 = two
//     adjacent dwords by ds_read2_b32 at 4-byte alignment, -2 = ds_read2st64_b32).
//     One launch reads blocks * 1024 * iters * 4 * width bytes.
//   probe_valu(op, iters, blocks, d_sink, stream)
//     iters * 16 independent vector instructions per lane (op 0 v_pk_add_u16,
//     1 v_pk_min_u16, 2 v_add_u32, 3 v_min_u32, 4 the two packed ones alternating,
//     5 v_pk_add_u16 with a scalar operand; 6..20 double-precision and integer
//     instructions of the candidate stage; 21..24 address and operand-select forms
//     of the min-plus stage).  One launch issues blocks * 256 * iters * 16
//     lane-instructions.
// Both return 0, -1 (null sink), -2 (unsupported combination) or -6 (launch
// refused).  d_sink is one uint32 of device memory; stream a hipStream_t.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace themis {
namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 1024;
constexpr int PROBE_LDS = 65536 + 256;

// WIDTH: bytes per lane per read (4, 8 or 16).  MIS: byte offset added to every
// address (0 = naturally aligned).
template <int WIDTH, int MIS>
__global__ __launch_bounds__(PROBE_THREADS) void k_lds_probe(uint32_t* __restrict__ sink,
                                                             int iters)
{
    extern __shared__ uint32_t lds[];
    for (int x = threadIdx.x; x < PROBE_LDS / 4; x += PROBE_THREADS) lds[x] = x;
    __syncthreads();
    // 1024 lanes * WIDTH bytes per sweep; four sweeps 16 KB apart per block of reads
    const uint32_t addr = (uint32_t)(uintptr_t)lds + (threadIdx.x * WIDTH) % 16384 + (MIS > 0 ? MIS : 0);
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
        if constexpr (WIDTH == 4) {
            uint32_t a, b, c, d;
            asm volatile(
                "ds_read_b32 %0, %4\n ds_read_b32 %1, %4 offset:16384\n"
                "ds_read_b32 %2, %4 offset:32768\n ds_read_b32 %3, %4 offset:49152\n"
                "s_waitcnt lgkmcnt(0)"
                : "=v"(a), "=v"(b), "=v"(c), "=v"(d) : "v"(addr));
            acc ^= a ^ b ^ c ^ d;
        } else if constexpr (WIDTH == 8 && MIS == -1) {
            // two adjacent dwords through ds_read2_b32, base only 4-byte aligned
            u32x2 a, b, c, d;
            const uint32_t ad = addr + 4;
            asm volatile(
                "ds_read2_b32 %0, %4 offset1:1\n ds_read2_b32 %1, %5 offset1:1\n"
                "ds_read2_b32 %2, %6 offset1:1\n ds_read2_b32 %3, %7 offset1:1\n"
                "s_waitcnt lgkmcnt(0)"
                : "=v"(a), "=v"(b), "=v"(c), "=v"(d)
                : "v"(ad), "v"(ad + 16384), "v"(ad + 32768), "v"(ad + 49152));
            acc ^= a.x ^ b.x ^ c.x ^ d.x;
        } else if constexpr (WIDTH == 8 && MIS == -2) {
            // two dwords 256 bytes apart through ds_read2st64_b32 (what a 4-byte
            // unit-stride loop unrolled by two compiles to)
            u32x2 a, b, c, d;
            const uint32_t ad = (uint32_t)(uintptr_t)lds + (threadIdx.x & 63) * 4 +
                                (threadIdx.x >> 6) * 512;
            asm volatile(
                "ds_read2st64_b32 %0, %4 offset1:1\n ds_read2st64_b32 %1, %5 offset1:1\n"
                "ds_read2st64_b32 %2, %6 offset1:1\n ds_read2st64_b32 %3, %7 offset1:1\n"
                "s_waitcnt lgkmcnt(0)"
                : "=v"(a), "=v"(b), "=v"(c), "=v"(d)
                : "v"(ad), "v"(ad + 16384), "v"(ad + 32768), "v"(ad + 49152));
            acc ^= a.x ^ b.x ^ c.x ^ d.x;
        } else if constexpr (WIDTH == 8) {
            u32x2 a, b, c, d;
            asm volatile(
                "ds_read_b64 %0, %4\n ds_read_b64 %1, %4 offset:16384\n"
                "ds_read_b64 %2, %4 offset:32768\n ds_read_b64 %3, %4 offset:49152\n"
                "s_waitcnt lgkmcnt(0)"
                : "=v"(a), "=v"(b), "=v"(c), "=v"(d) : "v"(addr));
            acc ^= a.x ^ b.x ^ c.x ^ d.x;
        } else {
            u32x4 a, b, c, d;
            asm volatile(
                "ds_read_b128 %0, %4\n ds_read_b128 %1, %4 offset:16384\n"
                "ds_read_b128 %2, %4 offset:32768\n ds_read_b128 %3, %4 offset:49152\n"
                "s_waitcnt lgkmcnt(0)"
                : "=v"(a), "=v"(b), "=v"(c), "=v"(d) : "v"(addr));
            acc ^= a.x ^ b.x ^ c.x ^ d.x;
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;  // keeps the reads alive
}

// VALU issue-rate probe: every lane runs `iters` rounds of 16 independent
// instructions of one kind (or add/min alternating), nothing else.
template <int OP>
__global__ __launch_bounds__(256) void k_valu_probe(uint32_t* __restrict__ sink, int iters,
                                                    uint32_t seed)
{
    uint32_t r[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) r[j] = seed * (threadIdx.x + 1) + j;
    const uint32_t c = seed | 0x00010001u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if constexpr (OP == 0) asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(r[j]) : "v"(c));
            if constexpr (OP == 1) asm volatile("v_pk_min_u16 %0, %0, %1" : "+v"(r[j]) : "v"(c));
            if constexpr (OP == 2) asm volatile("v_add_u32 %0, %0, %1" : "+v"(r[j]) : "v"(c));
            if constexpr (OP == 3) asm volatile("v_min_u32 %0, %0, %1" : "+v"(r[j]) : "v"(c));
            if constexpr (OP == 4) {
                if (j & 1)
                    asm volatile("v_pk_min_u16 %0, %0, %1" : "+v"(r[j]) : "v"(r[j - 1]));
                else
                    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(r[j]) : "v"(c));
            }
            if constexpr (OP == 5) asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(r[j]) : "s"(c));
        }
    }
    uint32_t x = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) x ^= r[j];
    if (x == 0x12345678u) sink[0] = x;
}

// The same for the double-precision and conversion instructions the candidate
// kernel is made of: 8 independent register pairs per lane, 16 instructions a round.
template <int OP>
__global__ __launch_bounds__(256) void k_valu64_probe(uint32_t* __restrict__ sink, int iters,
                                                      uint32_t seed)
{
    double r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = 1.0 + 1e-3 * (double)(seed * (threadIdx.x + 1) + j);
    const double c = 1.0 + 1e-9 * (double)seed;
    uint32_t u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) u[j] = seed + j;
    unsigned long long mask = 0x5555555555555555ull * seed;  // uniform: lives in an SGPR pair
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if constexpr (OP == 6) asm volatile("v_fma_f64 %0, %0, %1, %1" : "+v"(r[j]) : "v"(c));
                if constexpr (OP == 7) asm volatile("v_mul_f64 %0, %0, %1" : "+v"(r[j]) : "v"(c));
                if constexpr (OP == 8) asm volatile("v_add_f64 %0, %0, %1" : "+v"(r[j]) : "v"(c));
                if constexpr (OP == 9) asm volatile("v_floor_f64 %0, %0" : "+v"(r[j]));
                if constexpr (OP == 10) asm volatile("v_rcp_f64 %0, %0" : "+v"(r[j]));
                if constexpr (OP == 11) asm volatile("v_cvt_f64_u32 %0, %1" : "=v"(r[j]) : "v"(u[j]));
                if constexpr (OP == 12) asm volatile("v_cvt_u32_f64 %0, %1" : "=v"(u[j]) : "v"(r[j]));
                if constexpr (OP == 13) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(u[j]) : "v"(seed));
                if constexpr (OP == 14)
                    asm volatile("v_cmp_ge_f64 vcc, %0, %1" : : "v"(r[j]), "v"(c) : "vcc");
                if constexpr (OP == 15)
                    asm volatile("v_cndmask_b32 %0, %0, %1, vcc" : "+v"(u[j]) : "v"(seed) : "vcc");
                if constexpr (OP == 16) asm volatile("v_mul_u32_u24 %0, %0, %1" : "+v"(u[j]) : "v"(seed));
                if constexpr (OP == 17)
                    asm volatile("v_cndmask_b32_e64 %0, %0, %1, %2"
                                 : "+v"(u[j]) : "v"(seed), "s"(mask));
                if constexpr (OP == 18) asm volatile("v_max_f64 %0, %0, %1" : "+v"(r[j]) : "v"(c));
                if constexpr (OP == 19)
                    asm volatile("v_add_f64 %0, %0, %1 clamp" : "+v"(r[j]) : "v"(c));
                if constexpr (OP == 20)
                    asm volatile("v_cmp_ge_f64_e64 %0, %1, %2" : "=s"(mask) : "v"(r[j]), "v"(c));
                if constexpr (OP == 21)
                    asm volatile("v_mad_u32_u16 %0, %0, 4, %1" : "+v"(u[j]) : "v"(seed));
                if constexpr (OP == 22)
                    asm volatile("v_pk_add_u16 %0, %0, %1 op_sel:[0,1] op_sel_hi:[1,1]"
                                 : "+v"(u[j]) : "v"(seed));
                if constexpr (OP == 23)
                    asm volatile("v_lshl_add_u32 %0, %0, 2, %1" : "+v"(u[j]) : "v"(seed));
                if constexpr (OP == 24)
                    asm volatile("v_add_u32_sdwa %0, %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD "
                                 "src0_sel:WORD_0 src1_sel:DWORD" : "+v"(u[j]) : "v"(seed));
            }
    }
    double x = 0;
    uint32_t y = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        x += r[j];
        y ^= u[j];
    }
    if (x == 0.123456 || y == 0x12345678u || mask == 1ull) sink[0] = y;
}

template <int WIDTH, int MIS>
hipError_t launch_probe(uint32_t* sink, int iters, int blocks, hipStream_t st)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_lds_probe<WIDTH, MIS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PROBE_LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_lds_probe<WIDTH, MIS>), dim3(blocks), dim3(PROBE_THREADS), PROBE_LDS,
                       st, sink, iters);
    return hipGetLastError();
}

}  // namespace

// bytes read by one launch: blocks * 1024 lanes * iters * 4 reads * width
hipError_t launch_lds_probe(int width, int misalign, int iters, int blocks, uint32_t* sink,
                            hipStream_t st)
{
#define PROBE_CASE(W, M) \
    if (width == W && misalign == M) return launch_probe<W, M>(sink, iters, blocks, st)
    PROBE_CASE(4, 0);
    PROBE_CASE(4, 2);
    PROBE_CASE(8, 0);
    PROBE_CASE(8, 4);
    PROBE_CASE(8, 2);
    PROBE_CASE(8, -1);
    PROBE_CASE(8, -2);
    PROBE_CASE(16, 0);
    PROBE_CASE(16, 8);
    PROBE_CASE(16, 4);
    PROBE_CASE(16, 2);
#undef PROBE_CASE
    return hipErrorInvalidValue;
}

// one launch issues blocks * 256 lanes * iters * 16 instructions
hipError_t launch_valu_probe(int op, int iters, int blocks, uint32_t* sink, hipStream_t st)
{
#define VALU_CASE(O) \
    if (op == O) { \
        hipLaunchKernelGGL(k_valu_probe<O>, dim3(blocks), dim3(256), 0, st, sink, iters, 3u); \
        return hipGetLastError(); \
    }
    VALU_CASE(0) VALU_CASE(1) VALU_CASE(2) VALU_CASE(3) VALU_CASE(4) VALU_CASE(5)
#undef VALU_CASE
#define VALU64_CASE(O) \
    if (op == O) { \
        hipLaunchKernelGGL(k_valu64_probe<O>, dim3(blocks), dim3(256), 0, st, sink, iters, 3u); \
        return hipGetLastError(); \
    }
    VALU64_CASE(6) VALU64_CASE(7) VALU64_CASE(8) VALU64_CASE(9) VALU64_CASE(10) VALU64_CASE(11)
    VALU64_CASE(12) VALU64_CASE(13) VALU64_CASE(14) VALU64_CASE(15) VALU64_CASE(16)
    VALU64_CASE(17) VALU64_CASE(18) VALU64_CASE(19) VALU64_CASE(20)
    VALU64_CASE(21) VALU64_CASE(22) VALU64_CASE(23) VALU64_CASE(24)
#undef VALU64_CASE
    return hipErrorInvalidValue;
}

}  // namespace themis

extern "C" {

int probe_lds_read(int width, int misalign, int iters, int blocks, uint32_t* d_sink, void* stream)
{
    if (!d_sink) return -1;
    if (iters < 1 || blocks < 1 || blocks > 65536) return -2;
    hipError_t e = themis::launch_lds_probe(width, misalign, iters, blocks, d_sink,
                                            static_cast<hipStream_t>(stream));
    if (e == hipErrorInvalidValue) return -2;
    return e == hipSuccess ? 0 : -6;
}

int probe_valu(int op, int iters, int blocks, uint32_t* d_sink, void* stream)
{
    if (!d_sink) return -1;
    if (iters < 1 || blocks < 1 || blocks > 65536) return -2;
    hipError_t e = themis::launch_valu_probe(op, iters, blocks, d_sink,
                                             static_cast<hipStream_t>(stream));
    if (e == hipErrorInvalidValue) return -2;
    return e == hipSuccess ? 0 : -6;
}

}  // extern "C"
