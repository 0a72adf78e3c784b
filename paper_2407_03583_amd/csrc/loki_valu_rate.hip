// Sustained issue rate of the vector-ALU instruction classes the search is made of, measured
// with dependency-free streams (16 independent instructions per loop trip, up to 8 wavefronts
// per SIMD, many more blocks than fit at once).  A measurement aid for the roofline: the nominal peak assumes one vector instruction
// per SIMD every 4 cycles at 2.4 GHz; this tells what the GPU at hand actually sustains.
// Built into a library of its own (libloki_probe.so, include/loki_probe.h): the search library does not carry it.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "../../include/loki_probe.h"

// instruction classes (the `kind` of loki_measure_valu_rate)
#define LOKI_RATE_MUL_F64 0
#define LOKI_RATE_ADD_F64 1
#define LOKI_RATE_MAX_F64 2
#define LOKI_RATE_SEARCH_MIX 3
#define LOKI_RATE_ADD_U32 4
#define LOKI_RATE_FMA_F64 5
#define LOKI_RATE_RCP_F64 6
#define LOKI_RATE_MUL_LO_U32 7
#define LOKI_RATE_MUL_HI_U32 8
#define LOKI_RATE_MIN_U32 9
#define LOKI_RATE_LDS_READ_B64 10
#define LOKI_RATE_LAST LOKI_RATE_LDS_READ_B64

#pragma clang fp contract(off)

namespace loki {

namespace {

#define LOKI_REP16(OP)                                                                              \
    OP " %0, %0, %8\n" OP " %1, %1, %8\n" OP " %2, %2, %8\n" OP " %3, %3, %8\n" OP " %4, %4, %8\n"  \
    OP " %5, %5, %8\n" OP " %6, %6, %8\n" OP " %7, %7, %8\n" OP " %0, %0, %8\n" OP " %1, %1, %8\n"  \
    OP " %2, %2, %8\n" OP " %3, %3, %8\n" OP " %4, %4, %8\n" OP " %5, %5, %8\n" OP " %6, %6, %8\n"  \
    OP " %7, %7, %8\n"

#define LOKI_REP16_UNARY(OP)                                                                      \
    OP " %0, %0\n" OP " %1, %1\n" OP " %2, %2\n" OP " %3, %3\n" OP " %4, %4\n" OP " %5, %5\n"       \
    OP " %6, %6\n" OP " %7, %7\n" OP " %0, %0\n" OP " %1, %1\n" OP " %2, %2\n" OP " %3, %3\n"       \
    OP " %4, %4\n" OP " %5, %5\n" OP " %6, %6\n" OP " %7, %7\n"

#define LOKI_REP16_FMA(OP)                                                                                  \
    OP " %0, %0, %8, %8\n" OP " %1, %1, %8, %8\n" OP " %2, %2, %8, %8\n" OP " %3, %3, %8, %8\n"            \
    OP " %4, %4, %8, %8\n" OP " %5, %5, %8, %8\n" OP " %6, %6, %8, %8\n" OP " %7, %7, %8, %8\n"            \
    OP " %0, %0, %8, %8\n" OP " %1, %1, %8, %8\n" OP " %2, %2, %8, %8\n" OP " %3, %3, %8, %8\n"            \
    OP " %4, %4, %8, %8\n" OP " %5, %5, %8, %8\n" OP " %6, %6, %8, %8\n" OP " %7, %7, %8, %8\n"

// 16 reads of 8 bytes per lane (consecutive lanes 8 bytes apart: no bank conflicts), waited for once
#define LOKI_REP16_LDS                                                                                      \
    "ds_read_b64 %0, %8\n ds_read_b64 %1, %8 offset:2048\n ds_read_b64 %2, %8 offset:4096\n"                 \
    "ds_read_b64 %3, %8 offset:6144\n ds_read_b64 %4, %8\n ds_read_b64 %5, %8 offset:2048\n"                 \
    "ds_read_b64 %6, %8 offset:4096\n ds_read_b64 %7, %8 offset:6144\n ds_read_b64 %0, %8\n"                 \
    "ds_read_b64 %1, %8 offset:2048\n ds_read_b64 %2, %8 offset:4096\n ds_read_b64 %3, %8 offset:6144\n"     \
    "ds_read_b64 %4, %8\n ds_read_b64 %5, %8 offset:2048\n ds_read_b64 %6, %8 offset:4096\n"                 \
    "ds_read_b64 %7, %8 offset:6144\n s_waitcnt lgkmcnt(0)\n"

template <int KIND>
__global__ void __launch_bounds__(256) valu_rate_kernel(double *out, int iters, double seed) {
    double a0 = seed, a1 = seed * 2, a2 = seed * 3, a3 = seed * 4, a4 = seed * 5, a5 = seed * 6, a6 = seed * 7,
           a7 = seed * 8;
    const double c = 1.0 - 1e-9;
    uint32_t u0 = threadIdx.x + 1, u1 = u0 + 1, u2 = u0 + 2, u3 = u0 + 3, u4 = u0 + 4, u5 = u0 + 5, u6 = u0 + 6, u7 = u0 + 7;
    const uint32_t uc = 2654435761u;
    __shared__ double sLds[KIND == LOKI_RATE_LDS_READ_B64 ? 1024 : 1];
    // byte address in LDS: the low half of a generic pointer into LDS is the offset within LDS
    const uint32_t lds_at = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(&sLds[0])) + threadIdx.x * 8;
    if (KIND == LOKI_RATE_LDS_READ_B64) {
        for (int q = threadIdx.x; q < 1024; q += 256) sLds[q] = seed + q;
        __syncthreads();
    }
    for (int it = 0; it < iters; it++) {
        if (KIND == LOKI_RATE_FMA_F64)
            asm volatile(LOKI_REP16_FMA("v_fma_f64")
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                         : "v"(c));
        if (KIND == LOKI_RATE_RCP_F64)
            asm volatile(LOKI_REP16_UNARY("v_rcp_f64")
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                         : "v"(c));
        if (KIND == LOKI_RATE_MUL_LO_U32)
            asm volatile(LOKI_REP16("v_mul_lo_u32")
                         : "+v"(u0), "+v"(u1), "+v"(u2), "+v"(u3), "+v"(u4), "+v"(u5), "+v"(u6), "+v"(u7)
                         : "v"(uc));
        if (KIND == LOKI_RATE_MUL_HI_U32)
            asm volatile(LOKI_REP16("v_mul_hi_u32")
                         : "+v"(u0), "+v"(u1), "+v"(u2), "+v"(u3), "+v"(u4), "+v"(u5), "+v"(u6), "+v"(u7)
                         : "v"(uc));
        if (KIND == LOKI_RATE_MIN_U32)
            asm volatile(LOKI_REP16("v_min_u32")
                         : "+v"(u0), "+v"(u1), "+v"(u2), "+v"(u3), "+v"(u4), "+v"(u5), "+v"(u6), "+v"(u7)
                         : "v"(uc));
        if (KIND == LOKI_RATE_LDS_READ_B64)
            asm volatile(LOKI_REP16_LDS
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                         : "v"(lds_at)
                         : "memory");
        if (KIND == LOKI_RATE_MUL_F64)
            asm volatile(LOKI_REP16("v_mul_f64")
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                         : "v"(c));
        if (KIND == LOKI_RATE_ADD_F64)
            asm volatile(LOKI_REP16("v_add_f64")
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                         : "v"(c));
        if (KIND == LOKI_RATE_MAX_F64)
            asm volatile(LOKI_REP16("v_max_f64")
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                         : "v"(c));
        if (KIND == LOKI_RATE_SEARCH_MIX)  // the inner loop of the search: multiply, add, running maximum
            asm volatile(
                "v_mul_f64 %0, %4, %8\n v_add_f64 %0, %0, %5\n v_max_f64 %7, %7, %0\n"
                "v_mul_f64 %1, %4, %8\n v_add_f64 %1, %1, %5\n v_max_f64 %7, %7, %1\n"
                "v_mul_f64 %2, %4, %8\n v_add_f64 %2, %2, %5\n v_max_f64 %7, %7, %2\n"
                "v_mul_f64 %3, %4, %8\n v_add_f64 %3, %3, %5\n v_max_f64 %7, %7, %3\n"
                "v_mul_f64 %0, %6, %8\n v_add_f64 %0, %0, %5\n v_max_f64 %7, %7, %0\n"
                "v_mul_f64 %1, %6, %8\n"
                : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
                : "v"(c));
        if (KIND == LOKI_RATE_ADD_U32) {
            int x0 = it, x1 = it + 1, x2 = it + 2, x3 = it + 3;
            asm volatile(
                "v_add_u32 %0, %0, %4\n v_add_u32 %1, %1, %4\n v_add_u32 %2, %2, %4\n v_add_u32 %3, %3, %4\n"
                "v_add_u32 %0, %0, %4\n v_add_u32 %1, %1, %4\n v_add_u32 %2, %2, %4\n v_add_u32 %3, %3, %4\n"
                "v_add_u32 %0, %0, %4\n v_add_u32 %1, %1, %4\n v_add_u32 %2, %2, %4\n v_add_u32 %3, %3, %4\n"
                "v_add_u32 %0, %0, %4\n v_add_u32 %1, %1, %4\n v_add_u32 %2, %2, %4\n v_add_u32 %3, %3, %4\n"
                : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
                : "v"(it));
            a0 += x0 + x1 + x2 + x3;
        }
    }
    // the sink only keeps the arithmetic alive; blocks 2048 apart share a slot
    out[(blockIdx.x & 2047) * 256 + threadIdx.x] =
        a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7 + static_cast<double>(u0 ^ u1 ^ u2 ^ u3 ^ u4 ^ u5 ^ u6 ^ u7);
}

}  // namespace

// `out` needs 2048 * 256 doubles (a sink shared by blocks 2048 apart); every thread runs iters trips
// of 16 instructions
static hipError_t launch_valu_rate(int kind, double *out, int blocks, int iters, hipStream_t stream) {
    const dim3 grid(blocks), block(256);
    switch (kind) {
        case LOKI_RATE_MUL_F64: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_MUL_F64>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_ADD_F64: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_ADD_F64>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_MAX_F64: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_MAX_F64>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_SEARCH_MIX: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_SEARCH_MIX>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_ADD_U32: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_ADD_U32>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_FMA_F64: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_FMA_F64>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_RCP_F64: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_RCP_F64>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_MUL_LO_U32: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_MUL_LO_U32>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_MUL_HI_U32: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_MUL_HI_U32>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_MIN_U32: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_MIN_U32>, grid, block, 0, stream, out, iters, 0.5); break;
        case LOKI_RATE_LDS_READ_B64: hipLaunchKernelGGL(valu_rate_kernel<LOKI_RATE_LDS_READ_B64>, grid, block, 0, stream, out, iters, 0.5); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace loki

extern "C" int loki_measure_valu_rate(int kind, void *d_workspace, size_t workspace_bytes, void *hip_stream,
                                      double *wave_instructions_per_second, int *hip_error) {
    if (!d_workspace || !wave_instructions_per_second) return -1;
    if (kind < 0 || kind > LOKI_RATE_LAST) return -6;
    // many short blocks: the block dispatcher then keeps every SIMD full to the end, as in the search
    // (fewer trips for the classes that issue at a quarter of the rate or less)
    const bool slow = kind == LOKI_RATE_RCP_F64 || kind == LOKI_RATE_MUL_LO_U32 || kind == LOKI_RATE_MUL_HI_U32 ||
                      kind == LOKI_RATE_LDS_READ_B64;
    const int blocks = 32768, iters = slow ? 1000 : 6250, sink_blocks = 2048;
    if (workspace_bytes < size_t(sink_blocks) * 256 * sizeof(double) || (reinterpret_cast<uintptr_t>(d_workspace) % 8) != 0)
        return -4;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    double *out = static_cast<double *>(d_workspace);
    if (e == hipSuccess) e = loki::launch_valu_rate(kind, out, blocks, 100, stream);  // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, stream);
    if (e == hipSuccess) e = loki::launch_valu_rate(kind, out, blocks, iters, stream);
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) {
        if (hip_error) *hip_error = static_cast<int>(e);
        return -5;
    }
    *wave_instructions_per_second = double(blocks) * 4.0 * double(iters) * 16.0 / (double(ms) * 1e-3);
    return 0;
}
