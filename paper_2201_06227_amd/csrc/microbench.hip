// Micro-measurements of what one MI355X delivers to kernels shaped like the ones in this library: sustained
// issue rate of the matrix instructions they use, LDS read and write rates of 128-bit accesses, the rate at which
// rows of an L2-resident operand panel reach LDS through buffer loads with the LDS modifier (whole 128-byte
// lines per row against half lines), and a plain HBM copy.  Every kernel is a complete small program; the
// figures ground the per-kernel rooflines.  Benchmark instrumentation, not part of the method.
#include "common.hpp"

namespace egeria {

typedef int mb_v4i __attribute__((ext_vector_type(4)));
typedef int mb_v16i __attribute__((ext_vector_type(16)));
typedef float mb_v16f __attribute__((ext_vector_type(16)));
typedef float mb_v4f __attribute__((ext_vector_type(4)));
typedef double mb_v4d __attribute__((ext_vector_type(4)));
typedef __bf16 mb_v8bf __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) uint8_t mb_lds_byte;

namespace {

// KIND 0: i32_32x32x32_i8, 1: f32_32x32x16_bf16, 2: f32_32x32x2_f32, 3: f32_16x16x4_f32, 4: f64_16x16x4_f64.
// Four independent accumulator blocks per wave, issued round robin; the result is stored when it matches a
// value it cannot have, so the chain stays live.
template <int KIND>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, int *sink)
{
    const int t = threadIdx.x;
    if constexpr (KIND == 0) {
        mb_v16i acc[4] = {};
        const mb_v4i a = {t, 1, 2, 3}, b = {3, 2, 1, t};
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
        int s = 0;
        for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
        if (s == 0x7fffffff) sink[0] = s;
    } else if constexpr (KIND == 1) {
        mb_v16f acc[4] = {};
        mb_v8bf a, b;
        for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(t + e); b[e] = (__bf16)1.5f; }
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        float s = 0;
        for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
        if (s == 12345.f) sink[0] = 1;
    } else if constexpr (KIND == 2) {
        mb_v16f acc[4] = {};
        const float a = (float)t, b = 1.5f;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
        float s = 0;
        for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
        if (s == 12345.f) sink[0] = 1;
    } else if constexpr (KIND == 3) {
        mb_v4f acc[4] = {};
        const float a = (float)t, b = 1.5f;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
        float s = 0;
        for (int i = 0; i < 4; ++i) for (int r = 0; r < 4; ++r) s += acc[i][r];
        if (s == 12345.f) sink[0] = 1;
    } else {
        mb_v4d acc[4] = {};
        const double a = (double)t, b = 1.5;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[i], 0, 0, 0);
        double s = 0;
        for (int i = 0; i < 4; ++i) for (int r = 0; r < 4; ++r) s += acc[i][r];
        if (s == 12345.) sink[0] = 1;
    }
}

// One dependent chain of bf16 matrix instructions per wave (each takes the result of the one before as its
// accumulator); VALU: eight fp32 multiply-adds that depend on no matrix result follow each of them in issue
// order.  The work reported is that of the matrix instructions only, so the three variants compare directly:
// what a dependent chain reaches alone, and what is left of it when the vector ALU of the same SIMD is in use.
template <bool VALU>
__global__ __launch_bounds__(256) void mfma_chain_kernel(int iters, int *sink)
{
    const int t = threadIdx.x;
    mb_v16f acc = {};
    mb_v8bf a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(t + e); b[e] = (__bf16)1.5f; }
    float x[8];
    for (int e = 0; e < 8; ++e) x[e] = (float)(t + e);
    const float m = 1.0f - 1.0f / (float)(iters + 3), c = 0.25f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
            if (VALU) {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = fmaf(x[e], m, c);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
            }
        }
    }
    float s = 0;
    for (int r = 0; r < 16; ++r) s += acc[r];
    for (int e = 0; e < 8; ++e) s += x[e];
    if (s == 12345.f) sink[0] = 1;
}

// 128-bit LDS accesses without bank conflicts (lane l at byte 16 l of a 1 KiB row per wave), eight per iteration.
template <bool WRITE>
__global__ __launch_bounds__(256) void lds_rate_kernel(int iters, int *sink)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[32768];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 8192; i += 256) ((int *)lds)[i] = i;
    __syncthreads();
    const uint32_t off = (uint32_t)(uintptr_t)(mb_lds_byte *)lds + wave * 8192 + lane * 16;
    mb_v4i r[8] = {};
    mb_v4i v = {lane, 1, 2, 3};
    for (int it = 0; it < iters; ++it) {
        if (WRITE)
            asm volatile("ds_write_b128 %0, %1\n ds_write_b128 %0, %1 offset:1024\n ds_write_b128 %0, %1 offset:2048\n"
                         "ds_write_b128 %0, %1 offset:3072\n ds_write_b128 %0, %1 offset:4096\n ds_write_b128 %0, %1 offset:5120\n"
                         "ds_write_b128 %0, %1 offset:6144\n ds_write_b128 %0, %1 offset:7168\n s_waitcnt lgkmcnt(0)" ::"v"(off), "v"(v) : "memory");
        else
            asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:1024\n ds_read_b128 %2, %8 offset:2048\n"
                         "ds_read_b128 %3, %8 offset:3072\n ds_read_b128 %4, %8 offset:4096\n ds_read_b128 %5, %8 offset:5120\n"
                         "ds_read_b128 %6, %8 offset:6144\n ds_read_b128 %7, %8 offset:7168\n s_waitcnt lgkmcnt(0)"
                         : "=v"(r[0]), "=v"(r[1]), "=v"(r[2]), "=v"(r[3]), "=v"(r[4]), "=v"(r[5]), "=v"(r[6]), "=v"(r[7])
                         : "v"(off) : "memory");
    }
    __syncthreads();
    const mb_v4i s = r[0] ^ r[1] ^ r[2] ^ r[3] ^ r[4] ^ r[5] ^ r[6] ^ r[7];
    if (s[0] == 0x12345678 || ((int *)lds)[threadIdx.x] == 0x12345679) sink[0] = 1;
}

// Rows of an operand panel from L2 into LDS: every workgroup re-reads its own 64 KiB panel (resident in L2
// after the first pass), eight 1-KiB requests per wave and step, three steps in flight.  ROW_BYTES = 128: a
// request covers 8 rows x one whole 128-byte line; 64: 16 rows x half a line (row stride 128 bytes).
template <int ROW_BYTES>
__global__ __launch_bounds__(256) void panel_to_lds_kernel(const uint8_t *base, int iters, int *sink)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];       // four slots of 32 KiB
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int UPR = ROW_BYTES / 16, RPC = 64 / UPR, NLD = 8, KSTEPS = 128 / ROW_BYTES;
    constexpr uint32_t wg_bytes = 65536;
    const uint64_t a = (uint64_t)(base + (uint64_t)blockIdx.x * wg_bytes);
    mb_v4i d;
    d[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    d[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32) & 0xffff);
    d[2] = (int)wg_bytes;
    d[3] = 0x00020000;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(mb_lds_byte *)lds;
    uint32_t rowoff[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) rowoff[j] = (uint32_t)(((wave + 4 * j) * RPC + lane / UPR) * 128 + (lane % UPR) * 16);
    int k = 0, slot = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NLD; ++j)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :: "s"(lds0 + slot * 32768 + (wave + 4 * j) * 1024), "v"(rowoff[j] + k * ROW_BYTES), "s"(d) : "memory", "m0");
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        k = k + 1 == KSTEPS ? 0 : k + 1;
        slot = slot + 1 == 4 ? 0 : slot + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (lds[threadIdx.x] == 0x5a && iters < 0) sink[0] = 1;
}

__global__ __launch_bounds__(256) void copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, int64_t n4)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

}  // namespace

}  // namespace egeria

using namespace egeria;

#define EG_HIP(expr)                                   \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) return EGERIA_ERR_HIP;  \
    } while (0)

extern "C" egeria_status egeria_microbench(int32_t kind, int32_t iters, void *scratch, size_t scratch_bytes, float *ms_out,
                                           double *work_out, void *stream)
{
    if (!ms_out || !work_out || iters < 1 || !scratch || scratch_bytes < (size_t)(256u << 20)) return EGERIA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int cus = compute_units();
    hipEvent_t e0, e1;
    EG_HIP(hipEventCreate(&e0));
    EG_HIP(hipEventCreate(&e1));
    int *sink = (int *)scratch;
    const dim3 block(256);
    const dim3 two_per_cu((unsigned)(2 * cus)), one_per_cu((unsigned)cus);
    double work = 0.0;
    for (int rep = 0; rep < 2; ++rep) {                   // the first pass warms caches and code
        EG_HIP(hipEventRecord(e0, st));
        switch (kind) {
        case EGERIA_MICRO_MFMA_I8: hipLaunchKernelGGL(mfma_rate_kernel<0>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 4.0 * iters * 65536.0; break;
        case EGERIA_MICRO_MFMA_BF16: hipLaunchKernelGGL(mfma_rate_kernel<1>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 4.0 * iters * 32768.0; break;
        case EGERIA_MICRO_MFMA_F32_32: hipLaunchKernelGGL(mfma_rate_kernel<2>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 4.0 * iters * 4096.0; break;
        case EGERIA_MICRO_MFMA_F32_16: hipLaunchKernelGGL(mfma_rate_kernel<3>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 4.0 * iters * 2048.0; break;
        case EGERIA_MICRO_MFMA_F64: hipLaunchKernelGGL(mfma_rate_kernel<4>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 4.0 * iters * 2048.0; break;
        case EGERIA_MICRO_LDS_READ: hipLaunchKernelGGL(lds_rate_kernel<false>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 8.0 * iters * 1024.0; break;
        case EGERIA_MICRO_LDS_WRITE: hipLaunchKernelGGL(lds_rate_kernel<true>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 8.0 * iters * 1024.0; break;
        case EGERIA_MICRO_L2_TO_LDS_LINE:
        case EGERIA_MICRO_L2_TO_LDS_HALF: {
            static bool set[2] = {false, false};
            const int half = kind == EGERIA_MICRO_L2_TO_LDS_HALF;
            const void *fn = half ? (const void *)panel_to_lds_kernel<64> : (const void *)panel_to_lds_kernel<128>;
            if (!set[half]) {
                EG_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 32768));
                set[half] = true;
            }
            const uint8_t *panels = (const uint8_t *)scratch + 4096;
            if (half) hipLaunchKernelGGL(panel_to_lds_kernel<64>, one_per_cu, block, 4 * 32768, st, panels, iters, sink);
            else hipLaunchKernelGGL(panel_to_lds_kernel<128>, one_per_cu, block, 4 * 32768, st, panels, iters, sink);
            work = 1.0 * cus * 4 * 8.0 * iters * 1024.0;
            break;
        }
        case EGERIA_MICRO_BF16_CHAIN: hipLaunchKernelGGL(mfma_chain_kernel<false>, one_per_cu, block, 0, st, iters, sink); work = 1.0 * cus * 4 * 4.0 * iters * 32768.0; break;
        case EGERIA_MICRO_BF16_CHAIN_VALU: hipLaunchKernelGGL(mfma_chain_kernel<true>, one_per_cu, block, 0, st, iters, sink); work = 1.0 * cus * 4 * 4.0 * iters * 32768.0; break;
        case EGERIA_MICRO_BF16_CHAIN_VALU2: hipLaunchKernelGGL(mfma_chain_kernel<true>, two_per_cu, block, 0, st, iters, sink); work = 2.0 * cus * 4 * 4.0 * iters * 32768.0; break;
        case EGERIA_MICRO_HBM_COPY: {
            const int64_t n4 = (int64_t)((scratch_bytes / 2) / 16);
            hipLaunchKernelGGL(copy_kernel, dim3((unsigned)(cus * 8)), block, 0, st, (const float4 *)scratch,
                               (float4 *)((char *)scratch + scratch_bytes / 2), n4);
            work = 2.0 * 16.0 * (double)n4;
            break;
        }
        default: return EGERIA_ERR_INVALID_ARG;
        }
        EG_HIP(hipGetLastError());
        EG_HIP(hipEventRecord(e1, st));
        EG_HIP(hipEventSynchronize(e1));
    }
    EG_HIP(hipEventElapsedTime(ms_out, e0, e1));
    *work_out = work;
    EG_HIP(hipEventDestroy(e0));
    EG_HIP(hipEventDestroy(e1));
    return EGERIA_OK;
}
