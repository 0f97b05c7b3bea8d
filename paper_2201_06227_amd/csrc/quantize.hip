// Per-tensor symmetric int8 quantisation (Section 4.1 of the paper: the
// reference model is an int8 post-training-quantised snapshot).  Two coalesced
// HBM passes per tensor: an absolute-maximum reduction, then the map to codes.
#include "common.hpp"
#include <type_traits>

namespace egeria {

// ---- absolute maximum -------------------------------------------------------------
__device__ __forceinline__ uint32_t max4_bits(float4 v)
{
    uint32_t a = abs_bits(v.x), b = abs_bits(v.y), c = abs_bits(v.z), d = abs_bits(v.w);
    a = a > b ? a : b;
    c = c > d ? c : d;
    return a > c ? a : c;
}

// Each workgroup writes the maximum of its grid-stride share to partials[blockIdx.x]
// (bit pattern of |x|, so NaN and Inf order above every finite value).
// (workgroup blk of nblks; a device function so that other kernels can carry the pass along).
template <bool BF16>
__device__ __forceinline__ void absmax_share(const void *__restrict__ xv, int64_t n, uint32_t *__restrict__ partials,
                                             uint32_t *__restrict__ reset, int n_reset, int blk, int nblks)
{
    if (blk == 0) {
        for (int t = threadIdx.x; t < n_reset * kAmaxWays; t += blockDim.x)
            reset[(size_t)(t / kAmaxWays) * kAmaxWays * kAmaxStride + (t % kAmaxWays) * kAmaxStride] = 0u;
        // `reset` is the first atomic slot, kHeaderFixedWords words into the workspace: the header's
        // counter of re-evaluated attention values starts every chain at zero as well
        if (n_reset > 0 && threadIdx.x == 0) reset[kUnsureWord - kHeaderFixedWords] = 0u;
    }
    const int64_t tid = (int64_t)blk * blockDim.x + threadIdx.x;
    const int64_t nthreads = (int64_t)nblks * blockDim.x;
    uint32_t m = 0;
    if (!BF16) {
        const float *x = (const float *)xv;
        const int64_t n4 = n >> 2;
        const float4 *x4 = (const float4 *)x;
        int64_t i = tid;
        for (; i + 3 * nthreads < n4; i += 4 * nthreads) {           // four independent loads in flight
            const float4 v0 = x4[i], v1 = x4[i + nthreads], v2 = x4[i + 2 * nthreads], v3 = x4[i + 3 * nthreads];
            uint32_t a = max4_bits(v0), b = max4_bits(v1), c = max4_bits(v2), d = max4_bits(v3);
            a = a > b ? a : b;
            c = c > d ? c : d;
            a = a > c ? a : c;
            m = m > a ? m : a;
        }
        for (; i < n4; i += nthreads) {
            const uint32_t a = max4_bits(x4[i]);
            m = m > a ? m : a;
        }
        for (int64_t k = (n4 << 2) + tid; k < n; k += nthreads) {
            const uint32_t a = abs_bits(x[k]);
            m = m > a ? m : a;
        }
    } else {
        const uint16_t *x = (const uint16_t *)xv;
        const int64_t n8 = n >> 3;
        const uint4 *x8 = (const uint4 *)x;
        for (int64_t i = tid; i < n8; i += nthreads) {
            uint4 v = x8[i];
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t lo = (w[j] << 16) & 0x7fffffffu, hi = w[j] & 0x7fff0000u;
                lo = lo > hi ? lo : hi;
                m = m > lo ? m : lo;
            }
        }
        for (int64_t i = (n8 << 3) + tid; i < n; i += nthreads) {
            uint32_t a = ((uint32_t)x[i] << 16) & 0x7fffffffu;
            m = m > a ? m : a;
        }
    }
    m = wave_max_u32(m);
    __shared__ uint32_t sm[4];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) sm[wv] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t a = sm[0] > sm[1] ? sm[0] : sm[1], b = sm[2] > sm[3] ? sm[2] : sm[3];
        partials[blk] = a > b ? a : b;
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void absmax_kernel(const void *__restrict__ xv, int64_t n,
                                                     uint32_t *__restrict__ partials,
                                                     uint32_t *__restrict__ reset, int n_reset)
{
    absmax_share<BF16>(xv, n, partials, reset, n_reset, (int)blockIdx.x, (int)gridDim.x);
}

int absmax_blocks(int64_t n, egeria_dtype dt)
{
    const int64_t per = dt == EGERIA_F32 ? 4 : 8;
    int64_t blocks = (n / per + 256 * 4 - 1) / (256 * 4);            // about four vectors per thread
    if (blocks < 1) blocks = 1;
    if (blocks > kAbsPartials) blocks = kAbsPartials;
    return (int)blocks;
}

hipError_t launch_absmax(const void *x, egeria_dtype dt, int64_t n, uint32_t *partials, uint32_t *reset,
                         int n_reset, hipStream_t st)
{
    const dim3 grid((unsigned)absmax_blocks(n, dt)), block(256);
    if (dt == EGERIA_F32)
        return launch_k(EGERIA_KERNEL_ABSMAX, absmax_kernel<false>, grid, block, 0, st, x, n, partials, reset, n_reset);
    return launch_k(EGERIA_KERNEL_ABSMAX, absmax_kernel<true>, grid, block, 0, st, x, n, partials, reset, n_reset);
}

template <bool BF16>
__device__ __forceinline__ float load_elem(const void *x, int64_t i)
{
    if (BF16) return bf16_to_f32(((const uint16_t *)x)[i]);
    return ((const float *)x)[i];
}

// The map to codes of a [rows, cols] matrix: unit u = 16 consecutive codes of one row (one
// 16-byte store); this thread takes units first, first + stride, ...
template <bool BF16>
__device__ __forceinline__ void quantize_row_units(const void *__restrict__ x, int64_t rows, int64_t cols, int64_t ldq,
                                                   float inv, int8_t *__restrict__ q, int64_t first, int64_t stride)
{
    const int64_t upr = (ldq + 15) >> 4;                     // 16-byte units per row
    const int64_t units = rows * upr;
    const bool narrow = units < (1LL << 32);
    const bool vec_ok = BF16 ? ((cols & 7) == 0) : ((cols & 3) == 0);
    int64_t u = first;
    if (!BF16 && cols == ldq && (cols & 15) == 0 && ((uintptr_t)x & 15) == 0 && ((uintptr_t)q & 15) == 0) {
        // fp32 rows without padding are one contiguous run of whole units (cols a multiple of 16, so
        // the last unit ends where the tensor ends): four of a thread's units (sixteen 16-byte loads)
        // in flight together when it has that many (a single workgroup quantising a whole small
        // matrix would otherwise pay one memory round trip per unit)
        const float4 *x4 = (const float4 *)x;
        for (; u + 3 * stride < units; u += 4 * stride) {
            float4 v[4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) v[k][j] = x4[(u + k * stride) * 4 + j];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    w[j] = quant1(v[k][j].x, inv) | (quant1(v[k][j].y, inv) << 8) | (quant1(v[k][j].z, inv) << 16) |
                           (quant1(v[k][j].w, inv) << 24);
                *(uint4 *)(q + ((u + k * stride) << 4)) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    }
    for (; u < units; u += stride) {
        const int64_t row = div_u(u, upr, narrow);
        const int64_t c0 = (u - row * upr) << 4;
        const int64_t base = row * cols + c0;
        uint32_t w[4] = {0, 0, 0, 0};
        if (vec_ok && c0 + 16 <= cols) {
            if (!BF16) {
                const float4 *p = (const float4 *)((const float *)x + base);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float4 v = p[j];
                    w[j] = quant1(v.x, inv) | (quant1(v.y, inv) << 8) | (quant1(v.z, inv) << 16) |
                           (quant1(v.w, inv) << 24);
                }
            } else {
                const uint4 *p = (const uint4 *)((const uint16_t *)x + base);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    uint4 v = p[j];
                    uint32_t s[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        uint32_t lo = quant1(__uint_as_float(s[e] << 16), inv);
                        uint32_t hi = quant1(__uint_as_float(s[e] & 0xffff0000u), inv);
                        int o = j * 8 + e * 2;
                        w[o >> 2] |= (lo << ((o & 3) * 8)) | (hi << (((o + 1) & 3) * 8));
                    }
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (c0 + e < cols) w[e >> 2] |= quant1(load_elem<BF16>(x, base + e), inv) << ((e & 3) * 8);
        }
        int8_t *dst = q + row * ldq + c0;
        if (c0 + 16 <= ldq && (((row * ldq) & 15) == 0)) {
            *(uint4 *)dst = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            for (int e = 0; e < 16 && c0 + e < ldq; ++e) dst[e] = (int8_t)((w[e >> 2] >> ((e & 3) * 8)) & 0xff);
        }
    }
}

// ---- quantise [rows, cols] -> int8 [rows, ldq] ---------------------------------------
// One thread produces 16 consecutive codes of one row (one 16-byte store).
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_rows_kernel(
    const void *__restrict__ x, int64_t rows, int64_t cols, int64_t ldq,
    const uint32_t *__restrict__ slot, int n_slot, int slot_stride,
    const float *__restrict__ fixed_scale,
    int8_t *__restrict__ q, float *__restrict__ scale_out, float *__restrict__ scale_out2,
    uint32_t *__restrict__ flag)
{
    float scale;
    bool bad;
    const float inv = scales_from(slot, n_slot, slot_stride, fixed_scale, &scale, &bad);
    if (blockIdx.x == 0 && threadIdx.x == 0) publish(scale, bad, scale_out, scale_out2, flag);
    quantize_row_units<BF16>(x, rows, cols, ldq, inv, q, (int64_t)blockIdx.x * blockDim.x + threadIdx.x,
                             (int64_t)gridDim.x * blockDim.x);
}

hipError_t launch_quantize_rows(const void *x, egeria_dtype dt, int64_t rows, int64_t cols,
                                int64_t ldq, const uint32_t *slot, int n_slot, int slot_stride,
                                const float *fixed_scale,
                                int8_t *q, float *scale_out, float *scale_out2, uint32_t *flag,
                                hipStream_t st)
{
    const int64_t units = rows * ((ldq + 15) / 16);
    int64_t blocks = (units + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    const dim3 grid((unsigned)blocks), block(256);
    if (dt == EGERIA_F32)
        return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_rows_kernel<false>, grid, block, 0, st, x, rows, cols, ldq,
                        slot, n_slot, slot_stride, fixed_scale, q, scale_out, scale_out2, flag);
    return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_rows_kernel<true>, grid, block, 0, st, x, rows, cols, ldq, slot,
                    n_slot, slot_stride, fixed_scale, q, scale_out, scale_out2, flag);
}

// ---- quantise [n, c, hw] -> int8 [n, hw, cp] -------------------------------------------
// A workgroup transposes a tile of 64 pixels x 64 channels through LDS: reads
// are contiguous along the pixel axis, writes along the channel axis.
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_nchw_kernel(
    const void *__restrict__ x, int64_t n, int64_t c, int64_t hw, int64_t cp,
    const uint32_t *__restrict__ slot, int n_slot, int slot_stride,
    const float *__restrict__ fixed_scale,
    int8_t *__restrict__ q, float *__restrict__ scale_out, float *__restrict__ scale_out2,
    uint32_t *__restrict__ flag)
{
    float scale;
    bool bad;
    const float inv = scales_from(slot, n_slot, slot_stride, fixed_scale, &scale, &bad);
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0)
        publish(scale, bad, scale_out, scale_out2, flag);
    __shared__ uint8_t tile[64][64 + 4];                  // [pixel][channel], padded rows
    const int64_t img = blockIdx.z;
    const int64_t p0 = (int64_t)blockIdx.x * 64, c0 = (int64_t)blockIdx.y * 64;
    const int tp = threadIdx.x & 63, tc = threadIdx.x >> 6;   // pixel lane, channel phase
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int64_t ch = c0 + tc + 4 * i, p = p0 + tp;
        uint32_t code = 0;
        if (ch < c && p < hw) code = quant1(load_elem<BF16>(x, (img * c + ch) * hw + p), inv);
        tile[tp][tc + 4 * i] = (uint8_t)code;
    }
    __syncthreads();
    // 64 pixels x 4 units of 16 channels = 256 stores of 16 bytes
    const int pix = threadIdx.x >> 2, un = threadIdx.x & 3;
    const int64_t p = p0 + pix, ch0 = c0 + un * 16;
    if (p < hw && ch0 < cp) {
        const uint32_t *src = (const uint32_t *)&tile[pix][un * 16];
        *(uint4 *)(q + (img * hw + p) * cp + ch0) = make_uint4(src[0], src[1], src[2], src[3]);
    }
}

// Same map without the LDS stage, for fp32 input whose pixel count is a
// multiple of 4: a thread owns 4 consecutive pixels x 16 channels (sixteen
// 16-byte loads, lanes along the pixel axis, all in flight together) and
// writes four 16-byte channel groups.
// (this thread takes units first, first + stride, ...)
__device__ __forceinline__ void quantize_nchw_vec_units(const float *__restrict__ x, int64_t n, int64_t c, int64_t hw,
                                                        int64_t cp, float inv, int8_t *__restrict__ q, int64_t first,
                                                        int64_t stride)
{
    const int64_t pq = hw >> 2, cg = cp >> 4;
    const int64_t units = n * cg * pq;
    const bool narrow = units < (1LL << 32);
    for (int64_t u = first; u < units; u += stride) {
        const int64_t ig = div_u(u, pq, narrow);
        const int64_t p = (u - ig * pq) << 2;
        const int64_t img = div_u(ig, cg, narrow), g = ig - img * cg;
        const int64_t ch0 = g << 4;
        float4 v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e)
            v[e] = ch0 + e < c ? *(const float4 *)(x + (img * c + ch0 + e) * hw + p) : make_float4(0.f, 0.f, 0.f, 0.f);
        uint32_t w[4][4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) w[k][j] = 0;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const uint32_t sh = (e & 3) * 8;
            uint32_t c0 = quant1(v[e].x, inv), c1 = quant1(v[e].y, inv), c2 = quant1(v[e].z, inv), c3 = quant1(v[e].w, inv);
            if (ch0 + e >= c) c0 = c1 = c2 = c3 = 0;                  // pad channels are zero even when inv is not finite
            w[0][e >> 2] |= c0 << sh;
            w[1][e >> 2] |= c1 << sh;
            w[2][e >> 2] |= c2 << sh;
            w[3][e >> 2] |= c3 << sh;
        }
        int8_t *dst = q + (img * hw + p) * cp + ch0;
#pragma unroll
        for (int k = 0; k < 4; ++k) *(uint4 *)(dst + k * cp) = make_uint4(w[k][0], w[k][1], w[k][2], w[k][3]);
    }
}

__global__ __launch_bounds__(256) void quantize_nchw_vec_kernel(
    const float *__restrict__ x, int64_t n, int64_t c, int64_t hw, int64_t cp,
    const uint32_t *__restrict__ slot, int n_slot, int slot_stride,
    const float *__restrict__ fixed_scale,
    int8_t *__restrict__ q, float *__restrict__ scale_out, float *__restrict__ scale_out2,
    uint32_t *__restrict__ flag)
{
    float scale;
    bool bad;
    const float inv = scales_from(slot, n_slot, slot_stride, fixed_scale, &scale, &bad);
    if (blockIdx.x == 0 && threadIdx.x == 0) publish(scale, bad, scale_out, scale_out2, flag);
    quantize_nchw_vec_units(x, n, c, hw, cp, inv, q, (int64_t)blockIdx.x * blockDim.x + threadIdx.x,
                            (int64_t)gridDim.x * blockDim.x);
}

hipError_t launch_quantize_nchw(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t hw,
                                int64_t cp, const uint32_t *slot, int n_slot, int slot_stride,
                                const float *fixed_scale,
                                int8_t *q, float *scale_out, float *scale_out2, uint32_t *flag,
                                hipStream_t st)
{
    const dim3 grid((unsigned)((hw + 63) / 64), (unsigned)((cp + 63) / 64), (unsigned)n), block(256);
    if (dt == EGERIA_F32 && (hw & 3) == 0 && hw >= 4 && n > 0 && c > 0) {
        const int64_t units = n * (cp >> 4) * (hw >> 2);
        int64_t blocks = (units + 255) / 256;
        if (blocks > 16384) blocks = 16384;
        return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_nchw_vec_kernel, dim3((unsigned)blocks), block, 0, st,
                        (const float *)x, n, c, hw, cp, slot, n_slot, slot_stride, fixed_scale, q, scale_out, scale_out2,
                        flag);
    }
    if (dt == EGERIA_F32)
        return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_nchw_kernel<false>, grid, block, 0, st, x, n, c, hw, cp, slot,
                        n_slot, slot_stride, fixed_scale, q, scale_out, scale_out2, flag);
    return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_nchw_kernel<true>, grid, block, 0, st, x, n, c, hw, cp, slot,
                    n_slot, slot_stride, fixed_scale, q, scale_out, scale_out2, flag);
}

// ---- small tensors: one workgroup, one launch -----------------------------------------------
// Absolute maximum, scale and codes of a tensor of a few thousand values
// (convolution weights of a narrow layer, a small mini-batch): both passes in
// one workgroup, so the tensor costs one kernel launch instead of two.
// General form [nimg, c, hw] -> int8 [nimg, hw, cp]; a row-major matrix is the
// case hw = 1.
template <bool BF16>
__device__ __forceinline__ void quantize_small_body(const void *__restrict__ x, int nimg, int c, int hw, int cp,
                                                    int8_t *__restrict__ q, float *__restrict__ scale_out,
                                                    uint32_t *__restrict__ flag)
{
    const int total = nimg * c * hw;
    uint32_t m = 0;
    if (!BF16 && ((uintptr_t)x & 15) == 0) {
        // 16-byte loads, four of them requested together
        const float4 *x4 = (const float4 *)x;
        const int n4 = total >> 2;
        int i = threadIdx.x;
        for (; i + 768 < n4; i += 1024) {
            const float4 v0 = x4[i], v1 = x4[i + 256], v2 = x4[i + 512], v3 = x4[i + 768];
            uint32_t a = max4_bits(v0), b = max4_bits(v1), cc = max4_bits(v2), d = max4_bits(v3);
            a = a > b ? a : b;
            cc = cc > d ? cc : d;
            a = a > cc ? a : cc;
            m = m > a ? m : a;
        }
        for (; i < n4; i += 256) {
            const uint32_t a = max4_bits(x4[i]);
            m = m > a ? m : a;
        }
        for (int k = (n4 << 2) + threadIdx.x; k < total; k += 256) {
            const uint32_t a = abs_bits(((const float *)x)[k]);
            m = m > a ? m : a;
        }
    } else {
        for (int i = threadIdx.x; i < total; i += 256) {
            const uint32_t a = abs_bits(load_elem<BF16>(x, i));
            m = m > a ? m : a;
        }
    }
    m = wave_max_u32(m);
    __shared__ uint32_t sm[4];
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = m;
    __syncthreads();
    float scale;
    bool bad;
    const float inv = scales_from(sm, 4, 1, nullptr, &scale, &bad);
    if (threadIdx.x == 0) publish(scale, bad, scale_out, nullptr, flag);
    if (hw == 1) {                                   // rows of a matrix: 16 codes per thread and store
        quantize_row_units<BF16>(x, nimg, c, cp, inv, q, threadIdx.x, 256);
        return;
    }
    const int nout = nimg * hw * cp;
    for (int o = threadIdx.x; o < nout; o += 256) {
        const int ch = o % cp, pp = (o / cp) % hw, img = o / (cp * hw);
        uint32_t code = 0;
        if (ch < c) code = quant1(load_elem<BF16>(x, ((int64_t)img * c + ch) * hw + pp), inv);
        q[o] = (int8_t)code;
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void quantize_small_kernel(const void *__restrict__ x, int nimg, int c, int hw,
                                                             int cp, int8_t *__restrict__ q,
                                                             float *__restrict__ scale_out,
                                                             uint32_t *__restrict__ flag)
{
    quantize_small_body<BF16>(x, nimg, c, hw, cp, q, scale_out, flag);
}

hipError_t launch_quantize_small(const void *x, egeria_dtype dt, int nimg, int c, int hw, int cp, int8_t *q,
                                 float *scale_out, uint32_t *flag, hipStream_t st)
{
    if (dt == EGERIA_F32)
        return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_small_kernel<false>, dim3(1), dim3(256), 0, st, x, nimg, c, hw,
                        cp, q, scale_out, flag);
    return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_small_kernel<true>, dim3(1), dim3(256), 0, st, x, nimg, c, hw, cp,
                    q, scale_out, flag);
}

// ---- a whole snapshot of weight tensors in one or two launches ------------------------------
// Every workgroup finds its tensor in the launch's table (kernel argument) and
// works on a fixed share of it: first the maximum of its share of the values,
// then its share of the 16-byte output units [o][hw][cp / 16].
__device__ __forceinline__ int find_job(const WeightBatch &b, int blk)
{
    int j = 0;
    while (j + 1 < b.n && blk >= b.job[j + 1].first_block) ++j;
    return j;
}

__device__ __forceinline__ uint32_t job_share_absmax(const WeightJob &jb, int lb, uint32_t *sm)
{
    const int64_t n_in = (int64_t)jb.o * jb.c * jb.hw;
    const int64_t beg = (int64_t)lb * jb.epb;
    int64_t end = beg + jb.epb;
    if (end > n_in) end = n_in;
    uint32_t m = 0;
    if (!jb.bf16) {
        const float *x = (const float *)jb.x;
        const int64_t n4 = end > beg ? (end - beg) >> 2 : 0;
        const float4 *x4 = (const float4 *)(x + beg);                // epb is a multiple of 8
        int64_t i = threadIdx.x;
        for (; i + 768 < n4; i += 1024) {                            // four independent loads in flight
            const float4 v0 = x4[i], v1 = x4[i + 256], v2 = x4[i + 512], v3 = x4[i + 768];
            uint32_t a = max4_bits(v0), b = max4_bits(v1), c = max4_bits(v2), d = max4_bits(v3);
            a = a > b ? a : b;
            c = c > d ? c : d;
            a = a > c ? a : c;
            m = m > a ? m : a;
        }
        if (i < n4) {                                                // at most three strides are left: one round trip
            float4 t[3];
#pragma unroll
            for (int k = 0; k < 3; ++k) t[k] = x4[i + 256 * k < n4 ? i + 256 * k : n4 - 1];
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const uint32_t a = i + 256 * k < n4 ? max4_bits(t[k]) : 0u;
                m = m > a ? m : a;
            }
        }
        for (int64_t k = beg + (n4 << 2) + threadIdx.x; k < end; k += 256) {
            const uint32_t a = abs_bits(x[k]);
            m = m > a ? m : a;
        }
    } else {
        const uint16_t *x = (const uint16_t *)jb.x;
        for (int64_t k = beg + threadIdx.x; k < end; k += 256) {
            const uint32_t a = ((uint32_t)x[k] << 16) & 0x7fffffffu;
            m = m > a ? m : a;
        }
    }
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = m;
    __syncthreads();
    const uint32_t a = sm[0] > sm[1] ? sm[0] : sm[1], b = sm[2] > sm[3] ? sm[2] : sm[3];
    return a > b ? a : b;
}

// Tensors of one launch report to the same flag word at the same time.
__device__ __forceinline__ void publish_shared(float scale, bool bad, float *scale_out, uint32_t *flag)
{
    *scale_out = scale;
    uint32_t old = *flag;
    for (;;) {
        uint32_t want = (old & 0xffffff00u) == kFlagMagic ? old : kFlagMagic;
        if (bad) want |= kFlagNonFinite;
        if (want == old) break;
        const uint32_t seen = atomicCAS(flag, old, want);
        if (seen == old) break;
        old = seen;
    }
}

__device__ __forceinline__ void job_share_quantize(const WeightJob &jb, int lb, float inv)
{
    const int cpu = jb.cp >> 4;
    const int64_t units = (int64_t)jb.o * jb.hw * cpu;
    const int64_t beg = (int64_t)lb * jb.upb;
    int64_t end = beg + jb.upb;
    if (end > units) end = units;
    const bool rows_vec = jb.hw == 1 && !jb.bf16 && (jb.c & 3) == 0;
    const bool narrow = units < (1LL << 32);
    for (int64_t u = beg + threadIdx.x; u < end; u += 256) {
        const int64_t op = div_u(u, cpu, narrow);         // o * hw + pixel
        const int c0 = (int)(u - op * cpu) << 4;
        const int64_t oc = div_u(op, jb.hw, narrow);
        const int pix = (int)(op - oc * jb.hw);
        uint32_t w[4] = {0, 0, 0, 0};
        if (rows_vec && c0 + 16 <= jb.c) {
            const float4 *p = (const float4 *)((const float *)jb.x + oc * jb.c + c0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4 v = p[j];
                w[j] = quant1(v.x, inv) | (quant1(v.y, inv) << 8) | (quant1(v.z, inv) << 16) | (quant1(v.w, inv) << 24);
            }
        } else {
            // sixteen gathered values, requested together: unconditional loads (a channel beyond c reads
            // channel c - 1 and is dropped), since a load under a per-lane condition is awaited on its own
            float v[16];
            if (jb.bf16) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int ch = c0 + e < jb.c ? c0 + e : jb.c - 1;
                    v[e] = bf16_to_f32(((const uint16_t *)jb.x)[(oc * jb.c + ch) * jb.hw + pix]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int ch = c0 + e < jb.c ? c0 + e : jb.c - 1;
                    v[e] = ((const float *)jb.x)[(oc * jb.c + ch) * jb.hw + pix];
                }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (c0 + e < jb.c) w[e >> 2] |= quant1(v[e], inv) << ((e & 3) * 8);
        }
        *(uint4 *)(jb.q + (u << 4)) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// PHASE 0: every tensor of the launch fits one workgroup; maximum, scale and codes in one go.
// PHASE 1: per-workgroup maxima -> partials[blockIdx.x].   PHASE 2: scale from the partials, codes.
// Workgroups beyond the table's total_blocks (first launch of a snapshot only) take a share of
// an unrelated maximum pass that the caller wants in the same launch: the mini-batch the
// refreshed reference model is about to run on.
template <int PHASE>
__global__ __launch_bounds__(256) void quantize_weights_kernel(const WeightBatch b, uint32_t *__restrict__ partials,
                                                               uint32_t *__restrict__ flag, int total_blocks,
                                                               const InputMaxJob extra, const InputQuantJob xq)
{
    if ((int)blockIdx.x >= total_blocks) {
        const int blk = (int)blockIdx.x - total_blocks;
        if (PHASE == 2 && xq.kind != 0) {
            // second launch: the codes of the mini-batch whose maxima the first launch took
            float scale;
            bool bad;
            const float inv = scales_from(xq.slot, xq.n_slot, 1, nullptr, &scale, &bad);
            if (blk == 0 && threadIdx.x == 0) publish(scale, bad, xq.scale_out, nullptr, xq.flag);
            const int64_t first = (int64_t)blk * 256 + threadIdx.x, stride = (int64_t)xq.nblk * 256;
            if (xq.kind == 2) quantize_nchw_vec_units((const float *)xq.x, xq.rows, xq.cols, xq.hw, xq.ldq, inv, xq.q, first, stride);
            else if (xq.bf16) quantize_row_units<true>(xq.x, xq.rows, xq.cols, xq.ldq, inv, xq.q, first, stride);
            else quantize_row_units<false>(xq.x, xq.rows, xq.cols, xq.ldq, inv, xq.q, first, stride);
            return;
        }
        if (PHASE != 2 && extra.q) {
            // a small mini-batch [rows, cols]: maximum, scale and codes by this one workgroup
            if (extra.bf16) quantize_small_body<true>(extra.x, extra.rows, extra.cols, 1, extra.cp, extra.q, extra.scale_out, extra.flag);
            else quantize_small_body<false>(extra.x, extra.rows, extra.cols, 1, extra.cp, extra.q, extra.scale_out, extra.flag);
        } else if (PHASE != 2) {
            if (extra.bf16) absmax_share<true>(extra.x, extra.n, extra.partials, extra.reset, extra.n_reset, blk, extra.nblk);
            else absmax_share<false>(extra.x, extra.n, extra.partials, extra.reset, extra.n_reset, blk, extra.nblk);
        }
        return;
    }
    __shared__ uint32_t sm[4];
    const int j = find_job(b, (int)blockIdx.x);
    const WeightJob &jb = b.job[j];
    const int lb = (int)blockIdx.x - jb.first_block;
    if (PHASE == 1) {
        const uint32_t m = job_share_absmax(jb, lb, sm);
        if (threadIdx.x == 0) partials[blockIdx.x] = m;
        return;
    }
    float scale;
    bool bad;
    float inv;
    if (PHASE == 0) {
        (void)job_share_absmax(jb, lb, sm);
        inv = scales_from(sm, 4, 1, nullptr, &scale, &bad);
    } else {
        inv = scales_from(partials + jb.first_block, jb.nblk, 1, nullptr, &scale, &bad);
    }
    if (lb == 0 && threadIdx.x == 0) publish_shared(scale, bad, jb.scale, flag);
    job_share_quantize(jb, lb, inv);
}

// One scale per output channel: a wave owns channel oc of its tensor, takes the
// maximum of the channel's c * hw values, publishes the scale and writes the
// channel's codes [hw][cp].  No barrier, one launch.
__global__ __launch_bounds__(256) void quantize_weights_pc_kernel(const WeightBatch b, uint32_t *__restrict__ flag)
{
    const int j = find_job(b, (int)blockIdx.x);
    const WeightJob &jb = b.job[j];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int oc = ((int)blockIdx.x - jb.first_block) * 4 + wave;
    if (oc >= jb.o) return;
    const int64_t n_row = (int64_t)jb.c * jb.hw, base = (int64_t)oc * n_row;
    uint32_t m = 0;
    for (int64_t k = lane; k < n_row; k += 64) {
        const float v = jb.bf16 ? bf16_to_f32(((const uint16_t *)jb.x)[base + k]) : ((const float *)jb.x)[base + k];
        const uint32_t a = abs_bits(v);
        m = m > a ? m : a;
    }
    m = wave_max_u32(m);
    float scale;
    bool bad;
    const float inv = scale_from_bits(m, nullptr, &scale, &bad);
    if (lane == 0) publish_shared(scale, bad, jb.scale + oc, flag);
    const int cpu = jb.cp >> 4;
    const int units = jb.hw * cpu;
    for (int u = lane; u < units; u += 64) {
        const int pix = u / cpu, c0 = (u - pix * cpu) << 4;
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (c0 + e < jb.c) {
                const int64_t idx = base + (int64_t)(c0 + e) * jb.hw + pix;
                const float v = jb.bf16 ? bf16_to_f32(((const uint16_t *)jb.x)[idx]) : ((const float *)jb.x)[idx];
                w[e >> 2] |= quant1(v, inv) << ((e & 3) * 8);
            }
        *(uint4 *)(jb.q + ((int64_t)oc * units + u) * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

hipError_t launch_quantize_weights_pc(const WeightBatch &b, int total_blocks, uint32_t *flag, hipStream_t st)
{
    return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_weights_pc_kernel, dim3((unsigned)total_blocks), dim3(256), 0, st, b,
                    flag);
}

hipError_t launch_quantize_weights(const WeightBatch &b, int total_blocks, bool one_launch, uint32_t *partials,
                                   uint32_t *flag, hipStream_t st, const InputMaxJob *extra, const InputQuantJob *xq)
{
    InputMaxJob ex{};
    InputQuantJob qj{};
    if (extra) ex = *extra;
    if (extra && xq && !one_launch) qj = *xq;               // the codes need the maxima of an earlier launch
    const dim3 first((unsigned)(total_blocks + ex.nblk)), second((unsigned)(total_blocks + qj.nblk)), block(256);
    if (one_launch)
        return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_weights_kernel<0>, first, block, 0, st, b, partials, flag,
                        total_blocks, ex, InputQuantJob{});
    hipError_t e = launch_k(EGERIA_KERNEL_ABSMAX, quantize_weights_kernel<1>, first, block, 0, st, b, partials, flag,
                            total_blocks, ex, InputQuantJob{});
    if (e != hipSuccess) return e;
    return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_weights_kernel<2>, second, block, 0, st, b, partials, flag,
                    total_blocks, InputMaxJob{}, qj);
}

// ---- fused GELU + quantise ---------------------------------------------------------------
// The GELU output of a Transformer layer's first feed-forward GEMM is consumed
// only by the next quantiser, and its codes must equal those of the fp64
// evaluation rounded to fp32.  GELU is evaluated in fp32 first (cubic pieces from a
// table); a lane falls back to the fp64 form only when the error bound of that
// evaluation leaves two candidate codes (a few elements per 100 000).
__device__ __forceinline__ float gelu_exact(float v)
{
    const double d = (double)v;
    return (float)(0.5 * d * (1.0 + erf(d * 0.70710678118654752440)));
}

constexpr float kGeluShortcutMin = 0.5f;   // gelu(0.5) = 0.346 exceeds max |gelu| over v < 0 (0.17)

__global__ __launch_bounds__(256) void gelu_absmax_exact_kernel(const float *__restrict__ v, int64_t n,
                                                                const uint32_t *__restrict__ vmax,
                                                                uint32_t *__restrict__ exact_absmax)
{
    if (__uint_as_float(reduce_ways(vmax)) >= kGeluShortcutMin) return;   // the shortcut applies: nothing to do
    uint32_t m = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t a = abs_bits(gelu_exact(v[i]));
        m = m > a ? m : a;
    }
    __shared__ uint32_t sm4[4];
    block_atomic_max(m, exact_absmax, sm4);
}

hipError_t launch_gelu_absmax_exact(const float *v, int64_t n, const uint32_t *vmax, uint32_t *exact_absmax,
                                    hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 1023) / 1024;
    if (blocks > 1024) blocks = 1024;
    return launch_k(EGERIA_KERNEL_NONE, gelu_absmax_exact_kernel, dim3((unsigned)blocks), dim3(256), 0, st, v, n, vmax,
                    exact_absmax);
}

// fp32 GELU from a table of cubic pieces (gelu_table.inc: 256 pieces of width 1/16 on [-8, 8), generated
// with the measured error of the fp32 evaluation; beyond 8 gelu(v) rounds to v, below -8 it lies within
// 5e-15 of the table's first value).  |approximation - gelu| <= kGeluErrAbs + kGeluErrRel * |gelu|.
#include "gelu_table.inc"

// BIG: values of 8 and more may occur (the caller knows the tensor's maximum); otherwise the test is left out.
template <bool BIG>
__device__ __forceinline__ float gelu_table(float v, const float4 *__restrict__ tab)
{
    const float vc = fminf(fmaxf(v, -8.0f), 7.999999f);
    const int i = (int)fmaf(vc, 16.0f, 128.0f);                  // piece, 0..255
    const float t = vc - fmaf((float)i, 0.0625f, -8.0f);
    const float4 c = tab[i];
    const float g = fmaf(fmaf(fmaf(c.w, t, c.z), t, c.y), t, c.x);
    return (BIG && v >= 8.0f) ? v : g;
}

__device__ __forceinline__ uint32_t code_of(float t)
{
    float r = rintf(t);
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (uint32_t)((int)r) & 0xffu;
}

// Code of gelu(v) from the table.  The code clamp(rne(fp32(g * inv))) is monotone in g, so when both ends of
// the interval that the error bound leaves for g * inv round to the same integer, that integer is the code
// of the exact value; *unsure is set otherwise (a few values per 100 000) and the caller takes the fp64 form.
// err_abs_inv = kGeluErrAbs * inv.  (The relative part also covers the rounding of the two products.)
// (The interval [t - e, t + e] rounds to one integer if |t - rne(t)| + e < 1/2.  No clamp: the scale is the
// tensor's exact maximum of |gelu| over 127, so |t| stays below 127.5 by the table's error bound; with a
// non-finite maximum inv is 0 and every code is 0.)
template <bool BIG>
__device__ __forceinline__ uint32_t quant_gelu_fast(float v, float inv, float err_abs_inv, const float4 *__restrict__ tab,
                                                    bool *unsure)
{
    const float t = gelu_table<BIG>(v, tab) * inv;
    const float e = fmaf(kGeluErrRel + 3.0e-7f, fabsf(t), err_abs_inv);
    const float rt = rintf(t);
    *unsure = !(fabsf(t - rt) + e < 0.5f);
    return (uint32_t)((int)rt) & 0xffu;
}

__global__ __launch_bounds__(256) void quantize_gelu_rows_kernel(
    const float *__restrict__ v, int64_t rows, int64_t cols, int64_t ldq, const uint32_t *__restrict__ vmax,
    const uint32_t *__restrict__ exact_absmax, int8_t *__restrict__ q, float *__restrict__ scale_out,
    uint32_t *__restrict__ flag)
{
    // absolute maximum of gelu(v): gelu is increasing for v >= 0 and bounded by 0.17 for v < 0
    const float vm = __uint_as_float(reduce_ways(vmax));
    const bool bad = !(vm <= 3.402823466e+38f);
    const float exact = __uint_as_float(reduce_ways(exact_absmax));
    float absmax = vm >= kGeluShortcutMin ? gelu_exact(vm) : exact;
    if (bad) absmax = 0.0f;
    float scale = (float)((double)absmax / 127.0);
    float inv = (float)(127.0 / (double)absmax);
    if (!(inv <= 3.402823466e+38f) || !(scale > 0.0f)) { scale = 1.0f; inv = 0.0f; }
    if (blockIdx.x == 0 && threadIdx.x == 0) publish(scale, bad, scale_out, nullptr, flag);
    __shared__ float4 tab[256];                    // the table, once per workgroup (256 threads)
    tab[threadIdx.x] = kGeluTable[threadIdx.x];
    __syncthreads();
    const float err_abs_inv = kGeluErrAbs * inv;
    const int64_t upr = ldq >> 4;
    const int64_t units = rows * upr;
    const bool narrow = units < (1LL << 32);
    const bool vec_ok = (cols & 3) == 0;
    // a thread's units are `stride` apart: row and unit within the row advance by stride / upr and stride % upr
    // (one division at the start instead of one per unit)
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t step_rows = div_u(stride, upr, narrow), step_units = stride - step_rows * upr;
    auto run = [&](auto big_c) {
        constexpr bool BIG = decltype(big_c)::value;
        int64_t row = div_u(first, upr, narrow), cu = first - row * upr;
        for (int64_t u = first; u < units; u += stride) {
            const int64_t c0 = cu << 4;
            const int64_t base = row * cols + c0;
            uint32_t w[4] = {0, 0, 0, 0};
            uint32_t redo = 0;                         // elements that need the fp64 form
            if (vec_ok && c0 + 16 <= cols) {
                const float4 *p = (const float4 *)(v + base);
                float4 x[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) x[j] = p[j];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bool u0, u1, u2, u3;
                    w[j] = quant_gelu_fast<BIG>(x[j].x, inv, err_abs_inv, tab, &u0) |
                           (quant_gelu_fast<BIG>(x[j].y, inv, err_abs_inv, tab, &u1) << 8) |
                           (quant_gelu_fast<BIG>(x[j].z, inv, err_abs_inv, tab, &u2) << 16) |
                           (quant_gelu_fast<BIG>(x[j].w, inv, err_abs_inv, tab, &u3) << 24);
                    redo |= ((u0 ? 1u : 0u) | (u1 ? 2u : 0u) | (u2 ? 4u : 0u) | (u3 ? 8u : 0u)) << (4 * j);
                }
            } else {
                redo = 0xffffu;                        // ragged tail of a row: every element through the loop below
            }
            // one copy of the fp64 code, rolled: the values are re-read (they are in cache)
#pragma unroll 1
            while (redo) {
                const int e = __ffs((int)redo) - 1;
                redo &= redo - 1;
                if (c0 + e >= cols) continue;
                const uint32_t code = code_of(gelu_exact(v[base + e]) * inv);
                const uint32_t sh = (e & 3) * 8, keep = ~(0xffu << sh);
                if ((e >> 2) == 0) w[0] = (w[0] & keep) | (code << sh);
                if ((e >> 2) == 1) w[1] = (w[1] & keep) | (code << sh);
                if ((e >> 2) == 2) w[2] = (w[2] & keep) | (code << sh);
                if ((e >> 2) == 3) w[3] = (w[3] & keep) | (code << sh);
            }
            *(uint4 *)(q + row * ldq + c0) = make_uint4(w[0], w[1], w[2], w[3]);
            row += step_rows;
            cu += step_units;
            if (cu >= upr) { cu -= upr; ++row; }
        }
    };
    // values of 8 and more (where gelu(v) rounds to v and the table ends) only if the tensor's maximum says so
    if (vm >= 8.0f || bad) run(std::true_type{}); else run(std::false_type{});
}

hipError_t launch_quantize_gelu_rows(const float *v, int64_t rows, int64_t cols, int64_t ldq,
                                     const uint32_t *vmax, const uint32_t *exact_absmax, int8_t *q,
                                     float *scale_out, uint32_t *flag, hipStream_t st)
{
    const int64_t units = rows * (ldq / 16);
    int64_t blocks = (units + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_gelu_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, v,
                    rows, cols, ldq, vmax, exact_absmax, q, scale_out, flag);
}

__global__ __launch_bounds__(256) void gelu_exact_kernel(const float *v, int64_t n, float *y)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        y[i] = gelu_exact(v[i]);
}

hipError_t launch_gelu_exact(const float *v, int64_t n, float *y, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    return launch_k(EGERIA_KERNEL_NONE, gelu_exact_kernel, dim3((unsigned)blocks), dim3(256), 0, st, v, n, y);
}

// ---- dequantise ------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dequantize_kernel(const int8_t *__restrict__ q,
                                                         const float *__restrict__ scale, int64_t n,
                                                         float *__restrict__ x)
{
    const float s = *scale;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        x[i] = (float)q[i] * s;
}

hipError_t launch_dequantize(const int8_t *q, const float *scale, int64_t n, float *x, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    return launch_k(EGERIA_KERNEL_NONE, dequantize_kernel, dim3((unsigned)blocks), dim3(256), 0, st, q, scale, n, x);
}

}  // namespace egeria
