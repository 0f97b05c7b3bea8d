// Affine (asymmetric) uint8 activation codes: the framework's default activation
// code, to which Section 5 of the paper delegates the int8 arithmetic.  From the
// extrema of a tensor, every operation an IEEE fp32 one:
//   hi = max(max x, 0), lo = min(min x, 0)
//   scale = max((hi - lo) / 255, 2^-23);  zp = clamp(0 - rne(lo / scale), 0, 255)
//   q = clamp(rne(x * (1 / scale)) + zp, 0, 255)
// A code is stored as the int8 value q - 128, so the int8 x int8 matrix cores
// contract it unchanged: sum (q - zp) w = sum (q - 128) w + (128 - zp) sum w, and
// the sums of the weight codes (per output channel, and for 3x3 kernels per class
// of border pixel: a window position outside the image holds the real value zero,
// whose centred code is 0, while the contraction reads a stored 0 = code 128
// there) are made once per snapshot by colsum_kernel.
//
// Two launches per quantise point: the extrema as per-workgroup partial results
// (plain stores), then the codes, every workgroup reducing the partial results
// to the same scale and zero point.  HBM-bound: 4 n bytes read twice, n written.
#include "common.hpp"

namespace egeria {

namespace {

constexpr int kMinMaxBlocks = 1024;

template <bool BF16>
__global__ __launch_bounds__(256) void minmax_kernel(const void *__restrict__ x, int64_t n, uint32_t *__restrict__ partials)
{
    float hi = 0.0f, nlo = 0.0f;       // max(x, 0) and max(-x, 0)
    uint32_t worst = 0;                // largest |x| bit pattern: above 0x7f7fffff for NaN and infinities
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
    if (!BF16 && ((uintptr_t)x & 15) == 0) {
        const float4 *x4 = (const float4 *)x;
        const int64_t n4 = n >> 2;
        for (int64_t i = first; i < n4; i += stride) {
            const float4 v = x4[i];
            const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                hi = fmaxf(hi, e[k]);
                nlo = fmaxf(nlo, -e[k]);
                const uint32_t a = abs_bits(e[k]);
                worst = worst > a ? worst : a;
            }
        }
        for (int64_t i = (n4 << 2) + first; i < n; i += stride) {
            const float v = ((const float *)x)[i];
            hi = fmaxf(hi, v);
            nlo = fmaxf(nlo, -v);
            const uint32_t a = abs_bits(v);
            worst = worst > a ? worst : a;
        }
    } else {
        for (int64_t i = first; i < n; i += stride) {
            const float v = BF16 ? bf16_to_f32(((const uint16_t *)x)[i]) : ((const float *)x)[i];
            hi = fmaxf(hi, v);
            nlo = fmaxf(nlo, -v);
            const uint32_t a = abs_bits(v);
            worst = worst > a ? worst : a;
        }
    }
    // both are non-negative, so their bit patterns order like the values
    uint32_t hb = wave_max_u32(__float_as_uint(hi)), lb = wave_max_u32(__float_as_uint(nlo));
    worst = wave_max_u32(worst);
    __shared__ uint32_t sm[3][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sm[0][wave] = hb; sm[1][wave] = lb; sm[2][wave] = worst; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) {
            sm[0][0] = sm[0][0] > sm[0][w] ? sm[0][0] : sm[0][w];
            sm[1][0] = sm[1][0] > sm[1][w] ? sm[1][0] : sm[1][w];
            sm[2][0] = sm[2][0] > sm[2][w] ? sm[2][0] : sm[2][w];
        }
        const bool bad = sm[2][0] >= 0x7f800000u;
        partials[2 * blockIdx.x] = bad ? 0x7fc00000u : sm[0][0];
        partials[2 * blockIdx.x + 1] = sm[1][0];
    }
}

// [n, c, hw] (channel planes; hw = 1: rows of a matrix) -> codes [n, hw, cp], 16 per thread and store
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_affine_kernel(const void *__restrict__ x, int64_t n, int64_t c, int64_t hw,
                                                              int64_t cp, const uint32_t *__restrict__ partials, int nb,
                                                              int store_offset, uint8_t *__restrict__ q,
                                                              float *__restrict__ scale_out, int32_t *__restrict__ zp_out,
                                                              uint32_t *__restrict__ flag)
{
    uint32_t hb = 0, lb = 0;
    for (int i = threadIdx.x; i < nb; i += 256) {
        const uint32_t a = partials[2 * i], b = partials[2 * i + 1];
        hb = hb > a ? hb : a;
        lb = lb > b ? lb : b;
    }
    hb = wave_max_u32(hb);
    lb = wave_max_u32(lb);
    __shared__ uint32_t sm[2][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sm[0][wave] = hb; sm[1][wave] = lb; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        hb = hb > sm[0][w] ? hb : sm[0][w];
        lb = lb > sm[1][w] ? lb : sm[1][w];
    }
    const bool bad = hb >= 0x7f800000u || lb >= 0x7f800000u;
    if (bad) hb = lb = 0;
    const float hi = __uint_as_float(hb), lo = -__uint_as_float(lb);
    float scale = __fdiv_rn(__fsub_rn(hi, lo), 255.0f);
    scale = fmaxf(scale, 1.1920928955078125e-07f);
    int zp = 0 - (int)rintf(__fdiv_rn(lo, scale));
    zp = zp < 0 ? 0 : (zp > 255 ? 255 : zp);
    const float inv = __fdiv_rn(1.0f, scale);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        publish(scale, bad, scale_out, nullptr, flag);
        *zp_out = zp;
    }
    const int64_t upr = cp >> 4;
    const int64_t total = n * hw * upr;
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += (int64_t)gridDim.x * blockDim.x) {
        int64_t img, p, unit;
        if (hw == 1) {
            img = u / upr;
            unit = u - img * upr;
            p = 0;
        } else {
            p = u % hw;
            const int64_t rest = u / hw;
            unit = rest % upr;
            img = rest / upr;
        }
        union {
            uint8_t b[16];
            uint4 v;
        } pk;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t ch = unit * 16 + e;
            int code = store_offset;                       // pad channels: the stored byte is zero
            if (ch < c) {
                const int64_t i = (img * c + ch) * hw + p;
                const float v = BF16 ? bf16_to_f32(((const uint16_t *)x)[i]) : ((const float *)x)[i];
                code = (int)rintf(__fmul_rn(v, inv)) + zp;
                code = code < 0 ? 0 : (code > 255 ? 255 : code);
            }
            pk.b[e] = (uint8_t)(code - store_offset);
        }
        *(uint4 *)(q + ((img * hw + p) * cp + unit * 16)) = pk.v;
    }
}

// One wave per output channel: the sums of its int8 weight codes per window position, combined per border class.
__global__ __launch_bounds__(256) void colsum_kernel(const int8_t *__restrict__ w_q, int32_t out, int32_t taps, int32_t cp,
                                                     int32_t *__restrict__ colsum)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * 4 + wave;
    if (n >= out) return;
    int32_t s[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        s[t] = 0;
        if (t < taps) {
            const int8_t *row = w_q + ((int64_t)n * taps + t) * cp;
            for (int k = lane; k < cp; k += 64) s[t] += row[k];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) s[t] += __shfl_xor(s[t], off, kWave);
        }
    }
    if (lane != 0) return;
    if (taps == 1) {
        colsum[n] = s[0];
        return;
    }
    for (int cls = 0; cls < 16; ++cls) {
        int32_t v = 0;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const bool outside = (kh == 0 && (cls & 1)) || (kh == 2 && (cls & 2)) || (kw == 0 && (cls & 4)) ||
                                     (kw == 2 && (cls & 8));
                if (!outside) v += s[kh * 3 + kw];
            }
        colsum[(int64_t)cls * out + n] = v;
    }
}

}  // namespace

int minmax_blocks(int64_t n)
{
    int64_t b = (n + 4095) / 4096;
    if (b < 1) b = 1;
    return (int)(b > kMinMaxBlocks ? kMinMaxBlocks : b);
}

size_t affine_partial_bytes() { return (size_t)kMinMaxBlocks * 2 * sizeof(uint32_t); }

hipError_t launch_minmax(const void *x, egeria_dtype dt, int64_t n, uint32_t *partials, hipStream_t st)
{
    const dim3 grid((unsigned)minmax_blocks(n)), block(256);
    if (dt == EGERIA_BF16) return launch_k(EGERIA_KERNEL_ABSMAX, minmax_kernel<true>, grid, block, 0, st, x, n, partials);
    return launch_k(EGERIA_KERNEL_ABSMAX, minmax_kernel<false>, grid, block, 0, st, x, n, partials);
}

hipError_t launch_quantize_affine(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t hw, int64_t cp,
                                  const uint32_t *partials, int nb, int store_offset, void *q, float *scale_out,
                                  int32_t *zp_out, uint32_t *flag, hipStream_t st)
{
    int64_t blocks = (n * hw * (cp >> 4) + 255) / 256;
    if (blocks < 1) blocks = 1;                            // scale and zero point are still written
    if (blocks > 8192) blocks = 8192;
    const dim3 grid((unsigned)blocks), block(256);
    if (dt == EGERIA_BF16)
        return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_affine_kernel<true>, grid, block, 0, st, x, n, c, hw, cp, partials, nb,
                        store_offset, (uint8_t *)q, scale_out, zp_out, flag);
    return launch_k(EGERIA_KERNEL_QUANTIZE, quantize_affine_kernel<false>, grid, block, 0, st, x, n, c, hw, cp, partials, nb,
                    store_offset, (uint8_t *)q, scale_out, zp_out, flag);
}

hipError_t launch_colsum(const int8_t *w_q, int32_t out, int32_t taps, int32_t cp, int32_t *colsum, hipStream_t st)
{
    if (out <= 0) return hipSuccess;
    return launch_k(EGERIA_KERNEL_NONE, colsum_kernel, dim3((unsigned)((out + 3) / 4)), dim3(256), 0, st, w_q, out, taps, cp,
                    colsum);
}

}  // namespace egeria
