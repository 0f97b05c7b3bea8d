// Reference model at float16 / float32 precision (Section 6.4 of the paper,
// Table 2): operands in the layout the GEMM consumes.  A tensor [n, c, hw]
// (channel-major: a mini-batch of images, a convolution kernel, or with hw = 1
// the rows of a matrix) becomes [n, hw, cpe] of the reference precision, the
// channels rounded to nearest even and padded with zeros to cpe (a whole
// number of 16-byte units).  One thread makes one 16-byte unit; lanes run along
// the pixels of an image (coalesced reads of each channel plane) or, for
// matrices, along the units of a row.
#include "common.hpp"

namespace egeria {

namespace {

template <bool SRC_BF16, int ET>
__global__ __launch_bounds__(256) void cast_chlast_kernel(const void *__restrict__ x, int64_t n, int64_t c,
                                                          int64_t hw, int64_t cpe, uint8_t *__restrict__ out,
                                                          float *__restrict__ one)
{
    constexpr int EPU = ET == 1 ? 8 : 4;                  // elements per 16-byte unit
    if (one && blockIdx.x == 0 && threadIdx.x == 0) *one = 1.0f;
    const int64_t upr = cpe / EPU;                        // units per pixel
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
        float v[EPU];
#pragma unroll
        for (int e = 0; e < EPU; ++e) {
            const int64_t ch = unit * EPU + e;
            v[e] = 0.0f;
            if (ch < c) {
                const int64_t i = (img * c + ch) * hw + p;
                v[e] = SRC_BF16 ? bf16_to_f32(((const uint16_t *)x)[i]) : ((const float *)x)[i];
            }
        }
        uint8_t *dst = out + ((img * hw + p) * cpe + unit * EPU) * (ET == 1 ? 2 : 4);
        if (ET == 1) {
            union {
                _Float16 h[8];
                uint4 q;
            } pk;
#pragma unroll
            for (int e = 0; e < 8; ++e) pk.h[e] = (_Float16)v[e];     // round to nearest even
            *(uint4 *)dst = pk.q;
        } else {
            *(float4 *)dst = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

}  // namespace

hipError_t launch_cast_chlast(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t hw, int64_t cpe, int et,
                              void *out, float *one, hipStream_t st)
{
    const int64_t total = n * hw * (cpe / (et == 1 ? 8 : 4));
    int64_t blocks = (total + 255) / 256;
    if (blocks < 1) blocks = 1;                            // the 1.0f is still written
    if (blocks > 8192) blocks = 8192;
    const dim3 grid((unsigned)blocks), block(256);
    const bool bf = dt == EGERIA_BF16;
    if (et == 1) {
        if (bf) return launch_k(EGERIA_KERNEL_QUANTIZE, cast_chlast_kernel<true, 1>, grid, block, 0, st, x, n, c, hw, cpe, (uint8_t *)out, one);
        return launch_k(EGERIA_KERNEL_QUANTIZE, cast_chlast_kernel<false, 1>, grid, block, 0, st, x, n, c, hw, cpe, (uint8_t *)out, one);
    }
    if (bf) return launch_k(EGERIA_KERNEL_QUANTIZE, cast_chlast_kernel<true, 2>, grid, block, 0, st, x, n, c, hw, cpe, (uint8_t *)out, one);
    return launch_k(EGERIA_KERNEL_QUANTIZE, cast_chlast_kernel<false, 2>, grid, block, 0, st, x, n, c, hw, cpe, (uint8_t *)out, one);
}

}  // namespace egeria
