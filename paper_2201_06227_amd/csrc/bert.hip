// fp32 glue of a Transformer encoder layer of the reference model: under
// dynamic quantisation (Section 5 of the paper) only the linear layers are
// int8; self-attention and layer norm stay in fp32.
#include "common.hpp"

namespace egeria {

typedef float v16f __attribute__((ext_vector_type(16)));

// ---- y = LN(x + res): one wave per row -----------------------------------------------
__global__ __launch_bounds__(256) void layernorm_kernel(const float *__restrict__ x,
                                                        const float *__restrict__ res, int64_t rows,
                                                        int H, const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, float eps,
                                                        float *__restrict__ y,
                                                        uint32_t *__restrict__ absmax_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    uint32_t amax = 0;
    if (row < rows) {
        const float *xr = x + row * H;
        const float *rr = res ? res + row * H : nullptr;
        float s = 0.0f;
        for (int h = lane; h < H; h += 64) s += xr[h] + (rr ? rr[h] : 0.0f);
        const float mean = wave_sum(s) / (float)H;
        float q = 0.0f;
        for (int h = lane; h < H; h += 64) {
            const float v = (xr[h] + (rr ? rr[h] : 0.0f)) - mean;
            q += v * v;
        }
        const float var = wave_sum(q) / (float)H;
        const float rstd = 1.0f / sqrtf(var + eps);
        for (int h = lane; h < H; h += 64) {
            const float v = (xr[h] + (rr ? rr[h] : 0.0f)) - mean;
            float o = v * rstd;
            if (gamma) o = o * gamma[h];
            if (beta) o = o + beta[h];
            y[row * H + h] = o;
            const uint32_t ab = abs_bits(o);
            amax = amax > ab ? amax : ab;
        }
    }
    if (absmax_out) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)amax, off, kWave);
            amax = o > amax ? o : amax;
        }
        if (lane == 0 && amax) atomicMax(absmax_out, amax);
    }
}

hipError_t launch_layernorm(const float *x, const float *res, int64_t rows, int32_t H,
                            const float *gamma, const float *beta, float eps, float *y,
                            uint32_t *absmax_out, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(layernorm_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, x, res, rows,
                       (int)H, gamma, beta, eps, y, absmax_out);
    return hipGetLastError();
}

// ---- multi-head self-attention -----------------------------------------------------------
// A workgroup owns one (batch, head) pair and 128 queries, 32 per wave; key /
// value tiles of 32 rows pass through LDS.  The products run on
// v_mfma_f32_32x32x2f32 in the transposed form
//     S^T = K Q^T  (keys x queries),      O^T = V^T P^T  (head dim x queries),
// so that a lane always owns one query column: the soft-max statistics of a
// query are an in-lane reduction over its 16 key registers plus one exchange
// with the lane holding the other 16 keys, and the accumulator registers of
// S^T are, unchanged, the B operand of the second product.
constexpr int kDh = 64;             // head dimension covered (smaller heads are zero padded)
constexpr int kKeyTile = 32;
constexpr int kKPad = kDh + 4;

__global__ __launch_bounds__(256) void attention_kernel(const float *__restrict__ qkv, int B, int S,
                                                        int Hd, int heads, int dh, float scale,
                                                        float *__restrict__ ctx,
                                                        uint32_t *__restrict__ absmax_out)
{
    __shared__ __attribute__((aligned(16))) float sK[kKeyTile][kKPad];
    __shared__ __attribute__((aligned(16))) float sV[kKeyTile][kDh];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, hh = lane >> 5;
    const int qtiles = (S + 127) / 128;
    const int bh = blockIdx.x / qtiles, qt = blockIdx.x % qtiles;
    const int bi = bh / heads, hd = bh % heads;
    const int64_t tok0 = (int64_t)bi * S;
    const int64_t ld = 3 * (int64_t)Hd;
    const float *qbase = qkv + hd * dh, *kbase = qbase + Hd, *vbase = qbase + 2 * Hd;

    // this lane's query row as the B operand of S^T = K Q^T: 32 of its 64 values,
    // d = 8u + 4hh + e  (u = 0..7, e = 0..3)
    const int q = qt * 128 + wave * 32 + c;
    float qr[32];
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int d = 8 * u + 4 * hh + e;
            qr[4 * u + e] = (q < S && d < dh) ? qbase[(tok0 + q) * ld + d] * scale : 0.0f;
        }

    v16f o0, o1;                       // O^T rows d = 0..31 and 32..63, column = this lane's query
#pragma unroll
    for (int r = 0; r < 16; ++r) { o0[r] = 0.0f; o1[r] = 0.0f; }
    float mrun = -INFINITY, lrun = 0.0f;

    for (int j0 = 0; j0 < S; j0 += kKeyTile) {
        __syncthreads();
        // stage K and V rows j0 .. j0+31 (zero beyond S and beyond dh)
        for (int i = tid; i < kKeyTile * kDh; i += 256) {
            const int kr = i >> 6, d = i & 63;
            const bool ok = (j0 + kr) < S && d < dh;
            const int64_t off = (tok0 + j0 + kr) * ld + d;
            sK[kr][d] = ok ? kbase[off] : 0.0f;
            sV[kr][d] = ok ? vbase[off] : 0.0f;
        }
        __syncthreads();

        v16f st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.0f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float4 kv = *(const float4 *)&sK[c][8 * u + 4 * hh];
            st = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.x, qr[4 * u + 0], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.y, qr[4 * u + 1], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.z, qr[4 * u + 2], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_32x32x2f32(kv.w, qr[4 * u + 3], st, 0, 0, 0);
        }
        // register r of st is key j0 + 8*(r/4) + 4*hh + r%4 for this lane's query
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = j0 + (r >> 2) * 8 + hh * 4 + (r & 3);
            if (key >= S) st[r] = -INFINITY;
            mx = fmaxf(mx, st[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float mnew = fmaxf(mrun, mx);           // finite: every tile holds at least one key
        const float corr = expf(mrun - mnew);
        float ps = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            st[r] = expf(st[r] - mnew);
            ps += st[r];
        }
        ps += __shfl_xor(ps, 32, kWave);
        lrun = lrun * corr + ps;
        mrun = mnew;
#pragma unroll
        for (int r = 0; r < 16; ++r) { o0[r] *= corr; o1[r] *= corr; }
        // O^T += V^T P^T: step r contracts key 8*(r/4) + 4*hh + r%4 of the tile
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kr = (r >> 2) * 8 + hh * 4 + (r & 3);
            o0 = __builtin_amdgcn_mfma_f32_32x32x2f32(sV[kr][c], st[r], o0, 0, 0, 0);
            o1 = __builtin_amdgcn_mfma_f32_32x32x2f32(sV[kr][32 + c], st[r], o1, 0, 0, 0);
        }
    }

    uint32_t amax = 0;
    if (q < S) {
        const float invl = 1.0f / lrun;
        float *dst = ctx + (tok0 + q) * Hd + hd * dh;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int d = (r >> 2) * 8 + hh * 4 + (r & 3);
            if (d < dh) {
                const float v = o0[r] * invl;
                dst[d] = v;
                const uint32_t ab = abs_bits(v);
                amax = amax > ab ? amax : ab;
            }
            if (32 + d < dh) {
                const float v = o1[r] * invl;
                dst[32 + d] = v;
                const uint32_t ab = abs_bits(v);
                amax = amax > ab ? amax : ab;
            }
        }
    }
    if (absmax_out) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const uint32_t o = (uint32_t)__shfl_xor((int)amax, off, kWave);
            amax = o > amax ? o : amax;
        }
        if (lane == 0 && amax) atomicMax(absmax_out, amax);
    }
}

hipError_t launch_attention(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads,
                            float *ctx, uint32_t *absmax_out, hipStream_t st)
{
    const int dh = Hd / heads;
    const int qtiles = (S + 127) / 128;
    const int64_t grid = (int64_t)B * heads * qtiles;
    if (grid <= 0) return hipSuccess;
    if (dh > kDh || grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attention_kernel, dim3((unsigned)grid), dim3(256), 0, st, qkv, (int)B, (int)S, (int)Hd,
                       (int)heads, dh, 1.0f / sqrtf((float)dh), ctx, absmax_out);
    return hipGetLastError();
}

}  // namespace egeria
