// int8 x int8 -> int32 GEMM and implicit-GEMM 3x3 convolution on the gfx950
// matrix cores, with the dequantising epilogue fused (the reference model's
// linear and convolution layers, Section 4.1 of the paper).
//
//   acc[m, n] = sum_k a[m, k] * w[n, k]          (both operands K-contiguous)
//   y[m, n]   = act( fma((float)acc, sx*sw, bias[n]) [+ residual] )
//
// One workgroup of 4 waves owns a BM x BN tile of the output.  Per K step of 64
// bytes the tile's A and W rows are staged through LDS (16-byte units, rows
// padded to 80 bytes so that the 128-bit operand reads of a wave fall on
// distinct banks) while the next step's global loads are already in flight.
// Each wave issues v_mfma_i32_32x32x32_i8: lane l supplies 16 consecutive K
// bytes of row (l % 32) at K offset 16 * (l / 32) for A and for W alike, so
// the product is exact whatever the instruction's internal K order is.
#include "common.hpp"

namespace egeria {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;          // K bytes per step
constexpr int kLdsRow = 80;      // padded LDS row in bytes

template <int BM, int BN, int WM, int WN, bool CONV>
__global__ __launch_bounds__(256) void gemm_i8_kernel(const GemmArgs g)
{
    static_assert(WM * WN == 4, "four waves per workgroup");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_IT = (BM * 4 + 255) / 256, B_IT = (BN * 4 + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint8_t sA[BM * kLdsRow];
    __shared__ __attribute__((aligned(16))) uint8_t sB[BN * kLdsRow];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tiles_n = (g.N + BN - 1) / BN;
    const int64_t tile_m = blockIdx.x / tiles_n;
    const int tile_n = blockIdx.x % tiles_n;
    const int64_t m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int unit = tid & 3;                    // which 16-byte unit of the 64-byte K step

    // rows this thread stages
    int64_t a_m[A_IT];
    bool a_ok[A_IT];
    int a_oh[A_IT], a_ow[A_IT];
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
        const int r = (tid + it * 256) >> 2;
        a_m[it] = m0 + r;
        a_ok[it] = r < BM && a_m[it] < g.M;
        if (CONV) {
            a_ow[it] = (int)(a_m[it] % g.W);
            a_oh[it] = (int)((a_m[it] / g.W) % g.H);
        }
    }
    int b_n[B_IT];
    bool b_ok[B_IT];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
        const int r = (tid + it * 256) >> 2;
        b_n[it] = n0 + r;
        b_ok[it] = r < BN && b_n[it] < g.N;
    }

    uint4 ra[A_IT], rb[B_IT];
    auto load_tiles = [&](int kt) {
        const int k0 = kt * kBK + unit * 16;
        const bool k_ok = k0 < g.kp;
        int dh = 0, dw = 0, c0 = 0;
        if (CONV) {
            const int tap = k0 / g.cp;
            c0 = k0 - tap * g.cp;
            const int kh = tap / 3;
            dh = kh - 1;
            dw = tap - kh * 3 - 1;
        }
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            bool ok = a_ok[it] && k_ok;
            const int8_t *p;
            if (CONV) {
                ok = ok && (unsigned)(a_oh[it] + dh) < (unsigned)g.H && (unsigned)(a_ow[it] + dw) < (unsigned)g.W;
                p = g.a + (a_m[it] + (int64_t)dh * g.W + dw) * g.cp + c0;
            } else {
                p = g.a + a_m[it] * g.lda + k0;
            }
            ra[it] = ok ? *(const uint4 *)p : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
            const bool ok = b_ok[it] && k_ok;
            rb[it] = ok ? *(const uint4 *)(g.w + (int64_t)b_n[it] * g.kp + k0) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int r = (tid + it * 256) >> 2;
            if (r < BM) *(uint4 *)&sA[r * kLdsRow + unit * 16] = ra[it];
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
            const int r = (tid + it * 256) >> 2;
            if (r < BN) *(uint4 *)&sB[r * kLdsRow + unit * 16] = rb[it];
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int nk = (g.kp + kBK - 1) / kBK;
    load_tiles(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();                 // previous step's operand reads are done
        store_tiles();
        __syncthreads();
        if (kt + 1 < nk) load_tiles(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i fa[TM], fb[TN];
            const int koff = (ks * 2 + (lane >> 5)) * 16;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *(const v4i *)&sA[((wm * TM + i) * 32 + (lane & 31)) * kLdsRow + koff];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *(const v4i *)&sB[((wn * TN + j) * 32 + (lane & 31)) * kLdsRow + koff];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // ---- epilogue: lane l of a 32x32 block holds column l % 32 and rows
    // 8 * (r / 4) + 4 * (l / 32) + r % 4 for r = 0..15.
    const float s = (*g.sx) * (*g.sw);
    const float rs = g.res_q ? *g.res_scale : 0.0f;
    uint32_t amax = 0;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        const bool col_ok = col < g.N;
        const float bc = (g.bias && col_ok) ? g.bias[col] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + (wm * TM + i) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (!col_ok || row >= g.M) continue;
                const int a = acc[i][j][r];
                if (g.acc_out) g.acc_out[row * g.N + col] = a;
                float v = fmaf((float)a, s, bc);
                if (g.res_q) v = v + (float)g.res_q[row * g.res_ld + col] * rs;
                if (g.act == 1) v = v > 0.0f ? v : 0.0f;
                else if (g.act == 2) {          // erf-form GELU in fp64, rounded once: it feeds a quantiser
                    const double dv = (double)v;
                    v = (float)(0.5 * dv * (1.0 + erf(dv * 0.70710678118654752440)));
                }
                g.y[row * g.ldy + col] = v;
                const uint32_t ab = abs_bits(v);
                amax = amax > ab ? amax : ab;
            }
        }
    }
    if (g.absmax_out) {
        __shared__ uint32_t sm4[4];
        block_atomic_max(amax, g.absmax_out, sm4);
    }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_variant(const GemmArgs &g, hipStream_t st)
{
    const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    if (tiles <= 0) return hipSuccess;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    if (g.conv3x3)
        return launch_k(EGERIA_KERNEL_GEMM, gemm_i8_kernel<BM, BN, WM, WN, true>, dim3((unsigned)tiles), dim3(256), 0,
                        st, g);
    return launch_k(EGERIA_KERNEL_GEMM, gemm_i8_kernel<BM, BN, WM, WN, false>, dim3((unsigned)tiles), dim3(256), 0, st,
                    g);
}

hipError_t launch_gemm_i8(const GemmArgs &g, hipStream_t st)
{
    if (g.N <= 32) return launch_variant<128, 32, 4, 1>(g, st);
    return launch_variant<128, 128, 2, 2>(g, st);
}

}  // namespace egeria
