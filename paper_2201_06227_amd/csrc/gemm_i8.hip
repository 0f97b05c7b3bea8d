// int8 x int8 -> int32 GEMM and implicit-GEMM 3x3 convolution on the gfx950
// matrix cores, with the dequantising epilogue fused (the reference model's
// linear and convolution layers, Section 4.1 of the paper).
//
//   acc[m, n] = sum_k a[m, k] * w[n, k]          (both operands K-contiguous)
//   y[m, n]   = act( fma((float)acc, sx*sw, bias[n]) [+ residual] )
//
// One workgroup of 4 waves owns a BM x BN tile of the output (256x256 down to
// 128x32, chosen so that the grid still fills the chip).  Per K step of 64
// bytes the tile's A and W rows are staged through a double-buffered LDS stage
// (16-byte units, rows padded to 80 bytes so that the 128-bit operand reads of
// a wave fall on distinct banks): the next step's global loads are issued
// before the current step's MFMAs and land in the other buffer after them, so
// there is one barrier per step.  Each wave issues v_mfma_i32_32x32x32_i8:
// lane l supplies 16 consecutive K bytes of row (l % 32) at K offset
// 16 * (l / 32) for A and for W alike, so the product is exact whatever the
// instruction's internal K order is.  Workgroup ids are dealt so that each XCD
// works on a contiguous range of tiles (N fastest) and its L2 serves the
// re-reads of A rows and of the weights.
#include "common.hpp"

namespace egeria {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;          // K bytes per step
constexpr int kLdsRow = 80;      // padded LDS row in bytes

template <int BM, int BN, int WM, int WN, bool CONV>
__global__ __launch_bounds__(256) void gemm_i8_kernel(const GemmArgs g, int tiles, int tiles_per_xcd)
{
    static_assert(WM * WN == 4, "four waves per workgroup");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_IT = (BM * 4 + 255) / 256, B_IT = (BN * 4 + 255) / 256;
    constexpr int STAGE = (BM + BN) * kLdsRow;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];       // [2][BM + BN][80]

    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int tile = xcd * tiles_per_xcd + local;
    if (local >= tiles_per_xcd || tile >= tiles) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tiles_n = (g.N + BN - 1) / BN;
    const int64_t tile_m = tile / tiles_n;
    const int tile_n = tile % tiles_n;
    const int64_t m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int unit = tid & 3;                    // which 16-byte unit of the 64-byte K step
    // epilogue scalars, requested now so that their latency hides behind the K loop
    const float s = (*g.sx) * (*g.sw);
    const float rs = g.res_q ? *g.res_scale : 0.0f;

    // Operands are fetched with raw buffer loads: a lane whose row or K offset is
    // out of range is given an offset beyond the buffer and reads zeros, so the
    // main loop is straight-line code that the scheduler hints below can order.
    constexpr uint32_t kOob = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void *)g.a, 0, (int)g.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void *)g.w, 0, (int)g.w_bytes, 0x00020000);
    uint32_t a_base[A_IT];               // byte offset of the row (linear) or of the centre pixel (conv)
    bool a_ok[A_IT];
    int a_oh[A_IT], a_ow[A_IT];
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
        const int r = (tid + it * 256) >> 2;
        const int64_t m = m0 + r;
        a_ok[it] = r < BM && m < g.M;
        a_base[it] = a_ok[it] ? (uint32_t)(m * (CONV ? (int64_t)g.cp : g.lda)) : 0u;
        if (CONV) {
            a_ow[it] = (int)(m % g.W);
            a_oh[it] = (int)((m / g.W) % g.H);
        }
    }
    uint32_t b_base[B_IT];
    bool b_ok[B_IT];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
        const int r = (tid + it * 256) >> 2;
        b_ok[it] = r < BN && n0 + r < g.N;
        b_base[it] = b_ok[it] ? (uint32_t)(n0 + r) * (uint32_t)g.kp : 0u;
    }

    auto load_tiles = [&](int kt, v4u (&ra)[A_IT], v4u (&rb)[B_IT]) {
        const int k0 = kt * kBK + unit * 16;
        const bool k_ok = k0 < g.kp;
        int dh = 0, dw = 0, delta = k0;
        if (CONV) {
            const int tap = k0 / g.cp;
            const int kh = tap / 3;
            dh = kh - 1;
            dw = tap - kh * 3 - 1;
            delta = (dh * g.W + dw) * g.cp + (k0 - tap * g.cp);
        }
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            bool ok = a_ok[it] && k_ok;
            if (CONV) ok = ok && (unsigned)(a_oh[it] + dh) < (unsigned)g.H && (unsigned)(a_ow[it] + dw) < (unsigned)g.W;
            ra[it] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, ok ? a_base[it] + (uint32_t)delta : kOob, 0, 0);
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it)
            rb[it] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (b_ok[it] && k_ok) ? b_base[it] + (uint32_t)k0 : kOob, 0, 0);
    };
    auto store_tiles = [&](int stage, const v4u (&ra)[A_IT], const v4u (&rb)[B_IT]) {
        uint8_t *sA = lds + stage * STAGE, *sB = sA + BM * kLdsRow;
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
            const int r = (tid + it * 256) >> 2;
            if ((BM * 4) % 256 == 0 || r < BM) *(v4u *)&sA[r * kLdsRow + unit * 16] = ra[it];
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
            const int r = (tid + it * 256) >> 2;
            if ((BN * 4) % 256 == 0 || r < BN) *(v4u *)&sB[r * kLdsRow + unit * 16] = rb[it];
        }
    };
    // operand fragments of one 32-byte K half-step
    auto read_frags = [&](int stage, int ks, v4i (&fa)[TM], v4i (&fb)[TN]) {
        const uint8_t *sA = lds + stage * STAGE, *sB = sA + BM * kLdsRow;
        const int koff = (ks * 2 + (lane >> 5)) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *(const v4i *)&sA[((wm * TM + i) * 32 + (lane & 31)) * kLdsRow + koff];
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = *(const v4i *)&sB[((wn * TN + j) * 32 + (lane & 31)) * kLdsRow + koff];
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    auto mfma_all = [&](const v4i (&fa)[TM], const v4i (&fb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };

    // Software pipeline.  Global loads run two K steps ahead in two register
    // sets; LDS holds two stages; operand fragments are double buffered.  The
    // scheduler hints spread the step's memory instructions between its MFMAs:
    // an MFMA occupies the matrix pipe for 32 cycles during which the wave may
    // issue loads, LDS reads and LDS writes, and the LDS write port (a quarter
    // of the read rate) is the scarce resource.
    constexpr int NMF = TM * TN;                 // MFMAs per half step
    constexpr int NLD = A_IT + B_IT;             // global loads / LDS writes per step
    constexpr int NRD = TM + TN;                 // LDS operand reads per half step
    const int nk = (g.kp + kBK - 1) / kBK;
    v4u ra0[A_IT], rb0[B_IT], ra1[A_IT], rb1[B_IT];
    v4i fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    load_tiles(0, ra0, rb0);
    load_tiles(1, ra1, rb1);
    store_tiles(0, ra0, rb0);
    __syncthreads();
    read_frags(0, 0, fa0, fb0);
    // step kt: tile kt is in LDS stage kt & 1, tile kt + 1 is in (or on its way to)
    // the register set `rs`, tile kt + 2 is requested into the set `rl`
    auto step = [&](int kt, v4u (&rsa)[A_IT], v4u (&rsb)[B_IT], v4u (&rla)[A_IT], v4u (&rlb)[B_IT]) {
        load_tiles(kt + 2, rla, rlb);            // past the end of K the loader returns zeros
        read_frags(kt & 1, 1, fa1, fb1);
        store_tiles((kt + 1) & 1, rsa, rsb);
        mfma_all(fa0, fb0);
#pragma unroll
        for (int i = 0; i < NMF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA
            if (i < NLD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);          // one global load
            if (i < NRD) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);          // one LDS read
            if (i >= NMF - NLD) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // one LDS write
        }
        __syncthreads();
        read_frags((kt + 1) & 1, 0, fa0, fb0);
        mfma_all(fa1, fb1);
#pragma unroll
        for (int i = 0; i < NMF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < NRD) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    for (int kt = 0; kt < nk; kt += 2) {        // an odd count runs one extra step on zeros
        step(kt, ra1, rb1, ra0, rb0);
        step(kt + 1, ra0, rb0, ra1, rb1);
    }
    __syncthreads();

    // ---- epilogue.  Lane l of a 32x32 accumulator block holds column l % 32 and
    // rows 8 * (r / 4) + 4 * (l / 32) + r % 4 (r = 0..15).  One block row of the
    // wave tile at a time is passed through LDS (free now) so that each lane ends
    // up with four consecutive columns of one row: 16-byte loads of bias and
    // residual, 16-byte stores of the output.
    constexpr int EW = TN * 32, ELD = EW + 4;
    constexpr int QPR = EW / 4;                  // 4-column groups per row; divides 64
    constexpr int RPI = 64 / QPR;                // rows a wave covers per pass
    int *ebuf = (int *)lds + wave * 32 * ELD;
    const bool vec4 = (g.N & 3) == 0 && (g.ldy & 3) == 0;
    // a lane keeps the same four columns through the whole epilogue
    const int c4 = (lane % QPR) * 4;
    const int col = n0 + wn * EW + c4;
    const bool full = vec4 && col + 4 <= g.N;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (g.bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < g.N) bv[e] = g.bias[col + e];
    }
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                ebuf[((r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * ELD + j * 32 + (lane & 31)] = acc[i][j][r];
        __syncthreads();
#pragma unroll 4
        for (int pass = 0; pass < 32 / RPI; ++pass) {
            const int rr = pass * RPI + lane / QPR;
            const int64_t row = m0 + (wm * TM + i) * 32 + rr;
            if (row >= g.M || col >= g.N) continue;
            const int4 a4 = *(const int4 *)&ebuf[rr * ELD + c4];
            const int av[4] = {a4.x, a4.y, a4.z, a4.w};
            float rv[4] = {0.f, 0.f, 0.f, 0.f}, out[4];
            if (g.res_q) {
                const int8_t *rp = g.res_q + row * g.res_ld + col;
                if (full) {
                    const uint32_t w = *(const uint32_t *)rp;
#pragma unroll
                    for (int e = 0; e < 4; ++e) rv[e] = (float)(int8_t)((w >> (8 * e)) & 0xff) * rs;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < g.N) rv[e] = (float)rp[e] * rs;
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = fmaf((float)av[e], s, bv[e]);
                if (g.res_q) v = v + rv[e];
                if (g.act == 1) v = v > 0.0f ? v : 0.0f;
                out[e] = v;
                if (col + e < g.N) {
                    const uint32_t ab = g.amax_pos ? (v > 0.0f ? __float_as_uint(v) : 0u) : abs_bits(v);
                    amax = amax > ab ? amax : ab;
                }
            }
            if (full) {
                *(float4 *)(g.y + row * g.ldy + col) = make_float4(out[0], out[1], out[2], out[3]);
                if (g.acc_out) *(int4 *)(g.acc_out + row * g.N + col) = a4;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < g.N) {
                        g.y[row * g.ldy + col + e] = out[e];
                        if (g.acc_out) g.acc_out[row * g.N + col + e] = av[e];
                    }
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
    if (tiles > 0x3fffffffLL) return hipErrorInvalidValue;
    const int tpx = (int)((tiles + 7) / 8);
    const dim3 grid((unsigned)(tpx * 8)), block(256);
    constexpr size_t smem = (size_t)2 * (BM + BN) * kLdsRow;
    hipError_t e;
    if (g.conv3x3) {
        static bool set = false;
        if (!set) {
            e = hipFuncSetAttribute((const void *)gemm_i8_kernel<BM, BN, WM, WN, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
            set = true;
        }
        return launch_k(EGERIA_KERNEL_GEMM, gemm_i8_kernel<BM, BN, WM, WN, true>, grid, block, smem, st, g, (int)tiles,
                        tpx);
    }
    static bool set = false;
    if (!set) {
        e = hipFuncSetAttribute((const void *)gemm_i8_kernel<BM, BN, WM, WN, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        set = true;
    }
    return launch_k(EGERIA_KERNEL_GEMM, gemm_i8_kernel<BM, BN, WM, WN, false>, grid, block, smem, st, g, (int)tiles,
                    tpx);
}

// ---- 3x3 convolution with at most 16 input channels and at most 32 outputs ----------------
// (the first stages of CIFAR-style ResNets).  The problem is bandwidth bound and
// each output pixel needs only 9 x 16 bytes of input, so there is no LDS stage
// and no barrier: a wave owns 32 consecutive output pixels; lane l reads, for
// K step s, the 16 channel bytes of pixel l % 32 displaced by tap 2s + l / 32
// (half-waves read contiguous 512-byte runs) and the matching 16 weight bytes of
// output channel l % 32; five MFMAs cover the nine taps (the tenth is zero).
__global__ __launch_bounds__(256) void conv3x3_c16_kernel(const GemmArgs g)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 31, h = lane >> 5;
    const int64_t m = ((int64_t)blockIdx.x * 4 + wave) * 32 + p;
    const bool m_ok = m < g.M;
    const int ow = (int)(m % g.W), oh = (int)((m / g.W) % g.H);
    const float s = (*g.sx) * (*g.sw);
    const float rs = g.res_q ? *g.res_scale : 0.0f;
    v4i fa[5], fb[5];
#pragma unroll
    for (int st = 0; st < 5; ++st) {
        const int tap = 2 * st + h;
        const int kh = tap / 3, dh = kh - 1, dw = tap - kh * 3 - 1;
        const bool ok = m_ok && tap < 9 && (unsigned)(oh + dh) < (unsigned)g.H && (unsigned)(ow + dw) < (unsigned)g.W;
        fa[st] = ok ? *(const v4i *)(g.a + (m + (int64_t)dh * g.W + dw) * 16) : v4i{0, 0, 0, 0};
        fb[st] = (p < g.N && tap < 9) ? *(const v4i *)(g.w + (int64_t)p * g.kp + tap * 16) : v4i{0, 0, 0, 0};
    }
    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
#pragma unroll
    for (int st = 0; st < 5; ++st) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[st], fb[st], acc, 0, 0, 0);

    // lane holds output channel p and pixels 8 * (r / 4) + 4 * h + r % 4 of the wave's 32
    const int col = p;
    const bool col_ok = col < g.N;
    const float bc = (g.bias && col_ok) ? g.bias[col] : 0.0f;
    const int64_t mw = ((int64_t)blockIdx.x * 4 + wave) * 32;
    uint32_t amax = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t row = mw + (r >> 2) * 8 + h * 4 + (r & 3);
        if (!col_ok || row >= g.M) continue;
        const int a = acc[r];
        if (g.acc_out) g.acc_out[row * g.N + col] = a;
        float v = fmaf((float)a, s, bc);
        if (g.res_q) v = v + (float)g.res_q[row * g.res_ld + col] * rs;
        if (g.act == 1) v = v > 0.0f ? v : 0.0f;
        g.y[row * g.ldy + col] = v;
        const uint32_t ab = g.amax_pos ? (v > 0.0f ? __float_as_uint(v) : 0u) : abs_bits(v);
        amax = amax > ab ? amax : ab;
    }
    if (g.absmax_out) {
        __shared__ uint32_t sm4[4];
        block_atomic_max(amax, g.absmax_out, sm4);
    }
}

// Tile choice.  With fp32 outputs the epilogue (convert, scale, store) costs as
// much as the K loop unless K is long, so two 128x128 workgroups per CU, one in
// its K loop while the other stores, beat one 256-wide workgroup; the wide
// tiles pay off for long K, where the LDS and L1 traffic per MFMA matters.
hipError_t launch_gemm_i8(const GemmArgs &g, hipStream_t st)
{
    auto ntiles = [&](int bm, int bn) { return ((g.M + bm - 1) / bm) * (int64_t)((g.N + bn - 1) / bn); };
    if (g.conv3x3 && g.cp == 16 && g.N <= 32) {
        const int64_t blocks = (g.M + 127) / 128;
        if (blocks <= 0) return hipSuccess;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        return launch_k(EGERIA_KERNEL_GEMM, conv3x3_c16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, g);
    }
    if (g.N <= 32) return launch_variant<128, 32, 4, 1>(g, st);
    if (g.kp >= 2048) {
        if (ntiles(256, 256) >= 448) return launch_variant<256, 256, 2, 2>(g, st);
        if (ntiles(256, 128) >= 224) return launch_variant<256, 128, 2, 2>(g, st);
    }
    return launch_variant<128, 128, 2, 2>(g, st);
}

}  // namespace egeria
