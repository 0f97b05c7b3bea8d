// int8 x int8 -> int32 GEMM and implicit-GEMM 3x3 convolution on the gfx950
// matrix cores, with the dequantising epilogue fused (the reference model's
// linear and convolution layers, Section 4.1 of the paper).
//
//   acc[m, n] = sum_k a[m, k] * w[n, k]          (both operands K-contiguous)
//   y[m, n]   = act( fma((float)acc, sx*sw, bias[n]) [+ residual] )
//
// One workgroup of 4 (or, for the two largest tiles of big linear layers, 8)
// waves owns a BM x BN tile of the output (256x256 down to 128x32, chosen so
// that the grid still fills the chip).  Per K step of 64 or
// 128 bytes the tile's A and W rows go from global memory straight into a ring
// of LDS stages (buffer loads with the LDS modifier; 16-byte units, rotated by
// an exclusive-or of the row so that the 128-bit operand reads of a wave fall
// on distinct banks): while the matrix cores work on one stage the following
// steps are landing in the others, one barrier per step.  Each wave issues
// v_mfma_i32_32x32x32_i8: lane l supplies 16 consecutive K bytes of row
// (l % 32) at K offset 16 * (l / 32) for A and for W alike, so the product is
// exact whatever the instruction's internal K order is.  Workgroup ids are
// dealt so that each XCD works on a contiguous range of tiles (N fastest) and
// its L2 serves the re-reads of A rows and of the weights.
#include "common.hpp"
#include <type_traits>

namespace egeria {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// K bytes per step, BK: 128 (one 128-byte cache line of every row per request)
// or 64.  With 64-byte steps each line is fetched half now and half one step
// later; the stage is half as large, so more workgroups or stages fit a CU -
// but a request for half a line costs the L2 -> LDS path as much as one for a
// whole line (measured: 29 against 62 bytes per clock and compute unit), so the
// 64-byte shapes are bound by that path as soon as the matrix cores are fed
// well.  The eight-wave shapes take whole lines, two stages of them, and a
// tile large enough that one workgroup per compute unit keeps two waves on
// every SIMD.
// LDS stages of a tile shape: one being read, the others being filled.
constexpr int stages_for(int bm, int bn, int bk)
{
    const int stage = (bm + bn) * bk;
    if (bk == 64) {
        if (bm == 64 && bn == 768) return 3;           // the row-owning tile: three stages fill the 160 KB exactly
        if (bm * bn < 256 * 192) return 3;
        const int fit = 150 * 1024 / stage;
        return fit > 6 ? 6 : fit;
    }
    if (3 * stage > 150 * 1024) return 2;
    return 2 * stage <= 80 * 1024 ? 2 : 3;
}

typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// Element type of the two operands (ET): 0 = int8 (int32 sums, the reference
// model's default), 1 = float16, 2 = float32 (fp32 sums; the reference model at
// the higher precisions of the paper's Table 2).  The kernel moves bytes: a
// 16-byte unit is 16, 8 or 4 values of K, and one unit pair per lane feeds one
// MFMA (int8, float16) or four (float32, one value each).
template <int ET>
struct AccOf {
    typedef v16i type;
};
template <>
struct AccOf<1> {
    typedef v16f type;
};
template <>
struct AccOf<2> {
    typedef v16f type;
};
template <int ET>
struct ResOf {
    typedef int8_t type;
};
template <>
struct ResOf<1> {
    typedef _Float16 type;
};
template <>
struct ResOf<2> {
    typedef float type;
};
template <int ET>
__device__ __forceinline__ typename AccOf<ET>::type mma(v4i a, v4i b, typename AccOf<ET>::type c)
{
    if constexpr (ET == 0) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    } else if constexpr (ET == 1) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__int_as_float(a[e]), __int_as_float(b[e]), c, 0, 0, 0);
        return c;
    }
}
__device__ __forceinline__ int32_t acc_bits(int a) { return a; }
__device__ __forceinline__ int32_t acc_bits(float a) { return __float_as_int(a); }

typedef __attribute__((address_space(3))) uint8_t lds_byte;

// 16 bytes per lane from a buffer straight into LDS: lane l of the wave writes
// LDS bytes [lds_base + 16 l, lds_base + 16 l + 16) with what it reads at byte
// offset voff of the buffer (zeros if voff is out of range).  Written as an
// assembly statement so that the request stays outstanding across later LDS
// reads of other stages: completion is awaited with an explicit vmcnt wait,
// and ordering against other waves' reads with workgroup barriers.
__device__ __forceinline__ void load_to_lds_b128(v4i rsrc, uint32_t lds_base, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

// Workgroups of a tile shape that are meant to share a CU (one wave of each per
// SIMD): the register allocation is held to 512 / that many registers per lane,
// so that one workgroup's epilogue overlaps another's K loop.
constexpr int resident_target(int bm, int bn)
{
    return bm * bn > 256 * 128 ? 1 : (bm * bn > 128 * 128 ? 2 : 3);
}

template <int BM, int BN, int WM, int WN, bool CONV, int BK, int ET, bool LNF = false>
__global__ __launch_bounds__(64 * WM * WN, resident_target(BM, BN)) void gemm_i8_kernel(const GemmArgs g, int tiles,
                                                                               int tiles_per_xcd)
{
    typedef typename AccOf<ET>::type acc_t;
    typedef typename ResOf<ET>::type res_t;
    static_assert(BK == 64 || BK == 128, "K step of 64 or 128 bytes");
    constexpr int kBK = BK;
    constexpr int UPR = BK / 16;                 // 16-byte K units per row of a stage
    constexpr int kRowsPerChunk = 64 / UPR;      // rows one load instruction of a wave covers
    constexpr int SWR = 16 / UPR;                // rows that share a rotation of the K units
    constexpr int NSUB = BK / 32;                // 32-byte sub-steps (one MFMA deep) per step
    constexpr int NW = WM * WN, NT = 64 * NW;          // waves and threads per workgroup
    static_assert(NW == 4 || NW == 8, "four or eight waves per workgroup");
    static_assert(BM % kRowsPerChunk == 0 && BN % kRowsPerChunk == 0, "tiles are made of whole chunks");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_CH = BM / kRowsPerChunk, B_CH = BN / kRowsPerChunk; // 1-KiB chunks per K step
    constexpr int A_IT = (A_CH + NW - 1) / NW, B_IT = (B_CH + NW - 1) / NW;         // chunks per wave
    constexpr int STAGE = (BM + BN) * kBK;
    constexpr int NST = stages_for(BM, BN, BK);
    constexpr int NLD = A_IT + B_IT;                                    // loads per wave and K step
    static_assert((NST - 2) * NLD < 64, "outstanding loads must fit the wait counter");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];       // [NST][BM + BN][BK]

    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int tile = xcd * tiles_per_xcd + local;
    if (local >= tiles_per_xcd || tile >= tiles) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wm = wave / WN, wn = wave % WN;
    const int tiles_n = (g.N + BN - 1) / BN;
    const int64_t tile_m = tile / tiles_n;
    const int tile_n = tile % tiles_n;
    const int64_t m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    // epilogue scalars, requested now so that their latency hides behind the K loop
    const float sxv = *g.sx;
    const float s = g.sw_per_n ? 0.0f : sxv * (*g.sw);
    const float rs = g.res_q ? (ET == 0 ? *g.res_scale : 1.0f) : 0.0f;
    float q_inv = 0.0f;                          // multiplier of the optional int8 output
    if (g.q_out) q_inv = (float)(1.0 / (double)*g.q_scale);
    // affine activation codes: stored codes are q - 128, so 128 - zero point goes back in
    const int zmul = (ET == 0 && g.zp_in) ? 128 - *g.zp_in : 0;
    const int rmul = (ET == 0 && g.zp_res) ? 128 - *g.zp_res : 0;

    // Operands go from global memory straight into LDS (buffer loads with the
    // LDS modifier): one such instruction of a wave fills 1 KiB, lane l writing
    // bytes [16 l, 16 l + 16) of it, i.e. unit l % UPR of row l / UPR of a chunk
    // of 64 / UPR rows (UPR = BK / 16 units per row).  Which 16 bytes of K a
    // lane fetches for that slot is free, so the K units of row r are stored
    // rotated by (r / (16 / UPR)) % UPR (exclusive-or): the 128-bit operand
    // reads of 16 consecutive rows then fall on 16 distinct bank groups.  A lane whose row or K offset
    // is out of range is given an offset beyond the buffer and writes zeros.
    constexpr uint32_t kOob = 0x80000000u;
    auto descriptor = [](const void *p, int64_t bytes) {             // raw buffer: base, no stride, extent, dword format
        const uint64_t a = (uint64_t)p;
        v4i d;
        d[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
        d[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32) & 0xffff);
        d[2] = __builtin_amdgcn_readfirstlane((int)bytes);
        d[3] = 0x00020000;
        return d;
    };
    const v4i rsrc_a = descriptor(g.a, g.a_bytes), rsrc_w = descriptor(g.w, g.w_bytes);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_byte *)lds;      // LDS address of the stage array
    const int rloc = lane / UPR;                                 // row within the chunk
    // K unit this lane fetches: slot ^ ((row / SWR) % UPR) with row = chunk * (64 / UPR) + rloc and
    // chunk = wave + NW * it; the chunk's share of that is (chunk * 4) % UPR = (wave % 2) * 4 % UPR
    const int unit = (lane % UPR) ^ (((wave_u & 1) * 4 + rloc / SWR) % UPR);
    static_assert(A_CH % 2 == 0 && B_CH % 2 == 0, "a wave's chunks must keep their parity");
    uint32_t a_base[A_IT];               // byte offset of the row (linear) or of the centre pixel (conv)
    bool a_ok[A_IT];
    int a_oh[A_IT], a_ow[A_IT];
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
        const int r = ((wave_u + it * NW) % A_CH) * kRowsPerChunk + rloc;
        const int64_t m = m0 + r;
        a_ok[it] = m < g.M;
        a_base[it] = a_ok[it] ? (uint32_t)(m * (CONV ? (int64_t)g.cp : g.lda)) : 0u;
        if (CONV) {
            // the operand's extent is below 2^31 bytes, so m fits 32 bits (a 64-bit division is a long call)
            const uint32_t mrow = (uint32_t)m / (uint32_t)g.W;
            a_ow[it] = (int)((uint32_t)m - mrow * (uint32_t)g.W);
            a_oh[it] = (int)(mrow % (uint32_t)g.H);
        }
    }
    uint32_t b_base[B_IT];
    bool b_ok[B_IT];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
        const int r = ((wave_u + it * NW) % B_CH) * kRowsPerChunk + rloc;
        b_ok[it] = n0 + r < g.N;
        b_base[it] = b_ok[it] ? (uint32_t)(n0 + r) * (uint32_t)g.kp : 0u;
    }

    // Requests for K step kt into LDS stage `stage`, one 1-KiB chunk per call
    // (idx < A_IT: a chunk of A, else of W).  Every wave issues exactly NLD loads
    // per K step (the waits below count them): where a tile has fewer chunks
    // than that, waves fetch a chunk twice, writing the same bytes.
    struct StepAddr {
        int k0, dh, dw, delta;
        bool k_ok;
    };
    // The row-owning tile: every workgroup streams the whole weight matrix, so all of them would ask the L2 for
    // the same rows at the same time; each starts at a K step of its own instead (integer sums do not depend
    // on the order).  Steps past the end of K stay past the end.
    const int nk_all = (g.kp + kBK - 1) / kBK;
    const int k_rot = LNF ? tile % nk_all : 0;
    auto step_addr = [&](int kt) {
        StepAddr sa;
        if (LNF && kt < nk_all) kt = kt + k_rot < nk_all ? kt + k_rot : kt + k_rot - nk_all;
        sa.k0 = kt * kBK + unit * 16;
        sa.k_ok = sa.k0 < g.kp;
        sa.dh = 0;
        sa.dw = 0;
        sa.delta = sa.k0;
        if (CONV) {
            const int tap = sa.k0 / g.cp;
            const int kh = tap / 3;
            sa.dh = kh - 1;
            sa.dw = tap - kh * 3 - 1;
            sa.delta = (sa.dh * g.W + sa.dw) * g.cp + (sa.k0 - tap * g.cp);
        }
        return sa;
    };
    auto fetch_one = [&](const StepAddr &sa, int stage, int idx) {
        const uint32_t sA = lds0 + stage * STAGE, sB = sA + BM * kBK;
        if (idx < A_IT) {
            const int it = idx;
            const int chunk = (wave_u + it * NW) % A_CH;
            bool ok = a_ok[it] && sa.k_ok;
            if (CONV)
                ok = ok && (unsigned)(a_oh[it] + sa.dh) < (unsigned)g.H && (unsigned)(a_ow[it] + sa.dw) < (unsigned)g.W;
            load_to_lds_b128(rsrc_a, sA + chunk * 1024, ok ? a_base[it] + (uint32_t)sa.delta : kOob);
        } else {
            const int it = idx - A_IT;
            const int chunk = (wave_u + it * NW) % B_CH;
            load_to_lds_b128(rsrc_w, sB + chunk * 1024, (b_ok[it] && sa.k_ok) ? b_base[it] + (uint32_t)sa.k0 : kOob);
        }
    };
    auto fetch = [&](int kt, int stage) {
        const StepAddr sa = step_addr(kt);
#pragma unroll
        for (int idx = 0; idx < A_IT + B_IT; ++idx) fetch_one(sa, stage, idx);
    };
    // operand fragments of one 32-byte K sub-step ks: lane l supplies row l % 32, K unit 2 ks + l / 32
    const int frow = lane & 31;
    const int fsw = (frow / SWR) % UPR;
    auto read_frags = [&](int stage, int ks, v4i (&fa)[TM], v4i (&fb)[TN]) {
        const uint8_t *sA = lds + stage * STAGE, *sB = sA + BM * kBK;
        const int koff = ((ks * 2 + (lane >> 5)) ^ fsw) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *(const v4i *)&sA[((wm * TM + i) * 32 + frow) * kBK + koff];
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[j] = *(const v4i *)&sB[((wn * TN + j) * 32 + frow) * kBK + koff];
    };

    acc_t acc[TM][TN];
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
                acc[i][j] = mma<ET>(fa[i], fb[j], acc[i][j]);
    };

    // Software pipeline over a ring of NST LDS stages.  During step kt the
    // matrix cores work on stage kt % NST, K steps kt + 1 .. kt + NST - 2 are
    // landing in the following stages and K step kt + NST - 1 is requested into
    // the stage that step kt - 1 read (every wave has passed the barrier that
    // ended that step).  One barrier per step; a step is two or four 32-byte
    // sub-steps whose operand fragments are double-buffered in registers.
    constexpr int NMF = TM * TN;                 // MFMAs per sub-step
    constexpr int NRD = TM + TN;                 // LDS operand reads per sub-step
    constexpr int kWaitNext = 0x0f70 | (((NST - 2) * NLD) & 0xf) | ((((NST - 2) * NLD) >> 4) << 14);   // vmcnt only
    const int nk = (g.kp + kBK - 1) / kBK;
    v4i fa0[TM], fb0[TN], fa1[TM], fb1[TN];
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) fetch(p, p);
    __builtin_amdgcn_s_waitcnt(kWaitNext);       // K step 0 landed
    __syncthreads();
    read_frags(0, 0, fa0, fb0);
    auto hint = [&]() {                           // one LDS read after each of the first MFMAs
#pragma unroll
        for (int i = 0; i < NMF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < NRD) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    int st = 0;                                  // stage of K step kt
    for (int kt = 0; kt < nk; ++kt) {            // past the end of K the loads return zeros
        const int st1 = st == NST - 1 ? 0 : st + 1, stl = st == 0 ? NST - 1 : st - 1;
        read_frags(st, 1, fa1, fb1);
        const StepAddr sa = step_addr(kt + NST - 1);
        // the step's requests are spread between its first MFMAs: a burst of them
        // would fill the memory pipeline's queue and stall the wave's MFMA issue
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                acc[i][j] = mma<ET>(fa0[i], fb0[j], acc[i][j]);
                constexpr int per = (NLD + NMF - 1) / NMF;               // requests after each MFMA
#pragma unroll
                for (int q = 0; q < per; ++q)
                    if ((i * TN + j) * per + q < NLD) fetch_one(sa, stl, (i * TN + j) * per + q);
                if ((i * TN + j) * per < NLD) __builtin_amdgcn_sched_barrier(0);   // keep the MFMA before its requests
            }
        if (NSUB == 4) {
            read_frags(st, 2, fa0, fb0);
            mfma_all(fa1, fb1);
            hint();
            read_frags(st, 3, fa1, fb1);
            mfma_all(fa0, fb0);
            hint();
        }
        __builtin_amdgcn_s_waitcnt(kWaitNext);   // K step kt + 1 landed
        __syncthreads();
        read_frags(st1, 0, fa0, fb0);
        mfma_all(fa1, fb1);
        hint();
        st = st1;
        if (TM * TN == 16) {
            // 256 accumulators per lane: name the accumulation registers as their home, or the
            // allocator splits them between the two register files and spills inside the loop
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i][j]));
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the zero-filled K steps past the end

    // The int8 residual of the tile goes through LDS (the stage memory is free
    // now): one coalesced pass of 16-byte loads instead of one byte load per
    // output element issued from inside the epilogue, whose round trips would add up.
    constexpr bool RES_LDS = ET == 0;
    static_assert(!RES_LDS || (size_t)NST * STAGE >= (size_t)BM * BN, "the residual tile must fit the stage memory");
    if (RES_LDS && g.res_q) {
        constexpr int RU = BN / 16, RIT = (BM * RU + NT - 1) / NT;     // 16-byte units per row, units per thread
        v4i rv[RIT];
        __syncthreads();                                              // every wave has read its last operands
#pragma unroll
        for (int it = 0; it < RIT; ++it) {
            const int u = tid + it * NT, rr = u / RU, cu = u % RU;
            const int64_t m = m0 + rr;
            const int64_t col = n0 + cu * 16;
            rv[it] = v4i{0, 0, 0, 0};
            if (u < BM * RU && m < g.M && col < g.res_ld) rv[it] = *(const v4i *)(g.res_q + m * g.res_ld + col);
        }
#pragma unroll
        for (int it = 0; it < RIT; ++it) {
            const int u = tid + it * NT;
            if (u < BM * RU) *(v4i *)&lds[(u / RU) * BN + (u % RU) * 16] = rv[it];
        }
        __syncthreads();
    }

    // ---- epilogue, straight from the accumulators.  Lane l of a 32x32 block
    // holds column l % 32 and rows 8 * (r / 4) + 4 * (l / 32) + r % 4 (r = 0..15),
    // so for a fixed r each half of the wave owns 32 consecutive columns of one
    // row: every store instruction writes two full 128-byte row segments, and the
    // row part of the address is uniform (scalar arithmetic only).
    const int lcol = lane & 31, lrow = (lane >> 5) * 4;
    const int wm_u = __builtin_amdgcn_readfirstlane(wm), wn_u = __builtin_amdgcn_readfirstlane(wn);
    // Running maximum for the next quantiser, kept as a bit pattern so that a
    // NaN or an infinity stays visible.  Non-negative values (after ReLU, or
    // when only positive values are wanted) order like signed integers.
    const bool pos = g.amax_pos != 0;
    int32_t amax = 0;
    const bool interior = m0 + BM <= g.M && n0 + BN <= g.N && (g.y || g.q_out) && !g.acc_out && !g.zp_in && !g.zp_res;
    const uint32_t qoff = g.q_out ? (uint32_t)(lrow * g.q_ld + lcol) : 0u;
    const uint32_t yoff = (uint32_t)(lrow * g.ldy + lcol);
    const uint32_t roff = g.res_q ? (uint32_t)(lrow * g.res_ld + lcol) : 0u;
    const uint32_t aoff = (uint32_t)(lrow * g.N + lcol);
    // EDGE false: interior tile, no bounds tests, no observation outputs.
    // EDGE true : edge tiles and observed runs, every element tested.
    // QOUT (interior tiles): the tile also, or only, goes out as int8 codes.
    auto emit = [&](auto edge_c, auto res_c, auto relu_c, auto pos_c, auto qout_c) {
        constexpr bool EDGE = decltype(edge_c)::value, RES = decltype(res_c)::value, RELU = decltype(relu_c)::value;
        constexpr bool POS = decltype(pos_c)::value, QOUT = decltype(qout_c)::value;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col0 = n0 + (wn_u * TN + j) * 32;
            const bool col_ok = !EDGE || col0 + lcol < g.N;
            const float bj = (g.bias && col_ok) ? g.bias[col0 + lcol] : 0.0f;
            const float sj = g.sw_per_n ? (col_ok ? sxv * g.sw[col0 + lcol] : 0.0f) : s;   // one fp32 multiply
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int64_t row0 = m0 + (wm_u * TM + i) * 32;
                float *yb = g.y + row0 * g.ldy + col0;
                const res_t *rb = (const res_t *)g.res_q + row0 * g.res_ld + col0;
                int32_t *ab = g.acc_out + row0 * g.N + col0;
                int8_t *qb = g.q_out + row0 * g.q_ld + col0;
                const int rows_left = EDGE ? (int)(g.M - row0 < 32 ? g.M - row0 : 32) - lrow : 32;
                // the block stays in the accumulation registers until its turn
                asm volatile("" : "+a"(acc[i][j]));
                // float residuals of an interior block: all sixteen requested before the first is used
                // (interleaved with the stores of y the compiler keeps each load behind the store before it)
                float rpre[16];
                if constexpr (!RES_LDS && !EDGE && RES) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        rpre[r] = (float)rb[(size_t)(8 * (r >> 2) + (r & 3)) * g.res_ld + roff];
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rr = 8 * (r >> 2) + (r & 3);
                    if (EDGE && !(col_ok && rr < rows_left)) {
                        // pad columns of the int8 output are zero
                        if (g.q_out && !col_ok && col0 + lcol < g.q_ld && rr < rows_left) qb[(size_t)rr * g.q_ld + qoff] = 0;
                        continue;
                    }
                    auto a = acc[i][j][r];
                    if constexpr (EDGE && ET == 0) {
                        if (g.zp_in) {
                            // the sum of the centred codes: the weight codes of this output channel, over the
                            // window positions inside the image for this pixel, times 128 - zero point
                            int cls = 0;
                            if (CONV) {
                                const uint32_t m = (uint32_t)(row0 + lrow + rr);
                                const uint32_t mrow = m / (uint32_t)g.W;
                                const int ow = (int)(m - mrow * (uint32_t)g.W), oh = (int)(mrow % (uint32_t)g.H);
                                cls = (oh == 0 ? 1 : 0) | (oh == g.H - 1 ? 2 : 0) | (ow == 0 ? 4 : 0) | (ow == g.W - 1 ? 8 : 0);
                            }
                            a += zmul * g.colsum[(size_t)cls * g.N + col0 + lcol];
                        }
                    }
                    float v = fmaf((float)a, sj, bj);
                    if (EDGE ? g.res_q != nullptr : RES) {
                        if constexpr (RES_LDS)
                            v = v + (float)((int)(int8_t)lds[((wm_u * TM + i) * 32 + lrow + rr) * BN + (wn_u * TN + j) * 32 + lcol] + rmul) * rs;
                        else if constexpr (!EDGE && RES)
                            v = v + rpre[r] * rs;
                        else
                            v = v + (float)rb[(size_t)rr * g.res_ld + roff] * rs;
                    }
                    if (EDGE ? g.act == 1 : RELU) v = v > 0.0f ? v : 0.0f;
                    if (EDGE ? g.y != nullptr : (!QOUT || g.y != nullptr)) yb[(size_t)rr * g.ldy + yoff] = v;
                    if (EDGE ? g.q_out != nullptr : QOUT) qb[(size_t)rr * g.q_ld + qoff] = (int8_t)quant1(v, q_inv);
                    if (EDGE && g.acc_out) ab[(size_t)rr * g.N + aoff] = acc_bits(a);
                    int32_t bits = (int32_t)__float_as_uint(v);
                    if (EDGE ? !(g.act == 1 || pos) : !(RELU || POS)) bits &= 0x7fffffff;
                    amax = amax > bits ? amax : bits;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    using T = std::true_type;
    using F = std::false_type;
    if constexpr (LNF) {
        // The layer norm of the rows in the same launch: the workgroup owns whole rows (one tile across N).
        // A 32-row block of the fp32 output goes to LDS (the stage memory is free now), then each wave
        // normalises rows of it exactly as layernorm_vec_kernel does with a stored tensor: lane l holds the
        // 16-byte units l, l + 64, ... of the row, and the arithmetic is the shared ln_row_vec.  The residual
        // rows are requested before the barrier, gamma and beta once.
        static_assert(WM == 1 && ET == 0 && !CONV, "whole rows of a linear layer with int8 operands");
        constexpr int YS = BN + 8;                      // floats per row of the block in LDS (pad: the two rows a
                                                        // store instruction writes fall into different banks)
        constexpr int NV = BN / 256, RPW = 32 / NW;     // 16-byte units per lane and row; rows per wave and block
        static_assert(BN % 256 == 0 && 32 % NW == 0, "rows of 256 NV floats, a wave takes whole rows");
        static_assert((size_t)NST * STAGE >= (size_t)32 * YS * 4, "a 32-row block must fit the stage memory");
        float *yt = (float *)lds;
        const int H = g.N, nv = H >> 2;
        const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f), one4 = make_float4(1.f, 1.f, 1.f, 1.f);
        float4 gmv[NV], btv[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int c = lane + 64 * u, cc = c < nv ? c : nv - 1;
            gmv[u] = g.ln_gamma ? reinterpret_cast<const float4 *>(g.ln_gamma)[cc] : one4;
            btv[u] = g.ln_beta ? reinterpret_cast<const float4 *>(g.ln_beta)[cc] : zero4;
        }
        uint32_t amax_u = 0;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            __syncthreads();                            // the stage memory (or the block before) has been read
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = (wn_u * TN + j) * 32 + lcol;
                const bool col_ok = col < g.N;
                const float bj = (g.bias && col_ok) ? g.bias[col] : 0.0f;
                const float sj = g.sw_per_n ? (col_ok ? sxv * g.sw[col] : 0.0f) : s;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    yt[(lrow + 8 * (r >> 2) + (r & 3)) * YS + col] = fmaf((float)acc[i][j][r], sj, bj);
            }
            float4 rv[RPW][NV];
#pragma unroll
            for (int k = 0; k < RPW; ++k) {
                const int64_t row = m0 + i * 32 + wave_u + NW * k;
                const float4 *rr = reinterpret_cast<const float4 *>(g.ln_res + (row < g.M ? row : g.M - 1) * H);
#pragma unroll
                for (int u = 0; u < NV; ++u) {
                    const int c = lane + 64 * u;
                    rv[k][u] = rr[c < nv ? c : nv - 1];
                }
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < RPW; ++k) {
                const int lr = wave_u + NW * k;
                const int64_t row = m0 + i * 32 + lr;
                if (row < g.M) {
                    float4 xv[NV], o[NV];
#pragma unroll
                    for (int u = 0; u < NV; ++u) {
                        const int c = lane + 64 * u;
                        const bool in = c < nv;
                        xv[u] = in ? *reinterpret_cast<const float4 *>(&yt[lr * YS + 4 * c]) : zero4;
                        if (!in) rv[k][u] = zero4;
                    }
                    ln_row_vec<NV>(xv, rv[k], gmv, btv, lane, nv, H, g.ln_eps, o, amax_u);
#pragma unroll
                    for (int u = 0; u < NV; ++u) {
                        const int c = lane + 64 * u;
                        if (c < nv) reinterpret_cast<float4 *>(g.ln_out + row * H)[c] = o[u];
                    }
                }
            }
        }
        amax = (int32_t)amax_u;
    } else
    if (!interior || (g.q_out && (g.res_q || g.act != 1))) emit(T{}, F{}, F{}, F{}, F{});
    else if (g.q_out) emit(F{}, F{}, T{}, F{}, T{});
    else if (g.res_q) {
        if (g.act == 1) emit(F{}, T{}, T{}, F{}, F{}); else emit(F{}, T{}, F{}, F{}, F{});
    } else {
        if (g.act == 1) emit(F{}, F{}, T{}, F{}, F{});
        else if (pos) emit(F{}, F{}, F{}, T{}, F{});
        else emit(F{}, F{}, F{}, F{}, F{});
    }
    if (g.absmax_out) {
        __shared__ uint32_t smw[NW];
        if constexpr (NW == 4) {
            block_atomic_max((uint32_t)amax, g.absmax_out, smw);
        } else {
            uint32_t v = (uint32_t)amax;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
                v = o > v ? o : v;
            }
            if (lane == 0) smw[wave] = v;
            __syncthreads();
            if (tid == 0) {
                uint32_t a = 0;
#pragma unroll
                for (int w = 0; w < NW; ++w) a = smw[w] > a ? smw[w] : a;
                uint32_t *way = g.absmax_out + (blockIdx.x & (kAmaxWays - 1)) * kAmaxStride;
                if (a > __hip_atomic_load(way, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(way, a);
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int BK, int ET = 0, bool LNF = false>
static hipError_t launch_variant(const GemmArgs &g, hipStream_t st)
{
    const int64_t tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    if (tiles <= 0) return hipSuccess;
    if (tiles > 0x3fffffffLL) return hipErrorInvalidValue;
    const int tpx = (int)((tiles + 7) / 8);
    const dim3 grid((unsigned)(tpx * 8)), block(64 * WM * WN);
    constexpr size_t smem = (size_t)stages_for(BM, BN, BK) * (BM + BN) * BK;
    hipError_t e;
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    if (g.conv3x3) {
        static bool set[kMaxDevices] = {};                   // the attribute belongs to one device's code object
        if (!set[dev]) {
            e = hipFuncSetAttribute((const void *)gemm_i8_kernel<BM, BN, WM, WN, true, BK, ET>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
            set[dev] = true;
        }
        return launch_k(EGERIA_KERNEL_GEMM, gemm_i8_kernel<BM, BN, WM, WN, true, BK, ET>, grid, block, smem, st, g,
                        (int)tiles, tpx);
    }
    static bool set[kMaxDevices] = {};
    if (!set[dev]) {
        e = hipFuncSetAttribute((const void *)gemm_i8_kernel<BM, BN, WM, WN, false, BK, ET, LNF>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        set[dev] = true;
    }
    // (instrumentation: the launch that also normalises its rows is timed with the layer norms, whose bytes bound it)
    return launch_k(LNF ? EGERIA_KERNEL_LAYERNORM : EGERIA_KERNEL_GEMM, gemm_i8_kernel<BM, BN, WM, WN, false, BK, ET, LNF>,
                    grid, block, smem, st, g, (int)tiles, tpx);
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
    // the operand's extent is below 2^31 bytes, so pixel indices fit 32 bits (64-bit division is slow)
    const uint32_t mrow = (uint32_t)m / (uint32_t)g.W;
    const int ow = (int)((uint32_t)m - mrow * (uint32_t)g.W), oh = (int)(mrow % (uint32_t)g.H);
    const float s = (*g.sx) * (g.sw_per_n ? (p < g.N ? g.sw[p] : 0.0f) : *g.sw);   // lane's output channel is p
    const float rs = g.res_q ? *g.res_scale : 0.0f;
    // the residual of the workgroup's 128 pixels (16 bytes each, contiguous): requested now with
    // one 16-byte load per thread, handed to the epilogue through LDS
    __shared__ __attribute__((aligned(16))) uint8_t sres[128 * 16];
    const bool res16 = g.res_q != nullptr && g.res_ld == 16;
    v4i resv = {0, 0, 0, 0};
    if (res16 && threadIdx.x < 128) {
        const int64_t pix = (int64_t)blockIdx.x * 128 + threadIdx.x;
        if (pix < g.M) resv = *(const v4i *)(g.res_q + pix * 16);
    }
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
    const float q_inv = g.q_out ? (float)(1.0 / (double)*g.q_scale) : 0.0f;
    if (res16) {
        if (threadIdx.x < 128) *(v4i *)&sres[threadIdx.x * 16] = resv;
        __syncthreads();
    }
    uint32_t amax = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t row = mw + (r >> 2) * 8 + h * 4 + (r & 3);
        if (row >= g.M) continue;
        if (!col_ok) {
            if (g.q_out && col < g.q_ld) g.q_out[row * g.q_ld + col] = 0;     // pad columns of the int8 output
            continue;
        }
        const int a = acc[r];
        if (g.acc_out) g.acc_out[row * g.N + col] = a;
        float v = fmaf((float)a, s, bc);
        if (res16) v = v + (float)(int8_t)sres[(wave * 32 + (r >> 2) * 8 + h * 4 + (r & 3)) * 16 + col] * rs;
        else if (g.res_q) v = v + (float)g.res_q[row * g.res_ld + col] * rs;
        if (g.act == 1) v = v > 0.0f ? v : 0.0f;
        if (g.y) g.y[row * g.ldy + col] = v;
        if (g.q_out) g.q_out[row * g.q_ld + col] = (int8_t)quant1(v, q_inv);
        const uint32_t ab = g.amax_pos ? (v > 0.0f ? __float_as_uint(v) : 0u) : abs_bits(v);
        amax = amax > ab ? amax : ab;
    }
    if (g.absmax_out) {
        __shared__ uint32_t sm4[4];
        block_atomic_max(amax, g.absmax_out, sm4);
    }
}

// ---- the same convolution with the quantiser of its operands folded in -------------------
// A workgroup owns 128 consecutive output pixels.  It reduces the candidate
// maxima of the operand's quantise point to the scale (as every quantise kernel
// does), turns the fp32 values of its pixels and of the W + 1 pixels before and
// after them into int8 codes in LDS (16 bytes per pixel), and the five MFMAs
// of a wave read their operands from there.  The residual of the skip
// connection is either a block of ready codes or, likewise, the block input
// quantised on load.  Workgroup 0 stores the scales for later kernels.
// All global reads of this kernel are raw buffer loads: a request that must not
// happen (a pixel outside the tensor, a channel beyond c, a candidate beyond n) is
// given an offset outside the buffer and returns zero, so no load sits under a
// branch.  (A load under a branch is awaited where the branch ends: one memory
// round trip per load instead of one for all of them.)  Extents are below 2^31.
constexpr uint32_t kNoLoad = 0x80000000u;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const void *p, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)p, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float buffer_f32(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
}
template <bool BF16>
__device__ __forceinline__ float buffer_elem(__amdgpu_buffer_rsrc_t r, uint32_t index, bool ok)
{
    if (BF16) return __uint_as_float((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)(ok ? index * 2 : kNoLoad), 0, 0) << 16);
    return buffer_f32(r, ok ? index * 4 : kNoLoad);
}
// channels [4 gq, 4 gq + 4) of pixel pi of a [n, c, hw] tensor (zeros beyond c and where !ok)
template <bool BF16>
__device__ __forceinline__ float4 plane_values(__amdgpu_buffer_rsrc_t r, int c, uint32_t hw, uint32_t pi, int gq, bool ok)
{
    const uint32_t img = pi / hw, pp = pi - img * hw;                // pixel counts fit 31 bits here: 32-bit division
    const uint32_t base = (img * c + gq * 4) * hw + pp;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = buffer_elem<BF16>(r, base + e * hw, ok && gq * 4 + e < c);
    return make_float4(v[0], v[1], v[2], v[3]);
}
// item idx of the operand stage: four channels of one of the npix staged pixels.
// Rows of c floats: four consecutive threads share a pixel; channel planes:
// consecutive threads take consecutive pixels of one channel group.
template <int A_SRC>
__device__ __forceinline__ void operand_item(int idx, int npix, int &j, int &gq)
{
    if (A_SRC == 1) { j = idx >> 2; gq = idx & 3; }
    else { gq = idx / npix; j = idx - gq * npix; }
}
template <int A_SRC, bool BF16, bool C16>
__device__ __forceinline__ float4 load_operand_item(__amdgpu_buffer_rsrc_t r, int c, int M, uint32_t hw, int first_pix, int npix, int idx)
{
    int j, gq;
    operand_item<A_SRC>(idx, npix, j, gq);
    const int pi = first_pix + j;
    const bool ok = idx < npix * 4 && pi >= 0 && pi < M;
    if (A_SRC == 1) {
        const uint32_t row = (uint32_t)pi * (uint32_t)c;
        if (C16) {
            const v4u q = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(ok ? (row + gq * 4) * 4 : kNoLoad), 0, 0);
            return make_float4(__uint_as_float(q[0]), __uint_as_float(q[1]), __uint_as_float(q[2]), __uint_as_float(q[3]));
        }
        float t[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] = buffer_f32(r, (ok && gq * 4 + e < c) ? (row + gq * 4 + e) * 4 : kNoLoad);
        return make_float4(t[0], t[1], t[2], t[3]);
    }
    return plane_values<BF16>(r, c, hw, (uint32_t)pi, gq, ok);
}
// the lane's share of n candidate maxima, `stride` words apart (n <= 512)
__device__ __forceinline__ uint32_t buffer_candidates(const uint32_t *slot, int n, int stride)
{
    const __amdgpu_buffer_rsrc_t r = raw_buffer(slot, n > 0 ? ((int64_t)(n - 1) * stride + 1) * 4 : 0);
    const int lane = threadIdx.x & 63;
    uint32_t v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int i = lane + 64 * k;
        v[k] = __builtin_amdgcn_raw_buffer_load_b32(r, (int)(i < n ? (uint32_t)(i * stride) * 4 : kNoLoad), 0, 0);
    }
    uint32_t bits = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) bits = v[k] > bits ? v[k] : bits;
    return bits;
}
__device__ __forceinline__ uint32_t pack_codes(float4 v, float inv)
{
    return quant1(v.x, inv) | quant1(v.y, inv) << 8 | quant1(v.z, inv) << 16 | quant1(v.w, inv) << 24;
}

// XBF16: the channel planes read (operand of a_src 2, residual of res_src 1) hold bf16; C16 (a_src 1): rows of 16 floats
template <int A_SRC, bool XBF16, bool C16>
__global__ __launch_bounds__(256) void conv3x3_c16_fused_kernel(const GemmArgs g, const ConvFuse z)
{
    // [128][16] residual codes, bias [32], weight scale [32], [128 + 2 (W + 1)][16] operand codes
    extern __shared__ __attribute__((aligned(16))) uint8_t sdyn[];
    uint8_t *sres = sdyn, *sa = sdyn + 128 * 16 + 256;
    float *sbias = (float *)(sdyn + 128 * 16), *ssw = sbias + 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.x * 128, M = (int)g.M;
    const uint32_t hw = (uint32_t)g.H * (uint32_t)g.W;
    const int halo = g.W + 1, npix = 128 + 2 * halo;
    const int xes = XBF16 ? 2 : 4;

    // ---- every request the workgroup depends on goes out before anything is awaited:
    // the first 1024 items of the operand stage (all of it up to 62 pixels of width), the
    // residual, the weights and the candidate maxima
    const __amdgpu_buffer_rsrc_t ra = raw_buffer(z.a_f, A_SRC == 0 ? 0 : (int64_t)M * z.c * (A_SRC == 1 ? 4 : xes));
    constexpr int NB = 4;
    float4 raw[NB];
    if (A_SRC != 0) {
#pragma unroll
        for (int b = 0; b < NB; ++b) raw[b] = load_operand_item<A_SRC, XBF16, C16>(ra, z.c, M, hw, m0 - halo, npix, threadIdx.x + 256 * b);
    }
    // both forms of the residual are requested; the one that is not in use has an empty buffer
    const bool res_planes = z.res_src == 1, res_codes = !res_planes && g.res_q != nullptr;
    const __amdgpu_buffer_rsrc_t rrp = raw_buffer(z.res_f, res_planes ? (int64_t)M * z.res_c * xes : 0);
    const __amdgpu_buffer_rsrc_t rrq = raw_buffer(g.res_q, res_codes ? (int64_t)M * 16 : 0);
    float4 rraw[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int idx = threadIdx.x + 256 * b, gq = idx >> 7, j = idx & 127;
        rraw[b] = plane_values<XBF16>(rrp, z.res_c, hw, (uint32_t)(m0 + j), gq, res_planes && m0 + j < M);
    }
    const int rpi = m0 + (int)(threadIdx.x & 127);
    const v4i rv = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rrq, (int)((res_codes && rpi < M) ? (uint32_t)rpi * 16 : kNoLoad), 0, 0));
    const __amdgpu_buffer_rsrc_t rw = raw_buffer(g.w, g.w_bytes);
    v4i fb[5];
#pragma unroll
    for (int st = 0; st < 5; ++st) {
        const int tap = 2 * st + h;
        fb[st] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(
                                             rw, (int)((p < g.N && tap < 9) ? (uint32_t)(p * g.kp + tap * 16) : kNoLoad), 0, 0));
    }
    // bias and weight scale of output channel t, for threads t < 32 (zero beyond N)
    const __amdgpu_buffer_rsrc_t rb = raw_buffer(g.bias, g.bias ? (int64_t)g.N * 4 : 0);
    const __amdgpu_buffer_rsrc_t rs_w = raw_buffer(g.sw, g.sw_per_n ? (int64_t)g.N * 4 : 4);
    const uint32_t ct = threadIdx.x & 31;
    const float bias_t = buffer_f32(rb, ct * 4), sw_t = buffer_f32(rs_w, g.sw_per_n ? ct * 4 : 0u);
    uint32_t cand_a = 0, cand_r = 0;
    if (A_SRC != 0) cand_a = buffer_candidates(z.a_slot, z.a_nslot, z.a_stride);
    cand_r = buffer_candidates(z.res_slot, res_planes ? z.res_nslot : 0, z.res_stride);

    float scale_a;
    if (A_SRC != 0) {
        bool bad;
        const float inv = scale_from_bits(wave_max_u32(cand_a), z.a_fixed, &scale_a, &bad);
        if (blockIdx.x == 0 && threadIdx.x == 0) publish(scale_a, bad, z.a_scale_out, nullptr, z.flag);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int idx = threadIdx.x + 256 * b;
            int j, gq;
            operand_item<A_SRC>(idx, npix, j, gq);
            if (idx < npix * 4) *(uint32_t *)&sa[j * 16 + gq * 4] = pack_codes(raw[b], inv);
        }
        for (int idx = threadIdx.x + 256 * NB; idx < npix * 4; idx += 256) {       // wide images
            int j, gq;
            operand_item<A_SRC>(idx, npix, j, gq);
            *(uint32_t *)&sa[j * 16 + gq * 4] = pack_codes(load_operand_item<A_SRC, XBF16, C16>(ra, z.c, M, hw, m0 - halo, npix, idx), inv);
        }
    } else {
        scale_a = *g.sx;
    }
    if (threadIdx.x < 32) {
        sbias[threadIdx.x] = bias_t;
        ssw[threadIdx.x] = (int)threadIdx.x < g.N ? sw_t : 0.0f;
    }
    float rs = 0.0f;
    const bool has_res = z.res_src == 1 || g.res_q != nullptr;
    if (z.res_src == 1) {
        bool bad;
        const float inv = scale_from_bits(wave_max_u32(cand_r), z.res_fixed, &rs, &bad);
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int idx = threadIdx.x + 256 * b, gq = idx >> 7, j = idx & 127;
            *(uint32_t *)&sres[j * 16 + gq * 4] = pack_codes(rraw[b], inv);
        }
    } else if (g.res_q) {
        rs = *g.res_scale;
        if (threadIdx.x < 128) *(v4i *)&sres[threadIdx.x * 16] = rv;
    }
    __syncthreads();

    const int lp = wave * 32 + p;                                    // the lane's output pixel within the workgroup
    const int m = m0 + lp;
    const bool m_ok = m < M;
    const uint32_t mrow = (uint32_t)m / (uint32_t)g.W;
    const int ow = (int)((uint32_t)m - mrow * (uint32_t)g.W), oh = (int)(mrow % (uint32_t)g.H);
    v4i fa[5];
#pragma unroll
    for (int st = 0; st < 5; ++st) {
        const int tap = 2 * st + h;
        const int kh = tap / 3, dh = kh - 1, dw = tap - kh * 3 - 1;
        const bool ok = m_ok && tap < 9 && (unsigned)(oh + dh) < (unsigned)g.H && (unsigned)(ow + dw) < (unsigned)g.W;
        if (A_SRC != 0) fa[st] = ok ? *(const v4i *)&sa[(lp + halo + dh * g.W + dw) * 16] : v4i{0, 0, 0, 0};
        else fa[st] = ok ? *(const v4i *)(g.a + ((int64_t)m + dh * g.W + dw) * 16) : v4i{0, 0, 0, 0};
    }
    // Weights are the row operand and pixels the column operand, so a lane ends up with 16 output
    // channels of ONE pixel: channels 8 (r / 4) + 4 h + r % 4 in register r, i.e. four groups of four
    // consecutive channels, which go out as 16-byte stores.
    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
#pragma unroll
    for (int st = 0; st < 5; ++st) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[st], fa[st], acc, 0, 0, 0);

    const float q_inv = g.q_out ? (float)(1.0 / (double)*g.q_scale) : 0.0f;
    const int n_out = g.q_out && g.q_ld > g.N ? (int)g.q_ld : g.N;               // channels that receive anything
    const bool vec = g.y && (g.N & 3) == 0 && (g.ldy & 3) == 0 && ((uintptr_t)g.y & 15) == 0;
    uint32_t amax = 0;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
        const int ch0 = 8 * gi + 4 * h;
        if (8 * gi >= n_out) break;                                               // uniform
        if (!m_ok || ch0 >= n_out) continue;
        const float4 b4 = *(const float4 *)&sbias[ch0], w4 = *(const float4 *)&ssw[ch0];
        const float bb[4] = {b4.x, b4.y, b4.z, b4.w}, ww[4] = {w4.x, w4.y, w4.z, w4.w};
        const uint32_t rc = has_res ? *(const uint32_t *)&sres[lp * 16 + (ch0 & 15)] : 0u;
        float v[4];
        uint32_t codes = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float t = fmaf((float)acc[4 * gi + e], scale_a * ww[e], bb[e]);
            if (has_res) t = t + (float)(int8_t)(rc >> (8 * e)) * rs;
            if (g.act == 1) t = t > 0.0f ? t : 0.0f;
            const bool ch_ok = ch0 + e < g.N;
            if (g.absmax_out) {
                const uint32_t ab = g.amax_pos ? (t > 0.0f ? __float_as_uint(t) : 0u) : abs_bits(t);
                amax = (ch_ok && ab > amax) ? ab : amax;
            }
            if (g.q_out) codes |= (ch_ok ? quant1(t, q_inv) : 0u) << (8 * e);     // pad columns of the int8 output are zero
            v[e] = t;
        }
        if (g.y) {
            float *dst = g.y + (int64_t)m * g.ldy + ch0;
            if (vec) {
                *(float4 *)dst = make_float4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (ch0 + e < g.N) dst[e] = v[e];
            }
        }
        if (g.q_out && ch0 < g.q_ld) *(uint32_t *)(g.q_out + (int64_t)m * g.q_ld + ch0) = codes;
    }
    if (g.absmax_out) {
        __shared__ uint32_t sm4[4];
        block_atomic_max(amax, g.absmax_out, sm4);
    }
}

hipError_t launch_conv3x3_c16_fused(const GemmArgs &g, const ConvFuse &z, hipStream_t st)
{
    // what the kernel assumes: 16-byte pixels, a residual of 16 codes per pixel at most, no raw-accumulator
    // output, a halo that fits the LDS stage
    if (!g.conv3x3 || g.cp != 16 || g.N < 1 || g.N > 32 || g.kp != 9 * 16 || g.et != 0 || g.acc_out) return hipErrorInvalidValue;
    if (g.W < 1 || g.H < 1 || g.W > kConvFuseMaxWidth || g.M % ((int64_t)g.H * g.W) != 0) return hipErrorInvalidValue;
    if (g.M > 0x7fffffffLL - 2 * (kConvFuseMaxWidth + 1) - 128) return hipErrorInvalidValue;    // 32-bit pixel arithmetic
    if (z.a_src < 0 || z.a_src > 2 || (z.a_src != 0 && (!z.a_f || z.c < 1 || z.c > 16))) return hipErrorInvalidValue;
    if (z.a_src == 0 && (!g.a || !g.sx)) return hipErrorInvalidValue;
    if (z.res_src == 1 && (!z.res_f || z.res_c < 1 || z.res_c > 16 || g.N > 16)) return hipErrorInvalidValue;
    if (z.res_src == 0 && g.res_q && (g.res_ld != 16 || g.N > 16)) return hipErrorInvalidValue;
    const int64_t blocks = (g.M + 127) / 128;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t smem = 128 * 16 + 256 + (z.a_src != 0 ? (size_t)(128 + 2 * (g.W + 1)) * 16 : 0);
    const dim3 grid((unsigned)blocks), block(256);
    // what the kernel's 32-bit offsets assume
    if (g.M * 16 * 4 >= (1LL << 31) || g.w_bytes >= (1LL << 31) || z.a_nslot > 512 || z.res_nslot > 512) return hipErrorInvalidValue;
    // XBF16: element type of the planes read (the block input: operand of a_src 2, residual of res_src 1)
    const bool xbf16 = z.a_src == 2 ? z.a_bf16 != 0 : (z.res_src == 1 && z.res_bf16 != 0);
    if (z.a_src == 2 && z.res_src == 1 && (z.a_bf16 != 0) != (z.res_bf16 != 0)) return hipErrorInvalidValue;
#define EG_FUSED(A, B, C) launch_k(EGERIA_KERNEL_GEMM, conv3x3_c16_fused_kernel<A, B, C>, grid, block, smem, st, g, z)
    if (z.a_src == 0) return xbf16 ? EG_FUSED(0, true, false) : EG_FUSED(0, false, false);
    if (z.a_src == 1) {
        if (z.c == 16) return xbf16 ? EG_FUSED(1, true, true) : EG_FUSED(1, false, true);
        return xbf16 ? EG_FUSED(1, true, false) : EG_FUSED(1, false, false);
    }
    return xbf16 ? EG_FUSED(2, true, false) : EG_FUSED(2, false, false);
#undef EG_FUSED
}

// The tile shapes on offer: rows x columns of the output tile, K bytes per
// step, workgroups of that shape that fit a CU together (registers and LDS),
// and the relative cost of a unit of tile area (smaller tiles move more LDS
// and L1 bytes per MFMA).
struct TileShape {
    int bm, bn, bk, resident, waves;
    double penalty;
};
constexpr int kNumShapes = 11;
static const TileShape kShapes[kNumShapes] = {
    {256, 256, 64, 1, 4, 1.00},  {256, 192, 128, 1, 4, 1.03}, {256, 128, 64, 2, 4, 1.06}, {128, 192, 64, 2, 4, 1.10},
    {128, 128, 64, 3, 4, 1.20},  {128, 128, 128, 2, 4, 1.22}, {128, 64, 64, 4, 4, 1.40},  {128, 64, 128, 3, 4, 1.38},
    {256, 128, 128, 1, 4, 1.05}, {256, 256, 128, 1, 8, 1.00}, {256, 192, 128, 1, 8, 1.02},
};

static hipError_t launch_shape(int i, const GemmArgs &g, hipStream_t st)
{
    switch (i) {
    case 0: return launch_variant<256, 256, 2, 2, 64>(g, st);
    case 1: return launch_variant<256, 192, 2, 2, 128>(g, st);
    case 2: return launch_variant<256, 128, 2, 2, 64>(g, st);
    case 3: return launch_variant<128, 192, 2, 2, 64>(g, st);
    case 4: return launch_variant<128, 128, 2, 2, 64>(g, st);
    case 5: return launch_variant<128, 128, 2, 2, 128>(g, st);
    case 6: return launch_variant<128, 64, 2, 2, 64>(g, st);
    case 7: return launch_variant<128, 64, 2, 2, 128>(g, st);
    case 8: return launch_variant<256, 128, 2, 2, 128>(g, st);
    case 9: return launch_variant<256, 256, 2, 4, 128>(g, st);
    case 10: return launch_variant<256, 192, 4, 2, 128>(g, st);
    default: return hipErrorInvalidValue;
    }
}

// Tile choice.  A tile shape is priced by the work the chip does for it,
// padding included: workgroups run in rounds of (compute units) x (workgroups resident
// per CU), a partly filled last round costs as much as a full one, and the
// smaller shapes pay more LDS and L1 traffic per MFMA.  With fp32 outputs the
// epilogue (convert, scale, store) costs as much as the K loop unless K is
// long, so for short K only shapes with two workgroups per CU are considered
// (one is in its K loop while the other stores), and for very short K, where
// the kernel is a stream of stores, only the small shapes.
// The float16 / float32 reference precisions: three tile shapes, chosen by how
// many tiles the output makes.
template <int ET>
static hipError_t launch_float(const GemmArgs &g, hipStream_t st)
{
    if (g.q_out || g.absmax_out) return hipErrorInvalidValue;
    if (g.N <= 32) return launch_variant<128, 32, 4, 1, 64, ET>(g, st);
    const int64_t t128 = ((g.M + 127) / 128) * (int64_t)((g.N + 127) / 128);
    if (t128 >= 512) return launch_variant<128, 128, 2, 2, 64, ET>(g, st);
    return launch_variant<128, 64, 2, 2, 64, ET>(g, st);
}

bool gemm_layernorm_fusable(int32_t N, const void *ln_out, const void *ln_res, const void *gamma, const void *beta)
{
    auto ok16 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    return N >= 4 && N <= 768 && (N & 3) == 0 && ln_out && ln_res && ok16(ln_out) && ok16(ln_res) && ok16(gamma) && ok16(beta);
}

hipError_t launch_gemm_i8(const GemmArgs &g, hipStream_t st)
{
    if (g.ln_out) {
        // a linear layer and the layer norm of its rows in one launch: 64 whole rows per workgroup
        if (g.et != 0 || g.conv3x3 || g.act || g.res_q || g.q_out || g.acc_out || g.zp_in || g.zp_res) return hipErrorInvalidValue;
        if (!gemm_layernorm_fusable(g.N, g.ln_out, g.ln_res, g.ln_gamma, g.ln_beta)) return hipErrorInvalidValue;
        return launch_variant<64, 768, 1, 8, 64, 0, true>(g, st);
    }
    if (g.et == 1) return launch_float<1>(g, st);
    if (g.et == 2) return launch_float<2>(g, st);
    if (g.et != 0) return hipErrorInvalidValue;
    if (g.conv3x3 && g.cp == 16 && g.N <= 32 && !g.zp_in) {   // (symmetric codes only)
        const int64_t blocks = (g.M + 127) / 128;
        if (blocks <= 0) return hipSuccess;
        if (g.M >= (1LL << 31)) return hipErrorInvalidValue;            // 32-bit pixel arithmetic in the kernel
        return launch_k(EGERIA_KERNEL_GEMM, conv3x3_c16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, g);
    }
    if (g.N <= 32) return launch_variant<128, 32, 4, 1, 64>(g, st);
    int best = 0;
    double best_cost = 0.0;
    for (int i = 0; i < kNumShapes; ++i) {
        const TileShape &sh = kShapes[i];
        const int64_t tiles = ((g.M + sh.bm - 1) / sh.bm) * (int64_t)((g.N + sh.bn - 1) / sh.bn);
        if (sh.waves == 8) {
            // eight waves on one large tile with whole-line K steps: linear layers with a long K that fill every
            // compute unit.  (With K = 768 they win by 5-10 % when timed alone, where the fp32 output stays in the
            // last-level cache, and lose as much inside an encoder layer, where it goes to HBM and the shapes
            // with two workgroups per compute unit hide more of the store behind the other workgroup's K loop.)
            if (g.conv3x3 || g.kp < 2048 || tiles < compute_units()) continue;
        } else if (sh.resident == 1 && g.kp < 2048) {
            continue;
        }
        if (sh.bm * sh.bn > 128 * 128 && g.kp < 512) continue;     // store bound: many small workgroups in flight
        const int64_t slots = compute_units() * (int64_t)sh.resident;
        const int64_t rounds = (tiles + slots - 1) / slots;
        double cost = (double)rounds * sh.resident * sh.bm * sh.bn * sh.penalty;
        // K of a few steps: the kernel is a stream of fp32 stores, and the more workgroups a CU holds the
        // better they overlap (12544 x 1024 x 256: 128x64 with four per CU 17 us, 128x128 with two 21 us)
        if (g.kp < 512) cost *= 1.0 + 0.15 * (4 - sh.resident);
        if (best_cost == 0.0 || cost < best_cost) {
            best_cost = cost;
            best = i;
        }
    }
    return launch_shape(best, g, st);
}

}  // namespace egeria
