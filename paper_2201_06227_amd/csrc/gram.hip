// Training plasticity P = SP_loss(A_T, A_R) (Section 4.2, Eq. 1 of the paper;
// the loss is the cited similarity-preserving loss):
//   Gt = Q Q^T (b x b) for Q = A_T and Q = A_R reshaped to [b, D],
//   rows of Gt divided by their L2 norm, P = ||G_T - G_R||_F^2 / b^2.
//
// P is a squared *difference* of two nearly equal matrices, so forming both
// Gram matrices in fp32 and subtracting loses most of the digits once the
// layer has converged.  The kernels therefore contract
//   M = (T - R)(T + R)^T     and     B = R R^T
// (T, R the two activations): the Gram difference is exactly (M + M^T)/2, it is
// obtained to fp32 *relative* accuracy, and G_T's Gram is recovered as
// B + (M + M^T)/2 in fp64 in the finaliser.  Same bytes and the same number of
// matrix-core operations as two plain Gram products.
//
// Kernel 1 (gram_partial): split-K over D.  A workgroup owns one chunk of D and
//   one macro tile of both products: 64x64 (four 32x32 blocks, one per wave) for
//   b > 32, or the single 32x32 block for b <= 32 with the four waves splitting
//   each K tile.  Every fp32 product of the two contractions is formed exactly
//   on the bf16 matrix cores: an fp32 value is the sum of three bf16 values
//   (8 + 8 + 8 significant bits, obtained by truncation and exact subtraction),
//   so x * y = sum of nine bf16 x bf16 products, each exact in fp32; the six
//   largest are issued (v_mfma_f32_32x32x16_bf16, fp32 accumulation), the three
//   dropped ones sum to less than 2^-21 of the product.  Six bf16 MFMAs cost 0.375 of the
//   eight fp32 MFMAs they replace.  Sample rows are fetched with coalesced loads
//   one K tile ahead into registers, split once per element, and written to LDS
//   as bf16 planes (hi / mid / lo of T-R, T+R and R) in 16-byte units whose
//   position is xor-rotated by the row so that writes and the 128-bit operand
//   reads are bank-conflict free.  Lane l supplies row l % 32 and the 8 values of
//   unit l / 32 of a 16-deep slab, A and B operand alike, so the order of k
//   inside the sum never matters.
//   Each workgroup stores its M block twice, as is and transposed, so that
//   the next kernel reads rows only.
// Kernel 2 (sp_finalize): one workgroup per row i of the b x b matrices.  It
//   sums row i of M, M^T and B over the chunks in fp64 (fixed assignment of
//   chunks to thread groups, fixed order), forms row i of both Gram matrices,
//   their norms and the row's share of the squared difference; the last
//   workgroup to finish adds the b shares in index order and writes P.
//   Results are bit-reproducible from call to call.
#include "common.hpp"
#include <mutex>

namespace egeria {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct GramPlan {
    int mt;          // blocks of 32 per macro-tile side: 1 (b <= 32) or 2
    int nm;          // macro tiles per side
    int nmacro;      // nm * nm
    int kt;          // features per K tile: 64 (mt = 1) or 32 (mt = 2)
    int nsplit;      // chunks of D
    int nsplit_pad;  // rounded up to a multiple of 8 (chunks are dealt to XCDs)
    int64_t kc;      // chunk length, multiple of kt
};

static GramPlan plan_gram(int32_t b, int64_t D)
{
    GramPlan p;
    p.mt = b <= 32 ? 1 : 2;
    p.nm = p.mt == 1 ? 1 : (b + 63) / 64;
    p.nmacro = p.nm * p.nm;
    p.kt = p.mt == 1 ? 64 : 32;
    // about one workgroup per CU: measured per score (partials + finaliser, us) for targets of 128 / 256 /
    // 512 / 1024 workgroups: b = 32, D = 98304: 19.6 / 17.6 / 20.6 / 24.6; b = 64, D = 200704: 57.7 / 43.5 /
    // 43.8 / 55.9 (more chunks mean more partials for the finaliser to add)
    int64_t want = (compute_units() + p.nmacro - 1) / p.nmacro;
    int64_t cap = D / ((p.mt == 1 ? 4 : 2) * (int64_t)b);  // bound the partials by a fraction of the input bytes
    if (cap < 1) cap = 1;
    if (want > cap) want = cap;
    int64_t kc = (D + want - 1) / want;
    kc = (kc + p.kt - 1) / p.kt * p.kt;
    p.kc = kc;
    p.nsplit = (int)((D + kc - 1) / kc);
    p.nsplit_pad = (p.nsplit + 7) / 8 * 8;
    return p;
}

// workspace of the metric: [counter | row shares (b doubles) | partials [nsplit][3][b][b] (M, M^T, B)]
static size_t off_rowsum() { return 256; }
static size_t off_partials(int32_t b) { return 256 + align_up((size_t)b * sizeof(double), 256); }

size_t plasticity_partial_bytes(int32_t b, int64_t D)
{
    GramPlan p = plan_gram(b, D);
    return off_partials(b) + align_up((size_t)p.nsplit * 3 * (size_t)b * b * sizeof(float), 256);
}

// ---- four consecutive features of one sample row, as fp32 -------------------------------
// FAST: rows are 16-byte aligned and every K tile is whole, so the load is
// unconditional (the caller clamps row and tile to valid ones; what a clamped
// load returns only reaches outputs that are never stored).  Unconditional
// loads also let the compiler count outstanding requests exactly, which the
// two-tile-deep prefetch depends on.  Otherwise: zeros for a row beyond b or
// features beyond the chunk's end, scalar loads.
template <int DT, bool FAST>
__device__ __forceinline__ float4 load4(const void *__restrict__ base, int64_t row, bool row_ok,
                                        int64_t D, int64_t k, int64_t kend)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (FAST) {
        if (DT == 0) {
            v = *(const float4 *)((const float *)base + row * D + k);
        } else {
            const uint2 q = *(const uint2 *)((const uint16_t *)base + row * D + k);
            v.x = __uint_as_float(q.x << 16);
            v.y = __uint_as_float(q.x & 0xffff0000u);
            v.z = __uint_as_float(q.y << 16);
            v.w = __uint_as_float(q.y & 0xffff0000u);
        }
        return v;
    }
    if (!row_ok || k >= kend) return v;
    float e[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (k + i < kend)
            e[i] = DT == 0 ? ((const float *)base)[row * D + k + i]
                           : bf16_to_f32(((const uint16_t *)base)[row * D + k + i]);
    return make_float4(e[0], e[1], e[2], e[3]);
}

// The three bf16 parts of eight fp32 values, packed as the 16-byte operand unit
// of the bf16 MFMA.  hi = the value truncated to bf16, mid = the remainder
// truncated, lo = what is left; both subtractions are exact and lo has at most
// eight significant bits, so hi + mid + lo == x exactly.
struct Split8 {
    v4u h, m, l;
};
__device__ __forceinline__ uint32_t pack_hi16(float x1, float x0)
{
    return __builtin_amdgcn_perm(__float_as_uint(x1), __float_as_uint(x0), 0x07060302u);
}
__device__ __forceinline__ Split8 split8(const float (&x)[8])
{
    Split8 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float x0 = x[2 * e], x1 = x[2 * e + 1];
        const float r0 = x0 - __uint_as_float(__float_as_uint(x0) & 0xffff0000u);
        const float r1 = x1 - __uint_as_float(__float_as_uint(x1) & 0xffff0000u);
        const float l0 = r0 - __uint_as_float(__float_as_uint(r0) & 0xffff0000u);
        const float l1 = r1 - __uint_as_float(__float_as_uint(r1) & 0xffff0000u);
        o.h[e] = pack_hi16(x1, x0);
        o.m[e] = pack_hi16(r1, r0);
        o.l[e] = pack_hi16(l1, l0);
    }
    return o;
}

template <int MT, bool OFFD, int TDT, int RDT, bool FAST>
__global__ __launch_bounds__(256) void gram_partial_kernel(const void *__restrict__ at,
                                                           const void *__restrict__ ar, int b,
                                                           int64_t D, GramPlan p,
                                                           float *__restrict__ part,
                                                           uint32_t *__restrict__ counter)
{
    constexpr int ROWS = MT * 32;                 // rows per side of the macro tile
    constexpr int KT = MT == 1 ? 64 : 32;         // features per K tile
    constexpr int UPR = KT / 8;                   // 16-byte units (8 bf16) per row of a plane
    constexpr int SWR = 16 / UPR;                 // rows that share a rotation of the units
    constexpr int PLANE = ROWS * KT * 2;          // bytes of one bf16 plane
    constexpr int STAGE = (OFFD ? 12 : 9) * PLANE;
    static_assert(MT == 2 || !OFFD, "a macro tile of one block has no off-diagonal neighbours");
    static_assert(ROWS * UPR == 256, "one unit per thread and plane");
    // planes: 0-2 hi/mid/lo of T-R (rows i), 3-5 of R (rows i), 6-8 of T+R (rows j),
    // 9-11 of R (rows j; off-diagonal macro tiles only, else planes 3-5 serve)
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];     // [2 stages][planes][ROWS][KT] bf16

    // consecutive workgroup ids land on different XCDs: all macro tiles of one
    // chunk go to the same XCD so that its L2 serves the re-reads of that chunk
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int chunk = (slot / p.nmacro) * 8 + xcd;
    const int mtile = slot % p.nmacro;
    if (chunk >= p.nsplit) return;
    const int mi = mtile / p.nm, mj = mtile % p.nm;
    const bool diag = !OFFD || mi == mj;
    const int64_t k0 = (int64_t)chunk * p.kc;
    const int64_t k1 = k0 + p.kc < D ? k0 + p.kc : D;
    const int ntiles = (int)((k1 - k0 + KT - 1) / KT);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;

    // Staging: thread tid owns unit tid % UPR of row tid / UPR.  Its eight values
    // are features 4u .. 4u+3 and KT/2 + 4u .. KT/2 + 4u+3 of the tile (two 16-byte
    // loads, each contiguous over the threads of a row); which features share a
    // unit is free as long as every plane uses the same assignment.
    const int srow = tid / UPR, su = tid % UPR;
    int64_t row_i = (int64_t)mi * ROWS + srow, row_j = (int64_t)mj * ROWS + srow;
    const bool ok_i = row_i < b, ok_j = row_j < b;
    row_i = ok_i ? row_i : 0;                     // rows beyond b: a valid address for the unconditional loads
    row_j = ok_j ? row_j : 0;
    const uint32_t soff = (uint32_t)(srow * (UPR * 16) + ((su ^ ((srow / SWR) % UPR)) * 16));
    struct Staged {
        float4 t[2], r[2], tj[2], rj[2];
    };
    auto fetch = [&](int t, Staged &s) {
        // past the chunk's end: the last tile again (FAST; such a tile is never contracted) or zeros
        const int tt = FAST ? (t < ntiles ? t : ntiles - 1) : t;
        const int64_t kb = k0 + (int64_t)tt * KT + 4 * su;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int64_t k = kb + q * (KT / 2);
            s.t[q] = load4<TDT, FAST>(at, row_i, ok_i, D, k, k1);
            s.r[q] = load4<RDT, FAST>(ar, row_i, ok_i, D, k, k1);
            if (OFFD && !diag) {
                s.tj[q] = load4<TDT, FAST>(at, row_j, ok_j, D, k, k1);
                s.rj[q] = load4<RDT, FAST>(ar, row_j, ok_j, D, k, k1);
            }
        }
    };
    auto put = [&](int stage, int plane, const float (&x)[8]) {
        const Split8 sp = split8(x);
        uint8_t *base = lds + stage * STAGE + plane * PLANE + soff;
        *(v4u *)(base) = sp.h;
        *(v4u *)(base + PLANE) = sp.m;
        *(v4u *)(base + 2 * PLANE) = sp.l;
    };
    auto stash = [&](int stage, const Staged &s) {
        const float t8[8] = {s.t[0].x, s.t[0].y, s.t[0].z, s.t[0].w, s.t[1].x, s.t[1].y, s.t[1].z, s.t[1].w};
        const float r8[8] = {s.r[0].x, s.r[0].y, s.r[0].z, s.r[0].w, s.r[1].x, s.r[1].y, s.r[1].z, s.r[1].w};
        float d8[8], s8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) d8[e] = t8[e] - r8[e];
        put(stage, 0, d8);
        put(stage, 3, r8);
        if (OFFD && !diag) {
            const float tj8[8] = {s.tj[0].x, s.tj[0].y, s.tj[0].z, s.tj[0].w, s.tj[1].x, s.tj[1].y, s.tj[1].z, s.tj[1].w};
            const float rj8[8] = {s.rj[0].x, s.rj[0].y, s.rj[0].z, s.rj[0].w, s.rj[1].x, s.rj[1].y, s.rj[1].z, s.rj[1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) s8[e] = tj8[e] + rj8[e];
            put(stage, 6, s8);
            put(stage, 9, rj8);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) s8[e] = t8[e] + r8[e];
            put(stage, 6, s8);
        }
    };

    v16f accM, accB;
#pragma unroll
    for (int i = 0; i < 16; ++i) { accM[i] = 0.0f; accB[i] = 0.0f; }

    // operand rows of this wave inside the macro tile
    const int bi = MT == 1 ? 0 : (wave >> 1), bj = MT == 1 ? 0 : (wave & 1);
    const int rowA = bi * 32 + r, rowB = bj * 32 + r;
    const uint32_t offA = (uint32_t)(rowA * (UPR * 16)), swA = (uint32_t)((rowA / SWR) % UPR);
    const uint32_t offB = (uint32_t)(rowB * (UPR * 16)), swB = (uint32_t)((rowB / SWR) % UPR);
    const int planeRj = diag ? 3 : 9;

    // One 16-deep slab: unit 2 * slab + h of the operand rows, six partial
    // products per fp32 product, smallest first.
    auto slab = [&](int stage, int sl) {
        const uint32_t u = (uint32_t)(2 * sl + h);
        const uint8_t *pa = lds + stage * STAGE + offA + ((u ^ swA) * 16);
        const uint8_t *pb = lds + stage * STAGE + offB + ((u ^ swB) * 16);
        v8bf dA[3], rA[3], sB[3], rB[3];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            dA[c] = __builtin_bit_cast(v8bf, *(const v4u *)(pa + (0 + c) * PLANE));
            rA[c] = __builtin_bit_cast(v8bf, *(const v4u *)(pa + (3 + c) * PLANE));
            sB[c] = __builtin_bit_cast(v8bf, *(const v4u *)(pb + (6 + c) * PLANE));
            rB[c] = __builtin_bit_cast(v8bf, *(const v4u *)(pb + (planeRj + c) * PLANE));
        }
        constexpr int ia[6] = {2, 0, 1, 1, 0, 0}, ib[6] = {0, 2, 1, 0, 1, 0};   // (lo,hi) (hi,lo) (mid,mid) (mid,hi) (hi,mid) (hi,hi)
#pragma unroll
        for (int q = 0; q < 6; ++q) {
            accM = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dA[ia[q]], sB[ib[q]], accM, 0, 0, 0);
            accB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rA[ia[q]], rB[ib[q]], accB, 0, 0, 0);
        }
    };

    // Software pipeline: during step t the matrix cores contract tile t from LDS
    // stage t & 1 while tile t + 1, already in registers, is split into the other
    // stage; tile t + 2 is in flight (requested one step ago) and tile t + 3 is
    // requested into the registers that tile t + 1 has just left.  One barrier
    // per tile.
    auto contract = [&](int stage) {
        if (MT == 1) {
            slab(stage, wave);
        } else {
            slab(stage, 0);
            slab(stage, 1);
        }
    };
    Staged st0, st1;
    fetch(0, st0);
    fetch(1, st1);
    stash(0, st0);
    fetch(2, st0);
    __syncthreads();
    auto step = [&](int t, Staged &next) {
        contract(t & 1);
        stash((t + 1) & 1, next);
        fetch(t + 3, next);
        // issue order: the splitting arithmetic of the next tile and its LDS writes between the
        // MFMAs of this one (an MFMA occupies the matrix pipe for 8 passes, the vector ALU is free
        // meanwhile; the nine 16-byte LDS writes, spread out, do not queue up at the tile's end)
        constexpr int NMF = MT == 1 ? 12 : 24;
#pragma unroll
        for (int i = 0; i < NMF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, MT == 1 ? 12 : 6, 0);     // vector ALU
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                    // one LDS write
        }
        __syncthreads();
    };
    for (int t = 0; t < ntiles; t += 2) {
        step(t, st1);
        if (t + 1 < ntiles) step(t + 1, st0);
    }

    // lane l of a 32x32 block holds column l % 32, rows 8 * (i / 4) + 4 * (l / 32) + i % 4
    const size_t nelem = (size_t)b * b;
    float *dst = part + (size_t)chunk * 3 * nelem;               // M | M^T | B of this chunk
    if (id == 0 && tid == 0) *counter = 0u;                       // ticket of the finaliser
    if (MT == 1) {
        // the four waves hold partial sums over disjoint k: add them through LDS
        float *red = (float *)lds;                // [4][2][1024], the stage memory is free now
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            red[(wave * 2 + 0) * 1024 + i * 64 + lane] = accM[i];
            red[(wave * 2 + 1) * 1024 + i * 64 + lane] = accB[i];
        }
        __syncthreads();
        for (int e = tid; e < 2048; e += 256) {
            const int prod = e >> 10, w = e & 1023;
            const int i = w >> 6, l = w & 63;
            const float s = (red[(0 * 2 + prod) * 1024 + w] + red[(1 * 2 + prod) * 1024 + w]) +
                            (red[(2 * 2 + prod) * 1024 + w] + red[(3 * 2 + prod) * 1024 + w]);
            const int row = (i >> 2) * 8 + (l >> 5) * 4 + (i & 3), col = l & 31;
            if (row < b && col < b) {
                if (prod == 0) {
                    dst[(size_t)row * b + col] = s;
                    dst[nelem + (size_t)col * b + row] = s;
                } else {
                    dst[2 * nelem + (size_t)row * b + col] = s;
                }
            }
        }
    } else {
        const int col = mj * ROWS + bj * 32 + r;
        const bool quad_ok = (b & 3) == 0;        // four consecutive rows of a column: one 16-byte store of M^T
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = mi * ROWS + bi * 32 + (i >> 2) * 8 + h * 4 + (i & 3);
            if (row < b && col < b) {
                dst[(size_t)row * b + col] = accM[i];
                dst[2 * nelem + (size_t)row * b + col] = accB[i];
                if (!quad_ok) dst[nelem + (size_t)col * b + row] = accM[i];
            }
        }
        if (quad_ok && col < b) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = mi * ROWS + bi * 32 + q * 8 + h * 4;
                if (row < b)
                    *(float4 *)&dst[nelem + (size_t)col * b + row] =
                        make_float4(accM[4 * q], accM[4 * q + 1], accM[4 * q + 2], accM[4 * q + 3]);
            }
        }
    }
}

// One workgroup per row i (b <= 128).  The 256 threads form G = 256 / W groups of
// W >= b lanes (W = 32, 64 or 128); group g adds chunks g, g + G, ... of row i
// of M, M^T and B in fp64, lane j taking column j (coalesced 4 W-byte reads),
// and the G sums are added in group order.
__global__ __launch_bounds__(256) void sp_finalize_kernel(const float *__restrict__ part, int nsplit, int b,
                                                          double *__restrict__ rowsum,
                                                          uint32_t *__restrict__ counter,
                                                          float *__restrict__ p_out)
{
    __shared__ double sm[3][256];
    __shared__ double wsum[4];
    const int i = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int W = b <= 32 ? 32 : (b <= 64 ? 64 : 128), G = 256 / W;
    const int j = t & (W - 1), grp = t / W;
    const size_t nelem = (size_t)b * b, cstride = 3 * nelem;
    constexpr int U = 8;                                          // chunks in flight per thread (3 loads each)
    double am = 0.0, at = 0.0, ab = 0.0;
    if (j < b) {
        const float *p = part + (size_t)i * b + j;
        int c = grp;
        for (; c + (U - 1) * G < nsplit; c += U * G) {
            float vm[U], vt[U], vb[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float *pc = p + (size_t)(c + u * G) * cstride;
                vm[u] = pc[0];
                vt[u] = pc[nelem];
                vb[u] = pc[2 * nelem];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                am += (double)vm[u];
                at += (double)vt[u];
                ab += (double)vb[u];
            }
        }
        for (; c < nsplit; c += G) {
            const float *pc = p + (size_t)c * cstride;
            am += (double)pc[0];
            at += (double)pc[nelem];
            ab += (double)pc[2 * nelem];
        }
    }
    sm[0][t] = am;
    sm[1][t] = at;
    sm[2][t] = ab;
    __syncthreads();
    double gt = 0.0, gr = 0.0;
    if (t < W && t < b) {
        double m = 0.0, mt = 0.0, bb = 0.0;
        for (int g = 0; g < G; ++g) {
            m += sm[0][g * W + t];
            mt += sm[1][g * W + t];
            bb += sm[2][g * W + t];
        }
        gr = bb;                                   // row i of R R^T
        gt = bb + 0.5 * (m + mt);                  // row i of T T^T
    }
    // sums over the row: waves 0 and 1 hold the (at most 128) columns
    auto row_sum = [&](double v) {
        v = wave_sum(v);
        __syncthreads();
        if (lane == 0) wsum[wave] = v;
        __syncthreads();
        return wsum[0] + wsum[1];
    };
    double nt = sqrt(row_sum(gt * gt)), nr = sqrt(row_sum(gr * gr));
    nt = nt < 1e-12 ? 1e-12 : nt;
    nr = nr < 1e-12 ? 1e-12 : nr;
    const double d = (t < W && t < b) ? gt / nt - gr / nr : 0.0;
    const double share = row_sum(d * d);
    __shared__ uint32_t ticket_s;
    if (t == 0) {
        rowsum[i] = share;
        __threadfence();                                   // publish the share, then take a ticket
        ticket_s = atomicAdd(counter, 1u);
    }
    __syncthreads();
    if (ticket_s != (uint32_t)(b - 1) || wave != 0) return;
    __threadfence();                                       // see every other workgroup's share
    const double v0 = lane < b ? __hip_atomic_load(&rowsum[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0;
    const double v1 = lane + 64 < b ? __hip_atomic_load(&rowsum[lane + 64], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0;
    const double tot = wave_sum(v0 + v1);
    if (lane == 0) *p_out = (float)(tot / ((double)b * (double)b));
}

hipError_t launch_plasticity(const void *a_t, egeria_dtype t_dt, const void *a_r, egeria_dtype r_dt,
                             int32_t b, int64_t D, float *p_out, void *ws_part, hipStream_t st)
{
    const GramPlan p = plan_gram(b, D);
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    uint32_t *counter = (uint32_t *)ws_part;
    double *rowsum = (double *)((char *)ws_part + off_rowsum());
    float *part = (float *)((char *)ws_part + off_partials(b));
    // whole K tiles and 16-byte aligned rows: the unconditional-load variant
    const bool vec = D % p.kt == 0;
    const dim3 grid((unsigned)(p.nsplit_pad * p.nmacro)), block(256);
    const int tcode = t_dt == EGERIA_BF16 ? 1 : 0, rcode = r_dt == EGERIA_BF16 ? 1 : 0;
    hipError_t e = hipSuccess;
#define EGERIA_GRAM(MTV, OFF, T, R, V)                                                                 \
    do {                                                                                               \
        /* two stages of nine bf16 planes of 4 KiB, twelve when off-diagonal macro tiles exist */      \
        constexpr size_t smem = (size_t)2 * (OFF ? 12 : 9) * 4096;                                     \
        static bool attr_set[kMaxDevices] = {};                                                        \
        if (!attr_set[dev]) {                                                                          \
            e = hipFuncSetAttribute((const void *)gram_partial_kernel<MTV, OFF, T, R, V>,              \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);            \
            if (e != hipSuccess) return e;                                                             \
            attr_set[dev] = true;                                                                      \
        }                                                                                              \
        e = launch_k(EGERIA_KERNEL_GRAM, gram_partial_kernel<MTV, OFF, T, R, V>, grid, block, smem,    \
                     st, a_t, a_r, (int)b, D, p, part, counter);                                       \
    } while (0)
#define EGERIA_GRAM_DT(MTV, OFF)                                                                       \
    do {                                                                                               \
        if (vec) {                                                                                     \
            if (!tcode && !rcode) EGERIA_GRAM(MTV, OFF, 0, 0, true);                                   \
            else if (tcode && !rcode) EGERIA_GRAM(MTV, OFF, 1, 0, true);                               \
            else if (!tcode && rcode) EGERIA_GRAM(MTV, OFF, 0, 1, true);                               \
            else EGERIA_GRAM(MTV, OFF, 1, 1, true);                                                    \
        } else {                                                                                       \
            if (!tcode && !rcode) EGERIA_GRAM(MTV, OFF, 0, 0, false);                                  \
            else if (tcode && !rcode) EGERIA_GRAM(MTV, OFF, 1, 0, false);                              \
            else if (!tcode && rcode) EGERIA_GRAM(MTV, OFF, 0, 1, false);                              \
            else EGERIA_GRAM(MTV, OFF, 1, 1, false);                                                   \
        }                                                                                              \
    } while (0)
    if (p.mt == 1) EGERIA_GRAM_DT(1, false);
    else if (p.nm == 1) EGERIA_GRAM_DT(2, false);
    else EGERIA_GRAM_DT(2, true);
#undef EGERIA_GRAM_DT
#undef EGERIA_GRAM
    if (e != hipSuccess) return e;
    return launch_k(EGERIA_KERNEL_NONE, sp_finalize_kernel, dim3((unsigned)b), dim3(256), 0, st, (const float *)part,
                    p.nsplit, (int)b, rowsum, counter, p_out);
}

}  // namespace egeria

// ---- the metric for callers that cannot allocate ------------------------------------------
// egeria_plasticity takes its scratch memory (ticket counter, row shares, split-K partials) from a
// workspace the caller allocated.  Code under HIP graph capture, tight serving loops and harnesses
// that forbid allocation have nowhere to get one: egeria_plasticity_noalloc runs the same two
// kernels on a scratch array that lives in the library's own device image.  Each GPU holds its own
// copy of the array, at its own address, until the process ends; `scratch` below is only the
// host-side handle of the symbol, and the device address is looked up once per device.
namespace {
constexpr size_t kScratchBytes = (size_t)16 << 20;      // >= plasticity_partial_bytes(b, D) for every b <= 128 on 256 CUs
std::mutex g_scratch_mutex;
void *g_scratch_ptr[egeria::kMaxDevices] = {};
}  // namespace

// (no `used` attribute: the compiler exports a file-scope static device array that host code names, and
// the runtime finds it by that exported name; marked `used` it stays a local symbol of the code object)
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of this GPU's copy of the array (the current device's), looked up on first use.
static hipError_t scratch_address(void **out)
{
    const int dev = egeria::current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

extern "C" egeria_status egeria_plasticity_noalloc(const void *a_train, egeria_dtype t_dt, const void *a_ref,
                                                   egeria_dtype r_dt, int32_t b, int64_t D, float *p_out, void *stream)
{
    using namespace egeria;
    if (!a_train || !a_ref || !p_out || b < 1 || D < 1) return EGERIA_ERR_INVALID_ARG;
    if (((uintptr_t)a_train & 15u) || ((uintptr_t)a_ref & 15u) || ((uintptr_t)p_out & 3u)) return EGERIA_ERR_INVALID_ARG;
    if ((t_dt != EGERIA_F32 && t_dt != EGERIA_BF16) || (r_dt != EGERIA_F32 && r_dt != EGERIA_BF16))
        return EGERIA_ERR_INVALID_ARG;
    if (b > 128) return EGERIA_ERR_UNSUPPORTED;
    if (plasticity_partial_bytes(b, D) > kScratchBytes) return EGERIA_ERR_UNSUPPORTED;     // beyond the array
    void *ptr = nullptr;
    if (scratch_address(&ptr) != hipSuccess) return EGERIA_ERR_HIP;
    // the kernels take the array's device address as they take the caller's workspace in
    // egeria_plasticity; what must start at zero (the finaliser's ticket) is cleared by the first kernel
    if (launch_plasticity(a_train, t_dt, a_ref, r_dt, b, D, p_out, ptr, (hipStream_t)stream) != hipSuccess)
        return EGERIA_ERR_HIP;
    return EGERIA_OK;
}
