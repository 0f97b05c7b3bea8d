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
//   each K tile.  Sample rows are fetched with full-line coalesced loads into a
//   double-buffered LDS stage (the next tile's loads are in flight while the
//   current one is contracted) and read back as 128-bit v_mfma_f32_32x32x2f32
//   operands: lane l takes row l % 32 and four consecutive k at 8s + 4(l / 32),
//   A and B operand alike, so the order of k inside the sum never matters.
//   Each workgroup stores its M block twice, as is and transposed, so that
//   the next kernel reads rows only.
// Kernel 2 (sp_finalize): one workgroup per row i of the b x b matrices.  It
//   sums row i of M, M^T and B over the chunks in fp64 (fixed assignment of
//   chunks to thread groups, fixed order), forms row i of both Gram matrices,
//   their norms and the row's share of the squared difference; the last
//   workgroup to finish adds the b shares in index order and writes P.
//   Results are bit-reproducible from call to call.
#include "common.hpp"

namespace egeria {

typedef float v16f __attribute__((ext_vector_type(16)));

struct GramPlan {
    int mt;          // blocks of 32 per macro-tile side: 1 (b <= 32) or 2
    int nm;          // macro tiles per side
    int nmacro;      // nm * nm
    int kt;          // K tile in floats: 128 (mt = 1) or 32 (mt = 2)
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
    p.kt = p.mt == 1 ? 128 : 32;
    int64_t want = (512 + p.nmacro - 1) / p.nmacro;       // about two workgroups per CU
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

// ---- global -> register staging of one [rows x KT] tile -------------------------------
// Thread `tid` owns float4 slots tid, tid + 256, ... of the tile (row-major
// slots, KT/4 per row), so that a wave reads whole 128-byte lines.
template <int DT>
__device__ __forceinline__ float4 load4(const void *__restrict__ base, int64_t row, bool row_ok,
                                        int64_t D, int64_t k, int64_t kend, bool vec)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!row_ok || k >= kend) return v;
    if (vec && k + 4 <= kend) {
        if (DT == 0) {
            v = *(const float4 *)((const float *)base + row * D + k);
        } else {
            const uint2 q = *(const uint2 *)((const uint16_t *)base + row * D + k);
            v.x = __uint_as_float(q.x << 16);
            v.y = __uint_as_float(q.x & 0xffff0000u);
            v.z = __uint_as_float(q.y << 16);
            v.w = __uint_as_float(q.y & 0xffff0000u);
        }
    } else {
        float e[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (k + i < kend)
                e[i] = DT == 0 ? ((const float *)base)[row * D + k + i]
                               : bf16_to_f32(((const uint16_t *)base)[row * D + k + i]);
        v = make_float4(e[0], e[1], e[2], e[3]);
    }
    return v;
}

template <int MT, int TDT, int RDT>
__global__ __launch_bounds__(256) void gram_partial_kernel(const void *__restrict__ at,
                                                           const void *__restrict__ ar, int b,
                                                           int64_t D, GramPlan p, bool vec,
                                                           float *__restrict__ part,
                                                           uint32_t *__restrict__ counter)
{
    constexpr int ROWS = MT * 32;                 // rows per side of the macro tile
    constexpr int KT = MT == 1 ? 128 : 32;        // floats per K tile
    constexpr int LD = KT + 4;                    // padded LDS row
    constexpr int SLOTS = ROWS * KT / 4;          // float4 slots of one tensor tile
    constexpr int NIT = SLOTS / 256;              // slots per thread
    constexpr int NTEN = MT == 1 ? 2 : 4;         // tensors staged: T_i, R_i (, T_j, R_j)
    static_assert(SLOTS % 256 == 0, "tile must divide over the workgroup");
    extern __shared__ __attribute__((aligned(16))) float lds[];   // [2 stages][NTEN][ROWS][LD]

    // consecutive workgroup ids land on different XCDs: all macro tiles of one
    // chunk go to the same XCD so that its L2 serves the re-reads of that chunk
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int chunk = (slot / p.nmacro) * 8 + xcd;
    const int mtile = slot % p.nmacro;
    if (chunk >= p.nsplit) return;
    const int mi = mtile / p.nm, mj = mtile % p.nm;
    const bool diag = MT == 1 || mi == mj;
    const int64_t k0 = (int64_t)chunk * p.kc;
    const int64_t k1 = k0 + p.kc < D ? k0 + p.kc : D;
    const int ntiles = (int)((k1 - k0 + KT - 1) / KT);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;

    // rows / columns this thread stages
    int srow[NIT], scol[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int s = tid + it * 256;
        srow[it] = s / (KT / 4);
        scol[it] = (s % (KT / 4)) * 4;
    }
    // Two register sets: global loads run two K tiles ahead of the MFMAs (one
    // tile of MFMAs is shorter than an HBM round trip), LDS holds two stages.
    auto fetch = [&](int t, float4 (&st)[NTEN][NIT]) {
        const int64_t kb = k0 + (int64_t)t * KT;       // past the chunk's end load4 returns zeros
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int64_t ri = (int64_t)mi * ROWS + srow[it];
            st[0][it] = load4<TDT>(at, ri, ri < b, D, kb + scol[it], k1, vec);
            st[1][it] = load4<RDT>(ar, ri, ri < b, D, kb + scol[it], k1, vec);
            if (NTEN == 4 && !diag) {
                const int64_t rj = (int64_t)mj * ROWS + srow[it];
                st[2][it] = load4<TDT>(at, rj, rj < b, D, kb + scol[it], k1, vec);
                st[3][it] = load4<RDT>(ar, rj, rj < b, D, kb + scol[it], k1, vec);
            }
        }
    };
    auto stash = [&](int stage, const float4 (&st)[NTEN][NIT]) {
        float *base = lds + (size_t)stage * NTEN * ROWS * LD;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int o = srow[it] * LD + scol[it];
            *(float4 *)&base[0 * ROWS * LD + o] = st[0][it];
            *(float4 *)&base[1 * ROWS * LD + o] = st[1][it];
            if (NTEN == 4 && !diag) {
                *(float4 *)&base[2 * ROWS * LD + o] = st[2][it];
                *(float4 *)&base[3 * ROWS * LD + o] = st[3][it];
            }
        }
    };

    v16f accM, accB;
#pragma unroll
    for (int i = 0; i < 16; ++i) { accM[i] = 0.0f; accB[i] = 0.0f; }

    // operand rows of this wave inside the macro tile
    const int bi = MT == 1 ? 0 : (wave >> 1), bj = MT == 1 ? 0 : (wave & 1);
    const int rowA = bi * 32 + r, rowB = bj * 32 + r;
    const int kw0 = MT == 1 ? wave * 32 : 0;      // this wave's 32-float slice of the K tile

    auto contract = [&](int stage) {
        const float *base = lds + (size_t)stage * NTEN * ROWS * LD;
        const float *pTi = base + 0 * ROWS * LD + rowA * LD + kw0 + 4 * h;
        const float *pRi = base + 1 * ROWS * LD + rowA * LD + kw0 + 4 * h;
        const float *pTj = base + (diag ? 0 : 2) * ROWS * LD + rowB * LD + kw0 + 4 * h;
        const float *pRj = base + (diag ? 1 : 3) * ROWS * LD + rowB * LD + kw0 + 4 * h;
        float4 ti[4], ri[4], tj[4], rj[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            ti[s] = *(const float4 *)(pTi + 8 * s);
            ri[s] = *(const float4 *)(pRi + 8 * s);
            tj[s] = *(const float4 *)(pTj + 8 * s);
            rj[s] = *(const float4 *)(pRj + 8 * s);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            accM = __builtin_amdgcn_mfma_f32_32x32x2f32(ti[s].x - ri[s].x, tj[s].x + rj[s].x, accM, 0, 0, 0);
            accB = __builtin_amdgcn_mfma_f32_32x32x2f32(ri[s].x, rj[s].x, accB, 0, 0, 0);
            accM = __builtin_amdgcn_mfma_f32_32x32x2f32(ti[s].y - ri[s].y, tj[s].y + rj[s].y, accM, 0, 0, 0);
            accB = __builtin_amdgcn_mfma_f32_32x32x2f32(ri[s].y, rj[s].y, accB, 0, 0, 0);
            accM = __builtin_amdgcn_mfma_f32_32x32x2f32(ti[s].z - ri[s].z, tj[s].z + rj[s].z, accM, 0, 0, 0);
            accB = __builtin_amdgcn_mfma_f32_32x32x2f32(ri[s].z, rj[s].z, accB, 0, 0, 0);
            accM = __builtin_amdgcn_mfma_f32_32x32x2f32(ti[s].w - ri[s].w, tj[s].w + rj[s].w, accM, 0, 0, 0);
            accB = __builtin_amdgcn_mfma_f32_32x32x2f32(ri[s].w, rj[s].w, accB, 0, 0, 0);
        }
    };

    float4 st0[NTEN][NIT], st1[NTEN][NIT];
    fetch(0, st0);
    fetch(1, st1);
    stash(0, st0);
    __syncthreads();
    // step t: tile t is in LDS stage t & 1, tile t + 1 in the set `rs`, tile t + 2 is requested into `rl`
    auto step = [&](int t, float4 (&rs)[NTEN][NIT], float4 (&rl)[NTEN][NIT]) {
        fetch(t + 2, rl);
        contract(t & 1);
        stash((t + 1) & 1, rs);
        __syncthreads();
    };
    for (int t = 0; t < ntiles; t += 2) {         // an odd count runs one extra step on zeros
        step(t, st1, st0);
        step(t + 1, st0, st1);
    }

    // lane l of a 32x32 block holds column l % 32, rows 8 * (i / 4) + 4 * (l / 32) + i % 4
    const size_t nelem = (size_t)b * b;
    float *dst = part + (size_t)chunk * 3 * nelem;               // M | M^T | B of this chunk
    if (id == 0 && tid == 0) *counter = 0u;                       // ticket of the finaliser
    if (MT == 1) {
        // the four waves hold partial sums over disjoint k: add them through LDS
        float *red = lds;                         // [4][2][1024], the stage memory is free now
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
    uint32_t *counter = (uint32_t *)ws_part;
    double *rowsum = (double *)((char *)ws_part + off_rowsum());
    float *part = (float *)((char *)ws_part + off_partials(b));
    const bool vec = (t_dt == EGERIA_F32 ? (D % 4 == 0) : (D % 8 == 0)) &&
                     (r_dt == EGERIA_F32 ? (D % 4 == 0) : (D % 8 == 0));
    const dim3 grid((unsigned)(p.nsplit_pad * p.nmacro)), block(256);
    const int tcode = t_dt == EGERIA_BF16 ? 1 : 0, rcode = r_dt == EGERIA_BF16 ? 1 : 0;
    hipError_t e = hipSuccess;
#define EGERIA_GRAM(MTV, T, R)                                                                         \
    do {                                                                                               \
        constexpr int rows = MTV * 32, kt = MTV == 1 ? 128 : 32, nten = MTV == 1 ? 2 : 4;              \
        constexpr size_t smem = (size_t)2 * nten * rows * (kt + 4) * sizeof(float);                    \
        static bool attr_set = false;                                                                  \
        if (!attr_set) {                                                                               \
            e = hipFuncSetAttribute((const void *)gram_partial_kernel<MTV, T, R>,                      \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);            \
            if (e != hipSuccess) return e;                                                             \
            attr_set = true;                                                                           \
        }                                                                                              \
        e = launch_k(EGERIA_KERNEL_GRAM, gram_partial_kernel<MTV, T, R>, grid, block, smem, st, a_t,   \
                     a_r, (int)b, D, p, vec, part, counter);                                           \
    } while (0)
    if (p.mt == 1) {
        if (!tcode && !rcode) EGERIA_GRAM(1, 0, 0);
        else if (tcode && !rcode) EGERIA_GRAM(1, 1, 0);
        else if (!tcode && rcode) EGERIA_GRAM(1, 0, 1);
        else EGERIA_GRAM(1, 1, 1);
    } else {
        if (!tcode && !rcode) EGERIA_GRAM(2, 0, 0);
        else if (tcode && !rcode) EGERIA_GRAM(2, 1, 0);
        else if (!tcode && rcode) EGERIA_GRAM(2, 0, 1);
        else EGERIA_GRAM(2, 1, 1);
    }
#undef EGERIA_GRAM
    if (e != hipSuccess) return e;
    return launch_k(EGERIA_KERNEL_NONE, sp_finalize_kernel, dim3((unsigned)b), dim3(256), 0, st, (const float *)part,
                    p.nsplit, (int)b, rowsum, counter, p_out);
}

}  // namespace egeria
