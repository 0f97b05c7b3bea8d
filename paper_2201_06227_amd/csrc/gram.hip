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
// Kernel 1 (gram_partial): split-K over D.  A workgroup owns one 32x32 block
//   (ib, jb) of both products and one chunk of D; its four waves interleave
//   over the chunk, each lane reading 64 contiguous bytes of one sample row
//   straight into v_mfma_f32_32x32x2f32 operand registers (the order of k
//   inside the sum is free, so no transposition is needed).  The four waves'
//   accumulators are summed through LDS and written as one partial.
// Kernel 2 (gram_reduce): sums the partials over chunks in fp64.
// Kernel 3 (sp_finalize): one workgroup: row norms, normalise, squared
//   Frobenius difference, all in fp64; writes P as fp32.
#include "common.hpp"

namespace egeria {

typedef float v16f __attribute__((ext_vector_type(16)));

struct GramPlan {
    int side;        // ceil(b / 32)
    int nblk;        // side * side
    int nsplit;      // chunks of D
    int nsplit_pad;  // rounded up to a multiple of 8 (one chunk per XCD slot)
    int64_t kc;      // chunk length, multiple of 128
};

static GramPlan plan_gram(int32_t b, int64_t D)
{
    GramPlan p;
    p.side = (b + 31) / 32;
    p.nblk = p.side * p.side;
    int64_t want = (512 + p.nblk - 1) / p.nblk;           // about two workgroups per CU
    int64_t cap = D / (8 * (int64_t)b);                   // keep partials below ~1/8 of the input bytes
    if (cap < 1) cap = 1;
    if (want > cap) want = cap;
    int64_t kc = (D + want - 1) / want;
    kc = (kc + 127) / 128 * 128;
    p.kc = kc;
    p.nsplit = (int)((D + kc - 1) / kc);
    p.nsplit_pad = (p.nsplit + 7) / 8 * 8;
    return p;
}

size_t plasticity_partial_bytes(int32_t b, int64_t D)
{
    GramPlan p = plan_gram(b, D);
    size_t nelem = 2 * (size_t)b * b;
    return align_up((size_t)p.nsplit * nelem * sizeof(float), 256) + align_up(nelem * sizeof(double), 256);
}

// 16 consecutive values of one row, zero beyond the row / the chunk end.
template <int DT>
__device__ __forceinline__ void load16(const void *__restrict__ base, int64_t row, bool row_ok,
                                       int64_t D, int64_t k, int64_t kend, bool vec, float (&v)[16])
{
    if (!row_ok || k >= kend) {
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = 0.0f;
        return;
    }
    if (vec && k + 16 <= kend) {
        if (DT == 0) {
            const float4 *p = (const float4 *)((const float *)base + row * D + k);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float4 q = p[j];
                v[4 * j] = q.x; v[4 * j + 1] = q.y; v[4 * j + 2] = q.z; v[4 * j + 3] = q.w;
            }
        } else {
            const uint4 *p = (const uint4 *)((const uint16_t *)base + row * D + k);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint4 q = p[j];
                uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[8 * j + 2 * e] = __uint_as_float(w[e] << 16);
                    v[8 * j + 2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
                }
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float x = 0.0f;
            if (k + e < kend) {
                if (DT == 0) x = ((const float *)base)[row * D + k + e];
                else x = bf16_to_f32(((const uint16_t *)base)[row * D + k + e]);
            }
            v[e] = x;
        }
    }
}

template <int TDT, int RDT, bool DIAG>
__device__ __forceinline__ void gram_block(const void *__restrict__ at, const void *__restrict__ ar,
                                           int b, int64_t D, int64_t k0, int64_t k1, int ib, int jb,
                                           bool vec, v16f &accM, v16f &accB)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int64_t row_i = (int64_t)ib * 32 + r, row_j = (int64_t)jb * 32 + r;
    const bool ok_i = row_i < b, ok_j = row_j < b;
    float ti[16], ri[16], tj[16], rj[16];
    float nti[16], nri[16], ntj[16], nrj[16];
    int64_t k = k0 + wave * 32 + h * 16;
    load16<TDT>(at, row_i, ok_i, D, k, k1, vec, ti);
    load16<RDT>(ar, row_i, ok_i, D, k, k1, vec, ri);
    if (!DIAG) {
        load16<TDT>(at, row_j, ok_j, D, k, k1, vec, tj);
        load16<RDT>(ar, row_j, ok_j, D, k, k1, vec, rj);
    }
    for (; k - h * 16 < k1; k += 128) {
        const int64_t kn = k + 128;
        // next step's operands are requested before this step's products are issued
        load16<TDT>(at, row_i, ok_i, D, kn, k1, vec, nti);
        load16<RDT>(ar, row_i, ok_i, D, kn, k1, vec, nri);
        if (!DIAG) {
            load16<TDT>(at, row_j, ok_j, D, kn, k1, vec, ntj);
            load16<RDT>(ar, row_j, ok_j, D, kn, k1, vec, nrj);
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const float a_t = ti[t], a_r = ri[t];
            const float b_t = DIAG ? ti[t] : tj[t], b_r = DIAG ? ri[t] : rj[t];
            accM = __builtin_amdgcn_mfma_f32_32x32x2f32(a_t - a_r, b_t + b_r, accM, 0, 0, 0);
            accB = __builtin_amdgcn_mfma_f32_32x32x2f32(a_r, b_r, accB, 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            ti[t] = nti[t]; ri[t] = nri[t];
            if (!DIAG) { tj[t] = ntj[t]; rj[t] = nrj[t]; }
        }
    }
}

template <int TDT, int RDT>
__global__ __launch_bounds__(256) void gram_partial_kernel(const void *__restrict__ at,
                                                           const void *__restrict__ ar, int b,
                                                           int64_t D, GramPlan p, bool vec,
                                                           float *__restrict__ part)
{
    // consecutive workgroup ids land on different XCDs: give all blocks of one
    // chunk to the same XCD so that its L2 serves the re-reads of that chunk
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int chunk = (slot / p.nblk) * 8 + xcd;
    const int blk = slot % p.nblk;
    if (chunk >= p.nsplit) return;
    const int ib = blk / p.side, jb = blk % p.side;
    const int64_t k0 = (int64_t)chunk * p.kc;
    const int64_t k1 = k0 + p.kc < D ? k0 + p.kc : D;

    v16f accM, accB;
#pragma unroll
    for (int r = 0; r < 16; ++r) { accM[r] = 0.0f; accB[r] = 0.0f; }
    if (ib == jb) gram_block<TDT, RDT, true>(at, ar, b, D, k0, k1, ib, jb, vec, accM, accB);
    else gram_block<TDT, RDT, false>(at, ar, b, D, k0, k1, ib, jb, vec, accM, accB);

    __shared__ float red[4][2][1024];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        red[wave][0][r * 64 + lane] = accM[r];
        red[wave][1][r * 64 + lane] = accB[r];
    }
    __syncthreads();
    const size_t nelem = (size_t)b * b;
    float *dst = part + (size_t)chunk * 2 * nelem;
    for (int e = threadIdx.x; e < 2048; e += 256) {
        const int prod = e >> 10, w = e & 1023;
        const int r = w >> 6, l = w & 63;
        const float s = (red[0][prod][w] + red[1][prod][w]) + (red[2][prod][w] + red[3][prod][w]);
        const int row = ib * 32 + (r >> 2) * 8 + (l >> 5) * 4 + (r & 3);
        const int col = jb * 32 + (l & 31);
        if (row < b && col < b) dst[prod * nelem + (size_t)row * b + col] = s;
    }
}

__global__ __launch_bounds__(256) void gram_reduce_kernel(const float *__restrict__ part, int nsplit,
                                                          int nelem2, double *__restrict__ out)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nelem2) return;
    double s = 0.0;
    for (int c = 0; c < nsplit; ++c) s += (double)part[(size_t)c * nelem2 + e];
    out[e] = s;
}

// red = [M | B], each b x b doubles.
__global__ __launch_bounds__(256) void sp_finalize_kernel(const double *__restrict__ red, int b,
                                                          float *__restrict__ p_out)
{
    const double *M = red, *B = red + (size_t)b * b;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double acc = 0.0;
    for (int i = wave; i < b; i += 4) {
        double nt2 = 0.0, nr2 = 0.0;
        for (int j = lane; j < b; j += 64) {
            const double gr = B[(size_t)i * b + j];
            const double gt = gr + 0.5 * (M[(size_t)i * b + j] + M[(size_t)j * b + i]);
            nt2 += gt * gt;
            nr2 += gr * gr;
        }
        nt2 = wave_sum(nt2);
        nr2 = wave_sum(nr2);
        double nt = sqrt(nt2), nr = sqrt(nr2);
        nt = nt < 1e-12 ? 1e-12 : nt;
        nr = nr < 1e-12 ? 1e-12 : nr;
        for (int j = lane; j < b; j += 64) {
            const double gr = B[(size_t)i * b + j];
            const double gt = gr + 0.5 * (M[(size_t)i * b + j] + M[(size_t)j * b + i]);
            const double d = gt / nt - gr / nr;
            acc += d * d;
        }
    }
    acc = wave_sum(acc);
    __shared__ double sm[4];
    if (lane == 0) sm[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) *p_out = (float)(((sm[0] + sm[1]) + (sm[2] + sm[3])) / ((double)b * (double)b));
}

hipError_t launch_plasticity(const void *a_t, egeria_dtype t_dt, const void *a_r, egeria_dtype r_dt,
                             int32_t b, int64_t D, float *p_out, void *ws_part, hipStream_t st)
{
    const GramPlan p = plan_gram(b, D);
    const size_t nelem = (size_t)b * b;
    float *part = (float *)ws_part;
    double *red = (double *)((char *)ws_part + align_up((size_t)p.nsplit * 2 * nelem * sizeof(float), 256));
    const bool vec = (t_dt == EGERIA_F32 ? (D % 4 == 0) : (D % 8 == 0)) &&
                     (r_dt == EGERIA_F32 ? (D % 4 == 0) : (D % 8 == 0));
    const unsigned grid = (unsigned)(p.nsplit_pad * p.nblk);
#define EGERIA_GRAM(T, R)                                                                         \
    hipLaunchKernelGGL((gram_partial_kernel<T, R>), dim3(grid), dim3(256), 0, st, a_t, a_r, (int)b, D, \
                       p, vec, part)
    hipError_t e;
    {
        ProfileScope prof(EGERIA_KERNEL_GRAM, st);
        if (t_dt == EGERIA_F32 && r_dt == EGERIA_F32) EGERIA_GRAM(0, 0);
        else if (t_dt == EGERIA_BF16 && r_dt == EGERIA_F32) EGERIA_GRAM(1, 0);
        else if (t_dt == EGERIA_F32 && r_dt == EGERIA_BF16) EGERIA_GRAM(0, 1);
        else EGERIA_GRAM(1, 1);
        e = hipGetLastError();
    }
#undef EGERIA_GRAM
    if (e != hipSuccess) return e;
    const int nelem2 = (int)(2 * nelem);
    hipLaunchKernelGGL(gram_reduce_kernel, dim3((nelem2 + 255) / 256), dim3(256), 0, st, part, p.nsplit,
                       nelem2, red);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sp_finalize_kernel, dim3(1), dim3(256), 0, st, red, (int)b, p_out);
    return hipGetLastError();
}

}  // namespace egeria
