// Floating-point glue of a Transformer encoder layer of the reference model:
// under dynamic quantisation (Section 5 of the paper) only the linear layers
// are int8; self-attention and layer norm read and write fp32 tensors.
#include "common.hpp"
#include <type_traits>

namespace egeria {

// ---- y = LN(x + res): one wave per row, evaluated in fp64 and rounded once ----------------
// (its output feeds a quantiser; see the note on the attention kernel)
__global__ __launch_bounds__(256) void layernorm_kernel(const float *__restrict__ x,
                                                        const float *__restrict__ res, int64_t rows,
                                                        int H, const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, double eps,
                                                        float *__restrict__ y,
                                                        uint32_t *__restrict__ absmax_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    uint32_t amax = 0;
    if (row < rows) {
        const float *xr = x + row * H;
        const float *rr = res ? res + row * H : nullptr;
        double s = 0.0;
        for (int h = lane; h < H; h += 64) s += (double)xr[h] + (rr ? (double)rr[h] : 0.0);
        const double mean = wave_sum(s) / (double)H;
        double q = 0.0;
        for (int h = lane; h < H; h += 64) {
            const double v = ((double)xr[h] + (rr ? (double)rr[h] : 0.0)) - mean;
            q += v * v;
        }
        const double var = wave_sum(q) / (double)H;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int h = lane; h < H; h += 64) {
            const double v = (double)xr[h] + (rr ? (double)rr[h] : 0.0);
            const double gm = gamma ? (double)gamma[h] : 1.0, bt = beta ? (double)beta[h] : 0.0;
            const float o = (float)((v - mean) * rstd * gm + bt);
            y[row * H + h] = o;
            const uint32_t ab = abs_bits(o);
            amax = amax > ab ? amax : ab;
        }
    }
    if (absmax_out) {
        __shared__ uint32_t sm4[4];
        block_atomic_max(amax, absmax_out, sm4);
    }
}

// Same, for rows of at most 256*NV floats with H a multiple of 4: the row is
// read once with 16-byte loads and stays in registers (as the exact fp64 sums
// x + res) for the three passes.
template <int NV>
__global__ __launch_bounds__(256) void layernorm_vec_kernel(const float *__restrict__ x,
                                                            const float *__restrict__ res, int64_t rows,
                                                            int H, const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, double eps,
                                                            float *__restrict__ y,
                                                            uint32_t *__restrict__ absmax_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    const int nv = H >> 2;
    uint32_t amax = 0;
    if (row < rows) {
        // Every load of the row goes out before the first wait: unconditional, with the index clamped
        // and the value replaced afterwards (a load under a per-lane condition is awaited on its own,
        // and a row would cost a dozen memory round trips instead of one).  Absent operands read x.
        const float4 *xr = reinterpret_cast<const float4 *>(x + row * H);
        const float4 *rr = reinterpret_cast<const float4 *>((res ? res : x) + row * H);
        const float4 *gr = reinterpret_cast<const float4 *>(gamma ? gamma : x + row * H);
        const float4 *br = reinterpret_cast<const float4 *>(beta ? beta : x + row * H);
        const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f), one4 = make_float4(1.f, 1.f, 1.f, 1.f);
        float4 xv[NV], rv[NV], gmv[NV], btv[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = lane + 64 * i, cc = c < nv ? c : nv - 1;
            xv[i] = xr[cc];
            rv[i] = rr[cc];
            gmv[i] = gr[cc];
            btv[i] = br[cc];
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const bool in = lane + 64 * i < nv;
            if (!in) xv[i] = zero4;
            if (!in || !res) rv[i] = zero4;
            if (!gamma) gmv[i] = one4;
            if (!beta) btv[i] = zero4;
        }
        float4 o[NV];
        ln_row_vec<NV>(xv, rv, gmv, btv, lane, nv, H, eps, o, amax);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = lane + 64 * i;
            if (c < nv) reinterpret_cast<float4 *>(y + row * H)[c] = o[i];
        }
    }
    if (absmax_out) {
        __shared__ uint32_t sm4[4];
        block_atomic_max(amax, absmax_out, sm4);
    }
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

hipError_t launch_layernorm(const float *x, const float *res, int64_t rows, int32_t H,
                            const float *gamma, const float *beta, float eps, float *y,
                            uint32_t *absmax_out, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    const bool vec = (H % 4) == 0 && H <= 1024 && aligned16(x) && aligned16(res) && aligned16(gamma) &&
                     aligned16(beta) && aligned16(y);
    if (vec && H <= 256)
        return launch_k(EGERIA_KERNEL_LAYERNORM, layernorm_vec_kernel<1>, grid, block, 0, st, x, res, rows, (int)H,
                        gamma, beta, (double)eps, y, absmax_out);
    if (vec && H <= 768)
        return launch_k(EGERIA_KERNEL_LAYERNORM, layernorm_vec_kernel<3>, grid, block, 0, st, x, res, rows, (int)H,
                        gamma, beta, (double)eps, y, absmax_out);
    if (vec)
        return launch_k(EGERIA_KERNEL_LAYERNORM, layernorm_vec_kernel<4>, grid, block, 0, st, x, res, rows, (int)H,
                        gamma, beta, (double)eps, y, absmax_out);
    return launch_k(EGERIA_KERNEL_LAYERNORM, layernorm_kernel, grid, block, 0, st, x, res, rows, (int)H, gamma, beta,
                    (double)eps, y, absmax_out);
}

// ---- multi-head self-attention -----------------------------------------------------------
// Evaluated in fp64 and rounded once to fp32, like the layer norm above: the
// context feeds a quantiser, where a last-bit difference can flip an int8 code
// and the flip is then amplified by every later layer.
//
// A workgroup owns one (batch, head) pair and 64 * QB queries, 16 * QB per wave (QB
// blocks of 16); key / value tiles of 32 rows pass through LDS as fp32 and are
// widened when read.  The products run on v_mfma_f64_16x16x4f64 in the
// transposed form
//     S^T = K Q^T  (keys x queries),      O^T = V^T P^T  (head dim x queries),
// so that a lane always owns one query column (lane = column + 16 * g, register
// r = row 4r + g): the soft-max statistics of a query are an in-lane reduction
// plus two exchanges across g, and the accumulator registers of S^T are,
// unchanged, the B operand of the second product.
typedef double v4d __attribute__((ext_vector_type(4)));
constexpr int kDh = 64;             // head dimension covered (smaller heads are zero padded)
constexpr int kKeyTile = 32;
constexpr int kKVPad = kDh + 4;

template <int QB>
__global__ __launch_bounds__(256) void attention_kernel(const float *__restrict__ qkv, int B, int S,
                                                        int Hd, int heads, int dh, double scale,
                                                        float *__restrict__ ctx,
                                                        uint32_t *__restrict__ absmax_out, int total,
                                                        int per_xcd)
{
    __shared__ __attribute__((aligned(16))) float sKb[2][kKeyTile][kKVPad];   // two stages
    __shared__ __attribute__((aligned(16))) float sVb[2][kKeyTile][kKVPad];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    constexpr int QT = 64 * QB;          // queries per workgroup
    const int qtiles = (S + QT - 1) / QT;
    // Workgroup ids are dealt round-robin to the 8 XCDs; each XCD is given a
    // contiguous range of (batch, head, query tile) so that the query tiles of
    // one head, which re-read the same K and V, share an L2.
    const int vid = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || vid >= total) return;
    const int bh = vid / qtiles, qt = vid % qtiles;
    const int bi = bh / heads, hd = bh % heads;
    const int64_t tok0 = (int64_t)bi * S;
    const int64_t ld = 3 * (int64_t)Hd;
    const float *qbase = qkv + hd * dh, *kbase = qbase + Hd, *vbase = qbase + 2 * Hd;

    // query rows as the B operand of S^T = K Q^T: d = 16u + 4g + e (u, e = 0..3).  The loads are
    // unconditional (row and column clamped to valid ones, the value discarded afterwards): loads
    // under a per-lane condition are awaited one by one, sixteen memory round trips before the
    // first key tile instead of one.
    const bool vec4 = (dh & 3) == 0 && (Hd & 3) == 0;
    double qr[QB][16];
    int qidx[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int q = qt * QT + wave * (16 * QB) + qb * 16 + c;
        qidx[qb] = q;
        const float *qrow = qbase + (tok0 + (q < S ? q : S - 1)) * ld;
        float qv[16];
        if (vec4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int d0 = 16 * u + 4 * g;
                const float4 v = *(const float4 *)(qrow + (d0 < dh ? d0 : 0));
                qv[4 * u] = v.x; qv[4 * u + 1] = v.y; qv[4 * u + 2] = v.z; qv[4 * u + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int d = 16 * u + 4 * g + e;
                    qv[4 * u + e] = qrow[d < dh ? d : 0];
                }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int d = 16 * u + 4 * g + e;
                qr[qb][4 * u + e] = (q < S && d < dh) ? (double)qv[4 * u + e] : 0.0;
            }
    }

    v4d o[QB][4];                       // O^T: [query block][16-row block of the head dim]
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 4; ++r) o[qb][db][r] = 0.0;
    double mrun[QB], lrun[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { mrun[qb] = -INFINITY; lrun[qb] = 0.0; }

    // Key / value tiles: thread t stages float4 slots t and t + 256 of the
    // 32 x 64 tile (row = slot / 16); the next tile's global loads are issued
    // before the current tile is contracted and land in the other LDS stage.
    float4 pk[2], pv[2];
    auto fetch = [&](int j0) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int sl = tid + it * 256, kr = sl >> 4, d = (sl & 15) * 4;
            const int64_t off = (tok0 + j0 + kr) * ld + d;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b4 = a;
            if (j0 + kr < S) {
                if (vec4 && d + 4 <= dh) {
                    a = *(const float4 *)(kbase + off);
                    b4 = *(const float4 *)(vbase + off);
                } else {
                    float ea[4] = {0.f, 0.f, 0.f, 0.f}, eb[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (d + e < dh) { ea[e] = kbase[off + e]; eb[e] = vbase[off + e]; }
                    a = make_float4(ea[0], ea[1], ea[2], ea[3]);
                    b4 = make_float4(eb[0], eb[1], eb[2], eb[3]);
                }
            }
            pk[it] = a;
            pv[it] = b4;
        }
    };
    auto stash = [&](int stage) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int sl = tid + it * 256, kr = sl >> 4, d = (sl & 15) * 4;
            *(float4 *)&sKb[stage][kr][d] = pk[it];
            *(float4 *)&sVb[stage][kr][d] = pv[it];
        }
    };
    fetch(0);
    stash(0);
    __syncthreads();
    int stage = 0;
    for (int j0 = 0; j0 < S; j0 += kKeyTile, stage ^= 1) {
        const bool more = j0 + kKeyTile < S;
        if (more) fetch(j0 + kKeyTile);
        float (*sK)[kKVPad] = sKb[stage];
        float (*sV)[kKVPad] = sVb[stage];

        v4d st[2][QB];                  // [key block][query block]
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 4; ++r) st[kb][qb][r] = 0.0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const float4 kv = *(const float4 *)&sK[kb * 16 + c][16 * u + 4 * g];
                const double k4[4] = {(double)kv.x, (double)kv.y, (double)kv.z, (double)kv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        st[kb][qb] = __builtin_amdgcn_mfma_f64_16x16x4f64(k4[e], qr[qb][4 * u + e], st[kb][qb], 0, 0, 0);
            }
        }
        // register r of st[kb][qb] is key j0 + 16*kb + 4*r + g for this lane's query
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            double mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int key = j0 + kb * 16 + 4 * r + g;
                    st[kb][qb][r] = key >= S ? -INFINITY : st[kb][qb][r] * scale;   // q.k first, then 1/sqrt(dh)
                    mx = fmax(mx, st[kb][qb][r]);
                }
            mx = fmax(mx, __shfl_xor(mx, 16, kWave));
            mx = fmax(mx, __shfl_xor(mx, 32, kWave));
            const double mnew = fmax(mrun[qb], mx);      // finite: every tile holds at least one key
            const double corr = exp(mrun[qb] - mnew);
            double ps = 0.0;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    st[kb][qb][r] = exp(st[kb][qb][r] - mnew);
                    ps += st[kb][qb][r];
                }
            ps += __shfl_xor(ps, 16, kWave);
            ps += __shfl_xor(ps, 32, kWave);
            lrun[qb] = lrun[qb] * corr + ps;
            mrun[qb] = mnew;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 4; ++r) o[qb][db][r] *= corr;
        }
        // O^T += V^T P^T: step (kb, r) contracts keys 16*kb + 4*r + g, g = 0..3
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int kr = kb * 16 + 4 * r + g;
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const double vv = (double)sV[kr][db * 16 + c];
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        o[qb][db] = __builtin_amdgcn_mfma_f64_16x16x4f64(vv, st[kb][qb][r], o[qb][db], 0, 0, 0);
                }
            }
        if (more) stash(stage ^ 1);
        __syncthreads();
    }

    uint32_t amax = 0;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int q = qidx[qb];
        if (q >= S) continue;
        float *dst = ctx + (tok0 + q) * Hd + hd * dh;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int d = db * 16 + 4 * r + g;
                if (d < dh) {
                    const float v = (float)(o[qb][db][r] / lrun[qb]);
                    dst[d] = v;
                    const uint32_t ab = abs_bits(v);
                    amax = amax > ab ? amax : ab;
                }
            }
    }
    if (absmax_out) {
        __shared__ uint32_t sm4[4];
        block_atomic_max(amax, absmax_out, sm4);
    }
}

// ---- the same attention in fp32 arithmetic on the matrix cores, with certified int8 codes ----------
// Unobserved runs do not need the context as the fp64 evaluation gives it: all that leaves this stage
// is the int8 input of the next GEMM and its scale.  Three launches (two with the bf16-split kernel, whose
// workgroups settle the exact maximum themselves as they finish):
//   1. an approximate attention with fp32 products and sums: attention_split_kernel (further down: every
//      fp32 product as six bf16 partial products on the bf16 matrix cores; head dims in whole units of 8)
//      or attention_fast_kernel (here: the structure of the kernel above on v_mfma_f32_16x16x4f32, hardware
//      exp2; any head size).  It stores an approximate context and, per 64 queries of a head, a record: the
//      largest |context| it stored and an error bound E for its values (below).
//   2. attention_absmax_exact_kernel: the tensor's absolute maximum as the fp64 evaluation gives it.  Every
//      value that can be the maximum (|x| + E >= largest |x| - largest E; as a rule one) is re-evaluated in fp64.
//   3. quantize_attention_certify_kernel: the streaming map to codes.  code(x) = clamp(rne(x * inv)) is
//      monotone in x, so an approximate value whose interval [x - E, x + E] maps to one code has that
//      code; the others (a few in ten thousand) are re-evaluated in fp64, a wave per value, by the
//      workgroup that met them.
// The bound of a value x: E = 2^-24 * (max|v| of the head * (kErrBase + kErrPerScore * max|score| of the
// workgroup) + kErrRel |x|).  It is an empirical bound with margin, not a proof: bench.py --attention-error
// measures kernel 1 against the fp64 kernel on the twelve layers of the BERT-base-shaped stack (12.6 M
// values each) and prints the largest error / E per layer.
typedef float v4f __attribute__((ext_vector_type(4)));
constexpr float kErrBase = 2.0f, kErrPerScore = 0.5f;
// ... plus a part that grows with the value itself (the drift of the matrix cores' accumulation is
// proportional to the sums it carries): kErrRel * 2^-24 * |x|
constexpr float kErrRel = 12.0f * 5.9604645e-8f;
// error bound of one approximate context value x whose workgroup's record says err
__device__ __forceinline__ float value_err(float err, float x) { return fmaf(kErrRel, fabsf(x), err); }
struct AttnRecord {
    uint32_t amax_bits;     // largest |approximate context| of the workgroup's 64 queries x head dims
    float err;              // E for those values
};

__global__ __launch_bounds__(256) void attention_fast_kernel(const float *__restrict__ qkv, int B, int S, int Hd,
                                                             int heads, int dh, float scale, float *__restrict__ ctx,
                                                             AttnRecord *__restrict__ rec, int total, int per_xcd,
                                                             uint32_t *__restrict__ amax_slot,
                                                             uint32_t *__restrict__ err_slot)
{
    __shared__ __attribute__((aligned(16))) float sKb[2][kKeyTile][kKVPad];
    __shared__ __attribute__((aligned(16))) float sVb[2][kKeyTile][kKVPad];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    constexpr int QT = 64;
    const int qtiles = (S + QT - 1) / QT;
    const int vid = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || vid >= total) return;
    const int bh = vid / qtiles, qt = vid % qtiles;
    const int bi = bh / heads, hd = bh % heads;
    const int64_t tok0 = (int64_t)bi * S;
    const int64_t ld = 3 * (int64_t)Hd;
    const float *qbase = qkv + hd * dh, *kbase = qbase + Hd, *vbase = qbase + 2 * Hd;
    const bool vec4 = (dh & 3) == 0 && (Hd & 3) == 0;
    // query rows as the B operand of S^T = K Q^T: lane (c, g) holds dims 16u + 4g + e of query c
    float qr[16];
    const int q = qt * QT + wave * 16 + c;
    {
        const float *qrow = qbase + (tok0 + (q < S ? q : S - 1)) * ld;
        float qv[16];
        if (vec4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int d0 = 16 * u + 4 * g;
                const float4 v = *(const float4 *)(qrow + (d0 < dh ? d0 : 0));
                qv[4 * u] = v.x; qv[4 * u + 1] = v.y; qv[4 * u + 2] = v.z; qv[4 * u + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int d = 16 * u + 4 * g + e;
                    qv[4 * u + e] = qrow[d < dh ? d : 0];
                }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int d = 16 * u + 4 * g + e;
                qr[4 * u + e] = (q < S && d < dh) ? qv[4 * u + e] : 0.0f;
            }
    }
    v4f o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[db][r] = 0.0f;
    float mrun = -INFINITY, lrun = 0.0f;
    float smax = 0.0f;                  // largest |score| met by this lane
    uint32_t vmax = 0;                  // largest |v| staged by this thread (bit pattern)
    float4 pk[2], pv[2];
    auto fetch = [&](int j0) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int sl = tid + it * 256, kr = sl >> 4, d = (sl & 15) * 4;
            const int64_t off = (tok0 + j0 + kr) * ld + d;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b4 = a;
            if (j0 + kr < S) {
                if (vec4 && d + 4 <= dh) {
                    a = *(const float4 *)(kbase + off);
                    b4 = *(const float4 *)(vbase + off);
                } else {
                    float ea[4] = {0.f, 0.f, 0.f, 0.f}, eb[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (d + e < dh) { ea[e] = kbase[off + e]; eb[e] = vbase[off + e]; }
                    a = make_float4(ea[0], ea[1], ea[2], ea[3]);
                    b4 = make_float4(eb[0], eb[1], eb[2], eb[3]);
                }
            }
            pk[it] = a;
            pv[it] = b4;
        }
    };
    auto stash = [&](int stage) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int sl = tid + it * 256, kr = sl >> 4, d = (sl & 15) * 4;
            *(float4 *)&sKb[stage][kr][d] = pk[it];
            *(float4 *)&sVb[stage][kr][d] = pv[it];
            uint32_t a0 = abs_bits(pv[it].x), a1 = abs_bits(pv[it].y), a2 = abs_bits(pv[it].z), a3 = abs_bits(pv[it].w);
            a0 = a0 > a1 ? a0 : a1;
            a2 = a2 > a3 ? a2 : a3;
            a0 = a0 > a2 ? a0 : a2;
            vmax = vmax > a0 ? vmax : a0;
        }
    };
    fetch(0);
    stash(0);
    __syncthreads();
    int stage = 0;
    constexpr float kLog2e = 1.44269504088896340736f;
    for (int j0 = 0; j0 < S; j0 += kKeyTile, stage ^= 1) {
        const bool more = j0 + kKeyTile < S;
        if (more) fetch(j0 + kKeyTile);
        float (*sK)[kKVPad] = sKb[stage];
        float (*sV)[kKVPad] = sVb[stage];
        v4f st[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 4; ++r) st[kb][r] = 0.0f;
        // The matrix cores' accumulation is not round-to-nearest over a chain of instructions: measured against
        // fp64, a sum carried through n dependent MFMAs drifts by about n/4 ulp of its size, always towards
        // zero.  Chains are therefore kept short (four instructions from a zero accumulator) and their
        // results are added on the vector ALU, which rounds to nearest: the error of the context dropped
        // from 14 to 4 ulp of the tensor's maximum for 4 % more time.
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const float4 kv = *(const float4 *)&sK[kb * 16 + c][16 * u + 4 * g];
                const float k4[4] = {kv.x, kv.y, kv.z, kv.w};
                v4f part = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    part = __builtin_amdgcn_mfma_f32_16x16x4f32(k4[e], qr[4 * u + e], part, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) st[kb][r] += part[r];
            }
        }
        // register r of st[kb] is key j0 + 16 kb + 4 g + r for this lane's query
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = j0 + kb * 16 + 4 * g + r;
                const float sc = st[kb][r] * scale;
                smax = key < S ? fmaxf(smax, fabsf(sc)) : smax;
                st[kb][r] = key < S ? sc : -INFINITY;
                mx = fmaxf(mx, st[kb][r]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float mnew = fmaxf(mrun, mx);
        const float corr = __builtin_amdgcn_exp2f((mrun - mnew) * kLog2e);
        float ps = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                st[kb][r] = __builtin_amdgcn_exp2f((st[kb][r] - mnew) * kLog2e);
                ps += st[kb][r];
            }
        ps += __shfl_xor(ps, 16, kWave);
        ps += __shfl_xor(ps, 32, kWave);
        lrun = lrun * corr + ps;
        mrun = mnew;
        // this tile's V^T P^T from a zero accumulator (step (kb, r) contracts keys 16 kb + 4 g + r, g = 0..3),
        // then O^T = O^T * corr + tile on the vector ALU
        v4f ot[4];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 4; ++r) ot[db][r] = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int kr = kb * 16 + 4 * g + r;
#pragma unroll
                for (int db = 0; db < 4; ++db)
                    ot[db] = __builtin_amdgcn_mfma_f32_16x16x4f32(sV[kr][db * 16 + c], st[kb][r], ot[db], 0, 0, 0);
            }
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 4; ++r) o[db][r] = fmaf(o[db][r], corr, ot[db][r]);
        if (more) stash(stage ^ 1);
        __syncthreads();
    }

    uint32_t amax = 0;
    if (q < S) {
        float *dst = ctx + (tok0 + q) * Hd + hd * dh;
        const float inv = 1.0f / lrun;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const int d = db * 16 + 4 * g;              // registers 0..3: four consecutive head dims
            float v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                v[r] = o[db][r] * inv;
                const uint32_t ab = abs_bits(v[r]);
                amax = (d + r < dh && ab > amax) ? ab : amax;
            }
            if (vec4 && d + 4 <= dh) {
                *(float4 *)(dst + d) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (d + r < dh) dst[d + r] = v[r];
            }
        }
    }
    // the workgroup's record: largest |context| stored, and the error bound of its values
    __shared__ uint32_t red[3][4];
    amax = wave_max_u32(amax);
    vmax = wave_max_u32(vmax);
    const uint32_t sbits = wave_max_u32(__float_as_uint(smax));       // non-negative floats order like integers
    if (lane == 0) { red[0][wave] = amax; red[1][wave] = vmax; red[2][wave] = sbits; }
    __syncthreads();
    if (tid == 0) {
        uint32_t a = 0, v = 0, sb = 0;
        for (int w = 0; w < 4; ++w) {
            a = a > red[0][w] ? a : red[0][w];
            v = v > red[1][w] ? v : red[1][w];
            sb = sb > red[2][w] ? sb : red[2][w];
        }
        AttnRecord r;
        r.amax_bits = a;
        r.err = 5.9604645e-8f * __uint_as_float(v) * (kErrBase + kErrPerScore * __uint_as_float(sb));
        if (!(r.err <= 3.402823466e+38f)) r.amax_bits = 0x7f800000u;   // non-finite inputs: flagged downstream
        rec[vid] = r;
        // the largest of both over all workgroups, for the kernel that settles the exact maximum (atomically
        // combined words spread over ways; both are non-negative floats, whose bit patterns order like them)
        if (amax_slot) {
            uint32_t *wa = amax_slot + (blockIdx.x & (kAmaxWays - 1)) * kAmaxStride;
            uint32_t *we = err_slot + (blockIdx.x & (kAmaxWays - 1)) * kAmaxStride;
            const uint32_t eb = __float_as_uint(r.err);
            if (r.amax_bits > __hip_atomic_load(wa, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(wa, r.amax_bits);
            if (eb > __hip_atomic_load(we, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(we, eb);
        }
    }
}

// ---- kernel 1 on the bf16 matrix cores, every product an exact fp32 product -----------------------
// The fp32 matrix instruction runs at 1/16 of the bf16 one.  An fp32 value is the sum of three bf16
// values (8 + 8 + 8 significant bits: the value truncated, the remainder truncated, what is left; both
// subtractions are exact), so a product x * y is nine bf16 x bf16 products, each exact in fp32; the six
// largest are issued (v_mfma_f32_32x32x16_bf16, fp32 accumulation), the three dropped ones sum to less
// than 2^-22 of the product: six bf16 instructions for what sixteen times as many fp32 ones did.  Within a
// chain the small partial products come first, so that the sums carried through most of the chain are
// small against the result (the matrix cores' accumulation drifts with the sums it carries).
// Geometry: a workgroup is four waves x 32 queries of one head; a tile is 32 keys.  S^T = K Q^T and
// O^T = V^T P^T as above, so a lane owns a query column: lane l holds query l % 32 and, of a 32-row
// block, rows 8 (i / 4) + 4 (l / 32) + i % 4 in accumulator register i.  Operands: lane l supplies row
// l % 32 and the 8 values of unit l / 32 of a 16-deep slab.  For the second product the lane's own
// registers 8 s .. 8 s + 7 are its unit of slab s (which keys share a unit is free as long as the V
// operand uses the same assignment), so P never leaves the registers; V is written to LDS transposed,
// as bf16 planes [head dim][unit][slot] in that assignment.  K planes are [key][unit] with the units
// xor-rotated by the row; V rows are padded to 80 bytes: all 16-byte operand reads are conflict free.
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
// (defined further down; the kernel below ends with the exact evaluation of its candidates for the maximum)
__device__ __forceinline__ float context_exact(const float *__restrict__ qkv, int S, int Hd, int heads, int dh, double scale,
                                               uint32_t el, double *red);
template <typename F>
__device__ __forceinline__ void for_each_marked(bool mine, uint64_t *masks, F visit);
constexpr int kSplitQ = 128;             // queries per workgroup
constexpr int kSplitKeys = 32;           // keys per tile
constexpr int kSplitKRow = 128;          // bytes per key row of a K plane (8 units)
constexpr int kSplitVRow = 80;           // bytes per head-dim row of a V plane (4 units + pad)
constexpr int kSplitKPlane = kSplitKeys * kSplitKRow, kSplitVPlane = kDh * kSplitVRow;
constexpr int kSplitStage = 3 * (kSplitKPlane + kSplitVPlane);

struct Split3 {
    v4u h, m, l;
};
// two floats -> the bf16 truncation of each, x0 in the low half
__device__ __forceinline__ uint32_t pack_top16(float x1, float x0)
{
    return __builtin_amdgcn_perm(__float_as_uint(x1), __float_as_uint(x0), 0x07060302u);
}
__device__ __forceinline__ void split_pair(float x0, float x1, uint32_t &h, uint32_t &m, uint32_t &l)
{
    const float r0 = x0 - __uint_as_float(__float_as_uint(x0) & 0xffff0000u);
    const float r1 = x1 - __uint_as_float(__float_as_uint(x1) & 0xffff0000u);
    const float l0 = r0 - __uint_as_float(__float_as_uint(r0) & 0xffff0000u);
    const float l1 = r1 - __uint_as_float(__float_as_uint(r1) & 0xffff0000u);
    h = pack_top16(x1, x0);
    m = pack_top16(r1, r0);
    l = pack_top16(l1, l0);
}
__device__ __forceinline__ Split3 split_eight(const float (&x)[8])
{
    Split3 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        uint32_t wh, wm, wl;
        split_pair(x[2 * e], x[2 * e + 1], wh, wm, wl);
        o.h[e] = wh;
        o.m[e] = wm;
        o.l[e] = wl;
    }
    return o;
}

__global__ __launch_bounds__(256, 2) void attention_split_kernel(const float *__restrict__ qkv, int B, int S, int Hd,
                                                                 int heads, int dh, float scale, float *__restrict__ ctx,
                                                                 AttnRecord *__restrict__ rec, int total, int per_xcd,
                                                                 uint32_t *__restrict__ bound_slot,
                                                                 uint32_t *__restrict__ exact_slot)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * kSplitStage];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int qblocks = (S + kSplitQ - 1) / kSplitQ, qtiles = (S + 63) / 64;
    const int vid = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || vid >= total) return;
    const int bh = vid / qblocks, qb = vid % qblocks;
    const int bi = bh / heads, hd = bh % heads;
    const int64_t tok0 = (int64_t)bi * S;
    const int64_t ld = 3 * (int64_t)Hd;
    const float *qbase = qkv + hd * dh, *kbase = qbase + Hd, *vbase = qbase + 2 * Hd;

    // the wave's queries as the B operand of S^T = K Q^T: lane (r, h) holds dims 16 sl + 8 h .. + 7 of query r
    const int q = qb * kSplitQ + wave * 32 + r;
    Split3 qs[4];
    {
        const float *qrow = qbase + (tok0 + (q < S ? q : S - 1)) * ld;
        float4 raw[8];
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {
            const int d0 = 16 * sl + 8 * h;
            const int dc = d0 < dh ? d0 : 0;                     // head dims come in whole units of 8
            raw[2 * sl] = *(const float4 *)(qrow + dc);
            raw[2 * sl + 1] = *(const float4 *)(qrow + dc + 4);
        }
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {
            const bool ok = q < S && 16 * sl + 8 * h < dh;
            const float4 a = raw[2 * sl], b4 = raw[2 * sl + 1];
            const float x[8] = {ok ? a.x : 0.f, ok ? a.y : 0.f, ok ? a.z : 0.f, ok ? a.w : 0.f,
                                ok ? b4.x : 0.f, ok ? b4.y : 0.f, ok ? b4.z : 0.f, ok ? b4.w : 0.f};
            qs[sl] = split_eight(x);
        }
    }

    // staging.  K: thread t takes unit t % 8 (8 head dims) of key t / 8.  V: lane l of wave w takes head dims
    // 4 (4 w + l % 4) .. + 3 of keys 2 (l / 4) and 2 (l / 4) + 1 (two keys that are neighbours in a unit: one
    // 4-byte LDS word per head dim and plane; a wave's words fall into 64 different banks).
    const int skr = tid >> 3, sku = tid & 7;
    const int svd = 4 * (4 * wave + (lane & 3)), svk = 2 * (lane >> 2);
    const uint32_t koff = (uint32_t)(skr * kSplitKRow + ((sku ^ ((skr >> 1) & 7)) * 16));
    // key k of a tile: slab k / 16, unit 2 (k / 16) + (k / 4) % 2, slot 4 ((k / 8) % 2) + k % 4
    const uint32_t voff = (uint32_t)(svd * kSplitVRow + (2 * (svk >> 4) + ((svk >> 2) & 1)) * 16 + (4 * ((svk >> 3) & 1) + (svk & 3)) * 2);
    uint32_t vmax = 0;                  // largest |v| staged by this thread (bit pattern)
    float4 pk[2], pv[2];
    // Loads are unconditional, from clamped addresses: a key beyond S reads the last key's row (its score is
    // masked in the ragged tile, its P is exactly zero), head dims beyond dh read dims 0.. (the query is zero
    // there, and those rows of O^T are never stored).  No zeroing, so nothing waits for a load before its use.
    const float *kfetch = kbase + tok0 * ld + (8 * sku < dh ? 8 * sku : 0);
    const float *vfetch = vbase + tok0 * ld + (svd < dh ? svd : 0);
    auto fetch_k = [&](int j0) {
        const int row = j0 + skr < S ? j0 + skr : S - 1;
        const float *kp = kfetch + (int64_t)row * ld;
        pk[0] = *(const float4 *)kp;
        pk[1] = *(const float4 *)(kp + 4);
    };
    auto fetch_v = [&](int j0) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int row = j0 + svk + e < S ? j0 + svk + e : S - 1;
            pv[e] = *(const float4 *)(vfetch + (int64_t)row * ld);
        }
    };
    auto stash_k = [&](int buf) {
        uint8_t *kst = lds + buf * kSplitStage;
        const float x[8] = {pk[0].x, pk[0].y, pk[0].z, pk[0].w, pk[1].x, pk[1].y, pk[1].z, pk[1].w};
        const Split3 sp = split_eight(x);
        *(v4u *)(kst + koff) = sp.h;
        *(v4u *)(kst + kSplitKPlane + koff) = sp.m;
        *(v4u *)(kst + 2 * kSplitKPlane + koff) = sp.l;
    };
    auto stash_v = [&](int buf) {
        uint8_t *vst = lds + buf * kSplitStage + 3 * kSplitKPlane;
        const float v0[4] = {pv[0].x, pv[0].y, pv[0].z, pv[0].w}, v1[4] = {pv[1].x, pv[1].y, pv[1].z, pv[1].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t wh, wm, wl;
            split_pair(v0[e], v1[e], wh, wm, wl);
            uint8_t *dst = vst + voff + e * kSplitVRow;
            *(uint32_t *)dst = wh;
            *(uint32_t *)(dst + kSplitVPlane) = wm;
            *(uint32_t *)(dst + 2 * kSplitVPlane) = wl;
            const uint32_t a0 = abs_bits(v0[e]), a1 = abs_bits(v1[e]);
            vmax = vmax > a0 ? vmax : a0;
            vmax = vmax > a1 ? vmax : a1;
        }
    };

    // (plane of the K or V operand, plane of the Q or P operand), 0 = high part.  The small products come
    // first; a K / V plane is used for consecutive products so that few operand registers are live.
    constexpr int ia[6] = {2, 1, 1, 0, 0, 0}, ib[6] = {0, 1, 0, 2, 1, 0};
    const uint32_t ka_off = (uint32_t)(r * kSplitKRow), ka_sw = (uint32_t)((r >> 1) & 7);
    // raw scores (before the 1 / sqrt(dh) factor) of the tile in K buffer `buf`: register i is key
    // 8 (i / 4) + 4 h + i % 4 of the tile for this lane's query
    auto scores = [&](int buf) {
        const uint8_t *kst = lds + buf * kSplitStage;
        v16f acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
#pragma unroll
        for (int pr = 0; pr < 6; ++pr)
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                const v4u ak = *(const v4u *)(kst + ia[pr] * kSplitKPlane + ka_off + ((((uint32_t)(2 * sl + h)) ^ ka_sw) * 16));
                const v4u bq = ib[pr] == 0 ? qs[sl].h : (ib[pr] == 1 ? qs[sl].m : qs[sl].l);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, ak), __builtin_bit_cast(v8bf, bq), acc, 0, 0, 0);
            }
        return acc;
    };

    v16f o[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.0f;
    float mrun = -INFINITY, lrun = 0.0f;   // running maximum of the raw scores, running sum
    float smax = 0.0f;                  // largest |raw score| met by this lane
    const float c2 = scale * 1.44269504088896340736f;            // raw score -> exponent of 2

    // Software pipeline over the tiles.  Iteration t contracts S(t + 1), turns S(t) into P(t), contracts
    // P(t) V(t) and splits K(t + 2) and V(t + 1) (in registers since the iteration before) into the buffers
    // that S(t) and V(t - 1) have left: the scores of the next tile do not wait for this tile's soft-max, and
    // a tile's loads have a whole iteration to arrive.  One barrier per tile.  (Measured on this chip: the
    // vector instructions that follow a matrix instruction in a wave's issue order do not run beside it, and
    // two waves of a SIMD overlap them by about a third; the kernel's time is close to the sum of its 48
    // matrix and 430 vector instructions per tile, whatever their order.)
    const int ntiles = (S + kSplitKeys - 1) / kSplitKeys;
    fetch_k(0);
    fetch_v(0);
    stash_k(0);
    stash_v(0);
    fetch_k(kSplitKeys);
    fetch_v(kSplitKeys);
    stash_k(1);
    fetch_k(2 * kSplitKeys);
    __syncthreads();
    v16f sacc = scores(0);
    __syncthreads();                                             // K buffer 0 is rewritten in iteration 0
    // (the loads are unconditional; scores and staging of tiles past the end are skipped under uniform branches)
    auto iteration = [&](int t, auto ragged) {
        const int j0 = t * kSplitKeys;
        v16f snext = sacc;
        if (t + 1 < ntiles) snext = scores((t + 1) & 1);
        // soft-max of tile t
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) smax = fmaxf(smax, fabsf(sacc[i]));     // keys beyond S: zero rows, score 0
        if constexpr (decltype(ragged)::value) {                 // the ragged last tile: keys beyond S do not count
#pragma unroll
            for (int i = 0; i < 16; ++i)
                sacc[i] = j0 + 8 * (i >> 2) + 4 * h + (i & 3) < S ? sacc[i] : -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float mnew = fmaxf(mrun, mx);
        const float corr = __builtin_amdgcn_exp2f((mrun - mnew) * c2);
        const float shift = -mnew * c2;
        float ps = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            sacc[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], c2, shift));
            ps += sacc[i];
        }
        ps += __shfl_xor(ps, 32, kWave);
        lrun = lrun * corr + ps;
        mrun = mnew;
        // the lane's unit of slab s of P^T: its registers 8 s .. 8 s + 7
        Split3 pp[2];
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            const float x[8] = {sacc[8 * sl], sacc[8 * sl + 1], sacc[8 * sl + 2], sacc[8 * sl + 3],
                                sacc[8 * sl + 4], sacc[8 * sl + 5], sacc[8 * sl + 6], sacc[8 * sl + 7]};
            pp[sl] = split_eight(x);
        }
        // this tile's V^T P^T from zero accumulators (two independent chains, one per half of the head dims),
        // then O^T = O^T * corr + tile on the vector ALU
        {
            const uint8_t *vst = lds + (t & 1) * kSplitStage + 3 * kSplitKPlane;
            v16f ot[2];
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) ot[db][i] = 0.0f;
#pragma unroll
            for (int pr = 0; pr < 6; ++pr)
#pragma unroll
                for (int sl = 0; sl < 2; ++sl) {
                    const v4u bp = ib[pr] == 0 ? pp[sl].h : (ib[pr] == 1 ? pp[sl].m : pp[sl].l);
#pragma unroll
                    for (int db = 0; db < 2; ++db) {
                        const v4u av = *(const v4u *)(vst + ia[pr] * kSplitVPlane + (32 * db + r) * kSplitVRow + (2 * sl + h) * 16);
                        ot[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, av), __builtin_bit_cast(v8bf, bp), ot[db], 0, 0, 0);
                    }
                }
            if (t + 2 < ntiles) stash_k(t & 1);
            if (t + 1 < ntiles) stash_v((t + 1) & 1);
            fetch_k(j0 + 3 * kSplitKeys);
            fetch_v(j0 + 2 * kSplitKeys);
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] = fmaf(o[db][i], corr, ot[db][i]);
        }
        sacc = snext;
        __syncthreads();
    };
    const int nfull = S / kSplitKeys;
    for (int t = 0; t < nfull; ++t) iteration(t, std::false_type{});
    if (nfull < ntiles) iteration(nfull, std::true_type{});
    smax *= scale;

    // register i of block db is head dim 32 db + 8 (i / 4) + 4 h + i % 4 of this lane's query
    uint32_t amax = 0;
    if (q < S) {
        float *dst = ctx + (tok0 + q) * Hd + hd * dh;
        const float inv = 1.0f / lrun;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * db + 8 * g + 4 * h;
                if (d < dh) {                                    // head dims come in whole units of 8
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = o[db][4 * g + e] * inv;
                        const uint32_t ab = abs_bits(v[e]);
                        amax = ab > amax ? ab : amax;
                    }
                    *(float4 *)(dst + d) = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
    }
    // records: one per 64 queries (a pair of waves): largest |context| stored, and the error bound of its values
    __shared__ uint32_t red[3][4];
    __shared__ float rec_err[2], rec_low[2];
    __shared__ uint32_t non_finite;
    amax = wave_max_u32(amax);
    vmax = wave_max_u32(vmax);
    const uint32_t sbits = wave_max_u32(__float_as_uint(smax));       // non-negative floats order like integers
    if (lane == 0) { red[0][wave] = amax; red[1][wave] = vmax; red[2][wave] = sbits; }
    if (tid == 0) non_finite = 0;
    __syncthreads();
    if (tid < 2) {
        const int qt = qb * (kSplitQ / 64) + tid;
        rec_err[tid] = 0.0f;
        rec_low[tid] = 0.0f;
        if (qt < qtiles) {
            uint32_t v = 0;
            for (int w = 0; w < 4; ++w) v = v > red[1][w] ? v : red[1][w];
            const uint32_t a = red[0][2 * tid] > red[0][2 * tid + 1] ? red[0][2 * tid] : red[0][2 * tid + 1];
            const uint32_t sb = red[2][2 * tid] > red[2][2 * tid + 1] ? red[2][2 * tid] : red[2][2 * tid + 1];
            AttnRecord rc;
            rc.amax_bits = a;
            rc.err = 5.9604645e-8f * __uint_as_float(v) * (kErrBase + kErrPerScore * __uint_as_float(sb));
            if (!(rc.err <= 3.402823466e+38f)) rc.amax_bits = 0x7f800000u;   // non-finite inputs: flagged downstream
            rec[bh * qtiles + qt] = rc;
            if (bound_slot) {
                // The exact maximum of the tensor is found here too.  Every workgroup raises a shared word to a
                // lower bound of its own exact maximum (largest stored |x| minus its error bound); a value can be
                // the tensor's exact maximum only if |x| + E reaches the largest lower bound, whichever
                // workgroups have reported so far: the workgroup that holds the maximum always sees a bound that
                // its maximum passes.  Non-finite values: they are the "maximum".
                uint32_t *wb = bound_slot + ((blockIdx.x + tid) & (kAmaxWays - 1)) * kAmaxStride;
                if (rc.amax_bits >= 0x7f800000u) {
                    atomicMax(exact_slot + ((blockIdx.x + tid) & (kAmaxWays - 1)) * kAmaxStride, rc.amax_bits);
                    non_finite = 1;
                } else {
                    const float af = __uint_as_float(a);
                    // (the factor and the 2^-23 |x| term cover the rounding of this fp32 arithmetic itself)
                    const float low = fmaxf(af - fmaf(af, 1.2e-7f, value_err(rc.err, af) * 1.001f), 0.0f);
                    rec_err[tid] = rc.err;
                    rec_low[tid] = low;
                    const uint32_t lb = __float_as_uint(low);
                    if (lb > __hip_atomic_load(wb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(wb, lb);
                }
            }
        }
    }
    if (!bound_slot) return;                                     // the kernel alone (error measurement)
    __syncthreads();
    if (non_finite) return;
    // the largest lower bound reported so far (a stale value only admits more candidates)
    uint32_t gb = __hip_atomic_load(bound_slot + lane * kAmaxStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    gb = wave_max_u32(gb);
    const float e_r = rec_err[wave >> 1];
    const float floor_v = fmaxf(__uint_as_float(gb), rec_low[wave >> 1]);
    uint32_t cand = 0;                                           // bit 16 db + i: that register is a candidate
    if (q < S) {
        const float inv = 1.0f / lrun;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int d = 32 * db + 8 * (i >> 2) + 4 * h + (i & 3);
                const float x = fabsf(o[db][i] * inv);
                if (d < dh && x + fmaf(x, 1.2e-7f, value_err(e_r, x) * 1.001f) >= floor_v) cand |= 1u << (16 * db + i);
            }
    }
    if (!__syncthreads_or(cand != 0)) return;                    // as a rule: nothing to do
    __shared__ uint64_t masks[4];
    double *redd = (double *)lds;                                // the stage memory is free now
    const double scale_d = 1.0 / sqrt((double)dh);
    uint32_t best = 0;
    for (int sl = 0; sl < 32; ++sl) {
        if (!__syncthreads_or((cand >> sl) & 1u)) continue;
        for_each_marked(((cand >> sl) & 1u) != 0, masks, [&](int k) {
            const int wk = k >> 6, rk = k & 31, hk = (k >> 5) & 1;
            const int qk = qb * kSplitQ + wk * 32 + rk;
            const int dk = 32 * (sl >> 4) + 8 * ((sl & 15) >> 2) + 4 * hk + (sl & 3);
            const float x = context_exact(qkv, S, Hd, heads, dh, scale_d, (uint32_t)((tok0 + qk) * Hd + hd * dh + dk), redd);
            const uint32_t ab = abs_bits(x);
            best = best > ab ? best : ab;
        });
    }
    if (tid == 0 && best) atomicMax(exact_slot + (blockIdx.x & (kAmaxWays - 1)) * kAmaxStride, best);
}

// The context value of one (query token, head, dim) as the fp64 evaluation defines it:
// scores in fp64 (products summed over the head dims in ascending
// order, then the 1/sqrt(dh) factor), soft-max and the weighted sum of v in fp64, rounded once.  q, k and
// v rows are read from the packed qkv tensor.  Every load is unconditional (indices clamped to valid
// ones, the query zero beyond dh): a load under a condition is awaited on its own, and a key row would
// cost sixteen memory round trips instead of one.
// (kept compact and inlined once per kernel: called as a function it needs scratch memory for the
// caller's registers and ran five times slower)
__device__ __forceinline__ float context_exact(const float *__restrict__ qkv, int S, int Hd, int heads, int dh, double scale,
                                            uint32_t el, double *red)
{
    const bool vec4 = (dh & 3) == 0 && (Hd & 3) == 0;           // whole 16-byte units, 16-byte aligned rows
    const uint32_t mrow = el / (uint32_t)Hd, col = el - mrow * (uint32_t)Hd;
    const uint32_t bi = mrow / (uint32_t)S, hd = col / (uint32_t)dh, dd = col - hd * (uint32_t)dh;
    const int64_t ld = 3 * (int64_t)Hd;
    const float *q = qkv + (int64_t)mrow * ld + hd * dh;
    const float *kb = qkv + (int64_t)bi * S * ld + Hd + hd * dh, *vb = kb + Hd + dd;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int units = dh >> 2;
    // the query row goes through LDS (64 floats behind the 12 doubles of red): every thread needs all of it.
    // Its load and the first block's key and value loads are requested together, before the barriers: the
    // evaluation is a chain of memory round trips, and this takes one out of it.
    float *qs = (float *)(red + 12);
    float4 kv[16];
    float vj = 0.0f;
    auto request = [&](int j0) {
        const int j = j0 + tid;
        const int jj = j < S ? j : S - 1;
        const float *kr = kb + (int64_t)jj * ld;
        vj = vb[(int64_t)jj * ld];
        if (vec4) {
#pragma unroll
            for (int u = 0; u < 16; ++u) kv[u] = *(const float4 *)(kr + 4 * (u < units ? u : units - 1));
        }
    };
    const float qreg = (tid < 64 && tid < dh) ? q[tid] : 0.0f;
    request(0);
    __syncthreads();                                          // an earlier call has finished with red and qs
    if (tid < 64) qs[tid] = qreg;
    __syncthreads();
    double m = -INFINITY, l = 0.0, o = 0.0;
    for (int j0 = 0; j0 < S; j0 += 256) {
        const int j = j0 + tid;
        const int jj = j < S ? j : S - 1;
        const float *kr = kb + (int64_t)jj * ld;
        if (j0) request(j0);
        // a product of two fp32 values is exact in fp64, so each fma below is the multiply and the
        // add of the plain definition, in its order (dims ascending)
        double acc = 0.0;
        if (vec4) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (u < units) {
                    const float4 qv = *(const float4 *)&qs[4 * u];
                    acc = fma((double)qv.x, (double)kv[u].x, acc);
                    acc = fma((double)qv.y, (double)kv[u].y, acc);
                    acc = fma((double)qv.z, (double)kv[u].z, acc);
                    acc = fma((double)qv.w, (double)kv[u].w, acc);
                }
            }
        } else {
            for (int d = 0; d < dh; ++d) acc = fma((double)qs[d], (double)kr[d], acc);   // odd head sizes: plain loop
        }
        const double sc = j < S ? acc * scale : -INFINITY;
        double cm = sc;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) cm = fmax(cm, __shfl_xor(cm, off, kWave));
        __syncthreads();                                      // red is free (an earlier block, an earlier call)
        if (lane == 0) red[wave] = cm;
        __syncthreads();
        const double mnew = fmax(m, fmax(fmax(red[0], red[1]), fmax(red[2], red[3])));
        const double p = exp(sc - mnew);                 // exp(-inf) = 0 for the keys beyond S
        const double corr = j0 == 0 ? 0.0 : exp(m - mnew);
        const double ps = wave_sum(p), po = wave_sum(p * (double)vj);
        if (lane == 0) { red[4 + wave] = ps; red[8 + wave] = po; }
        __syncthreads();
        l = l * corr + ((red[4] + red[5]) + (red[6] + red[7]));
        o = o * corr + ((red[8] + red[9]) + (red[10] + red[11]));
        m = mnew;
    }
    return (float)(o / l);
}

// Workgroup-uniform walk over the values a predicate marks among 256 consecutive candidates: every thread
// passes its own flag, and `visit(k)` runs, in all threads, for every marked k = 0..255 in ascending order.
template <typename F>
__device__ __forceinline__ void for_each_marked(bool mine, uint64_t *masks, F visit)
{
    const uint64_t b = __ballot(mine);
    __syncthreads();                                          // masks is free
    if ((threadIdx.x & 63) == 0) masks[threadIdx.x >> 6] = b;
    __syncthreads();
    for (int w = 0; w < 4; ++w) {
        uint64_t mask = masks[w];
        while (mask) {
            const int src = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            visit(w * 64 + src);
        }
    }
}

// Exact absolute maximum of the context.  The largest stored |x| (A) and the largest E over all records come
// from two atomically combined words the first kernel filled; a value can be the exact maximum only if
// |x| + E_record >= A - E_max.  A thread tests one record (a workgroup per 256 records: one memory round
// trip for the whole grid, where a workgroup per record took six waves of workgroups); for the records that
// pass (as a rule one in the whole tensor) the workgroup rescans the record's 64 x dh values and
// re-evaluates those that pass the test.  The value that holds A passes, so the word `exact` ends up with
// the exact maximum (it starts at zero: cleared by the chain's first kernel).
__global__ __launch_bounds__(256) void attention_absmax_exact_kernel(const float *__restrict__ qkv,
                                                                     const float *__restrict__ ctx,
                                                                     const AttnRecord *__restrict__ rec, int nrec,
                                                                     const uint32_t *__restrict__ amax_slot,
                                                                     const uint32_t *__restrict__ err_slot,
                                                                     int S, int Hd, int heads, int dh, double scale,
                                                                     uint32_t *__restrict__ exact)
{
    __shared__ __attribute__((aligned(16))) double red[12 + 32];
    __shared__ uint64_t masks_rec[4], masks[4];
    __shared__ float err_s;
    const int tid = threadIdx.x;
    const int rid = blockIdx.x * 256 + tid;
    const AttnRecord mine = rec[rid < nrec ? rid : nrec - 1];
    const uint32_t a = reduce_ways(amax_slot);
    const float e = __uint_as_float(reduce_ways(err_slot));
    if (a >= 0x7f800000u) {                                   // NaN / Inf in the tensor: it is the "maximum"
        if (blockIdx.x == 0 && tid == 0) atomicMax(exact, a);
        return;
    }
    const float A = __uint_as_float(a);
    const float floor_v = A - value_err(e, A);                // values below this cannot be the maximum
    const float mine_max = __uint_as_float(mine.amax_bits);
    const bool holds = rid < nrec && mine_max + value_err(mine.err, mine_max) >= floor_v;
    const int qtiles = (S + 63) / 64;
    uint32_t best = 0;
    for_each_marked(holds, masks_rec, [&](int kr) {
        const int r = blockIdx.x * 256 + kr;
        __syncthreads();                                      // err_s is free
        if (tid == kr) err_s = mine.err;                      // the record is in that thread's registers
        __syncthreads();
        const float r_err = err_s;
        const int bh = r / qtiles, qt = r % qtiles;
        const int bi = bh / heads, hd = bh % heads;
        const int64_t tok0 = (int64_t)bi * S;
        const int nq = S - qt * 64 < 64 ? S - qt * 64 : 64;
        const int n_el = nq * dh;
        // the record's values, sixteen per thread requested together (indices clamped, the surplus masked
        // below); candidates are then taken 256 values at a time and re-evaluated one by one by the workgroup
        float xs[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int idx = k * 256 + tid < n_el ? k * 256 + tid : 0;
            xs[k] = fabsf(ctx[(tok0 + qt * 64 + idx / dh) * Hd + hd * dh + idx % dh]);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int base = k * 256;
            if (base < n_el) {
                const bool cand = base + tid < n_el && xs[k] + value_err(r_err, xs[k]) >= floor_v;
                for_each_marked(cand, masks, [&](int kv) {
                    const int cidx = base + kv;
                    const int qq = qt * 64 + cidx / dh, d = cidx % dh;
                    const float x = context_exact(qkv, S, Hd, heads, dh, scale, (uint32_t)((tok0 + qq) * Hd + hd * dh + d), red);
                    const uint32_t ab = abs_bits(x);
                    best = best > ab ? best : ab;
                });
            }
        }
    });
    if (tid == 0 && best) atomicMax(exact + (blockIdx.x & (kAmaxWays - 1)) * kAmaxStride, best);
}

// The int8 codes of the context under the tensor's exact scale: one workgroup per (batch element, head).
// It streams over the head's slice of the approximate context, 256 units a pass: a thread maps 16
// consecutive values of a token row (one 16-byte store; WIDE: head size and row length are multiples of
// 16) or a single value.  A value whose interval [x - E, x + E] maps to two codes gets a provisional code
// and goes on the workgroup's list in LDS (token * dh + dim within the head; the list has room for every
// value of a pass).  After each pass the workgroup re-evaluates the listed values in fp64 and overwrites
// their codes.  A re-evaluation needs all keys of its head (S x dh floats): read from global memory per
// value, that traffic (and the sixteen-byte pieces of 256 different rows each load instruction asks
// for) bounds the whole step.  KLDS (S <= 256, head size a multiple of 4): the workgroup copies the
// head's keys into LDS once, with coalesced loads, and each of its waves re-evaluates one listed value
// at a time from there: lane l holds keys l, l + 64, ..., a row of LDS each (rows padded by 16 bytes,
// so the lanes' 16-byte reads do not collide), the query row is broadcast from LDS, and only the value
// column (one float per key) comes from global memory.  Otherwise the workgroup-wide evaluation above
// is used, one value after the other.
constexpr int kKeysLds = 256;            // keys a workgroup can hold
constexpr int kKeyRow = kDh + 4;         // floats per key row in LDS (one 16-byte pad)

// true if the approximate value x with error bound err does not settle its code
// (The exact value y lies in [x - e, x + e]; its code is clamp(rne(fl(y * inv))) with fl(y * inv) within
// e * inv + 2^-23 |t| of t = fl(x * inv).  The two codes can differ only if that interval reaches the rounding
// boundary next to t, i.e. |t - rne(t)| + e * inv + 2^-23 |t| >= 1/2; the margins below are a little wider.)
__device__ __forceinline__ bool code_uncertain(float x, float err, float inv)
{
    const float t = x * inv;
    const float reach = fmaf(value_err(err, x) * 1.001f, inv, 2.4e-7f * fabsf(t)) + 1.0e-30f;
    return !(fabsf(t - rintf(t)) + reach < 0.5f);                  // also true for a non-finite bound
}

template <bool WIDE, bool KLDS>
__global__ __launch_bounds__(256, KLDS ? 2 : 3) void quantize_attention_certify_kernel(
    const float *__restrict__ qkv, const float *__restrict__ ctx, const AttnRecord *__restrict__ rec, int S, int Hd,
    int heads, int dh, double scale, const uint32_t *__restrict__ exact, int8_t *xq, int64_t ldq,
    float *__restrict__ scale_out, uint32_t *__restrict__ flag, uint32_t *__restrict__ unsure_total)
{
    constexpr int PER = WIDE ? 16 : 1;                            // values of a unit
    constexpr int NPRE = WIDE && KLDS ? 4 : 1;                    // passes whose loads are requested together
    constexpr uint32_t kList = 4096;                              // list entries served per round
    using Entry = std::conditional_t<KLDS, uint16_t, uint32_t>;   // KLDS: S * dh <= 256 * 64
    __shared__ Entry todo[kList];
    __shared__ uint32_t n_todo, more;
    __shared__ __attribute__((aligned(16))) double red[KLDS ? 2 : 12 + 32];
    __shared__ __attribute__((aligned(16))) float ks[KLDS ? kKeysLds * kKeyRow : 4];
    __shared__ __attribute__((aligned(16))) float qs[KLDS ? 4 * kDh : 4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t bh = blockIdx.x, bi = bh / (uint32_t)heads, hd = bh - bi * (uint32_t)heads;
    const uint32_t qtiles = (uint32_t)(S + 63) / 64u;
    const uint32_t tok0 = bi * (uint32_t)S;
    const int64_t ld = 3 * (int64_t)Hd;
    const float *qb = qkv + (int64_t)tok0 * ld + hd * dh, *kb = qb + Hd, *vb = kb + Hd;
    // units per token: 16-value groups of the head, or single columns (the last head also clears the pad
    // columns [Hd, ldq) of its tokens)
    const uint32_t upt = WIDE ? (uint32_t)dh / 16u : (uint32_t)dh + (hd + 1u == (uint32_t)heads ? (uint32_t)(ldq - Hd) : 0u);
    const uint32_t units = (uint32_t)S * upt;
    // a group of passes: unit `first + 256 i + tid` is this thread's in pass i (clamped to a valid one for
    // the loads; the surplus is masked where it is used)
    float4 v[NPRE][WIDE ? 4 : 1];
    auto request = [&](uint32_t first) {
#pragma unroll
        for (int i = 0; i < NPRE; ++i) {
            const uint32_t u = first + 256u * i + (uint32_t)tid, uc = u < units ? u : units - 1u;
            const uint32_t t = uc / upt, part = uc - t * upt;
            if (WIDE) {
                const float4 *p = (const float4 *)(ctx + (int64_t)(tok0 + t) * Hd + hd * (uint32_t)dh + part * 16u);
#pragma unroll
                for (int j = 0; j < 4; ++j) v[i][j] = p[j];
            } else {
                const uint32_t col = hd * (uint32_t)dh + part;
                v[i][0].x = ctx[(int64_t)(tok0 + t) * Hd + (col < (uint32_t)Hd ? col : (uint32_t)Hd - 1u)];
            }
        }
    };
    request(0);
    if (KLDS) {
        // the head's keys, eight 16-byte pieces per thread in flight (the first barrier below orders them
        // before any read)
        const int cpr = dh >> 2, total = S * cpr;
        for (int c0 = 0; c0 < total; c0 += 256 * 8) {
            float4 t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = c0 + i * 256 + tid;
                const int cc = c < total ? c : total - 1;
                t[i] = *(const float4 *)(kb + (int64_t)(cc / cpr) * ld + 4 * (cc % cpr));
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = c0 + i * 256 + tid;
                if (c < total) *(float4 *)&ks[(c / cpr) * kKeyRow + 4 * (c % cpr)] = t[i];
            }
        }
    }
    float sc_f;
    bool bad;
    const float inv = scale_from_bits(reduce_ways(exact), nullptr, &sc_f, &bad);
    if (blockIdx.x == 0 && threadIdx.x == 0) publish(sc_f, bad, scale_out, nullptr, flag);
    uint32_t met = 0;
    // the loop bounds are the same in every thread of the workgroup (barriers inside)
    for (uint32_t first = 0; first < units; first += 256u * NPRE) {
        if (first) request(first);
        // provisional codes; pend[i]: which of the unit's values do not settle their code
        uint32_t pend[NPRE], at[NPRE];
#pragma unroll
        for (int i = 0; i < NPRE; ++i) {
            const uint32_t u = first + 256u * i + (uint32_t)tid;
            pend[i] = 0;
            at[i] = 0;
            if (u < units) {
                const uint32_t t = u / upt, part = u - t * upt;
                const uint32_t m = tok0 + t;
                const float err = rec[bh * qtiles + t / 64u].err;
                if (WIDE) {
                    const uint32_t col = hd * (uint32_t)dh + part * 16u;
                    uint32_t w[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float4 x = v[i][j];
                        w[j] = quant1(x.x, inv) | quant1(x.y, inv) << 8 | quant1(x.z, inv) << 16 | quant1(x.w, inv) << 24;
                        pend[i] |= (code_uncertain(x.x, err, inv) ? 1u : 0u) << (4 * j) | (code_uncertain(x.y, err, inv) ? 2u : 0u) << (4 * j) |
                                   (code_uncertain(x.z, err, inv) ? 4u : 0u) << (4 * j) | (code_uncertain(x.w, err, inv) ? 8u : 0u) << (4 * j);
                    }
                    *(uint4 *)(xq + (int64_t)m * ldq + col) = make_uint4(w[0], w[1], w[2], w[3]);
                    at[i] = t * (uint32_t)dh + part * 16u;
                } else {
                    const uint32_t col = hd * (uint32_t)dh + part;
                    uint32_t code = 0;
                    if (col < (uint32_t)Hd) {
                        code = quant1(v[i][0].x, inv);
                        pend[i] = code_uncertain(v[i][0].x, err, inv) ? 1u : 0u;
                    }
                    xq[(int64_t)m * ldq + col] = (int8_t)code;   // pad columns: zero
                    at[i] = t * (uint32_t)dh + part;
                }
                if (bad) pend[i] = 0;
            }
        }
        // rounds: the pending values go on the list (as many as it holds), the workgroup serves the list
        bool again;
        do {
            __syncthreads();                                      // the list of the round before has been served
            if (tid == 0) { n_todo = 0; more = 0; }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NPRE; ++i) {
                while (pend[i]) {
                    const uint32_t slot = atomicAdd(&n_todo, 1u);
                    if (slot >= kList) { more = 1; break; }
                    const int e = __ffs((int)pend[i]) - 1;
                    pend[i] &= pend[i] - 1;
                    todo[slot] = (Entry)(at[i] + (uint32_t)e);
                }
            }
            __syncthreads();                                      // list complete, provisional codes stored
            const uint32_t n = n_todo < kList ? n_todo : kList;
            again = more != 0;
            met += n;
            if (KLDS) {
                const int cpr = dh >> 2, nk = (S + 63) >> 6;      // 16-byte pieces per row, keys per lane
                for (uint32_t k0 = 0; k0 < n; k0 += 4u) {         // a value per wave
                    const uint32_t k = k0 + (uint32_t)wave;
                    const bool active = k < n;
                    const uint32_t e = todo[active ? k : k0];
                    const uint32_t t = e / (uint32_t)dh, d = e - t * (uint32_t)dh;
                    float vj[4];
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        const int j = lane + 64 * kk;
                        vj[kk] = vb[(int64_t)(j < S ? j : S - 1) * ld + d];
                    }
                    qs[wave * kDh + lane] = lane < dh ? qb[(int64_t)t * ld + lane] : 0.0f;
                    __syncthreads();
                    if (active) {
                        // a product of two fp32 values is exact in fp64, so each fma is the multiply and the
                        // add of the plain definition, dims in ascending order
                        double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                        for (int u4 = 0; u4 < kDh / 4; ++u4) {
                            if (u4 < cpr) {
                                const float4 qv = *(const float4 *)&qs[wave * kDh + 4 * u4];
#pragma unroll
                                for (int kk = 0; kk < 4; ++kk) {
                                    if (kk < nk) {
                                        const int j = lane + 64 * kk;
                                        const float4 kv = *(const float4 *)&ks[(j < S ? j : S - 1) * kKeyRow + 4 * u4];
                                        acc[kk] = fma((double)qv.x, (double)kv.x, acc[kk]);
                                        acc[kk] = fma((double)qv.y, (double)kv.y, acc[kk]);
                                        acc[kk] = fma((double)qv.z, (double)kv.z, acc[kk]);
                                        acc[kk] = fma((double)qv.w, (double)kv.w, acc[kk]);
                                    }
                                }
                            }
                        }
                        double sc[4], mx = -INFINITY;
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) {
                            sc[kk] = lane + 64 * kk < S ? acc[kk] * scale : -INFINITY;
                            mx = fmax(mx, sc[kk]);
                        }
#pragma unroll
                        for (int off = 32; off > 0; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off, kWave));
                        double l = 0.0, o = 0.0;
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) {
                            const double pr = exp(sc[kk] - mx);      // exp(-inf) = 0 for the keys beyond S
                            l += pr;
                            o += pr * (double)vj[kk];
                        }
                        l = wave_sum(l);
                        o = wave_sum(o);
                        if (lane == 0) xq[(int64_t)(tok0 + t) * ldq + hd * dh + d] = (int8_t)quant1((float)(o / l), inv);
                    }
                    __syncthreads();                              // qs is free
                }
            } else {
                for (uint32_t k = 0; k < n; ++k) {
                    const uint32_t e = (uint32_t)__builtin_amdgcn_readfirstlane((int)todo[k]);
                    const uint32_t t = e / (uint32_t)dh, d = e - t * (uint32_t)dh;
                    const float x = context_exact(qkv, S, Hd, heads, dh, scale, (tok0 + t) * (uint32_t)Hd + hd * (uint32_t)dh + d, red);
                    if (tid == 0) xq[(int64_t)(tok0 + t) * ldq + hd * dh + d] = (int8_t)quant1(x, inv);
                }
            }
        } while (again);
    }
    if (tid == 0 && unsure_total && met) atomicAdd(unsure_total, met);
}

static bool attn_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t attention_records_bytes(int32_t B, int32_t S, int32_t heads)
{
    return align_up((size_t)B * heads * ((S + 63) / 64) * sizeof(AttnRecord), 256);
}

// Kernel 1: the bf16-split form when head dims come in whole units of 8 floats at 16-byte aligned addresses,
// else the fp32 form.  Both fill the same records (one per 64 queries of a head).
static hipError_t launch_attention_approx(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads, float *ctx,
                                          AttnRecord *rec, uint32_t *amax_slot, uint32_t *err_slot, uint32_t *exact_slot,
                                          hipStream_t st)
{
    const int dh = Hd / heads;
    const float scale = (float)(1.0 / sqrt((double)dh));
    if ((dh & 7) == 0 && (Hd & 3) == 0) {
        const int64_t grid = (int64_t)B * heads * ((S + kSplitQ - 1) / kSplitQ);
        const int per_xcd = (int)((grid + 7) / 8);
        return launch_k(EGERIA_KERNEL_ATTENTION, attention_split_kernel, dim3((unsigned)(per_xcd * 8)), dim3(256), 0, st,
                        qkv, (int)B, (int)S, (int)Hd, (int)heads, dh, scale, ctx, rec, (int)grid, per_xcd, amax_slot, exact_slot);
    }
    const int64_t grid = (int64_t)B * heads * ((S + 63) / 64);
    const int per_xcd = (int)((grid + 7) / 8);
    return launch_k(EGERIA_KERNEL_ATTENTION, attention_fast_kernel, dim3((unsigned)(per_xcd * 8)), dim3(256), 0, st, qkv,
                    (int)B, (int)S, (int)Hd, (int)heads, dh, scale, ctx, rec, (int)grid, per_xcd, amax_slot, err_slot);
}

// Kernel 1 alone (benchmark instrumentation: its error against the fp64 kernel): approximate context and the
// records {largest |x| as a bit pattern, error bound E}, B * heads * ceil(S / 64) of them.
hipError_t launch_attention_fast(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads, float *ctx,
                                 void *records, hipStream_t st)
{
    const int dh = Hd / heads;
    const int64_t grid = (int64_t)B * heads * ((S + 63) / 64);
    if (grid <= 0) return hipSuccess;
    if (dh > kDh || grid > 0x7ffffff0LL) return hipErrorInvalidValue;
    if (!attn_aligned16(qkv) || !attn_aligned16(ctx) || !attn_aligned16(records)) return hipErrorInvalidValue;
    return launch_attention_approx(qkv, B, S, Hd, heads, ctx, (AttnRecord *)records, nullptr, nullptr, nullptr, st);
}

hipError_t launch_attention_certified(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads, float *ctx,
                                      void *records, uint32_t *amax_slot, uint32_t *err_slot, uint32_t *exact_slot, int8_t *xq, int64_t ldq, float *scale_out,
                                      uint32_t *flag, uint32_t *unsure_total, hipStream_t st)
{
    const int dh = Hd / heads;
    const int qtiles = (S + 63) / 64;
    const int64_t grid = (int64_t)B * heads * qtiles;
    const int64_t M = (int64_t)B * S;
    if (grid <= 0) return hipSuccess;
    // what the kernels assume: heads of at most 64 dims, 32-bit indices of the context's values, rows that
    // 16-byte vector accesses may touch when the head size allows them
    if (dh > kDh || grid > 0x7ffffff0LL || M * Hd >= (1LL << 32) || ldq < Hd) return hipErrorInvalidValue;
    if (!attn_aligned16(qkv) || !attn_aligned16(ctx) || !attn_aligned16(xq) || !attn_aligned16(records)) return hipErrorInvalidValue;
    AttnRecord *rec = (AttnRecord *)records;
    const double scale = 1.0 / sqrt((double)dh);
    hipError_t e = launch_attention_approx(qkv, B, S, Hd, heads, ctx, rec, amax_slot, err_slot, exact_slot, st);
    if (e != hipSuccess) return e;
    const int nrec = (int)grid;
    // (the bf16-split kernel settles the exact maximum itself; the fp32 kernel leaves it to a launch of its own)
    if (!((dh & 7) == 0 && (Hd & 3) == 0)) e = launch_k(EGERIA_KERNEL_NONE, attention_absmax_exact_kernel, dim3((unsigned)((nrec + 255) / 256)), dim3(256), 0, st, qkv,
                 (const float *)ctx, (const AttnRecord *)rec, nrec, (const uint32_t *)amax_slot, (const uint32_t *)err_slot, (int)S,
                 (int)Hd, (int)heads, dh, scale, exact_slot);
    if (e != hipSuccess) return e;
    const bool wide = (dh & 15) == 0 && (Hd & 15) == 0 && ldq == Hd;
    if ((int64_t)S * (dh + (ldq - Hd)) >= (1LL << 31)) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((int64_t)B * heads);
    const bool klds = S <= kKeysLds && (dh & 3) == 0 && (Hd & 3) == 0;
    auto go = [&](auto kernel) {
        return launch_k(EGERIA_KERNEL_QUANTIZE, kernel, dim3(blocks), dim3(256), 0, st, qkv, (const float *)ctx,
                        (const AttnRecord *)rec, (int)S, (int)Hd, (int)heads, dh, scale, (const uint32_t *)exact_slot, xq,
                        ldq, scale_out, flag, unsure_total);
    };
    if (wide) return klds ? go(quantize_attention_certify_kernel<true, true>) : go(quantize_attention_certify_kernel<true, false>);
    return klds ? go(quantize_attention_certify_kernel<false, true>) : go(quantize_attention_certify_kernel<false, false>);
}

hipError_t launch_attention(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads,
                            float *ctx, uint32_t *absmax_out, hipStream_t st)
{
    const int dh = Hd / heads;
    constexpr int QB = 1;               // one 16-query block per wave: ~120 VGPRs, several waves per SIMD
    const int qtiles = (S + 64 * QB - 1) / (64 * QB);
    const int64_t grid = (int64_t)B * heads * qtiles;
    if (grid <= 0) return hipSuccess;
    if (dh > kDh || grid > 0x7ffffff0LL) return hipErrorInvalidValue;
    const int per_xcd = (int)((grid + 7) / 8);
    return launch_k(EGERIA_KERNEL_ATTENTION, attention_kernel<QB>, dim3((unsigned)(per_xcd * 8)), dim3(256), 0, st, qkv,
                    (int)B, (int)S, (int)Hd, (int)heads, dh, 1.0 / sqrt((double)dh), ctx, absmax_out, (int)grid, per_xcd);
}

}  // namespace egeria
