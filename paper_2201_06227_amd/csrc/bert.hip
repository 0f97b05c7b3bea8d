// Floating-point glue of a Transformer encoder layer of the reference model:
// under dynamic quantisation (Section 5 of the paper) only the linear layers
// are int8; self-attention and layer norm read and write fp32 tensors.
#include "common.hpp"

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
        double v[NV][4];
        double s = 0.0;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            v[i][0] = (double)xv[i].x + (double)rv[i].x;
            v[i][1] = (double)xv[i].y + (double)rv[i].y;
            v[i][2] = (double)xv[i].z + (double)rv[i].z;
            v[i][3] = (double)xv[i].w + (double)rv[i].w;
            s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
        }
        const double mean = wave_sum(s) / (double)H;
        double q = 0.0;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (lane + 64 * i < nv) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[i][e] -= mean;
                    q += v[i][e] * v[i][e];
                }
            }
        const double var = wave_sum(q) / (double)H;
        const double rstd = 1.0 / sqrt(var + eps);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = lane + 64 * i;
            if (c < nv) {
                const float4 gm = gmv[i], bt = btv[i];
                float4 o;
                o.x = (float)(v[i][0] * rstd * (double)gm.x + (double)bt.x);
                o.y = (float)(v[i][1] * rstd * (double)gm.y + (double)bt.y);
                o.z = (float)(v[i][2] * rstd * (double)gm.z + (double)bt.z);
                o.w = (float)(v[i][3] * rstd * (double)gm.w + (double)bt.w);
                reinterpret_cast<float4 *>(y + row * H)[c] = o;
                const uint32_t a0 = abs_bits(o.x), a1 = abs_bits(o.y), a2 = abs_bits(o.z), a3 = abs_bits(o.w);
                const uint32_t m01 = a0 > a1 ? a0 : a1, m23 = a2 > a3 ? a2 : a3;
                const uint32_t m = m01 > m23 ? m01 : m23;
                amax = amax > m ? amax : m;
            }
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
                qr[qb][4 * u + e] = (q < S && d < dh) ? (double)qv[4 * u + e] * scale : 0.0;
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
                    if (key >= S) st[kb][qb][r] = -INFINITY;
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
