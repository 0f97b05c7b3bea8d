// Shared declarations of the gfx950 kernels behind include/egeria.h.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/egeria.h"
#include "../../include/egeria_profile.h"

namespace egeria {

constexpr int kWave = 64;

// ---- workspace header -------------------------------------------------------
// word 0              : flag word, kFlagMagic | bits (bit 0: a quantiser met NaN/Inf);
//                       only thread 0 of block 0 of a quantise kernel touches it
// words 16 .. 16+S    : one absmax slot per quantise point whose tensor is produced
//                       by a kernel of the chain (bit pattern of a non-negative
//                       fp32, combined with integer atomicMax)
// next S words        : fp32 scales, one per quantise point
// next kAbsPartials   : per-workgroup maxima of the chain's input tensor (plain
//                       stores by the absmax kernel, reduced by the consumer, so
//                       no word of the header ever needs a separate reset launch)
constexpr uint32_t kFlagMagic = 0xE6E71A00u;
constexpr uint32_t kFlagNonFinite = 1u;
constexpr int kHeaderFixedWords = 16;
// word 4 of the header: how many attention-context values the certified quantiser re-evaluated in fp64
// during the last reference forward (cleared by the chain's first kernel; read by benchmarks and tests)
constexpr int kUnsureWord = 4;
constexpr int kAbsPartials = 512;
// An atomically combined maximum is spread over kAmaxWays words, kAmaxStride
// words apart (workgroup id modulo the ways picks the word): thousands of
// workgroups finishing together would otherwise serialise on one address.
constexpr int kAmaxWays = 64;
constexpr int kAmaxStride = 64;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- per-device host state -------------------------------------------------
// Function attributes, symbol addresses and streams belong to one device each:
// whatever the library sets up lazily is kept per device, indexed by the device
// that is current at the call.
constexpr int kMaxDevices = 16;
inline int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}
// Compute units of the current device (256 on MI355X), queried once per device;
// the tile and chunk choosers size their grids by it.
int compute_units();
inline size_t header_bytes(int slots)
{
    return align_up(4 * (size_t)(kHeaderFixedWords + slots * (kAmaxWays * kAmaxStride + 1) + kAbsPartials), 256);
}
inline uint32_t *ws_flag(void *ws) { return (uint32_t *)ws; }
inline uint32_t *ws_absmax(void *ws, int slot)
{
    return (uint32_t *)ws + kHeaderFixedWords + (size_t)slot * kAmaxWays * kAmaxStride;
}
inline float *ws_scale(void *ws, int slots, int slot)
{
    return (float *)ws + kHeaderFixedWords + (size_t)slots * kAmaxWays * kAmaxStride + slot;
}
inline uint32_t *ws_partials(void *ws, int slots)
{
    return (uint32_t *)ws + kHeaderFixedWords + (size_t)slots * (kAmaxWays * kAmaxStride + 1);
}

// ---- optional event timing of one kernel class (egeria_profile_begin / egeria_profile_end) ----
struct ProfileState {
    int cls = 0;
    hipEvent_t *start = nullptr;
    hipEvent_t *stop = nullptr;
    int n = 0;
    int count = 0;
};
extern ProfileState g_profile;

// Every kernel of the library is launched through here.  When timing of class
// `cls` is armed, the launch carries a start/stop event pair that receives the
// dispatch's own begin and end timestamps.
template <typename K, typename... Args>
inline hipError_t launch_k(int cls, K kernel, dim3 grid, dim3 block, size_t smem, hipStream_t st, Args... args)
{
    if (cls != 0 && g_profile.cls == cls && g_profile.count < g_profile.n) {
        const int i = g_profile.count++;
        hipExtLaunchKernelGGL(kernel, grid, block, smem, st, g_profile.start[i], g_profile.stop[i], 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, smem, st, args...);
    }
    return hipGetLastError();
}

// ---- launchers (each enqueues on `st` and returns hipGetLastError()) --------
// Per-workgroup maxima of |x| over n values into partials[0 .. absmax_blocks(n))
// (plain stores).  Block 0 also clears the ways of `n_reset` atomic slots that
// start at `reset` (the quantise points of the chain that follows).
int absmax_blocks(int64_t n, egeria_dtype dt);
hipError_t launch_absmax(const void *x, egeria_dtype dt, int64_t n, uint32_t *partials, uint32_t *reset,
                         int n_reset, hipStream_t st);

// Quantise a [rows, cols] matrix into int8 [rows, ldq] (ldq >= cols, multiple of
// 16, pad bytes zero) with the scale derived from max(slot[0 .. n_slot)) (or
// *fixed_scale).  Writes the scale to scale_out and, if non-null, scale_out2.
hipError_t launch_quantize_rows(const void *x, egeria_dtype dt, int64_t rows, int64_t cols,
                                int64_t ldq, const uint32_t *slot, int n_slot, int slot_stride,
                                const float *fixed_scale,
                                int8_t *q, float *scale_out, float *scale_out2, uint32_t *flag,
                                hipStream_t st);

// Quantise [n, c, hw] (channel-major) into int8 [n, hw, cp] (channel-last, cp =
// padded c, pad zero).
hipError_t launch_quantize_nchw(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t hw,
                                int64_t cp, const uint32_t *slot, int n_slot, int slot_stride,
                                const float *fixed_scale,
                                int8_t *q, float *scale_out, float *scale_out2, uint32_t *flag,
                                hipStream_t st);

// Fused GELU + quantise of a linear layer's pre-activations v [rows, cols]:
// codes of gelu(v) under the per-tensor scale of gelu(v), without storing
// gelu(v).  vmax holds max(v, 0) over the tensor (bit pattern); exact_absmax is
// a second word that launch_gelu_absmax_exact fills when vmax is too small for
// the shortcut absmax = gelu(vmax).
hipError_t launch_gelu_absmax_exact(const float *v, int64_t n, const uint32_t *vmax, uint32_t *exact_absmax,
                                    hipStream_t st);
hipError_t launch_quantize_gelu_rows(const float *v, int64_t rows, int64_t cols, int64_t ldq,
                                     const uint32_t *vmax, const uint32_t *exact_absmax, int8_t *q,
                                     float *scale_out, uint32_t *flag, hipStream_t st);
// y = gelu(v) evaluated in fp64, rounded once (observation points only).
hipError_t launch_gelu_exact(const float *v, int64_t n, float *y, hipStream_t st);

// One-launch quantisation of a small tensor [nimg, c, hw] -> int8 [nimg, hw, cp]
// (at most kSmallTensor values, dynamic scale only).
constexpr int64_t kSmallTensor = 16384;
hipError_t launch_quantize_small(const void *x, egeria_dtype dt, int nimg, int c, int hw, int cp, int8_t *q,
                                 float *scale_out, uint32_t *flag, hipStream_t st);

// A batch of weight tensors [o, c, hw] -> int8 [o, hw, cp] quantised together
// (dynamic per-tensor scales).  The table travels as a kernel argument.
struct WeightJob {
    const void *x;
    int8_t *q;
    float *scale;
    int32_t o, c, hw, cp;
    int32_t bf16;
    int32_t first_block;    // first workgroup of this tensor within the launch
    int32_t nblk;           // workgroups of this tensor (<= kAbsPartials)
    int32_t epb;            // input values per workgroup (multiple of 8)
    int32_t upb;            // 16-byte output units per workgroup
    int32_t per_channel;    // one scale per output channel: a wave per channel, nblk = ceil(o / 4)
};
constexpr int kWeightBatch = 32;
struct WeightBatch {
    WeightJob job[kWeightBatch];
    int32_t n;
};
// The first pass over an unrelated tensor (the mini-batch) that rides along in the snapshot's first
// launch.  q == nullptr: nblk = absmax_blocks(n, dt) extra workgroups doing what launch_absmax
// would.  q != nullptr (nblk = 1): what launch_quantize_small does for a [rows, cols] matrix.
struct InputMaxJob {
    const void *x;
    int64_t n;
    uint32_t *partials;
    uint32_t *reset;
    int32_t n_reset;
    int32_t bf16;
    int32_t nblk;
    int8_t *q;
    float *scale_out;
    uint32_t *flag;
    int32_t rows, cols, cp;
};
// The map to codes of that tensor, riding along in the snapshot's second launch (two-launch
// snapshots only): kind 1 = rows [rows, cols] -> [rows, ldq]; kind 2 = fp32 planes [rows = n,
// cols = c, hw] -> [n, hw, ldq = cp] with hw % 4 == 0.  slot: the n_slot maxima the first launch
// stored.  nblk extra workgroups.
struct InputQuantJob {
    int32_t kind;
    const void *x;
    int32_t bf16;
    int64_t rows, cols, hw, ldq;
    const uint32_t *slot;
    int32_t n_slot;
    int8_t *q;
    float *scale_out;
    uint32_t *flag;
    int32_t nblk;
};
// one_launch: every job has nblk == 1.  partials: total_blocks words.  extra, xq: nullable; xq is
// taken only together with extra and only by a two-launch snapshot.
hipError_t launch_quantize_weights(const WeightBatch &b, int total_blocks, bool one_launch, uint32_t *partials,
                                   uint32_t *flag, hipStream_t st, const InputMaxJob *extra, const InputQuantJob *xq);
// The same for jobs with one scale per output channel (job.scale is [o]); four channels per workgroup.
hipError_t launch_quantize_weights_pc(const WeightBatch &b, int total_blocks, uint32_t *flag, hipStream_t st);

hipError_t launch_dequantize(const int8_t *q, const float *scale, int64_t n, float *x, hipStream_t st);

// Reference precisions float16 (et = 1) and float32 (et = 2): [n, c, hw] of type dt ->
// [n, hw, cpe] of the reference precision, channels rounded to nearest even and padded with
// zeros to cpe elements (a whole number of 16-byte units).  hw = 1: the rows of a matrix.
// `one` (nullable) receives 1.0f: the scale the GEMM epilogue multiplies float sums by.
hipError_t launch_cast_chlast(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t hw, int64_t cpe, int et,
                              void *out, float *one, hipStream_t st);

// Affine uint8 activation codes (stored as q - 128): the extrema of n values as per-workgroup partial
// results (affine_partial_bytes() bytes of scratch hold them), then the codes of [n, c, hw] channel planes
// (hw = 1: matrix rows) as [n, hw, cp] bytes with zero pad channels; every workgroup reduces the nb =
// minmax_blocks(...) partial results to the scale and the zero point, which workgroup 0 stores.
// store_offset: 128 for the GEMM operand form, 0 for plain uint8 codes.
int minmax_blocks(int64_t n);
size_t affine_partial_bytes();
hipError_t launch_minmax(const void *x, egeria_dtype dt, int64_t n, uint32_t *partials, hipStream_t st);
hipError_t launch_quantize_affine(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t hw, int64_t cp,
                                  const uint32_t *partials, int nb, int store_offset, void *q, float *scale_out,
                                  int32_t *zp_out, uint32_t *flag, hipStream_t st);
// Sums of the int8 weight codes [out, taps, cp] per output channel: int32 [out] for taps = 1, and for a 3x3
// kernel (taps = 9) int32 [16, out], class c leaving out the window positions outside the image for a pixel
// in the first row (c & 1), last row (c & 2), first column (c & 4), last column (c & 8).
hipError_t launch_colsum(const int8_t *w_q, int32_t out, int32_t taps, int32_t cp, int32_t *colsum, hipStream_t st);

// int8 GEMM / implicit-GEMM convolution with fused dequantising epilogue.
struct GemmArgs {
    const int8_t *a;        // activations: [M, lda] (linear, 1x1 conv) or [B, H, W, cp] (3x3 conv)
    const int8_t *w;        // weights [N, kp]
    int64_t M;
    int32_t N;
    int32_t kp;             // padded reduction length in bytes (multiple of 16)
    int64_t lda;            // row stride of `a` in bytes (linear mode)
    int64_t a_bytes;        // extent of `a` in bytes (< 2^31)
    int64_t w_bytes;        // extent of `w` in bytes (< 2^31)
    int32_t conv3x3;        // 0: rows of `a` are contiguous; 1: 3x3 window gather, zero padding 1
    int32_t H, W, cp;       // image height, width and padded channels (conv3x3 mode)
    const float *sx;        // 1 fp32: scale of the activations
    const float *sw;        // scale of the weights: 1 fp32, or fp32 [N] when sw_per_n
    int32_t sw_per_n;
    const float *bias;      // [N] or null
    int32_t act;            // 0 none, 1 ReLU
    const int8_t *res_q;    // optional residual as int8 [M, res_ld] with scale *res_scale
    const float *res_scale;
    int64_t res_ld;
    float *y;               // fp32 out [M, ldy]
    int64_t ldy;
    int32_t *acc_out;       // optional raw accumulators [M, N]
    uint32_t *absmax_out;   // optional: atomicMax of |y| (bit pattern)
    int32_t amax_pos;       // 1: track max(y, 0) instead of |y| (input of the fused GELU quantiser)
    // optional: int8 codes of y under the static scale *q_scale, [M, q_ld] with zero pad
    // columns (the next layer's input); y may then be null
    int8_t *q_out;
    int64_t q_ld;
    const float *q_scale;
    // element type of a and w: 0 int8, 1 float16, 2 float32 (the float types: kp, lda, cp, a_bytes
    // and w_bytes stay in bytes; sx and sw point at 1.0f; res_q holds values of the same type,
    // res_ld in elements, res_scale unused; acc_out receives the fp32 sums' bit patterns; no q_out,
    // no absmax_out)
    int32_t et;
    // affine activation codes (int8 operands only): a holds q - 128; *zp_in is the zero point of a, colsum
    // the weight-code sums of launch_colsum; the accumulator becomes acc + (128 - zp) * colsum[class][n].
    // *zp_res: zero point of the residual codes (res_q holds q - 128 as well).  NULL: symmetric codes.
    const int32_t *zp_in;
    const int32_t *colsum;
    const int32_t *zp_res;
    // optional: the layer norm that follows a linear layer, in the same launch (int8 operands, N <= 768 a
    // multiple of 4, no activation, residual codes, observation or int8 output): ln_out [M, N] receives
    // LN(y + ln_res) with y the layer's fp32 output (never stored; g.y is ignored), ln_res fp32 [M, N],
    // ln_gamma / ln_beta fp32 [N] or null; absmax_out then tracks |ln_out|.  Same arithmetic, in the same
    // order, as launch_layernorm on the stored y.
    float *ln_out;
    const float *ln_res;
    const float *ln_gamma;
    const float *ln_beta;
    double ln_eps;
};
hipError_t launch_gemm_i8(const GemmArgs &g, hipStream_t st);
// true if launch_gemm_i8 can take the layer norm of an [M, N] output into the GEMM's launch
bool gemm_layernorm_fusable(int32_t N, const void *ln_out, const void *ln_res, const void *gamma, const void *beta);

// The narrow 3x3 convolution (at most 16 input channels, at most 32 outputs) with the quantiser of
// its operands folded in: the workgroup derives the scale of the quantise point itself, maps the
// fp32 values of its 128 output pixels and their halo to int8 codes in LDS (the same arithmetic as
// the quantise kernels, so the codes are the same) and contracts from there; the codes never travel
// through global memory.  The skip connection can be produced the same way from the block input.
struct ConvFuse {
    int32_t a_src;              // 0: g.a holds int8 codes; 1: fp32 rows [M, c]; 2: planes [n, c, H*W] (fp32 or bf16)
    const void *a_f;            // source of a_src 1 or 2
    int32_t a_bf16;
    int32_t c;                  // channels of that source (<= 16)
    const uint32_t *a_slot;     // candidate maxima of the quantise point (n, stride), or a fixed scale
    int32_t a_nslot, a_stride;
    const float *a_fixed;
    float *a_scale_out;         // workgroup 0 stores the scale here (and the non-finite flag in *flag)
    uint32_t *flag;
    int32_t res_src;            // 0: g.res_q (int8 [M, 16]) or none; 1: planes [n, res_c, H*W] quantised on load
    const void *res_f;
    int32_t res_bf16;
    int32_t res_c;
    const uint32_t *res_slot;
    int32_t res_nslot, res_stride;
    const float *res_fixed;
};
constexpr int kConvFuseMaxWidth = 256;      // image width up to which the halo of 128 pixels is staged
hipError_t launch_conv3x3_c16_fused(const GemmArgs &g, const ConvFuse &z, hipStream_t st);

// y = LN(x + res) over rows of length H, optional atomicMax of |y|.
hipError_t launch_layernorm(const float *x, const float *res, int64_t rows, int32_t H,
                            const float *gamma, const float *beta, float eps, float *y,
                            uint32_t *absmax_out, hipStream_t st);

// Multi-head self-attention on packed qkv [B, S, 3*Hd] -> ctx [B, S, Hd];
// optional atomicMax of |ctx|.
hipError_t launch_attention(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads,
                            float *ctx, uint32_t *absmax_out, hipStream_t st);

// The same attention for unobserved runs: fp32 matrix-core arithmetic, then the int8 codes [B*S, ldq] and
// the scale of the context as the fp64 evaluation defines them (values whose code the approximate result
// does not settle are re-evaluated in fp64).  ctx receives the approximate context (scratch), records
// attention_records_bytes(...) bytes of scratch, amax_slot, err_slot and exact_slot atomically combined maximum
// words (zero on entry), unsure_total (nullable) is incremented by the number of re-evaluated values.
size_t attention_records_bytes(int32_t B, int32_t S, int32_t heads);
hipError_t launch_attention_fast(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads, float *ctx,
                                 void *records, hipStream_t st);
hipError_t launch_attention_certified(const float *qkv, int32_t B, int32_t S, int32_t Hd, int32_t heads, float *ctx,
                                      void *records, uint32_t *amax_slot, uint32_t *err_slot, uint32_t *exact_slot,
                                      int8_t *xq, int64_t ldq, float *scale_out,
                                      uint32_t *flag, uint32_t *unsure_total, hipStream_t st);

// Training plasticity.  ws_part must hold plasticity_partial_bytes(b, D).
size_t plasticity_partial_bytes(int32_t b, int64_t D);
hipError_t launch_plasticity(const void *a_t, egeria_dtype t_dt, const void *a_r, egeria_dtype r_dt,
                             int32_t b, int64_t D, float *p_out, void *ws_part, hipStream_t st);

// ---- device helpers ------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
// |v| as a bit pattern whose unsigned order is the order of |v|; NaN and Inf
// compare above every finite value.
__device__ __forceinline__ uint32_t abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// Layer norm of one row held by a wave, evaluated in fp64 and rounded once: lane l holds the 16-byte units
// l, l + 64, ... of the row (x and residual already zeroed where absent or beyond the row's nv units, gamma
// one and beta zero where absent).  Returns the outputs of the lane's units and raises amax to the largest
// |output| bit pattern.  Every kernel that normalises a row goes through this one function, so they agree
// bit for bit.
template <int NV>
__device__ __forceinline__ void ln_row_vec(const float4 (&xv)[NV], const float4 (&rv)[NV], const float4 (&gmv)[NV],
                                           const float4 (&btv)[NV], int lane, int nv, int H, double eps,
                                           float4 (&o)[NV], uint32_t &amax)
{
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
        o[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (lane + 64 * i < nv) {
            const float4 gm = gmv[i], bt = btv[i];
            o[i].x = (float)(v[i][0] * rstd * (double)gm.x + (double)bt.x);
            o[i].y = (float)(v[i][1] * rstd * (double)gm.y + (double)bt.y);
            o[i].z = (float)(v[i][2] * rstd * (double)gm.z + (double)bt.z);
            o[i].w = (float)(v[i][3] * rstd * (double)gm.w + (double)bt.w);
            const uint32_t a0 = abs_bits(o[i].x), a1 = abs_bits(o[i].y), a2 = abs_bits(o[i].z), a3 = abs_bits(o[i].w);
            const uint32_t m01 = a0 > a1 ? a0 : a1, m23 = a2 > a3 ? a2 : a3;
            const uint32_t m = m01 > m23 ? m01 : m23;
            amax = amax > m ? amax : m;
        }
    }
}
// Workgroup-wide maximum of a bit pattern, then at most one atomicMax per
// workgroup, and none when the slot already holds a value at least as large.
__device__ __forceinline__ void block_atomic_max(uint32_t v, uint32_t *slot, uint32_t *sm4)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) sm4[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t a = sm4[0] > sm4[1] ? sm4[0] : sm4[1], c = sm4[2] > sm4[3] ? sm4[2] : sm4[3];
        a = a > c ? a : c;
        uint32_t *way = slot + (blockIdx.x & (kAmaxWays - 1)) * kAmaxStride;
        if (a > __hip_atomic_load(way, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(way, a);
    }
}
// Maximum over the ways of an atomically combined word; every lane of the wave
// must call it.
__device__ __forceinline__ uint32_t reduce_ways(const uint32_t *slot)
{
    uint32_t v = slot[(threadIdx.x & (kAmaxWays - 1)) * kAmaxStride];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}
// a / b for 0 <= a, 0 < b; in 32-bit arithmetic when `narrow` says both are below 2^32 (a 64-bit
// integer division is a call of some 150 instructions per lane, a 32-bit one a sixth of that).
__device__ __forceinline__ int64_t div_u(int64_t a, int64_t b, bool narrow)
{
    return narrow ? (int64_t)((uint32_t)a / (uint32_t)b) : a / b;
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
// int8 code of x under the multiplier inv = 1 / scale.
__device__ __forceinline__ uint32_t quant1(float x, float inv)
{
    float r = rintf(x * inv);                 // one fp32 multiply, round half to even
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (uint32_t)((int)r) & 0xffu;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}


// ---- scale from absmax --------------------------------------------------------------
// Called by every thread at the top of a quantise kernel.  Reduces the n_slot
// candidate maxima, returns the multiplier inv and the scale; *bad is set when
// the tensor holds a NaN or an infinity.
__device__ __forceinline__ float scale_from_bits(uint32_t bits, const float *__restrict__ fixed_scale, float *scale,
                                                 bool *bad)
{
    float inv, sc;
    *bad = bits >= 0x7f800000u;
    if (fixed_scale) {
        sc = *fixed_scale;
        inv = (float)(1.0 / (double)sc);
    } else {
        if (*bad) bits = 0;
        const float absmax = __uint_as_float(bits);
        sc = (float)((double)absmax / 127.0);
        inv = (float)(127.0 / (double)absmax);
    }
    if (!(inv <= 3.402823466e+38f) || !(sc > 0.0f)) { sc = 1.0f; inv = 0.0f; }
    *scale = sc;
    return inv;
}

// The lane's share of the n_slot candidate maxima: up to eight independent
// loads, requested together (one memory round trip, not one per candidate).
// The loads are unconditional (index clamped, value masked afterwards): a load
// under a branch is awaited at the end of the branch, one round trip each.
__device__ __forceinline__ uint32_t lane_candidates(const uint32_t *__restrict__ slot, int n_slot, int slot_stride)
{
    if (n_slot <= 0) return 0u;
    const int lane = threadIdx.x & 63;
    uint32_t v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int i = lane + 64 * k;
        v[k] = slot[(size_t)(i < n_slot ? i : n_slot - 1) * slot_stride];
    }
    uint32_t bits = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) bits = (lane + 64 * k < n_slot && v[k] > bits) ? v[k] : bits;
    for (int i = lane + 512; i < n_slot; i += 64) {
        const uint32_t w = slot[(size_t)i * slot_stride];
        bits = bits > w ? bits : w;
    }
    return bits;
}

__device__ __forceinline__ float scales_from(const uint32_t *__restrict__ slot, int n_slot, int slot_stride,
                                             const float *__restrict__ fixed_scale, float *scale, bool *bad)
{
    const uint32_t bits = wave_max_u32(lane_candidates(slot, n_slot, slot_stride));
    return scale_from_bits(bits, fixed_scale, scale, bad);
}

// Only thread 0 of block 0 of a quantise kernel reads or writes the flag word,
// and kernels that share a workspace are ordered on one stream, so plain
// accesses are enough.  Memory that does not yet carry the magic is initialised.
__device__ __forceinline__ void publish(float scale, bool bad, float *scale_out, float *scale_out2, uint32_t *flag)
{
    *scale_out = scale;
    if (scale_out2) *scale_out2 = scale;
    if (flag) {
        uint32_t f = *flag;
        if ((f & 0xffffff00u) != kFlagMagic) f = kFlagMagic;
        if (bad) f |= kFlagNonFinite;
        *flag = f;
    }
}
#endif

}  // namespace egeria
