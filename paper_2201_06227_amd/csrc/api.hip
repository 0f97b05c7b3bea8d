// C-ABI of libegeria (include/egeria.h): argument validation, workspace
// planning and the per-module launch sequences of the reference forward.
// Nothing here allocates device memory or synchronises, except egeria_check.
#include "common.hpp"
#include <mutex>
#include <vector>

using namespace egeria;

namespace egeria {
ProfileState g_profile;

int compute_units()
{
    static int cu[kMaxDevices] = {};
    const int dev = current_device();
    if (dev < 0) return 256;                        // no device (host-only sizing calls): the MI355X figure
    if (cu[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cu[dev] = v;
    }
    return cu[dev];
}
}

namespace {

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
inline int64_t pad16(int64_t k) { return (k + 15) / 16 * 16; }
// a basic block whose convolutions quantise their own operands on an unobserved run: at most 16
// channels, an image row that fits the LDS stage, and pixel counts the kernel's 32-bit byte
// offsets hold (2^25 pixels of 16 fp32 channels)
inline bool narrow_block(const egeria_block_desc *d, int64_t M)
{
    return d->kind == EGERIA_BASIC_BLOCK && d->c_in <= 16 && d->width <= kConvFuseMaxWidth && M < (1LL << 25);
}
// an FC mini-batch small enough for the one-workgroup quantiser (maximum, scale and codes in one launch)
inline bool fc_input_is_small(const egeria_block_desc *d)
{
    return (int64_t)d->batch * d->c_in <= kSmallTensor && (int64_t)d->batch * pad16(d->c_in) < (1LL << 30);
}

#define EG_HIP(expr)                                   \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) return EGERIA_ERR_HIP;  \
    } while (0)

// Workspace plan of one layer module: byte offsets from the workspace base.
struct Plan {
    bool ok = false;
    int slots = 0;          // quantise points
    int n_linear = 0;
    int n_layers = 1;
    int64_t M = 0;          // rows of every GEMM (batch, batch*h*w, batch*seq)
    int64_t D = 0;          // features per sample of the hooked activation
    size_t off_q[3] = {0, 0, 0};      // int8 activation buffers
    size_t off_f[5] = {0, 0, 0, 0, 0};  // fp32 intermediates
    size_t off_rec = 0;               // per-workgroup records of the fast attention kernel (Transformer kinds)
    size_t off_aff = 0;               // affine activation codes: partial extrema, then one zero point per quantise point
    size_t off_aref[2] = {0, 0};      // A_R ping-pong (egeria_plasticity_eval)
    size_t off_part = 0;              // metric partials
    size_t fwd_bytes = 0;             // header + forward buffers
    size_t total = 0;
};

// bytes of one operand row of c values at the module's reference precision, padded to 16
inline int64_t op_bytes(const egeria_block_desc *d, int64_t c)
{
    return pad16(c * (d->ref_precision == EGERIA_REF_F16 ? 2 : (d->ref_precision == EGERIA_REF_F32 ? 4 : 1)));
}

bool valid_desc(const egeria_block_desc *d)
{
    if (!d || d->batch < 1) return false;
    if (d->ref_precision < EGERIA_REF_INT8 || d->ref_precision > EGERIA_REF_F32) return false;
    if (d->act_scheme != EGERIA_ACT_SYMMETRIC && d->act_scheme != EGERIA_ACT_AFFINE) return false;
    switch (d->kind) {
    case EGERIA_FC_RELU:
        return d->c_in >= 1 && d->c_out >= 1;
    case EGERIA_BASIC_BLOCK:
        return d->c_in >= 1 && d->c_mid == d->c_in && d->c_out == d->c_in && d->height >= 1 && d->width >= 1;
    case EGERIA_BOTTLENECK:
        return d->c_in >= 1 && d->c_mid >= 1 && d->c_out >= 1 && d->height >= 1 && d->width >= 1 &&
               (!d->has_residual || d->c_out == d->c_in);
    case EGERIA_BERT_LAYER:
    case EGERIA_BERT_STACK:
        return d->seq >= 1 && d->hidden >= 1 && d->heads >= 1 && d->hidden % d->heads == 0 && d->ffn >= 1 &&
               d->n_layers >= 1 && (d->kind == EGERIA_BERT_STACK || d->n_layers == 1) && d->ln_eps >= 0.0f;
    default:
        return false;
    }
}

Plan make_plan(const egeria_block_desc *d)
{
    Plan p;
    if (!valid_desc(d)) return p;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    const int64_t b = d->batch;
    switch (d->kind) {
    case EGERIA_FC_RELU:
        p.slots = 1; p.n_linear = 1; p.M = b; p.D = d->c_out;
        take(header_bytes(p.slots));
        p.off_q[0] = take((size_t)(b * op_bytes(d, d->c_in)));
        break;
    case EGERIA_BASIC_BLOCK: {
        p.slots = 2; p.n_linear = 2; p.M = b * d->height * d->width; p.D = (int64_t)d->height * d->width * d->c_out;
        take(header_bytes(p.slots));
        const int64_t cp = op_bytes(d, d->c_in);
        p.off_q[0] = take((size_t)(p.M * cp));
        p.off_q[1] = take((size_t)(p.M * cp));
        p.off_f[0] = take((size_t)(p.M * d->c_in) * 4);
        break;
    }
    case EGERIA_BOTTLENECK: {
        p.slots = 3; p.n_linear = 3; p.M = b * d->height * d->width; p.D = (int64_t)d->height * d->width * d->c_out;
        take(header_bytes(p.slots));
        p.off_q[0] = take((size_t)(p.M * op_bytes(d, d->c_in)));
        p.off_q[1] = take((size_t)(p.M * op_bytes(d, d->c_mid)));
        p.off_q[2] = take((size_t)(p.M * op_bytes(d, d->c_mid)));
        p.off_f[0] = take((size_t)(p.M * d->c_mid) * 4);
        p.off_f[1] = take((size_t)(p.M * d->c_mid) * 4);
        break;
    }
    default: {
        p.n_layers = d->n_layers;
        // four quantise points per layer + one exact-absmax word for the GELU + one for the attention context
        // + one for the largest error bound of the fast attention kernel's records
        p.slots = 7 * p.n_layers;
        p.n_linear = 4 * p.n_layers; p.M = b * d->seq; p.D = (int64_t)d->seq * d->hidden;
        take(header_bytes(p.slots));
        p.off_q[0] = take((size_t)(p.M * op_bytes(d, d->hidden > d->ffn ? d->hidden : d->ffn)));
        p.off_f[0] = take((size_t)(p.M * 3 * d->hidden) * 4);   // qkv
        p.off_f[1] = take((size_t)(p.M * d->hidden) * 4);       // ctx
        p.off_f[2] = take((size_t)(p.M * d->hidden) * 4);       // attention / ffn projection
        p.off_f[3] = take((size_t)(p.M * d->hidden) * 4);       // post-attention layer norm
        p.off_f[4] = take((size_t)(p.M * d->ffn) * 4);          // ffn hidden
        p.off_rec = take(attention_records_bytes(d->batch, d->seq, d->heads));
        break;
    }
    }
    if (d->act_scheme == EGERIA_ACT_AFFINE) p.off_aff = take(affine_partial_bytes() + 4 * (size_t)p.slots);
    p.fwd_bytes = off;
    const size_t aref = (size_t)b * (size_t)p.D * 4;
    p.off_aref[0] = take(aref);
    p.off_aref[1] = p.n_layers > 1 ? take(aref) : p.off_aref[0];
    p.off_part = take(b <= 128 ? plasticity_partial_bytes((int32_t)b, p.D) : 0);
    p.total = off;
    p.ok = true;
    return p;
}

struct Fwd {
    const egeria_block_desc *d;
    const egeria_qweights *qw;
    const egeria_taps *taps;
    char *ws;
    Plan p;
    hipStream_t st;

    int n_in = 1;           // per-workgroup maxima the input's absmax kernel wrote
    bool input_max_done = false;    // an earlier launch has already taken the input's maxima
    bool input_codes_done = false;  // ... and its int8 codes and scale as well
    // where the absolute maximum of quantise point i is found: the input tensor's
    // per-workgroup maxima for point 0, an atomically combined word otherwise
    const uint32_t *amax(int i) const { return i == 0 ? ws_partials(ws, p.slots) : ws_absmax(ws, i); }
    int n_amax(int i) const { return i == 0 ? n_in : kAmaxWays; }
    int stride_amax(int i) const { return i == 0 ? 1 : kAmaxStride; }
    uint32_t *slot(int i) const { return ws_absmax(ws, i); }
    float *scale(int i) const { return ws_scale(ws, p.slots, i); }
    // static activation scales (Section 5, convolutional networks): the scale of quantise point i
    bool is_static() const { return qw->act_scale != nullptr; }
    const float *sscale(int i) const { return qw->act_scale ? qw->act_scale + i : nullptr; }
    const float *sx(int i) const { return qw->act_scale ? qw->act_scale + i : ws_scale(ws, p.slots, i); }
    bool wants_y(int i) const { const egeria_tap *t = tap(i); return t && t->y; }
    int8_t *qbuf(int i) const { return (int8_t *)(ws + p.off_q[i]); }
    float *fbuf(int i) const { return (float *)(ws + p.off_f[i]); }
    const egeria_tap *tap(int i) const { return taps ? &taps->tap[i] : nullptr; }

    // first kernel of every chain: the input's per-workgroup maxima; its block 0
    // also clears the atomically combined words of the later quantise points
    egeria_status input_absmax(const void *x, egeria_dtype dt, int64_t n)
    {
        n_in = absmax_blocks(n, dt);
        if (input_max_done) return EGERIA_OK;
        if (launch_absmax(x, dt, n, ws_partials(ws, p.slots), ws_absmax(ws, 0), p.slots, st) != hipSuccess)
            return EGERIA_ERR_HIP;
        return EGERIA_OK;
    }

    // affine activation codes: scratch of the extrema pass, zero point of quantise point i
    uint32_t *aff_partials() const { return (uint32_t *)(ws + p.off_aff); }
    int32_t *zp(int i) const { return (int32_t *)(ws + p.off_aff + affine_partial_bytes()) + i; }
    // quantise point `slot`: [n, c, hw] channel planes (hw = 1: matrix rows) -> stored codes in qbuf(qi)
    egeria_status quantize_affine(const void *src, egeria_dtype dt, int64_t n, int64_t c, int64_t hw, int qi, int slot) const
    {
        const int64_t total = n * c * hw;
        EG_HIP(launch_minmax(src, dt, total, aff_partials(), st));
        EG_HIP(launch_quantize_affine(src, dt, n, c, hw, pad16(c), aff_partials(), minmax_blocks(total), 128, qbuf(qi),
                                      scale(slot), zp(slot), ws_flag(ws), st));
        const egeria_tap *t = tap(slot);
        if (t && t->x_q) EG_HIP(hipMemcpyAsync(t->x_q, qbuf(qi), (size_t)(n * hw * pad16(c)), hipMemcpyDeviceToDevice, st));
        if (t && t->x_scale) EG_HIP(hipMemcpyAsync(t->x_scale, scale(slot), 4, hipMemcpyDeviceToDevice, st));
        if (t && t->x_zp) EG_HIP(hipMemcpyAsync(t->x_zp, zp(slot), 4, hipMemcpyDeviceToDevice, st));
        return EGERIA_OK;
    }

    egeria_status copy_tap_q(int i, const int8_t *src, size_t bytes, const float *sc) const
    {
        const egeria_tap *t = tap(i);
        if (!t) return EGERIA_OK;
        if (t->x_q) EG_HIP(hipMemcpyAsync(t->x_q, src, bytes, hipMemcpyDeviceToDevice, st));
        if (t->x_scale) EG_HIP(hipMemcpyAsync(t->x_scale, sc, 4, hipMemcpyDeviceToDevice, st));
        return EGERIA_OK;
    }
    egeria_status copy_tap_y(int i, const float *src, size_t bytes) const
    {
        const egeria_tap *t = tap(i);
        if (t && t->y) EG_HIP(hipMemcpyAsync(t->y, src, bytes, hipMemcpyDeviceToDevice, st));
        return EGERIA_OK;
    }
};

#define EG_OK(expr)                              \
    do {                                         \
        egeria_status s__ = (expr);              \
        if (s__ != EGERIA_OK) return s__;        \
    } while (0)

// One quantised linear layer on rows that are already int8.
egeria_status run_gemm(const Fwd &f, int li, const int8_t *a, int64_t lda, int64_t M, int32_t N, int32_t kp,
                       bool conv, int32_t H, int32_t W, int32_t cp, const float *sx, int act,
                       const int8_t *res_q, const float *res_scale, int64_t res_ld, float *y,
                       uint32_t *absmax_out, bool amax_pos = false, bool tap_y = true, int8_t *q_out = nullptr,
                       int64_t q_ld = 0, const float *q_scale = nullptr, const int32_t *zp_in = nullptr,
                       const int32_t *zp_res = nullptr)
{
    const egeria_qlinear &L = f.qw->linear[li];
    GemmArgs g{};
    g.a = a; g.w = L.w_q; g.M = M; g.N = N; g.kp = kp; g.lda = lda;
    g.a_bytes = conv ? M * (int64_t)cp : M * lda;
    g.w_bytes = (int64_t)N * kp;
    if (g.a_bytes >= (1LL << 31) || g.w_bytes >= (1LL << 31)) return EGERIA_ERR_UNSUPPORTED;
    g.conv3x3 = conv ? 1 : 0; g.H = H; g.W = W; g.cp = cp;
    g.sx = sx; g.sw = L.scale; g.sw_per_n = L.per_channel ? 1 : 0; g.bias = L.bias; g.act = act;
    g.et = f.d->ref_precision;
    if (g.et != EGERIA_REF_INT8) { g.sw = sx; g.sw_per_n = 0; }     // float sums: both scales are the 1.0f at sx
    g.res_q = res_q; g.res_scale = res_scale; g.res_ld = res_ld;
    g.y = y; g.ldy = N;
    const egeria_tap *t = f.tap(li);
    g.acc_out = t ? t->acc : nullptr;
    g.absmax_out = absmax_out;
    g.amax_pos = amax_pos ? 1 : 0;
    g.q_out = q_out; g.q_ld = q_ld; g.q_scale = q_scale;
    g.zp_in = zp_in; g.colsum = L.colsum; g.zp_res = zp_res;
    EG_HIP(launch_gemm_i8(g, f.st));
    return (tap_y && y) ? f.copy_tap_y(li, y, (size_t)M * N * 4) : EGERIA_OK;
}

// A linear layer of an encoder and the layer norm that follows it, out = LN(linear(a) + res): one launch when
// nothing observes the linear layer's output and the row length allows it, else the two kernels.
egeria_status run_gemm_layernorm(const Fwd &f, int li, const int8_t *a, int64_t lda, int64_t M, int32_t N, int32_t kp,
                                 const float *sx, float *y, const float *res, const egeria_norm *nm, float *out,
                                 uint32_t *absmax_out)
{
    const float *gamma = nm ? nm->gamma : nullptr, *beta = nm ? nm->beta : nullptr;
    // (a workgroup that owns whole rows streams the whole weight matrix through LDS: measured on the 12-layer
    // BERT-base shape, 41 us against 23 + 28 for K = 768, 85 against 56 + 28 for K = 3072)
    // 64 rows per workgroup: it takes most of the chip's compute units' worth of rows to pay (4096 rows, a
    // quarter of them: 0.207 -> 0.219 ms per one-layer evaluation)
    if (!f.taps && kp <= 1024 && (M + 63) / 64 >= (int64_t)compute_units() * 3 / 4 &&
        gemm_layernorm_fusable(N, out, res, gamma, beta)) {
        const egeria_qlinear &L = f.qw->linear[li];
        GemmArgs g{};
        g.a = a; g.w = L.w_q; g.M = M; g.N = N; g.kp = kp; g.lda = lda;
        g.a_bytes = M * lda;
        g.w_bytes = (int64_t)N * kp;
        if (g.a_bytes >= (1LL << 31) || g.w_bytes >= (1LL << 31)) return EGERIA_ERR_UNSUPPORTED;
        g.sx = sx; g.sw = L.scale; g.sw_per_n = L.per_channel ? 1 : 0; g.bias = L.bias;
        g.ldy = N;
        g.absmax_out = absmax_out;
        g.colsum = L.colsum;
        g.ln_out = out; g.ln_res = res; g.ln_gamma = gamma; g.ln_beta = beta; g.ln_eps = f.d->ln_eps;
        EG_HIP(launch_gemm_i8(g, f.st));
        return EGERIA_OK;
    }
    EG_OK(run_gemm(f, li, a, lda, M, N, kp, false, 0, 0, 0, sx, 0, nullptr, nullptr, 0, y, nullptr));
    EG_HIP(launch_layernorm(res, y, M, N, gamma, beta, f.d->ln_eps, out, absmax_out, f.st));
    return EGERIA_OK;
}

egeria_status forward_fc(Fwd &f, const void *x, egeria_dtype dt, float *a_ref)
{
    const egeria_block_desc *d = f.d;
    const int64_t kp = pad16(d->c_in);
    if (!f.is_static() && fc_input_is_small(d)) {
        // a small mini-batch: maximum, scale and codes in one workgroup and one launch
        if (!f.input_max_done)
            EG_HIP(launch_quantize_small(x, dt, (int)d->batch, (int)d->c_in, 1, (int)kp, f.qbuf(0), f.scale(0),
                                         ws_flag(f.ws), f.st));
    } else {
        if (!f.is_static()) EG_OK(f.input_absmax(x, dt, (int64_t)d->batch * d->c_in));
        if (!f.input_codes_done)
            EG_HIP(launch_quantize_rows(x, dt, d->batch, d->c_in, kp, f.amax(0), f.is_static() ? 0 : f.n_amax(0),
                                        f.stride_amax(0), f.sscale(0), f.qbuf(0), f.scale(0), nullptr, ws_flag(f.ws),
                                        f.st));
    }
    EG_OK(f.copy_tap_q(0, f.qbuf(0), (size_t)(d->batch * kp), f.scale(0)));
    return run_gemm(f, 0, f.qbuf(0), kp, d->batch, d->c_out, (int32_t)kp, false, 0, 0, 0, f.sx(0), 1,
                    nullptr, nullptr, 0, a_ref, nullptr);
}

// A convolution whose output only feeds the next one.  Dynamic scales: fp32
// output + its maximum, then a quantise pass.  Static scales: the epilogue
// writes the next layer's int8 input itself (fp32 only for an observed run).
egeria_status conv_to_int8(Fwd &f, int li, const int8_t *a, int64_t lda, int64_t M, int32_t N, int32_t kp, bool conv,
                           int32_t H, int32_t W, int32_t cp, int fb, int qi)
{
    const int32_t np = (int32_t)pad16(N);
    if (f.is_static()) {
        float *y = f.wants_y(li) ? f.fbuf(fb) : nullptr;
        EG_OK(run_gemm(f, li, a, lda, M, N, kp, conv, H, W, cp, f.sx(li), 1, nullptr, nullptr, 0, y, nullptr, false, true,
                       f.qbuf(qi), np, f.sscale(li + 1)));
    } else {
        EG_OK(run_gemm(f, li, a, lda, M, N, kp, conv, H, W, cp, f.sx(li), 1, nullptr, nullptr, 0, f.fbuf(fb),
                       f.slot(li + 1)));
        EG_HIP(launch_quantize_rows(f.fbuf(fb), EGERIA_F32, M, N, np, f.amax(li + 1), f.n_amax(li + 1),
                                    f.stride_amax(li + 1), nullptr, f.qbuf(qi), f.scale(li + 1), nullptr, ws_flag(f.ws),
                                    f.st));
    }
    return f.copy_tap_q(li + 1, f.qbuf(qi), (size_t)(M * np), f.sx(li + 1));
}

// A basic block of at most 16 channels on an unobserved run: no int8 tensor is
// written.  The first convolution quantises the block input while loading it;
// the second one does the same with the first one's fp32 output (dynamic
// scales) or reads the codes the first one's epilogue wrote (static scales),
// and forms the skip connection from the block input the same way.
egeria_status forward_narrow_block(Fwd &f, const void *x, egeria_dtype dt, float *a_ref)
{
    const egeria_block_desc *d = f.d;
    const bool st = f.is_static();
    auto base = [&](int li) {
        const egeria_qlinear &L = f.qw->linear[li];
        GemmArgs g{};
        g.w = L.w_q; g.M = f.p.M; g.N = li == 0 ? d->c_mid : d->c_out; g.kp = 9 * 16;
        g.w_bytes = (int64_t)g.N * g.kp;
        g.conv3x3 = 1; g.H = d->height; g.W = d->width; g.cp = 16;
        g.sx = f.sx(li); g.sw = L.scale; g.sw_per_n = L.per_channel ? 1 : 0; g.bias = L.bias; g.act = 1;
        g.ldy = g.N;
        return g;
    };
    GemmArgs g1 = base(0);
    ConvFuse z1{};
    z1.a_src = 2; z1.a_f = x; z1.a_bf16 = dt == EGERIA_BF16 ? 1 : 0; z1.c = d->c_in;
    z1.a_slot = f.amax(0); z1.a_nslot = st ? 0 : f.n_amax(0); z1.a_stride = f.stride_amax(0); z1.a_fixed = f.sscale(0);
    z1.a_scale_out = f.scale(0); z1.flag = ws_flag(f.ws);
    if (st) { g1.q_out = f.qbuf(1); g1.q_ld = 16; g1.q_scale = f.sscale(1); }
    else { g1.y = f.fbuf(0); g1.absmax_out = f.slot(1); }
    EG_HIP(launch_conv3x3_c16_fused(g1, z1, f.st));

    GemmArgs g2 = base(1);
    ConvFuse z2{};
    if (st) {
        g2.a = f.qbuf(1); g2.a_bytes = f.p.M * 16;
    } else {
        z2.a_src = 1; z2.a_f = f.fbuf(0); z2.c = d->c_mid;
        z2.a_slot = f.amax(1); z2.a_nslot = f.n_amax(1); z2.a_stride = f.stride_amax(1);
        z2.a_scale_out = f.scale(1); z2.flag = ws_flag(f.ws);
    }
    if (d->has_residual) {
        z2.res_src = 1; z2.res_f = x; z2.res_bf16 = z1.a_bf16; z2.res_c = d->c_in;
        z2.res_slot = f.amax(0); z2.res_nslot = z1.a_nslot; z2.res_stride = z1.a_stride; z2.res_fixed = f.sscale(0);
    }
    g2.y = a_ref;
    EG_HIP(launch_conv3x3_c16_fused(g2, z2, f.st));
    return EGERIA_OK;
}

egeria_status forward_conv_block(Fwd &f, const void *x, egeria_dtype dt, float *a_ref)
{
    const egeria_block_desc *d = f.d;
    const int64_t M = f.p.M, hw = (int64_t)d->height * d->width;
    const int32_t cin_p = (int32_t)pad16(d->c_in), cmid_p = (int32_t)pad16(d->c_mid);
    const int H = d->height, W = d->width;
    if (!f.is_static()) EG_OK(f.input_absmax(x, dt, M * d->c_in));
    if (!f.taps && narrow_block(d, M)) return forward_narrow_block(f, x, dt, a_ref);
    if (!f.input_codes_done)
        EG_HIP(launch_quantize_nchw(x, dt, d->batch, d->c_in, hw, cin_p, f.amax(0), f.is_static() ? 0 : f.n_amax(0),
                                    f.stride_amax(0), f.sscale(0), f.qbuf(0), f.scale(0), nullptr, ws_flag(f.ws), f.st));
    EG_OK(f.copy_tap_q(0, f.qbuf(0), (size_t)(M * cin_p), f.scale(0)));
    const int8_t *res = d->has_residual ? f.qbuf(0) : nullptr;
    if (d->kind == EGERIA_BASIC_BLOCK) {
        EG_OK(conv_to_int8(f, 0, f.qbuf(0), 0, M, d->c_mid, 9 * cin_p, true, H, W, cin_p, 0, 1));
        return run_gemm(f, 1, f.qbuf(1), 0, M, d->c_out, 9 * cmid_p, true, H, W, cmid_p, f.sx(1), 1, res, f.sx(0), cin_p,
                        a_ref, nullptr);
    }
    // bottleneck: 1x1 -> 3x3 -> 1x1
    EG_OK(conv_to_int8(f, 0, f.qbuf(0), cin_p, M, d->c_mid, cin_p, false, 0, 0, 0, 0, 1));
    EG_OK(conv_to_int8(f, 1, f.qbuf(1), 0, M, d->c_mid, 9 * cmid_p, true, H, W, cmid_p, 1, 2));
    return run_gemm(f, 2, f.qbuf(2), cmid_p, M, d->c_out, cmid_p, false, 0, 0, 0, f.sx(2), 1, res, f.sx(0), cin_p, a_ref,
                    nullptr);
}

// The FC and convolution modules at float16 / float32 reference precision
// (Section 6.4, Table 2).  Every layer input is cast to the reference precision
// in the layout the GEMM consumes; sums and outputs are fp32; the skip
// connection adds the cast block input.  Observation points: x_q receives the
// cast operand rows, acc the bit patterns of the fp32 sums, y the output.
egeria_status forward_float(Fwd &f, const void *x, egeria_dtype dt, float *a_ref)
{
    const egeria_block_desc *d = f.d;
    const int et = d->ref_precision, es = et == EGERIA_REF_F16 ? 2 : 4;
    float *one = f.scale(0);
    auto cast = [&](const void *src, egeria_dtype sdt, int64_t n, int64_t c, int64_t hw, int qi) -> egeria_status {
        EG_HIP(launch_cast_chlast(src, sdt, n, c, hw, op_bytes(d, c) / es, et, f.qbuf(qi), one, f.st));
        return EGERIA_OK;
    };
    auto tap_x = [&](int li, int qi, int64_t bytes) -> egeria_status {
        const egeria_tap *t = f.tap(li);
        if (t && t->x_q) EG_HIP(hipMemcpyAsync(t->x_q, f.qbuf(qi), (size_t)bytes, hipMemcpyDeviceToDevice, f.st));
        return EGERIA_OK;
    };
    if (d->kind == EGERIA_FC_RELU) {
        const int64_t kb = op_bytes(d, d->c_in);
        EG_OK(cast(x, dt, d->batch, d->c_in, 1, 0));
        EG_OK(tap_x(0, 0, d->batch * kb));
        return run_gemm(f, 0, f.qbuf(0), kb, d->batch, d->c_out, (int32_t)kb, false, 0, 0, 0, one, 1, nullptr, nullptr, 0,
                        a_ref, nullptr);
    }
    const int64_t M = f.p.M, hw = (int64_t)d->height * d->width;
    const int32_t cin_b = (int32_t)op_bytes(d, d->c_in), cmid_b = (int32_t)op_bytes(d, d->c_mid);
    const int H = d->height, W = d->width;
    EG_OK(cast(x, dt, d->batch, d->c_in, hw, 0));
    EG_OK(tap_x(0, 0, M * cin_b));
    const int8_t *res = d->has_residual ? f.qbuf(0) : nullptr;
    const int64_t res_ld = cin_b / es;
    if (d->kind == EGERIA_BASIC_BLOCK) {
        EG_OK(run_gemm(f, 0, f.qbuf(0), 0, M, d->c_mid, 9 * cin_b, true, H, W, cin_b, one, 1, nullptr, nullptr, 0, f.fbuf(0),
                       nullptr));
        EG_OK(cast(f.fbuf(0), EGERIA_F32, M, d->c_mid, 1, 1));
        EG_OK(tap_x(1, 1, M * cmid_b));
        return run_gemm(f, 1, f.qbuf(1), 0, M, d->c_out, 9 * cmid_b, true, H, W, cmid_b, one, 1, res, one, res_ld, a_ref,
                        nullptr);
    }
    EG_OK(run_gemm(f, 0, f.qbuf(0), cin_b, M, d->c_mid, cin_b, false, 0, 0, 0, one, 1, nullptr, nullptr, 0, f.fbuf(0),
                   nullptr));
    EG_OK(cast(f.fbuf(0), EGERIA_F32, M, d->c_mid, 1, 1));
    EG_OK(tap_x(1, 1, M * cmid_b));
    EG_OK(run_gemm(f, 1, f.qbuf(1), 0, M, d->c_mid, 9 * cmid_b, true, H, W, cmid_b, one, 1, nullptr, nullptr, 0, f.fbuf(1),
                   nullptr));
    EG_OK(cast(f.fbuf(1), EGERIA_F32, M, d->c_mid, 1, 2));
    EG_OK(tap_x(2, 2, M * cmid_b));
    return run_gemm(f, 2, f.qbuf(2), cmid_b, M, d->c_out, cmid_b, false, 0, 0, 0, one, 1, res, one, res_ld, a_ref, nullptr);
}

// Attention sizes (flops of the two products) from which unobserved runs take the certified fp32 kernels;
// egeria_profile_attention_threshold lets tests run them on small shapes too.
double g_attention_min_flops = 5.0e9;

// One encoder layer: `cur` -> `out`.  slot 4l must already hold absmax(cur).
egeria_status forward_bert_layer(const Fwd &f, int l, const float *cur, float *out, bool last)
{
    const egeria_block_desc *d = f.d;
    const int64_t M = f.p.M;
    const int32_t Hd = d->hidden, F = d->ffn;
    const int32_t hp = (int32_t)pad16(Hd), fp = (int32_t)pad16(F);
    const int s0 = 4 * l;
    const egeria_norm *nm = f.qw->norm ? &f.qw->norm[2 * l] : nullptr;
    float *qkv = f.fbuf(0), *ctx = f.fbuf(1), *proj = f.fbuf(2), *y1 = f.fbuf(3), *ff = f.fbuf(4);
    int8_t *xq = f.qbuf(0);

    if (!(l == 0 && f.input_codes_done))
        EG_HIP(launch_quantize_rows(cur, EGERIA_F32, M, Hd, hp, f.amax(s0), f.n_amax(s0), f.stride_amax(s0), nullptr, xq,
                                    f.scale(s0), nullptr, ws_flag(f.ws), f.st));
    EG_OK(f.copy_tap_q(s0, xq, (size_t)(M * hp), f.scale(s0)));
    EG_OK(run_gemm(f, s0, xq, hp, M, 3 * Hd, hp, false, 0, 0, 0, f.scale(s0), 0, nullptr, nullptr, 0, qkv, nullptr));
    // The certified approximate attention is two or three launches with some tens of microseconds of fixed cost; it
    // pays when the fp64 kernel would take longer than that (one layer of 32 x 128 tokens: fp64 46 us; the 12-layer
    // stack of 64 x 256 tokens: 315 us).
    const double attention_flops = 4.0 * d->batch * d->heads * (double)d->seq * d->seq * (Hd / d->heads);
    if (f.taps || attention_flops < g_attention_min_flops) {
        // observed runs (and small ones): the context itself in fp64, then the plain quantiser
        EG_HIP(launch_attention(qkv, d->batch, d->seq, Hd, d->heads, ctx, f.slot(s0 + 1), f.st));
        EG_HIP(launch_quantize_rows(ctx, EGERIA_F32, M, Hd, hp, f.amax(s0 + 1), f.n_amax(s0 + 1), f.stride_amax(s0 + 1),
                                    nullptr, xq, f.scale(s0 + 1), nullptr, ws_flag(f.ws), f.st));
        EG_OK(f.copy_tap_q(s0 + 1, xq, (size_t)(M * hp), f.scale(s0 + 1)));
    } else {
        // unobserved runs: fp32 matrix-core attention, codes and scale certified against the fp64 evaluation
        EG_HIP(launch_attention_certified(qkv, d->batch, d->seq, Hd, d->heads, ctx, f.ws + f.p.off_rec,
                                          f.slot(s0 + 1), f.slot(6 * f.p.n_layers + l), f.slot(5 * f.p.n_layers + l), xq, hp,
                                          f.scale(s0 + 1), ws_flag(f.ws),
                                          ws_flag(f.ws) + kUnsureWord, f.st));
    }
    EG_OK(run_gemm_layernorm(f, s0 + 1, xq, hp, M, Hd, hp, f.scale(s0 + 1), proj, cur, nm ? &nm[0] : nullptr, y1,
                             f.slot(s0 + 2)));

    EG_HIP(launch_quantize_rows(y1, EGERIA_F32, M, Hd, hp, f.amax(s0 + 2), f.n_amax(s0 + 2), f.stride_amax(s0 + 2), nullptr, xq, f.scale(s0 + 2), nullptr,
                                ws_flag(f.ws), f.st));
    EG_OK(f.copy_tap_q(s0 + 2, xq, (size_t)(M * hp), f.scale(s0 + 2)));
    // first feed-forward GEMM: pre-activations only, tracking their positive maximum;
    // GELU is applied inside the next quantiser
    uint32_t *exact_word = f.slot(4 * f.p.n_layers + l);
    EG_OK(run_gemm(f, s0 + 2, xq, hp, M, F, hp, false, 0, 0, 0, f.scale(s0 + 2), 0, nullptr, nullptr, 0, ff,
                   f.slot(s0 + 3), true, false));
    if (const egeria_tap *t = f.tap(s0 + 2))
        if (t->y) EG_HIP(launch_gelu_exact(ff, M * (int64_t)F, t->y, f.st));
    EG_HIP(launch_gelu_absmax_exact(ff, M * (int64_t)F, f.slot(s0 + 3), exact_word, f.st));
    EG_HIP(launch_quantize_gelu_rows(ff, M, F, fp, f.slot(s0 + 3), exact_word, xq, f.scale(s0 + 3), ws_flag(f.ws),
                                     f.st));
    EG_OK(f.copy_tap_q(s0 + 3, xq, (size_t)(M * fp), f.scale(s0 + 3)));
    EG_OK(run_gemm_layernorm(f, s0 + 3, xq, fp, M, Hd, fp, f.scale(s0 + 3), proj, y1, nm ? &nm[1] : nullptr, out,
                             last ? nullptr : f.slot(s0 + 4)));
    return EGERIA_OK;
}

// The FC and convolution modules with affine uint8 activation codes (Section 5: the framework's
// default activation code).  Every quantise point is an extrema pass and a code pass of its own; the
// contraction and the epilogue are the symmetric path's, with the zero points handed to the epilogue.
egeria_status forward_affine(Fwd &f, const void *x, egeria_dtype dt, float *a_ref)
{
    const egeria_block_desc *d = f.d;
    auto gemm = [&](int li, int qi, int64_t lda, int64_t M, int32_t N, int32_t kp, bool conv, int32_t cp, int slot,
                    const int8_t *res, int64_t res_ld, float *y) {
        return run_gemm(f, li, f.qbuf(qi), lda, M, N, kp, conv, d->height, d->width, cp, f.scale(slot), 1, res,
                        res ? f.scale(0) : nullptr, res_ld, y, nullptr, false, true, nullptr, 0, nullptr, f.zp(slot),
                        res ? f.zp(0) : nullptr);
    };
    if (d->kind == EGERIA_FC_RELU) {
        const int32_t kp = (int32_t)pad16(d->c_in);
        EG_OK(f.quantize_affine(x, dt, d->batch, d->c_in, 1, 0, 0));
        return gemm(0, 0, kp, d->batch, d->c_out, kp, false, 0, 0, nullptr, 0, a_ref);
    }
    const int64_t M = f.p.M, hw = (int64_t)d->height * d->width;
    const int32_t cin_p = (int32_t)pad16(d->c_in), cmid_p = (int32_t)pad16(d->c_mid);
    EG_OK(f.quantize_affine(x, dt, d->batch, d->c_in, hw, 0, 0));
    const int8_t *res = d->has_residual ? f.qbuf(0) : nullptr;
    if (d->kind == EGERIA_BASIC_BLOCK) {
        EG_OK(gemm(0, 0, 0, M, d->c_mid, 9 * cin_p, true, cin_p, 0, nullptr, 0, f.fbuf(0)));
        EG_OK(f.quantize_affine(f.fbuf(0), EGERIA_F32, M, d->c_mid, 1, 1, 1));
        return gemm(1, 1, 0, M, d->c_out, 9 * cmid_p, true, cmid_p, 1, res, cin_p, a_ref);
    }
    EG_OK(gemm(0, 0, cin_p, M, d->c_mid, cin_p, false, 0, 0, nullptr, 0, f.fbuf(0)));
    EG_OK(f.quantize_affine(f.fbuf(0), EGERIA_F32, M, d->c_mid, 1, 1, 1));
    EG_OK(gemm(1, 1, 0, M, d->c_mid, 9 * cmid_p, true, cmid_p, 1, nullptr, 0, f.fbuf(1)));
    EG_OK(f.quantize_affine(f.fbuf(1), EGERIA_F32, M, d->c_mid, 1, 2, 2));
    return gemm(2, 2, cmid_p, M, d->c_out, cmid_p, false, 0, 2, res, cin_p, a_ref);
}

// One encoder layer with affine uint8 activation codes: the four linear layers as above, attention in its
// fp64 evaluation, GELU (erf form, fp64 evaluation) on the fp32 output of the first feed-forward layer.
egeria_status forward_affine_bert_layer(const Fwd &f, int l, const float *cur, float *out)
{
    const egeria_block_desc *d = f.d;
    const int64_t M = f.p.M;
    const int32_t Hd = d->hidden, F = d->ffn;
    const int32_t hp = (int32_t)pad16(Hd), fp = (int32_t)pad16(F);
    const int s0 = 4 * l;
    const egeria_norm *nm = f.qw->norm ? &f.qw->norm[2 * l] : nullptr;
    float *qkv = f.fbuf(0), *ctx = f.fbuf(1), *proj = f.fbuf(2), *y1 = f.fbuf(3), *ff = f.fbuf(4);
    auto linear = [&](int li, const float *src, int32_t k, int32_t kp, int32_t n, float *y, bool tap_y) -> egeria_status {
        EG_OK(f.quantize_affine(src, EGERIA_F32, M, k, 1, 0, li));
        return run_gemm(f, li, f.qbuf(0), kp, M, n, kp, false, 0, 0, 0, f.scale(li), 0, nullptr, nullptr, 0, y, nullptr, false,
                        tap_y, nullptr, 0, nullptr, f.zp(li), nullptr);
    };
    EG_OK(linear(s0, cur, Hd, hp, 3 * Hd, qkv, true));
    EG_HIP(launch_attention(qkv, d->batch, d->seq, Hd, d->heads, ctx, nullptr, f.st));
    EG_OK(linear(s0 + 1, ctx, Hd, hp, Hd, proj, true));
    EG_HIP(launch_layernorm(cur, proj, M, Hd, nm ? nm[0].gamma : nullptr, nm ? nm[0].beta : nullptr, d->ln_eps, y1,
                            nullptr, f.st));
    EG_OK(linear(s0 + 2, y1, Hd, hp, F, ff, false));
    EG_HIP(launch_gelu_exact(ff, M * (int64_t)F, ff, f.st));
    EG_OK(f.copy_tap_y(s0 + 2, ff, (size_t)M * F * 4));
    EG_OK(linear(s0 + 3, ff, F, fp, Hd, proj, true));
    EG_HIP(launch_layernorm(y1, proj, M, Hd, nm ? nm[1].gamma : nullptr, nm ? nm[1].beta : nullptr, d->ln_eps, out,
                            nullptr, f.st));
    return EGERIA_OK;
}

// One encoder layer at float16 / float32 reference precision (Section 6.4): the four linear layers
// take their input cast to the reference precision and give fp32; attention (fp64 evaluation), GELU
// (erf form, fp64 evaluation) and the layer norms are the fp32 operators of the int8 path's
// observed runs.  Observation points as in forward_float; y of the first feed-forward layer is the
// GELU's output.
egeria_status forward_float_bert_layer(const Fwd &f, int l, const float *cur, float *out)
{
    const egeria_block_desc *d = f.d;
    const int64_t M = f.p.M;
    const int32_t Hd = d->hidden, F = d->ffn;
    const int et = d->ref_precision, es = et == EGERIA_REF_F16 ? 2 : 4;
    const int32_t hb = (int32_t)op_bytes(d, Hd), fb = (int32_t)op_bytes(d, F);
    const int s0 = 4 * l;
    const egeria_norm *nm = f.qw->norm ? &f.qw->norm[2 * l] : nullptr;
    float *qkv = f.fbuf(0), *ctx = f.fbuf(1), *proj = f.fbuf(2), *y1 = f.fbuf(3), *ff = f.fbuf(4);
    float *one = f.scale(0);
    int8_t *xq = f.qbuf(0);
    auto linear = [&](int li, const float *src, int32_t k, int32_t kb, int32_t n, float *y, bool tap_y) -> egeria_status {
        EG_HIP(launch_cast_chlast(src, EGERIA_F32, M, k, 1, kb / es, et, xq, one, f.st));
        const egeria_tap *t = f.tap(li);
        if (t && t->x_q) EG_HIP(hipMemcpyAsync(t->x_q, xq, (size_t)(M * kb), hipMemcpyDeviceToDevice, f.st));
        return run_gemm(f, li, xq, kb, M, n, kb, false, 0, 0, 0, one, 0, nullptr, nullptr, 0, y, nullptr, false, tap_y);
    };
    EG_OK(linear(s0, cur, Hd, hb, 3 * Hd, qkv, true));
    EG_HIP(launch_attention(qkv, d->batch, d->seq, Hd, d->heads, ctx, nullptr, f.st));
    EG_OK(linear(s0 + 1, ctx, Hd, hb, Hd, proj, true));
    EG_HIP(launch_layernorm(cur, proj, M, Hd, nm ? nm[0].gamma : nullptr, nm ? nm[0].beta : nullptr, d->ln_eps, y1,
                            nullptr, f.st));
    EG_OK(linear(s0 + 2, y1, Hd, hb, F, ff, false));
    EG_HIP(launch_gelu_exact(ff, M * (int64_t)F, ff, f.st));
    EG_OK(f.copy_tap_y(s0 + 2, ff, (size_t)M * F * 4));
    EG_OK(linear(s0 + 3, ff, F, fb, Hd, proj, true));
    EG_HIP(launch_layernorm(y1, proj, M, Hd, nm ? nm[1].gamma : nullptr, nm ? nm[1].beta : nullptr, d->ln_eps, out,
                            nullptr, f.st));
    return EGERIA_OK;
}

egeria_status check_common(const egeria_block_desc *desc, const egeria_qweights *qw, const void *x,
                           egeria_dtype x_dt, const egeria_taps *taps, void *ws, size_t ws_bytes, Plan &p)
{
    if (!desc || !qw || !x || !ws) return EGERIA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(ws)) return EGERIA_ERR_INVALID_ARG;
    p = make_plan(desc);
    if (!p.ok) return EGERIA_ERR_INVALID_ARG;
    if (x_dt != EGERIA_F32 && x_dt != EGERIA_BF16) return EGERIA_ERR_INVALID_ARG;
    if (desc->ref_precision != EGERIA_REF_INT8 && qw->act_scale) return EGERIA_ERR_UNSUPPORTED;
    if (desc->act_scheme == EGERIA_ACT_AFFINE && (qw->act_scale || desc->ref_precision != EGERIA_REF_INT8))
        return EGERIA_ERR_UNSUPPORTED;
    if (desc->kind >= EGERIA_BERT_LAYER) {
        if (x_dt != EGERIA_F32) return EGERIA_ERR_UNSUPPORTED;
        if (desc->hidden / desc->heads > 64) return EGERIA_ERR_UNSUPPORTED;
    }
    if (qw->n_linear != p.n_linear || !qw->linear) return EGERIA_ERR_INVALID_ARG;
    if (qw->act_scale && desc->kind >= EGERIA_BERT_LAYER) return EGERIA_ERR_UNSUPPORTED;
    if (qw->act_scale && (reinterpret_cast<uintptr_t>(qw->act_scale) & 3u)) return EGERIA_ERR_INVALID_ARG;
    if (qw->norm && qw->n_norm != 2 * p.n_layers) return EGERIA_ERR_INVALID_ARG;
    for (int i = 0; i < p.n_linear; ++i) {
        const egeria_qlinear &L = qw->linear[i];
        if (!L.w_q || !aligned16(L.w_q)) return EGERIA_ERR_INVALID_ARG;
        if (desc->ref_precision == EGERIA_REF_INT8 && !L.scale) return EGERIA_ERR_INVALID_ARG;
        if (desc->ref_precision != EGERIA_REF_INT8 && L.per_channel) return EGERIA_ERR_INVALID_ARG;
        if (desc->act_scheme == EGERIA_ACT_AFFINE && (!L.colsum || (reinterpret_cast<uintptr_t>(L.colsum) & 3u)))
            return EGERIA_ERR_INVALID_ARG;
    }
    if (taps && (taps->n != p.n_linear || !taps->tap)) return EGERIA_ERR_INVALID_ARG;
    if (p.M > 0x7fffffffLL || p.slots > 256) return EGERIA_ERR_UNSUPPORTED;
    (void)ws_bytes;
    return EGERIA_OK;
}

}  // namespace

extern "C" {

int64_t egeria_padded(int64_t k) { return pad16(k); }

size_t egeria_quantize_workspace_bytes(void) { return header_bytes(1); }

static egeria_status quantize_common(const void *x, egeria_dtype dt, int64_t n_total, const float *fixed_scale,
                                     int8_t *q, float *scale_out, void *ws, size_t ws_bytes)
{
    if (n_total < 0 || !scale_out || !ws) return EGERIA_ERR_INVALID_ARG;
    if (n_total > 0 && (!x || !q)) return EGERIA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(q) || !aligned16(ws)) return EGERIA_ERR_INVALID_ARG;
    if (dt != EGERIA_F32 && dt != EGERIA_BF16) return EGERIA_ERR_INVALID_ARG;
    if (ws_bytes < header_bytes(1)) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    return EGERIA_OK;
}

egeria_status egeria_quantize(const void *x, egeria_dtype dt, int64_t n, const float *fixed_scale, int8_t *q,
                              float *scale_out, void *ws, size_t ws_bytes, void *stream)
{
    EG_OK(quantize_common(x, dt, n, fixed_scale, q, scale_out, ws, ws_bytes));
    hipStream_t st = (hipStream_t)stream;
    if (!fixed_scale && n > 0 && n <= kSmallTensor) {
        EG_HIP(launch_quantize_small(x, dt, 1, (int)n, 1, (int)n, q, scale_out, ws_flag(ws), st));
        return EGERIA_OK;
    }
    const int nb = fixed_scale ? 0 : absmax_blocks(n, dt);
    if (!fixed_scale) EG_HIP(launch_absmax(x, dt, n, ws_partials(ws, 1), nullptr, 0, st));
    EG_HIP(launch_quantize_rows(x, dt, 1, n, n, ws_partials(ws, 1), nb, 1, fixed_scale, q, scale_out, nullptr, ws_flag(ws),
                                st));
    return EGERIA_OK;
}

egeria_status egeria_quantize_rows(const void *x, egeria_dtype dt, int64_t rows, int64_t cols,
                                   const float *fixed_scale, int8_t *q, float *scale_out, void *ws,
                                   size_t ws_bytes, void *stream)
{
    if (rows < 0 || cols < 0) return EGERIA_ERR_INVALID_ARG;
    EG_OK(quantize_common(x, dt, rows * cols, fixed_scale, q, scale_out, ws, ws_bytes));
    hipStream_t st = (hipStream_t)stream;
    if (!fixed_scale && rows * cols > 0 && rows * pad16(cols) <= kSmallTensor) {
        EG_HIP(launch_quantize_small(x, dt, (int)rows, (int)cols, 1, (int)pad16(cols), q, scale_out, ws_flag(ws), st));
        return EGERIA_OK;
    }
    const int nb = fixed_scale ? 0 : absmax_blocks(rows * cols, dt);
    if (!fixed_scale) EG_HIP(launch_absmax(x, dt, rows * cols, ws_partials(ws, 1), nullptr, 0, st));
    EG_HIP(launch_quantize_rows(x, dt, rows, cols, pad16(cols), ws_partials(ws, 1), nb, 1, fixed_scale, q, scale_out,
                                nullptr, ws_flag(ws), st));
    return EGERIA_OK;
}

egeria_status egeria_quantize_nchw(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t h, int64_t w,
                                   const float *fixed_scale, int8_t *q, float *scale_out, void *ws,
                                   size_t ws_bytes, void *stream)
{
    if (n < 0 || c < 0 || h < 0 || w < 0) return EGERIA_ERR_INVALID_ARG;
    EG_OK(quantize_common(x, dt, n * c * h * w, fixed_scale, q, scale_out, ws, ws_bytes));
    if (n > 65535 || pad16(c) / 64 > 65535) return EGERIA_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    if (!fixed_scale && n * c * h * w > 0 && n * h * w * pad16(c) <= kSmallTensor) {
        EG_HIP(launch_quantize_small(x, dt, (int)n, (int)c, (int)(h * w), (int)pad16(c), q, scale_out, ws_flag(ws), st));
        return EGERIA_OK;
    }
    const int nb = fixed_scale ? 0 : absmax_blocks(n * c * h * w, dt);
    if (!fixed_scale) EG_HIP(launch_absmax(x, dt, n * c * h * w, ws_partials(ws, 1), nullptr, 0, st));
    if (n * c * h * w == 0) {
        EG_HIP(launch_quantize_rows(x, dt, 0, 0, 0, ws_partials(ws, 1), nb, 1, fixed_scale, q, scale_out, nullptr,
                                    ws_flag(ws), st));
        return EGERIA_OK;
    }
    EG_HIP(launch_quantize_nchw(x, dt, n, c, h * w, pad16(c), ws_partials(ws, 1), nb, 1, fixed_scale, q, scale_out,
                                nullptr, ws_flag(ws), st));
    return EGERIA_OK;
}

size_t egeria_quantize_affine_workspace_bytes(void) { return 256 + affine_partial_bytes(); }

egeria_status egeria_quantize_affine(const void *x, egeria_dtype dt, int64_t n, uint8_t *q, float *scale_out,
                                     int32_t *zp_out, void *ws, size_t ws_bytes, void *stream)
{
    if (n < 0 || !scale_out || !zp_out || !ws) return EGERIA_ERR_INVALID_ARG;
    if (n > 0 && (!x || !q)) return EGERIA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(q) || !aligned16(ws)) return EGERIA_ERR_INVALID_ARG;
    if (dt != EGERIA_F32 && dt != EGERIA_BF16) return EGERIA_ERR_INVALID_ARG;
    if (ws_bytes < egeria_quantize_affine_workspace_bytes()) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    uint32_t *partials = (uint32_t *)((char *)ws + 256);
    EG_HIP(launch_minmax(x, dt, n, partials, st));
    EG_HIP(launch_quantize_affine(x, dt, 1, n, 1, pad16(n), partials, minmax_blocks(n), 0, q, scale_out, zp_out, ws_flag(ws),
                                  st));
    return EGERIA_OK;
}

size_t egeria_quantize_weights_workspace_bytes(int32_t n)
{
    if (n < 0) return 0;
    return align_up(4 * ((size_t)kHeaderFixedWords + (size_t)kWeightBatch * kAbsPartials), 256);
}

// extra: a maximum pass to carry along in the first launch of the first batch of per-tensor
// scales; *carried tells whether a launch took it.
static egeria_status quantize_weights_impl(const egeria_weight *w, int32_t n, void *ws, size_t ws_bytes, void *stream,
                                           const InputMaxJob *extra, bool *carried, const InputQuantJob *xq = nullptr,
                                           bool *xq_carried = nullptr)
{
    if (carried) *carried = false;
    if (xq_carried) *xq_carried = false;
    if (n < 0 || (n > 0 && !w) || !ws || !aligned16(ws)) return EGERIA_ERR_INVALID_ARG;
    if (ws_bytes < egeria_quantize_weights_workspace_bytes(n)) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    for (int i = 0; i < n; ++i) {
        const egeria_weight &t = w[i];
        if (t.out < 0 || t.in < 0 || t.kh < 1 || t.kw < 1) return EGERIA_ERR_INVALID_ARG;
        if (t.precision == EGERIA_REF_INT8 && !t.scale) return EGERIA_ERR_INVALID_ARG;
        if (t.dtype != EGERIA_F32 && t.dtype != EGERIA_BF16) return EGERIA_ERR_INVALID_ARG;
        if (t.precision < EGERIA_REF_INT8 || t.precision > EGERIA_REF_F32) return EGERIA_ERR_INVALID_ARG;
        if (t.precision != EGERIA_REF_INT8 && t.per_channel) return EGERIA_ERR_INVALID_ARG;
        if (t.colsum) {
            if (t.precision != EGERIA_REF_INT8 || (reinterpret_cast<uintptr_t>(t.colsum) & 3u)) return EGERIA_ERR_INVALID_ARG;
            if (!((t.kh == 1 && t.kw == 1) || (t.kh == 3 && t.kw == 3))) return EGERIA_ERR_UNSUPPORTED;
        }
        const int64_t total = (int64_t)t.out * t.in * t.kh * t.kw;
        if (total > 0 && (!t.w || !t.w_q)) return EGERIA_ERR_INVALID_ARG;
        if (!aligned16(t.w) || !aligned16(t.w_q)) return EGERIA_ERR_INVALID_ARG;
        const int es = t.precision == EGERIA_REF_F16 ? 2 : (t.precision == EGERIA_REF_F32 ? 4 : 1);
        if ((int64_t)t.out * t.kh * t.kw * pad16((int64_t)t.in * es) >= ((int64_t)1 << 31)) return EGERIA_ERR_UNSUPPORTED;
    }
    hipStream_t st = (hipStream_t)stream;
    // tensors of a float16 / float32 reference model: a cast into the GEMM's layout, no scale
    for (int i = 0; i < n; ++i) {
        const egeria_weight &t = w[i];
        if (t.precision == EGERIA_REF_INT8 || (int64_t)t.out * t.in == 0) continue;
        const int es = t.precision == EGERIA_REF_F16 ? 2 : 4;
        EG_HIP(launch_cast_chlast(t.w, (egeria_dtype)t.dtype, t.out, t.in, (int64_t)t.kh * t.kw,
                                  pad16((int64_t)t.in * es) / es, t.precision, t.w_q, nullptr, st));
    }
    uint32_t *partials = (uint32_t *)ws + kHeaderFixedWords;
    // tensors with one scale are batched separately from those with one scale per output channel
    for (int pc = 0; pc < 2; ++pc) {
        int i = 0;
        while (i < n) {
            WeightBatch b;
            b.n = 0;
            int blocks = 0;
            bool one = true;
            for (; i < n && b.n < kWeightBatch; ++i) {
                const egeria_weight &t = w[i];
                if (t.precision != EGERIA_REF_INT8 || (t.per_channel != 0) != (pc != 0)) continue;
                const int64_t total = (int64_t)t.out * t.in * t.kh * t.kw;
                WeightJob &jb = b.job[b.n++];
                jb.x = t.w;
                jb.q = t.w_q;
                jb.scale = t.scale;
                jb.o = t.out;
                jb.c = t.in;
                jb.hw = t.kh * t.kw;
                jb.cp = (int32_t)pad16(t.in);
                jb.bf16 = t.dtype == EGERIA_BF16;
                jb.per_channel = pc;
                // one workgroup for a small tensor, else about four 16-byte loads per thread
                int64_t nblk = total <= kSmallTensor ? 1 : (total + 4095) / 4096;
                if (nblk > kAbsPartials) nblk = kAbsPartials;
                if (pc) nblk = ((int64_t)t.out + 3) / 4;
                const int64_t units = (int64_t)t.out * jb.hw * (jb.cp / 16);
                jb.first_block = blocks;
                jb.nblk = (int32_t)nblk;
                jb.epb = (int32_t)(((total + nblk - 1) / (nblk > 0 ? nblk : 1) + 7) / 8 * 8);
                jb.upb = (int32_t)((units + nblk - 1) / (nblk > 0 ? nblk : 1));
                blocks += (int)nblk;
                one = one && nblk == 1;
            }
            if (b.n == 0 || blocks == 0) continue;
            if (pc) {
                EG_HIP(launch_quantize_weights_pc(b, blocks, ws_flag(ws), st));
            } else {
                const bool take = extra && carried && !*carried;
                const bool take_q = take && xq && xq_carried && !one;
                EG_HIP(launch_quantize_weights(b, blocks, one, partials, ws_flag(ws), st, take ? extra : nullptr,
                                               take_q ? xq : nullptr));
                if (take) *carried = true;
                if (take_q) *xq_carried = true;
            }
        }
    }
    // sums of the codes just written, for modules with affine activation codes
    for (int i = 0; i < n; ++i) {
        const egeria_weight &t = w[i];
        if (t.colsum) EG_HIP(launch_colsum(t.w_q, t.out, t.kh * t.kw, (int32_t)pad16(t.in), t.colsum, st));
    }
    return EGERIA_OK;
}

egeria_status egeria_quantize_weights(const egeria_weight *w, int32_t n, void *ws, size_t ws_bytes, void *stream)
{
    return quantize_weights_impl(w, n, ws, ws_bytes, stream, nullptr, nullptr);
}

egeria_status egeria_dequantize(const int8_t *q, const float *scale, int64_t n, float *x, void *stream)
{
    if (n < 0 || !scale) return EGERIA_ERR_INVALID_ARG;
    if (n > 0 && (!q || !x)) return EGERIA_ERR_INVALID_ARG;
    EG_HIP(launch_dequantize(q, scale, n, x, (hipStream_t)stream));
    return EGERIA_OK;
}

size_t egeria_workspace_bytes(const egeria_block_desc *desc)
{
    Plan p = make_plan(desc);
    return p.ok ? p.total : 0;
}

// Side stream of the stack evaluations (egeria_plasticity_eval / egeria_refresh_eval with
// n_layers > 1), with the events that order it against the caller's stream.  One per device,
// created on first use (default priority) on the device that is current then.  Every stack
// evaluation of a device shares it: g_side_mutex is held while such a call enqueues its work, so
// the record / wait pairs of two host threads never interleave (a wait refers to the event's last
// record at the time of the wait call), and the scores of concurrent calls simply queue up one
// call after the other on the side stream.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t produced[2] = {nullptr, nullptr};
    hipEvent_t scored[2] = {nullptr, nullptr};
};
static std::mutex g_side_mutex;

// call with g_side_mutex held
static SideStream *side_stream()
{
    static SideStream per_device[kMaxDevices];
    const int dev = current_device();
    if (dev < 0) return nullptr;
    SideStream &s = per_device[dev];
    if (!s.stream) {
        SideStream t;
        if (hipStreamCreateWithFlags(&t.stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
        for (int i = 0; i < 2; ++i) {
            if (hipEventCreateWithFlags(&t.produced[i], hipEventDisableTiming) != hipSuccess) return nullptr;
            if (hipEventCreateWithFlags(&t.scored[i], hipEventDisableTiming) != hipSuccess) return nullptr;
        }
        s = t;
    }
    return &s;
}

static egeria_status forward_impl(const egeria_block_desc *desc, const egeria_qweights *qw, const void *x,
                                  egeria_dtype x_dt, float *a_ref, const egeria_taps *taps,
                                  const void *const *a_train, egeria_dtype t_dt, float *p_out, void *ws,
                                  const Plan &p, hipStream_t st, bool input_max_done = false,
                                  bool input_codes_done = false)
{
    Fwd f{desc, qw, taps, (char *)ws, p, st};
    f.input_max_done = input_max_done;
    f.input_codes_done = input_codes_done;
    const bool eval = p_out != nullptr;
    const size_t aref_elems = (size_t)desc->batch * (size_t)p.D;
    if (desc->kind < EGERIA_BERT_LAYER) {
        float *out = a_ref ? a_ref : (float *)(f.ws + p.off_aref[0]);
        if (desc->ref_precision != EGERIA_REF_INT8) EG_OK(forward_float(f, x, x_dt, out));
        else if (desc->act_scheme == EGERIA_ACT_AFFINE) EG_OK(forward_affine(f, x, x_dt, out));
        else if (desc->kind == EGERIA_FC_RELU) EG_OK(forward_fc(f, x, x_dt, out));
        else EG_OK(forward_conv_block(f, x, x_dt, out));
        if (eval)
            EG_HIP(launch_plasticity(a_train[0], t_dt, out, EGERIA_F32, desc->batch, p.D, p_out, f.ws + p.off_part, st));
        return EGERIA_OK;
    }
    const bool float_ref = desc->ref_precision != EGERIA_REF_INT8;
    const bool affine = desc->act_scheme == EGERIA_ACT_AFFINE;
    if (!float_ref && !affine) EG_OK(f.input_absmax(x, x_dt, p.M * desc->hidden));
    const float *cur = (const float *)x;
    // The score of layer l only needs that layer's output, so it runs on a side
    // stream while the main stream goes on with layer l + 1 (the score is bound
    // by fp32 MFMA and HBM, the next layer starts with HBM-bound kernels).  The two
    // A_R buffers alternate: layer l + 2 may overwrite the buffer only after the
    // score of layer l has read it.  The side stream joins the main one at the end.
    std::unique_lock<std::mutex> side_lock(g_side_mutex, std::defer_lock);
    if (eval && p.n_layers > 1) side_lock.lock();
    SideStream *side = (eval && p.n_layers > 1) ? side_stream() : nullptr;
    if (eval && p.n_layers > 1 && !side) return EGERIA_ERR_HIP;
    for (int l = 0; l < p.n_layers; ++l) {
        float *out = a_ref ? a_ref + (size_t)l * aref_elems : (float *)(f.ws + p.off_aref[l & 1]);
        if (side && l >= 2) EG_HIP(hipStreamWaitEvent(st, side->scored[l & 1], 0));
        if (float_ref) EG_OK(forward_float_bert_layer(f, l, cur, out));
        else if (affine) EG_OK(forward_affine_bert_layer(f, l, cur, out));
        else EG_OK(forward_bert_layer(f, l, cur, out, l + 1 == p.n_layers));
        if (eval) {
            hipStream_t ms = side ? side->stream : st;
            if (side) {
                EG_HIP(hipEventRecord(side->produced[l & 1], st));
                EG_HIP(hipStreamWaitEvent(ms, side->produced[l & 1], 0));
            }
            EG_HIP(launch_plasticity(a_train[l], t_dt, out, EGERIA_F32, desc->batch, p.D, p_out + l,
                                     f.ws + p.off_part, ms));
            if (side) EG_HIP(hipEventRecord(side->scored[l & 1], ms));
        }
        cur = out;
    }
    if (side) {
        EG_HIP(hipStreamWaitEvent(st, side->scored[(p.n_layers - 1) & 1], 0));
        EG_HIP(hipStreamWaitEvent(st, side->scored[(p.n_layers - 2) & 1], 0));
    }
    return EGERIA_OK;
}

egeria_status egeria_ref_forward(const egeria_block_desc *desc, const egeria_qweights *qw, const void *x,
                                 egeria_dtype x_dt, float *a_ref, const egeria_taps *taps, void *ws,
                                 size_t ws_bytes, void *stream)
{
    Plan p;
    EG_OK(check_common(desc, qw, x, x_dt, taps, ws, ws_bytes, p));
    if (!a_ref || !aligned16(a_ref)) return EGERIA_ERR_INVALID_ARG;
    if (ws_bytes < p.fwd_bytes) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    return forward_impl(desc, qw, x, x_dt, a_ref, taps, nullptr, EGERIA_F32, nullptr, ws, p, (hipStream_t)stream);
}

size_t egeria_plasticity_workspace_bytes(int32_t b, int64_t D)
{
    if (b < 1 || b > 128 || D < 1) return 0;
    return plasticity_partial_bytes(b, D);
}

egeria_status egeria_plasticity(const void *a_train, egeria_dtype t_dt, const void *a_ref, egeria_dtype r_dt,
                                int32_t b, int64_t D, float *p_out, void *ws, size_t ws_bytes, void *stream)
{
    if (!a_train || !a_ref || !p_out || !ws || b < 1 || D < 1) return EGERIA_ERR_INVALID_ARG;
    if (!aligned16(a_train) || !aligned16(a_ref) || !aligned16(ws)) return EGERIA_ERR_INVALID_ARG;
    if ((t_dt != EGERIA_F32 && t_dt != EGERIA_BF16) || (r_dt != EGERIA_F32 && r_dt != EGERIA_BF16))
        return EGERIA_ERR_INVALID_ARG;
    if (b > 128) return EGERIA_ERR_UNSUPPORTED;
    if (ws_bytes < plasticity_partial_bytes(b, D)) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    EG_HIP(launch_plasticity(a_train, t_dt, a_ref, r_dt, b, D, p_out, ws, (hipStream_t)stream));
    return EGERIA_OK;
}

egeria_status egeria_plasticity_eval(const egeria_block_desc *desc, const egeria_qweights *qw, const void *x,
                                     egeria_dtype x_dt, const void *const *a_train, egeria_dtype t_dt,
                                     float *p_out, void *ws, size_t ws_bytes, void *stream)
{
    Plan p;
    EG_OK(check_common(desc, qw, x, x_dt, nullptr, ws, ws_bytes, p));
    if (!a_train || !p_out) return EGERIA_ERR_INVALID_ARG;
    if (t_dt != EGERIA_F32 && t_dt != EGERIA_BF16) return EGERIA_ERR_INVALID_ARG;
    for (int l = 0; l < p.n_layers; ++l)
        if (!a_train[l] || !aligned16(a_train[l])) return EGERIA_ERR_INVALID_ARG;
    if (desc->batch > 128) return EGERIA_ERR_UNSUPPORTED;
    if (ws_bytes < p.total) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    return forward_impl(desc, qw, x, x_dt, nullptr, nullptr, a_train, t_dt, p_out, ws, p, (hipStream_t)stream);
}

// Elements of the mini-batch whose maximum the forward takes in a launch of its own, or 0 if it
// has no such launch (static scales, a float reference precision, an FC input small enough for
// the one-launch quantiser).
static int64_t input_max_elems(const egeria_block_desc *d, const egeria_qweights *qw, const Plan &p)
{
    if (qw->act_scale || d->ref_precision != EGERIA_REF_INT8 || d->act_scheme != EGERIA_ACT_SYMMETRIC) return 0;
    if (d->kind == EGERIA_FC_RELU) return fc_input_is_small(d) ? 0 : (int64_t)d->batch * d->c_in;
    if (d->kind == EGERIA_BASIC_BLOCK || d->kind == EGERIA_BOTTLENECK) return p.M * d->c_in;
    return p.M * d->hidden;
}

egeria_status egeria_refresh_eval(const egeria_weight *w, int32_t n_w, void *ws_w, size_t ws_w_bytes,
                                  const egeria_block_desc *desc, const egeria_qweights *qw, const void *x,
                                  egeria_dtype x_dt, const void *const *a_train, egeria_dtype t_dt, float *p_out,
                                  void *ws, size_t ws_bytes, void *stream)
{
    Plan p;
    EG_OK(check_common(desc, qw, x, x_dt, nullptr, ws, ws_bytes, p));
    if (!a_train || !p_out) return EGERIA_ERR_INVALID_ARG;
    if (t_dt != EGERIA_F32 && t_dt != EGERIA_BF16) return EGERIA_ERR_INVALID_ARG;
    for (int l = 0; l < p.n_layers; ++l)
        if (!a_train[l] || !aligned16(a_train[l])) return EGERIA_ERR_INVALID_ARG;
    if (desc->batch > 128) return EGERIA_ERR_UNSUPPORTED;
    if (ws_bytes < p.total) return EGERIA_ERR_WORKSPACE_TOO_SMALL;
    InputMaxJob job{};
    job.n = input_max_elems(desc, qw, p);
    job.x = x;
    job.partials = ws_partials(ws, p.slots);
    job.reset = ws_absmax(ws, 0);
    job.n_reset = p.slots;
    job.bf16 = x_dt == EGERIA_BF16 ? 1 : 0;
    job.nblk = job.n > 0 ? absmax_blocks(job.n, x_dt) : 0;
    if (desc->kind == EGERIA_FC_RELU && !qw->act_scale && desc->ref_precision == EGERIA_REF_INT8 &&
        desc->act_scheme == EGERIA_ACT_SYMMETRIC && fc_input_is_small(desc)) {
        // the whole quantisation of a small FC input is one workgroup's work
        job.n = (int64_t)desc->batch * desc->c_in;
        job.nblk = 1;
        job.q = (int8_t *)((char *)ws + p.off_q[0]);
        job.scale_out = ws_scale(ws, p.slots, 0);
        job.flag = ws_flag(ws);
        job.rows = desc->batch; job.cols = desc->c_in; job.cp = (int32_t)pad16(desc->c_in);
    }
    // the codes of the mini-batch (a separate launch of the forward otherwise) can ride in the snapshot's
    // second launch: rows of an FC or Transformer input, fp32 channel planes of a convolution module that
    // does not quantise inside its convolutions
    InputQuantJob qj{};
    if (job.n > 0 && !job.q) {
        qj.x = x; qj.bf16 = job.bf16; qj.slot = job.partials; qj.n_slot = job.nblk;
        qj.q = (int8_t *)((char *)ws + p.off_q[0]); qj.scale_out = ws_scale(ws, p.slots, 0); qj.flag = ws_flag(ws);
        int64_t units = 0;
        if (desc->kind == EGERIA_FC_RELU) {
            qj.kind = 1; qj.rows = desc->batch; qj.cols = desc->c_in; qj.ldq = pad16(desc->c_in);
            units = qj.rows * (qj.ldq / 16);
        } else if (desc->kind == EGERIA_BERT_LAYER || desc->kind == EGERIA_BERT_STACK) {
            qj.kind = 1; qj.rows = p.M; qj.cols = desc->hidden; qj.ldq = pad16(desc->hidden);
            units = qj.rows * (qj.ldq / 16);
        } else {
            const int64_t hw = (int64_t)desc->height * desc->width, cp = pad16(desc->c_in);
            if (!narrow_block(desc, p.M) && x_dt == EGERIA_F32 && (hw & 3) == 0) {
                qj.kind = 2; qj.rows = desc->batch; qj.cols = desc->c_in; qj.hw = hw; qj.ldq = cp;
                units = qj.rows * (cp / 16) * (hw / 4);
            }
        }
        int64_t blocks = (units + 255) / 256;
        qj.nblk = (int32_t)(blocks > 8192 ? 8192 : blocks);
        if (qj.nblk < 1) qj.kind = 0;
    }
    bool carried = false, codes = false;
    EG_OK(quantize_weights_impl(w, n_w, ws_w, ws_w_bytes, stream, job.n > 0 ? &job : nullptr, &carried,
                                qj.kind != 0 ? &qj : nullptr, &codes));
    return forward_impl(desc, qw, x, x_dt, nullptr, nullptr, a_train, t_dt, p_out, ws, p, (hipStream_t)stream, carried,
                        codes);
}

egeria_status egeria_check(void *ws, void *stream)
{
    if (!ws) return EGERIA_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    uint32_t flag = 0;
    EG_HIP(hipMemcpyAsync(&flag, ws, 4, hipMemcpyDeviceToHost, st));
    EG_HIP(hipStreamSynchronize(st));
    if ((flag & 0xffffff00u) != kFlagMagic) return EGERIA_OK;     // workspace never used
    if (flag & kFlagNonFinite) {
        const uint32_t clean = kFlagMagic;
        EG_HIP(hipMemcpyAsync(ws, &clean, 4, hipMemcpyHostToDevice, st));
        EG_HIP(hipStreamSynchronize(st));
        return EGERIA_ERR_NONFINITE;
    }
    return EGERIA_OK;
}

static int g_profile_armed_class = 0;     // class to resume after egeria_profile_pause(1)

egeria_status egeria_profile_begin(int32_t kernel_class, int32_t max_launches)
{
    static std::vector<hipEvent_t> starts, stops;
    if (kernel_class <= EGERIA_KERNEL_NONE || kernel_class > EGERIA_KERNEL_CACHE_COPY || max_launches < 1)
        return EGERIA_ERR_INVALID_ARG;
    while ((int)starts.size() < max_launches) {
        hipEvent_t a, b;
        EG_HIP(hipEventCreate(&a));
        EG_HIP(hipEventCreate(&b));
        starts.push_back(a);
        stops.push_back(b);
    }
    g_profile.start = starts.data();
    g_profile.stop = stops.data();
    g_profile.n = max_launches;
    g_profile.count = 0;
    g_profile.cls = kernel_class;
    g_profile_armed_class = kernel_class;
    return EGERIA_OK;
}

egeria_status egeria_profile_pause(int32_t paused)
{
    if (paused) {
        if (g_profile.cls != 0) g_profile_armed_class = g_profile.cls;
        g_profile.cls = 0;
    } else if (g_profile_armed_class != 0) {
        g_profile.cls = g_profile_armed_class;
    }
    return EGERIA_OK;
}

egeria_status egeria_profile_end(float *ms_out, int32_t capacity, int32_t *n_out)
{
    if (!n_out || capacity < 0 || (capacity > 0 && !ms_out)) return EGERIA_ERR_INVALID_ARG;
    const int n = g_profile.count;
    g_profile.cls = 0;
    g_profile_armed_class = 0;
    g_profile.count = 0;
    *n_out = n;
    for (int i = 0; i < n && i < capacity; ++i) {
        EG_HIP(hipEventSynchronize(g_profile.stop[i]));
        EG_HIP(hipEventElapsedTime(&ms_out[i], g_profile.start[i], g_profile.stop[i]));
    }
    return EGERIA_OK;
}

egeria_status egeria_profile_attention(const float *qkv, int32_t B, int32_t S, int32_t hidden, int32_t heads,
                                       int32_t mode, float *ctx, void *records, void *stream)
{
    if (!qkv || !ctx || B < 1 || S < 1 || hidden < 1 || heads < 1 || hidden % heads != 0) return EGERIA_ERR_INVALID_ARG;
    if (!aligned16(qkv) || !aligned16(ctx) || (mode != 0 && mode != 1)) return EGERIA_ERR_INVALID_ARG;
    if (mode == 1 && (!records || !aligned16(records))) return EGERIA_ERR_INVALID_ARG;
    if (hidden / heads > 64) return EGERIA_ERR_UNSUPPORTED;
    if (mode == 0) EG_HIP(launch_attention(qkv, B, S, hidden, heads, ctx, nullptr, (hipStream_t)stream));
    else EG_HIP(launch_attention_fast(qkv, B, S, hidden, heads, ctx, records, (hipStream_t)stream));
    return EGERIA_OK;
}

double egeria_profile_attention_threshold(double min_flops)
{
    const double old = g_attention_min_flops;
    if (min_flops >= 0.0) g_attention_min_flops = min_flops;
    return old;
}

const char *egeria_status_string(egeria_status s)
{
    switch (s) {
    case EGERIA_OK: return "ok";
    case EGERIA_ERR_INVALID_ARG: return "invalid argument";
    case EGERIA_ERR_UNSUPPORTED: return "unsupported shape or type";
    case EGERIA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case EGERIA_ERR_NONFINITE: return "non-finite value met by a quantiser";
    case EGERIA_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

}  // extern "C"
