// C ABI of the library: argument validation, workspace carving and the launch sequences.
// Every operation is documented in include/abtrain.h.
#include <atomic>
#include <cmath>
#include <new>
#include <vector>

#include "common.h"

using namespace abt;

namespace {

std::atomic<int> g_max_sweeps{30};

// Chain kernel choice: for large batches the 128-row kernel where it supports the rank (32, 64, 96,
// 128, 192); else the 64-row kernel with loader and MFMA waves wherever that supports the rank
// (32, 64, 96, 128, 160, 192, 256, 320, 384), else the older kernel (224, 288, 352).
std::atomic<int> g_chain_rows{0};    // 0: automatic; 64 or 128: force that work-group height where the rank allows it
std::atomic<int> g_chain_parts{0};   // 0: automatic; n: force n column parts for 128-row work-groups

// Launch shape of the chain kernel.  Measured on gfx950 (forward of configs 2 and 3 and four other
// shapes): a 128-row work-group takes 1.58 times as long as a 64-row one on the same factors (its
// LDS traffic per slab, not its loaders, sets the pace), so it only pays through the rounds the
// grid needs on the 256 compute units: 4 rounds of 64-row work-groups against 2 of 128-row ones at
// M = 50432 (148 -> 127 us), 2 against 1 at M = 25216.  Column parts (several work-groups per row
// block) never paid in those measurements and are only used when forced.
struct ChainShape { int rows, parts; };

ChainShape choose_chain_shape(int64_t M, int p, int q, int R, bool second_stage, bool allow_parts) {
    const ChainShape small{64, 1};
    const int rows_forced = g_chain_rows.load(), parts_forced = g_chain_parts.load();
    if (rows_forced == 64 || !chain2_tall_supports(R, p, q)) return small;
    int parts = 1;
    if (allow_parts && second_stage && parts_forced > 1) {
        const int ntile = (int)ceil_div(q, 128);
        parts = parts_forced < ntile ? parts_forced : ntile;
    }
    if (rows_forced == 128 || !chain2_supports(R, p, q)) return ChainShape{128, parts};
    const double cost64 = (double)ceil_div(ceil_div(M, 64), 256);
    const double cost128 = 1.58 * (double)ceil_div(ceil_div(M, 128) * parts, 256);
    return cost128 < cost64 ? ChainShape{128, parts} : small;
}

// the gathered chain (factored convolution): same choice of work-group height, no column parts
hipError_t chain_gather(const void* image, const PatchGeom& g, const void* P, const void* Q, void* Yout, void* Tout,
                        int t_pitch, int64_t M, int q, int R, hipStream_t s) {
    const int p = g.kh * g.kw * ((g.Cin + 63) / 64) * 64;
    const ChainShape sh = choose_chain_shape(M, p, q, R, Yout != nullptr, false);
    if (sh.rows == 128) {
        // the tall launcher checks the image window of a 128-row block before it launches anything and
        // reports an invalid value when it does not fit 32-bit offsets: take the 64-row kernel then
        const hipError_t e = launch_chain2_tall_gather_bf16(image, g, P, Q, Yout, Tout, t_pitch, M, q, R, s);
        if (e != hipErrorInvalidValue) return e;
        (void)hipGetLastError();
    }
    return launch_chain2_gather_bf16(image, g, P, Q, Yout, Tout, t_pitch, M, q, R, s);
}

hipError_t chain(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                 int64_t M, int p, int q, int R, hipStream_t s) {
    const ChainShape sh = choose_chain_shape(M, p, q, R, Yout != nullptr, true);
    if (sh.rows == 128) return launch_chain2_tall_bf16(Xin, P, Q, Yout, Tout, M, p, q, R, sh.parts, s);
    if (chain2_supports(R, p, q)) return launch_chain2_bf16(Xin, P, Q, Yout, Tout, M, p, q, R, s);
    return launch_chain_bf16(Xin, P, Q, Yout, Tout, M, p, q, R, s);
}

// The entry points promise not to throw: what the host-side tables of a call may throw (allocation
// failure of a std::vector) becomes a status.
template <class F>
int guarded(F&& f) {
    try { return f(); }
    catch (const std::bad_alloc&) { return ABT_ENOMEM; }
    catch (...) { return ABT_EHIP; }
}
template <class F>
size_t guarded_size(F&& f) {
    try { return f(); }
    catch (...) { return 0; }
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t esize(int dt) { return dt == ABT_BF16 ? 2 : 4; }

int check_lr_shapes(int64_t M, int64_t m, int64_t n, int64_t r, int dt) {
    if (dt != ABT_F32 && dt != ABT_BF16) return ABT_EDTYPE;
    if (M < 1 || m < 1 || n < 1 || r < 1) return ABT_ESHAPE;
    if (M > 0x7fffffff || m > 0x7fffffff || n > 0x7fffffff || r > 0x7fffffff) return ABT_ESHAPE;
    if (dt == ABT_BF16) {
        if (m % 64 || n % 64 || r % 32 || r > 384) return ABT_ESHAPE;
        if (m > (1 << 20) || n > (1 << 20)) return ABT_ESHAPE;   // 32-bit byte offsets inside row blocks
    }
    return ABT_OK;
}

GemmF32 gemm(const float* A, const float* B, float* C, int64_t P, int64_t Q, int64_t K,
             int64_t lda, int64_t ldb, int64_t ldc, int tA, int tB, int acc) {
    GemmF32 g{};
    g.A = A; g.B = B; g.C = C; g.P = (int)P; g.Q = (int)Q; g.K = (int)K;
    g.lda = (int)lda; g.ldb = (int)ldb; g.ldc = (int)ldc;
    g.transA = tA; g.transB = tB; g.accumulate = acc; g.alpha = 1.0f;
    return g;
}

struct BwdLayout {  // bf16 backward workspace
    size_t At, Bt, dT, T, partials, total;
};

BwdLayout bwd_layout_bf16(int64_t M, int64_t m, int64_t n, int64_t r) {
    BwdLayout w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    w.At = take((size_t)r * m * 2);
    w.Bt = take((size_t)n * r * 2);
    w.dT = take((size_t)M * r * 2);
    w.T = take((size_t)M * r * 2);
    // the split count depends on which gradients are requested: size for the worst subset
    TnJob jobs[2] = {{nullptr, nullptr, nullptr, (int)m, 0}, {nullptr, nullptr, nullptr, (int)n, 1}};
    size_t part = tn_partials_bytes(M, jobs, 2, (int)r);
    const size_t only_a = tn_partials_bytes(M, jobs, 1, (int)r), only_b = tn_partials_bytes(M, jobs + 1, 1, (int)r);
    if (only_a > part) part = only_a;
    if (only_b > part) part = only_b;
    w.partials = take(part);
    w.total = off;
    return w;
}

int check_merge_layer(const abt_merge_desc& d) {
    if (!d.A_copies || !d.B_copies || !d.A_out || !d.B_out || !d.S_out || !d.k_out) return ABT_EINVAL;
    if (d.G < 1 || (d.mode != 0 && d.mode != 1)) return ABT_EINVAL;
    if (!(d.tau >= 0.0f && d.tau <= 1.0f) || d.k_fixed < 0) return ABT_EINVAL;
    if (d.m < 1 || d.n < 1 || d.k < 1 || d.k_cap < 1) return ABT_ESHAPE;
    if (d.k % 32) return ABT_ESHAPE;
    const int64_t K = d.mode == 0 ? d.k : d.k * d.G;
    if (K > 2048 || d.m > 0x7fffffff || d.n > 0x7fffffff || d.k_cap > 0x7fffffff) return ABT_ESHAPE;
    for (int g = 0; g < d.G; ++g) {
        if (!d.A_copies[g] || !d.B_copies[g]) return ABT_EINVAL;
        if (!aligned(d.A_copies[g], 16) || !aligned(d.B_copies[g], 16)) return ABT_EALIGN;
    }
    if (!aligned(d.A_out, 16) || !aligned(d.B_out, 16) || !aligned(d.S_out, 4) || !aligned(d.k_out, 4))
        return ABT_EALIGN;
    if (d.W_out && !aligned(d.W_out, 16)) return ABT_EALIGN;
    return ABT_OK;
}

}  // namespace

extern "C" {

const char* abt_status_string(int status) {
    switch (status) {
        case ABT_OK: return "ABT_OK";
        case ABT_EINVAL: return "ABT_EINVAL: invalid argument";
        case ABT_ESHAPE: return "ABT_ESHAPE: unsupported shape";
        case ABT_EALIGN: return "ABT_EALIGN: misaligned pointer";
        case ABT_EWORKSPACE: return "ABT_EWORKSPACE: workspace missing or too small";
        case ABT_EDTYPE: return "ABT_EDTYPE: unknown dtype";
        case ABT_ENOCONV: return "ABT_ENOCONV: Jacobi sweep cap reached";
        case ABT_EHIP: return "ABT_EHIP: HIP runtime error";
        case ABT_ENOMEM: return "ABT_ENOMEM: host memory allocation failed";
        case ABT_ETOOLARGE: return "ABT_ETOOLARGE: shape needs more than the static scratch array";
        default: return "unknown abt_status";
    }
}

namespace {

// output grid of a convolution with zero padding kh/2, kw/2 and stride s: ceil(H / s) x ceil(W / s)
inline int64_t conv_out(int64_t extent, int stride) { return (extent + stride - 1) / stride; }
inline int64_t conv_rows(const abt_conv_geom& g) { return g.N * conv_out(g.H, g.stride) * conv_out(g.W, g.stride); }
// the three gathers of a factored convolution
PatchGeom conv_patches_geom(const abt_conv_geom& g) {        // rows = output pixels, image = act
    return PatchGeom{(int)g.H, (int)g.W, (int)g.C, g.kh, g.kw, +1,
                     (int)conv_out(g.H, g.stride), (int)conv_out(g.W, g.stride), g.stride, 0};
}
PatchGeom conv_adjoint_geom(const abt_conv_geom& g, int r) {  // rows = input pixels, image = dT on the output grid
    return PatchGeom{(int)conv_out(g.H, g.stride), (int)conv_out(g.W, g.stride), r, g.kh, g.kw, -1,
                     (int)g.H, (int)g.W, 1, g.stride == 2 ? 1 : 0};
}

int check_conv(const abt_conv_geom* g, int64_t m, int64_t r, int dt) {
    if (!g) return ABT_EINVAL;
    if (dt != ABT_BF16) return ABT_EDTYPE;
    if (g->stride != 1 && g->stride != 2) return ABT_ESHAPE;
    if (g->N < 1 || g->H < 1 || g->W < 1 || g->C < 1 || m < 1 || r < 1 || g->kh < 1 || g->kw < 1) return ABT_ESHAPE;
    if (!(g->kh & 1) || !(g->kw & 1) || g->kh > 15 || g->kw > 15) return ABT_ESHAPE;
    if (g->C % 64 || m % 64 || r % 32 || r > 384 || r == 224 || r == 288 || r == 352) return ABT_ESHAPE;
    if (g->H > (1 << 20) || g->W > (1 << 20) || g->C > (1 << 20) || m > (1 << 20)) return ABT_ESHAPE;
    if ((int64_t)g->kh * g->kw * g->C > (1 << 20)) return ABT_ESHAPE;
    if (g->N > 0x7fffffff / (g->H * g->W)) return ABT_ESHAPE;     // pixel count fits an int
    // the window of the image that one 128-row block's patches touch is addressed with 32-bit offsets
    // (the launchers check their own windows again, with the exact geometry)
    if (((int64_t)g->stride * g->stride * (128 + 2 * g->W + 2) + 2 * g->stride * g->W +
         2 * ((g->kh / 2) * g->W + g->kw / 2)) * g->C * 2 >= kBufMaxBytes)
        return ABT_ESHAPE;
    return ABT_OK;
}

// column block of the activation gradient computed per launch: the widest supported tile that divides C
int conv_dact_chunk(int64_t C) {
    static const int sizes[] = {384, 320, 256, 192, 160, 128, 96, 64};
    for (int v : sizes) if (C % v == 0) return v;
    return 64;
}

struct ConvBwdLayout { size_t At, dT, T, Pst, partials, total; int r_pad; };

ConvBwdLayout conv_bwd_layout(const abt_conv_geom& g, int64_t m, int64_t r) {
    ConvBwdLayout w{};
    const int64_t M = conv_rows(g), taps = (int64_t)g.kh * g.kw;     // rows of Y, T, dY, dT
    w.r_pad = (int)((r + 63) / 64 * 64);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    w.At = take((size_t)r * m * 2);
    w.dT = take((size_t)M * r * 2);
    w.T = take((size_t)M * r * 2);
    w.Pst = take((size_t)g.C * taps * w.r_pad * 2);
    const TnJob ja{nullptr, nullptr, nullptr, (int)m, 0}, jb{nullptr, nullptr, nullptr, (int)(taps * g.C), 1};
    const TnJob both[2] = {ja, jb};
    const size_t pa = tn_partials_bytes(M, &ja, 1, (int)r), pb = tn_partials_bytes(M, &jb, 1, (int)r);
    const size_t pab = tn_partials_bytes(M, both, 2, (int)r);
    w.partials = take(pa > pb ? (pa > pab ? pa : pab) : (pb > pab ? pb : pab));
    w.total = off;
    return w;
}

}  // namespace

size_t lr_conv_bwd_workspace_bytes(const abt_conv_geom* geom, int64_t m, int64_t r, int dt) {
    if (check_conv(geom, m, r, dt) != ABT_OK) return 0;
    return conv_bwd_layout(*geom, m, r).total;
}

int lr_conv_fwd(const void* act, const void* A, const void* B, void* Y, void* T_save,
                const abt_conv_geom* geom, int64_t m, int64_t r, int dt, void* stream) {
    int st = check_conv(geom, m, r, dt);
    if (st != ABT_OK) return st;
    if (!act || !A || !B || !Y) return ABT_EINVAL;
    if (!aligned(act, 16) || !aligned(A, 16) || !aligned(B, 16) || !aligned(Y, 16) || !aligned(T_save, 16))
        return ABT_EALIGN;
    const abt_conv_geom& g = *geom;
    const int64_t M = conv_rows(g);
    const PatchGeom pg = conv_patches_geom(g);
    return chain_gather(act, pg, B, A, Y, T_save, (int)r, M, (int)m, (int)r, (hipStream_t)stream) == hipSuccess
               ? ABT_OK : ABT_EHIP;
}

int lr_conv_bwd(const void* dY, const void* act, const void* T, const void* A, const void* B,
                void* dAct, float* dA, float* dB,
                const abt_conv_geom* geom, int64_t m, int64_t r, int dt, int accumulate,
                void* workspace, size_t workspace_bytes, void* stream) {
    int st = check_conv(geom, m, r, dt);
    if (st != ABT_OK) return st;
    if (!dY || !act || !A || !B) return ABT_EINVAL;
    if (!aligned(dY, 16) || !aligned(act, 16) || !aligned(T, 16) || !aligned(A, 16) || !aligned(B, 16) ||
        !aligned(dAct, 16) || !aligned(dA, 16) || !aligned(dB, 16))
        return ABT_EALIGN;
    const abt_conv_geom& g = *geom;
    const ConvBwdLayout w = conv_bwd_layout(g, m, r);
    if (!workspace || workspace_bytes < w.total) return ABT_EWORKSPACE;
    if (!aligned(workspace, 256)) return ABT_EALIGN;
    if (!dAct && !dA && !dB) return ABT_OK;
    hipStream_t s = (hipStream_t)stream;
    char* ws = (char*)workspace;
    const int64_t M = conv_rows(g), M_in = g.N * g.H * g.W;     // output pixels (rows of dY, T, dT), input pixels
    const int taps = g.kh * g.kw;
    const int acc = accumulate ? 1 : 0;
    const PatchGeom fwd_geom = conv_patches_geom(g);
    void* dT = ws + w.dT;
    const void* Tp = T;
    if (!Tp && dA) {   // recompute T = patches(act) B^T (first stage of the chain only)
        if (chain_gather(act, fwd_geom, B, nullptr, nullptr, ws + w.T, (int)r, M, 64, (int)r, s) != hipSuccess)
            return ABT_EHIP;
        Tp = ws + w.T;
    }
    if (dAct || dB) {
        // dT = dY A = dY (A^T)^T: first stage of the plain chain on the transposed factor
        const TransposeJob tj{A, ws + w.At, (int)m, (int)r};
        if (launch_transpose_bf16(&tj, 1, s) != hipSuccess) return ABT_EHIP;
        if (chain(dY, ws + w.At, nullptr, nullptr, dT, M, (int)m, 64, (int)r, s) != hipSuccess) return ABT_EHIP;
    }
    if (dAct) {
        // dAct[q, c] = sum over taps and j of dT[(q - shift(tap)) / stride, j] B[j, tap, c] (only where
        // the division is exact): the same gathered product as the forward, on the image
        // dT [N, H', W', r] with mirrored shifts, against the re-laid-out factor Pst [C, taps r_pad];
        // rows are the input pixels; one launch per block of output channels
        if (launch_conv_bstack_bf16(B, ws + w.Pst, (int)r, (int)g.C, taps, w.r_pad, s) != hipSuccess) return ABT_EHIP;
        const PatchGeom adj = conv_adjoint_geom(g, (int)r);
        const int chunk = conv_dact_chunk(g.C);
        const int64_t pst_pitch = (int64_t)taps * w.r_pad;
        for (int64_t c0 = 0; c0 < g.C; c0 += chunk) {
            const char* Pc = ws + w.Pst + (size_t)c0 * pst_pitch * 2;
            if (chain_gather(dT, adj, Pc, nullptr, nullptr, (char*)dAct + c0 * 2, (int)g.C, M_in, 64, chunk, s) !=
                hipSuccess)
                return ABT_EHIP;
        }
    }
    // factor gradients: dA = dY^T T (plain) and dB = patches(act)^T dT (gathered), one launch
    TnJob jobs[2];
    int nj = 0;
    if (dA) jobs[nj++] = TnJob{dY, Tp, dA, (int)m, 0};
    if (dB) jobs[nj++] = TnJob{act, dT, dB, taps * (int)g.C, 1};
    if (dB) {
        if (launch_tn_gather_bf16(jobs, nj, fwd_geom, M, (int)r, acc, (float*)(ws + w.partials), s) != hipSuccess) return ABT_EHIP;
    } else if (dA) {
        if (launch_tn_bf16(jobs, 1, M, (int)r, acc, (float*)(ws + w.partials), s) != hipSuccess) return ABT_EHIP;
    }
    return ABT_OK;
}

int ab_adamw_step(const abt_adamw_tensor* tensors, int n, int64_t step,
                  double lr, double lr_scale, double beta1, double beta2, double eps,
                  double weight_decay, void* stream) {
    if (n < 0 || (n > 0 && !tensors) || step < 1) return ABT_EINVAL;
    if (!std::isfinite(lr) || !std::isfinite(lr_scale) || !std::isfinite(eps) || !std::isfinite(weight_decay) ||
        !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0) || eps < 0.0)
        return ABT_EINVAL;
    return guarded([&]() -> int {
    std::vector<AdamwTensor> v;
    v.reserve((size_t)n);
    for (int i = 0; i < n; ++i) {
        const abt_adamw_tensor& t = tensors[i];
        if (t.count < 0) return ABT_ESHAPE;
        if (t.count == 0) continue;
        if (!t.param || !t.grad || !t.exp_avg || !t.exp_avg_sq) return ABT_EINVAL;
        if (!aligned(t.param, 16) || !aligned(t.grad, 16) || !aligned(t.exp_avg, 16) ||
            !aligned(t.exp_avg_sq, 16) || !aligned(t.param_bf16, 16))
            return ABT_EALIGN;
        v.push_back(AdamwTensor{t.param, t.grad, t.exp_avg, t.exp_avg_sq, (uint16_t*)t.param_bf16, t.count});
    }
    if (v.empty()) return ABT_OK;
    AdamwHyper h;
    const double b1 = beta1, b2 = beta2;
    h.beta1 = (float)beta1; h.beta2 = (float)beta2;
    h.one_minus_beta1 = (float)(1.0 - b1); h.one_minus_beta2 = (float)(1.0 - b2);
    // 1 - beta^step, without cancellation when beta^step is close to 1
    const double bc1 = b1 > 0.0 ? -std::expm1((double)step * std::log(b1)) : 1.0;
    const double bc2 = b2 > 0.0 ? -std::expm1((double)step * std::log(b2)) : 1.0;
    h.inv_bc1 = (float)(1.0 / bc1);
    h.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
    h.eps = (float)eps; h.eta = (float)(lr * lr_scale); h.weight_decay = (float)weight_decay;
    return launch_adamw(v.data(), (int)v.size(), h, (hipStream_t)stream) == hipSuccess ? ABT_OK : ABT_EHIP;
    });
}

double ab_lr_rebound_scale(int64_t i, int64_t rebound_steps) {
    if (rebound_steps <= 0) return 1.0;
    if (i < 0) i = 0;
    if (i + 1 >= rebound_steps) return 1.0;
    return (double)(i + 1) / (double)rebound_steps;
}

int ab_reconstruct(const float* A, const float* B, float* W,
                   int64_t m, int64_t n, int64_t k, void* stream) {
    if (!A || !B || !W) return ABT_EINVAL;
    if (m < 1 || n < 1 || k < 1 || m > INT32_MAX || n > INT32_MAX || k > INT32_MAX) return ABT_ESHAPE;
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(W, 16)) return ABT_EALIGN;
    return launch_gemm_f32_one(gemm(A, B, W, m, n, k, k, n, n, 0, 0, 0), (hipStream_t)stream) == hipSuccess
               ? ABT_OK : ABT_EHIP;
}

int abt_set_chain_rows(int rows) {
    if (rows == 0 || rows == 64 || rows == 128) return g_chain_rows.exchange(rows);
    return g_chain_rows.load();
}

int abt_set_chain_parts(int parts) {
    if (parts >= 0 && parts <= 8) return g_chain_parts.exchange(parts);
    return g_chain_parts.load();
}

int abt_set_jacobi_max_sweeps(int max_sweeps) {
    return g_max_sweeps.exchange(max_sweeps < 1 ? 1 : (max_sweeps > 64 ? 64 : max_sweeps));
}

int abt_set_merge_groups(int groups) { return merge_set_groups(groups); }

int abt_set_merge_stage_timing(int on) { return merge_set_stage_timing(on); }

int ab_merge_stage_ms(float* ms) {
    if (!ms) return ABT_EINVAL;
    return merge_stage_ms(ms) == hipSuccess ? ABT_OK : ABT_EHIP;
}

size_t lr_linear_fwd_workspace_bytes(int64_t M, int64_t m, int64_t n, int64_t r, int dt) {
    if (check_lr_shapes(M, m, n, r, dt) != ABT_OK) return 0;
    return dt == ABT_F32 ? align_up((size_t)M * r * 4, 256) : 0;
}

size_t lr_linear_bwd_workspace_bytes(int64_t M, int64_t m, int64_t n, int64_t r, int dt) {
    if (check_lr_shapes(M, m, n, r, dt) != ABT_OK) return 0;
    if (dt == ABT_F32) return 2 * align_up((size_t)M * r * 4, 256);
    return bwd_layout_bf16(M, m, n, r).total;
}

int lr_linear_fwd(const void* X, const void* A, const void* B, void* Y, void* T_save,
                  int64_t M, int64_t m, int64_t n, int64_t r, int dt,
                  void* workspace, size_t workspace_bytes, void* stream) {
    int st = check_lr_shapes(M, m, n, r, dt);
    if (st != ABT_OK) return st;
    if (!X || !A || !B || !Y) return ABT_EINVAL;
    if (!aligned(X, 16) || !aligned(A, 16) || !aligned(B, 16) || !aligned(Y, 16) || !aligned(T_save, 16))
        return ABT_EALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (dt == ABT_BF16) {
        return chain(X, B, A, Y, T_save, M, (int)n, (int)m, (int)r, s) == hipSuccess ? ABT_OK : ABT_EHIP;
    }
    float* T = (float*)T_save;
    if (!T) {
        if (!workspace || workspace_bytes < lr_linear_fwd_workspace_bytes(M, m, n, r, dt)) return ABT_EWORKSPACE;
        if (!aligned(workspace, 256)) return ABT_EALIGN;
        T = (float*)workspace;
    }
    // T = X B^T ; Y = T A^T
    if (launch_gemm_f32_one(gemm((const float*)X, (const float*)B, T, M, r, n, n, n, r, 0, 1, 0), s) != hipSuccess) return ABT_EHIP;
    if (launch_gemm_f32_one(gemm(T, (const float*)A, (float*)Y, M, m, r, r, r, m, 0, 1, 0), s) != hipSuccess) return ABT_EHIP;
    return ABT_OK;
}

int lr_linear_bwd(const void* dY, const void* X, const void* T, const void* A, const void* B,
                  void* dX, float* dA, float* dB,
                  int64_t M, int64_t m, int64_t n, int64_t r, int dt, int accumulate,
                  void* workspace, size_t workspace_bytes, void* stream) {
    int st = check_lr_shapes(M, m, n, r, dt);
    if (st != ABT_OK) return st;
    if (!dY || !X || !A || !B) return ABT_EINVAL;
    if (!aligned(dY, 16) || !aligned(X, 16) || !aligned(T, 16) || !aligned(A, 16) || !aligned(B, 16) ||
        !aligned(dX, 16) || !aligned(dA, 16) || !aligned(dB, 16))
        return ABT_EALIGN;
    if (!workspace || workspace_bytes < lr_linear_bwd_workspace_bytes(M, m, n, r, dt)) return ABT_EWORKSPACE;
    if (!aligned(workspace, 256)) return ABT_EALIGN;
    hipStream_t s = (hipStream_t)stream;
    char* ws = (char*)workspace;
    const int acc = accumulate ? 1 : 0;
    if (!dX && !dA && !dB) return ABT_OK;

    if (dt == ABT_F32) {
        float* dT = (float*)ws;
        const float* Tp = (const float*)T;
        const bool need_dT = dX || dB;
        if (!Tp && dA) {
            float* Tw = (float*)(ws + align_up((size_t)M * r * 4, 256));
            if (launch_gemm_f32_one(gemm((const float*)X, (const float*)B, Tw, M, r, n, n, n, r, 0, 1, 0), s) != hipSuccess) return ABT_EHIP;
            Tp = Tw;
        }
        if (need_dT &&
            launch_gemm_f32_one(gemm((const float*)dY, (const float*)A, dT, M, r, m, m, r, r, 0, 0, 0), s) != hipSuccess) return ABT_EHIP;
        if (dX &&
            launch_gemm_f32_one(gemm(dT, (const float*)B, (float*)dX, M, n, r, r, n, n, 0, 0, 0), s) != hipSuccess) return ABT_EHIP;
        if (dA &&
            launch_gemm_f32_one(gemm((const float*)dY, Tp, dA, m, r, M, m, r, r, 1, 0, acc), s) != hipSuccess) return ABT_EHIP;
        if (dB &&
            launch_gemm_f32_one(gemm(dT, (const float*)X, dB, r, n, M, r, n, n, 1, 0, acc), s) != hipSuccess) return ABT_EHIP;
        return ABT_OK;
    }

    const BwdLayout w = bwd_layout_bf16(M, m, n, r);
    void* At = ws + w.At; void* Bt = ws + w.Bt; void* dT = ws + w.dT;
    const void* Tp = T;
    hipError_t e = hipSuccess;
    if (!Tp && dA) {  // recompute T = X B^T (first stage of the chain only)
        e = chain(X, B, nullptr, nullptr, ws + w.T, M, (int)n, (int)m, (int)r, s);
        if (e != hipSuccess) return ABT_EHIP;
        Tp = ws + w.T;
    }
    if (dX || dB) {
        // dT = dY A = dY (A^T)^T and dX = dT B = dT (B^T)^T: the forward chain on transposed factors
        const TransposeJob tj[2] = {{A, At, (int)m, (int)r}, {B, Bt, (int)r, (int)n}};
        e = launch_transpose_bf16(tj, dX ? 2 : 1, s);
        if (e != hipSuccess) return ABT_EHIP;
        e = chain(dY, At, dX ? Bt : nullptr, dX, dT, M, (int)m, (int)n, (int)r, s);
        if (e != hipSuccess) return ABT_EHIP;
    }
    TnJob jobs[2];
    int nj = 0;
    if (dA) jobs[nj++] = TnJob{dY, Tp, dA, (int)m, 0};
    if (dB) jobs[nj++] = TnJob{X, dT, dB, (int)n, 1};
    if (nj) {
        e = launch_tn_bf16(jobs, nj, M, (int)r, acc, (float*)(ws + w.partials), s);
        if (e != hipSuccess) return ABT_EHIP;
    }
    return ABT_OK;
}

// ------------------------------------------------------------------ G emulated groups per launch
namespace {
struct GroupedLayout { size_t At, Bt, dT, T, per_group, partials, total; };

GroupedLayout grouped_layout_bf16(int G, int64_t M, int64_t m, int64_t n, int64_t r) {
    GroupedLayout w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    w.At = take((size_t)r * m * 2);
    w.Bt = take((size_t)n * r * 2);
    w.dT = take((size_t)M * r * 2);
    w.T = take((size_t)M * r * 2);
    w.per_group = off;
    w.partials = (size_t)G * w.per_group;
    // Partials of any subset of the 2 G jobs: elements x splits with splits <= max(1, 256 / tiles) and
    // elements <= tiles x 128 x r, hence at most max(all elements, 256 x 128 x r) floats.
    const size_t all = (size_t)G * (size_t)(m + n) * r, cap = (size_t)256 * 128 * r;
    w.total = w.partials + align_up((all > cap ? all : cap) * sizeof(float), 256);
    return w;
}

int chain_rows_for_groups(int G, int64_t M, int p, int q, int R) {
    const int forced = g_chain_rows.load();
    if (forced == 64 || !chain2_tall_supports(R, p, q)) return 64;
    if (forced == 128 || !chain2_supports(R, p, q)) return 128;
    const double cost64 = (double)ceil_div(G * ceil_div(M, 64), 256);
    const double cost128 = 1.58 * (double)ceil_div(G * ceil_div(M, 128), 256);
    return cost128 < cost64 ? 128 : 64;
}

// one launch for the problems with a second stage and one for those without
hipError_t chain_grouped(const ChainProblem* pr, int G, int64_t M, int p, int q, int R, hipStream_t s) {
    if (!chain2_supports(R, p, q) && !chain2_tall_supports(R, p, q)) {
        for (int g = 0; g < G; ++g) {
            if (!pr[g].Yout && !pr[g].Tout) continue;
            const hipError_t e = chain(pr[g].Xin, pr[g].P, pr[g].Q, pr[g].Yout, pr[g].Tout, M, p, q, R, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    for (int second = 1; second >= 0; --second) {
        ChainProblem sel[kChainMaxGroups];
        int n = 0;
        for (int g = 0; g < G; ++g) {
            const bool has2 = pr[g].Yout != nullptr;
            if ((has2 && second) || (!has2 && !second && pr[g].Tout)) sel[n++] = pr[g];
        }
        if (n == 0) continue;
        const hipError_t e = launch_chain2_grouped_bf16(sel, n, M, p, q, R, chain_rows_for_groups(n, M, p, q, R), 1, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}
}  // namespace

size_t lr_linear_bwd_grouped_workspace_bytes(int G, int64_t M, int64_t m, int64_t n, int64_t r, int dt) {
    if (G < 1 || G > ABT_MAX_GROUPS || check_lr_shapes(M, m, n, r, dt) != ABT_OK) return 0;
    if (dt == ABT_F32) return (size_t)G * lr_linear_bwd_workspace_bytes(M, m, n, r, dt);
    return grouped_layout_bf16(G, M, m, n, r).total;
}

int lr_linear_fwd_grouped(const abt_lr_group* groups, int G,
                          int64_t M, int64_t m, int64_t n, int64_t r, int dt,
                          void* workspace, size_t workspace_bytes, void* stream) {
    const int st = check_lr_shapes(M, m, n, r, dt);
    if (st != ABT_OK) return st;
    if (!groups || G < 1 || G > ABT_MAX_GROUPS) return ABT_EINVAL;
    for (int g = 0; g < G; ++g) {
        const abt_lr_group& q = groups[g];
        if (!q.X || !q.A || !q.B || !q.Y || ((q.T_save != nullptr) != (groups[0].T_save != nullptr))) return ABT_EINVAL;
        if (!aligned(q.X, 16) || !aligned(q.A, 16) || !aligned(q.B, 16) || !aligned(q.Y, 16) || !aligned(q.T_save, 16))
            return ABT_EALIGN;
    }
    if (dt == ABT_F32) {
        const size_t each = lr_linear_fwd_workspace_bytes(M, m, n, r, dt);
        if (!groups[0].T_save && (!workspace || workspace_bytes < each * G)) return ABT_EWORKSPACE;
        for (int g = 0; g < G; ++g) {
            const int e = lr_linear_fwd(groups[g].X, groups[g].A, groups[g].B, groups[g].Y, groups[g].T_save, M, m, n, r, dt,
                                        workspace ? (char*)workspace + each * g : nullptr, each, stream);
            if (e != ABT_OK) return e;
        }
        return ABT_OK;
    }
    ChainProblem pr[kChainMaxGroups];
    for (int g = 0; g < G; ++g) pr[g] = ChainProblem{groups[g].X, groups[g].B, groups[g].A, groups[g].Y, groups[g].T_save};
    return chain_grouped(pr, G, M, (int)n, (int)m, (int)r, (hipStream_t)stream) == hipSuccess ? ABT_OK : ABT_EHIP;
}

int lr_linear_bwd_grouped(const abt_lr_group* groups, int G,
                          int64_t M, int64_t m, int64_t n, int64_t r, int dt, int accumulate,
                          void* workspace, size_t workspace_bytes, void* stream) {
    const int st = check_lr_shapes(M, m, n, r, dt);
    if (st != ABT_OK) return st;
    if (!groups || G < 1 || G > ABT_MAX_GROUPS) return ABT_EINVAL;
    for (int g = 0; g < G; ++g) {
        const abt_lr_group& q = groups[g];
        if (!q.dY || !q.X || !q.A || !q.B) return ABT_EINVAL;
        if (!aligned(q.dY, 16) || !aligned(q.X, 16) || !aligned(q.T, 16) || !aligned(q.A, 16) || !aligned(q.B, 16) ||
            !aligned(q.dX, 16) || !aligned(q.dA, 16) || !aligned(q.dB, 16))
            return ABT_EALIGN;
    }
    if (!workspace || workspace_bytes < lr_linear_bwd_grouped_workspace_bytes(G, M, m, n, r, dt)) return ABT_EWORKSPACE;
    if (!aligned(workspace, 256)) return ABT_EALIGN;
    char* ws = (char*)workspace;
    if (dt == ABT_F32) {
        const size_t each = lr_linear_bwd_workspace_bytes(M, m, n, r, dt);
        for (int g = 0; g < G; ++g) {
            const abt_lr_group& q = groups[g];
            const int e = lr_linear_bwd(q.dY, q.X, q.T, q.A, q.B, q.dX, q.dA, q.dB, M, m, n, r, dt, accumulate,
                                        ws + each * g, each, stream);
            if (e != ABT_OK) return e;
        }
        return ABT_OK;
    }
    hipStream_t s = (hipStream_t)stream;
    const GroupedLayout w = grouped_layout_bf16(G, M, m, n, r);
    auto at = [&](int g, size_t off) { return ws + (size_t)g * w.per_group + off; };
    // T = X B^T again for the groups that did not keep it and need it for dA
    ChainProblem pr[kChainMaxGroups];
    const void* Tp[kChainMaxGroups];
    bool any = false;
    for (int g = 0; g < G; ++g) {
        const abt_lr_group& q = groups[g];
        Tp[g] = q.T;
        pr[g] = ChainProblem{};
        if (!q.T && q.dA) {
            pr[g] = ChainProblem{q.X, q.B, nullptr, nullptr, at(g, w.T)};
            Tp[g] = at(g, w.T);
            any = true;
        }
    }
    if (any && chain_grouped(pr, G, M, (int)n, (int)m, (int)r, s) != hipSuccess) return ABT_EHIP;
    // dT = dY (A^T)^T, dX = dT (B^T)^T: the forward chain on the transposed factors of every group
    TransposeJob tj[kTransposeMaxJobs];
    int ntj = 0;
    any = false;
    for (int g = 0; g < G; ++g) {
        const abt_lr_group& q = groups[g];
        pr[g] = ChainProblem{};
        if (!q.dX && !q.dB) continue;
        tj[ntj++] = TransposeJob{q.A, at(g, w.At), (int)m, (int)r};
        if (q.dX) tj[ntj++] = TransposeJob{q.B, at(g, w.Bt), (int)r, (int)n};
        pr[g] = ChainProblem{q.dY, at(g, w.At), q.dX ? at(g, w.Bt) : nullptr, q.dX, at(g, w.dT)};
        any = true;
    }
    if (any) {
        if (launch_transpose_bf16(tj, ntj, s) != hipSuccess) return ABT_EHIP;
        if (chain_grouped(pr, G, M, (int)m, (int)n, (int)r, s) != hipSuccess) return ABT_EHIP;
    }
    // factor gradients of all groups in one launch (and one split reduction)
    TnJob jobs[kTnMaxJobs];
    int nj = 0;
    for (int g = 0; g < G; ++g) {
        const abt_lr_group& q = groups[g];
        if (q.dA) jobs[nj++] = TnJob{q.dY, Tp[g], q.dA, (int)m, 0};
        if (q.dB) jobs[nj++] = TnJob{q.X, at(g, w.dT), q.dB, (int)n, 1};
    }
    if (nj && tn_partials_bytes(M, jobs, nj, (int)r) > w.total - w.partials) return ABT_EWORKSPACE;   // cannot happen: see the layout
    if (nj && launch_tn_bf16(jobs, nj, M, (int)r, accumulate ? 1 : 0, (float*)(ws + w.partials), s) != hipSuccess)
        return ABT_EHIP;
    return ABT_OK;
}

// ------------------------------------------------------------------ backward without allocation
// The scratch of lr_linear_bwd_static: one array per GPU, held from the moment the library's code is
// loaded on that GPU until the process ends.  In host code the name below is only a handle; the
// array's device address comes from hipGetSymbolAddress, once per device, and only that address is
// ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[ABT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ABT_EHIP;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ABT_EHIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread gets the same address
    }
    *out = p;
    return ABT_OK;
}
}  // namespace

int lr_linear_bwd_static(const void* dY, const void* X, const void* T, const void* A, const void* B,
                         void* dX, float* dA, float* dB,
                         int64_t M, int64_t m, int64_t n, int64_t r, int dt, int accumulate, void* stream) {
    const int st = check_lr_shapes(M, m, n, r, dt);
    if (st != ABT_OK) return st;
    if (lr_linear_bwd_workspace_bytes(M, m, n, r, dt) > (size_t)ABT_STATIC_SCRATCH_BYTES) return ABT_ETOOLARGE;
    void* ws = nullptr;
    const int sp = static_scratch(&ws);
    if (sp != ABT_OK) return sp;
    return lr_linear_bwd(dY, X, T, A, B, dX, dA, dB, M, m, n, r, dt, accumulate, ws,
                         (size_t)ABT_STATIC_SCRATCH_BYTES, stream);
}

size_t ab_merge_batched_workspace_bytes(const abt_merge_desc* layers, int L) {
    if (!layers || L < 1) return 0;
    for (int l = 0; l < L; ++l)
        if (layers[l].G < 1 || layers[l].m < 1 || layers[l].n < 1 || layers[l].k < 1 || layers[l].k_cap < 1 ||
            (layers[l].mode != 0 && layers[l].mode != 1))
            return 0;
    return guarded_size([&] { return merge_workspace_bytes(layers, L); });
}

int ab_merge_batched(const abt_merge_desc* layers, int L, void* workspace, size_t workspace_bytes, void* stream) {
    if (!layers || L < 1) return ABT_EINVAL;
    for (int l = 0; l < L; ++l) {
        const int st = check_merge_layer(layers[l]);
        if (st != ABT_OK) return st;
    }
    return guarded([&]() -> int {
        if (!workspace || workspace_bytes < merge_workspace_bytes(layers, L)) return ABT_EWORKSPACE;
        if (!aligned(workspace, 256)) return ABT_EALIGN;
        return merge_run(layers, L, workspace, g_max_sweeps, (hipStream_t)stream) == hipSuccess ? ABT_OK : ABT_EHIP;
    });
}

size_t ab_merge_workspace_bytes(int G, int64_t m, int64_t n, int64_t k, int64_t k_cap, int mode) {
    abt_merge_desc d{};
    d.G = G; d.m = m; d.n = n; d.k = k; d.k_cap = k_cap; d.mode = mode;
    return ab_merge_batched_workspace_bytes(&d, 1);
}

int ab_merge(const float* const* A_copies, const float* const* B_copies, int G,
             int64_t m, int64_t n, int64_t k, float tau, int64_t k_fixed, int mode,
             float* A_out, float* B_out, float* S_out, int32_t* k_out, int64_t k_cap,
             float* W_out, void* workspace, size_t workspace_bytes, void* stream) {
    abt_merge_desc d{};
    d.A_copies = A_copies; d.B_copies = B_copies; d.G = G; d.mode = mode;
    d.m = m; d.n = n; d.k = k; d.tau = tau; d.k_fixed = k_fixed;
    d.A_out = A_out; d.B_out = B_out; d.S_out = S_out; d.k_out = k_out; d.k_cap = k_cap; d.W_out = W_out;
    return ab_merge_batched(&d, 1, workspace, workspace_bytes, stream);
}

// Dense W = W I (n <= m) or I W (n > m): the merge of one "copy" whose short-side factor is the
// identity.  Workspace: [merge workspace of the L layers][one K x K fp32 identity per distinct K].
}  // extern "C"

namespace {
int64_t factorize_K(int64_t m, int64_t n) { return m < n ? m : n; }

struct FactorizePlan {
    std::vector<abt_merge_desc> merge;      // A_copies / B_copies are filled in by the caller
    std::vector<int64_t> Ks;                // distinct K, in order of first use
    std::vector<size_t> eye_off;            // byte offset of each identity behind the merge workspace
    std::vector<int> eye_of_layer;
    size_t merge_bytes = 0, total = 0;
    int status = ABT_OK;
};

FactorizePlan plan_factorize(const abt_factorize_desc* layers, int L) {
    FactorizePlan p;
    if (!layers || L < 1) { p.status = ABT_EINVAL; return p; }
    p.merge.resize(L);
    p.eye_of_layer.resize(L);
    for (int l = 0; l < L; ++l) {
        const abt_factorize_desc& f = layers[l];
        if (f.m < 1 || f.n < 1 || f.k_cap < 1) { p.status = ABT_ESHAPE; return p; }
        const int64_t K = factorize_K(f.m, f.n);
        if (K % 32 || K > 2048) { p.status = ABT_ESHAPE; return p; }
        abt_merge_desc& d = p.merge[l];
        d = abt_merge_desc{};
        d.G = 1; d.mode = 0; d.m = f.m; d.n = f.n; d.k = K; d.tau = f.tau; d.k_fixed = f.k_fixed;
        d.A_out = f.A_out; d.B_out = f.B_out; d.S_out = f.S_out; d.k_out = f.k_out; d.k_cap = f.k_cap;
        int e = -1;
        for (size_t i = 0; i < p.Ks.size(); ++i) if (p.Ks[i] == K) e = (int)i;
        if (e < 0) { e = (int)p.Ks.size(); p.Ks.push_back(K); }
        p.eye_of_layer[l] = e;
    }
    p.merge_bytes = align_up(merge_workspace_bytes(p.merge.data(), L), 256);
    size_t off = p.merge_bytes;
    for (int64_t K : p.Ks) { p.eye_off.push_back(off); off += align_up(sizeof(float) * K * K, 256); }
    p.total = off;
    return p;
}
}  // namespace

extern "C" {

size_t ab_factorize_batched_workspace_bytes(const abt_factorize_desc* layers, int L) {
    return guarded_size([&]() -> size_t {
        const FactorizePlan p = plan_factorize(layers, L);
        return p.status == ABT_OK ? p.total : 0;
    });
}

int ab_factorize_batched(const abt_factorize_desc* layers, int L, void* workspace, size_t workspace_bytes,
                         void* stream) {
    return guarded([&]() -> int {
    FactorizePlan p = plan_factorize(layers, L);
    if (p.status != ABT_OK) return p.status;
    for (int l = 0; l < L; ++l) {
        if (!layers[l].W) return ABT_EINVAL;
        if (!aligned(layers[l].W, 16)) return ABT_EALIGN;
    }
    if (!workspace || workspace_bytes < p.total) return ABT_EWORKSPACE;
    if (!aligned(workspace, 256)) return ABT_EALIGN;
    // one pointer pair per layer: (W, I) or (I, W); the arrays are read before merge_run returns
    std::vector<const float*> a_ptr(L), b_ptr(L);
    for (int l = 0; l < L; ++l) {
        const float* eye = (const float*)((const char*)workspace + p.eye_off[p.eye_of_layer[l]]);
        const bool tall = layers[l].n <= layers[l].m;
        a_ptr[l] = tall ? layers[l].W : eye;
        b_ptr[l] = tall ? eye : layers[l].W;
        p.merge[l].A_copies = &a_ptr[l];
        p.merge[l].B_copies = &b_ptr[l];
        const int st = check_merge_layer(p.merge[l]);
        if (st != ABT_OK) return st;
    }
    for (size_t i = 0; i < p.Ks.size(); ++i)
        if (launch_identity_f32((float*)((char*)workspace + p.eye_off[i]), (int)p.Ks[i], (hipStream_t)stream) != hipSuccess)
            return ABT_EHIP;
    return merge_run(p.merge.data(), L, workspace, g_max_sweeps, (hipStream_t)stream) == hipSuccess ? ABT_OK : ABT_EHIP;
    });
}

size_t ab_factorize_workspace_bytes(int64_t m, int64_t n, int64_t k_cap) {
    abt_factorize_desc f{};
    f.m = m; f.n = n; f.k_cap = k_cap;
    return ab_factorize_batched_workspace_bytes(&f, 1);
}

int ab_factorize(const float* W, int64_t m, int64_t n, float tau, int64_t k_fixed,
                 float* A_out, float* B_out, float* S_out, int32_t* k_out, int64_t k_cap,
                 void* workspace, size_t workspace_bytes, void* stream) {
    abt_factorize_desc f{};
    f.W = W; f.m = m; f.n = n; f.tau = tau; f.k_fixed = k_fixed;
    f.A_out = A_out; f.B_out = B_out; f.S_out = S_out; f.k_out = k_out; f.k_cap = k_cap;
    return ab_factorize_batched(&f, 1, workspace, workspace_bytes, stream);
}

int ab_merge_info(const void* workspace, int layer, int32_t* sweeps, int32_t* n_sigma, void* stream) {
    if (!workspace || layer < 0) return ABT_EINVAL;
    int32_t info[4] = {0, 0, 0, 0};
    const hipError_t e = merge_read_info(workspace, layer, info, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return ABT_EINVAL;       // not a merge workspace, or no such layer in it
    if (e != hipSuccess) return ABT_EHIP;
    if (sweeps) *sweeps = info[0];
    if (n_sigma) *n_sigma = info[1];
    return info[2] ? ABT_OK : ABT_ENOCONV;
}

}  // extern "C"
