// Optimiser step of the group-training phase (Algorithm 1; the paper's experiments train with
// Adam with decoupled weight decay): one launch updates up to kAdamwMaxTensors tensors.
//
// The work is element-wise and bound by HBM: per element 16 bytes read (theta, g, m, v) and
// 12 written (theta, m, v), plus 2 for the optional bf16 copy of theta that the bf16 layer
// kernels read.  Every work-group takes one chunk of 4096 consecutive elements of one tensor; a
// table in the kernel arguments maps blockIdx.x to (tensor, chunk), so the many small factor
// tensors of a model (a few hundred thousand elements each) fill the chip in one launch.
#include "common.h"

namespace abt {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = kThreads * 16;   // elements per work-group: four 16-byte accesses per thread

struct AdamwTable {
    AdamwTensor t[kAdamwMaxTensors];
    int first_block[kAdamwMaxTensors + 1];   // work-groups [first_block[i], first_block[i+1]) serve tensor i
    int n;
    float beta1, beta2, one_minus_beta1, one_minus_beta2;
    float inv_bc1;        // 1 / (1 - beta1^step)
    float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^step)
    float eps, eta, weight_decay;
};

struct AdamwOut { float theta, m, v; };

__device__ __forceinline__ AdamwOut adamw_element(float theta, float g, float m, float v, const AdamwTable& a) {
    AdamwOut o;
    o.m = a.beta1 * m + a.one_minus_beta1 * g;
    o.v = a.beta2 * v + a.one_minus_beta2 * (g * g);
    const float denom = sqrtf(o.v) * a.inv_sqrt_bc2 + a.eps;
    const float u = (o.m * a.inv_bc1) / denom;
    o.theta = theta - a.eta * (u + a.weight_decay * theta);
    return o;
}

__global__ __launch_bounds__(kThreads) void adamw_kernel(const AdamwTable a) {
    // blockIdx.x -> tensor: the table is short and wave-uniform, a linear scan is enough
    int ti = 0;
    while (ti + 1 < a.n && (int)blockIdx.x >= a.first_block[ti + 1]) ++ti;
    const AdamwTensor t = a.t[ti];
    const int64_t base = (int64_t)((int)blockIdx.x - a.first_block[ti]) * kChunk;
    const int64_t left = t.count - base;
    if (left <= 0) return;
    const int here = left < kChunk ? (int)left : kChunk;

    float* const P = t.param + base;
    const float* const G = t.grad + base;
    float* const Mo = t.exp_avg + base;
    float* const V = t.exp_avg_sq + base;
    uint16_t* const Pb = t.param_bf16 ? t.param_bf16 + base : nullptr;

    // base is a multiple of 4096 elements, so 16-byte alignment of the tensors carries over
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int e = (it * kThreads + (int)threadIdx.x) * 4;
        if (e + 4 <= here) {
            const f32x4 th = *reinterpret_cast<const f32x4*>(P + e);
            const f32x4 g = *reinterpret_cast<const f32x4*>(G + e);
            const f32x4 m = *reinterpret_cast<const f32x4*>(Mo + e);
            const f32x4 v = *reinterpret_cast<const f32x4*>(V + e);
            f32x4 th1, m1, v1;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const AdamwOut o = adamw_element(th[j], g[j], m[j], v[j], a);
                th1[j] = o.theta; m1[j] = o.m; v1[j] = o.v;
            }
            *reinterpret_cast<f32x4*>(P + e) = th1;
            *reinterpret_cast<f32x4*>(Mo + e) = m1;
            *reinterpret_cast<f32x4*>(V + e) = v1;
            if (Pb) {
                u32x2 w;
                w[0] = pack2_bf16(th1[0], th1[1]);
                w[1] = pack2_bf16(th1[2], th1[3]);
                *reinterpret_cast<u32x2*>(Pb + e) = w;
            }
        } else {
            for (int j = e; j < here; ++j) {   // ragged tail of the tensor: at most three elements
                const AdamwOut o = adamw_element(P[j], G[j], Mo[j], V[j], a);
                P[j] = o.theta; Mo[j] = o.m; V[j] = o.v;
                if (Pb) Pb[j] = (uint16_t)(pack2_bf16(o.theta, 0.0f) & 0xffffu);
            }
        }
    }
}

}  // namespace

hipError_t launch_adamw(const AdamwTensor* tensors, int n, const AdamwHyper& h, hipStream_t s) {
    int done = 0;
    while (done < n) {
        AdamwTable a{};
        int blocks = 0, k = 0;
        while (done < n && k < kAdamwMaxTensors) {
            const AdamwTensor& t = tensors[done++];
            if (t.count <= 0) continue;
            const int64_t nb = ceil_div(t.count, kChunk);
            if (nb > (1 << 30) - blocks) {   // keep the block index in an int: flush what is gathered
                if (k == 0) return hipErrorInvalidValue;
                --done;
                break;
            }
            a.t[k] = t;
            a.first_block[k] = blocks;
            blocks += (int)nb;
            ++k;
        }
        if (k == 0) continue;
        a.first_block[k] = blocks;
        a.n = k;
        a.beta1 = h.beta1; a.beta2 = h.beta2;
        a.one_minus_beta1 = h.one_minus_beta1; a.one_minus_beta2 = h.one_minus_beta2;
        a.inv_bc1 = h.inv_bc1; a.inv_sqrt_bc2 = h.inv_sqrt_bc2;
        a.eps = h.eps; a.eta = h.eta; a.weight_decay = h.weight_decay;
        hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace abt
