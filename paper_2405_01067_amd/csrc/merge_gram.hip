// First stage of the merge (Algorithm 1: average the factor copies of all groups), fused with the
// Gram matrices the SVD of the merged matrix starts from:
//   mode 0:  Abar = mean_g A_g (m x K),  Bbar = mean_g B_g (K x n)           K = k
//   mode 1:  Abar = [A_1 .. A_G] / G,    Bbar = [B_1; ..; B_G]               K = G k
//   G_A = Abar^T Abar,  G_B = Bbar Bbar^T   (K x K, fp64, both triangles stored)
// The copies are read once from HBM: a work-group owns one 128 x 128 tile of the lower triangle
// of a Gram matrix and walks the whole contraction length (the m rows of Abar, the n columns of
// Bbar) in slabs of 32; it averages the copies on the way into LDS, widens to fp64 when the
// operands are read and accumulates with v_mfma_f64_16x16x4 (products of fp32 numbers are exact
// in fp64, so the Gram matrices carry only the rounding of the fp64 sums).  The work-groups of the
// diagonal tiles also write Abar / Bbar for the back-projection.  The tiles of one matrix sit
// next to each other on one XCD (block index modulo 8), so that the strips they share come out of
// that XCD's L2.
#include "merge_internal.h"

namespace abt {

namespace {

constexpr int GT = 128;        // tile edge
constexpr int GCC = 32;        // contraction indices per slab
constexpr int kGramPtrs = 64;  // copy pointers kept in LDS (more copies than that: fetched from the table)
constexpr int GPITCH = 272;    // floats per contraction index in LDS (two strips of 128 + 16: the four
                               // 16-lane rows of an operand read land in different quarters of the banks)

// column swizzle: contraction index cc stores column c at c ^ (8 ((cc >> 2) & 7)).  Keeps aligned
// groups of 8 columns together (16-byte stores of the A side), permutes inside aligned groups of 64,
// and makes the transposing stores of the B side (8 lanes per row, 8 rows per wave and instruction)
// hit 64 different banks.
__device__ __forceinline__ int gsw(int cc, int c) { return c ^ (((cc >> 2) & 7) << 3); }

// VEC: every row of the source matrices starts 16-byte aligned and holds a multiple of four
// elements (always true for the A side; for the B side when n % 4 == 0): 16-byte loads without
// predicates (addresses of out-of-range chunks are clamped into the matrix, their values dropped).
template <bool VEC>
__global__ __launch_bounds__(256, 1) void mean_gram_kernel(const LayerDev* __restrict__ layers,
                                                           const GramJob* __restrict__ jobs) {
    __shared__ float X[2][GCC * GPITCH];
    __shared__ const float* copy_ptr[kGramPtrs];
    const GramJob job = jobs[blockIdx.x];
    if (job.layer < 0) return;
    const LayerDev& L = layers[job.layer];
    const int K = L.K, k = L.k, G = L.G, mode = L.mode;
    const bool bside = job.which != 0;
    const int len = bside ? L.n : L.m;
    const bool diag = job.ti == job.tj;
    const int nstrip = diag ? 1 : 2;
    const int strip0 = job.ti * GT, strip1 = job.tj * GT;     // first column (A side) / row (B side) of the strips
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, n = lane & 15, kq = lane >> 4;
    const int wr = wave >> 1, wc = wave & 1;
    const bool idle = diag && wr == 0 && wc == 1;              // mirror image of the wave (1, 0)
    const float* const* src = bside ? L.B_ptrs : L.A_ptrs;
    float* mean_out = bside ? L.Bbar : L.Abar;
    const int ncopies = mode == 0 ? G : 1;
    const float scale = (mode == 0 || !bside) ? 1.0f / (float)G : 1.0f;
    // The pointers of the copies go to LDS once.  Fetched from the table in memory when a copy is
    // issued, each would be a load the data loads depend on, and waiting for it (loads return in
    // order) would also wait for every data load still in flight: one full memory latency per copy
    // with nothing overlapped.
    for (int g = t; g < G && g < kGramPtrs; g += 256) copy_ptr[g] = gload(src + g);
    __syncthreads();

    // ---- this thread's chunks of a slab: 4 per strip.  Chunk e of strip s (id = 256 e + t):
    //   A side: contraction row id >> 5 of the slab, columns 4 (id & 31) .. + 3 of the strip
    //   B side: strip row id >> 3, contraction columns 4 (id & 7) .. + 3 of the slab
    // fix[s][e]: element offset of the chunk inside a source matrix for slab 0 (mode 1: inside the copy the
    // chunk comes from, whose pointer is own[s][e]); live: the strip column / row exists (< K).
    int64_t fix[2][4];
    const float* own[2][4];
    bool live[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int id = 256 * e + t;
            const int sb = s == 0 ? strip0 : strip1;
            const int x = bside ? sb + (id >> 3) : sb + 4 * (id & 31);      // strip row / first strip column
            live[s][e] = s < nstrip && x < K;
            const int xc = live[s][e] ? x : 0;
            int gg = 0, xl = xc;
            if (mode != 0) { gg = xc / k; xl = xc - gg * k; }
            own[s][e] = mode != 0 ? gload(src + gg) : nullptr;
            fix[s][e] = bside ? (int64_t)xl * len + 4 * (id & 7) : (int64_t)(id >> 5) * k + xl;
        }
    const int64_t slab_step = bside ? GCC : (int64_t)GCC * k;
    // position of the chunk along the contraction inside a slab (A: its row; B: its first column)
    auto along = [&](int e) { const int id = 256 * e + t; return bside ? 4 * (id & 7) : (id >> 5); };

    // issue: loads only (every address is clamped into the matrix, so none needs a predicate and no
    // instruction between them waits for data); absorb: drops what was out of range and adds the rest
    auto issue = [&](int sl, int g, f32x4 (&pend)[2][4]) {
        const float* base = mode != 0 ? nullptr : (g < kGramPtrs ? copy_ptr[g] : gload(src + g));
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (s >= nstrip) break;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float* p0 = mode == 0 ? base : own[s][e];
                const int pos = sl * GCC + along(e);
                if (VEC) {
                    const int lim = bside ? len - 4 : len - 1;
                    const int back = pos > lim ? pos - lim : 0;
                    const float* p = p0 + fix[s][e] + sl * slab_step - (bside ? (int64_t)back : (int64_t)back * k);
                    pend[s][e] = gload(reinterpret_cast<const f32x4*>(p));
                } else {
                    f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (live[s][e]) {
                        const float* p = p0 + fix[s][e] + sl * slab_step;
                        if (!bside) { if (pos < len) v = gload(reinterpret_cast<const f32x4*>(p)); }
                        else {
#pragma unroll
                            for (int c = 0; c < 4; ++c) if (pos + c < len) v[c] = gload(p + c);
                        }
                    }
                    pend[s][e] = v;
                }
            }
        }
    };
    f32x4 sum[2][4];
    auto absorb = [&](int sl, const f32x4 (&pend)[2][4]) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (s >= nstrip) break;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = !VEC || (live[s][e] && sl * GCC + along(e) < len);
                sum[s][e] += ok ? pend[s][e] : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            }
        }
    };
    auto clear_sum = [&]() {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) sum[s][e] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    };
    // store the finished sums of slab sl into LDS buffer b (and, from the diagonal tile, the mean)
    auto store_slab = [&](int b, int sl) {
        float* Xb = X[b];
        const int c0 = sl * GCC;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (s >= nstrip) break;
            const int sb = s == 0 ? strip0 : strip1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int id = 256 * e + t;
                const f32x4 v = sum[s][e] * scale;
                if (!bside) {
                    const int cc = id >> 5, col = 4 * (id & 31);
                    *reinterpret_cast<f32x4*>(Xb + cc * GPITCH + gsw(cc, GT * s + col)) = v;
                    if (diag && c0 + cc < len && sb + col < K)
                        gstore(reinterpret_cast<f32x4*>(mean_out + (int64_t)(c0 + cc) * K + sb + col), v);
                } else {
                    const int row = id >> 3, cc0 = 4 * (id & 7);
#pragma unroll
                    for (int c = 0; c < 4; ++c) Xb[(cc0 + c) * GPITCH + gsw(cc0 + c, GT * s + row)] = v[c];
                    if (diag && sb + row < K) {
                        float* dst = mean_out + (int64_t)(sb + row) * len + c0 + cc0;
                        if (VEC) { if (c0 + cc0 < len) gstore(reinterpret_cast<f32x4*>(dst), v); }
                        else {
#pragma unroll
                            for (int c = 0; c < 4; ++c) if (c0 + cc0 + c < len) gstore(dst + c, v[c]);
                        }
                    }
                }
            }
        }
    };

    f64x4 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};
    const int offA = wr * 64, offB = (diag ? 0 : GT) + wc * 64;   // this wave's operand columns in the slab
    auto kstep = [&](const float* Xb, int q) {
        const int cc = 4 * q + kq;
        double av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            av[i] = (double)Xb[cc * GPITCH + gsw(cc, offA + 16 * i + n)];
            bv[i] = (double)Xb[cc * GPITCH + gsw(cc, offB + 16 * i + n)];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[i], bv[j], acc[i][j], 0, 0, 0);
    };

    // ---- prologue: slab 0
    f32x4 pend0[2][4], pend1[2][4];
    clear_sum();
    for (int g = 0; g < ncopies; ++g) { issue(0, g, pend0); absorb(0, pend0); }
    const int nslab = (len + GCC - 1) / GCC;
    for (int sl = 0; sl < nslab; ++sl) {
        const int b = sl & 1;
        store_slab(b, sl);
        __syncthreads();          // slab sl visible; everybody is done reading buffer b ^ 1 (slab sl - 1)
        const float* Xb = X[b];
        clear_sum();
        int q = 0;
        if (sl + 1 < nslab) {
            // the copies of the next slab arrive between the products: two copies in flight, copy g is
            // absorbed after its share of the eight steps
            issue(sl + 1, 0, pend0);
            for (int g = 0; g < ncopies; g += 2) {
                if (g + 1 < ncopies) issue(sl + 1, g + 1, pend1);
                for (const int qe = (g + 1) * 8 / ncopies; q < qe; ++q) if (!idle) kstep(Xb, q);
                absorb(sl + 1, pend0);
                if (g + 1 < ncopies) {
                    if (g + 2 < ncopies) issue(sl + 1, g + 2, pend0);
                    for (const int qe = (g + 2) * 8 / ncopies; q < qe; ++q) if (!idle) kstep(Xb, q);
                    absorb(sl + 1, pend1);
                }
            }
        }
        for (; q < 8; ++q) if (!idle) kstep(Xb, q);
    }

    // ---- store: element (i, j) of block (a, b) sits in lane (j, i % 4), register i / 4
    if (idle) return;
    double* out0 = bside ? L.GB : L.LA;
    double* out1 = bside ? L.LB : nullptr;
    const bool mirror = !diag || (wr == 1 && wc == 0);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int bb = 0; bb < 4; ++bb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = strip0 + wr * 64 + 16 * a + kq + 4 * v;
                const int j = strip1 + wc * 64 + 16 * bb + n;
                if (i < K && j < K) {
                    const double val = acc[a][bb][v];
                    gstore(out0 + (int64_t)i * K + j, val);
                    if (out1) gstore(out1 + (int64_t)i * K + j, val);
                    if (mirror) {
                        gstore(out0 + (int64_t)j * K + i, val);
                        if (out1) gstore(out1 + (int64_t)j * K + i, val);
                    }
                }
            }
}

}  // namespace

hipError_t launch_mean_gram(const LayerDev* layers, const GramJob* jobs, int njobs, int njobs_unaligned, hipStream_t s) {
    if (njobs > 0) hipLaunchKernelGGL(mean_gram_kernel<true>, dim3(njobs), dim3(256), 0, s, layers, jobs);
    if (njobs_unaligned > 0)
        hipLaunchKernelGGL(mean_gram_kernel<false>, dim3(njobs_unaligned), dim3(256), 0, s, layers, jobs + njobs);
    return hipGetLastError();
}

}  // namespace abt
