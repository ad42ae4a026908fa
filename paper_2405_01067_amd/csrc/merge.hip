// Merge of G group copies of a layer's factors and re-factorisation (Algorithm 1: average A and
// B over all workers, W <- A B; then Eq. 3 with the singular-value cut-off), for L layers at once.
//
// The merged matrix Wbar = Abar Bbar is never formed for the SVD.  With Gram matrices
// G_A = Abar^T Abar = L_A L_A^T and G_B = Bbar Bbar^T = L_B L_B^T (Cholesky, fp64) one has
// Abar = Q_A L_A^T and Bbar = L_B Q_B^T with orthonormal Q_A, Q_B, hence
//     Wbar = Q_A C Q_B^T,   C = L_A^T L_B   (K x K),
// and the SVD of the small core C = U_c Sigma V_c^T carries over: U = Q_A U_c, V = Q_B V_c.
// A one-sided (Hestenes) Jacobi iteration orthogonalises the columns of C: C V_c = U_c Sigma.
// The new factors of Eq. 3 are back-projections of the averaged ones, without any inverse:
//     A' = U Sigma^(1/2) = Abar P_A,   P_A = G_B Y diag(sigma^(-5/2))
//     B' = Sigma^(1/2) V^T = P_B Bbar, P_B = diag(sigma^(-3/2)) Y^T,      Y = L_A (C V_c)
// (from U_c Sigma = C V_c, V_c Sigma = C^T U_c and L L^T = G).  Everything K x K runs in fp64;
// the streaming ends (mean, back-projection) are fp32.
//
// mode 1 (mean of reconstructions) uses the same pipeline on the concatenations
// Abar = [A_1 .. A_G] / G (m x Gk) and Bbar = [B_1; ..; B_G] (Gk x n).
#include <atomic>
#include <mutex>
#include <vector>

#include "merge_internal.h"

namespace abt {

namespace {

// ------------------------------------------------------------------------------------------
// zero-fill by a kernel (fill kernels, not memset nodes, are what stays correct under graph replay)
// ------------------------------------------------------------------------------------------
__global__ void fill_i32_kernel(int* p, int64_t n, int v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void identity_f32_kernel(float* p, int K) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (int64_t)K * K) p[i] = (i / K == i % K) ? 1.0f : 0.0f;
}

// ------------------------------------------------------------------------------------------
// Stage 1: average (mode 0) or concatenate (mode 1) the G copies.  Pure streaming.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mean_kernel(const LayerDev* __restrict__ layers) {
    const LayerDev& L = layers[blockIdx.y];
    const int G = L.G;
    const float inv = 1.0f / (float)G;
    const int64_t nA = (int64_t)L.m * L.k, nB = (int64_t)L.k * L.n;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
    const int64_t start = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (L.mode == 0) {
        for (int64_t i = start; i < nA + nB; i += stride) {
            const bool isA = i < nA;                      // nA, nB are multiples of 4 (k % 32 == 0)
            const int64_t off = isA ? i : i - nA;
            const float* const* ptrs = isA ? L.A_ptrs : L.B_ptrs;
            f32x4 acc = *reinterpret_cast<const f32x4*>(ptrs[0] + off);
            for (int g = 1; g < G; ++g) acc += *reinterpret_cast<const f32x4*>(ptrs[g] + off);
            acc *= inv;
            *reinterpret_cast<f32x4*>((isA ? L.Abar : L.Bbar) + off) = acc;
        }
    } else {
        const int K = L.K;
        for (int64_t i = start; i < (nA + nB) * G; i += stride) {
            const int64_t per = nA + nB;
            const int g = (int)(i / per);
            const int64_t j = i - (int64_t)g * per;
            if (j < nA) {         // Abar[row][g*k + c] = A_g[row][c] / G
                const int64_t row = j / L.k, c = j % L.k;
                f32x4 v = *reinterpret_cast<const f32x4*>(L.A_ptrs[g] + j);
                v *= inv;
                *reinterpret_cast<f32x4*>(L.Abar + row * K + (int64_t)g * L.k + c) = v;
            } else {              // Bbar[g*k + c][:] = B_g[c][:]
                const int64_t off = j - nA;
                const f32x4 v = *reinterpret_cast<const f32x4*>(L.B_ptrs[g] + off);
                *reinterpret_cast<f32x4*>(L.Bbar + (int64_t)g * nB + off) = v;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Stage 2: Gram matrices in fp64 from fp32 data.  One work-group owns one 64 x 64 tile of the
// lower triangle and walks the whole contraction length, so the sums have a fixed order.
//   which = 0: G_A = Abar^T Abar (contraction over the m rows; stored into LA)
//   which = 1: G_B = Bbar Bbar^T (contraction over the n columns; stored into GB and LB)
// ------------------------------------------------------------------------------------------
struct GramTile { int layer, which, ti, tj; };

__global__ __launch_bounds__(256) void gram_kernel(const LayerDev* __restrict__ layers,
                                                   const GramTile* __restrict__ tiles) {
    __shared__ float As[16][68];
    __shared__ float Bs[16][68];
    const GramTile gt = tiles[blockIdx.x];
    const LayerDev& L = layers[gt.layer];
    const int K = L.K;
    const int i0 = gt.ti * 64, j0 = gt.tj * 64;
    const int len = gt.which == 0 ? L.m : L.n;
    const float* src = gt.which == 0 ? L.Abar : L.Bbar;
    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;

    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;

    for (int c0 = 0; c0 < len; c0 += 16) {
        // slab element (kk, x): which == 0 -> Abar[c0+kk][i0+x]; which == 1 -> Bbar[i0+x][c0+kk]
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int lin = e * 256 + t;
            int kk, x;
            if (gt.which == 0) { kk = lin >> 6; x = lin & 63; } else { x = lin >> 4; kk = lin & 15; }
            const int c = c0 + kk;
            float va = 0.0f, vb = 0.0f;
            if (c < len) {
                if (gt.which == 0) {
                    if (i0 + x < K) va = src[(int64_t)c * K + i0 + x];
                    if (j0 + x < K) vb = src[(int64_t)c * K + j0 + x];
                } else {
                    if (i0 + x < K) va = src[(int64_t)(i0 + x) * len + c];
                    if (j0 + x < K) vb = src[(int64_t)(j0 + x) * len + c];
                }
            }
            As[kk][x] = va;
            Bs[kk][x] = vb;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            double a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = (double)As[kk][ty * 4 + u]; b[u] = (double)Bs[kk][tx * 4 + u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fma(a[u], b[v], acc[u][v]);
        }
        __syncthreads();
    }
    double* out0 = gt.which == 0 ? L.LA : L.GB;
    double* out1 = gt.which == 0 ? nullptr : L.LB;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = i0 + ty * 4 + u, j = j0 + tx * 4 + v;
            if (i < K && j < K) {
                out0[(int64_t)i * K + j] = acc[u][v];
                out0[(int64_t)j * K + i] = acc[u][v];
                if (out1) { out1[(int64_t)i * K + j] = acc[u][v]; out1[(int64_t)j * K + i] = acc[u][v]; }
            }
        }
}

// ------------------------------------------------------------------------------------------
// Stage 3: Cholesky G = L L^T in place (lower triangle; the strict upper triangle is zeroed),
// blocked left-looking, one work-group per matrix.  Positive SEMI-definite input is allowed:
// a pivot that drops below 1e-14 * max diag(G) marks a direction already spanned by earlier
// columns; its column of L is set to zero (L L^T = G still holds to that accuracy).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cholesky_kernel(const LayerDev* __restrict__ layers) {
    __shared__ double Ljj[32][33];
    __shared__ double Lrow[32][33];
    __shared__ double red[256];
    const LayerDev& L = layers[blockIdx.x >> 1];
    double* Gm = (blockIdx.x & 1) ? L.LB : L.LA;
    const int K = L.K;
    const int t = threadIdx.x;

    double mx = 0.0, tr = 0.0;
    for (int i = t; i < K; i += 256) { const double d = Gm[(int64_t)i * K + i]; mx = fmax(mx, d); tr += d; }
    red[t] = mx;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s) red[t] = fmax(red[t], red[t + s]);
        __syncthreads();
    }
    const double floor_piv = red[0] * 1e-14;
    __syncthreads();
    red[t] = tr;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s) red[t] += red[t + s];
        __syncthreads();
    }
    if (t == 0) L.trace[blockIdx.x & 1] = red[0];
    __syncthreads();

    for (int j0 = 0; j0 < K; j0 += 32) {
        // (a) panel update: rows i >= j0, columns j0..j0+31, subtract the contribution of columns < j0
        for (int ibase = j0; ibase < K; ibase += 256) {
            const int i = ibase + t;
            double acc[32];
            if (i < K) {
#pragma unroll
                for (int c = 0; c < 32; ++c) acc[c] = Gm[(int64_t)i * K + j0 + c];
            }
            for (int t0 = 0; t0 < j0; t0 += 32) {
                __syncthreads();
                for (int e = t; e < 32 * 32; e += 256) Lrow[e >> 5][e & 31] = Gm[(int64_t)(j0 + (e >> 5)) * K + t0 + (e & 31)];
                __syncthreads();
                if (i < K) {
                    for (int tt = 0; tt < 32; ++tt) {
                        const double li = Gm[(int64_t)i * K + t0 + tt];
#pragma unroll
                        for (int c = 0; c < 32; ++c) acc[c] = fma(-li, Lrow[c][tt], acc[c]);
                    }
                }
            }
            if (i < K) {
#pragma unroll
                for (int c = 0; c < 32; ++c) Gm[(int64_t)i * K + j0 + c] = acc[c];
            }
        }
        __threadfence_block();
        __syncthreads();
        // (b) factor the 32 x 32 diagonal block in LDS
        for (int e = t; e < 32 * 32; e += 256) Ljj[e >> 5][e & 31] = Gm[(int64_t)(j0 + (e >> 5)) * K + j0 + (e & 31)];
        __syncthreads();
        if (t < 64) {
            const int r = t & 31;  // lanes 0..31 work, 32..63 idle (one wave keeps the steps in lockstep)
            for (int c = 0; c < 32; ++c) {
                const double d = Ljj[c][c];
                const bool ok = d > floor_piv;
                const double piv = ok ? sqrt(d) : 0.0;
                double v = 0.0;
                if (t < 32 && r >= c) v = (r == c) ? piv : (ok ? Ljj[r][c] / piv : 0.0);
                // one wave in lockstep: the fences only pin the order of the LDS accesses
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                __builtin_amdgcn_wave_barrier();
                if (t < 32 && r >= c) Ljj[r][c] = v;
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                __builtin_amdgcn_wave_barrier();
                if (t < 32 && r > c) {
                    for (int cc = c + 1; cc <= r; ++cc) Ljj[r][cc] -= v * Ljj[cc][c];
                }
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
        __syncthreads();
        // (c) write the diagonal block back (upper part zero) and solve the rows below
        for (int e = t; e < 32 * 32; e += 256) {
            const int r = e >> 5, c = e & 31;
            Gm[(int64_t)(j0 + r) * K + j0 + c] = (c <= r) ? Ljj[r][c] : 0.0;
        }
        for (int i = j0 + 32 + t; i < K; i += 256) {
            double x[32];
#pragma unroll
            for (int c = 0; c < 32; ++c) x[c] = Gm[(int64_t)i * K + j0 + c];
#pragma unroll
            for (int c = 0; c < 32; ++c) {
                double v = x[c];
#pragma unroll
                for (int d = 0; d < c; ++d) v = fma(-x[d], Ljj[c][d], v);
                const double piv = Ljj[c][c];
                x[c] = piv > 0.0 ? v / piv : 0.0;
            }
#pragma unroll
            for (int c = 0; c < 32; ++c) Gm[(int64_t)i * K + j0 + c] = x[c];
        }
        // zero the strict upper triangle right of this block row
        for (int e = t; e < 32 * (K - j0 - 32); e += 256) {
            const int r = e / (K - j0 - 32), c = e % (K - j0 - 32);
            Gm[(int64_t)(j0 + r) * K + j0 + 32 + c] = 0.0;
        }
        __threadfence_block();
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// fp64 GEMM for the K x K stages (grouped):  C = op(A) . op(B) with optional row gather on
// op(A), per-row / per-column scaling, fp64 and/or fp32 output.
// Tile 64 x 64, 256 threads, 4 x 4 outputs per thread, vector fp64 FMA.
// ------------------------------------------------------------------------------------------
struct GemmF64 {
    const double* A; const double* B;
    double* C; float* C32;            // either may be NULL
    int P, Q, K;
    int lda, ldb, ldc, ldc32;
    int transA, transB;               // as in GemmF32
    const int* row_gather;            // op(A) row i is read at row row_gather[i] (transA == 0 only)
    const double* row_scale32;        // C32[i][j] = row_scale32[i] * acc (NULL = 1)
    const double* col_scale32;        // C32[i][j] *= col_scale32[j]      (NULL = 1)
    const int32_t* limit; int limit_rows;  // tiles at or beyond *limit produce zeros
    int tile_begin, tiles_q;
};

__global__ __launch_bounds__(256) void gemm_f64_kernel(const GemmF64* __restrict__ descs, int ndesc) {
    __shared__ double As[16][68];
    __shared__ double Bs[16][68];
    int lo = 0, hi = ndesc - 1;
    const int tile = blockIdx.x;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (descs[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
    }
    const GemmF64 d = descs[lo];
    const int local = tile - d.tile_begin;
    const int i0 = (local / d.tiles_q) * 64, j0 = (local % d.tiles_q) * 64;
    const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
    const int lim = d.limit ? *d.limit : 0;
    const bool dead = d.limit && (d.limit_rows ? (i0 >= lim) : (j0 >= lim));

    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;

    if (!dead) {
        for (int k0 = 0; k0 < d.K; k0 += 16) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int lin = e * 256 + t;
                {
                    int kk, x;
                    if (d.transA) { kk = lin >> 6; x = lin & 63; } else { x = lin >> 4; kk = lin & 15; }
                    double v = 0.0;
                    if (i0 + x < d.P && k0 + kk < d.K) {
                        if (d.transA) v = d.A[(int64_t)(k0 + kk) * d.lda + i0 + x];
                        else {
                            const int row = d.row_gather ? d.row_gather[i0 + x] : i0 + x;
                            v = d.A[(int64_t)row * d.lda + k0 + kk];
                        }
                    }
                    As[kk][x] = v;
                }
                {
                    int kk, x;
                    if (d.transB) { x = lin >> 4; kk = lin & 15; } else { kk = lin >> 6; x = lin & 63; }
                    double v = 0.0;
                    if (j0 + x < d.Q && k0 + kk < d.K)
                        v = d.transB ? d.B[(int64_t)(j0 + x) * d.ldb + k0 + kk] : d.B[(int64_t)(k0 + kk) * d.ldb + j0 + x];
                    Bs[kk][x] = v;
                }
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                double a[4], b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty * 4 + u]; b[u] = Bs[kk][tx * 4 + u]; }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[u][v] = fma(a[u], b[v], acc[u][v]);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = i0 + ty * 4 + u, j = j0 + tx * 4 + v;
            if (i < d.P && j < d.Q) {
                if (d.C) d.C[(int64_t)i * d.ldc + j] = acc[u][v];
                if (d.C32) {
                    double val = acc[u][v];
                    if (d.row_scale32) val *= d.row_scale32[i];
                    if (d.col_scale32) val *= d.col_scale32[j];
                    d.C32[(int64_t)i * d.ldc32 + j] = (float)val;
                }
            }
        }
}

// ||C||_F^2 per layer, the scale of the "numerically zero column" test: eight work-groups per
// layer leave eight partial sums, which the readers add in a fixed order.
__global__ __launch_bounds__(256) void frob2_kernel(const LayerDev* __restrict__ layers) {
    __shared__ double red[256];
    const LayerDev& L = layers[blockIdx.y];
    const int64_t n = (int64_t)L.K * L.K;
    double ss = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += 8 * 256) ss = fma(L.Ct[i], L.Ct[i], ss);
    red[threadIdx.x] = ss;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) L.trace[2 + blockIdx.x] = red[0];
}
// ------------------------------------------------------------------------------------------
// Stage 5: one-sided Jacobi on the columns of C, held as the rows of Ct (K x K, fp64).
// Columns are grouped in blocks of jb; a sweep = one intra-block pass (all pairs inside every
// block) + nb - 1 cross rounds of a round-robin tournament over the blocks, each round pairing
// every block with one partner and rotating all jb x jb cross pairs.
// One wave owns one column pair at a time: three dot products reduced with wave shuffles, then
// the plane rotation that makes the two columns orthogonal.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// NX = ceil(K / 64) upper bound (elements of one column per lane).
template <int NX>
__global__ __launch_bounds__(1024) void jacobi_cross_kernel(const LayerDev* __restrict__ layers,
                                                            const int2* __restrict__ wg_map,
                                                            int sweep, int round) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    double* right = reinterpret_cast<double*>(lds_raw);   // [jb][K]
    const int2 wm = wg_map[blockIdx.x];                   // (layer, pair slot)
    const LayerDev& L = layers[wm.x];
    if (sweep_finished(L, sweep)) return;
    const int nb = L.nb, jb = L.jb, K = L.K;
    if (round >= nb - 1) return;
    // circle method: slot 0 pairs block nb-1 with `round`; slot j pairs (round + j) with (round - j)
    int bI, bJ;
    if (wm.y == 0) { bI = nb - 1; bJ = round; }
    else { bI = (round + wm.y) % (nb - 1); bJ = (round - wm.y + (nb - 1)) % (nb - 1); }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave >= jb) return;   // (block size equals jb waves; kept for safety)

    double* left_col = L.Ct + (int64_t)(bI * jb + wave) * K;
    double* right_blk = L.Ct + (int64_t)(bJ * jb) * K;
    double x[NX];
#pragma unroll
    for (int e = 0; e < NX; ++e) { const int r = lane + 64 * e; x[e] = r < K ? left_col[r] : 0.0; }
    for (int r = lane; r < K; r += 64) right[wave * K + r] = right_blk[(int64_t)wave * K + r];
    __syncthreads();

    const double floor2 = kZeroColumn2 * frob2(L);
    bool any_signif = false;
    for (int step = 0; step < jb; ++step) {
        double* ycol = right + ((wave + step) % jb) * K;
        double y[NX];
        double alpha = 0.0, beta = 0.0, gamma = 0.0;
#pragma unroll
        for (int e = 0; e < NX; ++e) {
            const int r = lane + 64 * e;
            y[e] = r < K ? ycol[r] : 0.0;
            alpha = fma(x[e], x[e], alpha);
            beta = fma(y[e], y[e], beta);
            gamma = fma(x[e], y[e], gamma);
        }
        alpha = wave_sum(alpha); beta = wave_sum(beta); gamma = wave_sum(gamma);
        double c, s; bool signif;
        if (jacobi_rotation(alpha, beta, gamma, floor2, c, s, signif)) {
#pragma unroll
            for (int e = 0; e < NX; ++e) {
                const int r = lane + 64 * e;
                const double xn = c * x[e] - s * y[e];
                const double yn = s * x[e] + c * y[e];
                x[e] = xn;
                if (r < K) ycol[r] = yn;
            }
        }
        any_signif |= signif;
        __syncthreads();
    }
#pragma unroll
    for (int e = 0; e < NX; ++e) { const int r = lane + 64 * e; if (r < K) left_col[r] = x[e]; }
    for (int r = lane; r < K; r += 64) right_blk[(int64_t)wave * K + r] = right[wave * K + r];
    if (any_signif && lane == 0) L.rotated[sweep] = 1;
}

// All pairs inside one block of jb columns (jb even): jb - 1 rounds of jb / 2 disjoint pairs.
template <int NX>
__global__ __launch_bounds__(512) void jacobi_intra_kernel(const LayerDev* __restrict__ layers,
                                                           const int2* __restrict__ wg_map, int sweep) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    double* cols = reinterpret_cast<double*>(lds_raw);    // [jb][K]
    const int2 wm = wg_map[blockIdx.x];                   // (layer, block)
    const LayerDev& L = layers[wm.x];
    if (sweep_finished(L, sweep)) return;
    const int jb = L.jb, K = L.K;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave >= jb / 2) return;
    double* blk = L.Ct + (int64_t)(wm.y * jb) * K;
    for (int cidx = wave; cidx < jb; cidx += jb / 2)
        for (int r = lane; r < K; r += 64) cols[cidx * K + r] = blk[(int64_t)cidx * K + r];
    __syncthreads();
    const double floor2 = kZeroColumn2 * frob2(L);
    bool any_signif = false;
    for (int round = 0; round < jb - 1; ++round) {
        int p, q;
        if (wave == 0) { p = jb - 1; q = round; }
        else { p = (round + wave) % (jb - 1); q = (round - wave + (jb - 1)) % (jb - 1); }
        double* xc = cols + p * K;
        double* yc = cols + q * K;
        double x[NX], y[NX];
        double alpha = 0.0, beta = 0.0, gamma = 0.0;
#pragma unroll
        for (int e = 0; e < NX; ++e) {
            const int r = lane + 64 * e;
            x[e] = r < K ? xc[r] : 0.0;
            y[e] = r < K ? yc[r] : 0.0;
            alpha = fma(x[e], x[e], alpha);
            beta = fma(y[e], y[e], beta);
            gamma = fma(x[e], y[e], gamma);
        }
        alpha = wave_sum(alpha); beta = wave_sum(beta); gamma = wave_sum(gamma);
        double c, s; bool signif;
        if (jacobi_rotation(alpha, beta, gamma, floor2, c, s, signif)) {
#pragma unroll
            for (int e = 0; e < NX; ++e) {
                const int r = lane + 64 * e;
                if (r < K) { xc[r] = c * x[e] - s * y[e]; yc[r] = s * x[e] + c * y[e]; }
            }
        }
        any_signif |= signif;
        __syncthreads();
    }
    for (int cidx = wave; cidx < jb; cidx += jb / 2) {
        double ss = 0.0;
        for (int r = lane; r < K; r += 64) {
            const double v = cols[cidx * K + r];
            blk[(int64_t)cidx * K + r] = v;
            ss = fma(v, v, ss);
        }
        ss = wave_sum(ss);
        if (lane == 0) L.nrm[wm.y * jb + cidx] = ss;       // refreshed from the data once per sweep
    }
    if (any_signif && lane == 0) L.rotated[sweep] = 1;
}

// ------------------------------------------------------------------------------------------
// Stage 6: singular values = column norms, sorted descending; rank rule; scale vectors.
// One work-group per layer.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void finalize_kernel(const LayerDev* __restrict__ layers, int max_sweeps) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const LayerDev& L = layers[blockIdx.x];
    const int K = L.K;
    int n2 = 1;
    while (n2 < K) n2 <<= 1;
    double* key = reinterpret_cast<double*>(lds_raw);      // [n2]
    int* idx = reinterpret_cast<int*>(key + n2);           // [n2]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;

    for (int c = wave; c < n2; c += 4) {
        double ss = 0.0;
        if (c < K) {
            const double* col = L.Ct + (int64_t)c * K;
            for (int r = lane; r < K; r += 64) ss = fma(col[r], col[r], ss);
            ss = wave_sum(ss);
        }
        if (lane == 0) { key[c] = c < K ? sqrt(ss) : -1.0; idx[c] = c; }
    }
    __syncthreads();
    // bitonic sort, descending by key (ties: lower original index first)
    for (int size = 2; size <= n2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = t; i < n2; i += 256) {
                const int j = i ^ stride;
                if (j > i) {
                    const bool desc = (i & size) == 0;
                    const double ki = key[i], kj = key[j];
                    const int ii = idx[i], ij = idx[j];
                    const bool i_first = (ki > kj) || (ki == kj && ii < ij);
                    if (desc ? !i_first : i_first) { key[i] = kj; key[j] = ki; idx[i] = ij; idx[j] = ii; }
                }
            }
            __syncthreads();
        }
    }
    // rank rule in fp32: keep sigma_i iff (float)sigma_i >= tau * (float)sigma_1
    __shared__ int count;
    if (t == 0) count = 0;
    __syncthreads();
    const float s1 = (float)key[0];
    const float cut = L.tau * s1;
    int mine = 0;
    for (int i = t; i < K; i += 256) mine += ((float)key[i] >= cut) ? 1 : 0;
    atomicAdd(&count, mine);
    __syncthreads();
    int kp = L.k_fixed > 0 ? L.k_fixed : (count < 1 ? 1 : count);
    if (kp > K) kp = K;
    if (kp > L.k_cap) kp = L.k_cap;
    const double floor_sig = key[0] * kSigmaFloor;
    for (int i = t; i < L.k_cap; i += 256) {
        const double sg = i < K ? key[i] : 0.0;
        L.S_out[i] = (float)sg;
        if (i < K) {
            const bool live = i < kp && sg > floor_sig && sg > 0.0;
            const double rs = live ? 1.0 / sqrt(sg) : 0.0;   // sigma^(-1/2)
            L.s3[i] = live ? rs / sg : 0.0;                  // sigma^(-3/2)
            L.s5[i] = live ? rs / (sg * sg) : 0.0;           // sigma^(-5/2)
        }
    }
    for (int i = t; i < K; i += 256) { L.sigma[i] = key[i]; L.perm[i] = idx[i]; }
    if (t == 0) {
        *L.k_out = kp;
        int sweeps = max_sweeps, conv = 0;
        for (int s = 0; s < max_sweeps; ++s)
            if (L.rotated[s] == 0) { sweeps = s + 1; conv = 1; break; }
        L.info[0] = sweeps; L.info[1] = K; L.info[2] = conv; L.info[3] = kp;
    }
}

// ------------------------------------------------------------------------------------------
// host-side plan
// ------------------------------------------------------------------------------------------
struct Plan {
    int L = 0;
    size_t off_info = 0, off_layers = 0, off_ptrs = 0, off_gram_tiles = 0, off_wg_cross = 0,
           off_wg_intra = 0, off_gemm64 = 0, off_gemm32 = 0, off_rotated = 0, off_data = 0, total = 0;
    int n_gram_tiles = 0, n_wg_cross = 0, n_wg_intra = 0, n_gemm64 = 0, n_gemm32 = 0, n_ptrs = 0;
    int nb_max = 0, K_max = 0, jb_max = 0;
    size_t lds_jacobi = 0;  // largest jb * K * 8 over the layers
    struct PerLayer {
        int K, jb, nb;
        size_t Abar, Bbar, LA, GB, LB, Ct, Yt, sigma, s3, s5, trace, nrm, perm, PA, PB;
    };
    std::vector<PerLayer> pl;
};

int jacobi_block(int K) { return K <= 768 ? 16 : (K <= 1024 ? 8 : 4); }

Plan make_plan(const abt_merge_desc* layers, int L) {
    Plan p;
    p.L = L;
    p.pl.resize(L);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    p.off_info = take(sizeof(int) * kInfoInts * L);
    p.off_layers = take(sizeof(LayerDev) * L);
    for (int l = 0; l < L; ++l) {
        const abt_merge_desc& d = layers[l];
        const int K = (int)(d.mode == 0 ? d.k : d.k * d.G);
        Plan::PerLayer& q = p.pl[l];
        q.K = K; q.jb = jacobi_block(K); q.nb = K / q.jb;
        p.n_ptrs += 2 * d.G;
        const int T = (K + 63) / 64;
        p.n_gram_tiles += 2 * (T * (T + 1) / 2);
        p.n_wg_cross += q.nb / 2;
        p.n_wg_intra += q.nb;
        if (q.nb > p.nb_max) p.nb_max = q.nb;
        if (K > p.K_max) p.K_max = K;
        if (q.jb > p.jb_max) p.jb_max = q.jb;
        if (sizeof(double) * q.jb * K > p.lds_jacobi) p.lds_jacobi = sizeof(double) * q.jb * K;
        p.n_gemm64 += 1;                        // per stage: one problem per layer
        p.n_gemm32 += 2 + (d.W_out ? 1 : 0);
    }
    p.off_ptrs = take(sizeof(void*) * p.n_ptrs);
    p.off_gram_tiles = take(sizeof(GramTile) * p.n_gram_tiles);
    p.off_wg_cross = take(sizeof(int2) * p.n_wg_cross);
    p.off_wg_intra = take(sizeof(int2) * p.n_wg_intra);
    p.off_gemm64 = take(sizeof(GemmF64) * p.n_gemm64 * 3);   // three fp64 stages, staged up front
    p.off_gemm32 = take(gemm_f32_desc_bytes() * p.n_gemm32);
    p.off_rotated = take(sizeof(int) * (kMaxSweepsCap + 1) * L);
    p.off_data = off;
    for (int l = 0; l < L; ++l) {
        const abt_merge_desc& d = layers[l];
        Plan::PerLayer& q = p.pl[l];
        const size_t K = q.K, kc = (size_t)d.k_cap;
        q.Abar = take(sizeof(float) * d.m * K);
        q.Bbar = take(sizeof(float) * K * d.n);
        q.LA = take(sizeof(double) * K * K);
        q.GB = take(sizeof(double) * K * K);
        q.LB = take(sizeof(double) * K * K);
        q.Ct = take(sizeof(double) * K * K);
        q.Yt = take(sizeof(double) * K * K);
        q.sigma = take(sizeof(double) * K);
        q.s3 = take(sizeof(double) * K);
        q.s5 = take(sizeof(double) * K);
        q.trace = take(sizeof(double) * 10);
        q.nrm = take(sizeof(double) * K);
        q.perm = take(sizeof(int) * K);
        q.PA = take(sizeof(float) * K * kc);
        q.PB = take(sizeof(float) * kc * K);
    }
    p.total = off;
    return p;
}

template <int NX>
hipError_t launch_jacobi_sweep(const Plan& p, const LayerDev* dl, const int2* cross, const int2* intra,
                               int sweep, hipStream_t s) {
    const size_t lds_cross = p.lds_jacobi;
    static size_t attr_bytes = 0;
    if (lds_cross > attr_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&jacobi_cross_kernel<NX>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_cross);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&jacobi_intra_kernel<NX>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_cross);
        if (e != hipSuccess) return e;
        attr_bytes = lds_cross;
    }
    hipLaunchKernelGGL(jacobi_intra_kernel<NX>, dim3(p.n_wg_intra), dim3(64 * (p.jb_max / 2)), lds_cross, s,
                       dl, intra, sweep);
    for (int round = 0; round < p.nb_max - 1; ++round)
        hipLaunchKernelGGL(jacobi_cross_kernel<NX>, dim3(p.n_wg_cross), dim3(64 * p.jb_max), lds_cross, s,
                           dl, cross, sweep, round);
    return hipGetLastError();
}


// ---- layer groups on side streams -----------------------------------------------------------
// One round of the block Jacobi iteration is a chain load -> Gram -> rotations -> update -> store,
// and all work-groups of a launch walk through it side by side: memory, matrix cores and LDS take
// turns instead of working together.  The layers are independent of each other, so they are split
// into up to four groups, each with a stream of its own (the caller's stream carries the first
// group); the groups drift apart and their phases overlap (measured on config 5: 58 -> 38 us per
// round of all 48 layers).  The streams have the default priority, are created once per process
// and are joined back into the caller's stream before merge_run returns.
constexpr int kMaxGroups = 4;
std::atomic<int> g_merge_groups{0};   // 0: as many as allowed; n: at most n groups (measurement switch)
struct SideStreams {
    hipStream_t stream[kMaxGroups - 1] = {};
    hipEvent_t fork = nullptr, join[kMaxGroups - 1] = {};
    hipEvent_t polled[kMaxGroups][2] = {};   // "the flags of sweep s have reached the host", per group, two in flight
    int* flags_host = nullptr;               // pinned: the device-to-host copies of the flags are asynchronous
    size_t flags_cap = 0;                    // ints
    int device = -1;
    bool ok = false;
};
std::mutex g_side_mutex;     // one batched merge at a time uses the side streams
SideStreams g_side;

bool pinned_flags_ready(size_t ints) {
    if (g_side.flags_cap >= ints) return true;
    if (g_side.flags_host) { (void)hipHostFree(g_side.flags_host); g_side.flags_host = nullptr; g_side.flags_cap = 0; }
    if (hipHostMalloc((void**)&g_side.flags_host, sizeof(int) * ints, hipHostMallocDefault) != hipSuccess) {
        g_side.flags_host = nullptr;
        return false;
    }
    g_side.flags_cap = ints;
    return true;
}

bool side_streams_ready() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (g_side.ok && g_side.device == dev) return true;
    if (g_side.ok) return false;             // created for another device: run on the caller's stream only
    SideStreams t;
    for (int i = 0; i < kMaxGroups - 1; ++i) {
        if (hipStreamCreateWithFlags(&t.stream[i], hipStreamNonBlocking) != hipSuccess) return false;
        if (hipEventCreateWithFlags(&t.join[i], hipEventDisableTiming) != hipSuccess) return false;
    }
    if (hipEventCreateWithFlags(&t.fork, hipEventDisableTiming) != hipSuccess) return false;
    for (int g = 0; g < kMaxGroups; ++g)
        for (int i = 0; i < 2; ++i)
            if (hipEventCreateWithFlags(&t.polled[g][i], hipEventDisableTiming) != hipSuccess) return false;
    t.device = dev; t.ok = true;
    g_side = t;
    return true;
}

}  // namespace

size_t merge_workspace_bytes(const abt_merge_desc* layers, int L) { return make_plan(layers, L).total; }

int merge_set_groups(int n) { return g_merge_groups.exchange(n < 0 ? 0 : n); }

hipError_t launch_identity_f32(float* dst, int K, hipStream_t s) {
    const int64_t n = (int64_t)K * K;
    hipLaunchKernelGGL(identity_f32_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, dst, K);
    return hipGetLastError();
}

hipError_t merge_read_info(const void* workspace, int layer, int32_t out[4], hipStream_t s) {
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) return e;
    return hipMemcpy(out, (const char*)workspace + sizeof(int) * kInfoInts * layer,
                     sizeof(int) * kInfoInts, hipMemcpyDeviceToHost);
}

hipError_t merge_run(const abt_merge_desc* layers, int L, void* workspace, int max_sweeps, hipStream_t s) {
    const Plan p = make_plan(layers, L);
    char* ws = (char*)workspace;
    if (max_sweeps > kMaxSweepsCap) max_sweeps = kMaxSweepsCap;
    if (max_sweeps < 1) max_sweeps = 1;

    // ---- host images of the header tables
    std::vector<LayerDev> hl(L);
    std::vector<const float*> hptrs(p.n_ptrs);
    std::vector<GramTile> gtiles; gtiles.reserve(p.n_gram_tiles);
    std::vector<int2> wcross; wcross.reserve(p.n_wg_cross);
    std::vector<int2> wintra; wintra.reserve(p.n_wg_intra);
    std::vector<GemmF64> g64(p.n_gemm64 * 3);
    std::vector<GemmF32> g32; g32.reserve(p.n_gemm32);
    const float* const* dptrs = (const float* const*)(ws + p.off_ptrs);
    int ptr_cursor = 0;
    int tb0 = 0, tb1 = 0, tb2 = 0;
    for (int l = 0; l < L; ++l) {
        const abt_merge_desc& d = layers[l];
        const Plan::PerLayer& q = p.pl[l];
        LayerDev& v = hl[l];
        v.A_ptrs = dptrs + ptr_cursor;
        for (int g = 0; g < d.G; ++g) hptrs[ptr_cursor + g] = d.A_copies[g];
        ptr_cursor += d.G;
        v.B_ptrs = dptrs + ptr_cursor;
        for (int g = 0; g < d.G; ++g) hptrs[ptr_cursor + g] = d.B_copies[g];
        ptr_cursor += d.G;
        v.G = d.G; v.mode = d.mode; v.m = (int)d.m; v.n = (int)d.n; v.k = (int)d.k; v.K = q.K;
        v.k_cap = (int)d.k_cap; v.k_fixed = (int)d.k_fixed; v.tau = d.tau;
        v.jb = q.jb; v.nb = q.nb;
        v.Abar = (float*)(ws + q.Abar); v.Bbar = (float*)(ws + q.Bbar);
        v.LA = (double*)(ws + q.LA); v.GB = (double*)(ws + q.GB); v.LB = (double*)(ws + q.LB);
        v.Ct = (double*)(ws + q.Ct); v.Yt = (double*)(ws + q.Yt);
        v.sigma = (double*)(ws + q.sigma); v.s3 = (double*)(ws + q.s3); v.s5 = (double*)(ws + q.s5);
        v.trace = (double*)(ws + q.trace);
        v.nrm = (double*)(ws + q.nrm);
        v.perm = (int*)(ws + q.perm);
        v.PA = (float*)(ws + q.PA); v.PB = (float*)(ws + q.PB);
        v.rotated = (int*)(ws + p.off_rotated) + (size_t)l * (kMaxSweepsCap + 1);
        v.info = (int*)(ws + p.off_info) + (size_t)l * kInfoInts;
        v.S_out = d.S_out; v.k_out = d.k_out;

        const int K = q.K, T = (K + 63) / 64;
        for (int which = 0; which < 2; ++which)
            for (int ti = 0; ti < T; ++ti)
                for (int tj = 0; tj <= ti; ++tj) gtiles.push_back(GramTile{l, which, ti, tj});
        for (int sidx = 0; sidx < q.nb / 2; ++sidx) wcross.push_back(make_int2(l, sidx));
        for (int b = 0; b < q.nb; ++b) wintra.push_back(make_int2(l, b));

        const int kc = (int)(d.k_cap < K ? d.k_cap : K);
        const int tq = (K + 63) / 64;
        // stage 4: Ct = L_B^T L_A   (Ct[j][i] = C[i][j], C = L_A^T L_B)
        GemmF64& a = g64[l];
        a = GemmF64{};
        a.A = v.LB; a.B = v.LA; a.C = v.Ct; a.P = K; a.Q = K; a.K = K;
        a.lda = K; a.ldb = K; a.ldc = K; a.transA = 1; a.transB = 0;
        a.tile_begin = tb0; a.tiles_q = tq; tb0 += tq * tq;
        // stage 7a: Yt[j][:] = (L_A c_perm(j))^T = Ct[perm(j)][:] L_A^T ; PB = diag(s3) Yt (fp32)
        GemmF64& b = g64[p.n_gemm64 + l];
        b = GemmF64{};
        b.A = v.Ct; b.B = v.LA; b.C = v.Yt; b.C32 = v.PB; b.P = kc; b.Q = K; b.K = K;
        b.lda = K; b.ldb = K; b.ldc = K; b.ldc32 = K; b.transA = 0; b.transB = 1;
        b.row_gather = v.perm; b.row_scale32 = v.s3; b.limit = d.k_out; b.limit_rows = 1;
        b.tile_begin = tb1; b.tiles_q = tq; tb1 += ((kc + 63) / 64) * tq;
        // stage 7b: PA = G_B Yt^T diag(s5)   (fp32 only)
        GemmF64& c = g64[2 * p.n_gemm64 + l];
        c = GemmF64{};
        c.A = v.GB; c.B = v.Yt; c.C32 = v.PA; c.P = K; c.Q = kc; c.K = K;
        c.lda = K; c.ldb = K; c.ldc32 = (int)d.k_cap; c.transA = 0; c.transB = 1;
        c.col_scale32 = v.s5; c.limit = d.k_out; c.limit_rows = 0;
        c.tile_begin = tb2; c.tiles_q = (kc + 63) / 64; tb2 += tq * ((kc + 63) / 64);
        // stage 8: back-projection (fp32 MFMA): A' = Abar PA, B' = PB Bbar, Wbar = Abar Bbar
        GemmF32 ga{};
        ga.A = v.Abar; ga.B = v.PA; ga.C = d.A_out; ga.P = (int)d.m; ga.Q = (int)d.k_cap; ga.K = K;
        ga.lda = K; ga.ldb = (int)d.k_cap; ga.ldc = (int)d.k_cap; ga.alpha = 1.0f;
        ga.limit = d.k_out; ga.limit_rows = 0;
        g32.push_back(ga);
        GemmF32 gb{};
        gb.A = v.PB; gb.B = v.Bbar; gb.C = d.B_out; gb.P = (int)d.k_cap; gb.Q = (int)d.n; gb.K = K;
        gb.lda = K; gb.ldb = (int)d.n; gb.ldc = (int)d.n; gb.alpha = 1.0f;
        gb.limit = d.k_out; gb.limit_rows = 1;
        g32.push_back(gb);
        if (d.W_out) {
            GemmF32 gw{};
            gw.A = v.Abar; gw.B = v.Bbar; gw.C = d.W_out; gw.P = (int)d.m; gw.Q = (int)d.n; gw.K = K;
            gw.lda = K; gw.ldb = (int)d.n; gw.ldc = (int)d.n; gw.alpha = 1.0f;
            g32.push_back(gw);
        }
    }

    // ---- upload the tables (pageable sources: staged by the runtime before each call returns)
    hipError_t e;
#define ABT_TRY(x) do { e = (x); if (e != hipSuccess) return e; } while (0)
    ABT_TRY(hipMemcpyAsync(ws + p.off_layers, hl.data(), sizeof(LayerDev) * L, hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_ptrs, hptrs.data(), sizeof(void*) * p.n_ptrs, hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_gram_tiles, gtiles.data(), sizeof(GramTile) * gtiles.size(), hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_wg_cross, wcross.data(), sizeof(int2) * wcross.size(), hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_wg_intra, wintra.data(), sizeof(int2) * wintra.size(), hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_gemm64, g64.data(), sizeof(GemmF64) * g64.size(), hipMemcpyHostToDevice, s));
    std::vector<char> g32img(gemm_f32_desc_bytes() * (g32.empty() ? 1 : g32.size()));
    const int tiles32 = gemm_f32_build_table(g32.data(), (int)g32.size(), g32img.data());
    ABT_TRY(hipMemcpyAsync(ws + p.off_gemm32, g32img.data(), gemm_f32_desc_bytes() * g32.size(), hipMemcpyHostToDevice, s));
    // the uploads must have left the host vectors before they are destroyed
    ABT_TRY(hipStreamSynchronize(s));

    const LayerDev* dl = (const LayerDev*)(ws + p.off_layers);
    {
        const int64_t n = (int64_t)(kMaxSweepsCap + 1) * L;
        hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s,
                           (int*)(ws + p.off_rotated), n, 0);
        // sweeps never run count as "nothing rotated" only if an earlier sweep converged; mark the
        // slots past the cap as dirty so finalize reports non-convergence correctly
    }
    hipLaunchKernelGGL(mean_kernel, dim3(64, L), dim3(256), 0, s, dl);
    hipLaunchKernelGGL(gram_kernel, dim3(p.n_gram_tiles), dim3(256), 0, s, dl,
                       (const GramTile*)(ws + p.off_gram_tiles));
    hipLaunchKernelGGL(cholesky_kernel, dim3(2 * L), dim3(256), 0, s, dl);
    const GemmF64* d64 = (const GemmF64*)(ws + p.off_gemm64);
    hipLaunchKernelGGL(gemm_f64_kernel, dim3(tb0), dim3(256), 0, s, d64, p.n_gemm64);
    hipLaunchKernelGGL(frob2_kernel, dim3(8, L), dim3(256), 0, s, dl);
    ABT_TRY(hipGetLastError());

    const int2* cross = (const int2*)(ws + p.off_wg_cross);
    const int2* intra = (const int2*)(ws + p.off_wg_intra);
    const int nx = (p.K_max + 63) / 64;
    std::vector<int> flags((size_t)(kMaxSweepsCap + 1) * L);
    auto converged = [&](int l, int sweep) {
        for (int q = 0; q <= sweep; ++q)
            if (flags[(size_t)l * (kMaxSweepsCap + 1) + q] == 0) return true;
        return false;
    };
    if (p.K_max <= 768) {
        // block form on the matrix cores, layers in groups (contiguous layer ranges with about the
        // same number of work-groups); wcross is layer-major, so a group is a slice of it
        std::unique_lock<std::mutex> lock(g_side_mutex);
        int ngroups = L < kMaxGroups ? L : kMaxGroups;
        if (g_merge_groups >= 1 && g_merge_groups < ngroups) ngroups = g_merge_groups;
        if (ngroups > 1 && !side_streams_ready()) ngroups = 1;
        struct Group { int l0, l1, wg0, wg1, rounds; bool done; hipStream_t s; };
        std::vector<Group> groups;
        {
            int l = 0, wg = 0;
            for (int g = 0; g < ngroups; ++g) {
                Group G{l, l, wg, wg, 0, false, g == 0 ? s : g_side.stream[g - 1]};
                const int target = (int)((int64_t)p.n_wg_cross * (g + 1) / ngroups);
                while (G.l1 < L && (G.wg1 < target || g == ngroups - 1)) {
                    G.wg1 += p.pl[G.l1].nb / 2;
                    if (p.pl[G.l1].nb - 1 > G.rounds) G.rounds = p.pl[G.l1].nb - 1;
                    ++G.l1;
                }
                l = G.l1; wg = G.wg1;
                if (G.l1 > G.l0) groups.push_back(G);
            }
        }
        if (groups.size() > 1) {
            ABT_TRY(hipEventRecord(g_side.fork, s));
            for (size_t g = 1; g < groups.size(); ++g) ABT_TRY(hipStreamWaitEvent(groups[g].s, g_side.fork, 0));
        }
        // The host learns whether a group has converged from its per-sweep flags.  Waiting for them
        // after every sweep would leave the GPU idle until the next sweep is enqueued, so the host
        // stays one sweep ahead: the flags of sweep s are copied to pinned memory behind that sweep,
        // sweep s + 1 is enqueued, and only then the host waits for the copy of sweep s and decides
        // about sweep s + 2.  (The launches of a sweep that turns out not to be needed exit at once.)
        const bool pipelined = side_streams_ready() && pinned_flags_ready(flags.size());
        hipError_t fail = hipSuccess;
        auto examine = [&](Group& G, int gi, int sweep) {       // flags of `sweep` have been copied
            if (G.done) return;
            if (pipelined) {
                fail = hipEventSynchronize(g_side.polled[gi][sweep & 1]);
                if (fail != hipSuccess) return;
            }
            const int* src = pipelined ? g_side.flags_host : flags.data();
            bool all_done = true;
            for (int l = G.l0; l < G.l1 && all_done; ++l) {
                bool done = false;
                for (int q = 0; q <= sweep; ++q) done |= src[(size_t)l * (kMaxSweepsCap + 1) + q] == 0;
                all_done = done;
            }
            G.done = all_done;
        };
        for (int sweep = 0; sweep < max_sweeps && fail == hipSuccess; ++sweep) {
            bool any = false;
            for (int round = 0; round < p.nb_max - 1 && fail == hipSuccess; ++round)
                for (Group& G : groups) {
                    if (G.done || round >= G.rounds) continue;
                    any = true;
                    fail = launch_jacobi_block_round(dl, cross + G.wg0, G.wg1 - G.wg0, p.K_max, sweep, round, G.s);
                    if (fail != hipSuccess) break;
                }
            if (!any || fail != hipSuccess) break;
            if (sweep + 1 >= max_sweeps) break;
            for (size_t gi = 0; gi < groups.size() && fail == hipSuccess; ++gi) {
                Group& G = groups[gi];
                if (G.done) continue;
                const size_t off = (size_t)G.l0 * (kMaxSweepsCap + 1);
                int* dst = pipelined ? g_side.flags_host : flags.data();
                fail = hipMemcpyAsync(dst + off, (const int*)(ws + p.off_rotated) + off,
                                      sizeof(int) * (kMaxSweepsCap + 1) * (G.l1 - G.l0), hipMemcpyDeviceToHost, G.s);
                if (fail == hipSuccess && pipelined) fail = hipEventRecord(g_side.polled[gi][sweep & 1], G.s);
                if (fail == hipSuccess && !pipelined) fail = hipStreamSynchronize(G.s);
            }
            // not pipelined: decide now; pipelined: decide on the sweep before this one
            const int look = pipelined ? sweep - 1 : sweep;
            if (look >= 1)
                for (size_t gi = 0; gi < groups.size() && fail == hipSuccess; ++gi) examine(groups[gi], (int)gi, look);
        }
        // join, also after an error: nothing of this call may stay behind on a side stream
        for (size_t g = 1; g < groups.size(); ++g) {
            hipError_t e2 = hipEventRecord(g_side.join[g - 1], groups[g].s);
            if (e2 == hipSuccess) e2 = hipStreamWaitEvent(s, g_side.join[g - 1], 0);
            if (e2 != hipSuccess) { hipStreamSynchronize(groups[g].s); if (fail == hipSuccess) fail = e2; }
        }
        if (fail != hipSuccess) return fail;
    } else {
        for (int sweep = 0; sweep < max_sweeps; ++sweep) {
            if (nx <= 16) ABT_TRY(launch_jacobi_sweep<16>(p, dl, cross, intra, sweep, s));
            else ABT_TRY(launch_jacobi_sweep<32>(p, dl, cross, intra, sweep, s));
            // A sweep is some hundred launches; once every layer has converged the remaining ones
            // would all exit at once.  Poll the per-sweep flags (a few KB) instead of issuing them.
            if (sweep >= 2 && sweep + 1 < max_sweeps) {
                ABT_TRY(hipMemcpyAsync(flags.data(), ws + p.off_rotated, sizeof(int) * flags.size(),
                                       hipMemcpyDeviceToHost, s));
                ABT_TRY(hipStreamSynchronize(s));
                bool all_done = true;
                for (int l = 0; l < L && all_done; ++l) all_done = converged(l, sweep);
                if (all_done) break;
            }
        }
    }
    int n2 = 1;
    while (n2 < p.K_max) n2 <<= 1;
    hipLaunchKernelGGL(finalize_kernel, dim3(L), dim3(256), (sizeof(double) + sizeof(int)) * n2, s, dl, max_sweeps);
    if (tb1 > 0) hipLaunchKernelGGL(gemm_f64_kernel, dim3(tb1), dim3(256), 0, s, d64 + p.n_gemm64, p.n_gemm64);
    if (tb2 > 0) hipLaunchKernelGGL(gemm_f64_kernel, dim3(tb2), dim3(256), 0, s, d64 + 2 * p.n_gemm64, p.n_gemm64);
    ABT_TRY(hipGetLastError());
    ABT_TRY(launch_gemm_f32_table(ws + p.off_gemm32, (int)g32.size(), tiles32, s));
#undef ABT_TRY
    return hipSuccess;
}

}  // namespace abt
