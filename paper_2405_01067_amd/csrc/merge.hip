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
// (from U_c Sigma = C V_c, V_c Sigma = C^T U_c and L L^T = G).  Everything K x K runs in fp64; the
// back-projection is fp32.  This file: the plan of a batched call (workspace layout, tables, stage
// order, layer groups on side streams), Cholesky, the K x K products and the finalisation; the
// average fused into the Gram kernel is in merge_gram.hip, the block Jacobi in merge_jacobi.hip.
//
// mode 1 (mean of reconstructions) uses the same pipeline on the concatenations
// Abar = [A_1 .. A_G] / G (m x Gk) and Bbar = [B_1; ..; B_G] (Gk x n).
#include <algorithm>
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
// Stage 3 for K <= kCholMaxK: the same factorisation, right-looking, with the panel in LDS and the
// trailing update on the fp64 matrix cores.  One work-group per matrix.  Per block column j0:
//   load the 32 x 32 diagonal block and the (K - j0 - 32) x 32 panel below it into LDS,
//   factor the diagonal block (one wave, 32 dependent steps), X = panel L_jj^(-T) (a thread per row),
//   write L's block column, and subtract X X^T from the lower triangle of the trailing matrix:
//   16 x 16 tiles, C tile from / to memory (L2), operands of v_mfma_f64_16x16x4 from the LDS panel.
// ------------------------------------------------------------------------------------------
constexpr int kCholMaxK = 544;     // (K - 32) x 34 doubles of panel: 136 KB
constexpr int kCholPitch = 34;     // doubles per panel row: 16 rows x 2 column groups of an operand read cover all banks

constexpr int kCholThreads = 256;  // (512 threads measured the same: the serial diagonal-block and row-solve phases dominate)

__global__ __launch_bounds__(kCholThreads) void cholesky_mfma_kernel(const LayerDev* __restrict__ layers) {
    constexpr int NT = kCholThreads;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const LayerDev& L = layers[blockIdx.x >> 1];
    double* Gm = (blockIdx.x & 1) ? L.LB : L.LA;
    const int K = L.K;
    if (K > kCholMaxK) return;
    double* Xp = reinterpret_cast<double*>(lds_raw);                 // [K - 32][kCholPitch]
    double (*Ljj)[33] = reinterpret_cast<double (*)[33]>(Xp + (size_t)(K > 32 ? K - 32 : 0) * kCholPitch);
    double* invp = &Ljj[0][0] + 32 * 33;                             // [32] reciprocal pivots (0: dropped column)
    double* red = invp + 32;                                         // [NT]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, n = lane & 15, kq = lane >> 4;

    double mx = 0.0, tr = 0.0;
    for (int i = t; i < K; i += NT) { const double d = gload(Gm + (int64_t)i * K + i); mx = fmax(mx, d); tr += d; }
    red[t] = mx;
    __syncthreads();
    for (int s = NT / 2; s > 0; s >>= 1) {
        if (t < s) red[t] = fmax(red[t], red[t + s]);
        __syncthreads();
    }
    const double floor_piv = red[0] * 1e-14;
    __syncthreads();
    red[t] = tr;
    __syncthreads();
    for (int s = NT / 2; s > 0; s >>= 1) {
        if (t < s) red[t] += red[t + s];
        __syncthreads();
    }
    if (t == 0) L.trace[blockIdx.x & 1] = red[0];
    __syncthreads();

    for (int j0 = 0; j0 < K; j0 += 32) {
        const int nr = K - j0 - 32;                  // rows below the diagonal block
        // ---- (1) diagonal block and panel -> LDS (rows of 256 bytes, coalesced)
        for (int e = t; e < 32 * 32; e += NT) Ljj[e >> 5][e & 31] = gload(Gm + (int64_t)(j0 + (e >> 5)) * K + j0 + (e & 31));
        // (eight 16-byte loads in flight per thread: a load that is stored to LDS right away costs a full
        // memory latency per loop trip)
        for (int e0 = 0; e0 < nr * 16; e0 += 8 * NT) {
            f64x2 buf[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + u * NT + t;
                const int ec = e < nr * 16 ? e : nr * 16 - 1;
                buf[u] = gload(reinterpret_cast<const f64x2*>(Gm + (int64_t)(j0 + 32 + (ec >> 4)) * K + j0 + 2 * (ec & 15)));
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + u * NT + t;
                if (e < nr * 16) *reinterpret_cast<f64x2*>(Xp + (e >> 4) * kCholPitch + 2 * (e & 15)) = buf[u];
            }
        }
        __syncthreads();
        // ---- (2) factor the diagonal block: one wave, lane r holds row r in registers; step c takes the
        // pivot and the finished column c from the other lanes with lane reads (no LDS, no waits)
        if (wave == 0) {
            const int r = lane & 31;
            double row[32];
#pragma unroll
            for (int c = 0; c < 32; ++c) row[c] = Ljj[r][c];
            auto lane_value = [](double v, int src) {
                const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
                const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
                return __hiloint2double(hi, lo);
            };
#pragma unroll
            for (int c = 0; c < 32; ++c) {
                const double d = lane_value(row[c], c);
                const bool ok = d > floor_piv;
                // 1 / sqrt(d): hardware estimate and two Newton steps (a square root and a division in
                // fp64 would be several times the rest of the step); the pivot itself is d / sqrt(d)
                const double dd = ok ? d : 1.0;
                double y = __builtin_amdgcn_rsq(dd);
                y = y * fma(-0.5 * dd, y * y, 1.5);
                y = y * fma(-0.5 * dd, y * y, 1.5);
                const double ip = ok ? y : 0.0;
                const double piv = ok ? dd * y : 0.0;
                const double v = (r == c) ? piv : (r > c ? row[c] * ip : 0.0);
                row[c] = v;
                if (lane == c) invp[c] = ip;
#pragma unroll
                for (int cc = c + 1; cc < 32; ++cc) row[cc] = fma(-v, lane_value(v, cc), row[cc]);
            }
            if (lane < 32) {
#pragma unroll
                for (int c = 0; c < 32; ++c) Ljj[r][c] = row[c];
            }
        }
        __syncthreads();
        // ---- (3) rows below: x = row L_jj^(-T), column by column so that the updates of a step are independent
        for (int r = t; r < nr; r += NT) {
            double x[32];
#pragma unroll
            for (int c = 0; c < 32; ++c) x[c] = Xp[r * kCholPitch + c];
#pragma unroll
            for (int c = 0; c < 32; ++c) {
                x[c] *= invp[c];
#pragma unroll
                for (int c2 = c + 1; c2 < 32; ++c2) x[c2] = fma(-x[c], Ljj[c2][c], x[c2]);
            }
#pragma unroll
            for (int c = 0; c < 32; ++c) Xp[r * kCholPitch + c] = x[c];
        }
        __syncthreads();
        // ---- (4) L's block column to memory: diagonal block (upper part zero), panel, zeros to the right
        for (int e = t; e < 32 * 32; e += NT) {
            const int r = e >> 5, c = e & 31;
            gstore(Gm + (int64_t)(j0 + r) * K + j0 + c, (c <= r) ? Ljj[r][c] : 0.0);
        }
        for (int e = t; e < nr * 16; e += NT)
            gstore(reinterpret_cast<f64x2*>(Gm + (int64_t)(j0 + 32 + (e >> 4)) * K + j0 + 2 * (e & 15)),
                   *reinterpret_cast<const f64x2*>(Xp + (e >> 4) * kCholPitch + 2 * (e & 15)));
        for (int e = t; e < 32 * nr; e += NT) {
            const int r = e / nr, c = e - r * nr;
            gstore(Gm + (int64_t)(j0 + r) * K + j0 + 32 + c, 0.0);
        }
        // ---- (5) trailing matrix, lower triangle: C(ti, tj) -= X(ti) X(tj)^T.  Lane l holds X[16 ti + l % 16][l / 16 + 4 s]
        // (s = 0..7) as A operand (negated) and the same of tile tj as B operand; the accumulator register v
        // is C[l / 16 + 4 v][l % 16] of the tile.
        const int T = nr >> 4;
        for (int ti = T - 1 - wave; ti >= 0; ti -= NT / 64) {
            double a[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) a[s] = -Xp[(16 * ti + n) * kCholPitch + 4 * s + kq];
            double* crow = Gm + (int64_t)(j0 + 32 + 16 * ti + kq) * K + j0 + 32 + n;
            // C tiles travel in groups of four, the next group's loads issued before the products of this
            // one: a load has 32 matrix instructions (about 2000 cycles) to come back from L2
            f64x4 cur[4], nxt[4];
            auto fetch4 = [&](f64x4 (&dst)[4], int base) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (base + u <= ti) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) dst[u][v] = gload(crow + (int64_t)(4 * v) * K + 16 * (base + u));
                    }
            };
            fetch4(cur, 0);
            for (int g0 = 0; g0 <= ti; g0 += 4) {
                if (g0 + 4 <= ti) fetch4(nxt, g0 + 4);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int tj = g0 + u;
                    if (tj <= ti) {
                        f64x4 acc = cur[u];
#pragma unroll
                        for (int s = 0; s < 8; ++s) {
                            const double b = Xp[(16 * tj + n) * kCholPitch + 4 * s + kq];
                            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[s], b, acc, 0, 0, 0);
                        }
#pragma unroll
                        for (int v = 0; v < 4; ++v) gstore(crow + (int64_t)(4 * v) * K + 16 * tj, acc[v]);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
            }
        }
        __threadfence_block();
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// fp64 GEMM for the K x K stages (grouped):  C = op(A) . op(B) with optional row gather on
// op(A), per-row / per-column scaling, fp64 and/or fp32 output.
// Tile 64 x 64, 256 threads = 4 waves of 32 x 32 (2 x 2 blocks of v_mfma_f64_16x16x4), slabs of 16
// staged through LDS, the next slab's global loads in flight during the products.
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

__global__ __launch_bounds__(256) void gemm_f64_kernel(const GemmF64* __restrict__ descs, int ndesc, int ntiles) {
    // k-major slabs of 16; pitch 80 doubles: the four 16-lane rows of an operand read (k, k + 1, ...)
    // start 160 words apart, i.e. in alternating halves of the 64 banks
    __shared__ double As[2][16][80];
    __shared__ double Bs[2][16][80];
    // Tiles are numbered problem by problem; block b works on tile (b % 8) * (grid / 8) + b / 8, so each
    // XCD (block index modulo 8) gets a contiguous eighth of the list: the tiles of one problem share
    // their operand panels through one L2 instead of pulling them into all eight.
    const int tile = (int)(blockIdx.x & 7) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3);
    if (tile >= ntiles) return;
    int lo = 0, hi = ndesc - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (descs[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
    }
    const GemmF64 d = descs[lo];
    const int local = tile - d.tile_begin;
    const int i0 = (local / d.tiles_q) * 64, j0 = (local % d.tiles_q) * 64;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, n = lane & 15, kq = lane >> 4;
    const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;      // this wave's 32 x 32 part of the tile
    const int lim = d.limit ? *d.limit : 0;
    const bool dead = d.limit && (d.limit_rows ? (i0 >= lim) : (j0 >= lim));

    // v_mfma_f64_16x16x4: A operand lane l = A[l % 16][l / 16], B operand = B[l / 16][l % 16],
    // accumulator register v of lane l = C[l / 16 + 4 v][l % 16]
    f64x4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};

    if (!dead) {
        // loads carry no predicate (indices are clamped into the matrices) so that none of them has
        // to be waited for before the next is issued; what was out of range is dropped when the slab
        // goes to LDS
        double ra[4], rb[4];
        bool oka[4], okb[4];
        // the rows of op(A) this thread fetches do not change from slab to slab: resolve the gather
        // once (inside the slab loop every index load would have to be waited for, and with it all
        // loads issued before)
        int rowA[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int lin = e * 256 + t;
            const int x = d.transA ? (lin & 63) : (lin >> 4);
            const int xi = i0 + x < d.P ? i0 + x : d.P - 1;
            rowA[e] = (!d.transA && d.row_gather) ? gload(d.row_gather + xi) : xi;
        }
        auto load_slab = [&](int k0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int lin = e * 256 + t;
                {
                    int kk, x;
                    if (d.transA) { kk = lin >> 6; x = lin & 63; } else { x = lin >> 4; kk = lin & 15; }
                    oka[e] = i0 + x < d.P && k0 + kk < d.K;
                    const int ki = k0 + kk < d.K ? k0 + kk : d.K - 1;
                    ra[e] = d.transA ? gload(d.A + (int64_t)ki * d.lda + rowA[e]) : gload(d.A + (int64_t)rowA[e] * d.lda + ki);
                }
                {
                    int kk, x;
                    if (d.transB) { x = lin >> 4; kk = lin & 15; } else { kk = lin >> 6; x = lin & 63; }
                    okb[e] = j0 + x < d.Q && k0 + kk < d.K;
                    const int xj = j0 + x < d.Q ? j0 + x : d.Q - 1, ki = k0 + kk < d.K ? k0 + kk : d.K - 1;
                    rb[e] = d.transB ? gload(d.B + (int64_t)xj * d.ldb + ki) : gload(d.B + (int64_t)ki * d.ldb + xj);
                }
            }
        };
        auto store_slab = [&](int b) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int lin = e * 256 + t;
                const double va = oka[e] ? ra[e] : 0.0, vb = okb[e] ? rb[e] : 0.0;
                if (d.transA) As[b][lin >> 6][lin & 63] = va; else As[b][lin & 15][lin >> 4] = va;
                if (d.transB) Bs[b][lin & 15][lin >> 4] = vb; else Bs[b][lin >> 6][lin & 63] = vb;
            }
        };
        // two LDS buffers, one barrier per slab: while slab s is multiplied out of buffer s % 2, slab
        // s + 1 (in registers since the iteration before) goes to the other buffer and the loads of
        // slab s + 2 are issued, so a load has two slabs of products to arrive
        const int nslab = (d.K + 15) / 16;
        load_slab(0);
        store_slab(0);
        if (nslab > 1) load_slab(16);
        __syncthreads();
        for (int sl = 0; sl < nslab; ++sl) {
            const int b = sl & 1;
            if (sl + 1 < nslab) {
                store_slab(b ^ 1);                       // everybody left buffer b ^ 1 before the last barrier
                if (sl + 2 < nslab) load_slab((sl + 2) * 16);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const double a0 = As[b][4 * q + kq][wi + n], a1 = As[b][4 * q + kq][wi + 16 + n];
                const double b0 = Bs[b][4 * q + kq][wj + n], b1 = Bs[b][4 * q + kq][wj + 16 + n];
                acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + wi + 16 * a + kq + 4 * v, j = j0 + wj + 16 * b + n;
                if (i < d.P && j < d.Q) {
                    const double val0 = acc[a][b][v];
                    if (d.C) d.C[(int64_t)i * d.ldc + j] = val0;
                    if (d.C32) {
                        double val = val0;
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
// The squared norms come from a launch of their own that spreads the K x K reads over the chip
// (one wave per column, four columns per work-group); the sort and the rank rule take one
// work-group per layer.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void colnorm_kernel(const LayerDev* __restrict__ layers) {
    const LayerDev& L = layers[blockIdx.y];
    const int K = L.K, lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= K) return;
    const double* col = L.Ct + (int64_t)c * K;
    double ss = 0.0;
    for (int r = lane; r < K; r += 64) { const double v = gload(col + r); ss = fma(v, v, ss); }
    ss = wave_sum(ss);
    if (lane == 0) L.nrm[c] = ss;
}

__global__ __launch_bounds__(256) void finalize_kernel(const LayerDev* __restrict__ layers, int max_sweeps) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const LayerDev& L = layers[blockIdx.x];
    const int K = L.K;
    int n2 = 1;
    while (n2 < K) n2 <<= 1;
    double* key = reinterpret_cast<double*>(lds_raw);      // [n2]
    int* idx = reinterpret_cast<int*>(key + n2);           // [n2]
    const int t = threadIdx.x;

    for (int c = t; c < n2; c += 256) { key[c] = c < K ? sqrt(L.nrm[c]) : -1.0; idx[c] = c; }
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
    size_t off_header = 0, off_info = 0, off_layers = 0, off_ptrs = 0, off_gram_tiles = 0, off_wg_cross = 0,
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

// Job list of the averaging + Gram stage.  The (layer, side) pairs are taken longest contraction
// first and dealt round-robin to the eight XCDs (block index modulo 8 picks the XCD); the tiles of
// one pair take consecutive slots of its XCD, so they run at about the same time on one L2.
// Returns the number of leading jobs that take the kernel with 16-byte loads; the rest (B sides with
// n % 4 != 0) follow.
int build_gram_jobs(const abt_merge_desc* layers, int L, std::vector<GramJob>& out) {
    struct Pair { int layer, which; int64_t len; int T; };
    std::vector<Pair> pairs;
    pairs.reserve(2 * (size_t)L);
    for (int l = 0; l < L; ++l) {
        const abt_merge_desc& d = layers[l];
        const int K = (int)(d.mode == 0 ? d.k : d.k * d.G);
        const int T = (K + 127) / 128;
        pairs.push_back(Pair{l, 0, d.m, T});
        if (d.n % 4 == 0) pairs.push_back(Pair{l, 1, d.n, T});
    }
    std::stable_sort(pairs.begin(), pairs.end(), [](const Pair& a, const Pair& b) {
        return a.len * a.T * (a.T + 1) > b.len * b.T * (b.T + 1);
    });
    std::vector<GramJob> per_xcd[8];
    for (size_t q = 0; q < pairs.size(); ++q) {
        // shortest list first keeps the XCDs level when the pairs differ in size
        int x = 0;
        for (int c = 1; c < 8; ++c) if (per_xcd[c].size() < per_xcd[x].size()) x = c;
        const Pair& pr = pairs[q];
        for (int ti = 0; ti < pr.T; ++ti)
            for (int tj = 0; tj <= ti; ++tj) per_xcd[x].push_back(GramJob{pr.layer, pr.which, ti, tj});
    }
    size_t slots = 0;
    for (int c = 0; c < 8; ++c) if (per_xcd[c].size() > slots) slots = per_xcd[c].size();
    out.assign(slots * 8, GramJob{-1, 0, 0, 0});
    for (int c = 0; c < 8; ++c)
        for (size_t i = 0; i < per_xcd[c].size(); ++i) out[i * 8 + c] = per_xcd[c][i];
    const int aligned = (int)out.size();
    for (int l = 0; l < L; ++l) {
        const abt_merge_desc& d = layers[l];
        if (d.n % 4 == 0) continue;
        const int K = (int)(d.mode == 0 ? d.k : d.k * d.G);
        const int T = (K + 127) / 128;
        for (int ti = 0; ti < T; ++ti)
            for (int tj = 0; tj <= ti; ++tj) out.push_back(GramJob{l, 1, ti, tj});
    }
    return aligned;
}

Plan make_plan(const abt_merge_desc* layers, int L) {
    Plan p;
    p.L = L;
    p.pl.resize(L);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    p.off_header = take(sizeof(int) * 4);                      // magic, L (merge_read_info bounds `layer` with it)
    p.off_info = take(sizeof(int) * kInfoInts * L);
    p.off_layers = take(sizeof(LayerDev) * L);
    for (int l = 0; l < L; ++l) {
        const abt_merge_desc& d = layers[l];
        const int K = (int)(d.mode == 0 ? d.k : d.k * d.G);
        Plan::PerLayer& q = p.pl[l];
        q.K = K; q.jb = jacobi_block(K); q.nb = K / q.jb;
        p.n_ptrs += 2 * d.G;
        p.n_wg_cross += q.nb / 2;
        p.n_wg_intra += q.nb;
        if (q.nb > p.nb_max) p.nb_max = q.nb;
        if (K > p.K_max) p.K_max = K;
        if (q.jb > p.jb_max) p.jb_max = q.jb;
        if (sizeof(double) * q.jb * K > p.lds_jacobi) p.lds_jacobi = sizeof(double) * q.jb * K;
        p.n_gemm64 += 1;                        // per stage: one problem per layer
        p.n_gemm32 += 2 + (d.W_out ? 1 : 0);
    }
    {
        std::vector<GramJob> jobs;
        build_gram_jobs(layers, L, jobs);
        p.n_gram_tiles = (int)jobs.size();
    }
    p.off_ptrs = take(sizeof(void*) * p.n_ptrs);
    p.off_gram_tiles = take(sizeof(GramJob) * p.n_gram_tiles);
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

// Stage timers (a measurement switch, off by default): events on the caller's stream at the stage
// boundaries of the last merge_run, read by merge_stage_ms.
constexpr int kStageMarks = ABT_MERGE_STAGES + 1;
std::atomic<int> g_stage_timing{0};
std::mutex g_stage_mutex;
hipEvent_t g_stage_event[kStageMarks] = {};
int g_stage_device = -1;
int g_stage_recorded = 0;        // marks recorded by the last timed merge_run

bool stage_events_ready() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (g_stage_device == dev) return true;
    if (g_stage_device >= 0) return false;      // created on another device
    for (int i = 0; i < kStageMarks; ++i)
        if (hipEventCreate(&g_stage_event[i]) != hipSuccess) return false;
    g_stage_device = dev;
    return true;
}

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

int merge_set_stage_timing(int on) { return g_stage_timing.exchange(on ? 1 : 0); }

hipError_t merge_stage_ms(float out[ABT_MERGE_STAGES]) {
    std::lock_guard<std::mutex> lock(g_stage_mutex);
    if (g_stage_recorded != kStageMarks) return hipErrorNotReady;
    hipError_t e = hipEventSynchronize(g_stage_event[kStageMarks - 1]);
    for (int i = 0; i < ABT_MERGE_STAGES && e == hipSuccess; ++i)
        e = hipEventElapsedTime(&out[i], g_stage_event[i], g_stage_event[i + 1]);
    return e;
}

hipError_t launch_identity_f32(float* dst, int K, hipStream_t s) {
    const int64_t n = (int64_t)K * K;
    hipLaunchKernelGGL(identity_f32_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, dst, K);
    return hipGetLastError();
}

constexpr int kWorkspaceMagic = 0x41425431;

hipError_t merge_read_info(const void* workspace, int layer, int32_t out[4], hipStream_t s) {
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) return e;
    int hdr[4] = {0, 0, 0, 0};
    e = hipMemcpy(hdr, workspace, sizeof(hdr), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return e;
    if (hdr[0] != kWorkspaceMagic || layer < 0 || layer >= hdr[1]) return hipErrorInvalidValue;
    // the info table follows the 256-byte header slot (see make_plan)
    return hipMemcpy(out, (const char*)workspace + 256 + sizeof(int) * kInfoInts * layer,
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
    std::vector<GramJob> gtiles;
    const int gram_aligned = build_gram_jobs(layers, L, gtiles);
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

        const int K = q.K;
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
    const int header[4] = {kWorkspaceMagic, L, 0, 0};
    ABT_TRY(hipMemcpyAsync(ws + p.off_header, header, sizeof(header), hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_layers, hl.data(), sizeof(LayerDev) * L, hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_ptrs, hptrs.data(), sizeof(void*) * p.n_ptrs, hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_gram_tiles, gtiles.data(), sizeof(GramJob) * gtiles.size(), hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_wg_cross, wcross.data(), sizeof(int2) * wcross.size(), hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_wg_intra, wintra.data(), sizeof(int2) * wintra.size(), hipMemcpyHostToDevice, s));
    ABT_TRY(hipMemcpyAsync(ws + p.off_gemm64, g64.data(), sizeof(GemmF64) * g64.size(), hipMemcpyHostToDevice, s));
    std::vector<char> g32img(gemm_f32_desc_bytes() * (g32.empty() ? 1 : g32.size()));
    const int tiles32 = gemm_f32_build_table(g32.data(), (int)g32.size(), g32img.data());
    ABT_TRY(hipMemcpyAsync(ws + p.off_gemm32, g32img.data(), gemm_f32_desc_bytes() * g32.size(), hipMemcpyHostToDevice, s));
    // the uploads must have left the host vectors before they are destroyed
    ABT_TRY(hipStreamSynchronize(s));

    std::unique_lock<std::mutex> stage_lock(g_stage_mutex, std::defer_lock);
    bool timed = false;
    if (g_stage_timing.load()) {
        stage_lock.lock();
        timed = stage_events_ready();
        g_stage_recorded = 0;
        if (!timed) stage_lock.unlock();
    }
    auto mark = [&](int i) -> hipError_t {
        if (!timed) return hipSuccess;
        g_stage_recorded = i + 1;
        return hipEventRecord(g_stage_event[i], s);
    };
    const LayerDev* dl = (const LayerDev*)(ws + p.off_layers);
    ABT_TRY(mark(0));
    {
        const int64_t n = (int64_t)(kMaxSweepsCap + 1) * L;
        hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s,
                           (int*)(ws + p.off_rotated), n, 0);
    }
    ABT_TRY(launch_mean_gram(dl, (const GramJob*)(ws + p.off_gram_tiles), gram_aligned, p.n_gram_tiles - gram_aligned, s));
    ABT_TRY(mark(1));
    if (p.K_max <= kCholMaxK) {
        const size_t lds = sizeof(double) * ((size_t)(p.K_max > 32 ? p.K_max - 32 : 0) * kCholPitch + 32 * 33 + 32 + kCholThreads);
        static std::atomic<size_t> chol_attr{0};
        if (lds > chol_attr.load()) {
            ABT_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&cholesky_mfma_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            chol_attr.store(lds);
        }
        hipLaunchKernelGGL(cholesky_mfma_kernel, dim3(2 * L), dim3(kCholThreads), lds, s, dl);
    } else {
        hipLaunchKernelGGL(cholesky_kernel, dim3(2 * L), dim3(256), 0, s, dl);
    }
    ABT_TRY(mark(2));
    const GemmF64* d64 = (const GemmF64*)(ws + p.off_gemm64);
    hipLaunchKernelGGL(gemm_f64_kernel, dim3(align_up(tb0, 8)), dim3(256), 0, s, d64, p.n_gemm64, tb0);
    hipLaunchKernelGGL(frob2_kernel, dim3(8, L), dim3(256), 0, s, dl);
    ABT_TRY(hipGetLastError());
    ABT_TRY(mark(3));

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
    ABT_TRY(mark(4));
    int n2 = 1;
    while (n2 < p.K_max) n2 <<= 1;
    hipLaunchKernelGGL(colnorm_kernel, dim3((p.K_max + 3) / 4, L), dim3(256), 0, s, dl);
    hipLaunchKernelGGL(finalize_kernel, dim3(L), dim3(256), (sizeof(double) + sizeof(int)) * n2, s, dl, max_sweeps);
    if (tb1 > 0) hipLaunchKernelGGL(gemm_f64_kernel, dim3(align_up(tb1, 8)), dim3(256), 0, s, d64 + p.n_gemm64, p.n_gemm64, tb1);
    if (tb2 > 0) hipLaunchKernelGGL(gemm_f64_kernel, dim3(align_up(tb2, 8)), dim3(256), 0, s, d64 + 2 * p.n_gemm64, p.n_gemm64, tb2);
    ABT_TRY(hipGetLastError());
    ABT_TRY(mark(5));
    ABT_TRY(launch_gemm_f32_table(ws + p.off_gemm32, (int)g32.size(), tiles32, s));
    ABT_TRY(mark(6));
#undef ABT_TRY
    return hipSuccess;
}

}  // namespace abt
