// Block form of the one-sided Jacobi iteration on the K x K core of the merge (the truncated SVD
// of Eq. 3 on the merged matrix), for K <= 768, on the fp64 matrix cores.
//
// The columns of C (rows of Ct) are grouped in blocks of 16; a round pairs every block with one
// partner (round-robin tournament over the blocks), one work-group per block pair.  For its 32
// columns P (K x 32) a work-group
//   1. forms the Gram matrix S = P^T P (32 x 32) with v_mfma_f64_16x16x4,
//   2. runs the cyclic Jacobi eigenvalue iteration on S in LDS: 16 steps of 16 disjoint rotations,
//      one step per cyclic shift of the partner block, every rotation applied to S from both sides
//      and accumulated in Q (32 x 32).  These are the plane rotations the column form of the
//      method would apply to the 256 column pairs of the two blocks, in the same order; they are
//      worked out on the 32 x 32 Gram matrix instead of on K-long columns,
//   3. applies them at once: P <- P Q, again on the matrix cores.
// Round 0 of a sweep first rotates the pairs inside each of the two blocks the same way (15 steps).
//
// The panel lives in registers from load to store, in the operand layout of step 3: a lane holds
// the rows r = l % 16 of its wave's row tiles and the columns l / 16 + 4 s (s = 0..7); with the
// product taken as (Q^T P^T) the result tile comes out of the matrix core in that same layout, so
// the update is in place.  Step 1 needs the transposed operand order (contraction over rows); each
// wave passes its row tiles through a private 4 KB LDS tile for that.
#include "merge_internal.h"

namespace abt {

namespace {

// swizzled address (in doubles) of element (row n, column c) of a 16 x 32 staging tile: stores of one
// column by 16 rows and loads of 16 consecutive columns of one row both spread over all banks
__device__ __forceinline__ int stage_addr(int n, int c) {
    return 32 * n + ((c + 16 * (n & 1) + 2 * (n >> 1)) & 31);
}

struct __align__(16) JacobiShared {
    double stage[4][16 * 32];       // per wave: transposition tile; afterwards the waves' partial Gram tiles
    // pitch 48: rows 96 words apart, so the cells of two neighbouring rows times sixteen columns that
    // a half wave touches at once fall into different halves of the 64 banks
    double S[2][32][48];            // read from one copy, written to the other, swapped every step
    double Q[32][48];
    f64x2 cs[2][16];                // (cosine, sine) of the 16 rotations of a step (two copies: steps alternate)
};

// The rotation of jacobi_rotation(), arranged for a short dependency chain (the 16 steps of a block
// pair are serial, and this is the longest link of a step): no branches, the tangent in fp32, the
// cosine from an fp32 reciprocal square root corrected by two terms of its series.  Any tangent
// gives a rotation that is orthogonal to fp64 rounding (c = (1 + t^2)^(-1/2), s = c t); a tangent
// good to 1e-7 leaves the pair with 1e-7 of its cosine.  `scale` is a power of two near
// 1 / ||C||_F^2: squared norms lie between kZeroColumn2 and 1 times ||C||_F^2, so scaled inputs of a
// pair that is rotated stay inside the fp32 range (|gamma| scale >= 1e-9 sqrt(1e-18 1e-18)).
__device__ __forceinline__ void fast_rotation(double alpha, double beta, double gamma, double floor2, double scale,
                                              double& c, double& s, bool& significant) {
    const double lim = alpha * beta;
    const double g2 = gamma * gamma;
    const bool live = alpha > floor2 && beta > floor2;
    significant = live && g2 > (kSignifTol * kSignifTol) * lim;
    const bool rot = live && g2 > (kRotateTol * kRotateTol) * lim;
    const float d = (float)((beta - alpha) * scale);
    const float g2x = (float)((gamma + gamma) * scale);
    const float zeta = d * __builtin_amdgcn_rcpf(g2x);
    const float az = fabsf(zeta);                        // an overflow of az^2 ends in t = 0 (|t| < 1e-19)
    const float ta = __builtin_amdgcn_rcpf(az + __builtin_amdgcn_sqrtf(fmaf(az, az, 1.0f)));
    const float tf = zeta >= 0.0f ? ta : -ta;
    const double c0 = (double)__builtin_amdgcn_rsqf(fmaf(tf, tf, 1.0f));
    const double tn = (double)tf;
    const double w = fma(tn, tn, 1.0);
    const double e = fma(-(c0 * c0), w, 1.0);            // c = c0 (1 - e)^(-1/2) = c0 (1 + e/2 + 3 e^2/8 + ...)
    const double cc = fma(c0, e * fma(0.375, e, 0.5), c0);
    c = rot ? cc : 1.0;
    s = rot ? cc * tn : 0.0;
}

// endpoints of pair p (0..15) in step st: the first `intra` steps pair columns inside each block
// (circle method on 16 players, pairs 0..7 in the first block, 8..15 in the second), the following
// 16 steps pair column p of the first block with column (p + t) mod 16 of the second.
__device__ __forceinline__ void pair_of(int st, int intra, int p, int& i, int& j) {
    if (st < intra) {
        const int base = p < 8 ? 0 : 16, u = p & 7;
        if (u == 0) { i = 15; j = st; }
        else { i = (st + u) % 15; j = (st - u + 15) % 15; }
        i += base; j += base;
    } else {
        i = p;
        j = 16 + ((p + st - intra) & 15);
    }
}

// NT: 16-row tiles per wave (two per 32-row chunk: its even and its odd rows), K <= 64 NT.
template <int NT>
__global__ __launch_bounds__(256, (NT <= 6 ? 3 : 1)) void jacobi_block_kernel(const LayerDev* __restrict__ layers,
                                                                               const int2* __restrict__ wg_map,
                                                                               int sweep, int round) {
    __shared__ JacobiShared sh;
    const int2 wm = wg_map[blockIdx.x];                   // (layer, pair slot)
    const LayerDev& L = layers[wm.x];
    if (sweep_finished(L, sweep)) return;
    const int K = L.K, nb = K >> 4;
    if (round >= nb - 1 || K > 64 * NT) return;
    // circle method: slot 0 pairs block nb-1 with `round`; slot j pairs (round + j) with (round - j)
    int bI, bJ;
    if (wm.y == 0) { bI = nb - 1; bJ = round; }
    else { bI = (round + wm.y) % (nb - 1); bJ = (round - wm.y + (nb - 1)) % (nb - 1); }
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 15, kq = lane >> 4;

    // ---- load the panel: D[t][s] = P[row(t, n)][column kq + 4 s], columns 0..15 = block I, 16..31 = block J
    double D[NT][8];
#pragma unroll
    for (int tt = 0; tt < NT / 2; ++tt) {
        const int row0 = 32 * (wave + 4 * tt) + 2 * n;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int col = (s < 4 ? bI * 16 + kq + 4 * s : bJ * 16 + kq + 4 * (s - 4));
            f64x2 v = {0.0, 0.0};
            if (row0 < K) v = gload(reinterpret_cast<const f64x2*>(L.Ct + (int64_t)col * K + row0));
            D[2 * tt][s] = v[0];
            D[2 * tt + 1][s] = v[1];
        }
    }

    // ---- S = P^T P: three 16 x 16 tiles (II, IJ, JJ), this wave's rows
    f64x4 gII = {0.0, 0.0, 0.0, 0.0}, gIJ = gII, gJJ = gII;
    double* stage = sh.stage[wave];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int s = 0; s < 8; ++s) stage[stage_addr(n, kq + 4 * s)] = D[t][s];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        double a0[4], a1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a0[q] = stage[stage_addr(4 * q + kq, n)];
            a1[q] = stage[stage_addr(4 * q + kq, 16 + n)];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            gII = __builtin_amdgcn_mfma_f64_16x16x4f64(a0[q], a0[q], gII, 0, 0, 0);
            gIJ = __builtin_amdgcn_mfma_f64_16x16x4f64(a0[q], a1[q], gIJ, 0, 0, 0);
            gJJ = __builtin_amdgcn_mfma_f64_16x16x4f64(a1[q], a1[q], gJJ, 0, 0, 0);
        }
    }
    // partial tiles of the four waves, added in wave order; result element (i, j) of a tile sits in
    // lane (j, i % 4), register i / 4
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        stage[0 * 256 + lane * 4 + v] = gII[v];
        stage[1 * 256 + lane * 4 + v] = gIJ[v];
    }
    __syncthreads();
    {
        const int l = tid >> 2, v = tid & 3, i = (l >> 4) + 4 * v, j = l & 15;
        const double sII = ((sh.stage[0][tid] + sh.stage[1][tid]) + sh.stage[2][tid]) + sh.stage[3][tid];
        const double sIJ = ((sh.stage[0][256 + tid] + sh.stage[1][256 + tid]) + sh.stage[2][256 + tid]) + sh.stage[3][256 + tid];
        sh.S[0][i][j] = sII;
        sh.S[0][i][16 + j] = sIJ;
        sh.S[0][16 + j][i] = sIJ;
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 4; ++v) stage[lane * 4 + v] = gJJ[v];
    __syncthreads();
    {
        const int l = tid >> 2, v = tid & 3, i = (l >> 4) + 4 * v, j = l & 15;
        sh.S[0][16 + i][16 + j] = ((sh.stage[0][tid] + sh.stage[1][tid]) + sh.stage[2][tid]) + sh.stage[3][tid];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            sh.Q[idx >> 5][idx & 31] = (idx >> 5) == (idx & 31) ? 1.0 : 0.0;
        }
    }
    __syncthreads();

    // ---- anything to rotate?  (pairs inside the blocks count in round 0 only)
    const double frob = frob2(L);
    const double floor2 = kZeroColumn2 * frob;
    const double scale = ldexp(1.0, -__builtin_amdgcn_frexp_exp(frob));
    const int intra = round == 0 ? 15 : 0;
    int need = 0;
    {
        const int i = tid >> 4, j = tid & 15;
        auto test = [&](int p, int q) {
            const double a = sh.S[0][p][p], b = sh.S[0][q][q], g = sh.S[0][p][q];
            if (a > floor2 && b > floor2 && g * g > (kRotateTol * kRotateTol) * (a * b)) need = 1;
        };
        test(i, 16 + j);
        if (intra && i < j) { test(i, j); test(16 + i, 16 + j); }
    }
    if (!__syncthreads_or(need)) return;     // the data is untouched: nothing to store

    // ---- cyclic Jacobi on S, accumulated in Q.  A thread owns the 2 x 2 cell rows(pair u) x
    // columns(pair v) of S and two rows of the columns(pair v) of Q.
    bool any_signif = false;
    if (tid < 16) {                                      // rotations of the first step
        int i, j;
        pair_of(0, intra, tid, i, j);
        double c, s; bool signif;
        fast_rotation(sh.S[0][i][i], sh.S[0][j][j], sh.S[0][i][j], floor2, scale, c, s, signif);
        any_signif |= signif;
        sh.cs[0][tid] = f64x2{c, s};
    }
    __syncthreads();
    // (a) round 0 only: the 15 steps inside the two blocks.  Two barriers per step: the rotations of
    // the next step are worked out from the new S by 16 threads while the others update Q.
    for (int st = 0; st < intra; ++st) {
        const double (*Sr)[48] = sh.S[st & 1];
        double (*Sw)[48] = sh.S[(st & 1) ^ 1];
        const int cu = tid >> 4, cv = tid & 15;
        int iu, ju, iv, jv;
        pair_of(st, intra, cu, iu, ju);
        pair_of(st, intra, cv, iv, jv);
        const f64x2 r1 = sh.cs[st & 1][cu], r2 = sh.cs[st & 1][cv];
        const double c1 = r1[0], s1 = r1[1], c2 = r2[0], s2 = r2[1];
        const double m00 = Sr[iu][iv], m01 = Sr[iu][jv], m10 = Sr[ju][iv], m11 = Sr[ju][jv];
        const double t00 = c1 * m00 - s1 * m10, t01 = c1 * m01 - s1 * m11;
        const double t10 = s1 * m00 + c1 * m10, t11 = s1 * m01 + c1 * m11;
        Sw[iu][iv] = c2 * t00 - s2 * t01; Sw[iu][jv] = s2 * t00 + c2 * t01;
        Sw[ju][iv] = c2 * t10 - s2 * t11; Sw[ju][jv] = s2 * t10 + c2 * t11;
        __syncthreads();
        if (tid < 16) {
            int i, j;
            pair_of(st + 1, intra, tid, i, j);
            double c, s; bool signif;
            fast_rotation(Sw[i][i], Sw[j][j], Sw[i][j], floor2, scale, c, s, signif);
            any_signif |= signif;
            sh.cs[(st + 1) & 1][tid] = f64x2{c, s};
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = cu + 16 * h;
            const double q0 = sh.Q[r][iv], q1 = sh.Q[r][jv];
            sh.Q[r][iv] = c2 * q0 - s2 * q1;
            sh.Q[r][jv] = s2 * q0 + c2 * q1;
        }
        __syncthreads();
    }
    // (b) the 16 steps between the blocks: step t pairs column u of the first block with column
    // (u + t) mod 16 of the second.  One barrier per step.  Cells are dealt to the threads by
    // diagonals: d = (v - u) mod 16 picks the wave and the 16-lane row, u the lane in the row.  The
    // rotation of pair u in step t + 1 needs three entries of the new S which step t leaves in
    // registers of one wave: S[u][j'] in the cell (u, u + 1) (j' = the next partner of u), S[u][u] and
    // S[j'][j'] in the diagonal cells of pairs u and u + 1.  So the lanes of the row d = 1 fetch the
    // two diagonal entries from row d = 0 by a lane permute and work the rotation out while the
    // other waves update Q; no second barrier, no trip through LDS.  Which wave holds these two
    // rows differs from work-group to work-group (the work-groups sharing a compute unit put this
    // serial part on different SIMDs).
    {
        const int wrot = (int)(blockIdx.x & 3);
        const int dd = (((wave - wrot) & 3) << 2) + (lane >> 4);
        const int du = lane & 15, dv = (du + dd) & 15;
        const bool rot_wave = wave == wrot;
        for (int t = 0; t < 16; ++t) {
            const int par = (intra + t) & 1;
            const double (*Sr)[48] = sh.S[par];
            double (*Sw)[48] = sh.S[par ^ 1];
            const int ju = 16 + ((du + t) & 15), jv = 16 + ((dv + t) & 15);
            const f64x2 r1 = sh.cs[par][du], r2 = sh.cs[par][dv];
            const double c1 = r1[0], s1 = r1[1], c2 = r2[0], s2 = r2[1];
            const double m00 = Sr[du][dv], m01 = Sr[du][jv], m10 = Sr[ju][dv], m11 = Sr[ju][jv];
            const double t00 = c1 * m00 - s1 * m10, t01 = c1 * m01 - s1 * m11;
            const double t10 = s1 * m00 + c1 * m10, t11 = s1 * m01 + c1 * m11;
            const double n00 = c2 * t00 - s2 * t01, n01 = s2 * t00 + c2 * t01;
            const double n10 = c2 * t10 - s2 * t11, n11 = s2 * t10 + c2 * t11;
            Sw[du][dv] = n00; Sw[du][jv] = n01; Sw[ju][dv] = n10; Sw[ju][jv] = n11;
            if (rot_wave && t < 15) {
                // lane 16 + u: alpha = S[u][u] from lane u, beta = S[j'][j'] from lane (u + 1) mod 16
                const double alpha = __shfl(n00, du, 64);
                const double beta = __shfl(n11, (du + 1) & 15, 64);
                if ((lane >> 4) == 1) {
                    double c, s; bool signif;
                    fast_rotation(alpha, beta, n01, floor2, scale, c, s, signif);
                    any_signif |= signif;
                    sh.cs[par ^ 1][du] = f64x2{c, s};
                }
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int r = du + 16 * h;
                const double q0 = sh.Q[r][dv], q1 = sh.Q[r][jv];
                sh.Q[r][dv] = c2 * q0 - s2 * q1;
                sh.Q[r][jv] = s2 * q0 + c2 * q1;
            }
            __syncthreads();
        }
    }
    if (any_signif) L.rotated[sweep] = 1;

    // ---- P <- P Q as (Q^T P^T): A operand = Q^T tile, B operand = the panel registers
    double qa[2][8];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int s = 0; s < 8; ++s) qa[ct][s] = sh.Q[kq + 4 * s][16 * ct + n];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        f64x4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = acc0;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(qa[0][s], D[t][s], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(qa[1][s], D[t][s], acc1, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) { D[t][v] = acc0[v]; D[t][4 + v] = acc1[v]; }
    }

    // ---- store
#pragma unroll
    for (int tt = 0; tt < NT / 2; ++tt) {
        const int row0 = 32 * (wave + 4 * tt) + 2 * n;
        if (row0 < K) {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int col = (s < 4 ? bI * 16 + kq + 4 * s : bJ * 16 + kq + 4 * (s - 4));
                gstore(reinterpret_cast<f64x2*>(L.Ct + (int64_t)col * K + row0), f64x2{D[2 * tt][s], D[2 * tt + 1][s]});
            }
        }
    }
}

}  // namespace

hipError_t launch_jacobi_block_round(const LayerDev* layers, const int2* wg_map, int n_wg, int K_max,
                                     int sweep, int round, hipStream_t s) {
    if (n_wg <= 0) return hipSuccess;
    const dim3 grid(n_wg), block(256);
    if (K_max <= 128) hipLaunchKernelGGL(jacobi_block_kernel<2>, grid, block, 0, s, layers, wg_map, sweep, round);
    else if (K_max <= 256) hipLaunchKernelGGL(jacobi_block_kernel<4>, grid, block, 0, s, layers, wg_map, sweep, round);
    else if (K_max <= 384) hipLaunchKernelGGL(jacobi_block_kernel<6>, grid, block, 0, s, layers, wg_map, sweep, round);
    else if (K_max <= 512) hipLaunchKernelGGL(jacobi_block_kernel<8>, grid, block, 0, s, layers, wg_map, sweep, round);
    else if (K_max <= 768) hipLaunchKernelGGL(jacobi_block_kernel<12>, grid, block, 0, s, layers, wg_map, sweep, round);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace abt
