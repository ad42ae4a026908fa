// Declarations shared by the merge sources: the per-layer device record, the constants of the
// Jacobi iteration and the rotation formula.
#pragma once

#include "common.h"

namespace abt {

constexpr int kInfoInts = 4;      // per layer: sweeps, n_sigma, converged, k'
constexpr int kMaxSweepsCap = 64;
constexpr double kRotateTol = 1e-9;    // |cos| above which a column pair is rotated
// A sweep in which no visited pair had |cos| above kSignifTol ends the iteration.  Every pair above
// kRotateTol was still rotated to orthogonality when visited, and the later rotations of that sweep
// disturb it only in second order: measured on the config-5 cores a sweep that starts at 1.2e-4 leaves
// 9e-8 behind (about 6 cos^2), so the cosines left at the end are below 1e-6, two orders under the
// 1e-4 the results are held to.
constexpr double kSignifTol = 3e-4;
constexpr double kSigmaFloor = 1e-7;   // sigma_i <= floor * sigma_1: singular vectors returned as zero
// A column of C with |c|^2 below kZeroColumn2 ||C||_F^2 (|c| < 1e-9 ||C||_F) is numerically zero
// and is left alone: what it holds is the rounding noise (about 1e-16 ||C||) of the large columns
// it was rotated with, so its angles are noise at the level the convergence test looks at and
// would keep the iteration from ending.  It belongs to a singular value far below
// kSigmaFloor sigma_1 (||C||_F <= sqrt(K) sigma_1).
constexpr double kZeroColumn2 = 1e-18;

struct LayerDev {
    const float* const* A_ptrs;
    const float* const* B_ptrs;
    int G, mode, m, n, k, K, k_cap, k_fixed;
    float tau;
    int jb, nb;            // Jacobi: columns per block, number of blocks
    float* Abar; float* Bbar;
    double* LA; double* GB; double* LB; double* Ct; double* Yt;
    double* sigma; double* s3; double* s5;
    double* trace;         // [10]: trace(G_A), trace(G_B), then eight partial sums of ||C||_F^2
    double* nrm;           // [K]: squared column norms of the rotated core (colnorm_kernel -> finalize_kernel)
    int* perm;
    float* PA; float* PB;
    int* rotated;          // [kMaxSweepsCap + 1]
    int* info;             // [kInfoInts]
    float* S_out; int32_t* k_out;
};


typedef __attribute__((ext_vector_type(2))) double f64x2;

__device__ __forceinline__ bool sweep_finished(const LayerDev& L, int sweep) {
    // the previous sweep found no significant pair: the iteration has converged
    return sweep > 0 && L.rotated[sweep - 1] == 0;
}

__device__ __forceinline__ double frob2(const LayerDev& L) {
    double s = 0.0;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += L.trace[2 + j];
    return s;
}

// Rotation for a pair with squared norms alpha, beta and inner product gamma; returns false when
// the pair counts as orthogonal.  x' = c x - s y, y' = s x + c y.
// A column whose squared norm is below `floor2` (kZeroColumn2 ||C||_F^2) is numerically zero and
// is left alone (rank-deficient cores).
__device__ __forceinline__ bool jacobi_rotation(double alpha, double beta, double gamma, double floor2,
                                                double& c, double& s, bool& significant, double* tangent = nullptr) {
    const double lim = alpha * beta;
    const double g2 = gamma * gamma;
    significant = false;
    if (!(alpha > floor2) || !(beta > floor2)) return false;
    significant = g2 > (kSignifTol * kSignifTol) * lim;
    if (!(g2 > (kRotateTol * kRotateTol) * lim)) return false;
    // tangent of the rotation angle, the smaller root of t^2 + 2 zeta t - 1 = 0 with
    // zeta = (beta - alpha) / (2 gamma), written so that it costs one square root and one division:
    // t = 2 gamma sign(d) / (|d| + sqrt(d^2 + 4 gamma^2)), d = beta - alpha
    const double d = beta - alpha;
    const double g2x = 2.0 * gamma;
    const double tn = (d >= 0.0 ? g2x : -g2x) / (fabs(d) + sqrt(fma(d, d, g2x * g2x)));
    // c = (1 + t^2)^(-1/2): hardware reciprocal square root refined by two Newton steps (the
    // rotation stays orthogonal to rounding: c^2 + s^2 = c^2 (1 + t^2))
    const double w = fma(tn, tn, 1.0);
    double y = __builtin_amdgcn_rsq(w);
    y = y * fma(-0.5 * w, y * y, 1.5);
    y = y * fma(-0.5 * w, y * y, 1.5);
    c = y;
    s = c * tn;
    if (tangent) *tangent = tn;
    return true;
}

// Average of the copies + Gram matrices (merge_gram.hip): one work-group per job; layer < 0 marks
// an empty slot; (ti, tj), ti >= tj, is a 128 x 128 tile of the lower triangle; which = 0: G_A
// (stored into LA), 1: G_B (stored into GB and LB).  The diagonal tiles also write Abar / Bbar.
struct GramJob { int layer, which, ti, tj; };
// `jobs` holds njobs entries for the kernel with 16-byte loads, then njobs_unaligned entries (B sides
// whose row length n is not a multiple of four) for the element-wise one.
hipError_t launch_mean_gram(const LayerDev* layers, const GramJob* jobs, int njobs, int njobs_unaligned, hipStream_t s);

// One round of the block Jacobi iteration for cores with K <= 768 (every layer of the batch):
// `n_wg` work-groups, wg_map[i] = (layer, pair slot).  Round 0 of a sweep also orthogonalises the
// columns inside every block.
hipError_t launch_jacobi_block_round(const LayerDev* layers, const int2* wg_map, int n_wg, int K_max,
                                     int sweep, int round, hipStream_t s);

}  // namespace abt
