// Shared declarations of the HIP side: vector types for the gfx950 MFMA builtins, bf16
// conversion, and the launcher prototypes that api.hip calls.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "abtrain.h"

namespace abt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) double f64x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWave = 64;

// fp32 -> bf16 bits, round-to-nearest-even, NaN kept quiet.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------ bf16 factored layer
// Fused chain  Tout[M,R] = Xin[M,p] . P[R,p]^T ;  Yout[M,q] = Tout . Q[q,R]^T  (bf16, fp32 acc).
// Yout or Tout may be NULL.  p, q multiples of 64; R in {32..384 step 32}.
hipError_t launch_chain_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                             int64_t M, int p, int q, int R, hipStream_t s);
// The same chain with 64-row work-groups, 8 waves and direct-to-LDS slab rings; covers
// R in {32, 64, 96, 128, 192, 256, 384} (chain2_supports).
bool chain2_supports(int R, int p);
hipError_t launch_chain2_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                              int64_t M, int p, int q, int R, hipStream_t s);
// dst[c, r] = src[r, c] for a bf16 matrix of `rows` x `cols`.
hipError_t launch_transpose_bf16(const void* src, void* dst, int rows, int cols, hipStream_t s);
// part[split][P,Q] = U[rows of split, P]^T . V[rows of split, Q]  (bf16 in, fp32 partials)
// followed by out[P,Q] (+)= sum over splits, in fixed order.  One of P, Q equals R.
// job: out[P,R] = U[M,P]^T . V[M,R]; with transposed != 0 the result is stored as out[R,P].
struct TnJob {
    const void* U; const void* V; float* out; int P; int transposed;
};
size_t tn_partials_bytes(int64_t M, const TnJob* jobs, int njobs, int R);
hipError_t launch_tn_bf16(const TnJob* jobs, int njobs, int64_t M, int R, int accumulate,
                          float* partials, hipStream_t s);

// ------------------------------------------------------------------ fp32 GEMM (MFMA)
// C[P,Q] = alpha * op(A) . op(B) (+ C if accumulate).  op(A) is P x K: transA == 0 reads
// A[P,K] (lda = row length), else A[K,P].  op(B) is K x Q: transB == 0 reads B[K,Q], else B[Q,K].
// col_limit: optional device int; output columns >= *col_limit are written as zero without
// being computed (rows when limit_rows != 0).
struct GemmF32 {
    const float* A; const float* B; float* C;
    int P, Q, K;
    int lda, ldb, ldc;
    int transA, transB;
    int accumulate;
    float alpha;
    const int32_t* limit;   // may be NULL
    int limit_rows;
};
// Single problem, descriptor passed by value.
hipError_t launch_gemm_f32_one(const GemmF32& d, hipStream_t s);
// n problems in one launch: build the table on the host (n * gemm_f32_desc_bytes() bytes,
// returns the tile count), copy it to the device, then launch from the device copy.
size_t gemm_f32_desc_bytes();
int gemm_f32_build_table(const GemmF32* descs_host, int n, void* host_image);
hipError_t launch_gemm_f32_table(const void* dev_image, int n, int tiles, hipStream_t s);

// ------------------------------------------------------------------ merge
// Host-side plan of a batched merge: validates nothing (api.hip does), lays out the workspace
// and enqueues every stage.
size_t merge_workspace_bytes(const abt_merge_desc* layers, int L);
hipError_t merge_run(const abt_merge_desc* layers, int L, void* workspace, int max_sweeps, hipStream_t s);
hipError_t merge_read_info(const void* workspace, int layer, int32_t out[4], hipStream_t s);

}  // namespace abt
