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

// Loads and stores through a pointer known to point into device memory.  A pointer read from a table
// is generic to the compiler, which then emits FLAT instructions; those count in the LDS counter as
// well as in the memory counter, so every wait for an LDS read would also wait for all global loads
// in flight (prefetches included).  These helpers emit GLOBAL instructions.
template <typename T>
__device__ __forceinline__ T gload(const T* p) {
    return *(const __attribute__((address_space(1))) T*)(p);
}
template <typename T>
__device__ __forceinline__ void gstore(T* p, const T& v) {
    *(__attribute__((address_space(1))) T*)(p) = v;
}

// Two fp32 -> packed bf16 (low half = lo), round-to-nearest-even: one v_cvt_pk_bf16_f32 on gfx950.
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Buffer addressing: a wave-uniform 128-bit descriptor (base, byte count) + wave-uniform byte
// offset + one 32-bit byte offset per lane.  Accesses past the byte count read zeros / are dropped.
// Only the per-lane offset is range-checked, not the wave-uniform one.  A byte count beyond
// kBufMaxBytes is clamped to it: per-lane offsets must stay below that (callers check sizes on the
// host), and kBufNowhere is a per-lane offset that no descriptor covers.
using rsrc_t = __amdgpu_buffer_rsrc_t;
constexpr int kBufMaxBytes = 0x7ffffff0;
constexpr int kBufNowhere = 0x7ffffff0;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, int64_t bytes) {
    const int n = bytes > kBufMaxBytes ? kBufMaxBytes : (bytes < 0 ? 0 : (int)bytes);
    // last word: raw buffer, 32-bit data format field as the gfx9 family expects for untyped access
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(rsrc_t r, int lane_off, int wave_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, wave_off, 0);
}
// A 16-byte store reads its data registers for a few cycles after it has issued, and the compiler
// does not keep the next instructions away from them when the wave-uniform offset is a register
// (seen: the address of the next store, written into the first data register one instruction after
// the store, went to memory in place of the data).  Nothing may follow for eight wait states: 64 lanes
// of 16 bytes leave the register file at 64 bytes per cycle.
__device__ __forceinline__ void store_data_guard() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 7");
    __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ void buf_store16(u32x4 v, rsrc_t r, int lane_off, int wave_off) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, lane_off, wave_off, 0);
    store_data_guard();
}

// A store with the non-temporal hint, for results that a launch writes once and that are too large
// to be found in the last-level cache by whoever reads them next: such lines should not push the
// factors, which every work-group re-reads, out of L2.  (The hint on the loads of the activations
// measured slower than plain loads; on the stores it is worth 6 % of a config-3 step.)
__device__ __forceinline__ void buf_store16_stream(u32x4 v, rsrc_t r, int lane_off, int wave_off) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, lane_off, wave_off, 2);
    store_data_guard();
}
// `stream` is uniform over the launch
__device__ __forceinline__ void buf_store16_maybe_stream(bool stream, u32x4 v, rsrc_t r, int lane_off, int wave_off) {
    if (stream) buf_store16_stream(v, r, lane_off, wave_off);
    else buf_store16(v, r, lane_off, wave_off);
}
// Outputs of a launch (Yout and Tout of the chain kernels) of this many bytes or more are stored with
// the hint: a quarter of the 256 MB last-level cache.
constexpr int64_t kStreamOutBytes = 64ll << 20;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------ bf16 factored layer
// Fused chain  Tout[M,R] = Xin[M,p] . P[R,p]^T ;  Yout[M,q] = Tout . Q[q,R]^T  (bf16, fp32 acc).
// Yout or Tout may be NULL.  p, q multiples of 64; R in {32..384 step 32}.
hipError_t launch_chain_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                             int64_t M, int p, int q, int R, hipStream_t s);
// The same chain with 64-row work-groups: four MFMA waves fed by four loader waves; covers
// R in {32, 64, 96, 128, 160, 192, 256, 320, 384} with p a multiple of 64 and p, q <= 2^20
// (32-bit byte offsets inside a work-group's rows and inside the factors) (chain2_supports).
bool chain2_supports(int R, int p, int q);
hipError_t launch_chain2_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                              int64_t M, int p, int q, int R, hipStream_t s);
// The same chain with 128-row work-groups (eight MFMA waves in two row groups fed by four loader
// waves): every slab of a factor serves twice the rows.  R in {32, 64, 96, 128, 192}.  With
// parts > 1 the grid gets that many work-groups per row block, each doing its share of the output
// tiles of stage 2 after repeating stage 1 (for batches too small to fill the chip otherwise).
bool chain2_tall_supports(int R, int p, int q);
hipError_t launch_chain2_tall_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                              int64_t M, int p, int q, int R, int parts, hipStream_t s);
// (For R = 192, 256 and 384 the plain 128-row launches go to the kernel of eight equal waves below; the
// gathered form has 128-row work-groups for R in {32, 64, 96, 128, 192, 384}.)
// Up to kChainMaxGroups problems of one shape in one launch (the emulated groups of a training step).
// rows = 64 or 128 (work-group height; the caller has checked chain2_supports / chain2_tall_supports);
// Yout must be NULL for all problems or for none; a problem with Yout == Tout == NULL is skipped.
constexpr int kChainMaxGroups = 8;
struct ChainProblem { const void* Xin; const void* P; const void* Q; void* Yout; void* Tout; };
hipError_t launch_chain2_grouped_bf16(const ChainProblem* problems, int G, int64_t M, int p, int q, int R,
                                      int rows, int parts, hipStream_t s);
// The same chain for R = 192, 256, 384 with 128-row work-groups of eight equal waves, slabs loaded
// straight into LDS; p, q multiples of 64, at most 2^20; `parts` as above; groups as above.
bool chain3_supports(int R, int p, int q);
hipError_t launch_chain3_bf16(const ChainProblem* problems, int G, int64_t M, int p, int q, int R, int parts, hipStream_t s);
// The same chain with the first operand gathered from a channels-last image [images, H, W, Cin]
// instead of read from a matrix: row i of the virtual operand is the kh x kw patch around a pixel
// (zero outside the image), columns ordered (tap, channel) with every tap padded to a multiple of
// 64 channels: p = kh kw ceil(Cin / 64) 64 columns, which is the row length of P [R, p].
// Rows are the pixels of a grid RH x RW per image (M = images RH RW); row (y, x) is centred on image
// pixel (mul y, mul x) and tap (ky, kx) reads the position sign (ky - kh/2, kx - kw/2) away from it,
// which with shift = 1 exists only where both coordinates are even, as pixel (ty / 2, tx / 2):
//   patches, stride 1:        RH x RW = H x W, mul = 1, shift = 0, sign = +1
//   patches, stride 2:        RH x RW = output grid, mul = 2, shift = 0, sign = +1
//   adjoint gather, stride 1: the same with sign = -1
//   adjoint gather, stride 2: image = gradient on the output grid, RH x RW = input grid, mul = 1,
//                             shift = 1, sign = -1.
// Tout rows are t_pitch elements apart (>= R).
struct PatchGeom { int H, W, Cin, kh, kw, sign, RH, RW, mul, shift; };
hipError_t launch_chain2_gather_bf16(const void* image, const PatchGeom& g, const void* P, const void* Q,
                                     void* Yout, void* Tout, int t_pitch, int64_t M, int q, int R, hipStream_t s);
hipError_t launch_chain2_tall_gather_bf16(const void* image, const PatchGeom& g, const void* P, const void* Q,
                                     void* Yout, void* Tout, int t_pitch, int64_t M, int q, int R, hipStream_t s);
// dst[c, r] = src[r, c] for a bf16 matrix of `rows` x `cols`.
struct TransposeJob { const void* src; void* dst; int rows, cols; };   // dst[cols, rows] = src[rows, cols]^T
constexpr int kTransposeMaxJobs = 16;   // per launch
hipError_t launch_transpose_bf16(const TransposeJob* jobs, int njobs, hipStream_t s);
// part[split][P,Q] = U[rows of split, P]^T . V[rows of split, Q]  (bf16 in, fp32 partials)
// followed by out[P,Q] (+)= sum over splits, in fixed order.  One of P, Q equals R.
// job: out[P,R] = U[M,P]^T . V[M,R]; with transposed != 0 the result is stored as out[R,P].
struct TnJob {
    const void* U; const void* V; float* out; int P; int transposed;
};
constexpr int kTnMaxJobs = 16;   // per launch (all with the same M and R)
size_t tn_partials_bytes(int64_t M, const TnJob* jobs, int njobs, int R);
hipError_t launch_tn_bf16(const TnJob* jobs, int njobs, int64_t M, int R, int accumulate,
                          float* partials, hipStream_t s);

// Pst [C, taps r_pad] (bf16) from B [r, taps C]: Pst[c, tap r_pad + j] = B[j, tap C + c], zero for j >= r.
hipError_t launch_conv_bstack_bf16(const void* B, void* Pst, int r, int C, int taps, int r_pad, hipStream_t s);
// One or two jobs; the U of the LAST one is the patch matrix of a channels-last image (g.sign is
// ignored: always +1): column tap Cin + c of row i is channel c of pixel (y + ky - kh/2, x + kx - kw/2),
// and its P = kh kw Cin.  A job before it is a plain one.  Partials as for launch_tn_bf16.
hipError_t launch_tn_gather_bf16(const TnJob* jobs, int njobs, const PatchGeom& g, int64_t M, int R, int accumulate,
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
hipError_t launch_identity_f32(float* dst, int K, hipStream_t s);   // dst[K, K] = I
// Stage timers of the batched merge: with the switch on, merge_run records events on the caller's
// stream at its stage boundaries and merge_stage_ms waits for the last and returns the elapsed
// milliseconds of the ABT_MERGE_STAGES stages (hipErrorNotReady if no timed merge has run).
int merge_set_stage_timing(int on);
hipError_t merge_stage_ms(float out[ABT_MERGE_STAGES]);
int merge_set_groups(int n);   // upper bound on the layer groups (streams) of the Jacobi stage; returns the previous one

// ------------------------------------------------------------------ optimiser step
// Adam with decoupled weight decay on up to any number of tensors (kAdamwMaxTensors per launch).
constexpr int kAdamwMaxTensors = 48;
struct AdamwTensor {
    float* param; const float* grad; float* exp_avg; float* exp_avg_sq; uint16_t* param_bf16; int64_t count;
};
struct AdamwHyper {   // everything the kernel needs, prepared on the host in double precision
    float beta1, beta2, one_minus_beta1, one_minus_beta2;
    float inv_bc1;        // 1 / (1 - beta1^step)
    float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^step)
    float eps, eta, weight_decay;   // eta = lr * lr_scale
};
hipError_t launch_adamw(const AdamwTensor* tensors, int n, const AdamwHyper& h, hipStream_t s);

}  // namespace abt
