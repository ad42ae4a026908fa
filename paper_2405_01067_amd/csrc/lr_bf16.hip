// bf16 factored layer on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// Forward  (Eq. 3 applied to a batch):  T = X B^T,  Y = T A^T      -> chain kernel
// Backward (chain rule through Eq. 3):  dT = dY A,  dX = dT B      -> the same chain kernel on
//                                                                     pre-transposed factors
//                                       dA = dY^T T, dB = dT^T X   -> lr_tn2.hip
//
// MFMA 32x32x16 bf16 register layout (lane l of 64, h = l / 32):
//   A operand: 8 bf16 = A[l % 32][8h .. 8h+7]   (row of the 32 x 16 left block)
//   B operand: 8 bf16 = B[8h .. 8h+7][l % 32]   (column of the 16 x 32 right block)
//   accumulator register v: C[8*(v/4) + 4h + v%4][l % 32]
// The contraction index may be permuted freely as long as both operands use the same
// permutation; the chain kernel relies on that to feed accumulators straight back as operands.
#include "common.h"

namespace abt {

namespace {

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
}

// =====================================================================================
// Chain kernel:  Tout[M,R] = Xin[M,p] . P[R,p]^T   then   Yout[M,q] = Tout . Q[q,R]^T
//
// 256 threads = 4 waves; a work-group owns 128 consecutive rows and every wave owns 32 of them
// from the first load to the last store, so T never crosses waves:
//   stage 1 computes T^T blocks (A operand = P rows from LDS, B operand = X rows straight from
//           global memory), which leaves each lane holding one row of T, 4 consecutive r per
//           accumulator quad;
//   those accumulators, rounded to bf16, are already a valid B operand for stage 2 under the
//           k-permutation  slot s of half h  <->  r = 16*kb + 8*(s/4) + 4h + s%4 ;
//   stage 2 computes Y^T blocks (A operand = Q rows from LDS, stored with that same permutation
//           applied inside every group of 16 columns), so each lane ends with 4 consecutive
//           output columns of one row: an 8-byte store.
// LDS holds only the factor slabs (double-buffered); T lives in registers.
// =====================================================================================
constexpr int CH_ROWS = 128;     // rows per work-group
constexpr int CH_BK = 64;        // stage-1 slab of the contraction dimension p
constexpr int CH_BN = 64;        // stage-2 chunk of output columns q
constexpr int CH_PITCH1 = (CH_BK + 8) * 2;  // bytes per P row in LDS (144: odd number of 16 B granules)

template <int R>
struct ChainLds {
    static constexpr int pitch2 = (R + 8) * 2;                 // bytes per Q row (odd granule count)
    static constexpr int stage1 = 2 * R * CH_PITCH1;
    static constexpr int stage2 = 2 * CH_BN * pitch2;
    static constexpr int bytes = stage1 > stage2 ? stage1 : stage2;
};

template <int R>
__global__ __launch_bounds__(256) void chain_bf16_kernel(const uint16_t* __restrict__ Xin,
                                                         const uint16_t* __restrict__ Pm,
                                                         const uint16_t* __restrict__ Qm,
                                                         uint16_t* __restrict__ Yout,
                                                         uint16_t* __restrict__ Tout,
                                                         int64_t M, int p, int q) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int RB = R / 32;   // 32-row blocks of r
    constexpr int KB2 = R / 16;  // stage-2 k16 steps
    constexpr int pitch2 = ChainLds<R>::pitch2;

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int lj = lane & 31, lh = lane >> 5;
    const int64_t row = (int64_t)blockIdx.x * CH_ROWS + wave * 32 + lj;
    const int64_t row_ld = row < M ? row : M - 1;  // tail rows read a valid row and store nothing

    // ------------------------------------------------------------------ stage 1
    f32x16 acc1[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc1[rb][v] = 0.0f;

    {
        constexpr int NLD = R / 32;  // 16-byte chunks of the P slab per thread (R rows x 8 chunks / 256)
        u32x4 gp[NLD];
        u32x4 xf[4], xn[4];
        const uint16_t* xrow = Xin + row_ld * p + 8 * lh;
        auto load_slab = [&](int k0) {
#pragma unroll
            for (int e = 0; e < NLD; ++e) {
                const int c = e * 256 + t;
                gp[e] = *reinterpret_cast<const u32x4*>(Pm + (int64_t)(c >> 3) * p + k0 + (c & 7) * 8);
            }
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
                xn[kb] = *reinterpret_cast<const u32x4*>(xrow + k0 + 16 * kb);
        };
        const int nslab = p / CH_BK;
        load_slab(0);
        for (int s = 0; s < nslab; ++s) {
            unsigned char* buf = lds + (s & 1) * (R * CH_PITCH1);
#pragma unroll
            for (int e = 0; e < NLD; ++e) {
                const int c = e * 256 + t;
                *reinterpret_cast<u32x4*>(buf + (c >> 3) * CH_PITCH1 + (c & 7) * 16) = gp[e];
            }
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) xf[kb] = xn[kb];
            __syncthreads();
            if (s + 1 < nslab) load_slab((s + 1) * CH_BK);
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    const u32x4 a = *reinterpret_cast<const u32x4*>(
                        buf + (rb * 32 + lj) * CH_PITCH1 + (16 * kb + 8 * lh) * 2);
                    acc1[rb] = mfma_bf16(a, xf[kb], acc1[rb]);
                }
            }
        }
    }

    // ------------------------------------------------------------------ T: round, keep, store
    // tf[kb2] is the stage-2 B operand for k16 step kb2: slots 0..3 = r 16kb2+4h+(0..3),
    // slots 4..7 = r 16kb2+8+4h+(0..3).
    u32x4 tf[KB2];
#pragma unroll
    for (int kb2 = 0; kb2 < KB2; ++kb2) {
        const int rb = kb2 >> 1, g0 = (kb2 & 1) * 2;
        tf[kb2][0] = pack2_bf16(acc1[rb][4 * g0 + 0], acc1[rb][4 * g0 + 1]);
        tf[kb2][1] = pack2_bf16(acc1[rb][4 * g0 + 2], acc1[rb][4 * g0 + 3]);
        tf[kb2][2] = pack2_bf16(acc1[rb][4 * g0 + 4], acc1[rb][4 * g0 + 5]);
        tf[kb2][3] = pack2_bf16(acc1[rb][4 * g0 + 6], acc1[rb][4 * g0 + 7]);
    }
    if (Tout != nullptr && row < M) {
        uint16_t* trow = Tout + row * R + 4 * lh;
#pragma unroll
        for (int kb2 = 0; kb2 < KB2; ++kb2) {
            u32x2 lo = {tf[kb2][0], tf[kb2][1]}, hi = {tf[kb2][2], tf[kb2][3]};
            *reinterpret_cast<u32x2*>(trow + 16 * kb2) = lo;
            *reinterpret_cast<u32x2*>(trow + 16 * kb2 + 8) = hi;
        }
    }
    if (Yout == nullptr) return;

    // ------------------------------------------------------------------ stage 2
    __syncthreads();  // stage-1 slabs are dead; the buffers are reused for Q chunks
    {
        constexpr int CPR = R / 8;            // 16-byte chunks per Q row
        constexpr int NLD = CH_BN * CPR / 256;  // chunks per thread (= R / 32)
        u32x4 gq[NLD];
        auto load_chunk = [&](int c0) {
            const uint16_t* base = Qm + (int64_t)c0 * R;  // rows c0..c0+63 are contiguous
#pragma unroll
            for (int e = 0; e < NLD; ++e)
                gq[e] = *reinterpret_cast<const u32x4*>(base + (int64_t)(e * 256 + t) * 8);
        };
        const int nchunk = q / CH_BN;
        load_chunk(0);
        for (int c = 0; c < nchunk; ++c) {
            unsigned char* buf = lds + (c & 1) * (CH_BN * pitch2);
#pragma unroll
            for (int e = 0; e < NLD; ++e) {
                const int lin = e * 256 + t;
                const int qr = lin / CPR, ch = lin % CPR;
                // columns 8ch..8ch+7 of the row: the first four go to slot group (ch&1) of half 0,
                // the last four to the same slot group of half 1 (see the permutation above).
                unsigned char* dst = buf + qr * pitch2 + ((ch >> 1) * 16 + (ch & 1) * 4) * 2;
                u32x2 lo = {gq[e][0], gq[e][1]}, hi = {gq[e][2], gq[e][3]};
                *reinterpret_cast<u32x2*>(dst) = lo;
                *reinterpret_cast<u32x2*>(dst + 16) = hi;
            }
            __syncthreads();
            if (c + 1 < nchunk) load_chunk((c + 1) * CH_BN);

            f32x16 acc2[CH_BN / 32];
#pragma unroll
            for (int mb = 0; mb < CH_BN / 32; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[mb][v] = 0.0f;
#pragma unroll
            for (int kb2 = 0; kb2 < KB2; ++kb2) {
#pragma unroll
                for (int mb = 0; mb < CH_BN / 32; ++mb) {
                    const u32x4 a = *reinterpret_cast<const u32x4*>(
                        buf + (mb * 32 + lj) * pitch2 + (16 * kb2 + 8 * lh) * 2);
                    acc2[mb] = mfma_bf16(a, tf[kb2], acc2[mb]);
                }
            }
            if (row < M) {
                uint16_t* yrow = Yout + row * q + c * CH_BN + 4 * lh;
#pragma unroll
                for (int mb = 0; mb < CH_BN / 32; ++mb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x2 o = {pack2_bf16(acc2[mb][4 * g + 0], acc2[mb][4 * g + 1]),
                                   pack2_bf16(acc2[mb][4 * g + 2], acc2[mb][4 * g + 3])};
                        *reinterpret_cast<u32x2*>(yrow + mb * 32 + 8 * g) = o;
                    }
            }
        }
    }
}

template <int R>
hipError_t launch_chain_r(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                          int64_t M, int p, int q, hipStream_t s) {
    constexpr int lds_bytes = ChainLds<R>::bytes;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&chain_bf16_kernel<R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t grid = ceil_div(M, CH_ROWS);
    hipLaunchKernelGGL(chain_bf16_kernel<R>, dim3((unsigned)grid), dim3(256), lds_bytes, s,
                       (const uint16_t*)Xin, (const uint16_t*)P, (const uint16_t*)Q,
                       (uint16_t*)Yout, (uint16_t*)Tout, M, p, q);
    return hipGetLastError();
}

// =====================================================================================
// bf16 transpose (for A^T and B^T, which turn dT = dY A and dX = dT B into the same
// "rows times rows" shape the chain kernel consumes).
// =====================================================================================
// One launch serves up to kTransposeMaxJobs matrices (rows and cols multiples of 8).  A work-group moves one
// 64 x 64 tile: 16-byte loads of row pieces into LDS, 16-byte stores of column pieces out of it.
struct TrJob { const uint16_t* src; uint16_t* dst; int rows, cols, tiles_x, tile_begin; };
struct TrArgs { TrJob job[kTransposeMaxJobs]; int njobs; };

__global__ __launch_bounds__(256) void transpose_bf16_kernel(TrArgs args) {
    __shared__ uint16_t tile[64][72];                  // pitch 144 B: 16-byte aligned rows
    int jid = 0;
    for (int i = 1; i < args.njobs; ++i)
        if ((int)blockIdx.x >= args.job[i].tile_begin) jid = i;
    const TrJob j = args.job[jid];
    const int t = (int)blockIdx.x - j.tile_begin;
    const int r0 = (t / j.tiles_x) * 64, c0 = (t % j.tiles_x) * 64;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int ci = e * 256 + threadIdx.x;          // 64 rows x 8 chunks of 8 elements
        const int row = ci >> 3, ch = ci & 7;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r0 + row < j.rows && c0 + ch * 8 < j.cols)
            v = *reinterpret_cast<const u32x4*>(j.src + (int64_t)(r0 + row) * j.cols + c0 + ch * 8);
        *reinterpret_cast<u32x4*>(&tile[row][ch * 8]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int ci = e * 256 + threadIdx.x;          // 64 output rows (source columns) x 8 chunks
        const int orow = ci >> 3, ch = ci & 7;
        if (c0 + orow < j.cols && r0 + ch * 8 < j.rows) {
            uint16_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = tile[ch * 8 + i][orow];
            u32x4 o = {(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16),
                       (uint32_t)v[4] | ((uint32_t)v[5] << 16), (uint32_t)v[6] | ((uint32_t)v[7] << 16)};
            *reinterpret_cast<u32x4*>(j.dst + (int64_t)(c0 + orow) * j.rows + r0 + ch * 8) = o;
        }
    }
}

// Re-layout of the factor B [r, taps C] of a factored convolution for the activation gradient:
// Pst [C, taps r_pad] with Pst[c, tap r_pad + j] = B[j, tap C + c] for j < r and 0 for r <= j < r_pad
// (every tap padded to a multiple of 64 columns, the slab width of the chain kernel).  One thread
// writes eight consecutive j (16 bytes).
__global__ __launch_bounds__(256) void conv_bstack_kernel(const uint16_t* __restrict__ B, uint16_t* __restrict__ Pst,
                                                          int r, int C, int taps, int r_pad) {
    const int per_row = taps * (r_pad / 8);
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)C * per_row) return;
    const int c = (int)(idx / per_row), rest = (int)(idx % per_row);
    const int tap = rest / (r_pad / 8), j0 = (rest % (r_pad / 8)) * 8;
    uint16_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = j0 + i < r ? B[(int64_t)(j0 + i) * taps * C + (int64_t)tap * C + c] : (uint16_t)0;
    u32x4 o = {(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16),
               (uint32_t)v[4] | ((uint32_t)v[5] << 16), (uint32_t)v[6] | ((uint32_t)v[7] << 16)};
    *reinterpret_cast<u32x4*>(Pst + (int64_t)c * taps * r_pad + (int64_t)tap * r_pad + j0) = o;
}

}  // namespace

hipError_t launch_conv_bstack_bf16(const void* B, void* Pst, int r, int C, int taps, int r_pad, hipStream_t s) {
    if (r < 1 || C < 1 || taps < 1 || r_pad % 64 || r_pad < r) return hipErrorInvalidValue;
    const int64_t n = (int64_t)C * taps * (r_pad / 8);
    hipLaunchKernelGGL(conv_bstack_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s,
                       (const uint16_t*)B, (uint16_t*)Pst, r, C, taps, r_pad);
    return hipGetLastError();
}

#define ABT_DISPATCH_R(R_, CALL)                          \
    switch (R_) {                                         \
        case 32: return CALL(32);                         \
        case 64: return CALL(64);                         \
        case 96: return CALL(96);                         \
        case 128: return CALL(128);                       \
        case 160: return CALL(160);                       \
        case 192: return CALL(192);                       \
        case 224: return CALL(224);                       \
        case 256: return CALL(256);                       \
        case 288: return CALL(288);                       \
        case 320: return CALL(320);                       \
        case 352: return CALL(352);                       \
        case 384: return CALL(384);                       \
        default: return hipErrorInvalidValue;             \
    }

hipError_t launch_chain_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                             int64_t M, int p, int q, int R, hipStream_t s) {
#define CALL(RR) launch_chain_r<RR>(Xin, P, Q, Yout, Tout, M, p, q, s)
    ABT_DISPATCH_R(R, CALL)
#undef CALL
}

hipError_t launch_transpose_bf16(const TransposeJob* jobs, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kTransposeMaxJobs) return hipErrorInvalidValue;
    TrArgs args{};
    args.njobs = njobs;
    int tiles = 0;
    for (int i = 0; i < njobs; ++i) {
        if (jobs[i].rows % 8 || jobs[i].cols % 8) return hipErrorInvalidValue;
        const int tx = (jobs[i].cols + 63) / 64, ty = (jobs[i].rows + 63) / 64;
        args.job[i] = TrJob{(const uint16_t*)jobs[i].src, (uint16_t*)jobs[i].dst, jobs[i].rows, jobs[i].cols, tx, tiles};
        tiles += tx * ty;
    }
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3(tiles), dim3(256), 0, s, args);
    return hipGetLastError();
}

}  // namespace abt
