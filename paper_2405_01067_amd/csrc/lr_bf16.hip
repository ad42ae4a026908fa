// bf16 factored layer on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// Forward  (Eq. 3 applied to a batch):  T = X B^T,  Y = T A^T      -> chain kernel
// Backward (chain rule through Eq. 3):  dT = dY A,  dX = dT B      -> the same chain kernel on
//                                                                     pre-transposed factors
//                                       dA = dY^T T, dB = dT^T X   -> split-row TN kernel + reduce
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
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ src,
                                                             uint16_t* __restrict__ dst,
                                                             int rows, int cols) {
    __shared__ uint16_t tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[(int64_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 64; i += 4)
        if (c0 + i < cols && r0 + tx < rows) dst[(int64_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

// =====================================================================================
// TN kernel:  part[split][P, R] = U[rows, P]^T . V[rows, R]   over the rows of one split.
// Both operands are stored with the contraction index (the batch row) as the slow dimension, so
// every thread transposes 8 x 8 bf16 patches in registers on the way into LDS; from there both
// MFMA operands are plain 16-byte reads.  One launch covers all jobs (dA and dB^T).
// Work-group tile: 128 (P) x R; waves 2 x 2 (R/32 even) or 4 x 1 (R/32 odd).
// =====================================================================================
constexpr int TN_BK = 64;                       // batch rows per slab
constexpr int TN_PITCH = (TN_BK + 8) * 2;       // bytes per transposed row in LDS
constexpr int TN_TP = 128;

struct TnDev {
    const uint16_t* U; const uint16_t* V; float* part; int P; int tile_begin;
};
struct TnArgs {
    TnDev job[2];
    int njobs;
    int64_t M;
    int64_t rows_per_split;
};

// 8 x 8 bf16 transpose: in[r] holds row r (8 values), out[c] receives column c.
__device__ __forceinline__ void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t a = in[2 * d][c >> 1], b = in[2 * d + 1][c >> 1];
            out[c][d] = (c & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
        }
}

template <int R>
struct TnCfg {
    static constexpr bool even = ((R / 32) % 2) == 0;
    static constexpr int WGP = even ? 2 : 4;   // waves along P
    static constexpr int WGQ = even ? 2 : 1;   // waves along R
    static constexpr int PB = even ? 2 : 1;    // 32-blocks per wave along P
    static constexpr int QB = even ? R / 64 : R / 32;
    static constexpr int lds_bytes = 2 * (TN_TP + R) * TN_PITCH;
};

template <int R>
__global__ __launch_bounds__(256) void tn_bf16_kernel(TnArgs args) {
    extern __shared__ __align__(16) unsigned char lds[];
    using C = TnCfg<R>;
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int lj = lane & 31, lh = lane >> 5;

    const int job_id = (args.njobs > 1 && (int)blockIdx.x >= args.job[1].tile_begin) ? 1 : 0;
    const TnDev job = args.job[job_id];
    const int p0 = ((int)blockIdx.x - job.tile_begin) * TN_TP;
    const int split = blockIdx.y;
    const int64_t k_begin = (int64_t)split * args.rows_per_split;
    int64_t k_end = k_begin + args.rows_per_split;
    if (k_end > args.M) k_end = args.M;

    const int wp = (wave / C::WGQ) * (C::PB * 32);
    const int wq = (wave % C::WGQ) * (C::QB * 32);

    f32x16 acc[C::PB][C::QB];
#pragma unroll
    for (int a = 0; a < C::PB; ++a)
#pragma unroll
        for (int b = 0; b < C::QB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // patch list of one slab: (TN_TP/8 + R/8) column groups x 8 row groups, 8 x 8 values each
    constexpr int CG_U = TN_TP / 8, CG_V = R / 8;
    constexpr int NPATCH = (CG_U + CG_V) * (TN_BK / 8);
    constexpr int PER_THREAD = (NPATCH + 255) / 256;

    u32x4 stage[PER_THREAD][8];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    auto load_slab = [&](int64_t k0) {
#pragma unroll
        for (int e = 0; e < PER_THREAD; ++e) {
            const int pid = e * 256 + t;
            if (pid < NPATCH) {
                // consecutive threads walk the column groups of one row group: coalesced rows
                const int cg = pid % (CG_U + CG_V), rg = pid / (CG_U + CG_V);
                const bool isU = cg < CG_U;
                const int col = isU ? p0 + cg * 8 : (cg - CG_U) * 8;
                const int ld = isU ? job.P : R;
                const uint16_t* base = isU ? job.U : job.V;
                const bool col_ok = isU ? (col < job.P) : true;
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int64_t k = k0 + rg * 8 + rr;
                    stage[e][rr] = (col_ok && k < k_end)
                                       ? *reinterpret_cast<const u32x4*>(base + k * ld + col) : zero4;
                }
            }
        }
    };
    auto store_slab = [&](unsigned char* buf) {
#pragma unroll
        for (int e = 0; e < PER_THREAD; ++e) {
            const int pid = e * 256 + t;
            if (pid < NPATCH) {
                const int cg = pid % (CG_U + CG_V), rg = pid / (CG_U + CG_V);
                u32x4 tr[8];
                transpose8x8(stage[e], tr);
                // LDS row = tile column (U columns first, then V columns); 8 batch rows = 16 bytes
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    *reinterpret_cast<u32x4*>(buf + (cg * 8 + c) * TN_PITCH + rg * 16) = tr[c];
            }
        }
    };

    const int64_t nrows = k_end > k_begin ? k_end - k_begin : 0;
    const int nslab = (int)((nrows + TN_BK - 1) / TN_BK);
    constexpr int buf_bytes = (TN_TP + R) * TN_PITCH;
    if (nslab > 0) load_slab(k_begin);
    for (int s = 0; s < nslab; ++s) {
        unsigned char* buf = lds + (s & 1) * buf_bytes;
        store_slab(buf);
        __syncthreads();
        if (s + 1 < nslab) load_slab(k_begin + (int64_t)(s + 1) * TN_BK);
        const unsigned char* ub = buf;
        const unsigned char* vb = buf + TN_TP * TN_PITCH;
#pragma unroll
        for (int kb = 0; kb < TN_BK / 16; ++kb) {
            u32x4 bf[C::QB];
#pragma unroll
            for (int b = 0; b < C::QB; ++b)
                bf[b] = *reinterpret_cast<const u32x4*>(vb + (wq + b * 32 + lj) * TN_PITCH + (16 * kb + 8 * lh) * 2);
#pragma unroll
            for (int a = 0; a < C::PB; ++a) {
                const u32x4 af = *reinterpret_cast<const u32x4*>(
                    ub + (wp + a * 32 + lj) * TN_PITCH + (16 * kb + 8 * lh) * 2);
#pragma unroll
                for (int b = 0; b < C::QB; ++b) acc[a][b] = mfma_bf16(af, bf[b], acc[a][b]);
            }
        }
    }

    float* part = job.part + (int64_t)split * job.P * R;
#pragma unroll
    for (int a = 0; a < C::PB; ++a)
#pragma unroll
        for (int b = 0; b < C::QB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int prow = p0 + wp + a * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (prow < job.P) part[(int64_t)prow * R + wq + b * 32 + lj] = acc[a][b][v];
            }
}

// out (+)= sum over splits of part[split]; part is [P, R]; out is [P, R] or, transposed, [R, P].
struct ReduceJob { const float* part; float* out; int P; int transposed; };
struct ReduceArgs { ReduceJob job[2]; int njobs; int R; int splits; int accumulate; int blocks0; };

__global__ __launch_bounds__(256) void tn_reduce_kernel(ReduceArgs a) {
    const int jid = (a.njobs > 1 && (int)blockIdx.x >= a.blocks0) ? 1 : 0;
    const ReduceJob j = a.job[jid];
    const int64_t idx = (int64_t)((int)blockIdx.x - (jid ? a.blocks0 : 0)) * 256 + threadIdx.x;
    const int64_t total = (int64_t)j.P * a.R;
    if (idx >= total) return;
    // idx enumerates the OUTPUT in its own row-major order, so stores are coalesced
    int64_t pidx;
    if (j.transposed) {
        const int64_t rr = idx / j.P, pp = idx % j.P;
        pidx = pp * a.R + rr;
    } else {
        pidx = idx;
    }
    float sum = 0.0f;
    for (int s = 0; s < a.splits; ++s) sum += j.part[(int64_t)s * total + pidx];
    if (a.accumulate) sum += j.out[idx];
    j.out[idx] = sum;
}

int tn_choose_splits(int64_t M, int total_tiles) {
    // aim at about two work-groups per compute unit, at least 4 slabs of rows per split
    int64_t want = (2 * 256 + total_tiles - 1) / total_tiles;
    int64_t max_by_rows = M / (4 * TN_BK);
    if (max_by_rows < 1) max_by_rows = 1;
    if (want > max_by_rows) want = max_by_rows;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    return (int)want;
}

template <int R>
hipError_t launch_tn_r(const TnArgs& args, int tiles, int splits, hipStream_t s) {
    constexpr int lds_bytes = TnCfg<R>::lds_bytes;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tn_bf16_kernel<R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(tn_bf16_kernel<R>, dim3(tiles, splits), dim3(256), lds_bytes, s, args);
    return hipGetLastError();
}

}  // namespace

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

hipError_t launch_transpose_bf16(const void* src, void* dst, int rows, int cols, hipStream_t s) {
    dim3 grid((cols + 63) / 64, (rows + 63) / 64);
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, s, (const uint16_t*)src,
                       (uint16_t*)dst, rows, cols);
    return hipGetLastError();
}

static int tn_total_tiles(const TnJob* jobs, int njobs) {
    int tiles = 0;
    for (int i = 0; i < njobs; ++i) tiles += (jobs[i].P + TN_TP - 1) / TN_TP;
    return tiles;
}

size_t tn_partials_bytes(int64_t M, const TnJob* jobs, int njobs, int R) {
    const int splits = tn_choose_splits(M, tn_total_tiles(jobs, njobs));
    size_t elems = 0;
    for (int i = 0; i < njobs; ++i) elems += (size_t)jobs[i].P * R;
    return elems * splits * sizeof(float);
}

hipError_t launch_tn_bf16(const TnJob* jobs, int njobs, int64_t M, int R, int accumulate,
                          float* partials, hipStream_t s) {
    if (njobs < 1 || njobs > 2) return hipErrorInvalidValue;
    const int tiles = tn_total_tiles(jobs, njobs);
    const int splits = tn_choose_splits(M, tiles);
    TnArgs args{};
    ReduceArgs red{};
    args.njobs = red.njobs = njobs;
    args.M = M;
    int64_t rps = ceil_div(M, splits);
    rps = ceil_div(rps, TN_BK) * TN_BK;
    args.rows_per_split = rps;
    red.R = R; red.splits = splits; red.accumulate = accumulate;
    float* part = partials;
    int tile_begin = 0, red_blocks = 0;
    for (int i = 0; i < njobs; ++i) {
        args.job[i].U = (const uint16_t*)jobs[i].U;
        args.job[i].V = (const uint16_t*)jobs[i].V;
        args.job[i].part = part;
        args.job[i].P = jobs[i].P;
        args.job[i].tile_begin = tile_begin;
        red.job[i].part = part;
        red.job[i].out = jobs[i].out;
        red.job[i].P = jobs[i].P;
        red.job[i].transposed = jobs[i].transposed;
        tile_begin += (jobs[i].P + TN_TP - 1) / TN_TP;
        const int blocks = (int)ceil_div((int64_t)jobs[i].P * R, 256);
        if (i == 0) red.blocks0 = blocks;
        red_blocks += blocks;
        part += (size_t)jobs[i].P * R * splits;
    }
    hipError_t e;
#define CALL(RR) launch_tn_r<RR>(args, tiles, splits, s)
    auto run = [&]() -> hipError_t { ABT_DISPATCH_R(R, CALL) };
#undef CALL
    e = run();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tn_reduce_kernel, dim3(red_blocks), dim3(256), 0, s, red);
    return hipGetLastError();
}

}  // namespace abt
