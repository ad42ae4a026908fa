// Chain kernel, 64-row work-groups:  Tout[M,R] = Xin[M,p] . P[R,p]^T  then  Yout[M,q] = Tout . Q[q,R]^T
// (bf16 in, fp32 accumulate).  Forward of the factored layer with (Xin,P,Q) = (X,B,A); the
// dT/dX half of the backward with (dY, A^T, B^T).
//
// A work-group owns 64 rows and runs 8 waves (two per SIMD).
//
//   stage 1: slabs of BK1 contraction columns: 64 rows of Xin and the R rows of P.  The waves form
//            CS column groups x KS contraction groups; a wave keeps a 64 x (R/CS) block of T^T in
//            accumulators and takes every KS-th k16 step.  The KS partial sums are then added in
//            a fixed tree order through LDS.
//   T:       rounded to bf16 once, written as a 64 x R tile to LDS (and to Tout), from where every
//            wave loads all of it as MFMA operands: T stays in registers for the whole of stage 2.
//   stage 2: a round produces 256 output columns, 32 per wave, from slabs of 256 rows of Q; the
//            finished 64 x 256 tile is staged in LDS and leaves as full 512-byte row segments.
//
// Slabs travel global -> registers -> LDS (two LDS slots, one barrier per slab).  The factor
// slabs come out of L2 and are fetched two slabs ahead (two register sets); the activation slab
// of stage 1 comes from HBM and is fetched six slabs ahead (a ring of six register sets, the slab
// loop is unrolled by six so that every ring index is a compile-time constant).
// (The direct-to-LDS loads of gfx950 were measured at about half the rate of this path per wave
// and are not used.)
//
// LDS slab layout: row-major, 16-byte chunks XOR-swizzled inside each row so that the 16 rows a
// quarter-wave reads for one MFMA operand fall on different banks.
//
// MFMA 32x32x16 bf16 layout (lane l, h = l/32): A operand = 8 values A[l%32][8h..8h+7], B operand
// = B[8h..8h+7][l%32], accumulator v = C[8(v/4) + 4h + v%4][l%32].
#include <cstdlib>

#include "common.h"

namespace abt {

namespace {

__device__ __forceinline__ bf16x8 as_bf(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ f32x16 mfma16(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(a), as_bf(b), c, 0, 0, 0);
}

// Work-group barrier of the slab loops: this wave's LDS traffic has completed, then s_barrier.
// Deliberately not __syncthreads(): that also drains the outstanding global loads, which are
// exactly the prefetches that must stay in flight across the barrier.
__device__ __forceinline__ void ring_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// chunk swizzle for rows of CPR 16-byte chunks: XOR the low bits of the chunk index with row bits
// chosen so that 16 consecutive rows, same logical chunk, hit 16 different 16-byte bank groups.
template <int CPR>
__device__ __forceinline__ int swz(int chunk, int row) {
    if constexpr (CPR % 16 == 0) return chunk ^ (row & 15);
    else if constexpr (CPR % 8 == 0) return chunk ^ ((row >> 1) & 7);
    else return chunk ^ ((row >> 2) & 3);
}

template <int R> struct Ch2;
template <> struct Ch2<32>  { static constexpr int CS = 1, KS = 8, BK1 = 128, BK2 = 32; };
template <> struct Ch2<64>  { static constexpr int CS = 2, KS = 4, BK1 = 64,  BK2 = 64; };
template <> struct Ch2<96>  { static constexpr int CS = 1, KS = 8, BK1 = 128, BK2 = 32; };
template <> struct Ch2<128> { static constexpr int CS = 2, KS = 4, BK1 = 64,  BK2 = 64; };
template <> struct Ch2<192> { static constexpr int CS = 2, KS = 4, BK1 = 64,  BK2 = 64; };
template <> struct Ch2<256> { static constexpr int CS = 4, KS = 2, BK1 = 64,  BK2 = 64; };
template <> struct Ch2<384> { static constexpr int CS = 4, KS = 2, BK1 = 64,  BK2 = 64; };

constexpr int DX = 6;   // activation slabs in flight (register ring); the slab loop is unrolled by DX

template <int R>
struct Ch2Lds {
    using C = Ch2<R>;
    static constexpr int CB = R / 32 / C::CS;
    static constexpr int xslab = 64 * C::BK1 * 2, pslab = R * C::BK1 * 2;
    static constexpr int stage1 = 2 * (xslab + pslab);
    static constexpr int qslab = 256 * C::BK2 * 2;
    static constexpr int ypitch = 256 * 2 + 16;
    static constexpr int ytile = 64 * ypitch;
    static constexpr int stage2 = 2 * qslab + ytile;
    static constexpr int red = (C::KS / 2) * C::CS * CB * 8192;   // first (largest) round of the tree
    static constexpr int tpitch = R * 2 + 16;
    static constexpr int ttile = 64 * tpitch;
    static constexpr int mid = red + ttile;
    static constexpr int ab = stage1 > stage2 ? stage1 : stage2;
    static constexpr int bytes = ab > mid ? ab : mid;
};

template <int R>
__global__ __launch_bounds__(512) void chain2_bf16_kernel(const uint16_t* __restrict__ Xin,
                                                          const uint16_t* __restrict__ Pm,
                                                          const uint16_t* __restrict__ Qm,
                                                          uint16_t* __restrict__ Yout,
                                                          uint16_t* __restrict__ Tout,
                                                          int64_t M, int p, int q) {
    extern __shared__ __align__(1024) unsigned char lds[];
    using C = Ch2<R>;
    using L = Ch2Lds<R>;
    constexpr int CS = C::CS, KS = C::KS, CB = L::CB;
    constexpr int BK1 = C::BK1, CPR1 = BK1 / 8, SPW = BK1 / (16 * KS);
    constexpr int NX = 64 * CPR1 / 512;          // 16-byte chunks per thread: activation slab
    constexpr int NPC = (R * CPR1 + 511) / 512;  // factor slab (the last one may be partial: guarded)
    static_assert(SPW >= 1 && NX >= 1, "slab shape");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 31, lh = lane >> 5;
    const int64_t row0 = (int64_t)blockIdx.x * 64;
    const int cs = wave % CS, ks = wave / CS;

    // ------------------------------------------------------------------ stage 1
    f32x16 acc1[2][CB];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc1[a][b][v] = 0.0f;

    unsigned char* const xs = lds;                       // [2][64][BK1]
    unsigned char* const ps = lds + 2 * L::xslab;        // [2][R][BK1]

    // per-thread chunk coordinates (constant over the slabs)
    int xoff[NX];
    const uint16_t* xsrc[NX];
#pragma unroll
    for (int e = 0; e < NX; ++e) {
        const int ci = e * 512 + tid;
        const int row = ci / CPR1, ch = ci % CPR1;
        xoff[e] = row * (BK1 * 2) + swz<CPR1>(ch, row) * 16;
        int64_t rr = row0 + row;
        if (rr >= M) rr = M - 1;                         // tail rows read a valid row, store nothing
        xsrc[e] = Xin + rr * p + ch * 8;
    }
    int poff[NPC];
    const uint16_t* psrc[NPC];
#pragma unroll
    for (int e = 0; e < NPC; ++e) {
        const int ci = e * 512 + tid;
        const int row = ci / CPR1, ch = ci % CPR1;
        poff[e] = row * (BK1 * 2) + swz<CPR1>(ch, row) * 16;
        psrc[e] = Pm + (int64_t)(row < R ? row : R - 1) * p + ch * 8;
    }

    const int ns1 = p / BK1;
    u32x4 xr[DX][NX], pr[2][NPC];
    auto load_x = [&](u32x4 (&dst)[NX], int s) {
#pragma unroll
        for (int e = 0; e < NX; ++e) dst[e] = *reinterpret_cast<const u32x4*>(xsrc[e] + (int64_t)s * BK1);
    };
    auto load_p = [&](u32x4 (&dst)[NPC], int s) {
#pragma unroll
        for (int e = 0; e < NPC; ++e) dst[e] = *reinterpret_cast<const u32x4*>(psrc[e] + (int64_t)s * BK1);
    };
    auto store_x = [&](const u32x4 (&src)[NX], int slot) {
#pragma unroll
        for (int e = 0; e < NX; ++e) *reinterpret_cast<u32x4*>(xs + slot * L::xslab + xoff[e]) = src[e];
    };
    auto store_p = [&](const u32x4 (&src)[NPC], int slot) {
#pragma unroll
        for (int e = 0; e < NPC; ++e)
            if (e * 512 + tid < R * CPR1) *reinterpret_cast<u32x4*>(ps + slot * L::pslab + poff[e]) = src[e];
    };

    // prologue: slab 0 into LDS slot 0; slabs 1..DX of X and 1..2 of P into the register rings
    if (ns1 > 0) {
        load_x(xr[0], 0);
        load_p(pr[0], 0);
        store_x(xr[0], 0);
        store_p(pr[0], 0);
#pragma unroll
        for (int d = 1; d <= DX; ++d)
            if (d < ns1) load_x(xr[d % DX], d);
        if (1 < ns1) load_p(pr[1], 1);
        if (2 < ns1) load_p(pr[0], 2);
    }
    ring_barrier();

    for (int s0 = 0; s0 < ns1; s0 += DX) {
#pragma unroll
        for (int d = 0; d < DX; ++d) {
            const int s = s0 + d;
            if (s < ns1) {
                // stage slab s+1 (slot (s+1)&1 was last read in iteration s-1, before its barrier)
                if (s + 1 < ns1) {
                    store_x(xr[(d + 1) % DX], (d + 1) & 1);
                    store_p(pr[(d + 1) & 1], (d + 1) & 1);
                }
                if (s + 1 + DX < ns1) load_x(xr[(d + 1) % DX], s + 1 + DX);
                if (s + 3 < ns1) load_p(pr[(d + 1) & 1], s + 3);
                // consume slab s
                const unsigned char* xb = xs + (d & 1) * L::xslab;
                const unsigned char* pb = ps + (d & 1) * L::pslab;
#pragma unroll
                for (int j = 0; j < SPW; ++j) {
                    const int kk = ks * SPW + j;          // k16 step inside the slab
                    const int qc = 2 * kk + lh;           // logical chunk of this lane's 8 values
                    u32x4 xf[2], pf[CB];
#pragma unroll
                    for (int a = 0; a < 2; ++a) {
                        const int row = 32 * a + lj;
                        xf[a] = *reinterpret_cast<const u32x4*>(xb + row * (BK1 * 2) + swz<CPR1>(qc, row) * 16);
                    }
#pragma unroll
                    for (int b = 0; b < CB; ++b) {
                        const int row = (cs * CB + b) * 32 + lj;
                        pf[b] = *reinterpret_cast<const u32x4*>(pb + row * (BK1 * 2) + swz<CPR1>(qc, row) * 16);
                    }
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int b = 0; b < CB; ++b) acc1[a][b] = mfma16(pf[b], xf[a], acc1[a][b]);
                }
                ring_barrier();
            }
        }
    }

    // ------------------------------------------------------------------ tree reduction over the KS groups
    {
        float* red = reinterpret_cast<float*>(lds);
#pragma unroll
        for (int half = KS / 2; half >= 1; half >>= 1) {
            if (ks >= half && ks < 2 * half) {
                float* dst = red + (size_t)(((ks - half) * CS + cs) * (2 * CB)) * 16 * 64;
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < CB; ++b)
#pragma unroll
                        for (int v = 0; v < 16; ++v) dst[((a * CB + b) * 16 + v) * 64 + lane] = acc1[a][b][v];
            }
            __syncthreads();
            if (ks < half) {
                const float* src = red + (size_t)((ks * CS + cs) * (2 * CB)) * 16 * 64;
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < CB; ++b)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc1[a][b][v] += src[((a * CB + b) * 16 + v) * 64 + lane];
            }
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ T tile (bf16) to LDS, Tout, operand registers
    unsigned char* ttile = lds + L::red;
    if (ks == 0) {
        // lane holds T[32a + lj][32(cs CB + b) + 8g + 4 lh + (0..3)] in acc1[a][b][4g .. 4g+3]
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 o = {pack2_bf16(acc1[a][b][4 * g + 0], acc1[a][b][4 * g + 1]),
                               pack2_bf16(acc1[a][b][4 * g + 2], acc1[a][b][4 * g + 3])};
                    *reinterpret_cast<u32x2*>(ttile + (32 * a + lj) * L::tpitch +
                                              (32 * (cs * CB + b) + 8 * g + 4 * lh) * 2) = o;
                }
    }
    __syncthreads();
    if (Tout != nullptr) {
        constexpr int CPT = R / 8;   // 16-byte chunks per T row
        for (int i = tid; i < 64 * CPT; i += 512) {
            const int row = i / CPT, ch = i % CPT;
            if (row0 + row < M)
                *reinterpret_cast<u32x4*>(Tout + (row0 + row) * R + ch * 8) =
                    *reinterpret_cast<const u32x4*>(ttile + row * L::tpitch + ch * 16);
        }
    }
    if (Yout == nullptr) return;

    constexpr int KB = R / 16;
    u32x4 tf[2][KB];   // B operands of stage 2: T[32a + lj][16kb + 8 lh .. +7]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
            tf[a][kb] = *reinterpret_cast<const u32x4*>(ttile + (32 * a + lj) * L::tpitch + (16 * kb + 8 * lh) * 2);
    __syncthreads();   // T tile consumed; stage 2 takes over the LDS

    // ------------------------------------------------------------------ stage 2
    constexpr int BK2 = C::BK2, CPR2 = BK2 / 8;
    constexpr int KSL = R / BK2;                 // slabs per round
    constexpr int NQ = 256 * CPR2 / 512;         // chunks per thread per slab
    unsigned char* const qs = lds;               // [2][256][BK2]
    unsigned char* const ytile = lds + 2 * L::qslab;
    const int nround = (q + 255) / 256;
    const int ns2 = nround * KSL;

    int qrow[NQ], qoff[NQ], qcol[NQ];
#pragma unroll
    for (int e = 0; e < NQ; ++e) {
        const int ci = e * 512 + tid;
        qrow[e] = ci / CPR2;
        const int ch = ci % CPR2;
        qcol[e] = ch * 8;
        qoff[e] = qrow[e] * (BK2 * 2) + swz<CPR2>(ch, qrow[e]) * 16;
    }
    u32x4 qr[2][NQ];
    auto load_q = [&](u32x4 (&dst)[NQ], int s) {
        const int round = s / KSL, kslab = s % KSL;
#pragma unroll
        for (int e = 0; e < NQ; ++e) {
            int row = round * 256 + qrow[e];
            if (row >= q) row = q - 1;
            dst[e] = *reinterpret_cast<const u32x4*>(Qm + (int64_t)row * R + kslab * BK2 + qcol[e]);
        }
    };
    auto store_q = [&](const u32x4 (&src)[NQ], int slot) {
#pragma unroll
        for (int e = 0; e < NQ; ++e) *reinterpret_cast<u32x4*>(qs + slot * L::qslab + qoff[e]) = src[e];
    };

    if (ns2 > 0) {
        load_q(qr[0], 0);
        store_q(qr[0], 0);
        if (1 < ns2) load_q(qr[1], 1);
        if (2 < ns2) load_q(qr[0], 2);
    }
    ring_barrier();

    f32x16 acc2[2];
    // rounds are processed in pairs so that the slab parity (LDS slot, register set) is a
    // compile-time constant even when a round has an odd number of slabs
    for (int rp = 0; rp < nround; rp += 2) {
#pragma unroll
        for (int rip = 0; rip < 2; ++rip) {
            const int round = rp + rip;
            if (round < nround) {
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc2[a][v] = 0.0f;
#pragma unroll
                for (int kslab = 0; kslab < KSL; ++kslab) {
                    const int u = rip * KSL + kslab;          // compile-time; its parity is the slab's
                    const int s = rp * KSL + u;
                    if (s + 1 < ns2) store_q(qr[(u + 1) & 1], (u + 1) & 1);
                    if (s + 3 < ns2) load_q(qr[(u + 1) & 1], s + 3);
                    const unsigned char* base = qs + (u & 1) * L::qslab;
#pragma unroll
                    for (int kk = 0; kk < BK2 / 16; ++kk) {
                        const int row = 32 * wave + lj;
                        const u32x4 qf = *reinterpret_cast<const u32x4*>(
                            base + row * (BK2 * 2) + swz<CPR2>(2 * kk + lh, row) * 16);
                        const int kb = kslab * (BK2 / 16) + kk;
                        acc2[0] = mfma16(qf, tf[0][kb], acc2[0]);
                        acc2[1] = mfma16(qf, tf[1][kb], acc2[1]);
                    }
                    ring_barrier();
                }
                // lane holds Y[32a + lj][32 wave + 8g + 4 lh + (0..3)] of this round's 64 x 256 tile
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x2 o = {pack2_bf16(acc2[a][4 * g + 0], acc2[a][4 * g + 1]),
                                   pack2_bf16(acc2[a][4 * g + 2], acc2[a][4 * g + 3])};
                        *reinterpret_cast<u32x2*>(ytile + (32 * a + lj) * L::ypitch + (32 * wave + 8 * g + 4 * lh) * 2) = o;
                    }
                ring_barrier();
                // 64 rows x 32 chunks of 16 bytes = 2048 chunks, 4 per thread, row-contiguous
                const int ncol = q - round * 256 < 256 ? q - round * 256 : 256;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ci = e * 512 + tid;
                    const int row = ci >> 5, ch = ci & 31;
                    if (row0 + row < M && ch * 8 < ncol)
                        *reinterpret_cast<u32x4*>(Yout + (row0 + row) * q + round * 256 + ch * 8) =
                            *reinterpret_cast<const u32x4*>(ytile + row * L::ypitch + ch * 16);
                }
            }
        }
    }
}

template <int R>
hipError_t launch_chain2_r(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                           int64_t M, int p, int q, hipStream_t s) {
    constexpr int lds_bytes = Ch2Lds<R>::bytes;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&chain2_bf16_kernel<R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(chain2_bf16_kernel<R>, dim3((unsigned)ceil_div(M, 64)), dim3(512), lds_bytes, s,
                       (const uint16_t*)Xin, (const uint16_t*)P, (const uint16_t*)Q,
                       (uint16_t*)Yout, (uint16_t*)Tout, M, p, q);
    return hipGetLastError();
}

}  // namespace

bool chain2_supports(int R, int p) {
    switch (R) {
        case 32: case 96: return p % 128 == 0;
        case 64: case 128: case 192: case 256: case 384: return p % 64 == 0;
        default: return false;
    }
}

hipError_t launch_chain2_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                              int64_t M, int p, int q, int R, hipStream_t s) {
    switch (R) {
        case 32: return launch_chain2_r<32>(Xin, P, Q, Yout, Tout, M, p, q, s);
        case 64: return launch_chain2_r<64>(Xin, P, Q, Yout, Tout, M, p, q, s);
        case 96: return launch_chain2_r<96>(Xin, P, Q, Yout, Tout, M, p, q, s);
        case 128: return launch_chain2_r<128>(Xin, P, Q, Yout, Tout, M, p, q, s);
        case 192: return launch_chain2_r<192>(Xin, P, Q, Yout, Tout, M, p, q, s);
        case 256: return launch_chain2_r<256>(Xin, P, Q, Yout, Tout, M, p, q, s);
        case 384: return launch_chain2_r<384>(Xin, P, Q, Yout, Tout, M, p, q, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace abt
