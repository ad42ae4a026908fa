// Chain kernel, 64-row work-groups:  Tout[M,R] = Xin[M,p] . P[R,p]^T  then  Yout[M,q] = Tout . Q[q,R]^T
// (bf16 in, fp32 accumulate).  Forward of the factored layer with (Xin,P,Q) = (X,B,A); the
// dT/dX half of the backward with (dY, A^T, B^T).
//
// A work-group owns 64 rows and runs 8 waves (two per SIMD).  Every operand slab travels
// global -> LDS with the direct-to-LDS loads of gfx950 (no staging registers), through a ring of
// up to four slabs, so several slabs are in flight while one is consumed.
//
//   stage 1: slabs hold 64 rows of Xin and the R rows of P, BK1 columns of the contraction each.
//            The waves form CS column groups x KS contraction groups; a wave keeps a 64 x (R/CS)
//            block of T^T in accumulators and takes every KS-th k16 step.  The KS partial sums
//            are then added in a fixed tree order through LDS.
//   T:       rounded to bf16 once, written as a 64 x R tile to LDS (and to Tout), from where every
//            wave loads all of it as MFMA operands: T stays in registers for the whole of stage 2.
//   stage 2: a round produces 256 output columns, 32 per wave; slabs hold 256 rows of Q.
//
// LDS slab layout: row-major, 16-byte chunks XOR-swizzled inside each row so that the 16 rows a
// quarter-wave reads for one MFMA operand fall on different banks.  One direct-to-LDS wave
// instruction fills 1 KiB = 64 consecutive chunk slots; lane l supplies slot base + 16 l.
//
// MFMA 32x32x16 bf16 layout (lane l, h = l/32): A operand = 8 values A[l%32][8h..8h+7], B operand
// = B[8h..8h+7][l%32], accumulator v = C[8(v/4) + 4h + v%4][l%32].
#include "common.h"

namespace abt {

namespace {

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

__device__ __forceinline__ bf16x8 as_bf(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ f32x16 mfma16(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(a), as_bf(b), c, 0, 0, 0);
}

// 16 bytes per lane, global -> LDS, asynchronous (counted by vmcnt).  `lds_block` is wave-uniform;
// lane l's data lands at lds_block + 16 l.  Issued from inline assembly on purpose: the compiler
// then does not track the transfer, and the explicit wait_vm() calls below decide how many slabs
// stay in flight (with the builtin it drains every transfer before each barrier).
__device__ __forceinline__ void dma16(const void* g, unsigned char* lds_block) {
    const uint32_t off = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void*)lds_block);
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(off) : "memory");
}

// wait until at most n of this wave's vector-memory operations are outstanding (n wave-uniform)
__device__ __forceinline__ void wait_vm(int n) {
#define ABT_VM(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
    switch (n) {
        ABT_VM(0) ABT_VM(1) ABT_VM(2) ABT_VM(3) ABT_VM(4) ABT_VM(5) ABT_VM(6) ABT_VM(7) ABT_VM(8)
        ABT_VM(9) ABT_VM(10) ABT_VM(11) ABT_VM(12) ABT_VM(13) ABT_VM(14) ABT_VM(15) ABT_VM(16)
        ABT_VM(17) ABT_VM(18) ABT_VM(19) ABT_VM(20) ABT_VM(21) ABT_VM(22) ABT_VM(23) ABT_VM(24)
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
#undef ABT_VM
}

// Work-group barrier for the slab rings: LDS reads/writes of this wave have completed, then
// s_barrier.  No global-memory fence (the ring only carries LDS data), so outstanding transfers of
// later slabs keep flying across it.
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

template <int R>
struct Ch2Lds {
    using C = Ch2<R>;
    static constexpr int CB = R / 32 / C::CS;
    static constexpr int slab1 = (64 + R) * C::BK1 * 2;
    static constexpr int nst1 = (4 * slab1 <= 144 * 1024) ? 4 : ((3 * slab1 <= 144 * 1024) ? 3 : 2);
    static constexpr int slab2 = 256 * C::BK2 * 2;
    static constexpr int nst2 = 4;
    static constexpr int red = (C::KS / 2) * C::CS * CB * 8192;   // first (largest) round of the tree
    static constexpr int tpitch = R * 2 + 16;
    static constexpr int ttile = 64 * tpitch;
    static constexpr int a = nst1 * slab1, b = nst2 * slab2, c = red + ttile;
    static constexpr int bytes = a > b ? (a > c ? a : c) : (b > c ? b : c);
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
    constexpr int NST1 = L::nst1, SLAB1 = L::slab1;
    constexpr int NI1 = (64 + R) * CPR1 / 64;          // wave instructions per stage-1 slab
    constexpr int LPW1 = (NI1 + 7) / 8;                // per wave (the last ones may be idle)
    static_assert(SPW >= 1, "slab must hold one k16 step per contraction group");

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

    // number of loads this wave issues per slab (instruction index = e * 8 + wave)
    int my_loads1 = 0;
#pragma unroll
    for (int e = 0; e < LPW1; ++e) my_loads1 += (e * 8 + wave < NI1) ? 1 : 0;

    auto issue1 = [&](int s) {
        unsigned char* base = lds + (s % NST1) * SLAB1;
        const int k0 = s * BK1;
#pragma unroll
        for (int e = 0; e < LPW1; ++e) {
            const int inst = e * 8 + wave;
            if (inst < NI1) {
                const int li = inst * 64 + lane;
                const int row = li / CPR1, pos = li % CPR1;
                const int c = swz<CPR1>(pos, row);
                const uint16_t* g;
                if (row < 64) {
                    int64_t rr = row0 + row;
                    if (rr >= M) rr = M - 1;
                    g = Xin + rr * p + k0 + c * 8;
                } else {
                    g = Pm + (int64_t)(row - 64) * p + k0 + c * 8;
                }
                dma16(g, base + inst * 1024);
            }
        }
    };

    const int ns1 = p / BK1;
    for (int s = 0; s < NST1 - 1 && s < ns1; ++s) issue1(s);
    for (int s = 0; s < ns1; ++s) {
        // loads of slabs s+1 .. min(ns1-1, s+NST1-2) may stay in flight
        int ahead = ns1 - 1 - s;
        if (ahead > NST1 - 2) ahead = NST1 - 2;
        wait_vm(ahead * my_loads1);
        ring_barrier();
        if (s + NST1 - 1 < ns1) issue1(s + NST1 - 1);
        const unsigned char* base = lds + (s % NST1) * SLAB1;
#pragma unroll
        for (int j = 0; j < SPW; ++j) {
            const int kk = ks * SPW + j;          // k16 step inside the slab
            const int qc = 2 * kk + lh;           // logical chunk of this lane's 8 values
            u32x4 xf[2], pf[CB];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int row = 32 * a + lj;
                xf[a] = *reinterpret_cast<const u32x4*>(base + row * (BK1 * 2) + swz<CPR1>(qc, row) * 16);
            }
#pragma unroll
            for (int b = 0; b < CB; ++b) {
                const int row = 64 + (cs * CB + b) * 32 + lj;
                pf[b] = *reinterpret_cast<const u32x4*>(base + row * (BK1 * 2) + swz<CPR1>(qc, row) * 16);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < CB; ++b) acc1[a][b] = mfma16(pf[b], xf[a], acc1[a][b]);
        }
    }
    __syncthreads();   // every wave is done with the ring; LDS is reused below

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
    __syncthreads();   // T tile consumed; the ring takes over the LDS again

    // ------------------------------------------------------------------ stage 2
    constexpr int BK2 = C::BK2, CPR2 = BK2 / 8, NST2 = L::nst2, SLAB2 = L::slab2;
    constexpr int KSL = R / BK2;                 // slabs per round
    constexpr int LPW2 = 256 * CPR2 / 64 / 8;    // loads per wave per slab
    const int nround = (q + 255) / 256;
    const int ns2 = nround * KSL;

    auto issue2 = [&](int s) {
        unsigned char* base = lds + (s % NST2) * SLAB2;
        const int round = s / KSL, kslab = s % KSL;
#pragma unroll
        for (int e = 0; e < LPW2; ++e) {
            const int inst = e * 8 + wave;
            const int li = inst * 64 + lane;
            const int row = li / CPR2, pos = li % CPR2;
            const int c = swz<CPR2>(pos, row);
            int qr = round * 256 + row;
            if (qr >= q) qr = q - 1;
            dma16(Qm + (int64_t)qr * R + kslab * BK2 + c * 8, base + inst * 1024);
        }
    };

    for (int s = 0; s < NST2 - 1 && s < ns2; ++s) issue2(s);
    f32x16 acc2[2];
    int s = 0;
    for (int round = 0; round < nround; ++round) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc2[a][v] = 0.0f;
#pragma unroll
        for (int kslab = 0; kslab < KSL; ++kslab, ++s) {
            int ahead = ns2 - 1 - s;
            if (ahead > NST2 - 2) ahead = NST2 - 2;
            wait_vm(ahead * LPW2);
            ring_barrier();
            if (s + NST2 - 1 < ns2) issue2(s + NST2 - 1);
            const unsigned char* base = lds + (s % NST2) * SLAB2;
#pragma unroll
            for (int kk = 0; kk < BK2 / 16; ++kk) {
                const int row = 32 * wave + lj;
                const u32x4 qf = *reinterpret_cast<const u32x4*>(
                    base + row * (BK2 * 2) + swz<CPR2>(2 * kk + lh, row) * 16);
                const int kb = kslab * (BK2 / 16) + kk;
                acc2[0] = mfma16(qf, tf[0][kb], acc2[0]);
                acc2[1] = mfma16(qf, tf[1][kb], acc2[1]);
            }
        }
        // lane holds Y[row0 + 32a + lj][256 round + 32 wave + 8g + 4 lh + (0..3)]
        const int col0 = round * 256 + 32 * wave;
        if (col0 < q) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int64_t row = row0 + 32 * a + lj;
                if (row < M) {
                    uint16_t* yrow = Yout + row * q + col0 + 4 * lh;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x2 o = {pack2_bf16(acc2[a][4 * g + 0], acc2[a][4 * g + 1]),
                                   pack2_bf16(acc2[a][4 * g + 2], acc2[a][4 * g + 3])};
                        *reinterpret_cast<u32x2*>(yrow + 8 * g) = o;
                    }
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
