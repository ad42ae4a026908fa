// Chain kernel for wide ranks and large batches (R = 192, 256, 384; 128-row work-groups):
//   Tout[M,R] = Xin[M,p] . P[R,p]^T  then  Yout[M,q] = Tout . Q[q,R]^T      (bf16 in, fp32 accumulate)
// the same contract as the 64-row / 128-row chain kernel with its two roles of waves, for the
// shapes where that one is held back by its loaders: at R = 384 a wave cannot keep 64 rows of T in
// registers next to two other waves on its SIMD, and four loader waves cannot put a factor slab
// into LDS as fast as the MFMA waves use it up.
//
// Here all eight waves of a work-group (two per SIMD, 256 registers each) do the same matrix work:
//   * slabs come in by buffer loads that write straight to LDS (16 bytes per lane, no registers: lane
//     l's data lands at the instruction's LDS base + 16 l, lanes outside the buffer descriptor write
//     zeros): an instruction fills 1 KB of a slab, and the XOR swizzle of the slab layout is applied
//     on the source side (lane l fetches the chunk that belongs at LDS position l).  A wave waits for
//     its own loads before the barrier that ends a slab, which makes the next slab visible to all.
//   * stage 1: slabs of 64 contraction columns (128 rows of Xin, R rows of P); wave (h, c) owns
//     rows 64h.. and columns (R/4)c.. of T in accumulators (R = 192: rows 32h.., columns 96c..).  Waves 0 and 1 load the Xin parts, three
//     slabs ahead (HBM latency) into four slots; waves 2..7 the P parts, one slab ahead into two.
//   * T: rounded to bf16 once, written as a 128 x R tile to LDS (and from there to Tout); every
//     wave then loads 32 rows of it as MFMA operands, which stay in registers for all of stage 2.
//   * stage 2: slabs of 128 rows of Q x 128 contraction columns (64 at R = 192), one slab ahead, every
//     wave loading an eighth; wave (b, c) owns rows 32b.. and columns 64c.. of each 128 x 128 output tile: every Q
//     operand read from LDS feeds one MFMA, every T operand is already in registers.  A finished
//     tile is rounded at once, staged in LDS piece by piece during the next slab (two buffers)
//     and leaves during the slab after that as full 256-byte row segments, four pieces per thread.
//   In both stages a wave keeps several operand reads in flight and holds the last step of a slab
//   back across the barrier, as the MFMA waves of the other chain kernel do.
//
// Measured on the stage-2 loop alone (factor resident in L2): 1.45 thousand cycles per slab against
// 1.02 thousand of MFMA time (1.14 without the loads); the same loop with register-staged loads and
// LDS stores: 1.75.  In the whole kernel a stage-2 tile (three slabs) takes 6.0 thousand cycles and
// a stage-1 slab 2.6 thousand (1.5 of MFMA time): the older wave of each SIMD reaches the barrier
// 800 - 1100 cycles before the younger one.
#include <atomic>

#include "common.h"

namespace abt {

namespace {

__device__ __forceinline__ bf16x8 as_bf3(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ f32x16 mfma3(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf3(a), as_bf3(b), c, 0, 0, 0);
}
// this wave's LDS traffic has completed, then s_barrier (global loads stay in flight)
__device__ __forceinline__ void wg_barrier3() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// this wave's global loads (the direct-to-LDS ones included) and stores have completed
__device__ __forceinline__ void wait_loads3() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
// 1 KB of a slab: lane l's 16 bytes go to LDS address dst + 16 l
__device__ __forceinline__ void dma16(rsrc_t r, unsigned char* dst, int lane_off, int wave_off) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)dst, 16, lane_off, wave_off, 0, 0);
}

constexpr int largest_divisor3(int n, int most) { return most <= 1 ? 1 : (n % most == 0 ? most : largest_divisor3(n, most - 1)); }

template <int R>
struct Ch3Cfg {
    static constexpr int ROWS = 128, NW = 8, NT = 64 * NW;
    static constexpr int BK1 = 64;                            // stage-1 slab: 64 contraction columns, 8 chunks per row
    // stage-1 split of the 128 x R tile of T over the eight waves: two row halves x four column
    // quarters when a quarter is whole 32-column blocks (R a multiple of 128), else four row blocks
    // of 32 x two column halves
    static constexpr int RA = R % 128 == 0 ? 2 : 1;           // 32-row blocks of T per wave
    static constexpr int CG = RA == 2 ? 4 : 2;                // column groups
    static constexpr int CB = R / 32 / CG;                    // 32-column blocks of T per wave
    static constexpr int xpart = ROWS * BK1 * 2;              // Xin part of a stage-1 slab: 16 KB, NXB slots
    static constexpr int ppart = R * BK1 * 2;                 // P part: two slots
    static constexpr int NXB = 4, LX = NXB - 1;               // Xin comes from HBM: its loads run LX slabs ahead
    static constexpr int NXW = 2;                             // waves that load Xin; the other six load P
    static constexpr int NI1X = xpart / 1024 / NXW;           // load instructions per slab of an Xin wave (8)
    static constexpr int NI1P = (R / 8 + NW - NXW - 1) / (NW - NXW);   // of a P wave (at most)
    // stage-2 slab: 128 rows of Q x BK2 contraction columns (128, or 64 where R is not a multiple of 128)
    static constexpr int BK2 = R % 128 == 0 ? 128 : 64, KSL = R / BK2, CPR2 = BK2 / 8;
    static constexpr int slab2 = 128 * BK2 * 2;
    static constexpr int NI2 = slab2 / 1024 / NW;             // load instructions per wave per slab (4 or 2)
    static constexpr int RPI2 = 64 / CPR2;                    // rows of a slab per load instruction (4 or 8)
    static constexpr int NS = BK2 / 16;                       // k16 steps per stage-2 slab
    static constexpr int NB = largest_divisor3(NS, 2);        // operand buffers of a wave in stage 2 (deeper rings measured slower)
    static constexpr int ypitch = 128 * 2 + 16;
    static constexpr int ytile = ROWS * ypitch;
    static constexpr int tpitch = R * 2 + 16;
    static constexpr int ttile = ROWS * tpitch;
    // the T tile sits above the first stage-2 slab slot, so that slab 0 of Q can arrive while T is in use
    static constexpr int a = NXB * xpart + 2 * ppart, b = slab2 + ttile, c = 2 * slab2 + 2 * ytile;
    static constexpr int lds_bytes = a > b ? (a > c ? a : c) : (b > c ? b : c);
    static_assert(R % 64 == 0 && R % BK2 == 0 && KSL >= 2 && NI1X == 8 && (NXB & (NXB - 1)) == 0 && LX <= 3, "slab shape");
    static_assert(CB * CG * 32 == R && (CPR2 == 16 || CPR2 == 8) && NI2 * NW * RPI2 == 128, "wave split");
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    static_assert(NS >= 2 && NS <= 9, "a staged tile leaves in eight pieces spread over the NS - 1 steps of a slab");
};

struct Ch3Ptrs {
    const uint16_t* X[kChainMaxGroups];
    const uint16_t* P[kChainMaxGroups];
    const uint16_t* Q[kChainMaxGroups];
    uint16_t* Y[kChainMaxGroups];
    uint16_t* T[kChainMaxGroups];
};

template <int R>
__global__ __launch_bounds__(512) void chain3_bf16_kernel(Ch3Ptrs ptrs, int64_t M, int p, int q,
                                                          int full_blocks, int tail_parts, int stream_out) {
    extern __shared__ __align__(1024) unsigned char lds[];
    const uint16_t* __restrict__ const Xin = ptrs.X[blockIdx.y];
    const uint16_t* __restrict__ const Pm = ptrs.P[blockIdx.y];
    const uint16_t* __restrict__ const Qm = ptrs.Q[blockIdx.y];
    uint16_t* __restrict__ const Yout = ptrs.Y[blockIdx.y];
    uint16_t* __restrict__ const Tout = ptrs.T[blockIdx.y];
    if (Yout == nullptr && Tout == nullptr) return;      // nothing asked of this group
    using L = Ch3Cfg<R>;
    constexpr int ROWS = L::ROWS, BK1 = L::BK1, CB = L::CB, BK2 = L::BK2, KSL = L::KSL, NS = L::NS, NB = L::NB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lj = lane & 31, lh = lane >> 5;
    // Work-groups [0, full_blocks) take one row block each and all of its output tiles; the row
    // blocks after those are shared by tail_parts work-groups each, every one repeating stage 1 and
    // doing its share of the stage-2 tiles.
    int rb = (int)blockIdx.x, part = 0, nparts = 1;
    if (rb >= full_blocks) {
        const int t = rb - full_blocks;
        rb = full_blocks + t / tail_parts;
        part = t % tail_parts;
        nparts = tail_parts;
    }
    const int64_t row0 = (int64_t)rb * ROWS;
    const int64_t rows_valid = M - row0 < ROWS ? M - row0 : ROWS;
    const int ns1 = p / BK1;
    const int ntile_all = (q + 127) / 128;
    const int tile0 = (int)((unsigned)part * (unsigned)ntile_all / (unsigned)nparts);
    const int ntile = (int)((unsigned)(part + 1) * (unsigned)ntile_all / (unsigned)nparts) - tile0;
    const int ns2 = ntile * KSL;
    // work-groups start their walks over the slabs and the tiles at different points
    const int rot1 = (int)((unsigned)rb % (unsigned)ns1);
    const int rot2 = (int)((unsigned)rb % (unsigned)ntile);
    auto slab1_of = [&](int s) { s += rot1; return s >= ns1 ? s - ns1 : s; };
    auto tile_of = [&](int t) { t += rot2; return tile0 + (t >= ntile ? t - ntile : t); };

    unsigned char* const ttile = lds + L::slab2;
    unsigned char* const ytile = lds + 2 * L::slab2;

    // ------------------------------------------------------------------ who loads what
    // Stage 1: a load instruction covers 8 rows of 8 chunks (rows 8 i + lane / 8 for instruction i).  Waves
    // 0 and 1 load the Xin part (instructions wave, wave + 2, ...), LX slabs ahead: it comes from HBM, and
    // a wave's loads complete in issue order, so "at most 8 n outstanding" tells an Xin wave that all but
    // its newest n slabs have landed.  Waves 2..7 load the P part (instructions wave - 2, wave + 4, ...),
    // one slab ahead, from L2.  The chunk at LDS position c of row r is logical chunk c ^ ((r >> 1) & 7);
    // all instructions of a wave have its parity, which leaves that XOR the same for all of them.
    // The row offset of Xin is part of the per-lane offset, the only part that the hardware
    // range-checks: rows past M arrive as zeros.
    const rsrc_t xres = make_rsrc(Xin + row0 * p, rows_valid * p * 2);
    const rsrc_t pres = make_rsrc(Pm, (int64_t)R * p * 2);
    const bool xwave = wave < L::NXW;
    const int r8 = lane >> 3;
    const int i0 = xwave ? wave : wave - L::NXW;        // first instruction of this wave
    const int chunk1 = (lane & 7) ^ ((4 * (i0 & 1) + (r8 >> 1)) & 7);
    const int v1 = ((8 * i0 + r8) * p + chunk1 * 8) * 2;
    auto issue1x = [&](int s) {
        unsigned char* dst = lds + (s & (L::NXB - 1)) * L::xpart + i0 * 1024;
        const int so = slab1_of(s) * (BK1 * 2);
#pragma unroll
        for (int j = 0; j < L::NI1X; ++j) dma16(xres, dst + j * (L::NXW * 1024), v1 + j * (8 * L::NXW) * p * 2, so);
    };
    auto issue1p = [&](int s) {
        unsigned char* dst = lds + L::NXB * L::xpart + (s & 1) * L::ppart + i0 * 1024;
        const int so = slab1_of(s) * (BK1 * 2);
        constexpr int NPW = L::NW - L::NXW;
#pragma unroll
        for (int j = 0; j < L::NI1P; ++j)
            if (i0 + j * NPW < R / 8) dma16(pres, dst + j * (NPW * 1024), v1, so + j * (8 * NPW) * p * 2);
    };
    // an Xin wave: all but its newest n slabs have landed; a P wave: all its loads have landed
    auto wait1 = [&](int n) {
        if (!xwave || n <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (n == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    };
    // Stage 2: an instruction covers RPI2 rows of CPR2 chunks: rows RPI2 (wave + 8u) + lane / CPR2; logical
    // chunk c ^ (r & 15) for 16-chunk rows, c ^ ((r >> 1) & 7) for 8-chunk rows (the same for all
    // instructions of a wave).  The descriptor covers the rows of the tile that exist: the rest
    // arrive as zeros and feed output columns that are never stored.
    const int r4 = lane / L::CPR2;
    const int row2 = L::RPI2 * wave + r4;
    const int chunk2 = (lane % L::CPR2) ^ (L::CPR2 == 16 ? (row2 & 15) : ((row2 >> 1) & 7));
    const int v2 = (row2 * R + chunk2 * 8) * 2;
    auto issue2 = [&](int s) {
        const int t = tile_of(s / KSL);
        const int rows = q - t * 128 < 128 ? q - t * 128 : 128;
        const rsrc_t qres = make_rsrc(Qm + (int64_t)t * 128 * R, (int64_t)rows * R * 2);
        unsigned char* dst = lds + (s & 1) * L::slab2 + wave * 1024;
        const int so = (s % KSL) * (BK2 * 2);
#pragma unroll
        for (int u = 0; u < L::NI2; ++u) dma16(qres, dst + u * 8192, v2 + u * (8 * L::RPI2) * R * 2, so);
    };

    // ------------------------------------------------------------------ stage 1
    constexpr int RA = L::RA;
    const int rg = RA == 2 ? wave >> 2 : wave >> 1;     // rows 32 RA rg ..
    const int cq = RA == 2 ? wave & 3 : wave & 1;       // columns 32 CB cq ..
    f32x16 acc1[RA][CB];
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc1[a][b][v] = 0.0f;
    struct Ops1 { u32x4 xf[RA]; u32x4 pf[CB]; };
    constexpr int SPW = BK1 / 16;                       // 4 steps per slab
    constexpr int NB1 = 2;                              // operand buffers (divides SPW: the held step sits in the last one)
    Ops1 ob[NB1];
    auto read1 = [&](Ops1& o, int s, int kk) {
        const unsigned char* xb = lds + (s & (L::NXB - 1)) * L::xpart;
        const unsigned char* pb = lds + L::NXB * L::xpart + (s & 1) * L::ppart;
        const int qc = 2 * kk + lh;                     // logical chunk of this lane's 8 values
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            const int row = 32 * (RA * rg + a) + lj;
            o.xf[a] = *reinterpret_cast<const u32x4*>(xb + row * (BK1 * 2) + ((qc ^ ((row >> 1) & 7)) * 16));
        }
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            const int row = (cq * CB + b) * 32 + lj;
            o.pf[b] = *reinterpret_cast<const u32x4*>(pb + row * (BK1 * 2) + ((qc ^ ((row >> 1) & 7)) * 16));
        }
    };
    auto mma1 = [&](const Ops1& o) {
#pragma unroll
        for (int a = 0; a < RA; ++a)
#pragma unroll
            for (int b = 0; b < CB; ++b) acc1[a][b] = mfma3(o.pf[b], o.xf[a], acc1[a][b]);
    };
    if (xwave) {
#pragma unroll
        for (int d = 0; d < L::LX; ++d)
            if (d < ns1) issue1x(d);
    } else {
        issue1p(0);
    }
    wait1((ns1 < L::LX ? ns1 : L::LX) - 1);
    wg_barrier3();                                      // slab 0 is in its slots
    for (int s = 0; s < ns1; ++s) {
        // into the slots whose reads ended before the last barrier.  The P loads go first and the Xin
        // loads one step later: loads come back in the order the compute unit asked for them, so a P slab
        // (from L2, needed for the next slab) must not queue behind the Xin slab of the same round (from
        // HBM, needed three slabs on); the Xin slab asked for a whole slab earlier is the last thing before it
        if (!xwave && s + 1 < ns1) issue1p(s + 1);
#pragma unroll
        for (int j = 0; j + 1 < NB1; ++j) read1(ob[j], s, j);
        __builtin_amdgcn_sched_barrier(0);
        if (s > 0) mma1(ob[NB1 - 1]);                   // last step of the slab before
        __builtin_amdgcn_sched_barrier(0);
        read1(ob[NB1 - 1], s, NB1 - 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j + 1 < SPW; ++j) {
            mma1(ob[j % NB1]);
            __builtin_amdgcn_sched_barrier(0);
            if (j + NB1 < SPW) read1(ob[j % NB1], s, j + NB1);
            if (j == 0 && xwave && s + L::LX < ns1) issue1x(s + L::LX);
            __builtin_amdgcn_sched_barrier(0);
        }
        // slab s + 1 must have landed; the newest Xin slab issued is min(s + LX, ns1 - 1)
        wait1((s + L::LX < ns1 ? s + L::LX : ns1 - 1) - (s + 1));
        wg_barrier3();
    }
    mma1(ob[NB1 - 1]);
    // ------------------------------------------------------------------ T tile (bf16) to LDS
    // lane holds T[32 (RA rg + a) + lj][32 (cq CB + b) + 8g + 4 lh + (0..3)] in acc1[a][b][4g .. 4g+3]
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 o = {pack2_bf16(acc1[a][b][4 * g + 0], acc1[a][b][4 * g + 1]),
                           pack2_bf16(acc1[a][b][4 * g + 2], acc1[a][b][4 * g + 3])};
                *reinterpret_cast<u32x2*>(ttile + (32 * (RA * rg + a) + lj) * L::tpitch +
                                          (32 * (cq * CB + b) + 8 * g + 4 * lh) * 2) = o;
            }
    if (Yout != nullptr) issue2(0);                     // slot 0 lies below the T tile
    wg_barrier3();                                      // T tile complete
    if (Tout != nullptr && part == 0) {
        const rsrc_t tres = make_rsrc(Tout + row0 * R, rows_valid * R * 2);
        constexpr int CPT = R / 8;                      // 16-byte chunks per T row
        for (int i = tid; i < ROWS * CPT; i += L::NT) {
            const int row = i / CPT, ch = i % CPT;
            buf_store16_maybe_stream(stream_out != 0, *reinterpret_cast<const u32x4*>(ttile + row * L::tpitch + ch * 16), tres, (row * R + ch * 8) * 2, 0);
        }
    }
    if (Yout == nullptr) return;

    // ------------------------------------------------------------------ stage 2
    const int trow0 = 32 * (wave >> 1), qrow0 = 64 * (wave & 1);
    constexpr int KB = R / 16;
    u32x4 tf[KB];                                       // T[trow0 + lj][16kb + 8 lh .. +7]
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
        tf[kb] = *reinterpret_cast<const u32x4*>(ttile + (trow0 + lj) * L::tpitch + (16 * kb + 8 * lh) * 2);
    const rsrc_t yres = make_rsrc(Yout + row0 * q, rows_valid * q * 2);
    wait_loads3();
    wg_barrier3();                                      // T tile consumed; Q slab 0 is in slot 0
    // address of step kk = address of step 0 with kk << 5 XORed in (chunk 2 kk + lh of 16 or 8 per row)
    const int qsw = L::CPR2 == 16 ? ((qrow0 + lj) & 15) : (((qrow0 + lj) >> 1) & 7);
    const int qaddr0 = (qrow0 + lj) * (BK2 * 2) + ((lh ^ qsw) * 16);
    struct Ops2 { u32x4 qf[2]; };
    auto read2 = [&](Ops2& dst, int s, int kk) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
            dst.qf[b] = *reinterpret_cast<const u32x4*>(lds + (s & 1) * L::slab2 + (qaddr0 ^ (kk << 5)) + b * 32 * (BK2 * 2));
    };
    f32x16 acc2[2];
    Ops2 ring[NB];
    auto mma2 = [&](const Ops2& o, int kb) {
        acc2[0] = mfma3(o.qf[0], tf[kb], acc2[0]);
        acc2[1] = mfma3(o.qf[1], tf[kb], acc2[1]);
    };
    // first step of a tile: the accumulators start from a zero operand instead of being cleared
    auto mma2_first = [&](const Ops2& o, int kb) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        acc2[0] = mfma3(o.qf[0], tf[kb], zero);
        acc2[1] = mfma3(o.qf[1], tf[kb], zero);
    };
    // A finished tile is rounded to bf16 right away (16 registers) and written to its staging buffer
    // piece by piece between the steps of the slab that follows, instead of all at once while the
    // matrix cores of this wave's SIMD wait: lane holds Y[trow0 + lj][qrow0 + 32b + 8g + 4 lh + (0..3)].
    u32x2 packed[2][4];
    auto pack_out = [&]() {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                packed[b][g] = u32x2{pack2_bf16(acc2[b][4 * g + 0], acc2[b][4 * g + 1]),
                                     pack2_bf16(acc2[b][4 * g + 2], acc2[b][4 * g + 3])};
    };
    auto stage_piece = [&](int t, int i) {
        const int b = i >> 2, g = i & 3;
        unsigned char* yt = ytile + (t & 1) * L::ytile;
        *reinterpret_cast<u32x2*>(yt + (trow0 + lj) * L::ypitch + (qrow0 + 32 * b + 8 * g + 4 * lh) * 2) = packed[b][g];
    };
    // a staged tile leaves as 2048 pieces of 16 bytes, four per thread: piece i = row i / 16, chunk i % 16
    u32x4 piece[4];
    auto flush_read = [&](int seq) {
        const unsigned char* yt = ytile + (seq & 1) * L::ytile;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = e * L::NT + tid;
            piece[e] = *reinterpret_cast<const u32x4*>(yt + (i >> 4) * L::ypitch + (i & 15) * 16);
        }
    };
    auto flush_store = [&](int seq) {
        const int t = tile_of(seq);
        const bool whole = q - t * 128 >= 128;          // else the tile has 64 columns (q is a multiple of 64)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = e * L::NT + tid;
            // pieces past a ragged tile go nowhere
            buf_store16_maybe_stream(stream_out != 0, piece[e], yres, whole || (i & 15) < 8 ? ((i >> 4) * q + (i & 15) * 8) * 2 : kBufNowhere, t * 256);
        }
    };
    int flushed = 0;
    for (int s0 = 0; s0 < ns2; s0 += KSL) {
        const int t = s0 / KSL;
#pragma unroll
        for (int kp = 0; kp < KSL; ++kp) {
            const int s = s0 + kp;
            if (s + 1 < ns2) issue2(s + 1);
            // tile f was staged during slab (f + 1) KSL, which ended with a barrier: it leaves during the
            // slab after that, read from LDS first and stored after the first steps
            const bool flush_now = s > KSL && (s - 1) % KSL == 0;
            if (flush_now) flush_read(flushed);
#pragma unroll
            for (int i = 0; i + 1 < NB; ++i) read2(ring[i], s, i);
            __builtin_amdgcn_sched_barrier(0);
            const bool stage_now = s > 0 && kp == 0;    // the tile before this one is complete after the held step
            if (s > 0) {
                // last step of the slab before this one
                mma2(ring[NB - 1], ((kp + KSL - 1) % KSL) * NS + NS - 1);
                if (kp == 0) pack_out();
            }
            __builtin_amdgcn_sched_barrier(0);
            read2(ring[NB - 1], s, NB - 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk + 1 < NS; ++kk) {
                if (kp == 0 && kk == 0) mma2_first(ring[0], 0);
                else mma2(ring[kk % NB], kp * NS + kk);
                __builtin_amdgcn_sched_barrier(0);
                if (kk + NB < NS) read2(ring[kk % NB], s, kk + NB);
                if (stage_now) {
#pragma unroll
                    for (int i = kk * 8 / (NS - 1); i < (kk + 1) * 8 / (NS - 1); ++i) stage_piece(t - 1, i);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // the next slab has landed.  The stores of a flush go out only now: loads and stores need not
            // complete in one common order, so no count of outstanding operations is used to tell the
            // slab's loads from stores issued before this wait; issued after it, the stores are on
            // their way during the next slab and complete long before its closing wait
            wait_loads3();
            if (flush_now) {
                flush_store(flushed);
                ++flushed;
            }
            wg_barrier3();
        }
    }
    mma2(ring[NB - 1], (KSL - 1) * NS + NS - 1);
    pack_out();
#pragma unroll
    for (int i = 0; i < 8; ++i) stage_piece(ntile - 1, i);
    wg_barrier3();                                      // the last tile is staged
    for (; flushed < ntile; ++flushed) {                // the last tile
        flush_read(flushed);
        flush_store(flushed);
    }
}

template <int R>
hipError_t launch_chain3_r(const Ch3Ptrs& ptrs, int G, bool second_stage, int64_t M, int p, int q, int parts, hipStream_t s) {
    using L = Ch3Cfg<R>;
    if (G < 1 || G > kChainMaxGroups || parts < 1 || parts > 64 || (second_stage && parts > (q + 127) / 128) ||
        (!second_stage && parts != 1))
        return hipErrorInvalidValue;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&chain3_bf16_kernel<R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, L::lds_bytes);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int64_t nblocks = ceil_div(M, L::ROWS);
    int64_t full = 0;
    int tail_parts = parts;
    if (parts == 1) {
        // the row blocks of a partly filled last round of the 256 compute units are shared by output
        // tiles when that round is at most half full and stage 2 is the larger part of the work
        full = nblocks;
        const int64_t tail = nblocks % 256;
        const int ntile = (q + 127) / 128;
        if (G == 1 && second_stage && nblocks > 256 && tail > 0 && 2 * tail <= 256) {
            int tp = (int)(256 / tail);
            if (tp > ntile) tp = ntile;
            // in units of stage-2 slabs: a stage-1 slab has 1.5 times the MFMA work
            const int ns1 = 3 * (p / L::BK1) / 2, whole = ns1 + ntile * L::KSL, shared = ns1 + (ntile + tp - 1) / tp * L::KSL;
            if (tp >= 2 && 10 * shared <= 7 * whole) {
                full = nblocks - tail;
                tail_parts = tp;
            }
        }
    }
    const int64_t grid = full + (nblocks - full) * tail_parts;
    hipLaunchKernelGGL((chain3_bf16_kernel<R>), dim3((unsigned)grid, (unsigned)G), dim3(L::NT), L::lds_bytes, s,
                       ptrs, M, p, q, (int)full, tail_parts, (int)(M * ((second_stage ? q : 0) + R) * 2 >= kStreamOutBytes));
    return hipGetLastError();
}

}  // namespace

bool chain3_supports(int R, int p, int q) {
    if (p % 64 != 0 || p < 64 || q < 64 || q % 64 != 0 || p > (1 << 20) || q > (1 << 20)) return false;
#ifdef ABT_NO_CHAIN3_384
    return R == 192 || R == 256;
#else
    return R == 192 || R == 256 || R == 384;
#endif
}

hipError_t launch_chain3_bf16(const ChainProblem* problems, int G, int64_t M, int p, int q, int R, int parts, hipStream_t s) {
    if (G < 1 || G > kChainMaxGroups || !problems || M < 1 || !chain3_supports(R, p, q)) return hipErrorInvalidValue;
    Ch3Ptrs t{};
    bool second_stage = false, first_stage_only = false;
    for (int g = 0; g < G; ++g) {
        t.X[g] = (const uint16_t*)problems[g].Xin; t.P[g] = (const uint16_t*)problems[g].P; t.Q[g] = (const uint16_t*)problems[g].Q;
        t.Y[g] = (uint16_t*)problems[g].Yout; t.T[g] = (uint16_t*)problems[g].Tout;
        if (t.Y[g]) second_stage = true;
        else if (t.T[g]) first_stage_only = true;
    }
    if (second_stage && first_stage_only) return hipErrorInvalidValue;
    switch (R) {
        case 192: return launch_chain3_r<192>(t, G, second_stage, M, p, q, parts, s);
        case 256: return launch_chain3_r<256>(t, G, second_stage, M, p, q, parts, s);
        case 384: return launch_chain3_r<384>(t, G, second_stage, M, p, q, parts, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace abt
