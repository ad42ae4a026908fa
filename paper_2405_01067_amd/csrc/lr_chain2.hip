// Chain kernel, 64-row work-groups (RG = 1) and 128-row work-groups (RG = 2):  Tout[M,R] = Xin[M,p] . P[R,p]^T  then  Yout[M,q] = Tout . Q[q,R]^T
// (bf16 in, fp32 accumulate).  Forward of the factored layer with (Xin,P,Q) = (X,B,A); the
// dT/dX half of the backward with (dY, A^T, B^T).
//
// A work-group owns 64 rows and runs 8 waves, two per SIMD, in two roles:
//   4 MFMA waves do all the matrix work: a wave owns all 64 rows (two MFMA row blocks), so every
//     factor operand it reads from LDS feeds two MFMAs and no operand is read by two waves;
//   4 loader waves issue every global load: whole slabs (activation and factor parts alike) go
//     through a ring of register sets, several slabs deep and consumed strictly in issue order,
//     so the in-order vector-memory counter tells a loader exactly when the oldest slab has
//     landed.  They also store T and write the finished output tiles.
//     The depth matters more than who loads: a CU needs roughly 64 KB of loads in flight at all
//     times to draw its ~50 B/clk from L2 (latency under load is about a thousand cycles); with
//     slabs fetched only one ahead the loop time was pinned to that latency.
// The waves meet at one s_barrier per slab; LDS holds two slab slots.
//
//   stage 1: slabs of 64 contraction columns: 64 rows of Xin and the R rows of P.  The MFMA waves
//            form RS row groups x CS column groups x KS contraction groups; a wave keeps its block
//            of T^T in accumulators and takes every KS-th k16 step.  The KS partial sums are then
//            added in a fixed tree order through LDS.
//   T:       rounded to bf16 once, written as a 64 x R tile to LDS (and from there to Tout); every
//            MFMA wave loads all of it as MFMA operands: T stays in registers for all of stage 2.
//   stage 2: a slab is 128 rows of Q (all R columns while that fits, else half) and yields a
//            64 x 128 output tile, 32 columns per MFMA wave; the tile is staged in LDS (two
//            buffers) and leaves two slabs later as full 256-byte row segments.
//   In both stages an MFMA wave keeps several operand reads in flight ahead of the MFMAs that use
//   them and holds the last step of a slab back across the barrier (a lone MFMA wave per SIMD has
//   nobody to hide its LDS latency behind: with reads issued step by step the loop time was about
//   three times the MFMA time).
// (The direct-to-LDS loads of gfx950 give one wave no more than register-staged loads do and are
// not used here; the kernel of eight equal waves in lr_chain3.hip is built on them.)
//
// LDS slab layout: row-major, 16-byte chunks XOR-swizzled inside each row so that the 16 rows a
// quarter-wave reads for one MFMA operand fall on different banks.
//
// MFMA 32x32x16 bf16 layout (lane l, h = l/32): A operand = 8 values A[l%32][8h..8h+7], B operand
// = B[8h..8h+7][l%32], accumulator v = C[8(v/4) + 4h + v%4][l%32].
//
// RG = 2, for large batches.  A 64-row work-group streams both factors through LDS for its 64 rows; a grid of them that needs
// several rounds on the 256 compute units leaves a partial last round.  Here a work-group owns 128
// rows as two row groups of 64: eight MFMA waves, four per row group, each group working exactly as
// the four MFMA waves of the 64-row kernel do, on its own rows of the Xin part of a slab, its own
// reduction scratch, T tile and output staging tiles, while both groups read the same P and Q slabs
// that four loader waves bring in once.  Measured: such a work-group takes 1.58 times as long as a
// 64-row one on the same factors (the slab is stored once but read by both groups, and twice the
// output is staged: LDS traffic per output tile goes from 128 KB to 208 KB at the same ~77 B/clk),
// so a compute unit gets through rows 1.27 times as fast, and a grid of half as many work-groups
// often needs fewer rounds.  Twelve waves leave 168 registers per lane, so the register rings are
// shallower and a stage-2 slab holds at most 96 contraction columns (two slabs per output tile for
// R = 192), which also keeps four staging tiles plus two slab slots inside the 160 KB of LDS.
// At R = 384 a wave cannot hold 64 rows of T (192 registers): stage 2 is then split by rows, a wave
// owning 32 rows of T and two 32-column blocks of the output tile (every Q operand read from LDS
// feeds one MFMA instead of two).
#include <atomic>
#include <type_traits>

#include "common.h"

namespace abt {

namespace {

__device__ __forceinline__ bf16x8 as_bf(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ f32x16 mfma16(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf(a), as_bf(b), c, 0, 0, 0);
}

// The only barrier used in this kernel (both roles execute the same sequence of them): this wave's
// LDS traffic has completed, then s_barrier.  Deliberately not __syncthreads(): that also drains
// outstanding global loads, which are exactly the prefetches that must stay in flight.
__device__ __forceinline__ void wg_barrier() {
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

// Work split of the four MFMA waves in stage 1: RS row groups x CS column groups x KS contraction
// groups (product 4).  Splitting the rows (RS = 2) would need no partial sums, but every wave then
// reads more operands from LDS per MFMA, and LDS bandwidth (shared with the loaders' stores) is
// what limits stage 1: measured slower than contraction groups plus a tree reduction.
template <int R> struct Ch2;
template <> struct Ch2<32>  { static constexpr int RS = 1, CS = 1, KS = 4; };
template <> struct Ch2<64>  { static constexpr int RS = 1, CS = 1, KS = 4; };
template <> struct Ch2<96>  { static constexpr int RS = 1, CS = 1, KS = 4; };
template <> struct Ch2<128> { static constexpr int RS = 1, CS = 2, KS = 2; };
template <> struct Ch2<160> { static constexpr int RS = 1, CS = 1, KS = 4; };
template <> struct Ch2<192> { static constexpr int RS = 1, CS = 2, KS = 2; };
template <> struct Ch2<256> { static constexpr int RS = 1, CS = 2, KS = 2; };
template <> struct Ch2<320> { static constexpr int RS = 1, CS = 2, KS = 2; };
template <> struct Ch2<384> { static constexpr int RS = 1, CS = 4, KS = 1; };

constexpr int NLW = 4;                          // loader waves
constexpr int NMW_ = 4;                         // MFMA waves per row group (RG row groups of 64 rows)
constexpr int NLT = 64 * NLW;                   // loader threads
constexpr int BK1 = 64, CPR1 = BK1 / 8;         // stage-1 slab: 64 contraction columns
constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }
constexpr int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }
constexpr int gcdi(int a, int b) { return b == 0 ? a : gcdi(b, a % b); }
constexpr int largest_divisor(int n, int most) { return most <= 1 ? 1 : (n % most == 0 ? most : largest_divisor(n, most - 1)); }

template <int R, int RG>
struct Ch2Cfg {
    using C = Ch2<R>;
    static constexpr int ROWS = 64 * RG;                      // rows per work-group
    static constexpr int CB = R / 32 / C::CS;                 // column blocks per wave
    static constexpr int RA = 2 / C::RS;                      // row blocks per wave
    static constexpr int SPW = BK1 / (16 * C::KS);            // k16 steps per wave per slab
    static constexpr int xpart = ROWS * BK1 * 2;              // slot = [ROWS rows of Xin][R rows of P]
    static constexpr int slab1 = (ROWS + R) * BK1 * 2;
    static constexpr int NCHX = ROWS * CPR1 / NLT;            // 16-byte chunks per loader thread (Xin part) = 2 RG
    static constexpr int NCHP = R * CPR1 / NLT;               // chunks per loader thread (P part) = R / 32
    // slabs in flight (register ring depth): twelve waves (RG = 2) leave 168 registers per lane
    static constexpr int D1 = RG == 1 ? clampi(32 / (NCHX + NCHP), 2, 6) : clampi(30 / (NCHX + NCHP), 2, 4);
    // stage 2: a slab is 128 rows of Q times BK2 = R / KSL columns
    // RG = 2: at most 96 contraction columns per slab beyond R = 128 (LDS: four staging tiles)
    static constexpr int KSL = RG == 1 ? (R <= 224 ? 1 : 2) : (R <= 128 ? 1 : (R <= 192 ? R / 96 : 4));
    // RG = 2 beyond R = 192: a wave cannot hold 64 rows of T (R / 2 registers of 168).  Each wave then
    // owns 32 rows of T and two column blocks of the output tile instead of 64 rows and one block.
    static constexpr bool RSPLIT = RG == 2 && R > 192;
    static constexpr int BK2 = R / KSL, CPR2 = BK2 / 8;
    static constexpr int slab2 = 128 * BK2 * 2;
    static constexpr int NCHQ = 128 * CPR2 / NLT;             // chunks per loader thread = BK2 / 16
    static constexpr int D2 = RG == 1 ? clampi(36 / NCHQ, 2, 6) : clampi(20 / NCHQ, 2, 4);   // stage-2 slabs in flight
    static constexpr int U2 = D2 * KSL / gcdi(D2, KSL);       // stage-2 trip count is padded to a multiple of this
    // operand buffers of an MFMA wave in stage 2 (registers: T takes R / 2 of them, twelve waves leave 168)
    static constexpr int NB2 = RG == 1 ? (R > 320 ? 2 : 6) : (RSPLIT ? 3 : (R > 128 ? 3 : 6));
    static constexpr int ypitch = 128 * 2 + 16;
    static constexpr int ytile = 64 * ypitch;
    static constexpr int red = (C::KS / 2) * C::CS * C::RS * RA * CB * 4096;   // first (largest) round of the tree
    static constexpr int tpitch = R * 2 + 16;
    static constexpr int ttile = 64 * tpitch;
    static constexpr int a = 2 * slab1, b = RG * (red + ttile), c = 2 * slab2 + RG * 2 * ytile;   // per row group: red, ttile, two ytiles
    static constexpr int lds_bytes = a > b ? (a > c ? a : c) : (b > c ? b : c);
    static constexpr int n_mid_barriers = C::KS > 1 ? 2 * ilog2(C::KS) : 1;  // tree + T tile written
    static_assert(SPW >= 1 && NCHX == 2 * RG && R % 32 == 0 && BK2 % 16 == 0 && R % KSL == 0, "slab shape");
    static_assert(C::RS * C::CS * C::KS == NMW_ && CB * C::CS * 32 == R && RA * C::RS == 2, "wave split");
};

// Gather form of the Xin operand (GATHER = true): Xin is not a matrix but a channels-last image
// [images, H, W, Cin], and row i of the virtual matrix is the patch around a pixel of it: virtual
// column (tap, block, c) with tap = ky kw + kx, `cpb` 64-column blocks per tap, reads channel
// 64 block + c of the pixel `sign (ky - kh/2, kx - kw/2)` away from the row's centre, zero outside the
// image and for channels >= Cin.  A slab of 64 contraction columns is then one tap and one channel
// block: 128 contiguous bytes per row, as in the plain case.  p = kh kw cpb 64.
// Rows are the pixels of a grid RH x RW per image, row-major; the centre of row (y, x) is the image
// pixel (mul y, mul x), and with shift > 0 the shifted position (ty, tx) only exists in the image
// where both are multiples of 2^shift, as pixel (ty >> shift, tx >> shift):
//   stride 1:                     RH x RW = H x W, mul = 1, shift = 0
//   strided patches (forward):    RH x RW = the output grid, mul = stride, shift = 0
//   their adjoint (image = the gradient on the output grid, rows = input pixels): mul = 1, shift = log2 stride.
struct Ch2Gather { int H, W, Cin, cpb, kh, kw, sign, RH, RW, mul, shift; };

// Source pixel (linear, over all images) at the centre of the first (end = 0) or last (end = 1)
// pixel of the grid row that row i lies in.  The centre is monotone in (image, y) and in x, so the
// centres of rows i0 .. i1 lie between ch2_centre(i0, 0) and ch2_centre(i1, 1).
__device__ __forceinline__ int ch2_centre(const Ch2Gather& gg, int i, int end) {
    const int per = gg.RH * gg.RW;
    const int img = i / per, rem = i - img * per;
    const int y = rem / gg.RW, x = end ? gg.RW - 1 : 0;
    return (img * gg.H + ((gg.mul * y) >> gg.shift)) * gg.W + ((gg.mul * x) >> gg.shift);
}

// Operands of up to kChainMaxGroups problems of one shape (the emulated groups of a training step:
// same M, p, q, R, each with its own activations and its own copy of the factors); blockIdx.y picks one.
struct Ch2Ptrs {
    const uint16_t* X[kChainMaxGroups];
    const uint16_t* P[kChainMaxGroups];
    const uint16_t* Q[kChainMaxGroups];
    uint16_t* Y[kChainMaxGroups];
    uint16_t* T[kChainMaxGroups];
};

template <int R, int RG, bool GATHER>
__global__ __launch_bounds__(64 * (NMW_ * RG + NLW)) void chain2_bf16_kernel(Ch2Ptrs ptrs,
                                                         int64_t M, int p, int q, int t_pitch, Ch2Gather gg,
                                                         int full_blocks, int tail_parts, int stream_out) {
    extern __shared__ __align__(1024) unsigned char lds[];
    const uint16_t* __restrict__ const Xin = ptrs.X[blockIdx.y];
    const uint16_t* __restrict__ const Pm = ptrs.P[blockIdx.y];
    const uint16_t* __restrict__ const Qm = ptrs.Q[blockIdx.y];
    uint16_t* __restrict__ const Yout = ptrs.Y[blockIdx.y];
    uint16_t* __restrict__ const Tout = ptrs.T[blockIdx.y];
    if (Yout == nullptr && Tout == nullptr) return;      // nothing asked of this group
    using C = Ch2<R>;
    using L = Ch2Cfg<R, RG>;
    constexpr int ROWS = L::ROWS, NMW = NMW_ * RG, NMT = 64 * NMW;
#define ABT_LOADER_WAVE (NMW_ * RG)
    constexpr int RS = C::RS, CS = C::CS, KS = C::KS, CB = L::CB, RA = L::RA, SPW = L::SPW;
    constexpr int BK2 = L::BK2, CPR2 = L::CPR2, KSL = L::KSL;
    constexpr int D1 = L::D1, D2 = L::D2;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Work-groups [0, full_blocks) take one row block each and all of its output tiles; the row
    // blocks after those are shared by tail_parts work-groups each, every one repeating stage 1 and
    // doing its share of the stage-2 tiles (for a batch too small to fill the chip, and for the
    // last, partly filled round of a large one).
    int rb = (int)blockIdx.x, part = 0, nparts = 1;
    if (rb >= full_blocks) {
        const int t = rb - full_blocks;
        rb = full_blocks + t / tail_parts;
        part = t % tail_parts;
        nparts = tail_parts;
    }
    const int64_t row0 = (int64_t)rb * ROWS;
    const int ns1 = p / BK1;
    const int n1p = (ns1 + D1 - 1) / D1 * D1;           // stage-1 trip count, padded to the loaders' ring
    // stage-2 output tiles of 128 columns: part `part` of `nparts` does the tiles
    // [tile0, tile0 + ntile) of the ntile_all; every part repeats stage 1 for its rows
    const int ntile_all = (q + 127) / 128;
    const int tile0 = (int)((unsigned)part * (unsigned)ntile_all / (unsigned)nparts);
    const int ntile = (int)((unsigned)(part + 1) * (unsigned)ntile_all / (unsigned)nparts) - tile0;
    const int ns2 = ntile * KSL;
    const int n2p = (ns2 + L::U2 - 1) / L::U2 * L::U2;  // stage-2 trip count, padded likewise
    // per row group g: reduction scratch at g * red, T tile at RG * red + g * ttile (stage 1 and T phase);
    // output staging tile (g, buffer) at 2 * slab2 + (2 g + buffer) * ytile (stage 2)
    unsigned char* const ttile = lds + RG * L::red;
    unsigned char* const ytile = lds + 2 * L::slab2;
    // Work-groups walk the contraction slabs (stage 1) and the output tiles (stage 2) from
    // different starting points, so that at any instant they touch different columns of
    // Xin / Yout and different rows of the factors.
    const int rot1 = (int)((unsigned)rb % (unsigned)ns1);
    const int rot2 = (int)((unsigned)rb % (unsigned)ntile);
    auto slab1_of = [&](int s) { if (s > ns1 - 1) s = ns1 - 1; s += rot1; return s >= ns1 ? s - ns1 : s; };
    auto tile_of = [&](int t) { if (t > ntile - 1) t = ntile - 1; t += rot2; return tile0 + (t >= ntile ? t - ntile : t); };

    if (wave >= NMW) {
        // ================================================================== loader waves
        // Every global access here is a buffer instruction: a wave-uniform descriptor and scalar
        // offset plus one 32-bit offset per lane.  Loads addressed by 64-bit per-lane pointers issue
        // at little more than half the rate while the MFMA waves on the same SIMDs are busy; buffer
        // loads do not slow down.  The descriptors cover exactly this work-group's valid rows and the
        // row offset is part of the per-lane offset (the only part the hardware range-checks), so
        // rows past M read as zeros and stores to them are dropped.
        const int lt = tid - NMT;
        const int64_t rows_valid = M - row0 < ROWS ? M - row0 : ROWS;
        // gather: the descriptor covers the pixels this work-group's patches can touch (from the start of
        // the grid row of its first row to the end of the grid row of its last, and the reach of the window)
        const int reach = GATHER ? (gg.kh / 2) * gg.W + gg.kw / 2 : 0;
        const bool plain = !GATHER || (gg.mul == 1 && gg.shift == 0);
        int64_t gpix0 = 0, gpix1 = 0;
        if constexpr (GATHER) {
            const int last = (int)(row0 + ROWS < M ? row0 + ROWS : M) - 1;
            const int64_t pixels = (M / ((int64_t)gg.RH * gg.RW)) * gg.H * gg.W;
            const int c0 = ch2_centre(gg, (int)row0, 0), c1 = ch2_centre(gg, last, 1);
            gpix0 = c0 > reach ? c0 - reach : 0;
            gpix1 = (int64_t)c1 + reach + 1 < pixels ? (int64_t)c1 + reach + 1 : pixels;
        }
        const rsrc_t xres = GATHER ? make_rsrc(Xin + gpix0 * gg.Cin, (gpix1 - gpix0) * gg.Cin * 2)
                                   : make_rsrc(Xin + row0 * p, rows_valid * p * 2);
        const rsrc_t pres = make_rsrc(Pm, (int64_t)R * p * 2);
        // stage-2 chunk assignment (computed first: the first Q slabs are requested before stage 1's
        // epilogue so that their latency hides behind the reduction and the T tile)
        int qoff[L::NCHQ], qsrc[L::NCHQ];
#pragma unroll
        for (int e = 0; e < L::NCHQ; ++e) {
            const int ci = e * NLT + lt;
            const int row = ci / CPR2, ch = ci % CPR2;
            qsrc[e] = (row * R + ch * 8) * 2;
            qoff[e] = row * (BK2 * 2) + swz<CPR2>(ch, row) * 16;
        }
        {
            // stage 1: one ring entry = this thread's chunks of one slab (64 rows of Xin, then the R
            // rows of P), D1 slabs ahead
            int xsrc[L::NCHX], off[L::NCHX];
            int gy[L::NCHX], gx[L::NCHX];                // gather: image coordinates of the thread's rows
#pragma unroll
            for (int e = 0; e < L::NCHX; ++e) {
                const int ci = e * NLT + lt;
                const int row = ci / CPR1, ch = ci % CPR1;
                off[e] = row * (BK1 * 2) + swz<CPR1>(ch, row) * 16;
                if constexpr (GATHER) {
                    const int64_t pix = row0 + row;
                    const int x = (int)(pix % gg.RW), y = (int)((pix / gg.RW) % gg.RH);
                    const int64_t img = pix / ((int64_t)gg.RW * gg.RH);
                    gx[e] = gg.mul * x;
                    gy[e] = pix < M ? gg.mul * y : -(1 << 20);   // rows past M: never valid
                    // plain: offset of the row's own pixel; else: offset of its image's first pixel
                    xsrc[e] = plain ? ((int)(pix - gpix0) * gg.Cin + ch * 8) * 2
                                    : ((int)(img * gg.H * gg.W - gpix0) * gg.Cin + ch * 8) * 2;
                } else {
                    gx[e] = gy[e] = 0;
                    xsrc[e] = (row * p + ch * 8) * 2;
                }
            }
            // per-lane and wave-uniform offset of chunk e of (virtual) slab vs
            auto xaddr = [&](int e, int vs, int& voff, int& soff) {
                if constexpr (GATHER) {
                    const int tap = vs / gg.cpb, cb = vs - tap * gg.cpb;
                    const int ky = tap / gg.kw, kx = tap - ky * gg.kw;
                    const int dy = gg.sign * (ky - gg.kh / 2), dx = gg.sign * (kx - gg.kw / 2);
                    const int ch8 = (lt % CPR1) * 8;
                    if (plain) {
                        const bool ok = (unsigned)(gy[e] + dy) < (unsigned)gg.H && (unsigned)(gx[e] + dx) < (unsigned)gg.W &&
                                        cb * 64 + ch8 < gg.Cin;
                        voff = ok ? xsrc[e] + ((dy * gg.W + dx) * gg.Cin + cb * 64) * 2 : kBufNowhere;
                    } else {
                        const int ty = gy[e] + dy, tx = gx[e] + dx, low = (1 << gg.shift) - 1;
                        const int sy = ty >> gg.shift, sx = tx >> gg.shift;
                        const bool ok = ty >= 0 && tx >= 0 && ((ty | tx) & low) == 0 && sy < gg.H && sx < gg.W &&
                                        cb * 64 + ch8 < gg.Cin;
                        voff = ok ? xsrc[e] + ((sy * gg.W + sx) * gg.Cin + cb * 64) * 2 : kBufNowhere;
                    }
                    soff = 0;
                } else {
                    voff = xsrc[e];
                    soff = vs * (BK1 * 2);
                }
            };
            // P chunk e of this thread: row 32 e + lt / 8, chunk lt % 8
            const int prow0 = lt / CPR1, pch = lt % CPR1;
            const int psrc = (prow0 * p + pch * 8) * 2;
            const int pstep = (NLT / CPR1) * p * 2;      // 32 rows of P, in bytes
            int poff[L::NCHP];
#pragma unroll
            for (int e = 0; e < L::NCHP; ++e) {
                const int row = e * (NLT / CPR1) + prow0;
                poff[e] = L::xpart + row * (BK1 * 2) + swz<CPR1>(pch, row) * 16;
            }
            u32x4 ring[D1][L::NCHX + L::NCHP];
            auto load = [&](u32x4 (&dst)[L::NCHX + L::NCHP], int s) {
                const int vs = slab1_of(s);
                const int so = vs * (BK1 * 2);
#pragma unroll
                for (int e = 0; e < L::NCHX; ++e) {
                    int vo, xo;
                    xaddr(e, vs, vo, xo);
                    dst[e] = buf_load16(xres, vo, xo);
                }
#pragma unroll
                for (int e = 0; e < L::NCHP; ++e) dst[L::NCHX + e] = buf_load16(pres, psrc, so + e * pstep);
            };
            auto store = [&](const u32x4 (&srcv)[L::NCHX + L::NCHP], int slot) {
#pragma unroll
                for (int e = 0; e < L::NCHX; ++e) *reinterpret_cast<u32x4*>(lds + slot * L::slab1 + off[e]) = srcv[e];
#pragma unroll
                for (int e = 0; e < L::NCHP; ++e)
                    *reinterpret_cast<u32x4*>(lds + slot * L::slab1 + poff[e]) = srcv[L::NCHX + e];
            };
            // steady state: chunk e of slab s+1 goes to LDS (slot s&1 is being read) and the same
            // chunk of slab s+1+D1 is requested, alternating: the LDS port and the vector-memory
            // address path then both stay busy instead of taking turns
            auto step1 = [&](u32x4 (&rg)[L::NCHX + L::NCHP], int s) {
                const int slot = (s + 1) & 1;
                const int vs = slab1_of(s + 1 + D1);
                const int so = vs * (BK1 * 2);
#pragma unroll
                for (int e = 0; e < L::NCHX; ++e) {
                    int vo, xo;
                    xaddr(e, vs, vo, xo);
                    *reinterpret_cast<u32x4*>(lds + slot * L::slab1 + off[e]) = rg[e];
                    rg[e] = buf_load16(xres, vo, xo);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int e = 0; e < L::NCHP; ++e) {
                    *reinterpret_cast<u32x4*>(lds + slot * L::slab1 + poff[e]) = rg[L::NCHX + e];
                    rg[L::NCHX + e] = buf_load16(pres, psrc, so + e * pstep);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            // all D1 slabs are requested before the first one is waited for
#pragma unroll
            for (int d = 0; d < D1; ++d) load(ring[d], d);
            store(ring[0], 0);
            load(ring[0], D1);
            wg_barrier();                                   // slab 0 is in slot 0
            for (int s0 = 0; s0 < n1p; s0 += D1) {
#pragma unroll
                for (int d = 0; d < D1; ++d) {
                    step1(ring[(d + 1) % D1], s0 + d);
                    wg_barrier();
                }
            }
        }
        // stage-2 ring: D2 slabs of Q in flight.  The descriptor is rebuilt per slab (scalar work) to
        // cover exactly the tile's rows: the wave-uniform offset of a buffer access is not range
        // checked, only the per-lane part is.  Rows of a ragged last tile that lie past the end of Q
        // then read as zeros; their output columns are never stored.
        u32x4 ring2[D2][L::NCHQ];
        auto load_q = [&](u32x4 (&dst)[L::NCHQ], int s) {
            if (s > ns2 - 1) s = ns2 - 1;
            const int t = tile_of(s / KSL);
            const int rows = q - t * 128 < 128 ? q - t * 128 : 128;
            const rsrc_t qres = make_rsrc(Qm + (int64_t)t * 128 * R, (int64_t)rows * R * 2);
            const int so = (s % KSL) * BK2 * 2;
#pragma unroll
            for (int e = 0; e < L::NCHQ; ++e) dst[e] = buf_load16(qres, qsrc[e], so);
        };
        // The first D2 slabs of Q are requested around the barriers of the T phase, one slab per
        // barrier and the rest after the last: requesting them all first would hold the MFMA waves
        // at the first of those barriers for as long as the requests take to issue.
#pragma unroll
        for (int i = 0; i <= L::n_mid_barriers; ++i) {
            if (Yout != nullptr) {
#pragma unroll
                for (int d = 0; d < D2; ++d)
                    if ((d < L::n_mid_barriers ? d : L::n_mid_barriers) == i) load_q(ring2[d], d);
            }
            if (i < L::n_mid_barriers) wg_barrier();
        }
        // T tile is in LDS: store it (the MFMA waves load their operands from it meanwhile)
        if (Tout != nullptr && part == 0) {
            // rows of Tout are t_pitch elements apart (R for a plain T; more when the tile is a
            // column block of a wider matrix); the descriptor ends with the last valid row
            const rsrc_t tres = make_rsrc(Tout + row0 * t_pitch, ((rows_valid - 1) * t_pitch + R) * 2);
            constexpr int CPT = R / 8;   // 16-byte chunks per T row
            for (int i = lt; i < ROWS * CPT; i += NLT) {
                const int row = i / CPT, ch = i % CPT;
                buf_store16_maybe_stream(stream_out != 0, *reinterpret_cast<const u32x4*>(ttile + (row >> 6) * L::ttile + (row & 63) * L::tpitch + ch * 16),
                            tres, (row * t_pitch + ch * 8) * 2, 0);
            }
        }
        if (Yout == nullptr) return;
        const rsrc_t yres = make_rsrc(Yout + row0 * q, rows_valid * q * 2);
        wg_barrier();                                    // T tile consumed: LDS belongs to stage 2
#pragma unroll
        for (int e = 0; e < L::NCHQ; ++e) *reinterpret_cast<u32x4*>(lds + qoff[e]) = ring2[0][e];
        load_q(ring2[0], D2);
        wg_barrier();                                    // Q slab 0 is in slot 0
        // stage 2: the Q slabs, and the finished output tiles: tile t was staged in LDS by the MFMA
        // waves during the last slab of t and leaves here, one slab later, as full 256-byte rows, in
        // four pieces per thread (64 rows x 16 chunks over 256 threads): the LDS reads are issued
        // first, the stores are spread between the slab's loads.
        constexpr int NY = ROWS * 16 / NLT;              // 16-byte pieces of a ROWS x 128 tile per thread
        u32x4 ypiece[NY];
        int ydst[NY];
        bool yleft[NY];
#pragma unroll
        for (int e = 0; e < NY; ++e) {
            const int ci = e * NLT + lt;
            ydst[e] = ((ci >> 4) * q + (ci & 15) * 8) * 2;
            yleft[e] = (ci & 15) < 8;                    // in the left 64 columns: all a ragged last tile has
        }
        auto flush_read = [&](int seq) {
#pragma unroll
            for (int e = 0; e < NY; ++e) {
                const int ci = e * NLT + lt;
                const int r = ci >> 4;
                const unsigned char* yt = ytile + ((r >> 6) * 2 + (seq & 1)) * L::ytile;
                ypiece[e] = *reinterpret_cast<const u32x4*>(yt + (r & 63) * L::ypitch + (ci & 15) * 16);
            }
        };
        auto flush_store = [&](int seq, int e) {
            const int t = tile_of(seq);
            const bool whole = q - t * 128 >= 128;
            if (whole || yleft[e]) buf_store16_maybe_stream(stream_out != 0, ypiece[e], yres, ydst[e], t * 256);
        };
        auto step2 = [&](u32x4 (&rg)[L::NCHQ], int s, bool flush, int seq) {
            const int slot = (s + 1) & 1;
            int sn = s + 1 + D2;
            if (sn > ns2 - 1) sn = ns2 - 1;
            const int tn = tile_of(sn / KSL);
            const int rows = q - tn * 128 < 128 ? q - tn * 128 : 128;
            const rsrc_t qres = make_rsrc(Qm + (int64_t)tn * 128 * R, (int64_t)rows * R * 2);
            const int so = (sn % KSL) * BK2 * 2;
            if (flush) flush_read(seq);
#pragma unroll
            for (int e = 0; e < L::NCHQ; ++e) {
                *reinterpret_cast<u32x4*>(lds + slot * L::slab2 + qoff[e]) = rg[e];
                rg[e] = buf_load16(qres, qsrc[e], so);
                __builtin_amdgcn_sched_barrier(0);
                if (e < NY && flush) flush_store(seq, e);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (flush) {
#pragma unroll
                for (int e = L::NCHQ; e < NY; ++e) flush_store(seq, e);
            }
        };
        int flushed = 0;
        for (int s0 = 0; s0 < n2p; s0 += D2) {
#pragma unroll
            for (int d = 0; d < D2; ++d) {
                const int s = s0 + d;
                // tile t is staged by the MFMA waves during slab (t + 1) KSL (they finish a slab's last
                // step one barrier late) and leaves during the slab after that
                const bool flush = s > KSL && (s - 1) % KSL == 0 && flushed < ntile;
                step2(ring2[(d + 1) % D2], s, flush, flushed);
                if (flush) ++flushed;
                wg_barrier();
            }
        }
        wg_barrier();                                    // the last tile is staged
        for (; flushed < ntile; ++flushed) {             // at most the last two tiles, one per staging buffer
            flush_read(flushed);
#pragma unroll
            for (int e = 0; e < NY; ++e) flush_store(flushed, e);
        }
        return;
    }

    // ====================================================================== MFMA waves
    const int lj = lane & 31, lh = lane >> 5;
    const int grp = wave >> 2, w4 = wave & 3;           // row group, wave inside the group
    const int cs = w4 % CS, rs = (w4 / CS) % RS, ks = w4 / (CS * RS);
    unsigned char* const ttile_g = ttile + grp * L::ttile;
    unsigned char* const red_g = lds + grp * L::red;

    // ------------------------------------------------------------------ stage 1
    f32x16 acc1[RA][CB];
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc1[a][b][v] = 0.0f;
    // One k16 step's operands.  The steps run as a software pipeline: the operands of step g + 1
    // are requested before the MFMAs of step g are issued, and the last step of a slab is held back
    // across the barrier, so that its MFMAs cover the latency of the next slab's first reads (a
    // slab's data may only be read after the barrier that publishes it).  Operand sets alternate
    // between two register buffers by the parity of the running step number.
    struct Ops1 { u32x4 xf[RA]; u32x4 pf[CB]; };
    Ops1 ob[2];
    auto read1 = [&](Ops1& o, int s, int j) {
        const unsigned char* base = lds + (s & 1) * L::slab1;
        const int kk = ks * SPW + j;                    // k16 step inside the slab
        const int qc = 2 * kk + lh;                     // logical chunk of this lane's 8 values
#pragma unroll
        for (int a = 0; a < RA; ++a) {
            const int row = 64 * grp + 32 * (rs * RA + a) + lj;
            o.xf[a] = *reinterpret_cast<const u32x4*>(base + row * (BK1 * 2) + swz<CPR1>(qc, row) * 16);
        }
#pragma unroll
        for (int b = 0; b < CB; ++b) {
            const int row = ROWS + (cs * CB + b) * 32 + lj;
            o.pf[b] = *reinterpret_cast<const u32x4*>(base + row * (BK1 * 2) + swz<CPR1>(qc, row) * 16);
        }
    };
    auto mma1 = [&](const Ops1& o) {
#pragma unroll
        for (int a = 0; a < RA; ++a)
#pragma unroll
            for (int b = 0; b < CB; ++b) acc1[a][b] = mfma16(o.pf[b], o.xf[a], acc1[a][b]);
    };
    // slab s: the held step of slab s - 1 sits in ob[1] (every slab has an even number of steps, or
    // a single one that is moved there)
    auto slab1 = [&](int s) {
        read1(ob[0], s, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (s > 0) mma1(ob[1]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (SPW == 1) {
            ob[1] = ob[0];
        } else {
#pragma unroll
            for (int j = 0; j + 1 < SPW; ++j) {
                read1(ob[(j + 1) & 1], s, j + 1);
                __builtin_amdgcn_sched_barrier(0);
                mma1(ob[j & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    static_assert(SPW == 1 || SPW % 2 == 0, "step parity");
    wg_barrier();                                       // slab 0 is in slot 0
    for (int s = 0; s < n1p; ++s) {
        if (s < ns1) slab1(s);
        wg_barrier();
    }
    mma1(ob[1]);                                        // the held last step (read before the last barrier)
    // ------------------------------------------------------------------ sum over the KS groups, T tile (bf16) to LDS
    // lane holds T[32(rs RA + a) + lj][32(cs CB + b) + 8g + 4 lh + (0..3)] in acc1[a][b][4g .. 4g+3]
    auto emit_T = [&](const f32x16 (&blk)[CB], int a) {
#pragma unroll
        for (int b = 0; b < CB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 o = {pack2_bf16(blk[b][4 * g + 0], blk[b][4 * g + 1]),
                           pack2_bf16(blk[b][4 * g + 2], blk[b][4 * g + 3])};
                *reinterpret_cast<u32x2*>(ttile_g + (32 * (rs * RA + a) + lj) * L::tpitch +
                                          (32 * (cs * CB + b) + 8 * g + 4 * lh) * 2) = o;
            }
    };
    if constexpr (KS == 2 && RA == 2) {
        // Two contraction groups: the partners swap halves instead of one sending everything.  Wave ks
        // sends its row block 1 - ks, adds what it receives to its row block ks and converts that
        // half of T itself: every wave stores and loads half as much, and all four convert.
        f32x4* red = reinterpret_cast<f32x4*>(red_g);
        auto swap_and_emit = [&](const f32x16 (&send)[CB], f32x16 (&keep)[CB], int a_keep) {
            f32x4* dst = red + (size_t)((ks * CS + cs) * CB) * 4 * 64;
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    dst[(b * 4 + g) * 64 + lane] = f32x4{send[b][4 * g], send[b][4 * g + 1], send[b][4 * g + 2], send[b][4 * g + 3]};
            wg_barrier();
            const f32x4* src = red + (size_t)(((1 - ks) * CS + cs) * CB) * 4 * 64;
#pragma unroll
            for (int b = 0; b < CB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v = src[(b * 4 + g) * 64 + lane];
                    keep[b][4 * g] += v[0]; keep[b][4 * g + 1] += v[1];
                    keep[b][4 * g + 2] += v[2]; keep[b][4 * g + 3] += v[3];
                }
            emit_T(keep, a_keep);
        };
        if (ks == 0) swap_and_emit(acc1[1], acc1[0], 0);
        else swap_and_emit(acc1[0], acc1[1], 1);
    } else {
        if constexpr (KS > 1) {
            // tree; layout: [wave slot][block (a,b)][quad g][lane][4 floats]: one 16-byte access per quad
            f32x4* red = reinterpret_cast<f32x4*>(red_g);
            const int wslot = rs * CS + cs;
#pragma unroll
            for (int half = KS / 2; half >= 1; half >>= 1) {
                if (ks >= half && ks < 2 * half) {
                    f32x4* dst = red + (size_t)(((ks - half) * (CS * RS) + wslot) * (RA * CB)) * 4 * 64;
#pragma unroll
                    for (int a = 0; a < RA; ++a)
#pragma unroll
                        for (int b = 0; b < CB; ++b)
#pragma unroll
                            for (int g = 0; g < 4; ++g)
                                dst[((a * CB + b) * 4 + g) * 64 + lane] =
                                    f32x4{acc1[a][b][4 * g], acc1[a][b][4 * g + 1], acc1[a][b][4 * g + 2], acc1[a][b][4 * g + 3]};
                }
                wg_barrier();
                if (ks < half) {
                    const f32x4* src = red + (size_t)((ks * (CS * RS) + wslot) * (RA * CB)) * 4 * 64;
#pragma unroll
                    for (int a = 0; a < RA; ++a)
#pragma unroll
                        for (int b = 0; b < CB; ++b)
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                const f32x4 v = src[((a * CB + b) * 4 + g) * 64 + lane];
                                acc1[a][b][4 * g] += v[0]; acc1[a][b][4 * g + 1] += v[1];
                                acc1[a][b][4 * g + 2] += v[2]; acc1[a][b][4 * g + 3] += v[3];
                            }
                }
                if (half > 1) wg_barrier();             // the next round overwrites what was just read
            }
        }
        if (ks == 0) {
#pragma unroll
            for (int a = 0; a < RA; ++a) emit_T(acc1[a], a);
        }
    }
    wg_barrier();                                       // last of the mid barriers: T tile complete
    if (Yout == nullptr) return;

    // Stage 2: wave w4 of a row group owns the group's 64 rows of T (in registers, as MFMA B operands)
    // and column block w4 (32 columns) of every 128-column output tile; in the row-split form, rows
    // 32 (w4 & 1) .. + 31 of the group and column blocks 2 (w4 >> 1), 2 (w4 >> 1) + 1.
    constexpr int KB = R / 16;
    constexpr int TA = L::RSPLIT ? 1 : 2;               // row blocks of T per wave
    constexpr int QB = L::RSPLIT ? 2 : 1;               // column blocks of the tile per wave
    const int trow0 = L::RSPLIT ? 32 * (w4 & 1) : 0;
    const int qrow0 = L::RSPLIT ? 64 * (w4 >> 1) : 32 * w4;
    u32x4 tf[TA][KB];   // T[trow0 + 32a + lj][16kb + 8 lh .. +7]
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
            tf[a][kb] = *reinterpret_cast<const u32x4*>(ttile_g + (trow0 + 32 * a + lj) * L::tpitch + (16 * kb + 8 * lh) * 2);
    wg_barrier();                                       // T tile consumed; stage 2 takes over the LDS
    wg_barrier();                                       // Q slab 0 is in slot 0
    // ------------------------------------------------------------------ stage 2
    // Software pipeline as in stage 1: a ring of NB operand buffers is refilled as soon as a step's
    // MFMAs are issued (NB - 1 reads stay in flight), and the last step of a slab is held back across
    // the barrier.  A tile's accumulators are therefore complete, and staged, one barrier later than
    // its last slab.
    constexpr int NS = BK2 / 16;                        // k16 steps per slab
    constexpr int NB = largest_divisor(NS, L::NB2);     // divides NS: the held step always sits in ring[NB - 1]
    // The swizzle XORs the low XB bits of the chunk index 2 kk + lh with row bits, and a row starts
    // at a multiple of 16 << XB bytes (BK2 is a multiple of 8 << XB elements), so the address
    // of step kk is that of step 0 with (kk mod PER) << 5 XORed in, plus a constant for kk / PER:
    // one lane address serves all steps (and all column blocks: 32 rows on leave the row bits alone).
    constexpr int XB = CPR2 % 16 == 0 ? 4 : (CPR2 % 8 == 0 ? 3 : 2);
    constexpr int PER = (1 << XB) / 2;
    static_assert((BK2 * 2) % (16 << XB) == 0, "row pitch and swizzle width");
    const int qaddr0 = (qrow0 + lj) * (BK2 * 2) + swz<CPR2>(lh, qrow0 + lj) * 16;
    struct Ops2 { u32x4 qf[QB]; };
    auto read2 = [&](Ops2& dst, int s, int kk) {
#pragma unroll
        for (int b = 0; b < QB; ++b)
            dst.qf[b] = *reinterpret_cast<const u32x4*>(lds + (s & 1) * L::slab2 + (qaddr0 ^ ((kk % PER) << 5)) +
                                                       (kk / PER) * (16 << XB) + b * 32 * (BK2 * 2));
    };
    f32x16 acc2[TA][QB];
    Ops2 ring[NB];
    auto mma2 = [&](const Ops2& o, int kb) {
#pragma unroll
        for (int a = 0; a < TA; ++a)
#pragma unroll
            for (int b = 0; b < QB; ++b) acc2[a][b] = mfma16(o.qf[b], tf[a][kb], acc2[a][b]);
    };
    auto stage_out = [&](int t) {
        // lane holds Y[trow0 + 32a + lj][qrow0 + 32b + 8g + 4 lh + (0..3)] of its group's 64 x 128 tile
        unsigned char* yt = ytile + (grp * 2 + (t & 1)) * L::ytile;
#pragma unroll
        for (int a = 0; a < TA; ++a)
#pragma unroll
            for (int b = 0; b < QB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x2 o = {pack2_bf16(acc2[a][b][4 * g + 0], acc2[a][b][4 * g + 1]),
                               pack2_bf16(acc2[a][b][4 * g + 2], acc2[a][b][4 * g + 3])};
                    *reinterpret_cast<u32x2*>(yt + (trow0 + 32 * a + lj) * L::ypitch +
                                              (qrow0 + 32 * b + 8 * g + 4 * lh) * 2) = o;
                }
    };
    auto clear2 = [&]() {
#pragma unroll
        for (int a = 0; a < TA; ++a)
#pragma unroll
            for (int b = 0; b < QB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[a][b][v] = 0.0f;
    };
    clear2();
    for (int s0 = 0; s0 < n2p; s0 += KSL) {
        const int t = s0 / KSL;
#pragma unroll
        for (int kslab = 0; kslab < KSL; ++kslab) {
            const int s = s0 + kslab;
            const bool live = s < ns2;                  // padded trips only keep the barrier count
            if (live) {
#pragma unroll
                for (int i = 0; i + 1 < NB; ++i) read2(ring[i], s, i);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (s > 0 && s - 1 < ns2) {
                // last step of the slab before this one
                mma2(ring[NB - 1], ((kslab + KSL - 1) % KSL) * NS + NS - 1);
                if (kslab == 0) {
                    stage_out(t - 1);
                    clear2();
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (live) {
                read2(ring[NB - 1], s, NB - 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kk = 0; kk + 1 < NS; ++kk) {
                    mma2(ring[kk % NB], kslab * NS + kk);
                    __builtin_amdgcn_sched_barrier(0);
                    if (kk + NB < NS) read2(ring[kk % NB], s, kk + NB);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            wg_barrier();
        }
    }
    if (n2p == ns2) {                                   // no padded trip has finished the last slab
        mma2(ring[NB - 1], (KSL - 1) * NS + NS - 1);
        stage_out(ntile - 1);
    }
    wg_barrier();                                       // the last tile is staged
}

#undef ABT_LOADER_WAVE

template <int R, int RG, bool GATHER>
hipError_t launch_chain_r(const Ch2Ptrs& ptrs, int G, bool second_stage,
                          int64_t M, int p, int q, int t_pitch, const Ch2Gather& gg, int parts, hipStream_t s) {
    using L = Ch2Cfg<R, RG>;
    constexpr int lds_bytes = L::lds_bytes;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    // column parts: each does its share of the 128-column output tiles (and repeats stage 1)
    if (G < 1 || G > kChainMaxGroups || parts < 1 || parts > 64 || (second_stage && parts > (q + 127) / 128) ||
        (!second_stage && parts != 1))
        return hipErrorInvalidValue;
    // (setting the attribute twice from two host threads is harmless; the flag only saves the call)
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&chain2_bf16_kernel<R, RG, GATHER>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int64_t nblocks = ceil_div(M, L::ROWS);
    int64_t full = 0;
    int tail_parts = parts;
    if (parts == 1) {
        // A large batch ends with a partly filled round of the 256 compute units.  When that round is
        // at most half full and stage 2 is the larger part of a work-group's slabs, its row blocks are
        // split over the idle units by output tiles (one problem per launch only).
        full = nblocks;
        const int64_t tail = nblocks % 256;
        const int ntile = (q + 127) / 128;
        if (G == 1 && second_stage && nblocks > 256 && tail > 0 && 2 * tail <= 256) {
            int tp = (int)(256 / tail);
            if (tp > ntile) tp = ntile;
            const int ns1 = p / BK1, whole = ns1 + ntile * L::KSL, shared = ns1 + (ntile + tp - 1) / tp * L::KSL;
            if (tp >= 2 && 10 * shared <= 7 * whole) {
                full = nblocks - tail;
                tail_parts = tp;
            }
        }
    }
    const int64_t grid = full + (nblocks - full) * tail_parts;
    hipLaunchKernelGGL((chain2_bf16_kernel<R, RG, GATHER>), dim3((unsigned)grid, (unsigned)G), dim3(64 * (NMW_ * RG + NLW)),
                       lds_bytes, s, ptrs, M, p, q, t_pitch, gg, (int)full, tail_parts,
                       (int)(M * ((second_stage ? q : 0) + t_pitch) * 2 >= kStreamOutBytes));
    return hipGetLastError();
}

template <bool GATHER>
hipError_t launch_chain_64(const Ch2Ptrs& ptrs, int G, bool second_stage,
                           int64_t M, int p, int q, int R, int t_pitch, const Ch2Gather& gg, hipStream_t s) {
    switch (R) {
#define ABT_CASE(RR) case RR: return launch_chain_r<RR, 1, GATHER>(ptrs, G, second_stage, M, p, q, t_pitch, gg, 1, s);
        ABT_CASE(32) ABT_CASE(64) ABT_CASE(96) ABT_CASE(128) ABT_CASE(160) ABT_CASE(192)
        ABT_CASE(256) ABT_CASE(320) ABT_CASE(384)
#undef ABT_CASE
        default: return hipErrorInvalidValue;
    }
}

template <bool GATHER>
hipError_t launch_chain_128(const Ch2Ptrs& ptrs, int G, bool second_stage,
                            int64_t M, int p, int q, int R, int t_pitch, const Ch2Gather& gg, int parts, hipStream_t s) {
    switch (R) {
#define ABT_CASE(RR) case RR: return launch_chain_r<RR, 2, GATHER>(ptrs, G, second_stage, M, p, q, t_pitch, gg, parts, s);
        ABT_CASE(32) ABT_CASE(64) ABT_CASE(96) ABT_CASE(128) ABT_CASE(192) ABT_CASE(384)
#undef ABT_CASE
        default: return hipErrorInvalidValue;
    }
}

Ch2Ptrs one_problem(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout) {
    Ch2Ptrs t{};
    t.X[0] = (const uint16_t*)Xin; t.P[0] = (const uint16_t*)P; t.Q[0] = (const uint16_t*)Q;
    t.Y[0] = (uint16_t*)Yout; t.T[0] = (uint16_t*)Tout;
    return t;
}

// checks shared by the two gathered launchers; rows = work-group height
bool gather_ok(const PatchGeom& g, int64_t M, int64_t p, int t_pitch, int R, int rows) {
    if (!(g.H >= 1 && g.W >= 1 && g.Cin >= 8 && g.Cin % 8 == 0 && g.kh >= 1 && g.kw >= 1 && (g.kh & 1) && (g.kw & 1) &&
          (g.sign == 1 || g.sign == -1) && g.RH >= 1 && g.RW >= 1 && (g.mul == 1 || g.mul == 2) &&
          (g.shift == 0 || g.shift == 1) && M % ((int64_t)g.RH * g.RW) == 0 && M <= 0x7fffffff && p <= (1 << 20) &&
          t_pitch >= R))
        return false;
    // 32-bit offsets inside a work-group's window of the image: `rows` consecutive rows and the grid
    // rows they start and end in have their centres within mul^2 (rows + 2 RW) + 2 mul W pixels of
    // one another; the reach of the window comes on top
    const int64_t span = (int64_t)g.mul * g.mul * (rows + 2 * g.RW + 2) + 2 * (int64_t)g.mul * g.W +
                         2 * ((g.kh / 2) * (int64_t)g.W + g.kw / 2);
    return span * g.Cin * 2 < kBufMaxBytes && (M / ((int64_t)g.RH * g.RW)) * g.H * g.W <= 0x7fffffff;
}

Ch2Gather device_geom(const PatchGeom& g) {
    return Ch2Gather{g.H, g.W, g.Cin, (g.Cin + 63) / 64, g.kh, g.kw, g.sign, g.RH, g.RW, g.mul, g.shift};
}

}  // namespace

bool chain2_supports(int R, int p, int q) {
    if (p % 64 != 0 || p > (1 << 20) || q > (1 << 20)) return false;
    switch (R) {
        case 32: case 64: case 96: case 128: case 160: case 192: case 256: case 320: case 384: return true;
        default: return false;
    }
}

// Ranks whose two reduction scratches, T tiles and staging tiles fit the LDS and whose T operands
// fit the 168 registers twelve waves leave (R = 384 would need 192 for them alone).
bool chain2_tall_supports(int R, int p, int q) {
    if (p % 64 != 0 || p > (1 << 20) || q > (1 << 20)) return false;
    switch (R) {
        case 32: case 64: case 96: case 128: case 192: case 384: return true;
        default: return chain3_supports(R, p, q);
    }
}

hipError_t launch_chain2_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                              int64_t M, int p, int q, int R, hipStream_t s) {
    return launch_chain_64<false>(one_problem(Xin, P, Q, Yout, Tout), 1, Yout != nullptr, M, p, q, R, R, Ch2Gather{}, s);
}

hipError_t launch_chain2_tall_bf16(const void* Xin, const void* P, const void* Q, void* Yout, void* Tout,
                              int64_t M, int p, int q, int R, int parts, hipStream_t s) {
    if (chain3_supports(R, p, q)) {                     // wide ranks: the kernel of eight equal waves
        const ChainProblem one{Xin, P, Q, Yout, Tout};
        return launch_chain3_bf16(&one, 1, M, p, q, R, parts, s);
    }
    return launch_chain_128<false>(one_problem(Xin, P, Q, Yout, Tout), 1, Yout != nullptr, M, p, q, R, R, Ch2Gather{}, parts, s);
}

hipError_t launch_chain2_gather_bf16(const void* image, const PatchGeom& g, const void* P, const void* Q,
                                     void* Yout, void* Tout, int t_pitch, int64_t M, int q, int R, hipStream_t s) {
    const int cpb = (g.Cin + 63) / 64;
    const int64_t p = (int64_t)g.kh * g.kw * cpb * 64;
    if (!gather_ok(g, M, p, t_pitch, R, 64) || !chain2_supports(R, (int)p, q)) return hipErrorInvalidValue;
    const Ch2Gather gg = device_geom(g);
    return launch_chain_64<true>(one_problem(image, P, Q, Yout, Tout), 1, Yout != nullptr, M, (int)p, q, R, t_pitch, gg, s);
}

hipError_t launch_chain2_tall_gather_bf16(const void* image, const PatchGeom& g, const void* P, const void* Q,
                                     void* Yout, void* Tout, int t_pitch, int64_t M, int q, int R, hipStream_t s) {
    const int cpb = (g.Cin + 63) / 64;
    const int64_t p = (int64_t)g.kh * g.kw * cpb * 64;
    if (!gather_ok(g, M, p, t_pitch, R, 128) || !chain2_tall_supports(R, (int)p, q) || R == 256) return hipErrorInvalidValue;
    const Ch2Gather gg = device_geom(g);
    return launch_chain_128<true>(one_problem(image, P, Q, Yout, Tout), 1, Yout != nullptr, M, (int)p, q, R, t_pitch, gg, 1, s);
}

hipError_t launch_chain2_grouped_bf16(const ChainProblem* problems, int G, int64_t M, int p, int q, int R,
                                      int rows, int parts, hipStream_t s) {
    if (G < 1 || G > kChainMaxGroups || !problems) return hipErrorInvalidValue;
    if (rows == 128 && chain3_supports(R, p, q)) return launch_chain3_bf16(problems, G, M, p, q, R, parts, s);
    Ch2Ptrs t{};
    const bool second_stage = problems[0].Yout != nullptr;
    for (int g = 0; g < G; ++g) {
        if ((problems[g].Yout != nullptr) != second_stage) return hipErrorInvalidValue;   // one launch shape for all
        t.X[g] = (const uint16_t*)problems[g].Xin; t.P[g] = (const uint16_t*)problems[g].P;
        t.Q[g] = (const uint16_t*)problems[g].Q; t.Y[g] = (uint16_t*)problems[g].Yout; t.T[g] = (uint16_t*)problems[g].Tout;
    }
    if (rows == 128) return launch_chain_128<false>(t, G, second_stage, M, p, q, R, R, Ch2Gather{}, parts, s);
    return launch_chain_64<false>(t, G, second_stage, M, p, q, R, R, Ch2Gather{}, s);
}

}  // namespace abt
