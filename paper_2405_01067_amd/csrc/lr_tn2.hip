// Factor gradients of the factored layer (bf16 in, fp32 out):
//     dA[m,R] = dY[M,m]^T . T[M,R]          dB[R,n] = dT[M,R]^T . X[M,n]
// Both are contractions over the M batch rows, the slow dimension of every operand.  One generic
// job:  part[split][P,R] = U[rows of split, P]^T . V[rows of split, R]   (dA: U = dY, V = T;
// dB: U = X, V = dT, result stored transposed), followed by a fixed-order sum over the splits.
//
// Work-group: 128 columns of U x all R columns of V over one split of the batch rows.  Four MFMA
// waves (2 x 2, or 4 x 1 when R/32 is odd) each own a block of the output tile.  Loader waves (two
// for the U part, R/64 for the V part; half as many with two blocks per thread for wide slabs)
// move slabs of 64 batch rows global -> register ring (two slabs in flight) -> LDS, two LDS slots,
// one barrier per slab.  Both operands lie in memory with the contraction index (batch row)
// slowest, while an MFMA operand needs 8 consecutive batch rows per lane: the loaders transpose
// 8 x 8 blocks in registers (byte permutes) on the way, so the MFMA waves read their operands
// with plain 16-byte LDS loads.  (Reading row-major slabs with the transposing LDS load
// ds_read_b64_tr_b16 instead was limited by the rate of those 8-byte reads.)
#include "common.h"

namespace abt {

namespace {

__device__ __forceinline__ void ring_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ f32x16 mfma16(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
constexpr int TP = 128;      // U columns per work-group
constexpr int BKM = 64;      // batch rows per slab
constexpr int NMW = 4;       // MFMA waves

template <int R>
struct Tn2 {
    static constexpr int RB = R / 32;
    static constexpr bool even = (RB % 2) == 0;
    static constexpr int WGP = even ? 2 : 4, WGQ = even ? 2 : 1;
    static constexpr int PB = even ? 2 : 1, QB = even ? RB / 2 : RB;
    static constexpr int NCOL = TP + R;                      // columns of a slab: U part, then V part
    static constexpr int slab = NCOL * BKM * 2;
    static constexpr int lds_bytes = 2 * slab;
    // loader work unit: an 8 x 8 block (8 batch rows x one 16-byte chunk of columns)
    static constexpr int BPT = NCOL > 320 ? 2 : 1;           // blocks per loader thread
    static constexpr int NUW = (TP / BPT + 63) / 64;         // loader waves for the U part
    static constexpr int NVW = (R / BPT + 63) / 64;          // loader waves for the V part
    static constexpr int NT = 64 * (NMW + NUW + NVW);
    // slabs in flight in the loaders' register ring: a CU wants about 64 KB of loads outstanding,
    // which two slabs only give when a slab is 40 KB or more (R >= 192)
    static constexpr int D = slab * 2 >= 64 * 1024 ? 2 : (slab * 3 >= 64 * 1024 ? 3 : 4);
    static_assert(lds_bytes <= 160 * 1024, "slab shape");
};

struct Tn2Job { const uint16_t* U; const uint16_t* V; float* part; int P; int tile_begin; int transposed; int gather; };
// Gather form of U (jobs with gather != 0): U is a channels-last image [M / (H W), H, W, C] and column
// tap C + c of row i of the virtual U is channel c of pixel (y + ky - kh/2, x + kx - kw/2) of the
// same image (tap = ky kw + kx), zero outside it.  job.P = kh kw C.
// Rows are the pixels of a grid RH x RW per image; row (y, x) is centred on image pixel (mul y, mul x)
// (mul = 1 with RH x RW = H x W: every pixel; mul = 2: the patches of a stride-2 convolution).
struct Tn2Gather { int H, W, C, kh, kw, RH, RW, mul; };
struct Tn2Args { Tn2Job job[kTnMaxJobs]; int njobs; int tiles; int splits; int64_t M; int64_t rows_per_split; Tn2Gather g; };

// LDS slab: column-major, 64 batch rows = 128 bytes per column, two columns per 256-byte line.  The
// sixteen 16-byte units of a line are XOR-swizzled with bits of the column-pair index p so that
// sixteen different bank groups are touched both by a loader store (16 lanes = 16 column chunks
// 8 columns apart, same unit: p bits 2..5 vary) and by an MFMA operand read (16 lanes = 16
// consecutive columns, same unit: p bits 0..2 and the column parity vary).
__device__ __forceinline__ int slab_addr(int col, int unit) {
    const int p = col >> 1;
    const int swz = ((p ^ (p >> 3)) & 3) | (p & 4) | (((p >> 5) & 1) << 3);
    const int u16 = (((col & 1) << 3) | unit) ^ swz;
    return p * 256 + u16 * 16;
}

// Loader role: moves NCOLS columns (multiple of 8) of a row-major bf16 matrix, 64 batch rows at a
// time, into LDS columns [col0, col0 + NCOLS) transposed: a thread loads an 8 x 8 block as eight
// 16-byte row pieces, transposes it in registers, and stores eight 16-byte column pieces.
// STREAM: the source is read once by the whole launch (the U strips): loads carry the non-temporal hint
// (0.7 % of a config-3 step; the same hint on the activation loads of the chain kernels measured slower).
template <int NCOLS, int BPT, int D, bool GATHER = false, bool STREAM = false>
__device__ __forceinline__ void tn_loader(const uint16_t* src, int pitch, int cols_valid, int col0, int lt,
                                          int64_t k_begin, int64_t k_end, int np, int slab_bytes,
                                          unsigned char* lds, const Tn2Gather tg = Tn2Gather{}, int vcol0 = 0,
                                          int64_t pixels = 0) {
    constexpr int NCC = NCOLS / 8;                       // 16-byte chunks per row
    constexpr int RGS = 8 / BPT;                         // row groups per block index
    const int cc = lt % NCC, rg0 = lt / NCC;
    const bool active = rg0 < RGS;
    // Offsets of the thread's first block; a second block (BPT = 2) lies 32 batch rows further:
    // 32 rows of `pitch` elements in memory, unit index + 4 = address ^ 64 in the LDS slab.
    int goff[8], loff[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        // global: row 8 rg + e, columns 8 cc ..; a chunk past the valid columns, or an idle
        // thread, gets an offset that no descriptor covers and loads zeros
        goff[e] = (active && cc * 8 < cols_valid) ? ((8 * rg0 + e) * pitch + cc * 8) * 2 : kBufNowhere;
        loff[e] = slab_addr(col0 + cc * 8 + e, rg0);         // LDS: column 8 cc + e, rows 8 rg .. 8 rg + 7
    }
    const int gstep = (active && cc * 8 < cols_valid) ? 32 * pitch * 2 : 0;
    u32x4 ring[D][BPT][8];
    auto descriptor = [&](int s) {
        const int64_t kr0 = k_begin + (int64_t)s * BKM;
        const int64_t left = k_end - kr0;                // <= 0 past the split: everything reads zeros
        // the row offset is part of the per-lane offset, the only part the hardware range-checks;
        // the descriptor ends at the split's last row
        return make_rsrc(src + kr0 * pitch, left * pitch * 2);
    };
    auto load_block = [&](u32x4 (&dst)[8], rsrc_t res, int b) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            dst[e] = STREAM ? __builtin_amdgcn_raw_buffer_load_b128(res, goff[e] + b * gstep, 0, 2)   // non-temporal
                            : buf_load16(res, goff[e] + b * gstep, 0);
    };
    // gather: this thread's eight virtual columns lie in one tap (C is a multiple of 8)
    const bool colok = active && cc * 8 < cols_valid;
    const int gtap = GATHER ? (vcol0 + cc * 8) / tg.C : 0;
    const int gc = GATHER ? (vcol0 + cc * 8) - gtap * tg.C : 0;
    const int gky = GATHER ? gtap / tg.kw : 0;
    const int gdy = GATHER ? gky - tg.kh / 2 : 0, gdx = GATHER ? (gtap - gky * tg.kw) - tg.kw / 2 : 0;
    const int reach = GATHER ? (tg.kh / 2) * tg.W + tg.kw / 2 : 0;
    const int64_t span = k_end - k_begin;
    const int rows_in_split = span > 0x7fffffff ? 0x7fffffff : (int)span;
    // Gather state of each of the thread's blocks for the slab that block fetches next: image
    // coordinates of its first row, and that row's byte offset (tap shift and channel included).
    // Slabs are fetched in order (0, 1, 2, ...), 64 rows apart: the state is carried with an
    // add-and-wrap per slab, no integer division and no descriptor arithmetic in the loop.  One
    // descriptor serves the whole split: it covers the pixels that the patches of the split's rows
    // can touch (the host keeps that window below 2 GiB).
    int bx[BPT], by[BPT], boff[BPT];
    const int step_x = GATHER ? BKM % tg.W : 0, step_y = GATHER ? (BKM / tg.W) % tg.H : 0;
    // window of the image the split's patches can touch: [sp0, sp1) in pixels over all images
    int64_t sp0 = k_begin > reach ? k_begin - reach : 0;
    int64_t sp1 = k_end + reach;
    if (GATHER && tg.mul != 1 && k_end > k_begin) {
        auto centre = [&](int64_t i) {     // centre pixel of row i (monotone in i)
            const int64_t per = (int64_t)tg.RH * tg.RW, img = i / per, rem = i - img * per;
            return (img * tg.H + tg.mul * (rem / tg.RW)) * tg.W + tg.mul * (rem % tg.RW);
        };
        const int64_t c0 = centre(k_begin), c1 = centre(k_end - 1);
        sp0 = c0 > reach ? c0 - reach : 0;
        sp1 = c1 + reach + 1;
    }
    if (sp1 > pixels) sp1 = pixels;
    const rsrc_t gres = make_rsrc(src + sp0 * tg.C, GATHER ? (sp1 - sp0) * tg.C * 2 : 0);
#pragma unroll
    for (int b = 0; b < BPT; ++b) {
        const int64_t first = k_begin + 8 * rg0 + 32 * b;
        bx[b] = GATHER ? (int)(first % tg.W) : 0;
        by[b] = GATHER ? (int)((first / tg.W) % tg.H) : 0;
        boff[b] = (((int)(first - sp0) + gdy * tg.W + gdx) * tg.C + gc) * 2;
    }
    // Strided rows (mul > 1): the state of a block is the grid position and image of its first row;
    // offsets are formed per row from the coordinates (a few multiplies per slab), the window of the
    // descriptor starts at pixel sp0.
    int sx[BPT], sy[BPT], simg[BPT];
    const bool strided = GATHER && tg.mul != 1;
#pragma unroll
    for (int b = 0; b < BPT; ++b) {
        const int64_t first = k_begin + 8 * rg0 + 32 * b;
        sx[b] = strided ? (int)(first % tg.RW) : 0;
        sy[b] = strided ? (int)((first / tg.RW) % tg.RH) : 0;
        simg[b] = strided ? (int)(first / ((int64_t)tg.RW * tg.RH)) : 0;
    }
    auto load_block_strided = [&](u32x4 (&dst)[8], int s, int b) {
        int x = sx[b], y = sy[b], img = simg[b];
        const int left = rows_in_split - (s * BKM + 8 * rg0 + 32 * b);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int ty = tg.mul * y + gdy, tx = tg.mul * x + gdx;
            const bool ok = colok && e < left && (unsigned)ty < (unsigned)tg.H && (unsigned)tx < (unsigned)tg.W;
            const int pix = (img * tg.H + ty) * tg.W + tx - (int)sp0;
            dst[e] = buf_load16(gres, ok ? (pix * tg.C + gc) * 2 : kBufNowhere, 0);
            if (++x == tg.RW) { x = 0; if (++y == tg.RH) { y = 0; ++img; } }
        }
        // advance the block's first row by one slab of 64 rows (64 = qy RW + qx)
        const int qy = BKM / tg.RW, qx = BKM - qy * tg.RW;
        int nx = sx[b] + qx, ny = sy[b] + qy;
        if (nx >= tg.RW) { nx -= tg.RW; ++ny; }
        simg[b] += ny / tg.RH;
        sy[b] = ny % tg.RH;
        sx[b] = nx;
    };
    auto load_block_gather = [&](u32x4 (&dst)[8], int s, int b) {
        if (strided) { load_block_strided(dst, s, b); return; }
        const int x = bx[b], y = by[b], off = boff[b];
        // advance to the next slab (this lambda is called once per slab and block, in slab order)
        boff[b] += BKM * tg.C * 2;
        bx[b] += step_x;
        const int carry = bx[b] >= tg.W ? 1 : 0;
        bx[b] -= carry ? tg.W : 0;
        by[b] += step_y + carry;
        by[b] -= by[b] >= tg.H ? tg.H : 0;
        const int left = rows_in_split - (s * BKM + 8 * rg0 + 32 * b);   // rows e < left are inside the split
        if (tg.W >= 4) {
            // Eight consecutive pixels cross at most one image-row boundary (two when W < 8), the
            // first after `ew` of them.  Rows between two boundaries share y, and among them the rows
            // whose shifted x stays inside the image form one interval: the valid rows are two
            // (three) intervals of [0, 8), built as a bit mask with a few operations per slab instead
            // of a chain of compares per row (a loader wave has no second wave on its SIMD to hide
            // instruction latencies behind, so its instruction count is its time).
            auto bits = [](int a, int b) -> unsigned {       // bits a .. b-1, clamped to [0, 8)
                a = a < 0 ? 0 : a;
                b = b > 8 ? 8 : b;
                return b > a ? (1u << b) - (1u << a) : 0u;
            };
            const int ew = tg.W - x;                          // first row (of 8) on the next image row
            const int y1 = y + 1 == tg.H ? 0 : y + 1;
            const bool vy0 = (unsigned)(y + gdy) < (unsigned)tg.H, vy1 = (unsigned)(y1 + gdy) < (unsigned)tg.H;
            const int ewc = ew < 8 ? ew : 8;
            const int lo0 = -gdx - x, hi0 = tg.W - gdx - x;
            unsigned mask = vy0 ? bits(lo0, hi0 < ewc ? hi0 : ewc) : 0u;
            const int lo1 = ew - gdx > ew ? ew - gdx : ew;
            const int ew2 = ew + tg.W;                        // second boundary (inside the block only if W < 8)
            const int hi1 = ew - gdx + tg.W;
            mask |= vy1 ? bits(lo1, hi1 < ew2 ? hi1 : ew2) : 0u;
            if (tg.W < 8) {
                const int y2 = y1 + 1 == tg.H ? 0 : y1 + 1;
                const bool vy2 = (unsigned)(y2 + gdy) < (unsigned)tg.H;
                const int lo2 = ew2 - gdx > ew2 ? ew2 - gdx : ew2;
                mask |= vy2 ? bits(lo2, ew2 - gdx + tg.W) : 0u;
            }
            mask &= bits(0, left);
            mask = colok ? mask : 0u;
            const int pitch2 = tg.C * 2;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                dst[e] = buf_load16(gres, (mask >> e) & 1u ? off + e * pitch2 : kBufNowhere, 0);
        } else {
            int xx = x, yy = y, o = off;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool ok = colok && e < left && (unsigned)(yy + gdy) < (unsigned)tg.H &&
                                (unsigned)(xx + gdx) < (unsigned)tg.W;
                dst[e] = buf_load16(gres, ok ? o : kBufNowhere, 0);
                o += tg.C * 2;
                if (++xx == tg.W) { xx = 0; if (++yy == tg.H) yy = 0; }
            }
        }
    };
    auto fetch = [&](u32x4 (&dst)[8], rsrc_t res, int s, int b) {
        if constexpr (GATHER) load_block_gather(dst, s, b);
        else load_block(dst, res, b);
    };
    auto store_block = [&](const u32x4 (&v)[8], unsigned char* base, int b) {
        // 8 x 8 transpose of 16-bit elements: word i of output column j packs rows 2i, 2i+1
        u32x4 out[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                out[j][i] = __builtin_amdgcn_perm(v[2 * i + 1][j >> 1], v[2 * i][j >> 1],
                                                  (j & 1) ? 0x07060302u : 0x05040100u);
        if (active) {
#pragma unroll
            for (int j = 0; j < 8; ++j) *reinterpret_cast<u32x4*>(base + (loff[j] ^ (b * 64))) = out[j];
        }
    };
    // all D slabs are requested before the first one is waited for
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const rsrc_t res = descriptor(d);
#pragma unroll
        for (int b = 0; b < BPT; ++b) fetch(ring[d][b], res, d, b);
    }
    {
        const rsrc_t res = descriptor(D);
#pragma unroll
        for (int b = 0; b < BPT; ++b) { store_block(ring[0][b], lds, b); fetch(ring[0][b], res, D, b); }
    }
    ring_barrier();                                      // slab 0 is in slot 0
    for (int s0 = 0; s0 < np; s0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int s = s0 + d;
            unsigned char* base = lds + ((s + 1) & 1) * slab_bytes;    // slab s+1; slot s&1 is being read
            const rsrc_t res = descriptor(s + 1 + D);
#pragma unroll
            for (int b = 0; b < BPT; ++b) {
                store_block(ring[(d + 1) % D][b], base, b);
                fetch(ring[(d + 1) % D][b], res, s + 1 + D, b);
                __builtin_amdgcn_sched_barrier(0);
            }
            ring_barrier();
        }
    }
}

template <int R, bool GATHER>
__global__ __launch_bounds__(Tn2<R>::NT) void tn2_bf16_kernel(Tn2Args args) {
    extern __shared__ __align__(1024) unsigned char lds[];
    using C = Tn2<R>;
    constexpr int D = C::D;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // Work-groups are dealt to the eight XCDs round-robin by their linear index, and each XCD has
    // its own L2.  The (split, tile) pairs are numbered split-major and every XCD takes one
    // contiguous eighth of them: the column tiles of one row split land on one XCD (two at most),
    // so the V rows they share are fetched from HBM once, not once per XCD, and every XCD gets the
    // same number of work-groups whatever the split count is.
    const int xcd = (int)blockIdx.x & 7, slot = (int)blockIdx.x >> 3;
    const int pair = xcd * ((int)gridDim.x >> 3) + slot;
    if (pair >= args.tiles * args.splits) return;
    const int tile = pair % args.tiles, split = pair / args.tiles;
    int jid = 0;                                         // the job whose tile range holds this tile
    for (int i = 1; i < args.njobs; ++i)
        if (tile >= args.job[i].tile_begin) jid = i;
    const Tn2Job job = args.job[jid];
    const int p0 = (tile - job.tile_begin) * TP;
    const int64_t k_begin = (int64_t)split * args.rows_per_split;
    int64_t k_end = k_begin + args.rows_per_split;
    if (k_end > args.M) k_end = args.M;
    const int64_t nrows = k_end > k_begin ? k_end - k_begin : 0;
    const int nslab = (int)((nrows + BKM - 1) / BKM);
    const int np = (nslab + D - 1) / D * D;              // trip count of every role, padded to the ring

    if (wave >= NMW + C::NUW) {
        tn_loader<R, C::BPT, D>(job.V, R, R, TP, tid - 64 * (NMW + C::NUW), k_begin, k_end, np, C::slab, lds);
        return;
    }
    if (wave >= NMW) {
        if constexpr (GATHER) {
            if (job.gather) {
                tn_loader<TP, C::BPT, D, true>(job.U, job.P, job.P - p0, 0, tid - 64 * NMW, k_begin, k_end, np, C::slab, lds,
                                               args.g, p0, (args.M / ((int64_t)args.g.RH * args.g.RW)) * args.g.H * args.g.W);
                return;
            }
        }
        tn_loader<TP, C::BPT, D, false, true>(job.U + p0, job.P, job.P - p0, 0, tid - 64 * NMW, k_begin, k_end, np, C::slab, lds);
        return;
    }

    // ====================================================================== MFMA waves
    const int lj = lane & 31, lh = lane >> 5;
    const int wp = (wave / C::WGQ) * (C::PB * 32);
    const int wq = (wave % C::WGQ) * (C::QB * 32);

    f32x16 acc[C::PB][C::QB];
#pragma unroll
    for (int a = 0; a < C::PB; ++a)
#pragma unroll
        for (int b = 0; b < C::QB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // operand addresses inside a slab for k16 = 0; step k16 moves two units on: address ^ (k16 << 5)
    int uad[C::PB], vad[C::QB];
#pragma unroll
    for (int a = 0; a < C::PB; ++a) uad[a] = slab_addr(wp + a * 32 + lj, lh);
#pragma unroll
    for (int b = 0; b < C::QB; ++b) vad[b] = slab_addr(TP + wq + b * 32 + lj, lh);

    ring_barrier();                                      // slab 0 is in slot 0
    for (int s = 0; s < np; ++s) {
        if (s < nslab) {
            const unsigned char* base = lds + (s & 1) * C::slab;
#pragma unroll
            for (int k16 = 0; k16 < BKM / 16; ++k16) {
                // lane (lj, lh) takes rows 16 k16 + 8 lh .. + 7 of column (block column + lj)
                u32x4 uf[C::PB];
#pragma unroll
                for (int a = 0; a < C::PB; ++a)
                    uf[a] = *reinterpret_cast<const u32x4*>(base + (uad[a] ^ (k16 << 5)));
#pragma unroll
                for (int b = 0; b < C::QB; ++b) {
                    const u32x4 vf = *reinterpret_cast<const u32x4*>(base + (vad[b] ^ (k16 << 5)));
#pragma unroll
                    for (int a = 0; a < C::PB; ++a) acc[a][b] = mfma16(uf[a], vf, acc[a][b]);
                }
            }
        }
        ring_barrier();
    }

    // accumulator v of block (a,b): U column p0 + wp + 32a + 8(v/4) + 4 lh + v%4, V column wq + 32b + lj
    float* part = job.part + (int64_t)split * job.P * R;
#pragma unroll
    for (int a = 0; a < C::PB; ++a)
#pragma unroll
        for (int b = 0; b < C::QB; ++b) {
            const int rcol = wq + b * 32 + lj;
            if (job.transposed) {      // part laid out [R, P]: four consecutive P per lane
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int prow = p0 + wp + a * 32 + 8 * g + 4 * lh;
                    if (prow < job.P) {
                        f32x4 o = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                        *reinterpret_cast<f32x4*>(part + (int64_t)rcol * job.P + prow) = o;
                    }
                }
            } else {                   // part laid out [P, R]
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int prow = p0 + wp + a * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (prow < job.P) part[(int64_t)prow * R + rcol] = acc[a][b][v];
                }
            }
        }
}

// out (+)= sum over splits of part[split], element-wise (part already has the layout of out).
struct Red2Job { const float* part; float* out; int64_t total; int block_begin; };
struct Red2Args { Red2Job job[kTnMaxJobs]; int njobs; int splits; int accumulate; };

__global__ __launch_bounds__(256) void tn2_reduce_kernel(Red2Args a) {
    int jid = 0;
    for (int i = 1; i < a.njobs; ++i)
        if ((int)blockIdx.x >= a.job[i].block_begin) jid = i;
    const Red2Job j = a.job[jid];
    const int64_t idx = ((int64_t)((int)blockIdx.x - j.block_begin) * 256 + threadIdx.x) * 4;
    if (idx >= j.total) return;   // totals are multiples of 4 (R % 32 == 0)
    f32x4 sum = *reinterpret_cast<const f32x4*>(j.part + idx);
    for (int s = 1; s < a.splits; ++s) sum += *reinterpret_cast<const f32x4*>(j.part + (int64_t)s * j.total + idx);
    if (a.accumulate) sum += *reinterpret_cast<const f32x4*>(j.out + idx);
    *reinterpret_cast<f32x4*>(j.out + idx) = sum;
}

int tn2_total_tiles(const TnJob* jobs, int njobs) {
    int tiles = 0;
    for (int i = 0; i < njobs; ++i) tiles += (jobs[i].P + TP - 1) / TP;
    return tiles;
}

int tn2_choose_splits(int64_t M, int total_tiles) {
    // one 8-wave work-group per compute unit and every work-group writes one fp32 partial tile:
    // aim at one full round of the 256 compute units, at least 8 slabs each
    int64_t want = 256 / total_tiles;
    int64_t max_by_rows = M / (8 * 64);
    if (max_by_rows < 1) max_by_rows = 1;
    if (want > max_by_rows) want = max_by_rows;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    return (int)want;
}

template <int R, bool GATHER>
hipError_t launch_tn2_r(const Tn2Args& args, int tiles, int splits, hipStream_t s) {
    constexpr int lds_bytes = Tn2<R>::lds_bytes;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tn2_bf16_kernel<R, GATHER>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((tn2_bf16_kernel<R, GATHER>), dim3(8 * ((tiles * splits + 7) / 8)), dim3(Tn2<R>::NT), lds_bytes, s, args);
    return hipGetLastError();
}

}  // namespace

size_t tn_partials_bytes(int64_t M, const TnJob* jobs, int njobs, int R) {
    const int splits = tn2_choose_splits(M, tn2_total_tiles(jobs, njobs));
    size_t elems = 0;
    for (int i = 0; i < njobs; ++i) elems += (size_t)jobs[i].P * R;
    return elems * splits * sizeof(float);
}

namespace {
// gather != NULL: the LAST job's U is gathered from an image, any job before it is plain
hipError_t launch_tn_common(const TnJob* jobs, int njobs, int64_t M, int R, int accumulate,
                            float* partials, const Tn2Gather* gather, hipStream_t s) {
    if (njobs < 1 || njobs > kTnMaxJobs || (gather && njobs > 2)) return hipErrorInvalidValue;
    const int tiles = tn2_total_tiles(jobs, njobs);
    const int splits = tn2_choose_splits(M, tiles);
    Tn2Args args{};
    Red2Args red{};
    args.njobs = red.njobs = njobs;
    args.tiles = tiles; args.splits = splits;
    args.M = M;
    if (gather) args.g = *gather;
    int64_t rps = ceil_div(M, splits);
    rps = ceil_div(rps, 64) * 64;
    args.rows_per_split = rps;
    red.splits = splits; red.accumulate = accumulate;
    float* part = partials;
    int tile_begin = 0, red_blocks = 0;
    for (int i = 0; i < njobs; ++i) {
        args.job[i].U = (const uint16_t*)jobs[i].U;
        args.job[i].V = (const uint16_t*)jobs[i].V;
        args.job[i].part = part;
        args.job[i].P = jobs[i].P;
        args.job[i].tile_begin = tile_begin;
        args.job[i].transposed = jobs[i].transposed;
        args.job[i].gather = (gather && i == njobs - 1) ? 1 : 0;
        red.job[i].part = part;
        red.job[i].out = jobs[i].out;
        red.job[i].total = (int64_t)jobs[i].P * R;
        tile_begin += (jobs[i].P + TP - 1) / TP;
        red.job[i].block_begin = red_blocks;
        red_blocks += (int)ceil_div((int64_t)jobs[i].P * R / 4, 256);
        part += (size_t)jobs[i].P * R * splits;
    }
    hipError_t e;
    switch (R) {
#define ABT_CASE(RR) case RR: e = gather ? launch_tn2_r<RR, true>(args, tiles, splits, s) \
                                         : launch_tn2_r<RR, false>(args, tiles, splits, s); break;
        ABT_CASE(32) ABT_CASE(64) ABT_CASE(96) ABT_CASE(128) ABT_CASE(160) ABT_CASE(192)
        ABT_CASE(224) ABT_CASE(256) ABT_CASE(288) ABT_CASE(320) ABT_CASE(352) ABT_CASE(384)
#undef ABT_CASE
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tn2_reduce_kernel, dim3(red_blocks), dim3(256), 0, s, red);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_tn_bf16(const TnJob* jobs, int njobs, int64_t M, int R, int accumulate,
                          float* partials, hipStream_t s) {
    return launch_tn_common(jobs, njobs, M, R, accumulate, partials, nullptr, s);
}

hipError_t launch_tn_gather_bf16(const TnJob* jobs, int njobs, const PatchGeom& g, int64_t M, int R, int accumulate,
                                 float* partials, hipStream_t s) {
    // patches only (no adjoint form here); 32-bit offsets inside the window of the image that one
    // slab's patches touch
    if (njobs < 1 || njobs > 2 ||
        g.H < 1 || g.W < 1 || g.Cin < 8 || g.Cin % 8 || g.kh < 1 || g.kw < 1 || !(g.kh & 1) || !(g.kw & 1) ||
        g.sign != 1 || g.shift != 0 || (g.mul != 1 && g.mul != 2) || g.RH < 1 || g.RW < 1 ||
        (g.mul == 1 && (g.RH != g.H || g.RW != g.W)) ||
        M % ((int64_t)g.RH * g.RW) != 0 || (M / ((int64_t)g.RH * g.RW)) * g.H * g.W > 0x7fffffff ||
        jobs[njobs - 1].P != g.kh * g.kw * g.Cin ||
        ((int64_t)64 + 2 * ((g.kh / 2) * (int64_t)g.W + g.kw / 2)) * g.Cin * 2 >= kBufMaxBytes)
        return hipErrorInvalidValue;
    // one descriptor per row split: its window of the image (the centres of the split's rows, the
    // reach of the window on both sides, the padded slabs of the loaders' ring) must stay below 2 GiB
    {
        const int splits = tn2_choose_splits(M, tn2_total_tiles(jobs, njobs));
        const int64_t rps = ceil_div(ceil_div(M, splits), 64) * 64;
        const int64_t reach = (g.kh / 2) * (int64_t)g.W + g.kw / 2;
        const int64_t span = (int64_t)g.mul * g.mul * (rps + 64 * 8 + g.RW + 2) + 2 * (int64_t)g.mul * g.W;
        if ((span + 2 * reach) * g.Cin * 2 >= kBufMaxBytes) return hipErrorInvalidValue;
    }
    const Tn2Gather tg{g.H, g.W, g.Cin, g.kh, g.kw, g.RH, g.RW, g.mul};
    return launch_tn_common(jobs, njobs, M, R, accumulate, partials, &tg, s);
}

}  // namespace abt
