// Factor gradients of the factored layer (bf16 in, fp32 out):
//     dA[m,R] = dY[M,m]^T . T[M,R]          dB[R,n] = dT[M,R]^T . X[M,n]
// Both are contractions over the M batch rows, the slow dimension of every operand.  One generic
// job:  part[split][P,R] = U[rows of split, P]^T . V[rows of split, R]   (dA: U = dY, V = T;
// dB: U = X, V = dT, result stored transposed), followed by a fixed-order sum over the splits.
//
// Work-group: 128 columns of U x all R columns of V over one split of the batch rows; 8 waves in
// two roles.  Four loader waves move slabs of 64 batch rows (32 for R > 256) global -> register
// ring (two slabs in flight) -> LDS exactly as they lie in memory (batch row major), two LDS slots,
// one barrier per slab.  Four MFMA waves (2 x 2, or 4 x 1 when R/32 is odd) each own a block of the
// output tile.  The MFMA operands, which need 8 consecutive batch rows per lane, are read with the
// transposing LDS load of gfx950 (ds_read_b64_tr_b16): in every group of 16 lanes, lane s supplies
// the address of 4 consecutive columns of batch row k0 + s/4 (columns 4 (s%4) ..), and lane l
// receives column l of the four rows k0 .. k0+3.
// LDS rows are a multiple of 256 bytes; their 64-byte units are XOR-swizzled with the low two bits
// of the row, so the four rows one transposing load touches lie in different banks.
#include "common.h"

namespace abt {

namespace {

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((ext_vector_type(4))) short s16x4;

__device__ __forceinline__ void ring_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ f32x16 mfma16(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
// transposing LDS read: 4 x b16 for this lane (see the header comment)
__device__ __forceinline__ u32x2 ds_tr(const unsigned char* p) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds_void*)p);
    return __builtin_bit_cast(u32x2, v);
}

constexpr int TP = 128;      // U columns per work-group
constexpr int UPITCH = TP * 2;
constexpr int NMT = 256, NLT = 256, NT = NMT + NLT;   // MFMA threads, loader threads

template <int R>
struct Tn2 {
    static constexpr int RB = R / 32;
    static constexpr bool even = (RB % 2) == 0;
    static constexpr int WGP = even ? 2 : 4, WGQ = even ? 2 : 1;
    static constexpr int PB = even ? 2 : 1, QB = even ? RB / 2 : RB;
    static constexpr int RP = (R + 127) / 128 * 128;        // padded V columns in LDS
    static constexpr int VPITCH = RP * 2;
    static constexpr int BKM = R <= 256 ? 64 : 32;          // batch rows per slab
    static constexpr int slab = BKM * (UPITCH + VPITCH);
    static constexpr int lds_bytes = 2 * slab;
    static constexpr int NU = BKM * (TP / 8) / NLT;          // 16-byte chunks per loader thread, U part
    static constexpr int NV = (BKM * (R / 8) + NLT - 1) / NLT;   // V part (the last one may be partial)
    static constexpr bool v_exact = BKM * (R / 8) % NLT == 0;
    static constexpr int D = 2;                              // slabs in flight in the loaders' register ring
    static_assert(lds_bytes <= 160 * 1024, "slab shape");
};

struct Tn2Job { const uint16_t* U; const uint16_t* V; float* part; int P; int tile_begin; int transposed; };
struct Tn2Args { Tn2Job job[2]; int njobs; int64_t M; int64_t rows_per_split; };

template <int R>
__global__ __launch_bounds__(NT) void tn2_bf16_kernel(Tn2Args args) {
    extern __shared__ __align__(1024) unsigned char lds[];
    using C = Tn2<R>;
    constexpr int BKM = C::BKM, D = C::D;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    const int jid = (args.njobs > 1 && (int)blockIdx.x >= args.job[1].tile_begin) ? 1 : 0;
    const Tn2Job job = args.job[jid];
    const int p0 = ((int)blockIdx.x - job.tile_begin) * TP;
    const int64_t k_begin = (int64_t)blockIdx.y * args.rows_per_split;
    int64_t k_end = k_begin + args.rows_per_split;
    if (k_end > args.M) k_end = args.M;
    const int64_t nrows = k_end > k_begin ? k_end - k_begin : 0;
    const int nslab = (int)((nrows + BKM - 1) / BKM);
    const int np = (nslab + D - 1) / D * D;              // trip count of both roles, padded to the ring

    if (wave >= NMT / 64) {
        // ================================================================== loader waves
        // Slabs go global -> register ring -> LDS exactly as they lie in memory.  Buffer loads: the
        // row offset is part of the per-lane offset, the only part the hardware range-checks, and
        // the descriptors (rebuilt per slab, scalar work) end at the split's last row, so rows past
        // it load zeros; a chunk in a column past P gets an offset that no descriptor covers.
        const int lt = tid - NMT;
        int uoff[C::NU], usrc[C::NU];
#pragma unroll
        for (int e = 0; e < C::NU; ++e) {
            const int ci = e * NLT + lt;
            const int row = ci / (TP / 8), ch = ci % (TP / 8);
            uoff[e] = row * UPITCH + ((((ch >> 2) ^ (row & 3)) << 2) | (ch & 3)) * 16;
            usrc[e] = p0 + ch * 8 < job.P ? (row * job.P + ch * 8) * 2 : kBufNowhere;
        }
        int voff[C::NV], vsrc[C::NV];
        bool vok[C::NV];
#pragma unroll
        for (int e = 0; e < C::NV; ++e) {
            const int ci = e * NLT + lt;
            const int row = ci / (R / 8), ch = ci % (R / 8);
            vok[e] = C::v_exact || ci < BKM * (R / 8);
            voff[e] = BKM * UPITCH + row * C::VPITCH + ((((ch >> 2) ^ (row & 3)) << 2) | (ch & 3)) * 16;
            vsrc[e] = vok[e] ? (row * R + ch * 8) * 2 : kBufNowhere;
        }
        u32x4 ring[D][C::NU + C::NV];
        auto load = [&](u32x4 (&dst)[C::NU + C::NV], int s) {
            const int64_t kr0 = k_begin + (int64_t)s * BKM;
            const int64_t left = k_end - kr0;                    // <= 0 past the split: everything reads zeros
            const rsrc_t ures = make_rsrc(job.U + kr0 * job.P + p0, (left * job.P - p0) * 2);
            const rsrc_t vres = make_rsrc(job.V + kr0 * R, left * R * 2);
#pragma unroll
            for (int e = 0; e < C::NU; ++e) dst[e] = buf_load16(ures, usrc[e], 0);
#pragma unroll
            for (int e = 0; e < C::NV; ++e) dst[C::NU + e] = buf_load16(vres, vsrc[e], 0);
        };
        // steady state: chunk e of slab s+1 goes to LDS (slot s&1 is being read) and the same chunk
        // of slab s+1+D is requested, alternating, so LDS port and address path work side by side
        auto step = [&](u32x4 (&rg)[C::NU + C::NV], int s) {
            unsigned char* base = lds + ((s + 1) & 1) * C::slab;
            const int64_t kr0 = k_begin + (int64_t)(s + 1 + D) * BKM;
            const int64_t left = k_end - kr0;
            const rsrc_t ures = make_rsrc(job.U + kr0 * job.P + p0, (left * job.P - p0) * 2);
            const rsrc_t vres = make_rsrc(job.V + kr0 * R, left * R * 2);
#pragma unroll
            for (int e = 0; e < C::NU; ++e) {
                *reinterpret_cast<u32x4*>(base + uoff[e]) = rg[e];
                rg[e] = buf_load16(ures, usrc[e], 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int e = 0; e < C::NV; ++e) {
                if (vok[e]) *reinterpret_cast<u32x4*>(base + voff[e]) = rg[C::NU + e];
                rg[C::NU + e] = buf_load16(vres, vsrc[e], 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        load(ring[0], 0);
#pragma unroll
        for (int e = 0; e < C::NU; ++e) *reinterpret_cast<u32x4*>(lds + uoff[e]) = ring[0][e];
#pragma unroll
        for (int e = 0; e < C::NV; ++e)
            if (vok[e]) *reinterpret_cast<u32x4*>(lds + voff[e]) = ring[0][C::NU + e];
#pragma unroll
        for (int d = 1; d <= D; ++d) load(ring[d % D], d);
        ring_barrier();                                  // slab 0 is in slot 0
        for (int s0 = 0; s0 < np; s0 += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                step(ring[(d + 1) % D], s0 + d);
                ring_barrier();
            }
        }
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

    // per lane: group g = lane / 16 selects (column half, row half); s = lane % 16
    const int ls = lane & 15, lg = lane >> 4;
    const int tr_row = 8 * (lg >> 1) + (ls >> 2);        // + 16 k16 + 4 rd
    const int tr_col = 16 * (lg & 1) + 4 * (ls & 3);     // + block column

    ring_barrier();                                      // slab 0 is in slot 0
    for (int s = 0; s < np; ++s) {
        if (s < nslab) {
            const unsigned char* ub = lds + (s & 1) * C::slab;
            const unsigned char* vb = ub + BKM * UPITCH;
#pragma unroll
            for (int k16 = 0; k16 < BKM / 16; ++k16) {
                u32x4 uf[C::PB], vf[C::QB];
                const int row = 16 * k16 + tr_row, row1 = row + 4;
#pragma unroll
                for (int a = 0; a < C::PB; ++a) {
                    const int col = wp + a * 32 + tr_col;
                    const u32x2 r0 = ds_tr(ub + row * UPITCH + (((col >> 5) ^ (row & 3)) << 6) + (col & 31) * 2);
                    const u32x2 r1 = ds_tr(ub + row1 * UPITCH + (((col >> 5) ^ (row1 & 3)) << 6) + (col & 31) * 2);
                    uf[a] = u32x4{r0[0], r0[1], r1[0], r1[1]};
                }
#pragma unroll
                for (int b = 0; b < C::QB; ++b) {
                    const int col = wq + b * 32 + tr_col;
                    const u32x2 r0 = ds_tr(vb + row * C::VPITCH + ((((col >> 5) & ~3) | (((col >> 5) & 3) ^ (row & 3))) << 6) + (col & 31) * 2);
                    const u32x2 r1 = ds_tr(vb + row1 * C::VPITCH + ((((col >> 5) & ~3) | (((col >> 5) & 3) ^ (row1 & 3))) << 6) + (col & 31) * 2);
                    vf[b] = u32x4{r0[0], r0[1], r1[0], r1[1]};
                }
#pragma unroll
                for (int a = 0; a < C::PB; ++a)
#pragma unroll
                    for (int b = 0; b < C::QB; ++b) acc[a][b] = mfma16(uf[a], vf[b], acc[a][b]);
            }
        }
        ring_barrier();
    }

    // accumulator v of block (a,b): U column p0 + wp + 32a + 8(v/4) + 4 lh + v%4, V column wq + 32b + lj
    float* part = job.part + (int64_t)blockIdx.y * job.P * R;
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
struct Red2Job { const float* part; float* out; int64_t total; };
struct Red2Args { Red2Job job[2]; int njobs; int splits; int accumulate; int blocks0; };

__global__ __launch_bounds__(256) void tn2_reduce_kernel(Red2Args a) {
    const int jid = (a.njobs > 1 && (int)blockIdx.x >= a.blocks0) ? 1 : 0;
    const Red2Job j = a.job[jid];
    const int64_t idx = ((int64_t)((int)blockIdx.x - (jid ? a.blocks0 : 0)) * 256 + threadIdx.x) * 4;
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

template <int R>
hipError_t launch_tn2_r(const Tn2Args& args, int tiles, int splits, hipStream_t s) {
    constexpr int lds_bytes = Tn2<R>::lds_bytes;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tn2_bf16_kernel<R>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(tn2_bf16_kernel<R>, dim3(tiles, splits), dim3(NT), lds_bytes, s, args);
    return hipGetLastError();
}

}  // namespace

size_t tn_partials_bytes(int64_t M, const TnJob* jobs, int njobs, int R) {
    const int splits = tn2_choose_splits(M, tn2_total_tiles(jobs, njobs));
    size_t elems = 0;
    for (int i = 0; i < njobs; ++i) elems += (size_t)jobs[i].P * R;
    return elems * splits * sizeof(float);
}

hipError_t launch_tn_bf16(const TnJob* jobs, int njobs, int64_t M, int R, int accumulate,
                          float* partials, hipStream_t s) {
    if (njobs < 1 || njobs > 2) return hipErrorInvalidValue;
    const int tiles = tn2_total_tiles(jobs, njobs);
    const int splits = tn2_choose_splits(M, tiles);
    Tn2Args args{};
    Red2Args red{};
    args.njobs = red.njobs = njobs;
    args.M = M;
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
        red.job[i].part = part;
        red.job[i].out = jobs[i].out;
        red.job[i].total = (int64_t)jobs[i].P * R;
        tile_begin += (jobs[i].P + TP - 1) / TP;
        const int blocks = (int)ceil_div((int64_t)jobs[i].P * R / 4, 256);
        if (i == 0) red.blocks0 = blocks;
        red_blocks += blocks;
        part += (size_t)jobs[i].P * R * splits;
    }
    hipError_t e;
    switch (R) {
#define ABT_CASE(RR) case RR: e = launch_tn2_r<RR>(args, tiles, splits, s); break;
        ABT_CASE(32) ABT_CASE(64) ABT_CASE(96) ABT_CASE(128) ABT_CASE(160) ABT_CASE(192)
        ABT_CASE(224) ABT_CASE(256) ABT_CASE(288) ABT_CASE(320) ABT_CASE(352) ABT_CASE(384)
#undef ABT_CASE
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tn2_reduce_kernel, dim3(red_blocks), dim3(256), 0, s, red);
    return hipGetLastError();
}

}  // namespace abt
