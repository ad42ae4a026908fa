// fp32 GEMM on the fp32 matrix cores of gfx950 (v_mfma_f32_32x32x2_f32), grouped over a list of
// independent problems.  Serves the fp32 flavour of the factored layer (all six products of the
// forward and backward) and the merge's back-projections A' = Abar P_A, B' = P_B Bbar, Wbar = Abar Bbar.
//
// Work-group: 256 threads = 4 waves in a 2 x 2 grid, output tile 128 x 128, each wave 64 x 64
// (2 x 2 MFMA blocks, 64 accumulator registers).  K is consumed in slabs of 16 staged through
// LDS in k-major order, so one lane's MFMA operand is a single 4-byte LDS read.
//
// MFMA 32x32x2 f32 register layout (lane l of 64): A operand = A[l % 32][l / 32],
// B operand = B[l / 32][l % 32], accumulator register v holds C[8*(v/4) + 4*(l/32) + v%4][l % 32].
#include "common.h"

namespace abt {

namespace {

constexpr int TILE = 128;
constexpr int SLAB = 16;
constexpr int PITCH = 132;  // floats per k-row in LDS; 132 = 4 mod 64 spreads a 16 x 4 patch over all banks

struct GemmF32Dev {
    GemmF32 d;
    int tile_begin;
    int tiles_q;
};

// Unpredicated load (indices clamped into the matrix; `ok` tells whether the element exists): a
// predicated one would have to be waited for before the next load is issued.
__device__ __forceinline__ float fetch(const float* base, int row, int col, int ld, int rows, int cols, bool& ok) {
    ok = row < rows && col < cols;
    const int r = row < rows ? row : rows - 1, c = col < cols ? col : cols - 1;
    return gload(base + (int64_t)r * ld + c);
}

__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmF32Dev* __restrict__ descs, int ndesc,
                                                       GemmF32Dev single, int use_single, int ntiles) {
    __shared__ float As2[2][SLAB * PITCH];
    __shared__ float Bs2[2][SLAB * PITCH];

    // Tiles are numbered problem by problem; block b works on tile (b % 8) * (grid / 8) + b / 8, so each
    // XCD (block index modulo 8) gets a contiguous eighth of the list and the tiles of one problem
    // share their operand panels through one L2.  The grid is the tile count rounded up to 8.
    const int tile = (int)(blockIdx.x & 7) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3);
    if (tile >= ntiles) return;
    GemmF32Dev g;
    if (use_single) {
        g = single;
    } else {
        int lo = 0, hi = ndesc - 1;
        while (lo < hi) {  // last descriptor whose tile_begin <= tile
            int mid = (lo + hi + 1) >> 1;
            if (descs[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
        }
        g = descs[lo];
    }
    const GemmF32& d = g.d;
    const int local = tile - g.tile_begin;
    const int i0 = (local / g.tiles_q) * TILE;
    const int j0 = (local % g.tiles_q) * TILE;

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wi = (wave >> 1) * 64, wj = (wave & 1) * 64;

    // Output columns (or rows) at or beyond *limit are defined to be zero: skip the arithmetic.
    int lim = d.limit ? *d.limit : (d.limit_rows ? d.P : d.Q);
    const bool dead = d.limit && (d.limit_rows ? (i0 >= lim) : (j0 >= lim));

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    if (!dead) {
        float ra[8], rb[8];
        bool oka[8], okb[8];
        auto load_slab = [&](int k0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int lin = e * 256 + t;
                if (d.transA) {  // A stored [K, P]
                    const int k = lin >> 7, i = lin & 127;
                    ra[e] = fetch(d.A, k0 + k, i0 + i, d.lda, d.K, d.P, oka[e]);
                } else {         // A stored [P, K]
                    const int i = lin >> 4, k = lin & 15;
                    ra[e] = fetch(d.A, i0 + i, k0 + k, d.lda, d.P, d.K, oka[e]);
                }
                if (d.transB) {  // B stored [Q, K]
                    const int j = lin >> 4, k = lin & 15;
                    rb[e] = fetch(d.B, j0 + j, k0 + k, d.ldb, d.Q, d.K, okb[e]);
                } else {         // B stored [K, Q]
                    const int k = lin >> 7, j = lin & 127;
                    rb[e] = fetch(d.B, k0 + k, j0 + j, d.ldb, d.K, d.Q, okb[e]);
                }
            }
        };
        auto store_slab = [&](int buf) {
            float* As = As2[buf];
            float* Bs = Bs2[buf];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int lin = e * 256 + t;
                const float va = oka[e] ? ra[e] : 0.0f, vb = okb[e] ? rb[e] : 0.0f;
                if (d.transA) As[(lin >> 7) * PITCH + (lin & 127)] = va;
                else          As[(lin & 15) * PITCH + (lin >> 4)] = va;
                if (d.transB) Bs[(lin & 15) * PITCH + (lin >> 4)] = vb;
                else          Bs[(lin >> 7) * PITCH + (lin & 127)] = vb;
            }
        };

        // two LDS buffers, one barrier per slab: while slab s is multiplied out of buffer s % 2, slab
        // s + 1 (in registers since the iteration before) goes to the other buffer and the loads of
        // slab s + 2 are issued, so a load has two slabs of products to arrive
        const int nslab = (d.K + SLAB - 1) / SLAB;
        load_slab(0);
        store_slab(0);
        if (nslab > 1) load_slab(SLAB);
        __syncthreads();
        for (int s = 0; s < nslab; ++s) {
            const float* As = As2[s & 1];
            const float* Bs = Bs2[s & 1];
            if (s + 1 < nslab) {
                store_slab((s & 1) ^ 1);                  // everybody left that buffer before the last barrier
                if (s + 2 < nslab) load_slab((s + 2) * SLAB);
            }
            const int li = lane & 31, lk = lane >> 5;
#pragma unroll
            for (int kk = 0; kk < SLAB; kk += 2) {
                float a0 = As[(kk + lk) * PITCH + wi + li];
                float a1 = As[(kk + lk) * PITCH + wi + 32 + li];
                float b0 = Bs[(kk + lk) * PITCH + wj + li];
                float b1 = Bs[(kk + lk) * PITCH + wj + 32 + li];
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            }
            __syncthreads();
        }
    }

    const int lj = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wi + a * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                const int col = j0 + wj + b * 32 + lj;
                if (row < d.P && col < d.Q) {
                    float* c = d.C + (int64_t)row * d.ldc + col;
                    const bool zero = d.limit && (d.limit_rows ? (row >= lim) : (col >= lim));
                    float val = zero ? 0.0f : d.alpha * acc[a][b][v];
                    if (d.accumulate && !zero) val += *c;
                    *c = val;
                }
            }
}

}  // namespace

hipError_t launch_gemm_f32_one(const GemmF32& d, hipStream_t s) {
    GemmF32Dev g;
    g.d = d;
    g.tile_begin = 0;
    g.tiles_q = (d.Q + TILE - 1) / TILE;
    const int tiles = ((d.P + TILE - 1) / TILE) * g.tiles_q;
    if (tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((tiles + 7) / 8 * 8), dim3(256), 0, s, nullptr, 0, g, 1, tiles);
    return hipGetLastError();
}

// Grouped launch in two steps so the caller can batch the upload with its other tables:
// gemm_f32_build_table fills `host_image` (n * gemm_f32_desc_bytes() bytes) and returns the tile
// count; after the caller has copied the image to device memory, launch_gemm_f32_table runs it.
size_t gemm_f32_desc_bytes() { return sizeof(GemmF32Dev); }

int gemm_f32_build_table(const GemmF32* descs_host, int n, void* host_image) {
    GemmF32Dev* tmp = static_cast<GemmF32Dev*>(host_image);
    int tiles = 0;
    for (int i = 0; i < n; ++i) {
        tmp[i].d = descs_host[i];
        tmp[i].tile_begin = tiles;
        tmp[i].tiles_q = (descs_host[i].Q + TILE - 1) / TILE;
        tiles += ((descs_host[i].P + TILE - 1) / TILE) * tmp[i].tiles_q;
    }
    return tiles;
}

hipError_t launch_gemm_f32_table(const void* dev_image, int n, int tiles, hipStream_t s) {
    if (n <= 0 || tiles <= 0) return hipSuccess;
    GemmF32Dev none{};
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((tiles + 7) / 8 * 8), dim3(256), 0, s,
                       (const GemmF32Dev*)dev_image, n, none, 0, tiles);
    return hipGetLastError();
}

}  // namespace abt
