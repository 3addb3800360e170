// Pieces shared by the MFMA GEMM kernels: operand fragment types, the block -> tile mapping and the epilogues.
#pragma once
#include "fg_common.h"

namespace fg {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

union Frag {
    uint4 u;
    bf16x8_t b;
    f16x8_t h;
};

template <typename T> __device__ __forceinline__ f32x16_t mfma32(const Frag &a, const Frag &b, f32x16_t c);
template <> __device__ __forceinline__ f32x16_t mfma32<bf16_t>(const Frag &a, const Frag &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.b, b.b, c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16_t mfma32<f16_t>(const Frag &a, const Frag &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a.h, b.h, c, 0, 0, 0);
}

constexpr int KT = 4;  // k tiles (of 16) per chunk: 64 k

// Block -> (column band bx, row block by, k split bz); false when the block has no tile.  With several row
// blocks the grid is one-dimensional and XCD-aware: blocks are dealt to the 8 XCDs round-robin by linear id, so
// XCD x takes the units g * 8 + x (a unit = one k split of a group of BG adjacent bands) and runs the
// row_blocks x BG tiles of a unit back to back.  The ~32 blocks resident on an XCD then share BG bands of W and
// the row blocks of X through its L2.  raster = BG, or 0 for a plain three-dimensional grid.
__device__ __forceinline__ bool map_block(int raster, int n_tiles, int tiles_per_band, int k_tiles, int chunks_per_split,
                                          int row_blocks, int &bx, int &by, int &bz)
{
    if (!raster) {
        bx = blockIdx.x; by = blockIdx.y; bz = blockIdx.z;
        return true;
    }
    const int BG = raster;
    const int n_bands = (n_tiles + tiles_per_band - 1) / tiles_per_band;
    const int n_bgroups = (n_bands + BG - 1) / BG;
    const int splits = (k_tiles / KT + chunks_per_split - 1) / chunks_per_split;
    const int per_group = row_blocks * BG;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int unit = (local / per_group) * 8 + xcd, within = local % per_group;   // unit = (k split, band group)
    if (unit >= n_bgroups * splits) return false;
    bz = unit / n_bgroups;
    by = within % row_blocks;
    bx = (unit % n_bgroups) * BG + within / row_blocks;
    return bx < n_bands;
}

// Epilogue of one wave's MT x NT tiles whose first row is wave_row0 and first tile column ntile0.
// EPI 0: fp32 partial slab bz.  EPI 1: gate / up tiles alternate and SwiGLU(gate) * up is stored as T.
// A lane holds column lane % 32 of each tile and rows 8 * (r / 4) + 4 * (lane / 32) + r % 4.  The stores go through a
// buffer descriptor that begins at the wave's first row and ends with the matrix (or with the wave's rows, whichever
// comes first): a store past the last row is dropped by the address check of the hardware, so the code is one
// straight line of independent (value, store) pairs with 32-bit offsets -- with a comparison and a branch per element
// the compiler kept them in order, and the exposed epilogue of a 256-row tile cost 11 % of the gate/up GEMM.
template <typename T, int MT, int NT, int EPI>
__device__ __forceinline__ void store_tiles(f32x16_t (&acc)[MT][NT], void *__restrict__ out, int M, int N, int wave_row0,
                                            int ntile0, int n_tiles, int bz, int lane)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-descriptor builtins exist in the device pass only
    const int col = lane & 31, rh = (lane >> 5) * 4;
    const int rows = min(M - wave_row0, 32 * MT);
    if (rows <= 0) return;
    if (EPI == 0) {
        float *base = reinterpret_cast<float *>(out) + ((size_t)bz * M + wave_row0) * N;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(base, 0, rows * N * 4, 0x00020000);
#pragma unroll
        for (int j = 0; j < NT; j++) {
            const int nt = ntile0 + j;
            if (nt >= n_tiles) continue;
            const int off0 = (rh * N + nt * 32 + col) * 4;
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int r = 0; r < 16; r++)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][r]), rs,
                                                          off0 + (i * 32 + 8 * (r >> 2) + (r & 3)) * N * 4, 0, 0);
        }
    } else {
        // gate / up tiles alternate: tile 2t = gate, 2t + 1 = up, both for output columns 32 t .. 32 t + 31
        const int F = N >> 1;
        T *base = reinterpret_cast<T *>(out) + (size_t)wave_row0 * F;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(base, 0, rows * F * 2, 0x00020000);
#pragma unroll
        for (int j = 0; j + 1 < NT; j += 2) {
            const int nt = ntile0 + j;
            if (nt + 1 >= n_tiles) continue;  // n_tiles is even and pairs start at even tiles
            const int off0 = (rh * F + (nt >> 1) * 32 + col) * 2;
            // four elements at a time, step by step (the operations of swiglu_f in its order): a wave issues in order, and
            // written element by element each exponential and reciprocal is waited for by the instruction behind it
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    float e[4];
#pragma unroll
                    for (int k = 0; k < 4; k++) e[k] = __expf(-acc[i][j][4 * q + k]);
#pragma unroll
                    for (int k = 0; k < 4; k++) e[k] = __builtin_amdgcn_rcpf(1.f + e[k]);
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        const T v = from_f<T>(acc[i][j][4 * q + k] * e[k] * acc[i][j + 1][4 * q + k]);
                        __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, v), rs,
                                                              off0 + (i * 32 + 8 * q + k) * F * 2, 0, 0);
                    }
                }
        }
    }
#endif
}

}  // namespace fg
