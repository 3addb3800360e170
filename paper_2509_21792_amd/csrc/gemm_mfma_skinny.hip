// Few-row shape of the 16-bit MFMA GEMM: out = X . W^T for up to 128 rows per block, bound by the HBM traffic of W
// (short-k shapes of up to 256 rows take two row blocks).
//
// A block owns 64 output columns (two 32-column bands of the packed W) and up to four 32-row tiles; its four waves
// split the contraction *inside* the block: of every 64-wide k chunk, wave w takes k tile w (16 wide).  Four waves
// side by side over 256 columns need a k split across blocks to fill the chip, and every such split is a slab of
// M x N fp32 written here and read back by the consumer; the split inside the block gives the same number of
// independent W streams with a quarter of the slabs -- none at all for the wide matrices (gate/up, LM head),
// so gate/up applies SwiGLU in its own epilogue and needs no separate pass.
//
// Each wave streams its W fragments straight from HBM in 1 KiB coalesced non-temporal loads, SK_DEPTH chunks
// ahead in a ring of register sets.  X (L2 resident) is staged through LDS in MFMA fragment order as in the
// streaming kernel, coalesced, one barrier per chunk; its global loads ride in the same ring, SK_DEPTH chunks
// ahead: the load counter retires in issue order, so an X load waited on any earlier would also wait for every W
// load issued before it and flatten the ring.  At the end the four partial accumulators meet in LDS, tile by tile:
//   EPI 0  fp32 partial slab of the block's k split (narrow outputs still want a few splits across blocks),
//   EPI 1  W is the gate/up interleaved matrix: silu(gate) * up, stored as T.
// Measured alternatives on the 7B-class gate/up at 8 rows (46.2 us as built): four bands per block 54.7 us (too few
// blocks), a ring of eight chunks 47.3 us (no gain, and two row tiles then spill); four bands per block for the narrow
// outputs at 64 rows (half the X staged per byte of W): QKV 11.8 against 11.0 us, O 10.7 against 9.8, down 29.4 against 28.8.  Three and four row tiles (65 - 128
// rows) need 208 - 256 registers: two blocks per CU, which is enough for the narrow outputs' grids of at most 256
// blocks.
#include "fg_common.h"
#include "gemm_mfma.h"

namespace fg {

typedef uint32_t sk_u32x4_t __attribute__((ext_vector_type(4)));
typedef float sk_f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 sk_load_stream(const uint4 *p)
{
    const sk_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const sk_u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int SK_DEPTH = 4;   // chunks in flight per wave (even: the LDS buffer of a chunk is its ring slot & 1)
constexpr int SK_NT = 2;      // 32-column bands per block

template <typename T, int MT, int EPI, int NT, int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(MT == 1 ? 4 : (MT == 2 ? 3 : 1)))) void gemm_mfma_skinny_kernel(const T *__restrict__ X, const uint4 *__restrict__ Wp,
                                                                void *__restrict__ out, int M, int N, int K, int chunks_per_split,
                                                                int row_blocks, int col_blocks, int splits)
{
    constexpr int BM = MT * 32;
    constexpr int XLOADS = BM * 8 / 256;   // 16-byte pieces of X per thread per chunk
    static_assert(BM * 8 % 256 == 0, "X staging must divide evenly");
    constexpr int XS = 2 * MT * KT * 64;                    // uint4 entries of the X double buffer
    constexpr int RED = 4 * NT * 1024 / 4;                  // uint4 entries of the reduction buffer (4 waves x NT tiles)
    __shared__ uint4 smem[XS > RED ? XS : RED];
    uint4 *xs = smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_tiles = N >> 5, k_tiles = K >> 4;
    // Block -> (column block, k split, row block).  Workgroups are dealt to the 8 XCDs round-robin by linear id: the
    // row blocks of one (column block, k split) unit get ids that differ by multiples of 8, so they run on the same
    // XCD at about the same time and the unit's W is fetched from HBM once (the other row blocks hit in that L2).
    const int grp8 = blockIdx.x / (8 * row_blocks), within = blockIdx.x % (8 * row_blocks);
    const int unit = grp8 * 8 + (within & 7), rb = within >> 3;
    if (unit >= col_blocks * splits) return;
    const int ntile0 = (unit % col_blocks) * NT, bz = unit / col_blocks;
    const int row0 = rb * BM;
    const int total_chunks = k_tiles / KT;
    const int c_begin = bz * chunks_per_split;
    const int c_end = min(c_begin + chunks_per_split, total_chunks);
    const int n_chunks = c_end - c_begin;
    const int last = max(c_end - 1, c_begin);

    f32x16_t acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    // W: lane pointer to k tile `wave` of chunk 0 of each of the block's bands (clamped on a ragged last block)
    const uint4 *wband[NT];
#pragma unroll
    for (int j = 0; j < NT; j++) {
        const int t = min(ntile0 + j, n_tiles - 1);
        wband[j] = Wp + ((size_t)t * k_tiles + wave) * 64 + lane;
    }
    // X staging, as in the streaming kernel: piece idx = i * 256 + tid is k piece idx % 8 of block row idx / 8;
    // rows past M are clamped (an output row depends on its own X row only, and rows >= M are never stored).
    // LDS slot of fragment (row tile, k tile): (k half) * 32 + row, XOR-swizzled by the k tile and the k half.
    const bf16_t *xsrc[XLOADS];
    int xdst[XLOADS];
#pragma unroll
    for (int i = 0; i < XLOADS; i++) {
        const int idx = i * 256 + tid;
        const int c = idx & 7, r = idx >> 3;
        const int row = min(row0 + r, M - 1);
        xsrc[i] = reinterpret_cast<const bf16_t *>(X) + (size_t)row * K + c * 8;
        xdst[i] = (((r >> 5) * KT + (c >> 1)) << 6) + ((((c & 1) << 5) + (r & 31)) ^ (((c >> 1) << 1) | ((c & 1) << 3)));
    }
    const int lsw = (lane ^ ((lane >> 5) << 3)) ^ (wave << 1);   // this wave's fragment slot (k tile = wave)

    sk_u32x4_t xr[D][XLOADS];   // a native vector type: the ring must stay in registers
    Frag wf[D][NT];
#define FG_SK_LOAD(slot, chunk)                                                                                       \
    do {                                                                                                              \
        const int cc_ = min((chunk), last);                                                                           \
        _Pragma("unroll") for (int i = 0; i < XLOADS; i++)                                                            \
            xr[slot][i] = *reinterpret_cast<const sk_u32x4_t *>(xsrc[i] + (size_t)cc_ * 64);                               \
        _Pragma("unroll") for (int j = 0; j < NT; j++) wf[slot][j].u = sk_load_stream(wband[j] + (size_t)cc_ * (KT * 64)); \
    } while (0)
#define FG_SK_STORE_X(slot, buf) \
    _Pragma("unroll") for (int i = 0; i < XLOADS; i++) reinterpret_cast<sk_u32x4_t *>(xs)[(buf) * (MT * KT * 64) + xdst[i]] = xr[slot][i]

    if (n_chunks > 0) {
#pragma unroll
        for (int d = 0; d < D; d++) FG_SK_LOAD(d, c_begin + d);
        FG_SK_STORE_X(0, 0);
        __syncthreads();
        // Whole rounds of the ring with no branch inside, so that the load counter's waits are exact.  Chunk c + d:
        // its X sits in LDS buffer d & 1, its W in ring slot d.  After the MFMAs, X of the next chunk (requested D
        // chunks ago, just before that chunk's W) goes to the other buffer, then the slot is refilled with chunk
        // c + d + D.  Past the end of the split the loads are clamped to its last chunk and the X fragment is
        // zeroed, so the surplus steps of the last round add nothing.
        for (int c = 0; c < n_chunks; c += D) {
#pragma unroll
            for (int d = 0; d < D; d++) {
                const bool live = c + d < n_chunks;
                Frag xa[MT];
#pragma unroll
                for (int i = 0; i < MT; i++) {
                    const sk_u32x4_t v = reinterpret_cast<const sk_u32x4_t *>(xs)[(d & 1) * (MT * KT * 64) + ((i * KT + wave) << 6) + lsw];
                    xa[i].u = live ? make_uint4(v.x, v.y, v.z, v.w) : make_uint4(0u, 0u, 0u, 0u);
                }
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int j = 0; j < NT; j++) acc[i][j] = mfma32<T>(xa[i], wf[d][j], acc[i][j]);
                FG_SK_STORE_X((d + 1) % D, (d + 1) & 1);
                FG_SK_LOAD(d, c_begin + c + d + D);
                __syncthreads();
            }
        }
    }
#undef FG_SK_LOAD
#undef FG_SK_STORE_X

    // The four k quarters meet in LDS, one row tile (32 rows x 64 columns) at a time.  A lane's 16 accumulators of
    // a tile are four groups of four consecutive rows (group q: rows 8 q + 4 (lane / 32) + 0..3, column lane % 32);
    // group q travels as one 16-byte entry and is summed by wave q, and groups whose rows are all past M stay home.
    sk_f32x4_t *red = reinterpret_cast<sk_f32x4_t *>(smem);   // [wave][tile][group][lane]
    const int F = N >> 1;
#pragma unroll
    for (int i = 0; i < MT; i++) {
        if (row0 + i * 32 >= M) break;
        __syncthreads();   // the X buffers / the previous tile's readers are done
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int q = 0; q < 4; q++)
                if (row0 + i * 32 + 8 * q < M)
                    red[((wave * NT + j) * 4 + q) * 64 + lane] =
                        (sk_f32x4_t){acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        __syncthreads();
        const int q = wave, m0 = row0 + i * 32 + 8 * q + 4 * (lane >> 5);
        if (row0 + i * 32 + 8 * q < M) {
            float s[NT][4];
#pragma unroll
            for (int j = 0; j < NT; j++) {
                const sk_f32x4_t a = red[((0 * NT + j) * 4 + q) * 64 + lane], b = red[((1 * NT + j) * 4 + q) * 64 + lane];
                const sk_f32x4_t c = red[((2 * NT + j) * 4 + q) * 64 + lane], d = red[((3 * NT + j) * 4 + q) * 64 + lane];
                s[j][0] = (a.x + b.x) + (c.x + d.x);
                s[j][1] = (a.y + b.y) + (c.y + d.y);
                s[j][2] = (a.z + b.z) + (c.z + d.z);
                s[j][3] = (a.w + b.w) + (c.w + d.w);
            }
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const int m = m0 + k;
                if (m >= M) continue;
                if (EPI == 0) {
#pragma unroll
                    for (int j = 0; j < NT; j++) {
                        const int nt = ntile0 + j;
                        if (nt < n_tiles) reinterpret_cast<float *>(out)[((size_t)bz * M + m) * N + nt * 32 + (lane & 31)] = s[j][k];
                    }
                } else {
                    // tiles alternate gate / up for the same 32 features
#pragma unroll
                    for (int j = 0; j + 1 < NT; j += 2) {
                        if (ntile0 + j + 1 >= n_tiles) continue;
                        const int f = ((ntile0 + j) >> 1) * 32 + (lane & 31);
                        reinterpret_cast<T *>(out)[(size_t)m * F + f] = from_f<T>(swiglu_f(s[j][k], s[j + 1][k]));
                    }
                }
            }
        }
    }
}

// Splits across blocks for the partial-slab epilogue.  Measured on the 7B-class shapes at 8 and 48 rows, the
// fastest grids are the ones just under one block per CU (down: 4 splits of 56 column blocks, 22 us against 24 - 26
// for 8 - 16 splits; O: 4; QKV: 3 of 72), so: the largest split that keeps the grid within 256 blocks and every
// split at least one round of the ring long, and among those the fewest splits that give the same longest split
// (the blocks run side by side, so the longest split is the duration).
int gemm_mfma_skinny_row_blocks(int M);
int gemm_mfma_skinny_split_for(int M, int N, int K)
{
    const int col_blocks = (N / 32 + SK_NT - 1) / SK_NT * gemm_mfma_skinny_row_blocks(M), chunks = K / 64;
    int s_hi = 256 / col_blocks;
    if (s_hi > 16) s_hi = 16;
    if (s_hi > chunks / SK_DEPTH) s_hi = chunks / SK_DEPTH;
    if (s_hi < 1) s_hi = 1;
    int best = 1, best_len = 1 << 30;
    for (int s = 1; s <= s_hi; s++) {
        const int len = ((chunks + s - 1) / s + SK_DEPTH - 1) / SK_DEPTH * SK_DEPTH;
        if (len < best_len) { best_len = len; best = s; }
    }
    return best;
}

template <typename T, int MT, int NT, int D = SK_DEPTH>
static void launch_skinny_mt(const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split, hipStream_t st)
{
    // chunks per split in whole rounds of the ring (a split past the end of k then writes a slab of zeros)
    const int chunks = K / 64, cps = ((chunks + split - 1) / split + D - 1) / D * D;
    const int col_blocks = (N / 32 + NT - 1) / NT, row_blocks = (M + MT * 32 - 1) / (MT * 32);
    const int units = col_blocks * split;
    dim3 grid((unsigned)((units + 7) / 8 * 8 * row_blocks));
    if (epilogue == 0)
        hipLaunchKernelGGL((gemm_mfma_skinny_kernel<T, MT, 0, NT, D>), grid, dim3(256), 0, st, reinterpret_cast<const T *>(x),
                           reinterpret_cast<const uint4 *>(wp), out, M, N, K, cps, row_blocks, col_blocks, split);
    else
        hipLaunchKernelGGL((gemm_mfma_skinny_kernel<T, MT, 1, NT, D>), grid, dim3(256), 0, st, reinterpret_cast<const T *>(x),
                           reinterpret_cast<const uint4 *>(wp), out, M, N, K, cps, row_blocks, col_blocks, split);
}

// Row tiles per block: one block of up to four tiles for up to 128 rows, otherwise the rows are cut evenly over
// blocks of three or four tiles.
int gemm_mfma_skinny_row_blocks(int M) { return (M + 127) / 128; }

template <typename T>
static void launch_skinny_typed(const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split, hipStream_t st)
{
    const int rb = gemm_mfma_skinny_row_blocks(M), per = (M + rb - 1) / rb;   // rows per block
    if (per <= 32) launch_skinny_mt<T, 1, SK_NT>(x, wp, out, M, N, K, epilogue, split, st);
    else if (per <= 64) launch_skinny_mt<T, 2, SK_NT>(x, wp, out, M, N, K, epilogue, split, st);
    else if (per <= 96) launch_skinny_mt<T, 3, SK_NT>(x, wp, out, M, N, K, epilogue, split, st);
    else launch_skinny_mt<T, 4, SK_NT>(x, wp, out, M, N, K, epilogue, split, st);
}

// Shapes were validated by the caller (launch_gemm_mfma).
int32_t launch_gemm_mfma_skinny(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue,
                                int split, hipStream_t st)
{
    if (M > 512) return fail(FG_ERR_SHAPE, "few-row GEMM takes at most 512 rows (got %d)", M);
    if (dtype == FG_BF16) launch_skinny_typed<bf16_t>(x, wp, out, M, N, K, epilogue, split, st);
    else launch_skinny_typed<f16_t>(x, wp, out, M, N, K, epilogue, split, st);
    FG_LAUNCH_CHECK("gemm_mfma_skinny");
    return FG_OK;
}

}  // namespace fg
