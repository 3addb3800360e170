// 16-bit (bf16 or fp16 operands, fp32 accumulate) GEMM on MFMA for gfx950: out = X . W^T with W pre-packed as
// MFMA operand fragments.
//
// W [N, K] is stored as 1 KiB tiles of 32 rows x 16 k: lane ((k % 16) / 8) * 32 + n % 32 of a tile holds the 8
// consecutive k of row n -- exactly the per-lane operand of v_mfma_f32_32x32x16_{bf16,f16} -- and the tiles of one
// 32-row band are contiguous in k.  A wave therefore streams its band of W straight from HBM into MFMA operand
// registers with fully coalesced 16-byte loads (1 KiB per wave instruction, no LDS round trip, no swizzle).
// The activation block X [M, K] (row-major, small or reused) is staged through LDS in the same fragment order,
// double buffered, one barrier per 64-wide k chunk.
//
// Block = WM x WN waves; a wave owns MT x NT tiles of 32 x 32 outputs.  WM = 1 with MT = ceil(M / 32) is the
// weight-streaming (memory-bound) shape: every byte of W is read exactly once per GEMM.  Split-K over
// blockIdx.z writes fp32 partial slabs that the consumer kernel sums (no atomics: results are deterministic).
#include "fg_common.h"
#include "gemm_mfma.h"

namespace fg {

// W is read exactly once per GEMM by this kernel (one row block): a streaming load that does not displace the
// activations and slabs in the caches.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4 *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <typename T, int MT, int NT, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM *WN * 64) void gemm_mfma_kernel(const T *__restrict__ X, const uint4 *__restrict__ Wp,
                                                                  void *__restrict__ out, int M, int N, int K,
                                                                  int chunks_per_split, int raster, int row_blocks)
{
    constexpr int THREADS = WM * WN * 64;
    constexpr int BM = WM * MT * 32;
    constexpr int XLOADS = BM * 8 / THREADS;  // 16-byte loads of X per thread per chunk
    static_assert(BM * 8 % THREADS == 0, "X staging must divide evenly");
    __shared__ uint4 xs[2][BM / 32 * KT * 64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int n_tiles = N >> 5, k_tiles = K >> 4;
    int bx, by, bz;
    if (!map_block(raster, n_tiles, WN * NT, k_tiles, chunks_per_split, row_blocks, bx, by, bz)) return;
    const int row0 = by * BM;
    const int ntile0 = (bx * WN + wn) * NT;
    const int total_chunks = k_tiles / KT;
    const int c_begin = bz * chunks_per_split;
    const int c_end = min(c_begin + chunks_per_split, total_chunks);
    const int n_chunks = c_end - c_begin;

    f32x16_t acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    // W band pointers (clamped for the ragged last block so loads stay in bounds; results are not stored)
    const uint4 *wband[NT];
#pragma unroll
    for (int j = 0; j < NT; j++) {
        int t = min(ntile0 + j, n_tiles - 1);
        wband[j] = Wp + ((size_t)t * k_tiles) * 64 + lane;
    }

    uint4 xr[XLOADS];
    Frag w[NT][KT];

    // X staging: thread t moves XLOADS 16-byte pieces per chunk; piece idx = i * THREADS + t is k-piece idx % 8
    // (c) of block row idx / 8 (r), so 8 consecutive lanes read 128 contiguous bytes of one row.  Rows past M are
    // clamped, not zeroed: an output row depends on its own X row only and rows >= M are never stored.
    // LDS holds the chunk in MFMA fragment order (fragment (row tile, k tile) = 64 slots of 16 bytes, slot
    // (k half) * 32 + row), with the slot XOR-swizzled by the k tile (bits 1-2) and the k half (bit 3): the 16
    // lanes of a store phase (8 pieces of 2 rows) then fall into 16 different bank groups, and the 16 consecutive
    // lanes of a fragment read still do.
    const bf16_t *xsrc[XLOADS];
    int xdst[XLOADS];
#pragma unroll
    for (int i = 0; i < XLOADS; i++) {
        int idx = i * THREADS + tid;
        int c = idx & 7, r = idx >> 3;
        int row = min(row0 + r, M - 1);
        xsrc[i] = reinterpret_cast<const bf16_t *>(X) + (size_t)row * K + c * 8;
        xdst[i] = (((r >> 5) * KT + (c >> 1)) << 6) + ((((c & 1) << 5) + (r & 31)) ^ (((c >> 1) << 1) | ((c & 1) << 3)));
    }
#define FG_LOAD_X(chunk)                                                                                  \
    _Pragma("unroll") for (int i = 0; i < XLOADS; i++) xr[i] = *reinterpret_cast<const uint4 *>(xsrc[i] + (size_t)(chunk) * 64)
#define FG_STORE_X(buf) _Pragma("unroll") for (int i = 0; i < XLOADS; i++) xs[buf][xdst[i]] = xr[i]

    if (n_chunks > 0) {
        FG_LOAD_X(c_begin);
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int kt = 0; kt < KT; kt++) w[j][kt].u = load_stream(wband[j] + (size_t)(c_begin * KT + kt) * 64);
        FG_STORE_X(0);
        __syncthreads();
        // One chunk per iteration.  Latency cover:
        //   W (HBM / L2)  fragment kt of the next chunk is requested into the registers of fragment kt right after
        //                 the MFMAs that consumed it, so a full chunk of MFMA work covers its latency;
        //   X (L2)        next chunk global -> registers at the top, registers -> the other LDS buffer at the bottom;
        //   LDS           the X fragments of k tile kt + 1 are read while the MFMAs of tile kt run (xa / xb
        //                 alternate); scheduling barriers keep the compiler from sinking the reads to their use.
        // The last iteration re-requests its own chunk (clamped index) instead of branching.
        Frag xa[MT], xb[MT];
        const int lsw = lane ^ ((lane >> 5) << 3);   // k-half part of the swizzle
        for (int c = 0; c < n_chunks; c++) {
            const int buf = c & 1;
            const int nxt = c_begin + min(c + 1, n_chunks - 1);
            FG_LOAD_X(nxt);
            const uint4 *xbase = &xs[buf][(wm * MT * KT) << 6];
#pragma unroll
            for (int i = 0; i < MT; i++) xa[i].u = xbase[((i * KT) << 6) + lsw];
#pragma unroll
            for (int kt = 0; kt < KT; kt += 2) {
#pragma unroll
                for (int i = 0; i < MT; i++) xb[i].u = xbase[((i * KT + kt + 1) << 6) + (lsw ^ ((kt + 1) << 1))];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int j = 0; j < NT; j++) acc[i][j] = mfma32<T>(xa[i], w[j][kt], acc[i][j]);
#pragma unroll
                for (int j = 0; j < NT; j++) w[j][kt].u = load_stream(wband[j] + (size_t)(nxt * KT + kt) * 64);
                __builtin_amdgcn_sched_barrier(0);
                if (kt + 2 < KT) {
#pragma unroll
                    for (int i = 0; i < MT; i++) xa[i].u = xbase[((i * KT + kt + 2) << 6) + (lsw ^ ((kt + 2) << 1))];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int j = 0; j < NT; j++) acc[i][j] = mfma32<T>(xb[i], w[j][kt + 1], acc[i][j]);
#pragma unroll
                for (int j = 0; j < NT; j++) w[j][kt + 1].u = load_stream(wband[j] + (size_t)(nxt * KT + kt + 1) * 64);
                __builtin_amdgcn_sched_barrier(0);
            }
            FG_STORE_X(buf ^ 1);
            __syncthreads();
        }
    }
#undef FG_LOAD_X
#undef FG_STORE_X

    store_tiles<T, MT, NT, EPI>(acc, out, M, N, row0 + wm * MT * 32, ntile0, n_tiles, bz, lane);
}

// ---- host side -----------------------------------------------------------------------------------------

template <typename T, int MT, int NT, int WM, int WN, int EPI>
static void launch_variant(const void *x, const void *wp, void *out, int M, int N, int K, int split, hipStream_t st)
{
    const int n_tiles = N / 32, per_block = WN * NT;
    const int total_chunks = K / 64;
    const int cps = (total_chunks + split - 1) / split;
    const int n_bands = (n_tiles + per_block - 1) / per_block, row_blocks = (M + WM * MT * 32 - 1) / (WM * MT * 32);
    if (row_blocks > 1) {
        const int BG = n_bands >= 32 ? 4 : (n_bands >= 16 ? 2 : 1);
        const int units = (n_bands + BG - 1) / BG * split;
        dim3 grid((unsigned)(8 * ((units + 7) / 8) * row_blocks * BG));
        hipLaunchKernelGGL((gemm_mfma_kernel<T, MT, NT, WM, WN, EPI>), grid, dim3(WM * WN * 64), 0, st,
                           reinterpret_cast<const T *>(x), reinterpret_cast<const uint4 *>(wp), out, M, N, K, cps, BG, row_blocks);
    } else {
        dim3 grid(n_bands, row_blocks, split);
        hipLaunchKernelGGL((gemm_mfma_kernel<T, MT, NT, WM, WN, EPI>), grid, dim3(WM * WN * 64), 0, st,
                           reinterpret_cast<const T *>(x), reinterpret_cast<const uint4 *>(wp), out, M, N, K, cps, 0, row_blocks);
    }
}

// Number of k splits of the weight-streaming kernel (fp32-partial epilogue only), by a small cost model in
// microseconds: streaming W takes its bytes over 5.3 TB/s, stretched when there are too few blocks to keep the
// memory system busy (about three blocks per CU for up to 32 rows, where a block is light, half of that above);
// every split adds a slab of M x N fp32 that is written here and read back by the consumer (about 2 TB/s for
// the pair).  Measured on the 7B-class and 1.5B-class shapes: gate/up at 48-128 rows wants 3 splits where a
// fixed block target gave 6 (60 -> 47 us at 48 rows, 81 -> 61 at 96), the narrow outputs keep the maximum.
static int choose_split(int M, int N, int K, int block_rows, int block_cols)
{
    const int bands = ((N + block_cols - 1) / block_cols) * ((M + block_rows - 1) / block_rows);
    const int total_chunks = K / 64;
    const double w_us = 2.0 * N * K / 5.3e6, slab_us = 4.0 * M * N / 2.0e6;
    const double sat = M <= 32 ? 800.0 : 400.0;
    int best = 1;
    double best_cost = 1e30;
    for (int s = 1; s <= 16 && s <= (total_chunks >= 2 ? total_chunks / 2 : 1); s++) {
        const int cps = (total_chunks + s - 1) / s;
        if ((total_chunks + cps - 1) / cps != s) continue;   // some split would be empty
        const double util = bands * s >= sat ? 1.0 : bands * s / sat;
        const double cost = w_us / util + s * slab_us;
        if (cost < best_cost) { best_cost = cost; best = s; }
    }
    return best;
}

int32_t launch_gemm_mfma_big(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue,
                             int split, int fixed_mt, const GemmEpi *epi, hipStream_t st);
int gemm_mfma_big_split_for(int M, int N, int K);
int gemm_mfma_big_unsplit_tiles(int M, int N, int K, int epilogue);
int gemm_mfma_big_stream_blocks(int N, int epilogue);
int32_t launch_gemm_mfma_skinny(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue,
                                int split, hipStream_t st);
int gemm_mfma_skinny_split_for(int M, int N, int K);
int32_t launch_gemm_mfma_decode(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split,
                                hipStream_t st);
int gemm_mfma_decode_split_for(int M, int N, int K);
bool gemm_mfma_decode_ok(int M, int N, int K, int epilogue);

// Which kernel runs a shape.  All thresholds are measurements on the 7B-class and 1.5B-class matrices; "wide" means
// at least 16384 output columns (gate/up, the LM head), "narrow" the QKV, O and down projections.  Times in us.
//   few-row kernel (gemm_mfma_skinny.hip, k split inside the block):
//     narrow outputs up to 64 rows, and up to 128 rows of a short reduction (QKV 15.0 / O 16.7 at 96 rows, level with
//       the pipelined kernel); the 7B down projection (18944 deep) takes 31.0 at 64 rows against 37 in the pipelined
//       kernel, but 36.4 / 43.7 at 96 / 128 rows against 32.6 / 33.5;
//     gate/up with its SwiGLU fused up to 31 rows (49.5 at 24 rows, level with the pipelined kernel; 51.0 / 56.2 / 60.2
//       at 32 / 48 / 64 rows against 49.7 / 50.8 / 52.2 there), up to 64 rows when the pipelined kernel would stream
//       through fewer than 192 blocks (the 1.5B-class gate/up, 140 blocks: level at 48 and 64 rows, 22 against 26 us per
//       layer at 96 rows, 23 against 30 at 128), and up to 128 rows when through fewer than 128;
//     the LM head up to 32 rows (167 against 177 at 8 rows, level at 32, behind above);
//   decode kernel (gemm_mfma_decode.hip, eight waves per block, no barrier in the main loop): gate/up with its SwiGLU
//     fused up to 16 rows -- 43.6 / 45.6 at 8 / 16 rows of the 7B-class model against 46.0 / 47.4 in the few-row kernel
//     (kernel durations from a trace).  Its partial-sum epilogue loses to the few-row kernel on every narrow output (O 8.9
//     against 6.9, QKV 12.0 against 7.8, down 25.9 against 22.0 at 8 rows) and on the LM head (186 against 168);
//   pipelined kernel (gemm_mfma_big.hip): every shape above 128 rows -- QKV 17.1 / 17.7 / 19.9 at 144 / 160 / 192 rows
//     against 24.5 in the few-row kernel, O 14.4 - 15.5 at 144 - 256 rows against 17 - 21 -- and from 65 rows the deep
//     narrow reductions (above) and the wide outputs that give at least 128 blocks (gate/up from 32 rows): one row of
//     128-row blocks, 192 columns wide so that 198 CUs stream, runs gate/up in 53.6 / 55.9 at 96 / 128 rows (61.4 / 64.2 with
//     256-column blocks) against 71.3 / 83.0 in the few-row and 89.9 / 91.1 in the streaming kernel, the LM head in 248 /
//     249 against 261 / 271 streamed;
//   streaming kernel (this file): the rest, i.e. the LM head at 33 - 64 rows (204 / 208 at 48 / 64 rows against 225 /
//     235 in 128-row blocks) and wide outputs of few blocks at 65 - 128 rows.
enum { KERNEL_STREAMING = 1, KERNEL_FEW = 2, KERNEL_BIG = 3, KERNEL_DECODE = 4 };
static int kernel_for(int M, int N, int K, int epilogue)
{
    if (epilogue >= EPI_ROPE) return KERNEL_BIG;
    if (N < 16384) return (M <= 64 || (M <= 128 && K < 8192)) ? KERNEL_FEW : KERNEL_BIG;
    if (M > 128) return KERNEL_BIG;
    const int stream_blocks = gemm_mfma_big_stream_blocks(N, epilogue == EPI_SWIGLU ? EPI_SWIGLU : EPI_SLABS);
    if ((M > 64 && stream_blocks >= 128) || (M > 31 && epilogue == EPI_SWIGLU && stream_blocks >= 192)) return KERNEL_BIG;
    if (epilogue == EPI_SWIGLU && M <= 16 && gemm_mfma_decode_ok(M, N, K, epilogue)) return KERNEL_DECODE;
    if (epilogue == EPI_SWIGLU) return (M <= 64 || (N + 63) / 64 <= 512) ? KERNEL_FEW : KERNEL_STREAMING;
    return M <= 32 ? KERNEL_FEW : KERNEL_STREAMING;
}
static int kernel_of_variant(int variant) { return variant == 1 ? KERNEL_STREAMING : (variant == 2 ? KERNEL_FEW : (variant == 6 ? KERNEL_DECODE : KERNEL_BIG)); }

// Whether the gate/up GEMM of M rows applies SwiGLU in its own epilogue (no slabs, no separate pass).
bool gemm_mfma_fuses_swiglu(int M, int N, int K) { return kernel_for(M, N, K, EPI_SWIGLU) != KERNEL_STREAMING; }

// Whether a GEMM of this shape runs the fused epilogue `kind` (RoPE + append, residual add, top-k partials): they
// exist in the pipelined kernel without a k split, which pays once the unsplit launch has tiles for three quarters
// of the CUs; below that the grid needs k splits, hence slabs, to fill the chip.  Measured on the 7B-class shapes, us
// per layer, unsplit with the fused epilogue against split with slabs and the separate row-wise kernel: at 1024 rows
// QKV 76 against 52, O 56 against 34, down 224 against 113 (112 - 144 tiles); at 2048 rows 96 / 62 / 244 against
// 93 / 68 / 250 (224 - 234 tiles).
bool gemm_mfma_fusable(int M, int N, int K, int kind)
{
    if (kind < EPI_ROPE) return true;
    if (kind > EPI_TOPK || (int64_t)M * K >= (1LL << 30)) return false;
    // the top-k epilogue is for LM heads: thousands of tiles, no k split at any row count the pipelined kernel takes
    if (kind == EPI_TOPK) return N >= 16384 && (M > 128 || (M > 64 && (N / 32 + 7) / 8 >= 128));
    return M > 256 && gemm_mfma_big_unsplit_tiles(M, N, K, kind) >= 192;
}

int gemm_mfma_split_for(int M, int N, int K)
{
    const int k = kernel_for(M, N, K, EPI_SLABS);
    if (k == KERNEL_FEW) return gemm_mfma_skinny_split_for(M, N, K);
    if (k == KERNEL_DECODE) return gemm_mfma_decode_split_for(M, N, K);
    if (k == KERNEL_BIG) return gemm_mfma_big_split_for(M, N, K);
    return choose_split(M, N, K, 256, 256);
}

static const char *const KERNEL_NAMES[] = {"", "gemm_mfma_kernel", "gemm_mfma_skinny_kernel", "gemm_mfma_big_kernel", "gemm_mfma_decode_kernel"};
const char *gemm_mfma_kernel_name(int M, int N, int K, int epilogue) { return KERNEL_NAMES[kernel_for(M, N, K, epilogue)]; }

template <typename T>
static int32_t launch_gemm_typed(const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split,
                                 hipStream_t st)
{
#define FG_GEMM_CASE(MT, NT, WM, WN)                                                                       \
    do {                                                                                                   \
        if (epilogue == 0) launch_variant<T, MT, NT, WM, WN, 0>(x, wp, out, M, N, K, split, st);           \
        else launch_variant<T, MT, NT, WM, WN, 1>(x, wp, out, M, N, K, split, st);                         \
    } while (0)
    if (M <= 32) FG_GEMM_CASE(1, 2, 1, 4);
    else if (M <= 64) FG_GEMM_CASE(2, 2, 1, 4);
    else if (M <= 128) FG_GEMM_CASE(4, 2, 1, 4);
    else FG_GEMM_CASE(8, 2, 1, 4);
#undef FG_GEMM_CASE
    FG_LAUNCH_CHECK("gemm_mfma");
    return FG_OK;
}

int32_t launch_gemm_mfma(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue,
                         int split_k, int *split_used, hipStream_t st, const GemmEpi *epi, int variant)
{
    if (M <= 0) return FG_OK;
    if (!is16(dtype)) return fail(FG_ERR_INVALID_ARG, "MFMA GEMM needs a 16-bit dtype");
    if (N % 32 || K % 64) return fail(FG_ERR_SHAPE, "16-bit GEMM needs n_out %% 32 == 0 and n_in %% 64 == 0 (got %d, %d)", N, K);
    if (epilogue == EPI_SWIGLU && (N % 64)) return fail(FG_ERR_SHAPE, "gate/up GEMM needs n_out %% 64 == 0");
    if ((int64_t)M * N >= (1LL << 31)) return fail(FG_ERR_SHAPE, "GEMM output of %d x %d exceeds 2^31 elements", M, N);
    if (variant < 0 || variant > 14) return fail(FG_ERR_INVALID_ARG, "unknown GEMM variant %d", variant);
    const int kernel = variant ? kernel_of_variant(variant) : kernel_for(M, N, K, epilogue);
    if (epilogue >= EPI_ROPE && kernel != KERNEL_BIG) return fail(FG_ERR_INVALID_ARG, "GEMM epilogue %d exists in the pipelined kernel only", epilogue);
    if (kernel == KERNEL_FEW && M > 512) return fail(FG_ERR_SHAPE, "the few-row kernel takes at most 512 rows (got %d)", M);
    if (kernel == KERNEL_DECODE && !gemm_mfma_decode_ok(M, N, K, epilogue)) return fail(FG_ERR_SHAPE, "the decode kernel takes at most 16 rows and the partial-sum and SwiGLU epilogues (got %d rows, epilogue %d)", M, epilogue);
    if (kernel == KERNEL_STREAMING && M > 256 && epilogue != EPI_SLABS && epilogue != EPI_SWIGLU) return fail(FG_ERR_INVALID_ARG, "bad epilogue");
    int split = 1;
    if (epilogue == EPI_SLABS) {
        if (split_k > 0) split = split_k;
        else if (kernel == KERNEL_FEW) split = gemm_mfma_skinny_split_for(M, N, K);
        else if (kernel == KERNEL_DECODE) split = gemm_mfma_decode_split_for(M, N, K);
        else if (kernel == KERNEL_BIG) split = gemm_mfma_big_split_for(M, N, K);
        else split = choose_split(M, N, K, 256, 256);
        if (split > K / 64) split = K / 64;
        int cps = (K / 64 + split - 1) / split;
        split = (K / 64 + cps - 1) / cps;
    }
    if (split_used) *split_used = split;
    if (kernel == KERNEL_FEW) return launch_gemm_mfma_skinny(dtype, x, wp, out, M, N, K, epilogue, split, st);
    if (kernel == KERNEL_DECODE) return launch_gemm_mfma_decode(dtype, x, wp, out, M, N, K, epilogue, split, st);
    if (kernel == KERNEL_BIG) return launch_gemm_mfma_big(dtype, x, wp, out, M, N, K, epilogue, split, variant == 3 ? 8 : (variant == 4 ? 4 : (variant == 5 ? 5 : (variant == 7 ? 14 : (variant == 8 ? 15 : (variant == 9 ? 18 : (variant == 10 ? 24 : (variant == 11 ? 6 : (variant == 12 ? 16 : (variant == 13 ? 7 : (variant == 14 ? 17 : 0)))))))))), epi, st);
    return dtype == FG_BF16 ? launch_gemm_typed<bf16_t>(x, wp, out, M, N, K, epilogue, split, st)
                            : launch_gemm_typed<f16_t>(x, wp, out, M, N, K, epilogue, split, st);
}

// ---- packing ---------------------------------------------------------------------------------------------
// Logical row n of the packed matrix: without src2 it is src row n; with src2 the rows alternate in blocks of
// 32: logical block 2t = src rows 32t.., block 2t + 1 = src2 rows 32t...
template <typename T>
__device__ __forceinline__ const T *logical_row(const T *src, const T *src2, int64_t n, int64_t K)
{
    if (!src2) return src + n * K;
    int64_t blk = n >> 5, r = n & 31;
    const T *base = (blk & 1) ? src2 : src;
    return base + ((blk >> 1) * 32 + r) * K;
}

__global__ void pack_bf16_kernel(const bf16_t *src, const bf16_t *src2, uint4 *dst, int64_t N, int64_t K)
{
    // one thread per 16-byte fragment element: (n tile, k tile, lane)
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (N / 32) * (K / 16) * 64;
    if (idx >= total) return;
    int lane = idx & 63;
    int64_t tile = idx >> 6;
    int64_t kt = tile % (K / 16), nt = tile / (K / 16);
    int64_t n = nt * 32 + (lane & 31), k = kt * 16 + (lane >> 5) * 8;
    dst[idx] = *reinterpret_cast<const uint4 *>(logical_row(src, src2, n, K) + k);
}

// the same fragment order straight from an fp32 matrix, rounded to bf16 on the way (draft training packs fp32 operands
// for every product: one pass instead of a cast pass and a pack pass)
__global__ void pack_cast_bf16_kernel(const float *src, uint4 *dst, int64_t N, int64_t K)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (N / 32) * (K / 16) * 64;
    if (idx >= total) return;
    int lane = idx & 63;
    int64_t tile = idx >> 6;
    int64_t kt = tile % (K / 16), nt = tile / (K / 16);
    int64_t n = nt * 32 + (lane & 31), k = kt * 16 + (lane >> 5) * 8;
    const float4 a = *reinterpret_cast<const float4 *>(src + n * K + k), b = *reinterpret_cast<const float4 *>(src + n * K + k + 4);
    uint4 o;
    o.x = (uint32_t)f2bf(a.x) | ((uint32_t)f2bf(a.y) << 16);
    o.y = (uint32_t)f2bf(a.z) | ((uint32_t)f2bf(a.w) << 16);
    o.z = (uint32_t)f2bf(b.x) | ((uint32_t)f2bf(b.y) << 16);
    o.w = (uint32_t)f2bf(b.z) | ((uint32_t)f2bf(b.w) << 16);
    dst[idx] = o;
}

// ... and from the transpose: src is [K, N] fp32, the packed matrix is its transpose [N, K].  The 32 lanes that share a
// k read 128 contiguous bytes of a source row.
__global__ void pack_cast_t_bf16_kernel(const float *src, uint4 *dst, int64_t N, int64_t K)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (N / 32) * (K / 16) * 64;
    if (idx >= total) return;
    int lane = idx & 63;
    int64_t tile = idx >> 6;
    int64_t kt = tile % (K / 16), nt = tile / (K / 16);
    int64_t n = nt * 32 + (lane & 31), k = kt * 16 + (lane >> 5) * 8;
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = src[(k + j) * N + n];
    uint4 o;
    o.x = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
    o.y = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
    o.z = (uint32_t)f2bf(v[4]) | ((uint32_t)f2bf(v[5]) << 16);
    o.w = (uint32_t)f2bf(v[6]) | ((uint32_t)f2bf(v[7]) << 16);
    dst[idx] = o;
}

int32_t launch_pack_cast_t_bf16(const float *src, void *dst, int64_t n_out, int64_t n_in, hipStream_t st)
{
    if (n_out % 32 || n_in % 64) return fail(FG_ERR_SHAPE, "pack needs n_out %% 32 == 0 and n_in %% 64 == 0 (got %lld, %lld)",
                                             (long long)n_out, (long long)n_in);
    const int64_t total = (n_out / 32) * (n_in / 16) * 64;
    hipLaunchKernelGGL(pack_cast_t_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, (uint4 *)dst, n_out, n_in);
    FG_LAUNCH_CHECK("pack_cast_t");
    return FG_OK;
}

int32_t launch_pack_cast_bf16(const float *src, void *dst, int64_t n_out, int64_t n_in, hipStream_t st)
{
    if (n_out % 32 || n_in % 64) return fail(FG_ERR_SHAPE, "pack needs n_out %% 32 == 0 and n_in %% 64 == 0 (got %lld, %lld)",
                                             (long long)n_out, (long long)n_in);
    const int64_t total = (n_out / 32) * (n_in / 16) * 64;
    hipLaunchKernelGGL(pack_cast_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, (uint4 *)dst, n_out, n_in);
    FG_LAUNCH_CHECK("pack_cast");
    return FG_OK;
}

__global__ void pack_f32_kernel(const float *src, const float *src2, float *dst, int64_t N, int64_t K)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * K) return;
    int64_t n = idx / K, k = idx % K;
    dst[idx] = logical_row(src, src2, n, K)[k];
}

int32_t launch_pack(int32_t dtype, const void *src, const void *src2, void *dst, int64_t n_out, int64_t n_in, hipStream_t st)
{
    int64_t N = src2 ? 2 * n_out : n_out;
    if (n_out % 32 || n_in % 64) return fail(FG_ERR_SHAPE, "pack needs n_out %% 32 == 0 and n_in %% 64 == 0 (got %lld, %lld)",
                                             (long long)n_out, (long long)n_in);
    if (is16(dtype)) {
        int64_t total = (N / 32) * (n_in / 16) * 64;
        hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const bf16_t *)src, (const bf16_t *)src2, (uint4 *)dst, N, n_in);
    } else if (dtype == FG_F32) {
        int64_t total = N * n_in;
        hipLaunchKernelGGL(pack_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const float *)src,
                           (const float *)src2, (float *)dst, N, n_in);
    } else
        return fail(FG_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    FG_LAUNCH_CHECK("pack");
    return FG_OK;
}

}  // namespace fg
