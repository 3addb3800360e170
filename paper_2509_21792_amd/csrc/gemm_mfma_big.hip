// Compute-bound shape of the 16-bit MFMA GEMM (more than 256 rows): out = X . W^T on 256 x 256 tiles.
//
// Block = 4 waves side by side, each owning 256 rows x 64 columns (8 x 2 tiles of v_mfma_f32_32x32x16).  With one
// wave per SIMD nothing hides a stall, so both operands are requested two 64-wide k chunks ahead:
//   W  packed fragments, global -> registers, two register sets that alternate by chunk; the set of chunk c is
//      refilled with chunk c + 2 fragment by fragment right after the MFMAs that consumed it;
//   X  row-major activations, global -> LDS directly (buffer_load_dwordx4 ... lds: 64 lanes x 16 bytes land in 1 KiB of
//      consecutive LDS), into a ring of three 32 KiB stages.  A stage holds 256 rows x 128 bytes; the 16-byte
//      piece p of row r holds the k octet p ^ ((r >> 1) & 7).  The permutation is applied to the *global*
//      address each lane requests (a row's eight lanes still cover its 128 contiguous bytes), and makes the
//      ds_read_b128 fragment reads (16 lanes = 16 rows, one octet) fall into 16 different bank groups.
// One barrier per chunk, placed before the last k tile: by then every wave has read all fragments of the current
// stage, so the stage can be handed to the loads of chunk c + 3 while the last 16 MFMAs run and the first
// fragments of the next chunk are read.
//
// vmcnt bookkeeping (loads retire in issue order).  Per chunk a wave issues, in this order: the W fragments of k
// tiles 0-2 (6 loads), [wait + barrier], the 8 X loads, the W fragments of k tile 3 (2 loads).  At the wait of
// chunk c the X loads of chunk c + 1 (issued two chunks earlier) must have landed; younger than them are
// 2 + 6 + 8 + 2 + 6 = 24 loads, hence s_waitcnt vmcnt(24).  The prologue issues its loads in the same interleaving
// so that the count holds from the first chunk on, and chunks past the end are clamped (re-requested), not
// skipped, so that it holds to the last.  Scheduling barriers pin the loads to their side of each wait.
#include "fg_common.h"
#include "gemm_mfma.h"

namespace fg {

constexpr int BIG_STAGES = 3;
constexpr int BIG_STAGE_U4 = 256 * 8;   // uint4 slots per stage: 256 rows x 8 pieces

// s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt << 4 | lgkmcnt << 8 | vmcnt[5:4] << 14
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | (7 << 4) | ((lgkm & 15) << 8) | ((vm >> 4) << 14); }

template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_big_kernel(const T *__restrict__ X, const uint4 *__restrict__ Wp,
                                                             void *__restrict__ out, int M, int N, int K, int chunks_per_split,
                                                             int raster, int row_blocks)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-descriptor builtins exist in the device pass only
    constexpr int MT = 8, NT = 2, WN = 4, BM = 256;
    // one variable per stage: the compiler orders LDS reads after direct-to-LDS loads per variable, so distinct
    // variables keep the reads of one stage from waiting on the loads in flight to the others
    __shared__ uint4 xs0[BIG_STAGE_U4], xs1[BIG_STAGE_U4], xs2[BIG_STAGE_U4];

    const int tid = threadIdx.x, lane = tid & 63, wn = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_tiles = N >> 5, k_tiles = K >> 4;
    int bx, by, bz;
    if (!map_block(raster, n_tiles, WN * NT, k_tiles, chunks_per_split, row_blocks, bx, by, bz)) return;
    const int row0 = by * BM;
    const int ntile0 = (bx * WN + wn) * NT;
    const int total_chunks = k_tiles / KT;
    const int c_begin = bz * chunks_per_split;
    const int c_end = min(c_begin + chunks_per_split, total_chunks);
    const int n_chunks = c_end - c_begin;
    if (n_chunks <= 0) return;

    f32x16_t acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
        for (int j = 0; j < NT; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    // W: lane pointer into each of the wave's two bands (clamped on a ragged last block; never stored)
    const uint4 *wband[NT];
#pragma unroll
    for (int j = 0; j < NT; j++) {
        int t = min(ntile0 + j, n_tiles - 1);
        wband[j] = Wp + ((size_t)t * k_tiles) * 64 + lane;
    }
    // X: wave wn brings rows 64 wn .. 64 wn + 63 of the block, 8 rows per load; lane = (row in the 8, piece p)
    int xoff[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int r = wn * 64 + i * 8 + (lane >> 3), p = lane & 7;
        const int row = min(row0 + r, M - 1);
        xoff[i] = (row * K + ((p ^ ((r >> 1) & 7)) << 3)) * 2;   // bytes
    }
    // X is addressed through a raw buffer descriptor (MUBUF loads can target LDS without being treated as
    // flat accesses by the compiler's wait-count bookkeeping): per-lane byte offset + per-chunk scalar offset
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(X), 0, M * K * 2, 0x00020000);
    // fragment reads: lane = (k half h, row l % 32): octet 2 kt + h of row 32 i + l % 32 sits in piece
    // (2 kt + h) ^ f with f = ((l % 32) >> 1) & 7, i.e. ((h ^ f) ^ (kt << 1))
    int xrd[KT];
    {
        const int r = lane & 31, h = lane >> 5, f = (r >> 1) & 7;
#pragma unroll
        for (int kt = 0; kt < KT; kt++) xrd[kt] = r * 8 + ((h ^ f) ^ (kt << 1));
    }

    Frag w0[NT][KT], w1[NT][KT], xa[MT], xb[MT];

#define FG_X_ISSUE(chunk, stage)                                                                          \
    _Pragma("unroll") for (int i = 0; i < 8; i++) __builtin_amdgcn_raw_ptr_buffer_load_lds(               \
        xrsrc, (stage) + (wn * 64 + i * 8) * 8, 16, xoff[i], __builtin_amdgcn_readfirstlane((chunk) * 128), 0, 0)
#define FG_W_LOAD(set, chunk, kt) \
    _Pragma("unroll") for (int j = 0; j < NT; j++) set[j][kt].u = wband[j][(size_t)((chunk) * KT + (kt)) * 64]
#define FG_X_READ(dst, stage_base, kt) \
    _Pragma("unroll") for (int i = 0; i < MT; i++) dst[i].u = (stage_base)[i * 256 + xrd[kt]]
#define FG_MFMA(xf, set, kt)                                                       \
    _Pragma("unroll") for (int i = 0; i < MT; i++) _Pragma("unroll") for (int j = 0; j < NT; j++) \
        acc[i][j] = mfma32<T>(xf[i], set[j][kt], acc[i][j])
#define FG_FENCE() __builtin_amdgcn_sched_barrier(0)

    const int last = c_end - 1;
    auto clampc = [&](int c) { return min(c, last); };

    // prologue: X(0), W(0) k tiles 0-2, X(1), W(0) k tile 3, W(1) k tiles 0-2, X(2), W(1) k tile 3
    FG_X_ISSUE(c_begin, xs0);
    FG_FENCE();
    FG_W_LOAD(w0, c_begin, 0); FG_W_LOAD(w0, c_begin, 1); FG_W_LOAD(w0, c_begin, 2);
    FG_FENCE();
    FG_X_ISSUE(clampc(c_begin + 1), xs1);
    FG_FENCE();
    FG_W_LOAD(w0, c_begin, 3);
    FG_W_LOAD(w1, clampc(c_begin + 1), 0); FG_W_LOAD(w1, clampc(c_begin + 1), 1); FG_W_LOAD(w1, clampc(c_begin + 1), 2);
    FG_FENCE();
    FG_X_ISSUE(clampc(c_begin + 2), xs2);
    FG_FENCE();
    FG_W_LOAD(w1, clampc(c_begin + 1), 3);
    FG_FENCE();
    // X(0) landed.  Only the 16 direct-to-LDS loads behind it are counted: the compiler may move the register
    // loads of the prologue, and a stricter wait costs nothing here.
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(16, 0));
    __builtin_amdgcn_s_barrier();
    FG_FENCE();
    FG_X_READ(xa, xs0, 0);

    // One chunk: `cur` holds its W fragments and is refilled with chunk c + 2; st = its stage, sn = the next one.
    // Within a k tile the instruction stream is laid out as 8 x {2 MFMAs, 1 fragment read (, 1 X load)} followed by
    // the two W loads, so that the LDS and memory instructions issue under the running MFMAs instead of in a clump.
#define FG_PIPE(with_x)                                                                               \
    _Pragma("unroll") for (int q = 0; q < 8; q++) {                                                   \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                            \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                            \
        if (with_x) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                \
    }                                                                                                 \
    __builtin_amdgcn_sched_group_barrier(0x020, 2, 0)
#define FG_CHUNK(cur, c, st, sn)                                                                      \
    do {                                                                                              \
        const uint4 *sb = (st);                                                                       \
        const int c2 = clampc((c) + 2), c3 = clampc((c) + 3);                                         \
        FG_FENCE();                                                                                   \
        FG_X_READ(xb, sb, 1);                                                                         \
        FG_MFMA(xa, cur, 0);                                                                          \
        FG_W_LOAD(cur, c2, 0);                                                                        \
        FG_PIPE(0);                                                                                   \
        FG_FENCE();                                                                                   \
        FG_X_READ(xa, sb, 2);                                                                         \
        FG_MFMA(xb, cur, 1);                                                                          \
        FG_W_LOAD(cur, c2, 1);                                                                        \
        FG_PIPE(0);                                                                                   \
        FG_FENCE();                                                                                   \
        FG_X_READ(xb, sb, 3);                                                                         \
        FG_MFMA(xa, cur, 2);                                                                          \
        FG_W_LOAD(cur, c2, 2);                                                                        \
        FG_PIPE(0);                                                                                     \
        FG_FENCE();                                                                                   \
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(24, 0));                                               \
        __builtin_amdgcn_s_barrier();                                                                 \
        FG_FENCE();                                                                                   \
        FG_X_ISSUE(c3, st);                                                                           \
        FG_X_READ(xa, (sn), 0);                                                                       \
        FG_MFMA(xb, cur, 3);                                                                          \
        FG_W_LOAD(cur, c2, 3);                                                                        \
        FG_PIPE(1);                                                                                   \
        FG_FENCE();                                                                                   \
    } while (0)

    // stages and W sets are static per code location: six chunks per trip, then a tail of up to five
    int c = c_begin;
    for (; c + 5 < c_end; c += 6) {
        FG_CHUNK(w0, c, xs0, xs1);
        FG_CHUNK(w1, c + 1, xs1, xs2);
        FG_CHUNK(w0, c + 2, xs2, xs0);
        FG_CHUNK(w1, c + 3, xs0, xs1);
        FG_CHUNK(w0, c + 4, xs1, xs2);
        FG_CHUNK(w1, c + 5, xs2, xs0);
    }
    if (c < c_end) FG_CHUNK(w0, c, xs0, xs1);
    if (c + 1 < c_end) FG_CHUNK(w1, c + 1, xs1, xs2);
    if (c + 2 < c_end) FG_CHUNK(w0, c + 2, xs2, xs0);
    if (c + 3 < c_end) FG_CHUNK(w1, c + 3, xs0, xs1);
    if (c + 4 < c_end) FG_CHUNK(w0, c + 4, xs1, xs2);
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));   // drain the clamped tail requests before the wave ends
#undef FG_CHUNK
#undef FG_PIPE
#undef FG_X_ISSUE
#undef FG_W_LOAD
#undef FG_X_READ
#undef FG_MFMA
#undef FG_FENCE

    store_tiles<T, MT, NT, EPI>(acc, out, M, N, row0, ntile0, n_tiles, bz, lane);
#endif
}

// Split and band-group choice by a small cost model (in microseconds).  The grid deals whole units (one k split of
// one group of BG bands, row_blocks x BG tiles) to the 8 XCDs, so the busiest XCD sets the number of rounds its 32
// CUs need; a round costs the split's chunks plus about 8 chunk-times of prologue and epilogue; every extra split
// adds an fp32 slab the consumer has to read back.
struct BigPlan { int split, bg; };
static BigPlan plan_big(int M, int N, int K, int fixed_split)
{
    const int n_bands = (N / 32 + 7) / 8, row_blocks = (M + 255) / 256, chunks = K / 64;
    BigPlan best{1, 1};
    double best_cost = 1e30;
    const int s_max = row_blocks == 1 ? 16 : 8;   // one row block: the slabs are small, the grid needs the splits
    for (int s = 1; s <= s_max; s++) {
        if (fixed_split > 0 && s != fixed_split) continue;
        if (fixed_split <= 0 && s > 1 && chunks / s < 8) break;
        const int cps = (chunks + s - 1) / s;
        if ((chunks + cps - 1) / cps != s) continue;   // some split would be empty
        for (int bg = 1; bg <= 4; bg *= 2) {
            const int units = (n_bands + bg - 1) / bg * s;
            const int xcd_blocks = (units + 7) / 8 * row_blocks * bg;
            const int rounds = (xcd_blocks + 31) / 32;
            double cost = rounds * (cps + 8) * 1.45 + (s - 1) * (double)M * N * 4 * 1.3 / 4.5e6;
            cost -= 0.01 * bg;   // equal otherwise: wider groups share more of X in L2
            if (cost < best_cost) { best_cost = cost; best = BigPlan{s, bg}; }
        }
    }
    if (fixed_split > 0 && best_cost == 1e30) best = BigPlan{fixed_split, 1};
    return best;
}

int gemm_mfma_big_split_for(int M, int N, int K) { return plan_big(M, N, K, 0).split; }

template <typename T>
static void launch_big_typed(const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split, int raster_on,
                             hipStream_t st)
{
    const int n_tiles = N / 32, per_block = 8;
    const int total_chunks = K / 64;
    const int cps = (total_chunks + split - 1) / split;
    const int n_bands = (n_tiles + per_block - 1) / per_block, row_blocks = (M + 255) / 256;
    dim3 grid(n_bands, row_blocks, split);
    int BG = 0;
    if (raster_on) {
        BG = plan_big(M, N, K, split).bg;
        const int units = (n_bands + BG - 1) / BG * split;
        grid = dim3((unsigned)(8 * ((units + 7) / 8) * row_blocks * BG));
    }
    if (epilogue == 0)
        hipLaunchKernelGGL((gemm_mfma_big_kernel<T, 0>), grid, dim3(256), 0, st, reinterpret_cast<const T *>(x),
                           reinterpret_cast<const uint4 *>(wp), out, M, N, K, cps, BG, row_blocks);
    else
        hipLaunchKernelGGL((gemm_mfma_big_kernel<T, 1>), grid, dim3(256), 0, st, reinterpret_cast<const T *>(x),
                           reinterpret_cast<const uint4 *>(wp), out, M, N, K, cps, BG, row_blocks);
}

// Shapes were validated by the caller (launch_gemm_mfma); M * K < 2^30 is needed by the 32-bit byte offsets.
int32_t launch_gemm_mfma_big(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue,
                             int split, int raster_on, hipStream_t st)
{
    if ((int64_t)M * K >= (1LL << 30)) return fail(FG_ERR_SHAPE, "GEMM input of %d x %d exceeds 2^30 elements", M, K);
    if (dtype == FG_BF16) launch_big_typed<bf16_t>(x, wp, out, M, N, K, epilogue, split, raster_on, st);
    else launch_big_typed<f16_t>(x, wp, out, M, N, K, epilogue, split, raster_on, st);
    FG_LAUNCH_CHECK("gemm_mfma_big");
    return FG_OK;
}

}  // namespace fg
