// Decode shape of the 16-bit MFMA GEMM: out = X . W^T for up to 16 rows, bound by streaming W from HBM once.
//
// A block is eight waves and NT bands of 32 output columns.  k is dealt in steps of 8 x KPW k tiles (16 wide): in step s
// wave w takes the KPW consecutive tiles (8 s + w) KPW ...  Unlike the few-row kernel there is no block-wide barrier in
// the main loop.  The W fragments come straight from HBM through a ring of register sets, D steps ahead, in 1 KiB
// coalesced non-temporal loads.  X rides in the same ring: a wave's piece of a step -- MR rows x KPW tiles, up to 128
// contiguous bytes of each row -- is loaded coalesced (lane = row x pieces + piece, 16 bytes each; the X loads of a slot
// are issued before its W loads, and the load counter retires in order, so waiting for them never waits for younger W
// loads), written to the wave's own corner of LDS and read back in operand order (lane = row + 32 x k half; same-wave
// LDS accesses complete in order, so this needs no barrier).  Loading in operand order directly gives every lane its own
// cache line: the texture path then takes 64 single-lane requests per instruction (7B-class down projection, 8 rows,
// unsplit: 43 us instead of 35).  At the end the eight partials of a band meet in LDS, eight rows at a time:
//   EPI_SLABS   fp32 partial slab of the block's k split, [split][M][N],
//   EPI_SWIGLU  W is the gate/up interleaved matrix: silu(gate) * up, stored as T [M, N / 2] (no k split).
//
// A CU draws some 35 GB/s from HBM however much it keeps in flight, so a matrix of more than a few tens of megabytes
// wants a block on nearly every CU: the wide outputs get one by their bands alone (7B-class gate/up: 198 blocks of six
// bands, one per CU -- a block needs more than half a CU's registers, so a grid beyond 256 blocks would run in two
// rounds), the narrow ones by a k split across blocks whose slabs the consumer adds, as in the other kernels.
//
// Tried and dropped here: complete sums per block (no k split) with the neighbouring row-wise steps fused in -- RMS norm
// of the residual stream on the way in, RoPE + cache append or the residual add on the way out.  Correct, but the narrow
// matrices then stream through 72 - 112 CUs (QKV + RoPE 16.5 us against 12.6 for the split GEMM and the separate
// kernel, O 10.8 against 6.8), and a fused norm costs the launch it saves: its loads and its reduction sit on the
// kernel's critical path just the same (gate/up 48.0 us fused against 4.3 + 43).  Letting the blocks of a k split meet
// through a ticket counter, the last one adding the slabs, costs 35 us per launch: the release / acquire fences this
// needs between XCDs write back and invalidate whole L2s.
#include "fg_common.h"
#include "gemm_mfma.h"

namespace fg {

typedef uint32_t dc_u32x4_t __attribute__((ext_vector_type(4)));
typedef float dc_f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 dc_load_stream(const uint4 *p)
{
    const dc_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const dc_u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int DC_WAVES = 8;
constexpr int DC_MAX_ROWS = 16;

template <typename T, int MR, int NT, int KPW, int D, int EPI>
__global__ __launch_bounds__(DC_WAVES * 64) void gemm_mfma_decode_kernel(const T *__restrict__ X, const uint4 *__restrict__ Wp,
                                                                       void *__restrict__ out, int M, int N, int K, int blocks_n,
                                                                       int steps_per_split)
{
    static_assert(EPI == EPI_SLABS || (EPI == EPI_SWIGLU && NT % 2 == 0), "SwiGLU takes gate / up band pairs");
    static_assert(MR == 8 || MR == 16, "LDS holds 8 or 16 rows");
    constexpr int PP = 2 * KPW, RPI = 64 / PP, XQ = (MR + RPI - 1) / RPI;   // X staging, see below
    constexpr int XS = DC_WAVES * PP * MR, RED = DC_WAVES * NT * 64;        // 16-byte entries
    __shared__ dc_u32x4_t smem[XS > RED ? XS : RED];
    dc_f32x4_t *red = reinterpret_cast<dc_f32x4_t *>(smem);                 // [wave][band][lane], after the main loop

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_tiles = N >> 5, k_tiles = K >> 4;
    const int n_steps_all = (k_tiles + DC_WAVES * KPW - 1) / (DC_WAVES * KPW);
    // block -> (band group bn, k split z); split z takes steps [z sps, (z + 1) sps)
    const int bn = blockIdx.x % blocks_n, z = blockIdx.x / blocks_n;
    const int step_lo = z * steps_per_split, n_steps = max(min(n_steps_all - step_lo, steps_per_split), 0);
    const int row = lane & 31, khalf = lane >> 5;

    const uint4 *wband[NT];
#pragma unroll
    for (int j = 0; j < NT; j++) wband[j] = Wp + (size_t)min(bn * NT + j, n_tiles - 1) * k_tiles * 64 + lane;

    // X staging: a step's piece of X is MR rows x PP 16-byte pieces (piece pp = 2 x tile + k half); a load instruction
    // covers RPI rows, lane = row x PP + piece; rows past M re-read row M - 1 (an output row depends on its own X row
    // only, and rows >= M are never stored)
    const int prow = lane / PP, pp = lane % PP;
    dc_u32x4_t *xw = smem + wave * (PP * MR);
    const T *x16[XQ];
#pragma unroll
    for (int q = 0; q < XQ; q++) x16[q] = X + (size_t)min(prow + q * RPI, M - 1) * K + (pp & 1) * 8;

    f32x16_t acc[NT];
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[j][r] = 0.f;

    dc_u32x4_t xr[D][XQ];   // a native vector type: the ring must stay in registers
    Frag wf[D][KPW][NT];
    // Steps past the end of the split (the last round of the ring) are dead: their loads are clamped to its last step
    // and their X operand is zeroed at use, as for k tiles past the end of k.
#define FG_DC_KT0(step) (((step_lo + max(min((step), n_steps - 1), 0)) * DC_WAVES + wave) * KPW)
#define FG_DC_LOAD(slot, step)                                                                                     \
    do {                                                                                                           \
        const int kt0_ = FG_DC_KT0(step);                                                                          \
        _Pragma("unroll") for (int q = 0; q < XQ; q++)                                                             \
            xr[slot][q] = *reinterpret_cast<const dc_u32x4_t *>(x16[q] + (size_t)min(kt0_ + (pp >> 1), k_tiles - 1) * 16); \
        _Pragma("unroll") for (int i = 0; i < KPW; i++)                                                            \
            _Pragma("unroll") for (int j = 0; j < NT; j++)                                                         \
                wf[slot][i][j].u = dc_load_stream(wband[j] + (size_t)min(kt0_ + i, k_tiles - 1) * 64);             \
    } while (0)

#pragma unroll
    for (int d = 0; d < D; d++) FG_DC_LOAD(d, d);
    // The loop below has no barrier to hold its loads in place, and left alone the scheduler sinks every load to just
    // before its use (load, wait for everything, MFMA: no ring at all).  Nothing may move across these fences.
    __builtin_amdgcn_sched_barrier(0);

    // whole rounds of the ring with no branch inside, so that the load counter's waits are exact
    for (int s0 = 0; s0 < n_steps; s0 += D) {
#pragma unroll
        for (int d = 0; d < D; d++) {
            const bool live = s0 + d < n_steps;
            const int kt0 = FG_DC_KT0(s0 + d);
            // this wave's piece of the step: registers -> its LDS corner (piece-major, the row XOR-ed with the piece so
            // that neither side meets bank conflicts) -> operand order
#pragma unroll
            for (int q = 0; q < XQ; q++)
                if (prow + q * RPI < MR) xw[pp * MR + ((prow + q * RPI) ^ (pp & (MR - 1)))] = xr[d][q];
            Frag xa[KPW];
#pragma unroll
            for (int i = 0; i < KPW; i++) {
                const dc_u32x4_t v = xw[(2 * i + khalf) * MR + ((row ^ (2 * i + khalf)) & (MR - 1))];   // rows past MR: some real row's
                xa[i].u = live && kt0 + i < k_tiles ? make_uint4(v.x, v.y, v.z, v.w) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int i = 0; i < KPW; i++)
#pragma unroll
                for (int j = 0; j < NT; j++) acc[j] = mfma32<T>(xa[i], wf[d][i][j], acc[j]);
            __builtin_amdgcn_sched_barrier(0);
            FG_DC_LOAD(d, s0 + d + D);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef FG_DC_LOAD
#undef FG_DC_KT0
    __syncthreads();   // the reduction buffer takes the place of the staging corners

    // The eight k-tile partials meet in LDS, eight rows at a time: a lane's 16 accumulators of a band are four groups
    // of four consecutive rows (group q: rows 8 q + 4 (lane / 32) + 0..3, column lane % 32).  Wave j sums band j
    // (SwiGLU: wave p sums the gate band 2 p and the up band 2 p + 1 of the same 32 features).
    constexpr int NSUM = EPI == EPI_SWIGLU ? 2 : 1;
    const int j0 = wave * NSUM, b0 = bn * NT + j0, col = lane & 31;
    const bool summing = wave < NT / NSUM && b0 + NSUM - 1 < n_tiles;
#pragma unroll
    for (int q = 0; q < MR / 8; q++) {
        if (8 * q >= M) break;
        if (q > 0) __syncthreads();
#pragma unroll
        for (int j = 0; j < NT; j++)
            red[(wave * NT + j) * 64 + lane] = (dc_f32x4_t){acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]};
        __syncthreads();
        if (!summing) continue;
        dc_f32x4_t s[NSUM];
#pragma unroll
        for (int u = 0; u < NSUM; u++) {
            s[u] = red[(j0 + u) * 64 + lane];
#pragma unroll
            for (int w = 1; w < DC_WAVES; w++) s[u] += red[(w * NT + j0 + u) * 64 + lane];
        }
        const int m0 = 8 * q + 4 * (lane >> 5);
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int m = m0 + k;
            if (m >= M) continue;
            if (EPI == EPI_SLABS) {
                reinterpret_cast<float *>(out)[((size_t)z * M + m) * N + b0 * 32 + col] = s[0][k];
            } else {
                const float g = s[0][k], u = s[NSUM - 1][k];
                reinterpret_cast<T *>(out)[(size_t)m * (N >> 1) + (b0 >> 1) * 32 + col] = from_f<T>(swiglu_f(g, u));
            }
        }
    }
}

bool gemm_mfma_decode_ok(int M, int N, int K, int epilogue)
{
    if (M < 1 || M > DC_MAX_ROWS || K % 64 || N % 32 || K < 64) return false;
    return epilogue == EPI_SLABS || (epilogue == EPI_SWIGLU && N % 64 == 0);
}

// Block shapes.  WIDE (gate/up, the LM head): six bands, one k tile per wave and step, two steps ahead (12 KiB in
// flight per wave).  Measured on the 7B-class gate/up at 8 rows, kernel durations: 42.8 us; three or four steps ahead
// 45.6 / 44.8, two tiles per step one or two steps ahead 44.9 / 46.0, eight bands (148 blocks) 50.8.  NARROW (QKV, O,
// down): one band, four k tiles per step (whole 128-byte lines of X), four steps ahead (16 KiB).
struct DcShape { int nt, kpw; };
static DcShape decode_shape(int N) { return N >= 16384 ? DcShape{6, 1} : DcShape{1, 4}; }

// k splits of the partial-slab epilogue: as many as keep the grid within one block per CU, every split at least two
// steps long, no empty split.
int gemm_mfma_decode_split_for(int M, int N, int K)
{
    (void)M;
    const DcShape sh = decode_shape(N);
    const int blocks_n = (N / 32 + sh.nt - 1) / sh.nt, n_steps = (K / 16 + DC_WAVES * sh.kpw - 1) / (DC_WAVES * sh.kpw);
    int s = 256 / blocks_n;
    if (s > 16) s = 16;
    if (s > n_steps / 2) s = n_steps / 2;
    if (s < 1) s = 1;
    const int sps = (n_steps + s - 1) / s;
    return (n_steps + sps - 1) / sps;
}

template <typename T, int MR, int NT, int KPW, int D, int EPI>
static void launch_decode(const void *x, const void *wp, void *out, int M, int N, int K, int split, hipStream_t st)
{
    const int blocks_n = (N / 32 + NT - 1) / NT, n_steps = (K / 16 + DC_WAVES * KPW - 1) / (DC_WAVES * KPW);
    const int sps = (n_steps + split - 1) / split;   // a split past the end of k writes a slab of zeros
    hipLaunchKernelGGL((gemm_mfma_decode_kernel<T, MR, NT, KPW, D, EPI>), dim3(blocks_n * split), dim3(DC_WAVES * 64), 0, st,
                       reinterpret_cast<const T *>(x), reinterpret_cast<const uint4 *>(wp), out, M, N, K, blocks_n, sps);
}

template <typename T, int MR>
static void launch_decode_rows(const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split, hipStream_t st)
{
    const bool wide = decode_shape(N).nt == 6;
    if (epilogue == EPI_SWIGLU) {
        if (wide) launch_decode<T, MR, 6, 1, 2, EPI_SWIGLU>(x, wp, out, M, N, K, 1, st);
        else launch_decode<T, MR, 2, 2, 4, EPI_SWIGLU>(x, wp, out, M, N, K, 1, st);
    } else {
        if (wide) launch_decode<T, MR, 6, 1, 2, EPI_SLABS>(x, wp, out, M, N, K, split, st);
        else launch_decode<T, MR, 1, 4, 4, EPI_SLABS>(x, wp, out, M, N, K, split, st);
    }
}

// Shapes were validated by the caller (launch_gemm_mfma).
int32_t launch_gemm_mfma_decode(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split,
                                hipStream_t st)
{
    if (!gemm_mfma_decode_ok(M, N, K, epilogue))
        return fail(FG_ERR_SHAPE, "decode GEMM: shape %d x %d x %d with epilogue %d not supported", M, N, K, epilogue);
    if (dtype == FG_BF16) {
        if (M <= 8) launch_decode_rows<bf16_t, 8>(x, wp, out, M, N, K, epilogue, split, st);
        else launch_decode_rows<bf16_t, 16>(x, wp, out, M, N, K, epilogue, split, st);
    } else {
        if (M <= 8) launch_decode_rows<f16_t, 8>(x, wp, out, M, N, K, epilogue, split, st);
        else launch_decode_rows<f16_t, 16>(x, wp, out, M, N, K, epilogue, split, st);
    }
    FG_LAUNCH_CHECK("gemm_mfma_decode");
    return FG_OK;
}

}  // namespace fg
