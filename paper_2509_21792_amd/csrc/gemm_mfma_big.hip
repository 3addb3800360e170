// Compute-bound shape of the 16-bit MFMA GEMM (more than 256 rows): out = X . W^T on (32 MT) x 256 tiles, MT = 8, 5 or 4
// (6 / 7 for one row block of 161 - 192 / 193 - 224 rows of a wide output: 67 against 80 us for the 7B-class gate/up at
// 192 rows).
//
// Block = 4 waves side by side, each owning 32 MT rows x 64 columns (MT x 2 tiles of v_mfma_f32_32x32x16).  MT = 8
// fills the register file with one wave per SIMD, so nothing hides a stall and both operands are requested two
// 64-wide k chunks ahead; MT = 4 leaves room for a second block per CU, whose main loop covers the first one's
// prologue and epilogue (and doubles the number of tiles for the narrow outputs, which otherwise leave CUs idle):
//   W  packed fragments, global -> registers, two register sets that alternate by chunk; the set of chunk c is
//      refilled with chunk c + 2 fragment by fragment right after the MFMAs that consumed it;
//   X  row-major activations, global -> LDS directly (buffer_load_dwordx4 ... lds: 64 lanes x 16 bytes land in 1 KiB of
//      consecutive LDS), into a ring of three stages.  A stage holds 32 MT rows x 128 bytes; the 16-byte
//      piece p of row r holds the k octet p ^ ((r >> 1) & 7).  The permutation is applied to the *global*
//      address each lane requests (a row's eight lanes still cover its 128 contiguous bytes), and makes the
//      ds_read_b128 fragment reads (16 lanes = 16 rows, one octet) fall into 16 different bank groups.
// One barrier per chunk, placed before the last k tile: by then every wave has read all fragments of the current
// stage, so the stage can be handed to the loads of chunk c + 3 while the last MFMAs run and the first
// fragments of the next chunk are read.
//
// vmcnt bookkeeping (loads retire in issue order).  Per chunk a wave issues, in this order: the W fragments of k
// tiles 0-2 (6 loads), [wait + barrier], the MT X loads, the W fragments of k tile 3 (2 loads).  At the wait of
// chunk c the X loads of chunk c + 1 (issued two chunks earlier) must have landed; younger than them are
// 2 + 6 + MT + 2 + 6 = 16 + MT loads, hence s_waitcnt vmcnt(16 + MT).  The prologue issues its loads in the same
// interleaving so that the count holds from the first chunk on, and chunks past the end are clamped (re-requested),
// not skipped, so that it holds to the last.  Scheduling barriers pin the loads to their side of each wait.
//
// Launches of one row block of a wide output use blocks of 192 columns instead: three waves own columns, the fourth only
// brings its share of X and keeps the barriers (see plan_big for why).
//
// Epilogues (no k split for the last three): fp32 slabs; SwiGLU of interleaved gate / up tiles; the QKV projection's
// RoPE + KV append + q rows; residual add into the fp32 stream; per-block top-k / log-sum-exp partials of an LM head.
#include "fg_common.h"
#include "gemm_mfma.h"

namespace fg {

constexpr int BIG_STAGES = 3;

// s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt << 4 | lgkmcnt << 8 | vmcnt[5:4] << 14
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | (7 << 4) | ((lgkm & 15) << 8) | ((vm >> 4) << 14); }

// ---- epilogues of a wave's MT x 2 tiles (columns of tiles nt0 and nt1, rows row0 ..) ---------------------------------
// A lane holds column lane % 32 of each tile and rows 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4 of the block.

// QKV projection: a wave's two tiles are the columns e and e + hd/2 of one head, so a lane holds both members of every
// rotate-half pair of its rows.  q and k rows leave through a 4 KiB transposing tile in LDS (one per wave, 32 rows at a
// time): the accumulator layout has a lane on one column of 16 rows, the stores want 16 contiguous bytes of one row --
// 8 consecutive head dims, which are contiguous in q rows and in both K page layouts.  LDS serves a wave's accesses in
// order, so the tile needs no barrier.  v takes the same tile the other way round (see there).
template <typename T, int MT>
__device__ __forceinline__ void epilogue_rope(f32x16_t (&acc)[MT][2], const GemmEpi &ep, int M, int row0, int nt0, int n_tiles,
                                              int lane, T *tile)
{
    if (nt0 >= n_tiles) return;
    const int hd = ep.hd, half = hd >> 1, Hq = ep.Hq, Hkv = ep.Hkv;
    const int head = (nt0 * 32) / hd;              // the same for the whole wave
    const int ebase = nt0 * 32 - head * hd;        // head dim of the low tile's first column
    const int c = lane & 31, rh = (lane >> 5) * 4;
    const size_t page_elems = (size_t)16 * hd;
    if (head >= Hq + Hkv) {
        // v: the pages are transposed ([dim][token], a dim's 16 tokens = 32 bytes), so what is contiguous in memory is a
        // run of rows (the consecutive cache slots of one sequence's new nodes) at one dim.  Stored from the accumulator
        // layout, a wave instruction puts 64 two-byte values into 64 different sectors and a sector is written once per
        // node (33 MB of write traffic for 2 MB of v at 2048 rows, 18 us of this kernel's 94).  Through the tile, with
        // the lanes of a store running over eight consecutive rows first, a sector gets its new tokens in one write.
        // A row's columns are rotated by two per row in the tile, so that the eight rows a group of lanes reads lie in
        // eight different banks.
        const int hk = head - Hq - Hkv;
        T *vp = reinterpret_cast<T *>(ep.v_pool) + ((size_t)ep.layer * ep.n_pages * Hkv + hk) * page_elems;
        const int lr = lane & 7, lc = lane >> 3;
        // the cache cells of all the lane's rows in one batch of loads (every round trip of this epilogue is exposed)
        int cellv[MT][4];
#pragma unroll
        for (int i = 0; i < MT; i++)
#pragma unroll
            for (int a = 0; a < 4; a++) {
                const int m = row0 + i * 32 + lr + 8 * a;
                cellv[i][a] = m < M ? ep.dest[m] : -1;
            }
#pragma unroll
        for (int i = 0; i < MT; i++) {
            if (row0 + i * 32 >= M) break;
            T *dst[4];   // where this lane's four rows of the tile go: the row's page and slot (nullptr: not appended)
#pragma unroll
            for (int a = 0; a < 4; a++) {
                const int cell = cellv[i][a];
                dst[a] = cell >= 0 ? vp + (size_t)(cell >> 4) * Hkv * page_elems + (cell & 15) : nullptr;
            }
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int rr = 8 * (r >> 2) + rh + (r & 3);
                tile[rr * 64 + ((c + 2 * rr) & 63)] = from_f<T>(acc[i][0][r]);
                tile[rr * 64 + ((32 + c + 2 * rr) & 63)] = from_f<T>(acc[i][1][r]);
            }
#pragma unroll
            for (int it = 0; it < 32; it++) {
                const int a = it & 3, rr = lr + 8 * a, cc = lc + 8 * (it >> 2);
                const T v = tile[rr * 64 + ((cc + 2 * rr) & 63)];
                const int e = cc < 32 ? ebase + cc : ebase + half + cc - 32;
                if (dst[a]) dst[a][e * 16] = v;
            }
        }
        return;
    }
    const bool is_q = head < Hq;
    T *kp = reinterpret_cast<T *>(ep.k_pool);
    const int hk = head - Hq;
    // Every global round trip of this epilogue is exposed (one wave per SIMD, nothing else to run), so there are as few
    // as possible: the positions of all the lane's rows in one batch (groups of four consecutive rows; the position
    // array is padded to a multiple of 64 entries by its 256-byte alignment in the workspace), then the table entries
    // one row tile ahead of the tile being rotated.
    int4 p4[MT][4];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int m0 = row0 + i * 32 + 8 * q + rh;
            p4[i][q] = m0 < M ? *reinterpret_cast<const int4 *>(ep.pos + m0) : make_int4(0, 0, 0, 0);
        }
    int cellk[MT][4];   // k rows: the cache cell of row (lane / 8) + 8 t of each row tile, fetched with the positions
    if (!is_q) {
#pragma unroll
        for (int i = 0; i < MT; i++)
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const int m = row0 + i * 32 + (lane >> 3) + 8 * t;
                cellk[i][t] = m < M ? ep.dest[m] : -1;
            }
    }
    // table and q rows through buffer descriptors: 32-bit offsets, and a q row past the last one is dropped by the
    // address check instead of by a branch
    typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t trs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float2 *>(ep.rope_tab), 0, ep.max_pos * half * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t qrs = __builtin_amdgcn_make_buffer_rsrc(ep.q_out, 0, M * Hq * hd * 2, 0x00020000);
    float2 cs[2][16];
    auto load_table = [&](int i, float2 (&dst)[16]) {
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int4 v = p4[i][r >> 2];
            const int pr = (r & 3) == 0 ? v.x : ((r & 3) == 1 ? v.y : ((r & 3) == 2 ? v.z : v.w));
            const int p = min(max(pr, 0), ep.max_pos - 1);
            const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(trs, (p * half + ebase + c) * 8, 0, 0);
            dst[r] = make_float2(__uint_as_float(t.x), __uint_as_float(t.y));
        }
    };
    load_table(0, cs[0]);
#pragma unroll
    for (int i = 0; i < MT; i++) {
        if (i + 1 < MT) load_table(i + 1, cs[(i + 1) & 1]);
        if (row0 + i * 32 < M) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int rr = 8 * (r >> 2) + rh + (r & 3);
                const float a = acc[i][0][r], b = acc[i][1][r];
                const float2 t = cs[i & 1][r];
                tile[rr * 64 + c] = from_f<T>(a * t.x - b * t.y);
                tile[rr * 64 + 32 + c] = from_f<T>(b * t.x + a * t.y);
            }
            // 256 pieces of 16 bytes: piece = (row, segment); segments 0-3 are dims ebase + 8 s .., 4-7 the rotated partners
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const int piece = lane + 64 * t, rr = piece >> 3, seg = piece & 7;
                const uint4 v = *reinterpret_cast<const uint4 *>(tile + rr * 64 + seg * 8);
                const int m = row0 + i * 32 + rr;
                const int e = seg < 4 ? ebase + seg * 8 : ebase + half + (seg - 4) * 8;
                if (is_q) {
                    __builtin_amdgcn_raw_buffer_store_b128((u32x4_t){v.x, v.y, v.z, v.w}, qrs, ((m * Hq + head) * hd + e) * 2, 0, 0);
                } else {
                    const int cell = cellk[i][t], page = cell >> 4, tk = cell & 15;
                    if (cell >= 0) {   // -1: beyond the page table (or past the last row), not appended
                        T *o = kp + (((size_t)ep.layer * ep.n_pages + page) * Hkv + hk) * page_elems;
                        *reinterpret_cast<uint4 *>(o + k_page_offset(ep.k_frag, hd, tk, e)) = v;
                    }
                }
            }
        }
    }
}

// LM head: per row and per 256-column block, the topk largest outputs (value, column; ties to the lower column) and
// the block's (max, sum exp(x - max)), so that no [M, vocab] tensor has to exist.  The accumulator layout has a lane on
// one column of 16 rows; the selection wants a row's 256 columns together.  16 rows at a time go through a
// 16 x 256 fp32 tile in LDS (stage 0 of the main loop, free by now): the four waves write their 64 columns each, then a
// row belongs to 16 consecutive lanes, a lane holding the columns 4 s + 64 v + u (s = lane % 16; v, u = 0..3 -- the
// float4 reads of 16 lanes cover all 64 banks).  topk rounds follow: every lane offers its best entry that comes after
// the previous winner in the order (value descending, column ascending), a 4-step exchange inside the 16 lanes picks
// the round's winner.
// float bits -> unsigned whose order is the values' order (and back); no NaNs here
__device__ __forceinline__ unsigned topk_ord(float x)
{
    const unsigned u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float topk_unord(unsigned k) { return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k); }

template <int MT>
__device__ __forceinline__ void epilogue_topk(f32x16_t (&acc)[MT][2], const GemmEpi &ep, int M, int N, int row0, int bx, int n_bands,
                                              int wn, int lane, float *tile)
{
    const int c = lane & 31, hsel = lane >> 5, tid = wn * 64 + lane;
    const int row16 = tid >> 4, seg = tid & 15;
    const int K = ep.topk;
#pragma unroll
    for (int i = 0; i < MT; i++) {
#pragma unroll
        for (int half = 0; half < 2; half++) {
            // (no early exit from the unrolled loops: the accumulators must stay in registers, indexed by constants)
            if (row0 + i * 32 + half * 16 < M) {   // the same for the whole block
            __syncthreads();                              // the previous tile's readers are done
#pragma unroll
            for (int qq = 0; qq < 2; qq++)
#pragma unroll
                for (int k = 0; k < 4; k++)
#pragma unroll
                    for (int j = 0; j < 2; j++)
                        tile[(8 * qq + 4 * hsel + k) * 256 + wn * 64 + j * 32 + c] = acc[i][j][4 * (2 * half + qq) + k];
            __syncthreads();
            // An entry travels as one 64-bit key: the value's bits mapped so that unsigned order is value order, above the
            // complemented column -- a larger key comes first in (value descending, column ascending).  A round is then
            // "the largest key below the previous winner": two compares and four selects per entry and no branch (written
            // with the pair comparison the compiler produced a compare-and-branch ladder per entry, ~20 instructions).
            // Columns past the matrix get the key 0 | ~0x7fffffff, below every real entry; -0 is folded into +0 first so
            // that the two still tie.
            unsigned long long key[16];
#pragma unroll
            for (int vv = 0; vv < 4; vv++) {
                const float4 x = *reinterpret_cast<const float4 *>(tile + row16 * 256 + seg * 4 + 64 * vv);
                const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const int cc = bx * 256 + seg * 4 + 64 * vv + u;
                    key[4 * vv + u] = cc < N ? ((unsigned long long)topk_ord(xs[u] + 0.f) << 32) | (unsigned)~cc : 0x80000000ull;
                }
            }
            const int m = row0 + i * 32 + half * 16 + row16;
            unsigned long long prev = ~0ull;
            float bmax = -INFINITY;
            for (int k = 0; k < K; k++) {
                unsigned long long best = 0;
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const unsigned long long cand = key[e] < prev ? key[e] : 0ull;
                    best = cand > best ? cand : best;
                }
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) {
                    const unsigned long long ob = ((unsigned long long)__shfl_xor((unsigned)(best >> 32), o, 64) << 32) |
                                                  __shfl_xor((unsigned)best, o, 64);
                    best = ob > best ? ob : best;
                }
                const unsigned hi = (unsigned)(best >> 32);
                const float bv = hi ? topk_unord(hi) : -INFINITY;          // nothing left in the block: (-inf, no column)
                const int bi = hi ? (int)~(unsigned)best : 0x7fffffff;
                if (k == 0) bmax = bv;
                prev = best;
                if (seg == 0 && m < M) {
                    const size_t at = ((size_t)m * n_bands + bx) * K + k;
                    ep.part_val[at] = bv;
                    ep.part_idx[at] = bi;
                }
            }
            if (ep.part_ms) {
                float sum = 0.f;
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const unsigned hi = (unsigned)(key[e] >> 32);
                    const float ve = hi ? topk_unord(hi) : -INFINITY;
                    sum += ve > -INFINITY ? __expf(ve - bmax) : 0.f;
                }
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o, 64);
                if (seg == 0 && m < M) {
                    ep.part_ms[((size_t)m * n_bands + bx) * 2] = bmax;
                    ep.part_ms[((size_t)m * n_bands + bx) * 2 + 1] = sum;
                }
            }
            }
        }
    }
}

// WA = waves of the block that own columns: 4, or 3 or 2 for launches that are weight streams (see plan_big): the block
// is then 192 or 128 columns wide, and its other waves only bring their share of X and keep the block's barriers.
template <typename T, int MT, int EPI, int WA = 4>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(MT == 4 ? 2 : 1))) void gemm_mfma_big_kernel(const T *__restrict__ X, const uint4 *__restrict__ Wp,
                                                             void *__restrict__ out, int M, int N, int K, int chunks_per_split,
                                                             int n_bands, int row_blocks, int per_xcd, int n_tile_total, GemmEpi ep)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-descriptor builtins exist in the device pass only
    constexpr int NT = 2, WN = 4, BM = MT * 32;
    static_assert(WA == 4 || ((WA == 3 || WA == 2) && (EPI == EPI_SLABS || EPI == EPI_SWIGLU)), "the narrower blocks have the barrier-free epilogues");
    constexpr int STAGE_U4 = BM * 8;   // uint4 slots per stage: BM rows x 8 pieces
    // one variable per stage: the compiler orders LDS reads after direct-to-LDS loads per variable, so distinct
    // variables keep the reads of one stage from waiting on the loads in flight to the others
    __shared__ uint4 xs0[STAGE_U4], xs1[STAGE_U4], xs2[STAGE_U4];

    const int tid = threadIdx.x, lane = tid & 63, wn = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_tiles = N >> 5, k_tiles = K >> 4;
    // Block -> tile.  Workgroups are dealt to the 8 XCDs round-robin by linear id; XCD x takes the tiles
    // x * per_xcd .. (x + 1) * per_xcd - 1 of the order (k split, column band, row block), row block fastest: every XCD
    // gets the same number of tiles (to within one), and the ~32 tiles resident on it are a few adjacent bands times
    // all row blocks, which share W bands and X row blocks through its L2.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int tile_id = xcd * per_xcd + local;
    if (local >= per_xcd || tile_id >= n_tile_total) return;
    const int per_split = n_bands * row_blocks;
    const int bz = tile_id / per_split, rem = tile_id - bz * per_split;
    const int bx = rem / row_blocks, by = rem - bx * row_blocks;
    const int row0 = by * BM;
    // the wave's two column tiles: adjacent ones, except for the QKV epilogue with 128-wide heads, where a wave takes
    // the tiles 64 columns apart that hold the two members of the rotate-half pairs
    int ntile[NT];
    if (EPI == EPI_ROPE && ep.hd == 128) {
        ntile[0] = bx * 8 + (wn >> 1) * 4 + (wn & 1);
        ntile[1] = ntile[0] + 2;
    } else {
        ntile[0] = (bx * WA + wn) * NT;
        ntile[1] = ntile[0] + 1;
    }
    const int total_chunks = k_tiles / KT;
    const int c_begin = bz * chunks_per_split;
    const int c_end = min(c_begin + chunks_per_split, total_chunks);
    const int n_chunks = c_end - c_begin;
    if (n_chunks <= 0) return;

    // The accumulators start at zero -- or, for the residual epilogue, at the tile of h they are added to: those loads
    // fly with the prologue's, and the epilogue is then a plain store.
    f32x16_t acc[MT][NT];
    if (EPI == EPI_RESIDUAL) {
        // through a descriptor that ends with the matrix (or the block's rows): a row past it reads as zero, no branches
        const int rows = min(M - row0, BM);
        const __amdgpu_buffer_rsrc_t hrs = __builtin_amdgcn_make_buffer_rsrc(ep.h + (size_t)row0 * N, 0, rows * N * 4, 0x00020000);
#pragma unroll
        for (int j = 0; j < NT; j++) {
            const unsigned off0 = ntile[j] < n_tiles ? (unsigned)(((lane >> 5) * 4 * N + ntile[j] * 32 + (lane & 31)) * 4) : 0xc0000000u;
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int r = 0; r < 16; r++)
                    acc[i][j][r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                        hrs, (int)(off0 + (unsigned)((i * 32 + 8 * (r >> 2) + (r & 3)) * N * 4)), 0, 0));
        }
    } else {
#pragma unroll
        for (int i = 0; i < MT; i++)
#pragma unroll
            for (int j = 0; j < NT; j++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;
    }

    // W: lane pointer into each of the wave's two bands (clamped on a ragged last block; never stored)
    const uint4 *wband[NT];
#pragma unroll
    for (int j = 0; j < NT; j++) {
        int t = min(ntile[j], n_tiles - 1);
        wband[j] = Wp + ((size_t)t * k_tiles) * 64 + lane;
    }
    // X: wave wn brings rows 8 MT wn .. 8 MT (wn + 1) - 1 of the block, 8 rows per load; lane = (row in the 8, piece p)
    int xoff[MT];
#pragma unroll
    for (int i = 0; i < MT; i++) {
        const int r = wn * (MT * 8) + i * 8 + (lane >> 3), p = lane & 7;
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
    _Pragma("unroll") for (int i = 0; i < MT; i++) __builtin_amdgcn_raw_ptr_buffer_load_lds(              \
        xrsrc, (stage) + (wn * (MT * 8) + i * 8) * 8, 16, xoff[i], __builtin_amdgcn_readfirstlane((chunk) * 128), 0, 0)
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

    if constexpr (WA < WN) {
        if (wn >= WA) {
            // A wave without columns: the same X loads and barriers as the others, nothing else.  At the barrier of chunk
            // c its loads of chunk c + 1 must have landed; younger than them are those of chunk c + 2 alone.
            FG_X_ISSUE(c_begin, xs0);
            FG_X_ISSUE(clampc(c_begin + 1), xs1);
            FG_X_ISSUE(clampc(c_begin + 2), xs2);
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * MT, 0));
            __builtin_amdgcn_s_barrier();
#define FG_HELPER(c, st)                                        \
    do {                                                        \
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(MT, 0));         \
        __builtin_amdgcn_s_barrier();                           \
        FG_FENCE();                                             \
        FG_X_ISSUE(clampc((c) + 3), st);                        \
        FG_FENCE();                                             \
    } while (0)
            int c = c_begin;
            for (; c + 2 < c_end; c += 3) {
                FG_HELPER(c, xs0);
                FG_HELPER(c + 1, xs1);
                FG_HELPER(c + 2, xs2);
            }
            if (c < c_end) FG_HELPER(c, xs0);
            if (c + 1 < c_end) FG_HELPER(c + 1, xs1);
#undef FG_HELPER
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
            return;
        }
    }

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
    // X(0) landed.  Only the 2 MT direct-to-LDS loads behind it are counted: the compiler may move the register
    // loads of the prologue, and a stricter wait costs nothing here.
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(2 * MT, 0));
    __builtin_amdgcn_s_barrier();
    FG_FENCE();
    FG_X_READ(xa, xs0, 0);

    // One chunk: `cur` holds its W fragments and is refilled with chunk c + 2; st = its stage, sn = the next one.
    // Within a k tile the instruction stream is laid out as MT x {2 MFMAs, 1 fragment read (, 1 X load)} followed by
    // the two W loads, so that the LDS and memory instructions issue under the running MFMAs instead of in a clump.
#define FG_PIPE(with_x)                                                                               \
    _Pragma("unroll") for (int q = 0; q < MT; q++) {                                                  \
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
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(16 + MT, 0));                                          \
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

    if (EPI == EPI_ROPE) {
        __syncthreads();   // every wave has drained its loads into, and finished reading, the stages: stage 0 is free
        epilogue_rope<T, MT>(acc, ep, M, row0, ntile[0], n_tiles, lane, reinterpret_cast<T *>(xs0) + wn * 2048);
    } else if (EPI == EPI_RESIDUAL) {
        store_tiles<T, MT, NT, EPI_SLABS>(acc, ep.h, M, N, row0, ntile[0], n_tiles, 0, lane);
    } else if (EPI == EPI_TOPK) {
        epilogue_topk<MT>(acc, ep, M, N, row0, bx, n_bands, wn, lane, reinterpret_cast<float *>(xs0));
    } else {
        store_tiles<T, MT, NT, EPI>(acc, out, M, N, row0, ntile[0], n_tiles, bz, lane);
    }
#endif
}

// Split and block-height choice.  Tiles are dealt evenly to the 8 XCDs and then to their 32 CUs, so the busiest CU runs
// ceil(ceil(tiles / 8) / 32) blocks one after the other (or side by side, sharing the matrix pipe: the same time); a
// block costs the split's chunks plus about 8 chunk-times of prologue and epilogue, a chunk 1.45 us for 256 rows and in
// proportion (+9 %) for shorter blocks; every extra split adds an fp32 slab the consumer has to read back.  Measured
// on the 7B-class shapes (us, 2048 rows): QKV 99 in 256-row blocks (144 tiles), 103 in 128-row blocks (288), against
// 61 predicted for 160-row blocks (234 tiles, one round); O 92 / 55 (256 / 128 rows); down 414 / 241, 236 with two
// splits of 256-row blocks.  The wide outputs (gate/up, LM head) have thousands of tiles.  128-row blocks, two to a CU,
// put each one's prologue and epilogue under the other's main loop but draw half as much again from L2 per flop
// (53.0 M against 35.5 M line requests for gate/up at 2048 rows); 256-row blocks leave their epilogue exposed, which
// an exact-division SwiGLU made expensive.  With the reciprocal-instruction SwiGLU a block's time is close to
// proportional to its height, with 8 % more per row for 160-row blocks and 17 % more for 128-row ones, and the launch
// takes as many of them as the busiest CU runs one after the other: ceil(tiles / 256) rounds.  That count decides the
// height of the wide outputs (wide_height below); it reproduces every measured ordering of gate/up (us, 256- / 160- /
// 128-row blocks): 64 at 128 rows in one 128-row block; 82 / 68 / 106 at 160 rows; 86 / 116 / 106 at 256; 160 / 132 /
// 109 at 384; 152 in 128-row blocks at 512; 197 / - / 208 at 768; level at 1024; 294 / - / 310 at 1280; 461 / - / 486
// at 2048; 886 / - / 927 at 4096.
// The residual and top-k epilogues exist for 128- and 160-row blocks only: with 256 accumulator registers per lane the
// extra live values of those epilogues (the tile of h, the selection's scratch) do not fit and the compiler spills.
// A launch of at most 256 blocks with one block per CU is a weight stream, and a CU draws a bounded rate from HBM
// whatever it keeps in flight -- 47 - 55 GB/s in a pure read stream with 32 KiB in flight as with 128, about 30 here (gate/up in one row of 148 blocks: 55 - 64 us from 32 to 128 rows, the same with operands
// four chunks ahead instead of two; the decode kernel's 198 blocks: 43 us): what counts is the number of CUs that
// stream.  Such launches of a wide output therefore use the narrowest blocks (128 or 192 columns: wa = 2 or 3 column
// waves) that still give one round: 198 blocks for the 7B-class gate/up, 140 for the 1.5B-class one.
struct BigPlan { int split, mt, wa; };
static bool tall_blocks_ok(int epilogue) { return epilogue != EPI_RESIDUAL && epilogue != EPI_TOPK; }
static int column_waves(int M, int N, int mt, int split, int epilogue)
{
    if (N < 16384 || split != 1 || (epilogue != EPI_SLABS && epilogue != EPI_SWIGLU) || M > 32 * mt) return 4;
    for (int wa = 2; wa < 4; wa++)   // the narrowest block that still gives one round
        if ((N / 32 + 2 * wa - 1) / (2 * wa) <= 256) return wa;
    return 4;
}
// Blocks of the launch for one row block of a wide output (what the kernel choice looks at).
int gemm_mfma_big_stream_blocks(int N, int epilogue)
{
    const int wa = column_waves(1, N, 4, 1, epilogue);
    return (N / 32 + 2 * wa - 1) / (2 * wa);
}
static int wide_height(int M, int n_bands)
{
    static const int heights[5] = {8, 7, 6, 5, 4};
    static const double per_block[5] = {1.0, 1.03 * 7 / 8, 1.05 * 6 / 8, 1.08 * 5 / 8, 1.17 * 4 / 8};
    int best = 8;
    double best_cost = 1e30;
    for (int i = 0; i < 5; i++) {
        // 224- and 192-row blocks: built for one row block of 193 - 224 / 161 - 192 rows only
        if ((heights[i] == 7 && M > 224) || (heights[i] == 6 && M > 192)) continue;
        const long tiles = (long)n_bands * ((M + 32 * heights[i] - 1) / (32 * heights[i]));
        // over several rounds a 160-row block costs 19 % more per row than a 256-row one, not 8 (1792 rows: 450 us in
        // seven rounds of 160-row blocks against 432 in five of 256-row ones)
        const double per = heights[i] == 5 && tiles > 256 ? 1.19 * 5 / 8 : per_block[i];
        const double cost = (double)((tiles + 255) / 256) * per;
        if (cost < best_cost) { best_cost = cost; best = heights[i]; }   // ties go to the taller block: less L2 traffic
    }
    return best;
}
static BigPlan plan_big(int M, int N, int K, int fixed_split, int fixed_mt, int epilogue = EPI_SLABS)
{
    const int n_bands = (N / 32 + 7) / 8, chunks = K / 64;
    if (!tall_blocks_ok(epilogue) && fixed_mt == 8) fixed_mt = 0;
    if (N >= 16384 && fixed_mt <= 0) fixed_mt = tall_blocks_ok(epilogue) ? wide_height(M, n_bands) : 4;
    BigPlan best{fixed_split > 0 ? fixed_split : 1, fixed_mt > 0 ? fixed_mt : 8, 4};
    double best_cost = 1e30;
    static const int heights[5] = {8, 7, 6, 5, 4};
    for (int mt : heights) {
        if ((fixed_mt > 0 && mt != fixed_mt) || ((mt == 6 || mt == 7) && fixed_mt != mt)) continue;
        if (mt == 8 && !tall_blocks_ok(epilogue)) continue;
        const int row_blocks = (M + 32 * mt - 1) / (32 * mt);
        const int s_max = row_blocks == 1 ? 16 : 8;   // one row block: the slabs are small, the grid needs the splits
        const double chunk_us = 1.45 * mt / 8 * (mt == 8 ? 1.0 : 1.09);
        for (int s = 1; s <= s_max; s++) {
            if (fixed_split > 0 && s != fixed_split) continue;
            if (fixed_split <= 0 && s > 1 && chunks / s < 8) break;
            const int cps = (chunks + s - 1) / s;
            if ((chunks + cps - 1) / cps != s) continue;   // some split would be empty
            const int per_xcd = (n_bands * row_blocks * s + 7) / 8, per_cu = (per_xcd + 31) / 32;
            double cost = per_cu * (cps + (mt == 4 && per_cu >= 2 ? 2 : 8)) * chunk_us;
            cost += (s - 1) * (double)M * N * 4 * 1.3 / 4.5e6;
            if (cost < best_cost) { best_cost = cost; best = BigPlan{s, mt, 4}; }
        }
    }
    best.wa = column_waves(M, N, best.mt, best.split, epilogue);
    return best;
}

int gemm_mfma_big_split_for(int M, int N, int K) { return plan_big(M, N, K, 0, 0).split; }

// Tiles of the launch when the shape runs without a k split (what the fused epilogues need).
int gemm_mfma_big_unsplit_tiles(int M, int N, int K, int epilogue)
{
    const BigPlan p = plan_big(M, N, K, 1, 0, epilogue);
    return (N / 32 + 7) / 8 * ((M + 32 * p.mt - 1) / (32 * p.mt));
}

template <typename T, int MT>
static void launch_big_typed(const void *x, const void *wp, void *out, int M, int N, int K, int epilogue, int split, int wa,
                             const GemmEpi &ep, hipStream_t st)
{
    const int n_tiles = N / 32, per_block = 2 * wa;
    const int total_chunks = K / 64;
    const int cps = (total_chunks + split - 1) / split;
    const int n_bands = (n_tiles + per_block - 1) / per_block, row_blocks = (M + 32 * MT - 1) / (32 * MT);
    const int total = n_bands * row_blocks * split, per_xcd = (total + 7) / 8;
    const dim3 grid((unsigned)(8 * per_xcd));
#define FG_BIG_LAUNCH_K(...)                                                                                        \
    hipLaunchKernelGGL((gemm_mfma_big_kernel<__VA_ARGS__>), grid, dim3(256), 0, st, reinterpret_cast<const T *>(x), \
                       reinterpret_cast<const uint4 *>(wp), out, M, N, K, cps, n_bands, row_blocks, per_xcd, total, ep)
#define FG_BIG_LAUNCH(E) FG_BIG_LAUNCH_K(T, MT, E)
    switch (epilogue) {
    case EPI_SLABS:
        if (wa == 3) FG_BIG_LAUNCH_K(T, MT, EPI_SLABS, 3);
        else if (wa == 2) FG_BIG_LAUNCH_K(T, MT, EPI_SLABS, 2);
        else FG_BIG_LAUNCH(EPI_SLABS);
        break;
    case EPI_SWIGLU:
        if (wa == 3) FG_BIG_LAUNCH_K(T, MT, EPI_SWIGLU, 3);
        else if (wa == 2) FG_BIG_LAUNCH_K(T, MT, EPI_SWIGLU, 2);
        else FG_BIG_LAUNCH(EPI_SWIGLU);
        break;
    case EPI_ROPE:
        if constexpr (MT != 6 && MT != 7) FG_BIG_LAUNCH(EPI_ROPE);
        break;
    default:
        if constexpr (MT != 8 && MT != 7 && MT != 6) {   // the plan never pairs these epilogues with 256-, 224- or 192-row blocks
            if (epilogue == EPI_TOPK) FG_BIG_LAUNCH(EPI_TOPK);
            else FG_BIG_LAUNCH(EPI_RESIDUAL);
        }
        break;
    }
#undef FG_BIG_LAUNCH
#undef FG_BIG_LAUNCH_K
}

// Shapes were validated by the caller (launch_gemm_mfma); M * K < 2^30 is needed by the 32-bit byte offsets.
// fixed_mt: 0 = the plan's block height and width, else 8, 7, 6, 5 or 4 (row tiles of 32 per block) with 256-column blocks,
// or 18, 17, 16, 15, 14 / 24 = the same heights with 192- / 128-column blocks (partial-sum and SwiGLU epilogues).
int32_t launch_gemm_mfma_big(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue,
                             int split, int fixed_mt, const GemmEpi *epi, hipStream_t st)
{
    const int fixed_wa = fixed_mt == 0 ? 0 : (fixed_mt > 20 ? 2 : (fixed_mt > 10 ? 3 : 4));
    fixed_mt %= 10;
    if (fixed_wa && fixed_wa < 4 && epilogue != EPI_SLABS && epilogue != EPI_SWIGLU)
        return fail(FG_ERR_INVALID_ARG, "128- and 192-column blocks have the partial-sum and SwiGLU epilogues only (got %d)", epilogue);
    if ((int64_t)M * K >= (1LL << 30)) return fail(FG_ERR_SHAPE, "GEMM input of %d x %d exceeds 2^30 elements", M, K);
    if (epilogue >= EPI_ROPE && split != 1) return fail(FG_ERR_INVALID_ARG, "fused GEMM epilogue %d cannot run with a k split", epilogue);
    if (epilogue > EPI_TOPK) return fail(FG_ERR_UNIMPLEMENTED, "GEMM epilogue %d", epilogue);
    if (epilogue == EPI_TOPK && (epi->topk < 1 || epi->topk > 8 || !epi->part_val || !epi->part_idx))
        return fail(FG_ERR_INVALID_ARG, "top-k epilogue needs 1 <= k <= 8 and its partial buffers");
    if (epilogue >= EPI_ROPE && !epi) return fail(FG_ERR_INVALID_ARG, "GEMM epilogue %d needs its arguments", epilogue);
    if (epilogue == EPI_ROPE && (epi->hd != 64 && epi->hd != 128)) return fail(FG_ERR_SHAPE, "RoPE epilogue needs head_dim 64 or 128");
    if (epilogue == EPI_ROPE && ((int64_t)M * epi->Hq * epi->hd >= (1LL << 30) || (int64_t)epi->max_pos * epi->hd >= (1LL << 28)))
        return fail(FG_ERR_SHAPE, "RoPE epilogue: q output or rotation table beyond its 32-bit byte offsets");
    if ((fixed_mt == 6 || fixed_mt == 7) && epilogue != EPI_SLABS && epilogue != EPI_SWIGLU)
        return fail(FG_ERR_INVALID_ARG, "192- and 224-row blocks have the partial-sum and SwiGLU epilogues only (got %d)", epilogue);
    BigPlan p = plan_big(M, N, K, split, fixed_mt, epilogue);
    if (fixed_wa) p.wa = fixed_wa;
    const GemmEpi ep = epi ? *epi : GemmEpi();
#define FG_BIG_MT(T)                                                                                   \
    do {                                                                                               \
        if (p.mt == 8) launch_big_typed<T, 8>(x, wp, out, M, N, K, epilogue, split, p.wa, ep, st);           \
        else if (p.mt == 7) launch_big_typed<T, 7>(x, wp, out, M, N, K, epilogue, split, p.wa, ep, st);      \
        else if (p.mt == 6) launch_big_typed<T, 6>(x, wp, out, M, N, K, epilogue, split, p.wa, ep, st);      \
        else if (p.mt == 5) launch_big_typed<T, 5>(x, wp, out, M, N, K, epilogue, split, p.wa, ep, st);      \
        else launch_big_typed<T, 4>(x, wp, out, M, N, K, epilogue, split, p.wa, ep, st);                     \
    } while (0)
    if (dtype == FG_BF16) FG_BIG_MT(bf16_t);
    else FG_BIG_MT(f16_t);
#undef FG_BIG_MT
    FG_LAUNCH_CHECK("gemm_mfma_big");
    return FG_OK;
}

}  // namespace fg
