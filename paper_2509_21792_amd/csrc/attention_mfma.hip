// Tree-masked GQA attention over the paged cache on MFMA (16-bit operands, fp32 softmax and accumulation).
//
// Work item = (sequence, kv head, chunk of key positions).  All query rows that share the kv head -- the
// G = Hq / Hkv query heads of every new node, G * N rows -- ride the same pass over K and V, so each K/V byte
// is fetched from HBM once per (sequence, kv head) whatever N is.  A wave owns QW tiles of 16 query rows and
// walks the chunk 32 key positions (two 16-token pages) at a time:
//   S^T = K . Q^T        v_mfma_f32_16x16x32, A = K fragments straight from global memory (pages in fragment order),
//                        B = Q fragments held in registers for the whole pass;
//   online softmax       per query column; lanes l, l+16, l+32, l+48 hold the same column, 4 keys each;
//   O^T += V^T . P^T     A = V^T fragments straight from global memory (pages store V transposed, so the 4
//                        tokens a lane needs are 8 contiguous bytes), B = P^T taken from the S^T accumulators
//                        in place: the contraction order is chosen so that no cross-lane shuffle is needed.
// The contraction over head_dim is permuted as well (lane group g covers the contiguous quarter g of the row),
// and the cache keeps K pages in that fragment order, so that every K load of a wave is one contiguous KiB.
// Measured and set aside: K / V of two steps in flight through LDS stages (direct-to-LDS buffer loads, query
// fragments back in registers) instead of one step in a second register set: 305 against 291 us per layer at
// B = 256, N = 8.  A later attempt kept V in two alternating register sets and sent only K two steps ahead through
// two LDS stages (one variable each): parity-exact and slower again, 9.0 against 7.1 ms per verify step -- the compiler
// orders every LDS read, the per-step reads of the parked Q fragments included, behind all direct-to-LDS loads still in
// flight, so each step starts by waiting for the K loads it has just issued.  Chunks write (m, l, O) partials; a merge kernel
// combines them.  Key positions >= committed length are in-round nodes and are masked per query row with the
// node's 64-bit ancestor set.
#include <stdlib.h>

#include <type_traits>

#include "fg_common.h"

namespace fg {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

union Frag16 {
    uint4 u;
    uint2 u2[2];
    bf16x8_t b;
    f16x8_t h;
    uint16_t s[8];
};

template <typename T> __device__ __forceinline__ f32x4_t mfma16(const Frag16 &a, const Frag16 &b, f32x4_t c);
template <> __device__ __forceinline__ f32x4_t mfma16<bf16_t>(const Frag16 &a, const Frag16 &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.b, b.b, c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4_t mfma16<f16_t>(const Frag16 &a, const Frag16 &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, c, 0, 0, 0);
}
// two fp32 -> one packed pair of T, round to nearest even (v_cvt_pk_bf16_f32 / v_cvt_f16_f32 + pack)
template <typename T> __device__ __forceinline__ uint32_t pack2(float a, float b);
template <> __device__ __forceinline__ uint32_t pack2<bf16_t>(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t r;
    r[0] = (__bf16)a;
    r[1] = (__bf16)b;
    return *reinterpret_cast<uint32_t *>(&r);
}
template <> __device__ __forceinline__ uint32_t pack2<f16_t>(float a, float b)
{
    typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
    f16x2_t r;
    r[0] = (_Float16)a;
    r[1] = (_Float16)b;
    return *reinterpret_cast<uint32_t *>(&r);
}

constexpr float RESCALE_LOG2 = 8.f;

// Reductions over the four lanes l, l + 16, l + 32, l + 48 (one query column) with the row-swap instructions of
// gfx950: swapping a register with a copy of itself leaves (lower half, lower half) and (upper, upper).
__device__ __forceinline__ float group_max(float x)
{
    unsigned u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    u = __float_as_uint(x);
    r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float group_sum(float x)
{
    unsigned u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    u = __float_as_uint(x);
    r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

struct AttnPlan {
    int QR;        // padded query rows per (sequence, kv head): multiple of 16
    int waves;     // waves per block
    int CK;        // key positions per chunk (multiple of 32)
    int n_chunks;  // chunks covering max_keys
};

template <int QW>
static AttnPlan plan_attention(int B, int N, int Hq, int Hkv, int max_keys)
{
    AttnPlan p;
    const int G = Hq / Hkv, QT = (G * N + 15) / 16;
    p.QR = QT * 16;
    p.waves = (QT + QW - 1) / QW;
    const long pairs = (long)B * Hkv * p.waves;
    // work items aimed at: about two per wave slot of the chip.  Measured at B = 8, N = 1 (a 3.08 ms step): 256 items
    // 3.18 ms, 512 to 4096 items 3.08 - 3.09
    constexpr long target = 2048;
    long splits = (target + pairs - 1) / pairs;
    if (splits < 1) splits = 1;
    long ck = (max_keys + splits - 1) / splits;
    // keeps the partial (m, l, O) traffic under ~1/2 of the K/V traffic; binds for small batches only, where shorter
    // chunks mean more waves at work (B = 8, N = 24: 0.94 ms of attention per step with 4 QR, 0.80 with 2 QR or QR)
    long ck_min = 2L * p.QR;
    if (ck < ck_min) ck = ck_min;
    ck = (ck + 31) / 32 * 32;
    p.CK = (int)ck;
    p.n_chunks = (max_keys + p.CK - 1) / p.CK;
    if (p.n_chunks < 1) p.n_chunks = 1;
    return p;
}

// Query tiles per wave.  Four make one wave carry all rows of an item up to N = 9 with 7 query heads per kv head, so that
// K / V are streamed once, past L2: the choice when the batch alone fills the chip (B = 256, N = 8: 7.3 ms of attention
// per step against 9.1 with two).  A small batch wants waves instead: with two tiles per wave an item's rows spread over
// twice the waves, two to a SIMD, and the extra passes over K / V hit in L2 (B = 8, N = 8: 0.82 -> 0.59 ms per step;
// B = 8, N = 24: 1.36 -> 0.80; B = 64, N = 24: 2.61 -> 2.47; B = 128, N = 32 with long caches: 6.71 -> 6.92, so the
// switch sits at 1024 (sequence, kv head, wave) triples).
static int pick_qw(int B, int N, int Hq, int Hkv)
{
    const int QT = ((Hq / Hkv) * N + 15) / 16;
    return (QT <= 2 || (long)B * Hkv * ((QT + 3) / 4) < 1024) ? 2 : 4;
}

// K / V loads.  Every cache line of K (pages in fragment order) and of V^T is touched by exactly one load
// instruction of a wave.  When an item has a single wave (STREAM) its K / V are read once per launch and the
// loads are non-temporal: measured on the 7B-class cache at B = 256, 327 -> 288 us per layer at N = 8 and
// 283 -> 242 at N = 1.  Items shared by two or three waves keep ordinary loads, so that the later waves hit in L2
// (with streaming loads 105 -> 108 us at B = 64, N = 24).
typedef uint32_t attn_u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t attn_u32x2_t __attribute__((ext_vector_type(2)));
template <bool STREAM, typename T> __device__ __forceinline__ uint4 load16(const T *p)
{
    if (!STREAM) return *reinterpret_cast<const uint4 *>(p);
    const attn_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const attn_u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
template <bool STREAM, typename T> __device__ __forceinline__ uint2 load8(const T *p)
{
    if (!STREAM) return *reinterpret_cast<const uint2 *>(p);
    const attn_u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const attn_u32x2_t *>(p));
    return make_uint2(v.x, v.y);
}

template <typename T, int HD, int QW, bool STREAM>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(QW == 2 ? 2 : 1, QW == 2 ? 2 : 1))) void attn_mfma_kernel(const T *__restrict__ q, const T *__restrict__ k_pool,
                                                         const T *__restrict__ v_pool, const int32_t *__restrict__ page_table,
                                                         const uint64_t *__restrict__ mask, float *__restrict__ part_o,
                                                         float *__restrict__ part_ml, int layer, int n_pages,
                                                         int max_pages, int N, int n_prev, int Hq, int Hkv, int QR, int CK,
                                                         int n_chunks, int n_items, int waves, float scale,
                                                         const int4 *__restrict__ order)
{
    constexpr int KK = HD / 32;   // MFMAs per S^T tile (contraction over head_dim)
    constexpr int HT = HD / 16;   // 16-row tiles of O^T
    // One wave per block.  Blocks are dealt to the 8 XCDs round-robin, so the waves that share one
    // (sequence, kv head, chunk) item get block ids that differ by multiples of 8: they land on the same XCD
    // and the item's K/V is fetched into one L2 only.
    const int grp8 = blockIdx.x / (8 * waves), within = blockIdx.x % (8 * waves);
    const int idx = grp8 * 8 + (within & 7), wave = within >> 3;
    if (idx >= n_items) return;
    const int4 desc = order[idx];   // longest items first (see attn_order_kernel): item, cache slot, committed length
    const int item = desc.x, s = desc.y, L = desc.z;
    const int chunk = item % n_chunks, hk = (item / n_chunks) % Hkv, b = item / (n_chunks * Hkv);
    const int lane = threadIdx.x;
    const int c = lane & 15, grp = lane >> 4;
    const int G = Hq / Hkv, n_tot = n_prev + N, rows = G * N;
    const int qt0 = wave * QW;
    if (qt0 * 16 >= rows) return;
    const int total = min(L + n_tot, max_pages * 16);
    // the sequence's keys are cut into nc = ceil(total / CK) chunks of equal size (a multiple of 32): items of one
    // launch then differ in work by at most the ratio of the longest to the shortest chunk, not by 0 .. CK
    const int nc = min((total + CK - 1) / CK, n_chunks);
    const int ck = ((total + max(nc, 1) - 1) / max(nc, 1) + 31) / 32 * 32;
    const int t_begin = chunk * ck;
    if (chunk >= nc || t_begin >= total) {
        // a chunk beyond the sequence: publish l = 0 so that the merge can read every chunk without knowing the length
        if (grp == 0) {
#pragma unroll
            for (int w = 0; w < QW; w++) {
                const int qi = (qt0 + w) * 16 + c;
                if (qi < rows) {
                    const size_t row = (((size_t)b * Hkv + hk) * n_chunks + chunk) * QR + qi;
                    *reinterpret_cast<float2 *>(part_ml + row * 2) = make_float2(0.f, 0.f);
                }
            }
        }
        return;
    }
    const int t_end = min(t_begin + ck, total);

    // query fragments (parked in LDS: each lane reads back only what it wrote, so no barrier is needed; this
    // frees QW * KK * 4 registers for the K / V double buffer) and per-column masks
    __shared__ uint4 qs[QW * KK * 64];
    uint64_t qmask[QW];
#pragma unroll
    for (int w = 0; w < QW; w++) {
        int qi = (qt0 + w) * 16 + c;
        bool ok = qi < rows;
        int j = ok ? qi / G : 0, g = ok ? qi % G : 0;
        qmask[w] = ok ? mask[(size_t)b * N + j] : 0ull;
        const T *qp = q + ((size_t)b * N + j) * Hq * HD + (size_t)(hk * G + g) * HD + grp * (HD / 4);
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
            qs[(w * KK + kk) * 64 + lane] = ok ? *reinterpret_cast<const uint4 *>(qp + kk * 8) : make_uint4(0, 0, 0, 0);
        }
    }

    float m_run[QW], l_run[QW];
    f32x4_t o[QW][HT];
#pragma unroll
    for (int w = 0; w < QW; w++) {
        m_run[w] = -INFINITY;
        l_run[w] = 0.f;
#pragma unroll
        for (int h = 0; h < HT; h++) o[w][h] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    }

    const float c2 = scale * 1.4426950408889634f;   // scores are exponentiated in base 2
    const size_t head_stride = (size_t)16 * HD;  // elements per (page, kv head)
    const int32_t *pt = page_table + (size_t)s * max_pages;

    // One step = 32 key positions (two pages).  The K / V fragments of step t + 1 are requested into a second
    // register set before the arithmetic of step t starts, so that with one wave per SIMD the memory latency is
    // covered by a whole step of MFMA and softmax work.
    // The two pages of the step that starts at key position t0 (the second may lie beyond the sequence: clamped, its
    // keys are masked).  Page ids are wave-uniform loads; they are fetched one step before the K / V loads that need
    // them, so that a step's K / V requests do not wait behind a page-table round trip of their own.
    auto pages_of = [&](int t0, int &pg0, int &pg1) {
        const int pi0 = min(t0 >> 4, max_pages - 1), pi1 = min(pi0 + 1, max_pages - 1);
        pg0 = min(max(pt[pi0], 0), n_pages - 1);
        pg1 = min(max(pt[pi1], 0), n_pages - 1);
    };
    auto load_pages = [&](int pg0, int pg1, Frag16 (&kf)[2][KK], Frag16 (&vf)[HT]) {
        const T *kb[2], *vb[2];
        kb[0] = k_pool + (((size_t)layer * n_pages + pg0) * Hkv + hk) * head_stride;
        kb[1] = k_pool + (((size_t)layer * n_pages + pg1) * Hkv + hk) * head_stride;
        vb[0] = v_pool + (((size_t)layer * n_pages + pg0) * Hkv + hk) * head_stride;
        vb[1] = v_pool + (((size_t)layer * n_pages + pg1) * Hkv + hk) * head_stride;

#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int kk = 0; kk < KK; kk++)
                kf[kt][kk].u = load16<STREAM>(kb[kt] + kk * 512 + lane * 8);   // fragment kk of the page: 1 KiB, contiguous
#pragma unroll
        for (int h = 0; h < HT; h++) {
            vf[h].u2[0] = load8<STREAM>(vb[0] + (size_t)(h * 16 + c) * 16 + grp * 4);
            vf[h].u2[1] = load8<STREAM>(vb[1] + (size_t)(h * 16 + c) * 16 + grp * 4);
        }
    };
    auto load_step = [&](int t0, Frag16 (&kf)[2][KK], Frag16 (&vf)[HT]) {
        int pg0, pg1;
        pages_of(t0, pg0, pg1);
        load_pages(pg0, pg1, kf, vf);
    };
    auto used = [&](int w) { return (qt0 + w) * 16 < rows; };   // wave-uniform: tiles past the last query row idle
    // One step over all tiles of the wave, in phases so that the independent tiles' MFMA and VALU chains overlap:
    //   1  raw scores S^T = K . Q^T;
    //   2  masking (MASKED steps: those that reach past the chunk or into the in-round nodes) and the test for a
    //      moved exponent reference;
    //   3  weights 2^(c2 (s - m_run)), their per-lane sums, the packed P^T fragments;
    //   4  O^T += V^T . P^T.
    // Lazy rescaling: m_run (one value per query column, identical in the four lane groups that share the column)
    // only moves when some score exceeds it by more than RESCALE_LOG2 in base-2 units, or when the column had no
    // valid key yet.  Each lane tests its own 8 scores, nothing crosses lanes; the weights are at most
    // 2^RESCALE_LOG2 and exact to the same relative precision.  The FAST variant has no code that touches the
    // accumulators outside the MFMAs (so they can stay in the accumulation registers for the whole loop): when
    // some lane fires it returns false with nothing changed, and the step is redone by the variant that reduces
    // the column maxima across the lane groups and rescales l and the accumulators.
    auto compute_step = [&](auto masked_tag, auto fast_tag, int t0, Frag16 (&kf)[2][KK], Frag16 (&vf)[HT]) -> bool {
        constexpr bool MASKED = decltype(masked_tag)::value, FAST = decltype(fast_tag)::value;
        static_assert(!(MASKED && FAST), "masked steps run the full variant");
        const bool tail = MASKED && t0 + 32 > t_end;   // some key positions of this step are outside the chunk
        // an offset the compiler cannot see through keeps the loop-invariant query reads inside the loop
        // (hoisted, they would take their QW * KK * 4 registers back)
        int q_off;
        asm volatile("v_mov_b32 %0, 0" : "=v"(q_off));
        if (tail) {
            // values of positions that are never attended may be anything: zero them so 0 * x stays 0
#pragma unroll
            for (int h = 0; h < HT; h++)
#pragma unroll
                for (int jj = 0; jj < 8; jj++) {
                    int t = t0 + (jj >> 2) * 16 + grp * 4 + (jj & 3);
                    if (t >= t_end) vf[h].s[jj] = 0;
                }
        }
        f32x4_t sacc[QW][2];
        float mx[QW];
        bool any_grow = false;
#pragma unroll
        for (int w = 0; w < QW; w++) {
            if (!used(w)) continue;
            Frag16 qfr[KK];
#pragma unroll
            for (int kk = 0; kk < KK; kk++) qfr[kk].u = qs[(w * KK + kk) * 64 + lane + q_off];
#pragma unroll
            for (int kt = 0; kt < 2; kt++) {
                sacc[w][kt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KK; kk++) sacc[w][kt] = mfma16<T>(kf[kt][kk], qfr[kk], sacc[w][kt]);
            }
        }
#pragma unroll
        for (int w = 0; w < QW; w++) {
            mx[w] = -INFINITY;
            if (!used(w)) continue;
#pragma unroll
            for (int jj = 0; jj < 8; jj++) {
                float v = sacc[w][jj >> 2][jj & 3];
                if (MASKED) {   // branch-free: in range, and either committed prefix or an ancestor bit
                    const int t = t0 + (jj >> 2) * 16 + grp * 4 + (jj & 3);
                    const uint32_t anc = (uint32_t)(qmask[w] >> min(max(t - L, 0), 63)) & 1u;
                    const bool valid = (t < t_end) & ((t < L) | (anc != 0u));
                    v = valid ? v : -INFINITY;
                    sacc[w][jj >> 2][jj & 3] = v;
                }
                mx[w] = fmaxf(mx[w], v);
            }
            any_grow |= (mx[w] - m_run[w]) * c2 > RESCALE_LOG2;   // -inf vs finite: inf; -inf vs -inf: NaN (false)
        }
        if (__builtin_amdgcn_ballot_w64(any_grow) != 0ull) {
            if (FAST) return false;
#pragma unroll
            for (int w = 0; w < QW; w++) {
                if (!used(w)) continue;
                const float cm = group_max(mx[w]);
                const float m_new = fmaxf(m_run[w], cm);
                const float m_use = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f((m_run[w] - m_use) * c2);   // exp2(-inf) = 0 on the first valid step
                l_run[w] *= alpha;
#pragma unroll
                for (int h = 0; h < HT; h++) o[w][h] = o[w][h] * alpha;
                m_run[w] = m_new;
            }
        }
        Frag16 pf[QW];
#pragma unroll
        for (int w = 0; w < QW; w++) {
            if (!used(w)) continue;
            const float mb = (m_run[w] == -INFINITY ? 0.f : m_run[w]) * c2;
            float pv[8];
#pragma unroll
            for (int jj = 0; jj < 8; jj++) {
                pv[jj] = __builtin_amdgcn_exp2f(fmaf(sacc[w][jj >> 2][jj & 3], c2, -mb));
                l_run[w] += pv[jj];
            }
            pf[w].u = make_uint4(pack2<T>(pv[0], pv[1]), pack2<T>(pv[2], pv[3]), pack2<T>(pv[4], pv[5]), pack2<T>(pv[6], pv[7]));
        }
#pragma unroll
        for (int w = 0; w < QW; w++) {
            if (!used(w)) continue;
#pragma unroll
            for (int h = 0; h < HT; h++) o[w][h] = mfma16<T>(vf[h], pf[w], o[w][h]);
        }
        return true;
    };
    // Plain steps (entirely inside the chunk and the committed prefix) first, with the next step's fragments
    // requested into a second register set before the arithmetic starts; then the at most three masked steps in a
    // loop of their own, so that the variants' registers are never live together.
    Frag16 kf[2][KK], vf[HT];
    const int t_plain = t_begin + max(min(t_end, L) - t_begin, 0) / 32 * 32;
    int t0 = t_begin;
    if (t0 < t_plain) {
        Frag16 kn[2][KK], vn[HT];
        auto rotate = [&]() {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int kk = 0; kk < KK; kk++) kf[kt][kk].u = kn[kt][kk].u;
#pragma unroll
            for (int h = 0; h < HT; h++) vf[h].u = vn[h].u;
        };
        load_step(t0, kf, vf);
        int pn0, pn1;                      // pages of the next step to be requested (t0 + 32, then t0 + 64, ...)
        pages_of(t0 + 32, pn0, pn1);
        while (t0 < t_plain) {
            {   // a full step: the first of the chunk, and any step whose reference has to move
                const bool has_next = t0 + 32 < t_plain;
                if (has_next) {
                    load_pages(pn0, pn1, kn, vn);
                    pages_of(t0 + 64, pn0, pn1);
                }
                compute_step(std::false_type{}, std::false_type{}, t0, kf, vf);
                if (has_next) rotate();
                t0 += 32;
            }
            while (t0 < t_plain) {
                const bool has_next = t0 + 32 < t_plain;
                if (has_next) {
                    load_pages(pn0, pn1, kn, vn);
                    pages_of(t0 + 64, pn0, pn1);
                }
                if (!compute_step(std::false_type{}, std::true_type{}, t0, kf, vf)) {   // redo it as a full step
                    // the pages of t0 + 64 were just fetched; the outer loop requests t0 + 32 again
                    pages_of(t0 + 32, pn0, pn1);
                    break;
                }
                if (has_next) rotate();
                t0 += 32;
            }
        }
    }
    for (; t0 < t_end; t0 += 32) {
        load_step(t0, kf, vf);
        compute_step(std::true_type{}, std::false_type{}, t0, kf, vf);
    }

    // partials: O^T lane holds head_dim rows h*16 + 4*grp + i of query column c
#pragma unroll
    for (int w = 0; w < QW; w++) {
        const float l_col = group_sum(l_run[w]);   // the lanes kept their own partial sums
        int qi = (qt0 + w) * 16 + c;
        if (qi >= rows) continue;
        size_t row = (((size_t)b * Hkv + hk) * n_chunks + chunk) * QR + qi;
#pragma unroll
        for (int h = 0; h < HT; h++)
            *reinterpret_cast<f32x4_t *>(part_o + row * HD + h * 16 + grp * 4) = o[w][h];
        if (grp == 0) {
            part_ml[row * 2] = m_run[w] * scale;   // the reference the weights were taken against, natural-log units
            part_ml[row * 2 + 1] = l_col;
        }
    }
}

// Launch order of the (sequence, kv head, chunk) items: longest first.  Blocks are dispatched in index order and
// a CU slot takes the next block when it finishes one, so with the long items up front the short ones fill the
// gaps at the end (longest-processing-time-first list scheduling) instead of a long item starting last.  One block:
// counting sort by size class (128 classes of the chunk length CK; empty items last); the order within a class
// is whatever the atomics give, which only affects scheduling.  Each entry carries what the attention kernel
// would otherwise fetch through two more dependent loads: (item, cache slot, committed length, 0).
__global__ __launch_bounds__(1024) void attn_order_kernel(const int32_t *__restrict__ seq_len, const int32_t *__restrict__ slot,
                                                            int n_slots, int max_pages, int n_tot, int Hkv, int CK, int n_chunks,
                                                            int n_items, int4 *__restrict__ order)
{
    constexpr int NB = 130;
    __shared__ int cnt[NB], base[NB];
    for (int i = threadIdx.x; i < NB; i += 1024) cnt[i] = 0;
    __syncthreads();
    auto describe = [&](int item, int &s, int &L) {
        const int chunk = item % n_chunks, b = item / (n_chunks * Hkv);
        s = min(max(slot[b], 0), n_slots - 1);
        L = seq_len[s];
        const int total = min(L + n_tot, max_pages * 16);
        const int nc = min((total + CK - 1) / CK, n_chunks);
        if (chunk >= nc) return NB - 1;
        const int ck = ((total + nc - 1) / nc + 31) / 32 * 32;
        const int keys = min(ck, total - chunk * ck);
        return keys <= 0 ? NB - 1 : 128 - min(128, (int)((int64_t)keys * 128 / CK));
    };
    int s, L;
    for (int item = threadIdx.x; item < n_items; item += 1024) atomicAdd(&cnt[describe(item, s, L)], 1);
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < NB; i++) { base[i] = run; run += cnt[i]; }
    }
    __syncthreads();
    for (int item = threadIdx.x; item < n_items; item += 1024) {
        const int cls = describe(item, s, L);
        order[atomicAdd(&base[cls], 1)] = make_int4(item, s, L, 0);
    }
}

// Combine the chunks of one (row, query head): out = sum_c O_c e^(m_c - m) / sum_c l_c e^(m_c - m).  Every chunk
// slot of the launch holds (m, l) -- l = 0 for chunks beyond the sequence, whose O is then never used -- so nothing
// here waits on the sequence length: the (m, l) loads and the first CB chunks' O loads are in flight together.
template <typename T, int HD, int CB>
__device__ __forceinline__ void merge_row(const float *__restrict__ part_o, const float *__restrict__ part_ml, size_t row0,
                                          int QR, int n_chunks, int lane, float (&acc)[HD / 64], float &den)
{
    float m = -INFINITY;
    float2 ml0 = make_float2(0.f, 0.f);
    if (lane < n_chunks) ml0 = *reinterpret_cast<const float2 *>(part_ml + (row0 + (size_t)lane * QR) * 2);
    // O of the first CB chunks (indices clamped: the surplus copies get weight 0)
    float v0[CB][HD / 64];
#pragma unroll
    for (int cc = 0; cc < CB; cc++) {
        const float *po = part_o + (row0 + (size_t)min(cc, n_chunks - 1) * QR) * HD + lane;
#pragma unroll
        for (int i = 0; i < HD / 64; i++) v0[cc][i] = po[64 * i];
    }
    m = ml0.y > 0.f ? ml0.x : -INFINITY;
    for (int ch = 64 + lane; ch < n_chunks; ch += 64) {
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + (row0 + (size_t)ch * QR) * 2);
        m = fmaxf(m, ml.y > 0.f ? ml.x : -INFINITY);
    }
    m = wave_max(m);
    float wgt = ml0.y > 0.f ? __expf(ml0.x - m) : 0.f;
    den = ml0.y * wgt;
#pragma unroll
    for (int cc = 0; cc < CB; cc++) {
        const float wc = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(wgt), cc));
#pragma unroll
        for (int i = 0; i < HD / 64; i++) acc[i] += wc != 0.f ? v0[cc][i] * wc : 0.f;
    }
    // the rest, eight chunks' loads at a time
    for (int base = 0; base < n_chunks; base += 64) {
        if (base) {
            const int ch = base + lane;
            wgt = 0.f;
            if (ch < n_chunks) {
                const float2 ml = *reinterpret_cast<const float2 *>(part_ml + (row0 + (size_t)ch * QR) * 2);
                wgt = ml.y > 0.f ? __expf(ml.x - m) : 0.f;
                den += ml.y * wgt;
            }
        }
        const int cnt = min(64, n_chunks - base);
#pragma unroll 8
        for (int cc = base ? 0 : CB; cc < cnt; cc++) {
            const float wc = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(wgt), cc));
            const float *po = part_o + (row0 + (size_t)(base + cc) * QR) * HD + lane;
#pragma unroll
            for (int i = 0; i < HD / 64; i++) {
                const float v = po[64 * i];
                acc[i] += wc != 0.f ? v * wc : 0.f;
            }
        }
    }
}

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                                        T *__restrict__ out, int N, int Hq, int Hkv, int QR, int n_chunks)
{
    // one wave per (row, query head), four heads per block
    const int r = blockIdx.x, hq = blockIdx.y * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (hq >= Hq) return;
    const int b = r / N, j = r % N, G = Hq / Hkv, hk = hq / G, g = hq % G;
    const int qi = j * G + g;
    const size_t row0 = (((size_t)b * Hkv + hk) * n_chunks) * QR + qi;   // chunk ch is row0 + ch * QR
    float den = 0.f, acc[HD / 64];
#pragma unroll
    for (int i = 0; i < HD / 64; i++) acc[i] = 0.f;
    if (n_chunks <= 4) merge_row<T, HD, 4>(part_o, part_ml, row0, QR, n_chunks, lane, acc, den);
    else if (n_chunks <= 16) merge_row<T, HD, 16>(part_o, part_ml, row0, QR, n_chunks, lane, acc, den);
    else merge_row<T, HD, 32>(part_o, part_ml, row0, QR, n_chunks, lane, acc, den);
    den = wave_sum(den);
    const float inv = den > 0.f ? 1.f / den : 0.f;
#pragma unroll
    for (int i = 0; i < HD / 64; i++) out[(size_t)r * Hq * HD + (size_t)hq * HD + lane + 64 * i] = from_f<T>(acc[i] * inv);
}

// The same combination when there are at most four chunk slots (large batches: a sequence is one to three chunks).
// A thread owns four consecutive dims of one (row, query head) and recomputes the row's few weights itself, so there
// is no cross-lane step at all: eight loads per thread, all in flight together, 32 (row, head) pairs per block at
// head_dim 128 instead of four.  27 -> 14 us per layer at B = 256, N = 8.
template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_merge_few_kernel(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                                            T *__restrict__ out, int M, int N, int Hq, int Hkv, int QR, int n_chunks)
{
    constexpr int TPP = HD / 4;   // threads per (row, head)
    const int pair = blockIdx.x * (256 / TPP) + threadIdx.x / TPP, e4 = (threadIdx.x % TPP) * 4;
    if (pair >= M * Hq) return;
    const int r = pair / Hq, hq = pair % Hq;
    const int b = r / N, j = r % N, G = Hq / Hkv, hk = hq / G, g = hq % G;
    const size_t row0 = (((size_t)b * Hkv + hk) * n_chunks) * QR + (j * G + g);   // chunk ch is row0 + ch * QR
    float2 ml[4];
    f32x4_t v[4];
#pragma unroll
    for (int c = 0; c < 4; c++) {
        const size_t row = row0 + (size_t)min(c, n_chunks - 1) * QR;   // clamped: the surplus copies are not used
        ml[c] = *reinterpret_cast<const float2 *>(part_ml + row * 2);
        v[c] = *reinterpret_cast<const f32x4_t *>(part_o + row * HD + e4);
    }
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < 4; c++)
        if (c < n_chunks && ml[c].y > 0.f) m = fmaxf(m, ml[c].x);
    float den = 0.f;
    f32x4_t acc = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; c++) {
        const float w = (c < n_chunks && ml[c].y > 0.f) ? __expf(ml[c].x - m) : 0.f;
        den += ml[c].y * w;
        if (w != 0.f) acc += v[c] * w;   // O of an empty chunk may hold anything
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
    *reinterpret_cast<uint2 *>(out + (size_t)r * Hq * HD + (size_t)hq * HD + e4) =
        make_uint2(pack2<T>(acc[0] * inv, acc[1] * inv), pack2<T>(acc[2] * inv, acc[3] * inv));
}

bool attention_mfma_supported(const fg_kv_cache *kv, int Hq, int N)
{
    return is16(kv->dtype) && (kv->head_dim == 128 || kv->head_dim == 64) && kv->page_size == 16 &&
           Hq % kv->n_kv_heads == 0 && Hq / kv->n_kv_heads <= 8 && N >= 1 && N <= FG_MAX_NODES;
}

int64_t attention_mfma_ws_bytes(int B, int N, int Hq, int Hkv, int hd, int max_keys)
{
    if (B < 1 || N < 1 || Hkv < 1 || Hq % Hkv) return 0;
    AttnPlan p = pick_qw(B, N, Hq, Hkv) == 2 ? plan_attention<2>(B, N, Hq, Hkv, max_keys) : plan_attention<4>(B, N, Hq, Hkv, max_keys);
    int64_t rows = (int64_t)B * Hkv * p.n_chunks * p.QR;
    return align_up(rows * hd * 4, 256) + align_up(rows * 2 * 4, 256) + align_up((int64_t)B * Hkv * p.n_chunks * 16, 256);
}

template <typename T, int HD, int QW>
static int32_t launch_typed(const fg_kv_cache *kv, int layer, const fg_tree *t, TreeDev td, int Hq, const void *q, void *out,
                            int max_keys, void *ws, int64_t ws_bytes, int reuse_order, hipStream_t st)
{
    const int B = t->B, N = t->N, Hkv = kv->n_kv_heads;
    AttnPlan p = plan_attention<QW>(B, N, Hq, Hkv, max_keys);
    int64_t rows = (int64_t)B * Hkv * p.n_chunks * p.QR;
    const int n_items = B * Hkv * p.n_chunks;
    int64_t need = align_up(rows * HD * 4, 256) + align_up(rows * 2 * 4, 256) + align_up((int64_t)n_items * 16, 256);
    if (!ws || ws_bytes < need) return fail(FG_ERR_CAPACITY, "attention workspace too small (%lld < %lld)", (long long)ws_bytes, (long long)need);
    float *part_o = (float *)ws;
    float *part_ml = (float *)((char *)ws + align_up(rows * HD * 4, 256));
    int4 *order = (int4 *)((char *)part_ml + align_up(rows * 2 * 4, 256));
    const float scale = 1.0f / sqrtf((float)HD);
    if (!reuse_order) {   // lengths do not change within a step: the layers after the first reuse the order
        hipLaunchKernelGGL(attn_order_kernel, dim3(1), dim3(1024), 0, st, kv->seq_len, t->slot, kv->n_slots, kv->max_pages_per_seq,
                           t->n_prev + N, Hkv, p.CK, p.n_chunks, n_items, order);
        FG_LAUNCH_CHECK("attn_order");
    }
    dim3 grid((unsigned)((n_items + 7) / 8 * 8 * p.waves));
#define FG_ATTN_LAUNCH(STREAM)                                                                                      \
    hipLaunchKernelGGL((attn_mfma_kernel<T, HD, QW, STREAM>), grid, dim3(64), 0, st, (const T *)q, (const T *)kv->k_pool, \
                       (const T *)kv->v_pool, kv->page_table, td.mask, part_o, part_ml, layer, kv->n_pages,            \
                       kv->max_pages_per_seq, N, t->n_prev, Hq, Hkv, p.QR, p.CK, p.n_chunks, n_items, p.waves, scale,  \
                       order)
    if (p.waves == 1) FG_ATTN_LAUNCH(true);
    else FG_ATTN_LAUNCH(false);
#undef FG_ATTN_LAUNCH
    FG_LAUNCH_CHECK("attn_mfma");
    if (p.n_chunks <= 4)
        hipLaunchKernelGGL((attn_merge_few_kernel<T, HD>), dim3((unsigned)(((int64_t)B * N * Hq + 256 / (HD / 4) - 1) / (256 / (HD / 4)))),
                           dim3(256), 0, st, part_o, part_ml, (T *)out, B * N, N, Hq, Hkv, p.QR, p.n_chunks);
    else
        hipLaunchKernelGGL((attn_merge_kernel<T, HD>), dim3(B * N, (Hq + 3) / 4), dim3(256), 0, st, part_o, part_ml,
                           (T *)out, N, Hq, Hkv, p.QR, p.n_chunks);
    FG_LAUNCH_CHECK("attn_merge");
    return FG_OK;
}

int32_t launch_attention_mfma(const fg_kv_cache *kv, int layer, const fg_tree *t, TreeDev td, int Hq, const void *q, void *out,
                              int max_keys, void *ws, int64_t ws_bytes, int reuse_order, hipStream_t st)
{
    const int qw = pick_qw(t->B, t->N, Hq, kv->n_kv_heads);
#define FG_ATTN(T, HD)                                                                                          \
    return qw == 2 ? launch_typed<T, HD, 2>(kv, layer, t, td, Hq, q, out, max_keys, ws, ws_bytes, reuse_order, st) \
                   : launch_typed<T, HD, 4>(kv, layer, t, td, Hq, q, out, max_keys, ws, ws_bytes, reuse_order, st)
    if (kv->dtype == FG_BF16) {
        if (kv->head_dim == 128) { FG_ATTN(bf16_t, 128); } else { FG_ATTN(bf16_t, 64); }
    } else {
        if (kv->head_dim == 128) { FG_ATTN(f16_t, 128); } else { FG_ATTN(f16_t, 64); }
    }
#undef FG_ATTN
}

}  // namespace fg
