// Ceiling probes (measurement only, no part of the method): what this GPU sustains for the two resources the hot
// path is bound by, so that a kernel's fraction of the nominal peak can be set beside its fraction of what any
// kernel could reach.
//   read    every wave streams 1 KiB per instruction (16 bytes per lane), four loads in flight, and keeps an XOR
//           of what it read; nothing is written but one word per block
//   copy    the same stream, written back: the plain copy whose FETCH_SIZE / WRITE_SIZE readings scale the HBM
//           traffic counters of the other kernels
//   read, L2-resident   every block streams one small region many times: the L2 -> L1 fill rate of a CU
//   read, deep          one contiguous slice per block with 8 - 32 loads per lane in flight: what a single CU draws from HBM
//   mfma    a register-resident loop of v_mfma_f32_32x32x16_{bf16,f16}: operands stay in registers, four independent
//           accumulator tiles per wave, no memory traffic in the loop
#include "fg_common.h"
#include "gemm_mfma.h"

namespace fg {

typedef uint32_t probe_u32x4_t __attribute__((ext_vector_type(4)));

template <int NT>
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *__restrict__ src, int64_t n_vec, uint32_t *sink)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t acc = 0;
    auto ld = [&](int64_t at) {
        if (NT) {
            const probe_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t *>(src + at));
            return make_uint4(v.x, v.y, v.z, v.w);
        }
        return src[at];
    };
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        const uint4 a = ld(i), b = ld(i + stride), c = ld(i + 2 * stride), d = ld(i + 3 * stride);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n_vec; i += stride) {
        const uint4 a = ld(i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    // one word per block, and only when the data says so: the store exists to keep the loads alive
    if (acc == 0x9e3779b9u && threadIdx.x == 0) sink[blockIdx.x] = acc;
}

// The same read stream in 4 KiB pieces at scattered addresses: a wave reads one 4 KiB page (four 1 KiB loads in
// flight), and the pages are visited in a hashed order -- the access pattern of a paged KV cache whose pages were
// handed out in no particular order (one K or V page of one kv head is 16 tokens x 128 dims x 2 bytes = 4 KiB).
__global__ __launch_bounds__(256) void probe_read_paged_kernel(const uint4 *__restrict__ src, int64_t n_pages, uint32_t *sink)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (int64_t)gridDim.x * 4;
    uint32_t acc = 0;
    for (int64_t i = wave; i < n_pages; i += n_waves) {
        // a bijection of [0, n_pages) when n_pages is a power of two: odd multiplier, then a xor-shift
        uint64_t p = ((uint64_t)i * 0x9E3779B97F4A7C15ULL) & (uint64_t)(n_pages - 1);
        p ^= p >> 7;
        p &= (uint64_t)(n_pages - 1);
        const uint4 *page = src + p * 256 + lane;
        const probe_u32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t *>(page));
        const probe_u32x4_t b = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t *>(page + 64));
        const probe_u32x4_t c = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t *>(page + 128));
        const probe_u32x4_t d = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t *>(page + 192));
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    if (acc == 0x9e3779b9u && lane == 0) sink[blockIdx.x] = acc;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n_vec)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n_vec; i += stride) dst[i] = src[i];
}

// `random` != 0: operands are four A and four B fragments of hashed values in [-2, 2) that rotate through the loop, so
// that the operand buses toggle as they do on real data (what the matrix cores draw, and with it the clock the power
// limit leaves, depends on it); 0: one constant fragment pair, the least the loop can draw.
template <typename T>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int random, float *sink)
{
    Frag a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        uint32_t w[8];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            // two 16-bit values per word: sign and mantissa bits from the hash, exponent of 1.0 or 0.5
            const uint64_t h = mix64(((uint64_t)threadIdx.x << 8) + i * 8 + j);
            const uint32_t lo = (uint32_t)h, hi = (uint32_t)(h >> 32);
            // bf16: exponent field 0x3f80 / 0x3f00; fp16: 0x3c00 / 0x3800
            constexpr bool bf = sizeof(T) == 2 && T(0.5f) == T(0);   // bf16_t is an integer storage type: 0.5f converts to 0
            const uint32_t e0 = bf ? (0x3f00u + ((lo >> 20) & 0x80u)) : (0x3800u + ((lo >> 20) & 0x400u));
            const uint32_t e1 = bf ? (0x3f00u + ((hi >> 20) & 0x80u)) : (0x3800u + ((hi >> 20) & 0x400u));
            const uint32_t m0 = bf ? (lo & 0x807fu) : (lo & 0x83ffu), m1 = bf ? (hi & 0x807fu) : (hi & 0x83ffu);
            const uint32_t one = bf ? 0x3f80u : 0x3c00u;
            const uint32_t v0 = random ? (e0 | m0) : one, v1 = random ? (e1 | m1) : one;
            w[j] = v0 | (v1 << 16);
        }
        a[i].u = make_uint4(w[0], w[1], w[2], w[3]);
        b[i].u = make_uint4(w[4], w[5], w[6], w[7]);
    }
    f32x16_t c0, c1, c2, c3;
#pragma unroll
    for (int r = 0; r < 16; r++) { c0[r] = 0.f; c1[r] = 0.f; c2[r] = 0.f; c3[r] = 0.f; }
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int u = 0; u < 4; u++) {
            c0 = mfma32<T>(a[u], b[u], c0);
            c1 = mfma32<T>(a[(u + 1) & 3], b[u], c1);
            c2 = mfma32<T>(a[(u + 2) & 3], b[(u + 1) & 3], c2);
            c3 = mfma32<T>(a[(u + 3) & 3], b[(u + 2) & 3], c3);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r++) s += c0[r] + c1[r] + c2[r] + c3[r];
    if (s == 1.2345f) sink[blockIdx.x * 256 + threadIdx.x] = s;   // keeps the loop alive; practically never true
}

// What a CU draws from L2: EVERY block streams the whole (small, power-of-two sized) region `passes` times, eight 16-byte
// loads per lane in flight.  The region stays in L2 and in none of the 32 KiB L1s, so the bytes a block reads are L2 -> L1
// fills: the path the operands of the large GEMMs take.
__global__ __launch_bounds__(256) void probe_read_l2_kernel(const uint4 *__restrict__ src, int n_vec, int passes, uint32_t *sink)
{
    const int mask = n_vec - 1;
    int idx = (blockIdx.x * 977 + threadIdx.x) & mask;
    uint32_t acc = 0;
    for (int it = 0; it < passes * (n_vec / 2048); it++) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = src[(idx + u * 256) & mask];
#pragma unroll
        for (int u = 0; u < 8; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        idx = (idx + 2048) & mask;
    }
    if (acc == 0x9e3779b9u && threadIdx.x == 0) sink[blockIdx.x] = acc;
}

constexpr int PROBE_L2_PASSES = 256;

// What one block draws from HBM when it keeps DEPTH 16-byte loads per lane in flight (DEPTH x 4 KiB per block): the
// blocks take contiguous slices of the buffer, so with at most one block per CU the rate per block is the rate per CU.
// It levels off far below the L2 -> L1 rate: a launch of fewer blocks than CUs is bound by how many CUs stream.
template <int DEPTH>
__global__ __launch_bounds__(256) void probe_read_deep_kernel(const uint4 *__restrict__ src, int64_t vec_per_block, uint32_t *sink)
{
    const uint4 *p = src + (int64_t)blockIdx.x * vec_per_block + threadIdx.x;
    const int64_t steps = vec_per_block / 256;   // a multiple of DEPTH (the host rounds the slice down)
    uint32_t acc = 0;
    probe_u32x4_t v[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; d++) v[d] = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t *>(p + (int64_t)d * 256));
    for (int64_t s0 = DEPTH; s0 < steps; s0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; d++) {   // slot d is consumed and refilled: DEPTH - 1 loads stay in flight
            acc ^= v[d].x ^ v[d].y ^ v[d].z ^ v[d].w;
            v[d] = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4_t *>(p + (s0 + d) * 256));
        }
    }
#pragma unroll
    for (int d = 0; d < DEPTH; d++) acc ^= v[d].x ^ v[d].y ^ v[d].z ^ v[d].w;
    if (acc == 0x9e3779b9u && threadIdx.x == 0) sink[blockIdx.x] = acc;
}

int32_t launch_probe_read(const void *src, int64_t bytes, int nontemporal, int blocks, void *sink, hipStream_t st)
{
    const int64_t n_vec = bytes / 16;
    if (nontemporal == 3) {   // L2-resident region, read PROBE_L2_PASSES times by every block
        hipLaunchKernelGGL(probe_read_l2_kernel, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, (int)n_vec, PROBE_L2_PASSES,
                           (uint32_t *)sink);
        FG_LAUNCH_CHECK("probe_read_l2");
        return FG_OK;
    }
    if (nontemporal >= 4) {   // contiguous slice per block, 8 / 16 / 32 loads per lane in flight
        const int depth = nontemporal == 4 ? 8 : (nontemporal == 5 ? 16 : 32);
        const int64_t per_block = n_vec / blocks / (256 * depth) * (256 * depth);
        if (per_block < 256 * depth) return fail(FG_ERR_INVALID_ARG, "fg_probe_read: buffer too small for %d blocks of this depth", blocks);
        if (depth == 8) hipLaunchKernelGGL(probe_read_deep_kernel<8>, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, per_block, (uint32_t *)sink);
        else if (depth == 16) hipLaunchKernelGGL(probe_read_deep_kernel<16>, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, per_block, (uint32_t *)sink);
        else hipLaunchKernelGGL(probe_read_deep_kernel<32>, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, per_block, (uint32_t *)sink);
        FG_LAUNCH_CHECK("probe_read_deep");
        return FG_OK;
    }
    if (nontemporal == 2) {   // scattered 4 KiB pages; the caller checked that bytes is a power of two
        hipLaunchKernelGGL(probe_read_paged_kernel, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, bytes / 4096, (uint32_t *)sink);
        FG_LAUNCH_CHECK("probe_read_paged");
        return FG_OK;
    }
    if (nontemporal) hipLaunchKernelGGL(probe_read_kernel<1>, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, n_vec, (uint32_t *)sink);
    else hipLaunchKernelGGL(probe_read_kernel<0>, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, n_vec, (uint32_t *)sink);
    FG_LAUNCH_CHECK("probe_read");
    return FG_OK;
}

int32_t launch_probe_copy(const void *src, void *dst, int64_t bytes, int blocks, hipStream_t st)
{
    hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, bytes / 16);
    FG_LAUNCH_CHECK("probe_copy");
    return FG_OK;
}

int32_t launch_probe_mfma(int32_t dtype, int iters, int random, int blocks, void *sink, hipStream_t st)
{
    if (dtype == FG_BF16) hipLaunchKernelGGL(probe_mfma_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, iters, random, (float *)sink);
    else hipLaunchKernelGGL(probe_mfma_kernel<f16_t>, dim3(blocks), dim3(256), 0, st, iters, random, (float *)sink);
    FG_LAUNCH_CHECK("probe_mfma");
    return FG_OK;
}

}  // namespace fg
