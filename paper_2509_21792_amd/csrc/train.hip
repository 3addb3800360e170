// Online draft learning (Sec. 4.2 "Draft Model Learning with Online Target Feedback"; Alg. 1, the draft training
// phase): loss and gradients of the one-layer draft head on the tokens and hidden states the generation phase cached,
// and the AdamW update.  Parameters, gradients and activations are fp32; the generation path gets the updated head by
// re-packing the parameters (fg_pack_weight).  The matrix products of a step run either in a register-tiled fp32 GEMM
// (the parity mode) or, operands rounded to bf16, in the generation path's MFMA GEMM; norm, RoPE, causal attention,
// SwiGLU and the loss are plain row-wise kernels, each with its backward.
#include "fg_common.h"

namespace fg {

// ---- fp32 GEMM: C[m, n] = sum_k A(m, k) B(k, n) (+ add[m, n]) ----------------------------------------------------
// A(m, k) sits at A[m * lda + k] (AK: k contiguous) or A[k * lda + m] (m contiguous); B(k, n) at B[n * ldb + k] (BK: k
// contiguous) or B[k * ldb + n] (n contiguous).  128 x 128 tile, 256 threads, 8 x 8 outputs per thread, 16-wide k steps
// through LDS.  Contiguous dimensions and leading dimensions are multiples of 4 (checked by the launcher), so global
// loads are float4 with whole-vector guards.
constexpr int SG_BM = 128, SG_BN = 128, SG_BK = 16;

template <bool AK, bool BK>
__global__ __launch_bounds__(256) void sgemm_kernel(const float *__restrict__ A, const float *__restrict__ Bm, float *__restrict__ C,
                                                    const float *__restrict__ add, int M, int N, int K, int lda, int ldb, int ldc)
{
    __shared__ float As[SG_BK][SG_BM + 4], Bs[SG_BK][SG_BN + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * SG_BM, n0 = blockIdx.x * SG_BN;
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 8; j++) acc[i][j] = 0.f;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k0 = 0; k0 < K; k0 += SG_BK) {
        // stage the two tiles (2048 elements each: two float4 per thread)
#pragma unroll
        for (int it = 0; it < 2; it++) {
            if (AK) {   // vectors along k: row = index / 4, k quad = index % 4
                const int idx = tid + it * 256, r = idx >> 2, kq = (idx & 3) * 4;
                const int m = m0 + r, k = k0 + kq;
                const float4 v = (m < M && k < K) ? *reinterpret_cast<const float4 *>(A + (size_t)m * lda + k) : zero4;
                As[kq][r] = v.x; As[kq + 1][r] = v.y; As[kq + 2][r] = v.z; As[kq + 3][r] = v.w;
            } else {    // vectors along m: k = index / 32, m quad = index % 32
                const int idx = tid + it * 256, kk = idx >> 5, mq = (idx & 31) * 4;
                const int m = m0 + mq, k = k0 + kk;
                const float4 v = (m < M && k < K) ? *reinterpret_cast<const float4 *>(A + (size_t)k * lda + m) : zero4;
                *reinterpret_cast<float4 *>(&As[kk][mq]) = v;
            }
            if (BK) {
                const int idx = tid + it * 256, r = idx >> 2, kq = (idx & 3) * 4;
                const int n = n0 + r, k = k0 + kq;
                const float4 v = (n < N && k < K) ? *reinterpret_cast<const float4 *>(Bm + (size_t)n * ldb + k) : zero4;
                Bs[kq][r] = v.x; Bs[kq + 1][r] = v.y; Bs[kq + 2][r] = v.z; Bs[kq + 3][r] = v.w;
            } else {
                const int idx = tid + it * 256, kk = idx >> 5, nq = (idx & 31) * 4;
                const int n = n0 + nq, k = k0 + kk;
                const float4 v = (n < N && k < K) ? *reinterpret_cast<const float4 *>(Bm + (size_t)k * ldb + n) : zero4;
                *reinterpret_cast<float4 *>(&Bs[kk][nq]) = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < SG_BK; kk++) {
            const float4 a0 = *reinterpret_cast<const float4 *>(&As[kk][ty * 8]), a1 = *reinterpret_cast<const float4 *>(&As[kk][ty * 8 + 4]);
            const float4 b0 = *reinterpret_cast<const float4 *>(&Bs[kk][tx * 8]), b1 = *reinterpret_cast<const float4 *>(&Bs[kk][tx * 8 + 4]);
            const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int i = 0; i < 8; i++)
#pragma unroll
                for (int j = 0; j < 8; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int m = m0 + ty * 8 + i;
        if (m >= M) continue;
#pragma unroll
        for (int jq = 0; jq < 2; jq++) {
            const int n = n0 + tx * 8 + jq * 4;
            if (n >= N) continue;      // N is a multiple of 4: a quad is inside or outside as a whole
            float4 v = make_float4(acc[i][jq * 4], acc[i][jq * 4 + 1], acc[i][jq * 4 + 2], acc[i][jq * 4 + 3]);
            if (add) {
                const float4 o = *reinterpret_cast<const float4 *>(add + (size_t)m * ldc + n);
                v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
            }
            *reinterpret_cast<float4 *>(C + (size_t)m * ldc + n) = v;
        }
    }
}

// op 0: C = A[M,K] . B[N,K]^T (forward);  1: C = A[M,K] . B[K,N] (input gradient);  2: C = A[K,M]^T . B[K,N] (weight gradient)
static int32_t sgemm(int op, const float *A, const float *B, float *C, const float *add, int M, int N, int K, hipStream_t st)
{
    if (M <= 0 || N <= 0 || K <= 0) return FG_OK;
    if (N % 4 || (op != 2 && K % 4) || (op == 2 && M % 4)) return fail(FG_ERR_SHAPE, "training GEMM needs dimensions in multiples of 4 (%d, %d, %d)", M, N, K);
    const dim3 grid((N + SG_BN - 1) / SG_BN, (M + SG_BM - 1) / SG_BM);
    if (op == 0) hipLaunchKernelGGL((sgemm_kernel<true, true>), grid, dim3(256), 0, st, A, B, C, add, M, N, K, K, K, N);
    else if (op == 1) hipLaunchKernelGGL((sgemm_kernel<true, false>), grid, dim3(256), 0, st, A, B, C, add, M, N, K, K, N, N);
    else hipLaunchKernelGGL((sgemm_kernel<false, false>), grid, dim3(256), 0, st, A, B, C, add, M, N, K, M, N, N);
    FG_LAUNCH_CHECK("sgemm");
    return FG_OK;
}

// ---- the same three products on the matrix cores (bf16 operands, fp32 accumulate) --------------------------------------
// The 16-bit GEMM of the generation path computes out = X . W^T for a packed W; each product is brought into that form
// by casting (and, where the contraction runs over the other index, transposing) its fp32 operands into scratch and
// packing the second one.  Gradients are tiny numbers: bf16 keeps fp32's exponent range, so nothing underflows.
__global__ void cast_bf16_kernel(const float *__restrict__ src, bf16_t *__restrict__ dst, size_t n)
{
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 3 < n) {
        const float4 v = *reinterpret_cast<const float4 *>(src + i);
        uint2 u;
        u.x = (uint32_t)f2bf(v.x) | ((uint32_t)f2bf(v.y) << 16);
        u.y = (uint32_t)f2bf(v.z) | ((uint32_t)f2bf(v.w) << 16);
        *reinterpret_cast<uint2 *>(dst + i) = u;
    } else {
        for (size_t j = i; j < n; j++) dst[j] = f2bf(src[j]);
    }
}

// dst [C, R] (bf16) = transpose of src [R, C] (fp32), 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void transpose_cast_bf16_kernel(const float *__restrict__ src, bf16_t *__restrict__ dst, int R, int C)
{
    __shared__ float tile[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8)
        tile[i][tx] = (r0 + i < R && c0 + tx < C) ? src[(size_t)(r0 + i) * C + c0 + tx] : 0.f;
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < C && r0 + tx < R) dst[(size_t)(c0 + i) * R + r0 + tx] = f2bf(tile[tx][i]);
}

struct Mfma16 {          // scratch of the matrix-core path
    bf16_t *x16;         // the first operand, cast (and transposed)
    bf16_t *wp;          // the second operand, cast (and transposed) and packed
    int64_t x_cap, w_cap;
    // the packed form of the last second operand, so that the two LM-head products of the forward pass pack it once
    const float *last_src = nullptr;
    int last_op = -1;
    // the frozen LM head packed ahead of time by the caller (both operand orders), or nullptr
    const float *head_src = nullptr;
    const bf16_t *head_fwd = nullptr, *head_bwd = nullptr;
};

static int32_t gemm16(Mfma16 &s, int op, const float *A, const float *B, float *C, const float *add, int M, int N, int K, hipStream_t st)
{
    if (M <= 0 || N <= 0 || K <= 0) return FG_OK;
    if (N % 32 || K % 64) return fail(FG_ERR_SHAPE, "matrix-core training GEMM needs an output width in multiples of 32 and a contraction in multiples of 64 (%d, %d)", N, K);
    if ((int64_t)M * K > s.x_cap || (int64_t)N * K > s.w_cap) return fail(FG_ERR_CAPACITY, "matrix-core training GEMM scratch too small");
    auto cast = [&](const float *src, bf16_t *dst, size_t n) {
        hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)((n / 4 + 255) / 256 + 1)), dim3(256), 0, st, src, dst, n);
    };
    auto tcast = [&](const float *src, bf16_t *dst, int R, int Cc) {
        hipLaunchKernelGGL(transpose_cast_bf16_kernel, dim3((Cc + 31) / 32, (R + 31) / 32), dim3(256), 0, st, src, dst, R, Cc);
    };
    // first operand as [M, K] bf16
    if (op == 2) tcast(A, s.x16, K, M);           // A is [K, M]
    else cast(A, s.x16, (size_t)M * K);
    // second operand as [N, K] bf16, packed
    const bf16_t *wp = s.wp;
    if (s.head_src && B == s.head_src && op != 2) wp = op == 0 ? s.head_fwd : s.head_bwd;
    else if (!(s.last_src == B && s.last_op == op)) {
        // rounded (and transposed) and packed in one pass: B is [N, K], or [K, N] for the other two operand orders
        const int32_t rc = op == 0 ? launch_pack_cast_bf16(B, s.wp, N, K, st) : launch_pack_cast_t_bf16(B, s.wp, N, K, st);
        if (rc) return rc;
        s.last_src = B;
        s.last_op = op;
    }
    if (add) {
        if (add != C) FG_HIP(hipMemcpyAsync(C, add, (size_t)M * N * 4, hipMemcpyDeviceToDevice, st));
        GemmEpi ep;
        ep.h = C;
        return launch_gemm_mfma(FG_BF16, s.x16, wp, nullptr, M, N, K, EPI_RESIDUAL, 1, nullptr, st, &ep);
    }
    return launch_gemm_mfma(FG_BF16, s.x16, wp, C, M, N, K, EPI_SLABS, 1, nullptr, st);
}

// ---- row-wise kernels ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum256(float v, float *red)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}
__device__ __forceinline__ float block_max256(float v, float *red)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// cat[r] = embed[token r] ++ feat[r]
__global__ void train_concat_kernel(const float *embed, const int32_t *tokens, int vocab, const float *feat, float *cat, int d)
{
    const int r = blockIdx.x, tok = min(max(tokens[r], 0), vocab - 1);
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        cat[(size_t)r * 2 * d + c] = embed[(size_t)tok * d + c];
        cat[(size_t)r * 2 * d + d + c] = feat[(size_t)r * d + c];
    }
}

// y = x * inv * g, inv = (mean(x^2) + eps)^(-1/2) kept per row for the backward pass
__global__ __launch_bounds__(256) void rms_fwd_kernel(const float *x, const float *g, float *y, float *inv_out, int d, float eps)
{
    __shared__ float red[4];
    const int r = blockIdx.x;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) { const float v = x[(size_t)r * d + c]; ss += v * v; }
    ss = block_sum256(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    if (threadIdx.x == 0) inv_out[r] = inv;
    for (int c = threadIdx.x; c < d; c += 256) y[(size_t)r * d + c] = x[(size_t)r * d + c] * inv * g[c];
}

// dx = add + inv * (g . dy) - x * inv^3 * sum_k (g . dy)_k x_k / d
__global__ __launch_bounds__(256) void rms_bwd_kernel(const float *dy, const float *x, const float *g, const float *inv_in,
                                                      const float *add, float *dx, int d)
{
    __shared__ float red[4];
    const int r = blockIdx.x;
    const float inv = inv_in[r];
    float dot = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) dot += g[c] * dy[(size_t)r * d + c] * x[(size_t)r * d + c];
    dot = block_sum256(dot, red);
    const float k3 = inv * inv * inv * dot / (float)d;
    for (int c = threadIdx.x; c < d; c += 256) {
        const size_t at = (size_t)r * d + c;
        dx[at] = add[at] + inv * g[c] * dy[at] - x[at] * k3;
    }
}

// dg[c] = sum over rows of dy * x * inv, in two steps so that the chip has work: a thread owns a column of a chunk of
// 64 rows and walks them in order, then a thread per column adds the chunks in order (fixed order, no atomics)
constexpr int DG_ROWS = 64;
__global__ void rms_dgain_part_kernel(const float *dy, const float *x, const float *inv, float *part, int M, int d)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x, r0 = blockIdx.y * DG_ROWS, r1 = min(r0 + DG_ROWS, M);
    if (c >= d) return;
    float s = 0.f;
    for (int r = r0; r < r1; r++) s += dy[(size_t)r * d + c] * x[(size_t)r * d + c] * inv[r];
    part[(size_t)blockIdx.y * d + c] = s;
}
__global__ void rms_dgain_sum_kernel(const float *part, float *dg, int chunks, int d)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= d) return;
    float s = 0.f;
    for (int k = 0; k < chunks; k++) s += part[(size_t)k * d + c];
    dg[c] = s;
}

// rotate-half RoPE of the q and k heads of qkv [M, qkvd] in place at position row % T; dir = +1 forward, -1 the
// transpose (the backward pass).  Angles in double, as the table of the generation path is built.
__global__ void train_rope_kernel(float *qkv, int T, int n_rot_heads, int hd, int qkvd, double theta, int dir)
{
    const int r = blockIdx.x, half = hd >> 1, pos = r % T;
    for (int w = threadIdx.x; w < n_rot_heads * half; w += blockDim.x) {
        const int head = w / half, i = w % half;
        const double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
        const float c = (float)cos(ang), s = (float)sin(ang) * (float)dir;
        float *p = qkv + (size_t)r * qkvd + (size_t)head * hd;
        const float a = p[i], b = p[i + half];
        p[i] = a * c - b * s;
        p[i + half] = b * c + a * s;
    }
}

// causal attention inside each chain: one block per (sequence, query head, query position).  P [B, Hq, T, T] is kept.
__global__ __launch_bounds__(256) void train_attn_fwd_kernel(const float *qkv, float *P, float *att, int T, int Hq, int Hkv, int hd,
                                                             int qkvd, float scale)
{
    extern __shared__ float sc[];   // T scores
    __shared__ float red[4];
    const int t = blockIdx.x, hq = blockIdx.y, b = blockIdx.z, hk = hq / (Hq / Hkv);
    const float *q = qkv + (size_t)(b * T + t) * qkvd + (size_t)hq * hd;
    float mx = -INFINITY;
    for (int s = threadIdx.x; s <= t; s += 256) {
        const float *k = qkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + hk) * hd;
        float a = 0.f;
        for (int e = 0; e < hd; e++) a += q[e] * k[e];
        a *= scale;
        sc[s] = a;
        mx = fmaxf(mx, a);
    }
    mx = block_max256(mx, red);
    float den = 0.f;
    for (int s = threadIdx.x; s <= t; s += 256) { const float e = expf(sc[s] - mx); sc[s] = e; den += e; }
    den = block_sum256(den, red);
    float *prow = P + (((size_t)b * Hq + hq) * T + t) * T;
    for (int s = threadIdx.x; s < T; s += 256) {
        const float p = s <= t ? sc[s] / den : 0.f;
        prow[s] = p;
        if (s <= t) sc[s] = p;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < hd; e += 256) {
        float o = 0.f;
        for (int s = 0; s <= t; s++) o += sc[s] * qkv[(size_t)(b * T + s) * qkvd + (size_t)(Hq + Hkv + hk) * hd + e];
        att[(size_t)(b * T + t) * Hq * hd + (size_t)hq * hd + e] = o;
    }
}

// dS = P . (dP - sum_s dP P) * scale (kept, [B, Hq, T, T]) and dq; one block per (sequence, query head, query position)
__global__ __launch_bounds__(256) void train_attn_bwd_q_kernel(const float *qkv, const float *P, const float *datt, float *dS,
                                                               float *dqkv, int T, int Hq, int Hkv, int hd, int qkvd, float scale)
{
    extern __shared__ float ds[];   // T entries
    __shared__ float red[4];
    const int t = blockIdx.x, hq = blockIdx.y, b = blockIdx.z, hk = hq / (Hq / Hkv);
    const float *dout = datt + (size_t)(b * T + t) * Hq * hd + (size_t)hq * hd;
    const float *prow = P + (((size_t)b * Hq + hq) * T + t) * T;
    float dot = 0.f;
    for (int s = threadIdx.x; s <= t; s += 256) {
        const float *v = qkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + Hkv + hk) * hd;
        float dp = 0.f;
        for (int e = 0; e < hd; e++) dp += dout[e] * v[e];
        ds[s] = dp;
        dot += dp * prow[s];
    }
    dot = block_sum256(dot, red);
    float *dsrow = dS + (((size_t)b * Hq + hq) * T + t) * T;
    for (int s = threadIdx.x; s < T; s += 256) {
        const float g = s <= t ? prow[s] * (ds[s] - dot) * scale : 0.f;
        dsrow[s] = g;
        if (s <= t) ds[s] = g;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < hd; e += 256) {
        float a = 0.f;
        for (int s = 0; s <= t; s++) a += ds[s] * qkv[(size_t)(b * T + s) * qkvd + (size_t)(Hq + hk) * hd + e];
        dqkv[(size_t)(b * T + t) * qkvd + (size_t)hq * hd + e] = a;
    }
}

// dk[s] = sum over the kv head's query heads and t >= s of dS[t, s] q[t];  dv[s] = the same sum of P[t, s] dout[t];
// one block per (sequence, kv head, key position), a thread per head dim: fixed summation order, no atomics
__global__ void train_attn_bwd_kv_kernel(const float *qkv, const float *P, const float *dS, const float *datt, float *dqkv, int T,
                                         int Hq, int Hkv, int hd, int qkvd)
{
    const int s = blockIdx.x, hk = blockIdx.y, b = blockIdx.z, G = Hq / Hkv;
    for (int e = threadIdx.x; e < hd; e += blockDim.x) {
        float dk = 0.f, dv = 0.f;
        for (int g = 0; g < G; g++) {
            const int hq = hk * G + g;
            for (int t = s; t < T; t++) {
                const size_t at = (((size_t)b * Hq + hq) * T + t) * T + s;
                dk += dS[at] * qkv[(size_t)(b * T + t) * qkvd + (size_t)hq * hd + e];
                dv += P[at] * datt[(size_t)(b * T + t) * Hq * hd + (size_t)hq * hd + e];
            }
        }
        dqkv[(size_t)(b * T + s) * qkvd + (size_t)(Hq + hk) * hd + e] = dk;
        dqkv[(size_t)(b * T + s) * qkvd + (size_t)(Hq + Hkv + hk) * hd + e] = dv;
    }
}

// ---- tiled causal attention (chains of up to 1024 entries, head_dim 64 or 128) ------------------------------------------
// The three kernels above take a block per position and read K / V rows straight from global memory, a row per thread:
// right, and two orders of magnitude off the chip (3.4 + 3.4 + 1.3 ms for 8 chains of 256 entries).  The tiled forms
// below do the same sums -- over keys in ascending order, over head dims in ascending order, no atomics, so a step stays
// bitwise repeatable -- with the operand rows staged through LDS 64 at a time and a tile of 16 positions per block.
constexpr int TA_TQ = 16, TA_TK = 64;
constexpr int TA_SS = 20;   // floats per key in the score array: the tile's 16 positions + 4 of padding (16-byte rows, fewer bank conflicts)

// stage rows r0 .. r0 + 63 of a [*, hd] operand (row stride `stride` floats, rows clamped to n_rows - 1) into
// tile [64][hd + 1] (the odd row stride keeps a column walk conflict-free)
__device__ __forceinline__ void ta_stage(float *tile, const float *src, size_t stride, int r0, int n_rows, int hd)
{
    const int q4 = hd >> 2;
    for (int idx = threadIdx.x; idx < TA_TK * q4; idx += 256) {
        const int r = idx / q4, c = (idx - r * q4) * 4;
        const float4 v = *reinterpret_cast<const float4 *>(src + (size_t)min(r0 + r, n_rows - 1) * stride + c);
        float *d = tile + r * (hd + 1) + c;
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    }
}

// MODE 0, forward: S = (q . K^T) scale over the keys up to each position, P = softmax(S) (kept, [B, Hq, T, T]), att = P . V.
// MODE 1, backward to q: dP = datt . V^T, dS = P (dP - sum_s dP P) scale (kept), dq = dS . K.
// One block per (tile of 16 positions, query head, chain).  LDS: aT [hd][16], tile [64][hd + 1], sc [Tp][20] (key-major, so
// that the last phase reads the scores of four positions in one instruction).
template <int MODE>
__global__ __launch_bounds__(256) void train_attn_tile_kernel(const float *__restrict__ qkv, float *__restrict__ P, float *__restrict__ dS,
                                                              const float *__restrict__ datt, float *__restrict__ out, int T, int Tp, int Hq,
                                                              int Hkv, int hd, int qkvd, float scale)
{
    extern __shared__ __align__(16) float ta_lds[];
    float *aT = ta_lds, *tile = aT + hd * TA_TQ, *sc = tile + (TA_TK * (hd + 1) + 3) / 4 * 4;
    const int t0 = blockIdx.x * TA_TQ, hq = blockIdx.y, b = blockIdx.z, hk = hq / (Hq / Hkv), tid = threadIdx.x;
    const int t_last = min(t0 + TA_TQ, T) - 1;
    const float *kbase = qkv + (size_t)b * T * qkvd + (size_t)(Hq + hk) * hd;
    const float *vbase = qkv + (size_t)b * T * qkvd + (size_t)(Hq + Hkv + hk) * hd;
    // A rows (q, scaled, or datt), transposed so that a thread reads four positions of one head dim at once
    for (int idx = tid; idx < TA_TQ * hd; idx += 256) {
        const int i = idx / hd, e = idx - i * hd, t = min(t0 + i, T - 1);
        aT[e * TA_TQ + i] = MODE == 0 ? qkv[(size_t)(b * T + t) * qkvd + (size_t)hq * hd + e] * scale
                                      : datt[(size_t)(b * T + t) * Hq * hd + (size_t)hq * hd + e];
    }
    // phase 1: scores against B1 = K (forward) or V (backward); thread = (key of the tile, group of four positions)
    const int kj = tid & 63, qg = tid >> 6;
    for (int k0 = 0; k0 <= t_last; k0 += TA_TK) {
        __syncthreads();
        ta_stage(tile, MODE == 0 ? kbase : vbase, qkvd, k0, T, hd);
        __syncthreads();
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        const float *krow = tile + kj * (hd + 1);
        for (int e = 0; e < hd; e++) {
            const float kv = krow[e];
            const float4 a4 = *reinterpret_cast<const float4 *>(aT + e * TA_TQ + qg * 4);
            acc[0] += a4.x * kv; acc[1] += a4.y * kv; acc[2] += a4.z * kv; acc[3] += a4.w * kv;
        }
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int s = k0 + kj, t = t0 + qg * 4 + i;
            sc[s * TA_SS + qg * 4 + i] = (s <= t && t < T) ? acc[i] : (MODE == 0 ? -INFINITY : 0.f);
        }
    }
    __syncthreads();
    // phase 2: the row-wise step; 16 threads per position, partial sums over s = sub, sub + 16, .. then a fixed tree
    {
        const int i = tid >> 4, sub = tid & 15, t = t0 + i;
        const int n = t < T ? t + 1 : 0;                       // keys of this position
        float *row = sc + i;                                   // element s of the position's row: row[s * TA_SS]
        const size_t grow = (((size_t)b * Hq + hq) * T + min(t, T - 1)) * T;
        if (MODE == 0) {
            float mx = -INFINITY;
            for (int s2 = sub; s2 < n; s2 += 16) mx = fmaxf(mx, row[s2 * TA_SS]);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 16));
            float den = 0.f;
            for (int s2 = sub; s2 < n; s2 += 16) { const float e2 = expf(row[s2 * TA_SS] - mx); row[s2 * TA_SS] = e2; den += e2; }
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) den += __shfl_xor(den, o, 16);
            for (int s2 = sub; s2 < T; s2 += 16) {
                const float pv = s2 < n ? row[s2 * TA_SS] / den : 0.f;
                if (t < T) P[grow + s2] = pv;
                row[s2 * TA_SS] = pv;
            }
        } else {
            float dot = 0.f;
            for (int s2 = sub; s2 < n; s2 += 16) dot += row[s2 * TA_SS] * P[grow + s2];
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 16);
            for (int s2 = sub; s2 < T; s2 += 16) {
                const float g2 = s2 < n ? P[grow + s2] * (row[s2 * TA_SS] - dot) * scale : 0.f;
                if (t < T) dS[grow + s2] = g2;
                row[s2 * TA_SS] = g2;
            }
        }
    }
    // phase 3: out = scores . B2 with B2 = V (forward) or K (backward); thread = (head dim, group of positions)
    const int groups = 256 / hd, rpg = TA_TQ / groups, e = tid % hd, g = tid / hd;   // hd 128: 2 groups of 8; hd 64: 4 of 4
    float o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 <= t_last; k0 += TA_TK) {
        __syncthreads();
        ta_stage(tile, MODE == 0 ? vbase : kbase, qkvd, k0, T, hd);
        __syncthreads();
        const int cnt = min(TA_TK, t_last + 1 - k0);
        for (int s2 = 0; s2 < cnt; s2++) {
            const float bv = tile[s2 * (hd + 1) + e];
            const float *ps = sc + (k0 + s2) * TA_SS + g * rpg;
            const float4 p0 = *reinterpret_cast<const float4 *>(ps);
            o8[0] += p0.x * bv; o8[1] += p0.y * bv; o8[2] += p0.z * bv; o8[3] += p0.w * bv;
            if (rpg == 8) {
                const float4 p1 = *reinterpret_cast<const float4 *>(ps + 4);
                o8[4] += p1.x * bv; o8[5] += p1.y * bv; o8[6] += p1.z * bv; o8[7] += p1.w * bv;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int t = t0 + g * rpg + i;
        if (i < rpg && t < T) {
            if (MODE == 0) out[(size_t)(b * T + t) * Hq * hd + (size_t)hq * hd + e] = o8[i];
            else out[(size_t)(b * T + t) * qkvd + (size_t)hq * hd + e] = o8[i];
        }
    }
}

// dk[s] = sum over the kv head's query heads (in order) and t >= s (ascending) of dS[t, s] q[t]; dv[s] likewise from P and
// datt.  One block per (tile of 16 keys, kv head, chain); q and datt rows go through LDS 64 positions at a time, with the
// matching [64][16] pieces of dS and P (zero above the diagonal as stored, so nothing is masked here).
__global__ __launch_bounds__(256) void train_attn_tile_kv_kernel(const float *__restrict__ qkv, const float *__restrict__ P,
                                                                 const float *__restrict__ dS, const float *__restrict__ datt,
                                                                 float *__restrict__ dqkv, int T, int Hq, int Hkv, int hd, int qkvd)
{
    extern __shared__ __align__(16) float ta_lds[];
    float *qt = ta_lds, *dt = qt + TA_TK * (hd + 1), *dsT = dt + TA_TK * (hd + 1), *pT = dsT + TA_TK * TA_TQ;   // 64 (hd + 1) is a multiple of 4
    const int s0 = blockIdx.x * TA_TQ, hk = blockIdx.y, b = blockIdx.z, G = Hq / Hkv, tid = threadIdx.x;
    const int groups = 256 / hd, rpg = TA_TQ / groups, e = tid % hd, g = tid / hd;
    float dk[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, dv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int gq = 0; gq < G; gq++) {
        const int hq = hk * G + gq;
        const size_t prow0 = ((size_t)b * Hq + hq) * T;
        for (int tt = (s0 / TA_TK) * TA_TK; tt < T; tt += TA_TK) {
            __syncthreads();
            ta_stage(qt, qkv + (size_t)b * T * qkvd + (size_t)hq * hd, qkvd, tt, T, hd);
            ta_stage(dt, datt + (size_t)b * T * Hq * hd + (size_t)hq * hd, (size_t)Hq * hd, tt, T, hd);
            for (int idx = tid; idx < TA_TK * TA_TQ; idx += 256) {
                const int r = idx >> 4, j = idx & 15, t = tt + r, s2 = s0 + j;
                const bool in = t < T && s2 < T;
                dsT[idx] = in ? dS[(prow0 + t) * T + s2] : 0.f;
                pT[idx] = in ? P[(prow0 + t) * T + s2] : 0.f;
            }
            __syncthreads();
            const int cnt = min(TA_TK, T - tt);
            for (int r = 0; r < cnt; r++) {
                const float qv = qt[r * (hd + 1) + e], dov = dt[r * (hd + 1) + e];
                const float4 d0 = *reinterpret_cast<const float4 *>(dsT + r * TA_TQ + g * rpg);
                const float4 p0 = *reinterpret_cast<const float4 *>(pT + r * TA_TQ + g * rpg);
                dk[0] += d0.x * qv; dk[1] += d0.y * qv; dk[2] += d0.z * qv; dk[3] += d0.w * qv;
                dv[0] += p0.x * dov; dv[1] += p0.y * dov; dv[2] += p0.z * dov; dv[3] += p0.w * dov;
                if (rpg == 8) {
                    const float4 d1 = *reinterpret_cast<const float4 *>(dsT + r * TA_TQ + g * rpg + 4);
                    const float4 p1 = *reinterpret_cast<const float4 *>(pT + r * TA_TQ + g * rpg + 4);
                    dk[4] += d1.x * qv; dk[5] += d1.y * qv; dk[6] += d1.z * qv; dk[7] += d1.w * qv;
                    dv[4] += p1.x * dov; dv[5] += p1.y * dov; dv[6] += p1.z * dov; dv[7] += p1.w * dov;
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int s2 = s0 + g * rpg + i;
        if (i < rpg && s2 < T) {
            dqkv[(size_t)(b * T + s2) * qkvd + (size_t)(Hq + hk) * hd + e] = dk[i];
            dqkv[(size_t)(b * T + s2) * qkvd + (size_t)(Hq + Hkv + hk) * hd + e] = dv[i];
        }
    }
}

static bool train_attn_tiled_ok(int T, int hd) { return (hd == 64 || hd == 128) && T <= 1024; }
static size_t train_attn_tile_lds(int T, int hd)
{
    // the tile is rounded up to whole 16-byte rows so that the score array behind it stays aligned
    return sizeof(float) * ((size_t)hd * TA_TQ + (size_t)(TA_TK * (hd + 1) + 3) / 4 * 4 + (size_t)TA_SS * ((T + 63) / 64 * 64));
}
// more than 64 KiB of dynamic LDS has to be allowed per kernel
static int32_t allow_lds(const void *kernel, size_t bytes)
{
    if (bytes <= 65536) return FG_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(FG_ERR_HIP, "cannot reserve %zu bytes of LDS", bytes);
    }
    return FG_OK;
}
static size_t train_attn_tile_kv_lds(int hd) { return sizeof(float) * (2 * (size_t)TA_TK * (hd + 1) + 2 * (size_t)TA_TK * TA_TQ); }

__global__ void train_swiglu_fwd_kernel(const float *gate, const float *up, float *act, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { const float g = gate[i]; act[i] = g / (1.f + expf(-g)) * up[i]; }
}

__global__ void train_swiglu_bwd_kernel(const float *dact, const float *gate, const float *up, float *dgate, float *dup, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float g = gate[i], sg = 1.f / (1.f + expf(-g));
    dup[i] = dact[i] * g * sg;
    dgate[i] = dact[i] * up[i] * (sg + g * sg * (1.f - sg));
}

// running (maximum, sum of exp(x - maximum)) of a stream of values, and the merge of two of them
struct MaxSum { float m, s; };
__device__ __forceinline__ void maxsum_add(MaxSum &a, float x)
{
    if (x > a.m) { a.s = a.s * expf(a.m - x) + 1.f; a.m = x; }
    else a.s += expf(x - a.m);
}
__device__ __forceinline__ MaxSum maxsum_merge(MaxSum a, MaxSum b)
{
    const float m = fmaxf(a.m, b.m);
    if (m == -INFINITY) return MaxSum{m, 0.f};
    return MaxSum{m, a.s * expf(a.m - m) + b.s * expf(b.m - m)};
}
__device__ __forceinline__ MaxSum block_maxsum256(MaxSum v, MaxSum *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = maxsum_merge(v, MaxSum{__shfl_xor(v.m, o, 64), __shfl_xor(v.s, o, 64)});
    __syncthreads();   // the previous use of red is over
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return maxsum_merge(maxsum_merge(red[0], red[1]), maxsum_merge(red[2], red[3]));
}

// Per row: the regression term and its gradient, the cross-entropy term between softmax(zt) and softmax(z), and the
// gradient of the total with respect to z, written over z.  Rows past n_valid get zero gradients and no loss.
__global__ __launch_bounds__(256) void train_loss_kernel(const float *h2, const float *feat_tgt, float *z, const float *zt,
                                                         const int32_t *n_valid, const int32_t *n_tot_dev, int T, int d, int V,
                                                         float w_ce, float *dh2, float *row_loss)
{
    __shared__ float red[4];
    __shared__ MaxSum red2[4];
    const int r = blockIdx.x, b = r / T, t = r % T;
    float *zr = z + (size_t)r * V;
    const float *ztr = zt + (size_t)r * V;
    if (t >= n_valid[b]) {
        for (int v = threadIdx.x; v < V; v += 256) zr[v] = 0.f;
        for (int e = threadIdx.x; e < d; e += 256) dh2[(size_t)r * d + e] = 0.f;
        if (threadIdx.x == 0) { row_loss[2 * r] = 0.f; row_loss[2 * r + 1] = 0.f; }
        return;
    }
    const float n_tot = (float)n_tot_dev[0];
    float reg = 0.f;
    for (int e = threadIdx.x; e < d; e += 256) {
        const float df = h2[(size_t)r * d + e] - feat_tgt[(size_t)r * d + e], ad = fabsf(df);
        reg += ad < 1.f ? 0.5f * df * df : ad - 0.5f;
        dh2[(size_t)r * d + e] = (ad < 1.f ? df : (df < 0.f ? -1.f : 1.f)) / (float)d / n_tot;
    }
    reg = block_sum256(reg, red) / (float)d;
    // log-sum-exp of both rows in one pass: a running (maximum, sum of exp(x - maximum)) per thread, merged in a fixed order
    MaxSum aq = {-INFINITY, 0.f}, ap = {-INFINITY, 0.f};
    for (int v = threadIdx.x; v < V; v += 256) { maxsum_add(aq, zr[v]); maxsum_add(ap, ztr[v]); }
    aq = block_maxsum256(aq, red2);
    ap = block_maxsum256(ap, red2);
    const float lq = aq.m + logf(aq.s), lp = ap.m + logf(ap.s);
    float ce = 0.f;
    for (int v = threadIdx.x; v < V; v += 256) {
        const float pv = expf(ztr[v] - lp), zq = zr[v], qv = expf(zq - lq);
        ce -= pv * (zq - lq);
        zr[v] = w_ce * (qv - pv) / n_tot;
    }
    ce = block_sum256(ce, red);
    if (threadIdx.x == 0) { row_loss[2 * r] = reg; row_loss[2 * r + 1] = ce; }
}

// n_tot = sum of n_valid (one thread: B is small); later: loss = sum of the row terms in row order / n_tot
__global__ void train_count_kernel(const int32_t *n_valid, int B, int T, int32_t *n_tot)
{
    int s = 0;
    for (int b = 0; b < B; b++) s += min(max(n_valid[b], 0), T);
    n_tot[0] = max(s, 1);
}
__global__ void train_loss_reduce_kernel(const float *row_loss, int M, const int32_t *n_tot, float *loss)
{
    __shared__ float red[4];
    float a = 0.f, c = 0.f;
    for (int r = threadIdx.x; r < M; r += 256) { a += row_loss[2 * r]; c += row_loss[2 * r + 1]; }
    a = block_sum256(a, red);
    c = block_sum256(c, red);
    if (threadIdx.x == 0) { loss[0] = a / (float)n_tot[0]; loss[1] = c / (float)n_tot[0]; }
}

__global__ void adamw_kernel(float *p, const float *g, float *m, float *v, size_t n, float lr, float b1, float b2, float eps,
                             float wd, float c1, float c2)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float gi = g[i];
    const float mi = b1 * m[i] + (1.f - b1) * gi, vi = b2 * v[i] + (1.f - b2) * gi * gi;
    m[i] = mi;
    v[i] = vi;
    p[i] -= lr * ((mi / c1) / (sqrtf(vi / c2) + eps) + wd * p[i]);
}

// ---- the step ----------------------------------------------------------------------------------------------------------
struct TrainWs {
    float *cat, *h0, *a1, *inv1, *qkv, *P, *dS, *att, *h1, *a2, *inv2, *gate, *up, *act, *h2, *z, *zt, *dh2, *dact, *dgate, *dup,
        *da, *dh1, *datt, *dqkv, *dx, *row_loss, *dg_part;
    int32_t *n_tot;
    Mfma16 mm;
};

static int64_t carve_train(const fg_model_cfg &c, int B, int T, void *base, int64_t cap, TrainWs *w)
{
    const int64_t M = (int64_t)B * T, d = c.d_model, F = c.d_ffn, V = c.vocab, hq = (int64_t)c.n_q_heads * c.head_dim;
    const int64_t qkvd = (int64_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    int64_t off = 0;
    auto take = [&](int64_t n) {
        off = align_up(off, 256);
        float *p = (float *)((char *)base + off);
        off += n * 4;
        return p;
    };
    TrainWs s;
    s.cat = take(M * 2 * d); s.h0 = take(M * d); s.a1 = take(M * d); s.inv1 = take(M); s.qkv = take(M * qkvd);
    s.P = take((int64_t)B * c.n_q_heads * T * T); s.dS = take((int64_t)B * c.n_q_heads * T * T); s.att = take(M * hq);
    s.h1 = take(M * d); s.a2 = take(M * d); s.inv2 = take(M); s.gate = take(M * F); s.up = take(M * F); s.act = take(M * F);
    s.h2 = take(M * d); s.z = take(M * V); s.zt = take(M * V); s.dh2 = take(M * d); s.dact = take(M * F); s.dgate = take(M * F);
    s.dup = take(M * F); s.da = take(M * d); s.dh1 = take(M * d); s.datt = take(M * hq); s.dqkv = take(M * qkvd); s.dx = take(M * d);
    s.row_loss = take(M * 2); s.dg_part = take((M + DG_ROWS - 1) / DG_ROWS * d); s.n_tot = (int32_t *)take(64);
    if (is16(c.dtype)) {
        // largest first operand: the logit gradients [M, V]; largest second operand: the LM head [V, d]
        const int64_t big = V > F ? V : F, wide = F > 2 * d ? F : 2 * d, rows = M > d ? M : d;
        s.mm.x_cap = M * (big > 2 * d ? big : 2 * d);
        s.mm.w_cap = V * d > wide * rows ? V * d : wide * rows;
        s.mm.x16 = (bf16_t *)take((s.mm.x_cap + 1) / 2);
        s.mm.wp = (bf16_t *)take((s.mm.w_cap + 1) / 2);
    }
    if (w) *w = s;
    if (base && off > cap) return -1;
    return align_up(off, 256);
}

int64_t draft_train_ws_bytes(const fg_model_cfg &c, int B, int T) { return carve_train(c, B, T, nullptr, 0, nullptr); }

// The frozen LM head [V, d] in the two packed forms a matrix-core step multiplies with: as the second operand of
// logits = x . head^T (n_out = V, n_in = d), and of dx = dlogits . head (n_out = d, n_in = V, i.e. the transpose).
int64_t draft_train_head_bytes(const fg_model_cfg &c) { return 2 * align_up((int64_t)c.vocab * c.d_model * 2, 256); }
int32_t launch_draft_train_pack_head(const fg_model_cfg &c, const float *lm_head, void *packed, hipStream_t st)
{
    char *p = (char *)packed;
    int32_t rc = launch_pack_cast_bf16(lm_head, p, c.vocab, c.d_model, st);
    if (rc) return rc;
    return launch_pack_cast_t_bf16(lm_head, p + align_up((int64_t)c.vocab * c.d_model * 2, 256), c.d_model, c.vocab, st);
}

int32_t launch_draft_train_grad(const fg_model_cfg &c, const float *embed, const float *lm_head, const fg_draft_params *w,
                                const int32_t *tokens, const float *feat_in, const float *feat_tgt, const int32_t *n_valid, int B,
                                int T, float w_ce, fg_draft_params *g, float *loss, const void *head_packed, void *ws,
                                int64_t ws_bytes, hipStream_t st)
{
    TrainWs s;
    if (carve_train(c, B, T, ws, ws_bytes, &s) < 0) return fail(FG_ERR_CAPACITY, "fg_draft_train_grad: workspace too small");
    if (head_packed && c.dtype == FG_BF16) {
        s.mm.head_src = lm_head;
        s.mm.head_fwd = (const bf16_t *)head_packed;
        s.mm.head_bwd = (const bf16_t *)((const char *)head_packed + align_up((int64_t)c.vocab * c.d_model * 2, 256));
    }
    const int M = B * T, d = c.d_model, F = c.d_ffn, V = c.vocab, Hq = c.n_q_heads, Hkv = c.n_kv_heads, hd = c.head_dim;
    const int hq = Hq * hd, qkvd = (Hq + 2 * Hkv) * hd;
    const float scale = 1.0f / sqrtf((float)hd);
    const size_t lds = (size_t)T * sizeof(float);
    int32_t rc;
    // fp32 throughout, or the GEMMs on the matrix cores with bf16 operands (fp16 would flush the gradients to zero)
    const bool mfma = c.dtype == FG_BF16;
    auto gemm = [&](int op, const float *A, const float *Bm, float *C, const float *add, int Mo, int No, int Ko, hipStream_t) -> int32_t {
        return mfma ? gemm16(s.mm, op, A, Bm, C, add, Mo, No, Ko, st) : sgemm(op, A, Bm, C, add, Mo, No, Ko, st);
    };
    // forward
    hipLaunchKernelGGL(train_count_kernel, dim3(1), dim3(1), 0, st, n_valid, B, T, s.n_tot);
    hipLaunchKernelGGL(train_concat_kernel, dim3(M), dim3(256), 0, st, embed, tokens, V, feat_in, s.cat, d);
    if ((rc = gemm(0, s.cat, w->fc, s.h0, nullptr, M, d, 2 * d, st))) return rc;
    hipLaunchKernelGGL(rms_fwd_kernel, dim3(M), dim3(256), 0, st, s.h0, w->norm_attn, s.a1, s.inv1, d, c.rms_eps);
    if ((rc = gemm(0, s.a1, w->wqkv, s.qkv, nullptr, M, qkvd, d, st))) return rc;
    hipLaunchKernelGGL(train_rope_kernel, dim3(M), dim3(256), 0, st, s.qkv, T, Hq + Hkv, hd, qkvd, (double)c.rope_theta, 1);
    const bool tiled = train_attn_tiled_ok(T, hd);
    const int Tp = (T + 63) / 64 * 64, tq = (T + TA_TQ - 1) / TA_TQ;
    if (tiled && ((rc = allow_lds((const void *)train_attn_tile_kernel<0>, train_attn_tile_lds(T, hd))) ||
                  (rc = allow_lds((const void *)train_attn_tile_kernel<1>, train_attn_tile_lds(T, hd))) ||
                  (rc = allow_lds((const void *)train_attn_tile_kv_kernel, train_attn_tile_kv_lds(hd)))))
        return rc;
    if (tiled)
        hipLaunchKernelGGL(train_attn_tile_kernel<0>, dim3(tq, Hq, B), dim3(256), train_attn_tile_lds(T, hd), st, s.qkv, s.P, nullptr,
                           nullptr, s.att, T, Tp, Hq, Hkv, hd, qkvd, scale);
    else
        hipLaunchKernelGGL(train_attn_fwd_kernel, dim3(T, Hq, B), dim3(256), lds, st, s.qkv, s.P, s.att, T, Hq, Hkv, hd, qkvd, scale);
    if ((rc = gemm(0, s.att, w->wo, s.h1, s.h0, M, d, hq, st))) return rc;
    hipLaunchKernelGGL(rms_fwd_kernel, dim3(M), dim3(256), 0, st, s.h1, w->norm_ffn, s.a2, s.inv2, d, c.rms_eps);
    if ((rc = gemm(0, s.a2, w->w_gate, s.gate, nullptr, M, F, d, st))) return rc;
    if ((rc = gemm(0, s.a2, w->w_up, s.up, nullptr, M, F, d, st))) return rc;
    const size_t nf = (size_t)M * F;
    hipLaunchKernelGGL(train_swiglu_fwd_kernel, dim3((unsigned)((nf + 255) / 256)), dim3(256), 0, st, s.gate, s.up, s.act, nf);
    if ((rc = gemm(0, s.act, w->w_down, s.h2, s.h1, M, d, F, st))) return rc;
    if ((rc = gemm(0, s.h2, lm_head, s.z, nullptr, M, V, d, st))) return rc;
    if ((rc = gemm(0, feat_tgt, lm_head, s.zt, nullptr, M, V, d, st))) return rc;
    // loss, d loss / d z (over z) and the regression part of d loss / d h2
    hipLaunchKernelGGL(train_loss_kernel, dim3(M), dim3(256), 0, st, s.h2, feat_tgt, s.z, s.zt, n_valid, s.n_tot, T, d, V, w_ce, s.dh2,
                       s.row_loss);
    hipLaunchKernelGGL(train_loss_reduce_kernel, dim3(1), dim3(256), 0, st, s.row_loss, M, s.n_tot, loss);
    // backward
    if ((rc = gemm(1, s.z, lm_head, s.dh2, s.dh2, M, d, V, st))) return rc;              // through the frozen LM head
    if ((rc = gemm(2, s.dh2, s.act, g->w_down, nullptr, d, F, M, st))) return rc;
    if ((rc = gemm(1, s.dh2, w->w_down, s.dact, nullptr, M, F, d, st))) return rc;
    hipLaunchKernelGGL(train_swiglu_bwd_kernel, dim3((unsigned)((nf + 255) / 256)), dim3(256), 0, st, s.dact, s.gate, s.up, s.dgate,
                       s.dup, nf);
    if ((rc = gemm(2, s.dgate, s.a2, g->w_gate, nullptr, F, d, M, st))) return rc;
    if ((rc = gemm(2, s.dup, s.a2, g->w_up, nullptr, F, d, M, st))) return rc;
    if ((rc = gemm(1, s.dgate, w->w_gate, s.da, nullptr, M, d, F, st))) return rc;
    if ((rc = gemm(1, s.dup, w->w_up, s.da, s.da, M, d, F, st))) return rc;
    const int dg_chunks = (M + DG_ROWS - 1) / DG_ROWS;
    auto dgain = [&](const float *dy, const float *x, const float *inv, float *dg) {
        hipLaunchKernelGGL(rms_dgain_part_kernel, dim3((d + 255) / 256, dg_chunks), dim3(256), 0, st, dy, x, inv, s.dg_part, M, d);
        hipLaunchKernelGGL(rms_dgain_sum_kernel, dim3((d + 255) / 256), dim3(256), 0, st, s.dg_part, dg, dg_chunks, d);
    };
    dgain(s.da, s.h1, s.inv2, g->norm_ffn);
    hipLaunchKernelGGL(rms_bwd_kernel, dim3(M), dim3(256), 0, st, s.da, s.h1, w->norm_ffn, s.inv2, s.dh2, s.dh1, d);
    if ((rc = gemm(2, s.dh1, s.att, g->wo, nullptr, d, hq, M, st))) return rc;
    if ((rc = gemm(1, s.dh1, w->wo, s.datt, nullptr, M, hq, d, st))) return rc;
    if (tiled) {
        hipLaunchKernelGGL(train_attn_tile_kernel<1>, dim3(tq, Hq, B), dim3(256), train_attn_tile_lds(T, hd), st, s.qkv, s.P, s.dS,
                           s.datt, s.dqkv, T, Tp, Hq, Hkv, hd, qkvd, scale);
        hipLaunchKernelGGL(train_attn_tile_kv_kernel, dim3(tq, Hkv, B), dim3(256), train_attn_tile_kv_lds(hd), st, s.qkv, s.P, s.dS,
                           s.datt, s.dqkv, T, Hq, Hkv, hd, qkvd);
    } else {
        hipLaunchKernelGGL(train_attn_bwd_q_kernel, dim3(T, Hq, B), dim3(256), lds, st, s.qkv, s.P, s.datt, s.dS, s.dqkv, T, Hq, Hkv,
                           hd, qkvd, scale);
        hipLaunchKernelGGL(train_attn_bwd_kv_kernel, dim3(T, Hkv, B), dim3(hd <= 64 ? 64 : 128), 0, st, s.qkv, s.P, s.dS, s.datt,
                           s.dqkv, T, Hq, Hkv, hd, qkvd);
    }
    hipLaunchKernelGGL(train_rope_kernel, dim3(M), dim3(256), 0, st, s.dqkv, T, Hq + Hkv, hd, qkvd, (double)c.rope_theta, -1);
    if ((rc = gemm(2, s.dqkv, s.a1, g->wqkv, nullptr, qkvd, d, M, st))) return rc;
    if ((rc = gemm(1, s.dqkv, w->wqkv, s.da, nullptr, M, d, qkvd, st))) return rc;
    dgain(s.da, s.h0, s.inv1, g->norm_attn);
    hipLaunchKernelGGL(rms_bwd_kernel, dim3(M), dim3(256), 0, st, s.da, s.h0, w->norm_attn, s.inv1, s.dh1, s.dx, d);
    if ((rc = gemm(2, s.dx, s.cat, g->fc, nullptr, d, 2 * d, M, st))) return rc;
    FG_LAUNCH_CHECK("draft_train_grad");
    return FG_OK;
}

int32_t launch_adamw(float *p, const float *g, float *m, float *v, int64_t n, float lr, float b1, float b2, float eps, float wd,
                     int step, hipStream_t st)
{
    if (n <= 0) return FG_OK;
    const float c1 = 1.f - powf(b1, (float)step), c2 = 1.f - powf(b2, (float)step);
    hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, g, m, v, (size_t)n, lr, b1, b2, eps, wd, c1, c2);
    FG_LAUNCH_CHECK("adamw");
    return FG_OK;
}

}  // namespace fg
