// fp32 GEMM for the fp32 parity configuration: out[M, N] = X[M, K] . W[N, K]^T, plain FMA, LDS tiled.
// Not a performance path (the fp32 model is launch-latency bound); it exists so that the whole pipeline can be
// checked against the fp32 oracle at 1e-4 without bf16 rounding in the way.
#include "fg_common.h"

namespace fg {

constexpr int TB = 64, TK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ X, const float *__restrict__ W,
                                                       float *__restrict__ out, int M, int N, int K)
{
    __shared__ float xs[TK][TB + 1], ws[TK][TB + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * TB, n0 = blockIdx.x * TB;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += TK) {
        for (int i = tid; i < TB * TK; i += 256) {
            int r = i / TK, c = i % TK;
            int m = m0 + r, n = n0 + r, k = k0 + c;
            xs[c][r] = (m < M && k < K) ? X[(size_t)m * K + k] : 0.f;
            ws[c][r] = (n < N && k < K) ? W[(size_t)n * K + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < TK; c++) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; i++) { a[i] = xs[c][ty * 4 + i]; b[i] = ws[c][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) out[(size_t)m * N + n] = acc[i][j];
        }
}

int32_t launch_gemm_f32(const float *x, const float *w, float *out, int M, int N, int K, hipStream_t st)
{
    if (M <= 0) return FG_OK;
    dim3 grid((N + TB - 1) / TB, (M + TB - 1) / TB);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, x, w, out, M, N, K);
    FG_LAUNCH_CHECK("gemm_f32");
    return FG_OK;
}

}  // namespace fg
