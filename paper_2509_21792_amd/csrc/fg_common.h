// Internal helpers of libfastgrpo: error state, small device utilities, launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "fastgrpo.h"

namespace fg {

// ---- error state (thread local) -------------------------------------------------------------------
int32_t fail(int32_t code, const char *fmt, ...);
#define FG_HIP(call)                                                                                   \
    do {                                                                                               \
        hipError_t e_ = (call);                                                                        \
        if (e_ != hipSuccess) return fg::fail(FG_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_));     \
    } while (0)
#define FG_LAUNCH_CHECK(name)                                                                          \
    do {                                                                                               \
        hipError_t e_ = hipGetLastError();                                                             \
        if (e_ != hipSuccess) return fg::fail(FG_ERR_HIP, "launch of %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// ---- element types --------------------------------------------------------------------------------
typedef uint16_t bf16_t;  // storage only
typedef _Float16 f16_t;

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even (inputs are finite here)
    return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf2f(v); }
template <> __device__ __forceinline__ float to_f<f16_t>(f16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return f2bf(v); }
template <> __device__ __forceinline__ f16_t from_f<f16_t>(float v) { return (f16_t)v; }

// SwiGLU of one (gate, up) pair in fp32: silu(g) * u, with the hardware's exp2 and reciprocal approximations (each within
// 1 ulp of fp32; an exact division costs about ten instructions more per element and is lost in the 16-bit store anyway).
// Every kernel that applies SwiGLU calls this, so a fused epilogue and the separate kernel give identical bits.
__device__ __forceinline__ float swiglu_f(float g, float u) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u; }

static inline size_t dtype_size(int32_t dtype) { return dtype == FG_F32 ? 4 : 2; }
static inline bool dtype_ok(int32_t dtype) { return dtype == FG_F32 || dtype == FG_BF16 || dtype == FG_F16; }
static inline bool is16(int32_t dtype) { return dtype == FG_BF16 || dtype == FG_F16; }

// K page layout of one (layer, page, kv head): page_size x head_dim elements.  16-bit caches with 16-token pages
// and head_dim a multiple of 32 keep a page in MFMA operand order -- head_dim / 32 fragments of 64 x 8 elements,
// fragment kk = [lane = grp * 16 + token][8] holding dims grp * (head_dim / 4) + kk * 8 .. + 7 -- so that the
// attention kernel fetches a fragment as one contiguous 1 KiB; everything else is token-major [token][dim].
// Four consecutive dims that start at a multiple of four are contiguous in both layouts.
static inline bool k_fragment_major(int32_t dtype, int head_dim, int page_size)
{
    return is16(dtype) && page_size == 16 && head_dim % 32 == 0;
}
__host__ __device__ __forceinline__ int k_page_offset(bool fragment_major, int head_dim, int t, int e)
{
    if (!fragment_major) return t * head_dim + e;
    const int q = head_dim >> 2, grp = e / q, r = e - grp * q;
    return (((r >> 3) * 4 + grp) * 16 + t) * 8 + (r & 7);
}

// run a statement with T bound to the element type of `dtype`
#define FG_DISPATCH(dtype, T, ...)                                       \
    do {                                                                 \
        if ((dtype) == FG_BF16) { using T = fg::bf16_t; __VA_ARGS__; }   \
        else if ((dtype) == FG_F16) { using T = fg::f16_t; __VA_ARGS__; } \
        else { using T = float; __VA_ARGS__; }                           \
    } while (0)
static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// ---- wave / block reductions (wave64) -------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- counter-based uniforms (SplitMix64 finaliser) ------------------------------------------------
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
__device__ __forceinline__ uint64_t row_key(uint64_t seed, uint64_t row) { return mix64(seed ^ (row * 0xD1B54A32D192ED03ULL)); }
__device__ __forceinline__ float uniform_from_key(uint64_t key, uint64_t v)
{
    uint64_t bits = mix64(key + v);
    return ((float)(bits >> 41) + 0.5f) * (1.0f / 8388608.0f);
}
__device__ __forceinline__ float gumbel_from_key(uint64_t key, uint64_t v) { return -logf(-logf(uniform_from_key(key, v))); }

// ---- launchers (one per kernel family; all asynchronous on `st`) -------------------------------------
struct TreeDev {             // per-call derived tree data in the workspace
    int32_t *pos;            // [B*N] position of each new node
    uint64_t *mask;          // [B*N] in-round ancestors-or-self of each new node (bit i = in-round node i)
    int32_t *dest;           // [B*N] cache cell of each new node: page * 16 + position in the page (same in every layer)
};

// Epilogues of the 16-bit GEMM.  SLABS and SWIGLU exist in every kernel; ROPE, RESIDUAL and TOPK only in the pipelined
// kernel without a k split (gemm_mfma_fusable says whether a shape gets them; the caller otherwise takes SLABS and runs
// the separate row-wise kernel).
enum { EPI_SLABS = 0, EPI_SWIGLU = 1, EPI_ROPE = 2, EPI_RESIDUAL = 3, EPI_TOPK = 4 };
struct GemmEpi {
    // EPI_ROPE: the GEMM is the QKV projection.  q and k heads are rotated (pairing i, i + hd/2) at pos[row]; q rows go
    // to q_out [M, Hq * hd], the node's k and v into its cache cell dest[row] (page * 16 + slot) of `layer`.
    const int32_t *pos = nullptr, *dest = nullptr;
    void *k_pool = nullptr, *v_pool = nullptr, *q_out = nullptr;
    const float2 *rope_tab = nullptr;
    int layer = 0, n_pages = 0, Hq = 0, Hkv = 0, hd = 0, max_pos = 0, k_frag = 0;
    // EPI_RESIDUAL: h [M, N] fp32 += x . W^T
    float *h = nullptr;
    // EPI_TOPK: per row and 256-column block the topk largest outputs (value, column; ties to the lower column) and
    // the block's (max, sum of exp(x - max)): part_val / part_idx [M][blocks][topk], part_ms [M][blocks][2]
    int topk = 0;
    float *part_val = nullptr;
    int32_t *part_idx = nullptr;
    float *part_ms = nullptr;
};
// variant: 0 = the library's choice of kernel; 1 streaming, 2 few-row, 3 / 4 / 5 pipelined with 256- / 128- / 160-row
// blocks (kernel-level measurements and tests)
int32_t launch_gemm_mfma(int32_t dtype, const void *x, const void *wp, void *out, int M, int N, int K, int epilogue,
                         int split_k, int *split_used, hipStream_t st, const GemmEpi *epi = nullptr, int variant = 0);
bool gemm_mfma_fusable(int M, int N, int K, int kind);
int32_t launch_gemm_f32(const float *x, const float *w, float *out, int M, int N, int K, hipStream_t st);
int32_t launch_pack(int32_t dtype, const void *src, const void *src2, void *dst, int64_t n_out, int64_t n_in, hipStream_t st);
int32_t launch_pack_cast_bf16(const float *src, void *dst, int64_t n_out, int64_t n_in, hipStream_t st);   // fp32 source, bf16 fragments
int32_t launch_pack_cast_t_bf16(const float *src, void *dst, int64_t n_out, int64_t n_in, hipStream_t st); // src is [n_in, n_out]

int32_t launch_embed(int32_t dtype, const void *embed, const int32_t *tokens, int vocab, float *h, int M, int d, hipStream_t st);
int32_t launch_concat_embed(int32_t dtype, const void *embed, const int32_t *tokens, int vocab, const void *feat,
                            const int32_t *feat_index, int N, int feat_rows, void *cat, int M, int d, hipStream_t st);
// h (+)= sum of S partial slabs; optional norm output a = rmsnorm(h) * gain (dtype), optional copy of h as dtype
int32_t launch_add_rmsnorm(int32_t dtype, float *h, const float *partials, int S, int init, const void *gain, void *a,
                           void *h_copy, int M, int d, float eps, hipStream_t st);
int32_t launch_rope_append(int32_t dtype, const float *qkv_partials, int S, const fg_tree *t, TreeDev td, const fg_kv_cache *kv,
                           int layer, const float *rope_tab, int max_pos, int Hq, void *q_out, hipStream_t st);
int32_t launch_swiglu_f32(const float *gu, float *act, int M, int F, hipStream_t st);
int32_t launch_argmax_top2(const float *logits, int M, int V, int32_t *idx, float *top2, hipStream_t st);


}  // namespace fg
