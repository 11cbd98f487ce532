// Device-side helpers shared by the libpoly kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/poly.h"
#include "../../include/poly_profile.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define POLY_WAVE 64

// Device-visible bookkeeping at the head of the workspace.
struct PolyMeta {
    int32_t R;       // row_offsets[F] as read on the device (0 when the inputs are rejected)
    int32_t status;  // POLY_OK or POLY_ERANGE
    int32_t F_ok;    // number of frames, or 0 when the inputs are rejected
    int32_t pad[61];
};

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

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; }

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f)); }

// erf-GELU without transcendental instructions, for results that are rounded to bf16 afterwards:
//     GELU(x) = x * Phi(x),   Phi(x) - 1/2 = erf(x / sqrt 2) / 2 ~= xc * Q(xc^2),   xc = clamp(x, -4.4, 4.4),
// Q a degree-8 polynomial (weighted least-squares fit on Chebyshev nodes of [0, 4.4^2]).  The constant is a hair
// under 1/2 so that Phi reaches exactly 0 on the negative tail (max with 0) instead of a tiny positive slope.
// Measured against the double-precision definition: absolute error below 4e-5 on |x| <= 8, relative error below
// 3.2e-4 wherever |GELU| > 0.05 -- a sixth of half a bf16 ulp.  14 plain fp32 instructions.
__device__ __forceinline__ float gelu_poly(float x)
{
    const float xc = __builtin_amdgcn_fmed3f(x, -4.4f, 4.4f);
    const float s = xc * xc;
    float q = fmaf(3.446953140e-11f, s, -3.649543778e-09f);
    q = fmaf(q, s, 1.703905070e-07f);
    q = fmaf(q, s, -4.655028533e-06f);
    q = fmaf(q, s, 8.353321027e-05f);
    q = fmaf(q, s, -1.050237101e-03f);
    q = fmaf(q, s, 9.626936167e-03f);
    q = fmaf(q, s, -6.605132669e-02f);
    q = fmaf(q, s, 3.987498879e-01f);
    return x * fmaxf(fmaf(xc, q, 0.499994f), 0.f);
}
// four at a time, written so that the four dependency chains advance together: one chain alone leaves the vector
// pipeline idle between dependent instructions
__device__ __forceinline__ f32x4 gelu_poly4(f32x4 x)
{
    f32x4 xc, s, q;
#pragma unroll
    for (int i = 0; i < 4; ++i) xc[i] = __builtin_amdgcn_fmed3f(x[i], -4.4f, 4.4f);
    s = xc * xc;
#pragma unroll
    for (int i = 0; i < 4; ++i) q[i] = fmaf(3.446953140e-11f, s[i], -3.649543778e-09f);
    const float c[7] = {1.703905070e-07f, -4.655028533e-06f, 8.353321027e-05f, -1.050237101e-03f, 9.626936167e-03f, -6.605132669e-02f, 3.987498879e-01f};
#pragma unroll
    for (int j = 0; j < 7; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) q[i] = fmaf(q[i], s[i], c[j]);
#pragma unroll
    for (int i = 0; i < 4; ++i) q[i] = x[i] * fmaxf(fmaf(xc[i], q[i], 0.499994f), 0.f);
    return q;
}

// erf-GELU through a table of Phi in LDS, for kernels whose inner loop is bound by the number of instructions it
// issues: GELU(x) = x * Phi(x), Phi linearly interpolated between samples 1/64 apart on [-4.5, 4.5] (clamped
// outside: Phi(-4.5) = 3.4e-6, 1 - Phi(4.5) = 3.4e-6).  Interpolation error <= h^2 / 8 * max|Phi''| = 7.4e-6.
// Entry i holds (Phi(x_i), Phi(x_{i+1}) - Phi(x_i)), x_i = (i - 288) / 64, i = 0 .. 576: 4616 bytes.
constexpr int GELU_TAB_ENTRIES = 577;
__device__ __forceinline__ void gelu_tab_build(float *tab, int tid, int nthreads)
{
    for (int i = tid; i < GELU_TAB_ENTRIES; i += nthreads) {
        const float x0 = (i - 288) * (1.0f / 64), x1 = x0 + 1.0f / 64;
        const float p0 = 0.5f * erfcf(-x0 * 0.70710678118654752440f), p1 = i < GELU_TAB_ENTRIES - 1 ? 0.5f * erfcf(-x1 * 0.70710678118654752440f) : p0;
        tab[2 * i] = p0;
        tab[2 * i + 1] = p1 - p0;
    }
}
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f32x4 gelu_tab4(f32x4 x, const float *tab)
{
    f32x4 fr;
    f32x2 e[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float t = fmaf(__builtin_amdgcn_fmed3f(x[i], -4.5f, 4.5f), 64.0f, 288.0f), fl = floorf(t);
        fr[i] = t - fl;
        e[i] = *(const f32x2 *)(tab + 2 * (int)fl);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) fr[i] = x[i] * fmaf(fr[i], e[i][1], e[i][0]);
    return fr;
}

// ---- launch with optional per-stage timing (profile.hip) ----
bool poly_prof_next(int stage, hipEvent_t *a, hipEvent_t *b);

#define POLY_LAUNCH(stage, kernel, grid, block, st, ...)                                         \
    do {                                                                                         \
        hipEvent_t ea_, eb_;                                                                     \
        if (poly_prof_next(stage, &ea_, &eb_))                                                   \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ea_, eb_, 0, __VA_ARGS__);         \
        else                                                                                     \
            hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);                         \
    } while (0)

#define POLY_LAUNCH_SHMEM(stage, kernel, grid, block, shmem, st, ...)                            \
    do {                                                                                         \
        hipEvent_t ea_, eb_;                                                                     \
        if (poly_prof_next(stage, &ea_, &eb_))                                                   \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, st, ea_, eb_, 0, __VA_ARGS__);     \
        else                                                                                     \
            hipLaunchKernelGGL(kernel, grid, block, shmem, st, __VA_ARGS__);                     \
    } while (0)

// ---- stage launchers (defined in the .hip files, used by the entry points in api.hip) ----

enum { EPI_STORE = 0, EPI_GELU = 1, EPI_RESID = 2 };

// C = A Wt^T with per-block structure.  Rows come in blocks of T; input block xb feeds the output
// blocks [out_off[xb], out_off[xb+1]) (or block xb itself when out_off is null).  Each output block ob
// may add its own low-rank term S[ob] Bt[adapter_of_out[ob]]^T before the epilogue.
struct GemmArgs {
    const void *A;    // elt [n_in*T][K]
    const void *Wt;   // elt [N][K]
    const float *bias;  // [N] or null
    int T, K, N;
    int n_in;             // upper bound of the number of input blocks (grid size)
    const int *n_in_dev;  // true count on the device, or null (= n_in)
    const int *out_off;   // [n_in+1] or null
    const void *S;        // elt [n_out*T][RP], zero padded to RP columns, or null
    int RP;
    const void *Bt;       // elt [n_adapters][N][r]
    int r;
    const int *adapter_of_out;  // [n_out], < 0 = no adapter
    const int *set_off;   // null: output block ob has the one low-rank term (S[ob], adapter_of_out[ob]).  Else [n_out+1]: output block
                          // ob sums the terms (S[sb], adapter_of_out[sb]) for sb in [set_off[ob], set_off[ob+1]) -- several adapters
                          // on one hidden state; S and adapter_of_out are then indexed by sb
    int mode;             // EPI_*
    void *out;            // EPI_STORE / EPI_GELU: elt [n_out*Tout][N]; EPI_RESID: float, same shape
    int Tout, t_off;      // output row of (ob, t) is ob*Tout + t_off + t
    const float *res;     // EPI_RESID: float [..*Tout][N] added (row res_block*Tout + t_off + t), or null
    const int *res_block_of_out;  // null = ob
    const float *pos;     // EPI_RESID: float [Tout][N] added (row t_off + t), or null
    // set by launch_gemm only.  Tb > 0: the nb input blocks of Tb rows are tiled as ONE run of nb * Tb rows (T = nb * Tb,
    // n_in = 1; n_in_dev still counts blocks and Tout = Tb still places the output blocks), so that row tiles ignore block
    // boundaries; row t of the run belongs to input block t / Tb
    int Tb, nb;
};

int launch_gemm(const GemmArgs &g, int dtype, hipStream_t st);

// Row-tile linear for K <= 192 (rowlin.hip): y = [LN](x) Wt^T + b + scale ([LN](x) At_k^T) Bt_k^T with the
// LayerNorm and the low-rank shrink computed inside the kernel.
struct RowLinArgs {
    const float *x_ln;            // LayerNorm mode: fp32 rows [n_in*T][K] (null = plain mode)
    const float *ln_g, *ln_b;     // [K]
    float eps;
    const bf16_t *a_in;           // plain mode: bf16 rows [n_in*T][K]
    const int *in_block_of_out;   // null = identity
    int T, K, N;
    int n_out;                    // upper bound of the number of output blocks (grid size)
    const int *n_out_dev;         // true count on the device, or null
    const bf16_t *Wt;             // [N][K]
    const float *bias;            // [N] or null
    const bf16_t *At, *Bt;        // [n_adapters][r][K], [n_adapters][N][r]; null = no adapters
    int r;
    float scale;
    const int *adapter_of_out;
    int mode;                     // EPI_STORE / EPI_GELU: bf16 out [n_out*T][N]; EPI_RESID: fp32 out = res + y
    void *out;
    const float *res;             // EPI_RESID: fp32 [..*T][N]
    const int *res_block_of_out;  // null = ob
};
bool rowlin_supported(int K, int N, int r, bool lora, bool f32out);

// x <- x + GELU(LayerNorm(x) W1 + b1) W2 + b2 on blocks of T rows (mlp.hip); bf16 weights stored contraction-fastest
struct MlpArgs {
    float *x;                    // [n_out][T][D] fp32, updated in place
    const float *ln_g, *ln_b;    // [D]
    float eps;
    int T, D, Dm, n_out;
    const int *n_out_dev;        // optional device-side block count (the smaller of the two is used)
    const bf16_t *W1t;           // [Dm][D]
    const float *b1;             // [Dm]
    const bf16_t *W2t;           // [D][Dm]
    const float *b2;             // [D]
};
bool mlp_supported(int D, int Dm);
int launch_mlp(const MlpArgs &a, hipStream_t st);

// The row-wise part of a layer in one launch (rowlayer.hip):
//   A (if o != null)        x' = res + o Wp + bp + scale (o Ap_k) Bp_k,  else x' = x_out
//   B                       x_out = x' + GELU(LayerNorm2(x') W1 + b1) W2 + b2
//   C (if qkv_out != null)  qkv_out = LayerNorm1'(x_out) Wq + bq + scale (.. Aq_k) Bq_k     (the next layer's qkv)
// bf16 weights stored contraction-fastest, adapter stacks indexed by adapter_of_out[block]
struct RowLayerArgs {
    int T, D, Dm, n_out;
    const int *n_out_dev;            // optional device-side block count (the smaller of the two is used)
    const int *adapter_of_out;       // [n_out] or null
    int r;
    float scale, eps;
    // A
    const bf16_t *o;                 // [n_out][T][D]
    const bf16_t *Wpt;               // [D][D]
    const float *bp;                 // [D]
    const bf16_t *Apt, *Bpt;         // [n_adapters][r][D], [n_adapters][D][r]; null = no adapters on proj
    const float *res;                // [..][T][D] fp32 residual stream going in
    const int *res_block_of_out;     // null = same block
    // B
    const float *ln2_g, *ln2_b;      // [D]
    const bf16_t *W1t;               // [Dm][D]
    const float *b1;                 // [Dm]
    const bf16_t *W2t;               // [D][Dm]
    const float *b2;                 // [D]
    float *x_out;                    // [n_out][T][D] fp32 residual stream going out (may be the same buffer as res)
    // C
    const float *lnq_g, *lnq_b;      // [D]
    const bf16_t *Wqt;               // [3 D][D]
    const float *bq;                 // [3 D]
    const bf16_t *Aqt, *Bqt;         // [n_adapters][r][D], [n_adapters][3 D][r]; null = no adapters on qkv
    bf16_t *qkv_out;                 // [n_out][T][3 D]
};
bool rowlayer_supported(int D, int Dm, int r);
int launch_rowlayer(const RowLayerArgs &a, hipStream_t st);
int launch_rowlin(const RowLinArgs &a, hipStream_t st);

// y = LayerNorm(x) row-wise; x float [n*T][D] -> elt [n*T][D]
int launch_layernorm(const float *x, void *y, const float *gain, const float *shift, int D, float eps, int T,
                     int n_blocks, const int *n_blocks_dev, int dtype, hipStream_t st);

// S[ob] = scale * X[in_block_of_out[ob]] At[adapter_of_out[ob]]^T, zero padded to RP columns.  pair_off (nullable): CSR offsets
// [n_in + 1] of the output blocks of every input block, when the output blocks of one input block are consecutive (fan-out):
// lets one workgroup serve two of them from one read of the input rows
int launch_shrink(const void *X, int T, int K, const void *At, int r, int RP, float scale, int n_out,
                  const int *n_out_dev, const int *in_block_of_out, const int *adapter_of_out, const int *pair_off, void *S,
                  int dtype, hipStream_t st);

// softmax attention of every (block, head); qkv elt [n*T][3D] -> out elt [n*T][D]
int launch_attention(const void *qkv, void *out, int T, int D, int heads, int n_blocks, const int *n_blocks_dev,
                     int dtype, hipStream_t st);

// ---- bookkeeping and row-wise stages (rowops.hip) ----
int launch_prep(const int32_t *row_offsets, const int32_t *adapter_ids, int F, int R_cap, int n_adapters, PolyMeta *meta,
                int32_t *frame_of_row, int32_t *adapter_of_row, int32_t *dev_status, hipStream_t st);
// patches <- frames (im2col), x[f][0][:] <- cls + pos[0], merged[0 .. n_merged) <- 0; and, when row_offsets is given, the work of
// launch_prep as one more block of the same launch
int launch_im2col(const void *frames, void *patches, int F, int H, int W, int p, int dtype, float *x, const float *cls, const float *pos,
                  int T_tok, int D, float *merged, size_t n_merged, const int32_t *row_offsets, const int32_t *adapter_ids, int R_cap,
                  int n_adapters, PolyMeta *meta, int32_t *frame_of_row, int32_t *adapter_of_row, int32_t *dev_status, hipStream_t st);
// base head of the lagged loop: scores of frame f -> lag[f + 1][K] and out[f][K] (nullable); lag[0] = carry (or zeros)
int launch_base_head(const float *x, int T, int D, const float *gain, const float *shift, float eps, const void *Wb, const float *bb,
                     int K, int F, float *lag, float *out, const float *carry, int dtype, hipStream_t st);
int launch_head(const float *x, const int *src_block_of_row, int T, int D, const float *gain, const float *shift, float eps,
                const void *head_w, const float *head_b, int C, const int *adapter_of_row, const int *frame_of_row,
                const int32_t *class_map, int K, const PolyMeta *meta, int R_cap, float *logits, float *scores, float *merged, int dtype,
                hipStream_t st);
