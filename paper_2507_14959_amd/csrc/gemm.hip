// Block-structured linear  y = x W + b  (+ s (x A_k) B_k)  with fused epilogues (Sec. 3.1).
//
// bf16: 128 x BN x 32 tiles, 4 waves in a 2 x 2 grid, v_mfma_f32_32x32x16_bf16, fp32 accumulators.
// The low-rank expand (x A_k) B_k is one more K step of the same MFMA per 16 ranks, fed with the
// shrink output S and the adapter's Bt slab, so W + A_k B_k is never formed and the base product of
// an input block is shared by all the row-blocks that fan out of it.
// fp32: 64 x 64 x 16 tiles on the vector ALUs (reference-precision path).
#include "poly_dev.h"

namespace {

template <typename T> __device__ __forceinline__ void epilogue_store_elt(const GemmArgs &g, int ob, int t, int col, float v)
{
    // caller guarantees t < T and col < N
    if (g.bias) v += g.bias[col];
    const size_t o = ((size_t)ob * g.Tout + g.t_off + t) * g.N + col;
    if (g.mode == EPI_RESID) {
        if (g.res) {
            const int rb = g.res_block_of_out ? g.res_block_of_out[ob] : ob;
            v += g.res[((size_t)rb * g.Tout + g.t_off + t) * g.N + col];
        }
        if (g.pos) v += g.pos[(size_t)(g.t_off + t) * g.N + col];
        ((float *)g.out)[o] = v;
    } else {
        if (g.mode == EPI_GELU) v = gelu_erf(v);
        ((T *)g.out)[o] = from_f32<T>(v);
    }
}

// decode the flat block index: n-tile fastest, then m-tile, then input block
__device__ __forceinline__ bool decode_tile(const GemmArgs &g, int BM, int BN, int &xb, int &t0, int &n0, int &ob0, int &ob1)
{
    const int tiles_n = (g.N + BN - 1) / BN, tiles_m = (g.T + BM - 1) / BM;
    int id = blockIdx.x;
    const int tn = id % tiles_n; id /= tiles_n;
    const int tm = id % tiles_m; xb = id / tiles_m;
    const int n_in = g.n_in_dev ? min(*g.n_in_dev, g.n_in) : g.n_in;
    if (xb >= n_in) return false;
    ob0 = xb; ob1 = xb + 1;
    if (g.out_off) { ob0 = g.out_off[xb]; ob1 = g.out_off[xb + 1]; }
    t0 = tm * BM; n0 = tn * BN;
    return ob0 < ob1;
}

// ------------------------------------------------------------------ bf16 MFMA

template <int BN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const GemmArgs g)
{
    constexpr int BM = 128, BK = 32, LS = BK + 8;  // LDS row stride in elements (80 B, 16-byte aligned)
    constexpr int NJ = BN / 64;                     // 32-wide column subtiles per wave
    __shared__ __attribute__((aligned(16))) bf16_t As[BM * LS];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * LS];

    int xb, t0, n0, ob0, ob1;
    if (!decode_tile(g, BM, BN, xb, t0, n0, ob0, ob1)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, lm = lane & 31, lh = lane >> 5;
    const bf16_t *A = (const bf16_t *)g.A + (size_t)xb * g.T * g.K;
    const bf16_t *Wt = (const bf16_t *)g.Wt;

    // global -> register staging: 16-byte vectors, 4 per tile row
    constexpr int AV = BM * 4 / 256, BV = BN * 4 / 256;
    bf16x8 ra[AV], rb[BV];
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int v = tid + i * 256, row = v >> 2, kv = (v & 3) * 8;
            const bool ok = (t0 + row < g.T) && (k0 + kv + 8 <= g.K);
            ra[i] = ok ? *(const bf16x8 *)(A + (size_t)(t0 + row) * g.K + k0 + kv) : zero8;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int v = tid + i * 256, row = v >> 2, kv = (v & 3) * 8;
            const bool ok = (n0 + row < g.N) && (k0 + kv + 8 <= g.K);
            rb[i] = ok ? *(const bf16x8 *)(Wt + (size_t)(n0 + row) * g.K + k0 + kv) : zero8;
        }
    };
    auto stage_tiles = [&]() {
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int v = tid + i * 256, row = v >> 2, kv = (v & 3) * 8;
            *(bf16x8 *)(As + row * LS + kv) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int v = tid + i * 256, row = v >> 2, kv = (v & 3) * 8;
            *(bf16x8 *)(Bs + row * LS + kv) = rb[i];
        }
    };

    f32x16 acc[2][NJ];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bool live[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) live[i] = t0 + wm * 64 + i * 32 < g.T;

    load_tiles(0);
    for (int k0 = 0; k0 < g.K; k0 += BK) {
        stage_tiles();
        __syncthreads();
        if (k0 + BK < g.K) load_tiles(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8 fa[2], fb[NJ];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = *(const bf16x8 *)(As + (wm * 64 + i * 32 + lm) * LS + kk + lh * 8);
#pragma unroll
            for (int j = 0; j < NJ; ++j) fb[j] = *(const bf16x8 *)(Bs + (wn * (BN / 2) + j * 32 + lm) * LS + kk + lh * 8);
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (live[i]) {
#pragma unroll
                    for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    for (int ob = ob0; ob < ob1; ++ob) {
        f32x16 c[2][NJ];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) c[i][j] = acc[i][j];

        const int k_ad = (g.S && g.adapter_of_out) ? g.adapter_of_out[ob] : -1;
        if (k_ad >= 0) {
            // expand: one more K step per 16 ranks; A operand = S rows, B operand = Bt_k rows
            const bf16_t *S = (const bf16_t *)g.S + (size_t)ob * g.T * g.RP;
            const bf16_t *Bt = (const bf16_t *)g.Bt + (size_t)k_ad * g.N * g.r;
            for (int s0 = 0; s0 < g.RP; s0 += 16) {
                const int j0 = s0 + lh * 8;
                bf16x8 fa[2], fb[NJ];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int t = t0 + wm * 64 + i * 32 + lm;
                    fa[i] = t < g.T ? *(const bf16x8 *)(S + (size_t)t * g.RP + j0) : zero8;
                }
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int col = n0 + wn * (BN / 2) + j * 32 + lm;
                    bf16x8 f = zero8;
                    if (col < g.N) {
                        const bf16_t *p = Bt + (size_t)col * g.r + j0;
                        if ((g.r & 7) == 0) {
                            if (j0 + 8 <= g.r) f = *(const bf16x8 *)p;
                        } else {
#pragma unroll
                            for (int q = 0; q < 8; ++q)
                                if (j0 + q < g.r) f[q] = p[q];
                        }
                    }
                    fb[j] = f;
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    if (live[i]) {
#pragma unroll
                        for (int j = 0; j < NJ; ++j) c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], c[i][j], 0, 0, 0);
                    }
            }
        }

#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (!live[i]) continue;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int col = n0 + wn * (BN / 2) + j * 32 + lm;
                if (col >= g.N) continue;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int t = t0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
                    if (t < g.T) epilogue_store_elt<bf16_t>(g, ob, t, col, c[i][j][e]);
                }
            }
        }
    }
}

// ------------------------------------------------------------------ fp32 vector ALU

__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs g)
{
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];

    int xb, t0, n0, ob0, ob1;
    if (!decode_tile(g, BM, BN, xb, t0, n0, ob0, ob1)) return;

    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const float *A = (const float *)g.A + (size_t)xb * g.T * g.K;
    const float *Wt = (const float *)g.Wt;
    const int lrow = tid >> 2, lk = (tid & 3) * 4;  // one 4-wide k strip of one tile row per thread

    float acc[4][4] = {};
    for (int k0 = 0; k0 < g.K; k0 += BK) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = k0 + lk + q;
            As[lk + q][lrow] = (t0 + lrow < g.T && k < g.K) ? A[(size_t)(t0 + lrow) * g.K + k] : 0.f;
            Bs[lk + q][lrow] = (n0 + lrow < g.N && k < g.K) ? Wt[(size_t)(n0 + lrow) * g.K + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    for (int ob = ob0; ob < ob1; ++ob) {
        const int k_ad = (g.S && g.adapter_of_out) ? g.adapter_of_out[ob] : -1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = t0 + ty * 4 + i;
            if (t >= g.T) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = n0 + tx * 4 + j;
                if (col >= g.N) continue;
                float v = acc[i][j];
                if (k_ad >= 0) {
                    const float *S = (const float *)g.S + ((size_t)ob * g.T + t) * g.RP;
                    const float *Bt = (const float *)g.Bt + ((size_t)k_ad * g.N + col) * g.r;
                    float d = 0.f;
                    for (int q = 0; q < g.r; ++q) d = fmaf(S[q], Bt[q], d);
                    v += d;
                }
                epilogue_store_elt<float>(g, ob, t, col, v);
            }
        }
    }
}

}  // namespace

int launch_gemm(const GemmArgs &g, int dtype, hipStream_t st)
{
    if (g.n_in <= 0 || g.T <= 0) return POLY_OK;
    if (dtype == POLY_BF16) {
        if (g.K % 8 != 0 || (g.S && g.RP % 16 != 0)) return POLY_EINVAL;
        const int tiles_m = (g.T + 127) / 128;
        // wide outputs take 128-column tiles; narrow ones 64 so that small batches still fill the CUs
        const bool wide = g.N >= 1024 || (long)g.n_in * tiles_m * ((g.N + 127) / 128) >= 1024;
        if (wide) {
            const long blocks = (long)g.n_in * tiles_m * ((g.N + 127) / 128);
            if (blocks > 0x7fffffffL) return POLY_EINVAL;
            POLY_LAUNCH(POLY_STAGE_GEMM, gemm_bf16_kernel<128>, dim3((unsigned)blocks), dim3(256), st, g);
        } else {
            const long blocks = (long)g.n_in * tiles_m * ((g.N + 63) / 64);
            POLY_LAUNCH(POLY_STAGE_GEMM, gemm_bf16_kernel<64>, dim3((unsigned)blocks), dim3(256), st, g);
        }
    } else {
        const long blocks = (long)g.n_in * ((g.T + 63) / 64) * ((g.N + 63) / 64);
        if (blocks > 0x7fffffffL) return POLY_EINVAL;
        POLY_LAUNCH(POLY_STAGE_GEMM, gemm_f32_kernel, dim3((unsigned)blocks), dim3(256), st, g);
    }
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}
