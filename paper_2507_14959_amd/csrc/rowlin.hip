// Row-tile linear for narrow models (K = D <= 192): one workgroup owns 64 token rows and ALL output columns.
//
//     y = [LayerNorm](x) W + b + s ([LayerNorm](x) A_k) B_k      (Sec. 3.1), epilogue: store | GELU | + residual
//
// Why a second linear kernel: at D = 192 a 128 x 64 GEMM tile moves more bytes through L2 than it computes on,
// and LayerNorm and the LoRA shrink were separate launches whose results went through HBM.  Here the
// activation rows of the tile are produced once (LayerNorm in registers, or a straight copy), kept in LDS and
// then in MFMA operand registers for the whole kernel; only W streams past, 64 output columns at a time,
// through a five-stage LDS ring filled with global_load_lds_dwordx4.  The shrink x A_k is 12 more MFMAs on the resident
// rows; its accumulator layout is already a valid operand layout for the expand once the ranks of Bt_k are
// read in the matching order, so S never leaves registers.
#include "poly_dev.h"
#include "rowtile.h"

#include <stdlib.h>

namespace {

constexpr int RL_ROWS = 64;    // token rows per workgroup
constexpr int RL_BNC = 64;     // output columns per W chunk
constexpr int RL_NS = 5;       // LDS stages of the W stream
constexpr int RL_MAXCH = 12;   // chunks per workgroup: N <= 768
constexpr int RL_THREADS = 512;

// One workgroup = 8 waves = two groups of 2 x 2 waves.  Both groups hold the same 64 activation rows as MFMA
// operand registers; group g takes the W chunks c with c % 2 == g, so two chunks are multiplied at a time and
// every SIMD has two waves whose MFMA and vector work (LayerNorm, GELU, conversions) overlap.  The
// accumulators of all of a wave's chunks (up to 6 x 16 registers) stay resident, so the chunk loop is nothing
// but the W stream: wait, barrier, refill, 12 MFMAs.  Stores happen once, at the end.
template <int KT, int MODE>   // K = 64 * KT; MODE = EPI_STORE / EPI_GELU / EPI_RESID, fixed at compile time to keep the epilogue branch-free
__global__ __launch_bounds__(RL_THREADS) void rowlin_kernel(const RowLinArgs a)
{
    constexpr int K = 64 * KT;
    constexpr int A_EL = KT * RL_ROWS * 64;          // resident activation rows, one [64][64] tile per 64 k
    constexpr int W_EL = KT * RL_BNC * 64;           // one W chunk: KT tiles of [64][64]
    constexpr int NLD = KT;                          // W loads per wave and chunk
    constexpr int MAXIT = RL_MAXCH / 2;              // chunk pairs
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Ws = lds + A_EL;
    float *bias_s = (float *)(lds + A_EL + RL_NS * W_EL);   // [N] bias, copied once: the epilogue must not wait on global loads

    const int tiles = (a.T + RL_ROWS - 1) / RL_ROWS;
    const int ob = blockIdx.x / tiles, t0 = (blockIdx.x % tiles) * RL_ROWS;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, wr = (wave >> 1) & 1, wc = wave & 1, lm = lane & 31, lh = lane >> 5;
    const int nchunks = (a.N + RL_BNC - 1) / RL_BNC;
    const int niter = (nchunks + 1) >> 1;

    // W chunk -> LDS stage: KT tiles x 8 groups of 8 rows; wave w takes row group w of every tile
    const int lr = lane >> 3;
    auto issue_w = [&](int chunk) {
        bf16_t *st = Ws + (chunk % RL_NS) * W_EL;
        const int row = wave * 8 + lr;
        const int col = min(chunk * RL_BNC + row, a.N - 1);                   // columns past N are never stored
        const bf16_t *src = a.Wt + (size_t)col * K + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
            glds16(src + kt * 64, __builtin_amdgcn_readfirstlane(lds_addr_of(st + kt * (RL_BNC * 64) + wave * 512)));
    };
    // the W stream needs nothing but the kernel arguments: start it before anything else (all stages are free)
    const int npro = min(RL_NS, nchunks);
    for (int c = 0; c < npro; ++c) issue_w(c);
    // the rest of W: into L2 now, so that the ring refills below are L2 hits
    l2_warm(a.Wt, (long)a.N * K * 2, lds_addr_of(bias_s + RL_MAXCH * RL_BNC), tid, RL_THREADS);

    const int n_out = a.n_out_dev ? min(*a.n_out_dev, a.n_out) : a.n_out;
    if (ob >= n_out) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    const int xb = a.in_block_of_out ? a.in_block_of_out[ob] : ob;
    const int k_ad = (a.At && a.adapter_of_out) ? a.adapter_of_out[ob] : -1;

    // ---- activation rows of this tile -> LDS (rows past T are clamped: their results are never stored)
    {
        constexpr int PER = K / 8;                   // 8 threads per row, K/8 contiguous elements each
        const int row = tid >> 3, part = tid & 7;
        if (a.x_ln == nullptr) {
            const bf16_t *src = a.a_in + ((size_t)xb * a.T + min(t0 + row, a.T - 1)) * K + part * PER;
#pragma unroll
            for (int c = 0; c < PER / 8; ++c) {
                const int k = part * PER + 8 * c;
                *(bf16x8 *)(As + (k >> 6) * (RL_ROWS * 64) + tile_off(row, (k & 63) >> 3)) = *(const bf16x8 *)(src + 8 * c);
            }
        } else {
            ln_rows_to_lds<KT, 8>(a.x_ln + (size_t)xb * a.T * K, a.T, t0, a.ln_g, a.ln_b, a.eps, As, tid);
        }
    }
    for (int i = tid; i < a.N; i += RL_THREADS) bias_s[i] = a.bias ? a.bias[i] : 0.f;
    // the activation rows were written with ordinary LDS stores: make them visible, but do not drain the W
    // stream (a fenced barrier would): wait for this wave's LDS stores, then a bare barrier
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- operands of the low-rank branch.  They are requested only now, after the prologue has consumed its own
    // loads: requested earlier, the compiler's wait bookkeeping carries them into the W stream as "maybe pending"
    // and drains the stream before every chunk.  Shrink: At rows as the A operand (rank = lm).
    // Expand: lane (column, lh) supplies ranks 4*lh + {0..3} and 8 + 4*lh + {0..3} (see the shrink below).
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    bf16x8 ft[KT * 4], fbt[MAXIT];
    if (k_ad >= 0) {
        const bf16_t *At = a.At + ((size_t)k_ad * a.r + min(lm, a.r - 1)) * K + lh * 8;
#pragma unroll
        for (int kk = 0; kk < KT * 4; ++kk) ft[kk] = lm < a.r ? *(const bf16x8 *)(At + kk * 16) : zero8;
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) {
            bf16x8 f = zero8;
            const int ch = 2 * it + grp, col = ch * RL_BNC + wc * 32 + lm;
            if (ch < nchunks && col < a.N) {
                const bf16_t *bt = a.Bt + ((size_t)k_ad * a.N + col) * a.r;
                if ((a.r & 3) == 0) {
                    if (4 * lh + 4 <= a.r) { const bf16x4 lo = *(const bf16x4 *)(bt + 4 * lh); f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3]; }
                    if (8 + 4 * lh + 4 <= a.r) { const bf16x4 hi = *(const bf16x4 *)(bt + 8 + 4 * lh); f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3]; }
                } else {
#pragma unroll
                    for (int sl = 0; sl < 8; ++sl) {
                        const int rank = (sl < 4 ? 4 * lh + sl : 8 + 4 * lh + (sl - 4));
                        if (rank < a.r) f[sl] = bt[rank];
                    }
                }
            }
            fbt[it] = f;
        }
    }

    // ---- activation fragments -> registers (B operand of the transposed product): rows wr*32 + lm
    bf16x8 fa[KT * 4];
#pragma unroll
    for (int kk = 0; kk < KT * 4; ++kk)
        fa[kk] = *(const bf16x8 *)(As + (kk >> 2) * (RL_ROWS * 64) + tile_off(wr * 32 + lm, 2 * (kk & 3) + lh));

    // ---- shrink: c[n][m] = sum_k At[n][k] x[m][k]; lane (lm, lh) ends up with ranks 4*lh + {0..3} (c[0..3]) and
    // 8 + 4*lh + {0..3} (c[4..7]) of row lm -- exactly the 8 contraction slots it must supply to the expand
    bf16x8 fs = zero8;
    if (k_ad >= 0) {
        f32x16 c;
#pragma unroll
        for (int e = 0; e < 16; ++e) c[e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KT * 4; ++kk) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ft[kk], fa[kk], c, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) fs[j] = (bf16_t)(a.scale * c[j]);
        // everything that was loaded into registers is forced to have arrived here, in one wait that the compiler
        // sees (the empty asm "uses" the registers): inside the stream below only the LDS-bound loads are in flight
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) asm volatile("" ::"v"(fbt[it]));
    }

    // ---- the W stream: iteration it multiplies chunks 2*it (group 0) and 2*it + 1 (group 1);
    // acc[it] = rows wr*32.. x columns (2*it + grp)*64 + wc*32..
    f32x16 acc[MAXIT];
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
        if (it < niter) {     // uniform; written as a guard (not a break) so that the loop unrolls and acc stays in registers
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[it][e] = 0.f;
            // chunks 2*it and 2*it + 1 must have landed; later chunks may stay in flight (loads return in order).
            // Issued so far: the prologue's min(NS, nchunks) chunks, then two more per earlier iteration.
            const int last_issued = min(nchunks - 1, it == 0 ? RL_NS - 1 : 2 * it + RL_NS - 3);
            const int ahead = max(0, last_issued - (2 * it + 1));
            if (ahead >= 3) rl_wait_barrier<3 * NLD>();
            else if (ahead == 2) rl_wait_barrier<2 * NLD>();
            else if (ahead == 1) rl_wait_barrier<NLD>();
            else rl_wait_barrier<0>();
            // every wave is past chunks 2*it - 2 and 2*it - 1: their stages take chunks 2*it + NS - 2 and 2*it + NS - 1
            if (it >= 1) {
                if (2 * it + RL_NS - 2 < nchunks) issue_w(2 * it + RL_NS - 2);
                if (2 * it + RL_NS - 1 < nchunks) issue_w(2 * it + RL_NS - 1);
            }
            const int ch = 2 * it + grp;
            if (ch < nchunks) {
                const bf16_t *st = Ws + (ch % RL_NS) * W_EL;
#pragma unroll
                for (int kk = 0; kk < KT * 4; ++kk) {
                    const bf16x8 fw = *(const bf16x8 *)(st + (kk >> 2) * (RL_BNC * 64) + tile_off(wc * 32 + lm, 2 * (kk & 3) + lh));
                    acc[it] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fa[kk], acc[it], 0, 0, 0);
                }
                if (k_ad >= 0) acc[it] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fbt[it], fs, acc[it], 0, 0, 0);
            }
        }
    }

    // ---- epilogue.  acc[it][e]: row wr*32 + lm, column (2*it + grp)*64 + wc*32 + 8*(e/4) + 4*lh + e%4.
    // A lane owns one row, so storing from registers would touch 32 cache lines per instruction with 8 or 16
    // bytes each.  Instead the finished tile (bias, GELU applied, output type) is laid out row-major in LDS --
    // the activation rows and the W ring are dead by now -- and copied out with consecutive threads on
    // consecutive 16-byte pieces of a row, which is also where the residual rows are read.
    constexpr bool f32out = MODE == EPI_RESID;
    const int row_bytes = a.N * (f32out ? 4 : 2);
    const int stride = ((row_bytes + 255) & ~255) + 16;     // rows start 4 banks apart
    char *tile = (char *)lds;
    asm volatile("s_barrier" ::: "memory");                  // every wave is done reading the W ring
    {
        char *trow = tile + (wr * 32 + lm) * stride + (wc * 32 + 4 * lh) * (f32out ? 4 : 2);
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) {
            const int ch = 2 * it + grp;
            if (ch < nchunks) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = ch * RL_BNC + wc * 32 + 8 * g + 4 * lh;
                    f32x4 v = {acc[it][4 * g], acc[it][4 * g + 1], acc[it][4 * g + 2], acc[it][4 * g + 3]};
                    if (f32out) {
                        // raw sums; bias and residual are added by the copy-out below, where accesses are coalesced
                        if (col < a.N) *(f32x4 *)(trow + (ch * RL_BNC + 8 * g) * 4) = v;
                    } else {
                        v += *(const f32x4 *)(bias_s + min(col, a.N - 4));
                        if (MODE == EPI_GELU) {
#pragma unroll
                            for (int z = 0; z < 4; ++z) v[z] = gelu_poly(v[z]);
                        }
                        const bf16x4 w = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                        if (col < a.N) *(bf16x4 *)(trow + (ch * RL_BNC + 8 * g) * 2) = w;
                    }
                }
            }
        }
    }
    __syncthreads();
    const int pieces = row_bytes >> 4;                       // 16-byte pieces per row
    const int rows = min(RL_ROWS, a.T - t0);
    char *out = (char *)a.out + ((size_t)ob * a.T + t0) * row_bytes;
    if (f32out) {
        const int rblk = a.res ? (a.res_block_of_out ? a.res_block_of_out[ob] : ob) : 0;
        const char *res = a.res ? (const char *)a.res + ((size_t)rblk * a.T + t0) * row_bytes : nullptr;
        for (int idx = tid; idx < rows * pieces; idx += RL_THREADS) {
            const int row = idx / pieces, p = idx - row * pieces;
            f32x4 v = *(const f32x4 *)(tile + row * stride + p * 16) + *(const f32x4 *)(bias_s + 4 * p);
            if (res) v += *(const f32x4 *)(res + (size_t)row * row_bytes + p * 16);
            *(f32x4 *)(out + (size_t)row * row_bytes + p * 16) = v;
        }
    } else {
        for (int idx = tid; idx < rows * pieces; idx += RL_THREADS) {
            const int row = idx / pieces, p = idx - row * pieces;
            *(f32x4 *)(out + (size_t)row * row_bytes + p * 16) = *(const f32x4 *)(tile + row * stride + p * 16);
        }
    }
}

template <int KT, int MODE> int launch_kt_mode(const RowLinArgs &a, hipStream_t st)
{
    constexpr int LDS = (KT * RL_ROWS * 64 + RL_NS * KT * RL_BNC * 64) * 2 + RL_MAXCH * RL_BNC * 4 + 256;   // + dump words of the L2 warm-up
    auto kern = rowlin_kernel<KT, MODE>;
    if (LDS > 64 * 1024) {
        static bool attr_set = false;   // raising the dynamic LDS limit is a per-kernel, process-wide setting
        if (!attr_set) {
            if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess) return POLY_EHIP;
            attr_set = true;
        }
    }
    const int tiles = (a.T + RL_ROWS - 1) / RL_ROWS;
    POLY_LAUNCH_SHMEM(POLY_STAGE_GEMM, kern, dim3((unsigned)(a.n_out * tiles)), dim3(RL_THREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}

template <int KT> int launch_kt(const RowLinArgs &a, hipStream_t st)
{
    switch (a.mode) {
    case EPI_STORE: return launch_kt_mode<KT, EPI_STORE>(a, st);
    case EPI_GELU: return launch_kt_mode<KT, EPI_GELU>(a, st);
    case EPI_RESID: return launch_kt_mode<KT, EPI_RESID>(a, st);
    default: return POLY_EINVAL;
    }
}

}  // namespace

bool rowlin_supported(int K, int N, int r, bool lora, bool f32out)
{
    if (!((K == 64 || K == 128 || K == 192) && N >= 8 && N % 8 == 0 && N <= RL_MAXCH * RL_BNC && (!lora || (r >= 1 && r <= 16)))) return false;
    // the finished tile is staged over the activation rows and the W ring: it must fit there
    const long stage = (long)RL_ROWS * ((((long)N * (f32out ? 4 : 2) + 255) & ~255L) + 16);
    return stage <= (long)(1 + RL_NS) * (K / 64) * RL_ROWS * 64 * 2;
}

int launch_rowlin(const RowLinArgs &a, hipStream_t st)
{
    if (a.n_out <= 0 || a.T <= 0) return POLY_OK;
    if (!rowlin_supported(a.K, a.N, a.r, a.At != nullptr, a.mode == EPI_RESID)) return POLY_EINVAL;
    if ((long)a.N * a.K > 0x7fffffffL) return POLY_EINVAL;
    switch (a.K / 64) {
    case 1: return launch_kt<1>(a, st);
    case 2: return launch_kt<2>(a, st);
    default: return launch_kt<3>(a, st);
    }
}
