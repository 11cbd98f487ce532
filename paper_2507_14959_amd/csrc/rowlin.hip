// Row-tile linear for narrow models (K = D <= 192): one workgroup owns 64 token rows and ALL output columns.
//
//     y = [LayerNorm](x) W + b + s ([LayerNorm](x) A_k) B_k      (Sec. 3.1), epilogue: store | GELU | + residual
//
// Why a second linear kernel: at D = 192 a 128 x 64 GEMM tile moves more bytes through L2 than it computes on,
// and LayerNorm and the LoRA shrink were separate launches whose results went through HBM.  Here the
// activation rows of the tile are produced once (LayerNorm in registers, or a straight copy), kept in LDS and
// then in MFMA operand registers for the whole kernel; only W streams past, 64 output columns at a time,
// through a five-stage LDS ring filled with global_load_lds_dwordx4.  The shrink x A_k is 12 more MFMAs on the
// resident rows; its accumulator layout is already a valid operand layout for the expand once the ranks of
// Bt_k are read in the matching order, so S never leaves registers.
//
// Eight waves with two jobs (every workgroup of a launch streams the same W out of L2 at the same time, L2 hands
// each of them about 30 bytes per clock, and a wave that issues a load into that saturated path is held at the
// issue stage until the path takes it -- so the waves that compute issue no loads while they compute):
//   waves 0-3 (2 x 2 over a 64 x 64 chunk): activation rows, shrink, 12 MFMAs per chunk with the accumulators of
//             all chunks resident (9 x 16 registers), expand, staging of the finished tile;
//   waves 4-7: W into the ring, Bt_k of the block's adapter into LDS, the residual rows into registers
//             (requested at the very start, used by the copy-out, which these waves then do alone).
#include "poly_dev.h"
#include "rowtile.h"

#include <stdlib.h>

#include <type_traits>

namespace {

constexpr int RL_ROWS = 64;    // token rows per workgroup
constexpr int RL_BNC = 64;     // output columns per W chunk
constexpr int RL_NS = 5;       // LDS stages of the W stream
constexpr int RL_MAXCH = 9;    // chunks per workgroup: N <= 576
constexpr int RL_MAXRES = 12;  // 16-byte pieces of residual per loader thread: fp32 output of N <= 192 columns
constexpr int RL_THREADS = 512;

template <int KT, int MODE>   // K = 64 * KT; MODE = EPI_STORE / EPI_GELU / EPI_RESID, fixed at compile time to keep the epilogue branch-free
__global__ __launch_bounds__(RL_THREADS) void rowlin_kernel(const RowLinArgs a)
{
    constexpr int K = 64 * KT;
    constexpr int A_EL = KT * RL_ROWS * 64;          // resident activation rows, one [64][64] tile per 64 k; later Bt_k
    constexpr int W_EL = KT * RL_BNC * 64;           // one W chunk: KT tiles of [64][64]
    constexpr int NLD = 2 * KT;                      // W loads per loader wave and chunk: 16 rows of each tile, 8 rows per load
    constexpr bool f32out = MODE == EPI_RESID;
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Ws = lds + A_EL;
    float *bias_s = (float *)(lds + A_EL + RL_NS * W_EL);   // [N] bias, copied once: the epilogue must not wait on global loads
    float *dump_s = bias_s + RL_MAXCH * RL_BNC;             // 64 words nobody reads (target of the L2 warm-up loads)
    float *gb_s = dump_s + 64;                              // LayerNorm gain [K] and shift [K]

    const int tiles = (a.T + RL_ROWS - 1) / RL_ROWS;
    const int ob = blockIdx.x / tiles, t0 = (blockIdx.x % tiles) * RL_ROWS;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave >= 4;
    const int wr = (wave >> 1) & 1, wc = wave & 1, lm = lane & 31, lh = lane >> 5;
    const int lw = wave & 3, lr = lane >> 3, lt = tid & 255;
    const int nchunks = (a.N + RL_BNC - 1) / RL_BNC;
    const int row_bytes = a.N * (f32out ? 4 : 2);
    const int stride = ((row_bytes + 255) & ~255) + 16;     // staging tile: rows start 4 banks apart
    const int pieces = row_bytes >> 4;                       // 16-byte pieces per output row
    const int rows = min(RL_ROWS, a.T - t0);

    // W chunk -> LDS stage: KT tiles of 64 rows; loader wave w takes rows 16w .. 16w + 15 of every tile, 8 rows (1 KB) per load
    auto issue_w = [&](int chunk) {
        bf16_t *st = Ws + (chunk % RL_NS) * W_EL;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int row = lw * 16 + half * 8 + lr;
            const int col = min(chunk * RL_BNC + row, a.N - 1);                   // columns past N are never stored
            const bf16_t *src = a.Wt + (size_t)col * K + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
                glds16(src + kt * 64, __builtin_amdgcn_readfirstlane(lds_addr_of(st + kt * (RL_BNC * 64) + (lw * 16 + half * 8) * 64)));
        }
    };
    // The activation rows are requested before anything else when their address does not depend on metadata: they
    // come from HBM (another kernel has just written them), and whatever is requested first is served first.
    // The computing waves take them: 4 threads per row; a thread takes the 16-byte pieces part, part + 4, ... so
    // that the lanes of a row read 64 contiguous bytes per instruction.
    f32x4 xv[K / 16];
    bf16x8 pv[K / 32];
    auto load_rows = [&](int xb) {
        if (a.x_ln) {
            ln_load<KT, 4>(a.x_ln + (size_t)xb * a.T * K, a.T, t0, tid, xv);
        } else {
            const bf16_t *src = a.a_in + ((size_t)xb * a.T + min(t0 + (tid >> 2), a.T - 1)) * K + 8 * (tid & 3);
#pragma unroll
            for (int i = 0; i < K / 32; ++i) pv[i] = *(const bf16x8 *)(src + 32 * i);
        }
    };
    const bool early = a.in_block_of_out == nullptr;
    f32x4 gbv = {0.f, 0.f, 0.f, 0.f};
    float bv[(RL_MAXCH * RL_BNC + 255) / 256];
    if (!loader) {
        if (early) load_rows(ob);
        // gain, shift and bias as well: requested after the W stream has started they would arrive behind it
        if (a.x_ln) gbv = ln_gb_load<KT>(a.ln_g, a.ln_b, tid);
#pragma unroll
        for (int j = 0; j < (RL_MAXCH * RL_BNC + 255) / 256; ++j) bv[j] = a.bias ? a.bias[min(tid + 256 * j, a.N - 1)] : 0.f;   // no per-lane condition: see ln_gb_load
    }

    const int n_out = a.n_out_dev ? min(*a.n_out_dev, a.n_out) : a.n_out;
    if (ob >= n_out) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    const int xb = a.in_block_of_out ? a.in_block_of_out[ob] : ob;
    const int k_ad = (a.At && a.adapter_of_out) ? a.adapter_of_out[ob] : -1;
    // the W stream (workgroups past the block count have left without moving data): only the chunks of step 0 for now --
    // the activation rows are still on their way and would be slowed down by more; the rest of the ring follows at
    // the first barrier, which the computing waves reach once their loads have arrived
    int last = min(2, nchunks) - 1;                  // newest chunk requested
    if (loader) {
        for (int c = 0; c <= last; ++c) issue_w(c);
        // the rest of W: into L2 now, so that the ring refills below are L2 hits
        l2_warm(a.Wt, (long)a.N * K * 2, lds_addr_of(dump_s), lt, 256);
    }

    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    f32x16 acc[RL_MAXCH];                            // acc[c][e]: row wr*32 + lm, column c*64 + wc*32 + 8*(e/4) + 4*lh + e%4
    f32x4 res[RL_MAXRES];                            // loader threads: residual pieces lt, lt + 256, ...
    char *tile = (char *)lds;                        // staging tile of the epilogue (activation rows and ring are dead by then)

    if (loader) {
        // ================================================================ loader waves
        if (f32out && a.res) {
            const int rblk = a.res_block_of_out ? a.res_block_of_out[ob] : ob;
            const char *rsrc = (const char *)a.res + ((size_t)rblk * a.T + t0) * row_bytes;
#pragma unroll
            for (int j = 0; j < RL_MAXRES; ++j) {
                const int idx = lt + 256 * j;
                if (idx < rows * pieces) res[j] = *(const f32x4 *)(rsrc + (size_t)(idx / pieces) * row_bytes + (idx % pieces) * 16);
            }
        }
        if (a.x_ln) {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LayerNorm gain and shift are in LDS
            for (int q = last + 1; q < min(RL_NS, nchunks); ++q) issue_w(q);
            last = min(RL_NS, nchunks) - 1;
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // activation rows are in LDS
        for (int sp = 0; 2 * sp < nchunks; ++sp) {
            // step sp multiplies chunks 2 sp and 2 sp + 1: they must have landed; newer ones may stay in flight (loads
            // complete in issue order)
            const int ahead = last - min(2 * sp + 1, nchunks - 1);
            if (ahead >= 3) rl_wait_barrier<3 * NLD>();
            else if (ahead == 2) rl_wait_barrier<2 * NLD>();
            else if (ahead == 1) rl_wait_barrier<NLD>();
            else rl_wait_barrier<0>();
            if (sp == 0 && k_ad >= 0) {
                // every computing wave holds its activation fragments by now: Bt_k [N][r] takes their place, as it is
                const char *bsrc = (const char *)(a.Bt + (size_t)k_ad * a.N * a.r);
                const int n16 = (a.N * a.r) >> 3;
                for (int i0 = lw * 64; i0 < n16; i0 += 256)
                    if (i0 + lane < n16) glds16(bsrc + (size_t)(i0 + lane) * 16, __builtin_amdgcn_readfirstlane(lds_addr_of(As) + i0 * 16));
            }
            // every wave is past the chunks of step sp - 1: refill the ring behind them
            const int upto = min(2 * sp - 1 + RL_NS, nchunks - 1);
            for (int q = last + 1; q <= upto; ++q) issue_w(q);
            last = max(last, upto);
        }
        rl_wait_barrier<0>();                                             // Bt_k has landed; the ring is dead
        asm volatile("s_barrier" ::: "memory");                           // expand done: Bt_k is dead
    } else {
        // ================================================================ computing waves
        // shrink operand: At_k rows as the A operand (rank = lm); requested first, used after the activation rows
        bf16x8 ft[KT * 4];
        if (k_ad >= 0) {
            const bf16_t *At = a.At + ((size_t)k_ad * a.r + min(lm, a.r - 1)) * K + lh * 8;
#pragma unroll
            for (int kk = 0; kk < KT * 4; ++kk) ft[kk] = lm < a.r ? *(const bf16x8 *)(At + kk * 16) : zero8;
        }
        // activation rows of this tile -> LDS (rows past T repeat row T - 1: their results are never stored)
        if (!early) load_rows(xb);
#pragma unroll
        for (int j = 0; j < (RL_MAXCH * RL_BNC + 255) / 256; ++j)
            if (tid + 256 * j < a.N) bias_s[tid + 256 * j] = bv[j];
        if (a.x_ln == nullptr) {
#pragma unroll
            for (int i = 0; i < K / 32; ++i) {
                const int k = 8 * (4 * i + (tid & 3));
                *(bf16x8 *)(As + (k >> 6) * (RL_ROWS * 64) + tile_off(tid >> 2, (k & 63) >> 3)) = pv[i];
            }
        } else {
            ln_gb_store<KT>(gbv, gb_s, tid);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // gain and shift are in LDS
            ln_finish<KT, 4>(xv, gb_s, a.eps, As, tid);
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

        // activation fragments -> registers (B operand of the transposed product): rows wr*32 + lm
        bf16x8 fa[KT * 4];
#pragma unroll
        for (int kk = 0; kk < KT * 4; ++kk)
            fa[kk] = *(const bf16x8 *)(As + (kk >> 2) * (RL_ROWS * 64) + tile_off(wr * 32 + lm, 2 * (kk & 3) + lh));

        // shrink: c[n][m] = sum_k At[n][k] x[m][k]; lane (lm, lh) ends up with ranks 4*lh + {0..3} (c[0..3]) and
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
        }

        // the W stream: two chunks per barrier, as two independent accumulator chains.  The accumulators start from the
        // bias.  Operands are fetched one K step (16) ahead of the MFMAs that use them: LDS latency is a hundred-odd
        // cycles, and the compiler on its own keeps only two or three reads in flight.
        auto bias_init = [&](int c) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 b = *(const f32x4 *)(bias_s + min(c * RL_BNC + wc * 32 + 8 * g + 4 * lh, a.N - 4));
#pragma unroll
                for (int z = 0; z < 4; ++z) acc[c][4 * g + z] = b[z];
            }
        };
        auto stream_step = [&](int c0, auto PAIR) {
            constexpr bool pair = decltype(PAIR)::value;
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const bf16_t *st0 = Ws + (c0 % RL_NS) * W_EL, *st1 = Ws + ((c0 + 1) % RL_NS) * W_EL;
            bf16x8 fw0[2][KT], fw1[2][KT];
            auto load = [&](int kk, int sl) {
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    fw0[sl][kt] = *(const bf16x8 *)(st0 + kt * (RL_BNC * 64) + tile_off(wc * 32 + lm, 2 * kk + lh));
                    if (pair) fw1[sl][kt] = *(const bf16x8 *)(st1 + kt * (RL_BNC * 64) + tile_off(wc * 32 + lm, 2 * kk + lh));
                }
            };
            load(0, 0);
            bias_init(c0);
            if (pair) bias_init(c0 + 1);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                if (kk < 3) load(kk + 1, (kk + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    acc[c0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw0[kk & 1][kt], fa[kt * 4 + kk], acc[c0], 0, 0, 0);
                    if (pair) acc[c0 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw1[kk & 1][kt], fa[kt * 4 + kk], acc[c0 + 1], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
#pragma unroll
        for (int sp = 0; sp < (RL_MAXCH + 1) / 2; ++sp) {
            // uniform conditions, written as guards (not a break) so that the loop unrolls and acc stays in registers
            if (2 * sp + 1 < nchunks) {
                if (2 * sp + 1 < RL_MAXCH) stream_step(2 * sp, std::true_type{});
            } else if (2 * sp < nchunks) {
                stream_step(2 * sp, std::false_type{});
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // Bt_k has landed; every wave is done with the ring
        // expand: lane (column, lh) supplies ranks 4*lh + {0..3} and 8 + 4*lh + {0..3} of Bt_k's row, the order the shrink left in fs
        if (k_ad >= 0) {
            // r is a multiple of 4: each half of the operand is one 8-byte read, at a clamped offset and zeroed where the
            // rank does not exist (no branches: lanes of one wave differ in lh)
            const bf16_t *BtL = As;
            const bool lo_ok = 4 * lh + 4 <= a.r, hi_ok = 8 + 4 * lh + 4 <= a.r;
            const int lo_o = lo_ok ? 4 * lh : 0, hi_o = hi_ok ? 8 + 4 * lh : 0;
            const bf16x4 zero4 = {0, 0, 0, 0};
#pragma unroll
            for (int c = 0; c < RL_MAXCH; ++c) {
                if (c < nchunks) {
                    const bf16_t *bt = BtL + (size_t)min(c * RL_BNC + wc * 32 + lm, a.N - 1) * a.r;
                    const bf16x4 lo = lo_ok ? *(const bf16x4 *)(bt + lo_o) : zero4, hi = hi_ok ? *(const bf16x4 *)(bt + hi_o) : zero4;
                    const bf16x8 f = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, fs, acc[c], 0, 0, 0);
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // Bt_k is dead: the staging tile may overwrite it
        // A lane owns one row, so storing from registers would touch 32 cache lines per instruction with 8 or 16
        // bytes each.  Instead the finished tile (bias, GELU applied, output type) is laid out row-major in LDS
        // and copied out with consecutive threads on consecutive 16-byte pieces of a row.
        char *trow = tile + (wr * 32 + lm) * stride + (wc * 32 + 4 * lh) * (f32out ? 4 : 2);
        auto stage_chunk = [&](int c, auto FULL) {
            constexpr bool full = decltype(FULL)::value;   // all 64 columns of the chunk exist: no per-lane predicate
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = c * RL_BNC + wc * 32 + 8 * g + 4 * lh;
                f32x4 v = {acc[c][4 * g], acc[c][4 * g + 1], acc[c][4 * g + 2], acc[c][4 * g + 3]};
                if (f32out) {
                    if (full || col < a.N) *(f32x4 *)(trow + (c * RL_BNC + 8 * g) * 4) = v;
                } else {
                    if (MODE == EPI_GELU) v = gelu_poly4(v);
                    const bf16x4 w = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                    if (full || col < a.N) *(bf16x4 *)(trow + (c * RL_BNC + 8 * g) * 2) = w;
                }
            }
        };
#pragma unroll
        for (int c = 0; c < RL_MAXCH; ++c) {
            if ((c + 1) * RL_BNC <= a.N) stage_chunk(c, std::true_type{});
            else if (c < nchunks) stage_chunk(c, std::false_type{});
        }
    }
    __syncthreads();
    char *out = (char *)a.out + ((size_t)ob * a.T + t0) * row_bytes;
    if (f32out) {
        // the loader threads hold the residual pieces; they finish the tile alone
        if (loader) {
#pragma unroll
            for (int j = 0; j < RL_MAXRES; ++j) {
                const int idx = lt + 256 * j;
                if (idx < rows * pieces) {
                    const int row = idx / pieces, p = idx - row * pieces;
                    f32x4 v = *(const f32x4 *)(tile + row * stride + p * 16);
                    if (a.res) v += res[j];
                    *(f32x4 *)(out + (size_t)row * row_bytes + p * 16) = v;
                }
            }
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
    constexpr int LDS = (KT * RL_ROWS * 64 + RL_NS * KT * RL_BNC * 64) * 2 + RL_MAXCH * RL_BNC * 4 + 256 + KT * 512;   // + dump words of the L2 warm-up, LayerNorm gain and shift
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
    if (!((K == 64 || K == 128 || K == 192) && N >= 8 && N % 8 == 0 && N <= RL_MAXCH * RL_BNC && (!lora || (r >= 4 && r <= 16 && r % 4 == 0)))) return false;
    if (f32out && N > 16 * RL_MAXRES) return false;                      // residual pieces held in registers
    if (lora && (long)N * r * 2 > (long)(K / 64) * RL_ROWS * 64 * 2) return false;   // Bt_k takes the place of the activation rows
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
