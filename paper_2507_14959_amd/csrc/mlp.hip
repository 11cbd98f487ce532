// MLP half of a pre-LN transformer layer for narrow models (D <= 192), on tiles of 64 token rows, in place:
//
//     x <- x + GELU(LayerNorm(x) W1 + b1) W2 + b2
//
// (the feed-forward sub-block of the ViT backbone; no low-rank branch on fc1 / fc2 -- layers that adapt these
// two linears take the separate kernels).  The operation is row-wise, so the tiles run over all rows of the
// launch regardless of block boundaries.  One workgroup owns 64 rows.  LayerNorm(x) is produced once and kept
// as MFMA operand registers; the hidden activation never leaves the chip: it exists one 64-column chunk at a
// time, as a bf16 tile in LDS between the two products.  W1 and W2 stream through a five-stage LDS ring in
// 24 KB items: W1's rows of a chunk, and the 64-wide K slice of W2 that the chunk feeds.
//
// Eight waves with two jobs.  Every workgroup of the launch streams the same weights out of L2 at the same
// time, and L2 delivers about 30 bytes per clock to each of them; a wave that issues a load into that
// saturated path is held at the issue stage until the path takes it.  So the loads are not issued by the
// waves that compute:
//   waves 0-3 (2 x 2 over the 64 x 64 chunk): per step h, first product of chunk h (accumulator in registers),
//             bias + GELU of chunk h - 1 into the hidden tile, second product of chunk h - 2 from the hidden
//             tile -- the GELU arithmetic is issued between the MFMAs of the same wave and runs in their shadow;
//   waves 4-7: nothing but global_load_lds_dwordx4 into the ring, counted with vmcnt.
// One barrier per step hands ring stages and hidden tiles back and forth.
#include "poly_dev.h"
#include "rowtile.h"

#include <type_traits>

namespace {

constexpr int ML_NS = 5;           // LDS stages of the weight stream
constexpr int ML_THREADS = 512;
constexpr int ML_MAX_DM = 768;

template <int KT>
__global__ __launch_bounds__(ML_THREADS) void mlp_kernel(const MlpArgs a)
{
    constexpr int D = 64 * KT;
    constexpr int A_EL = (KT < 2 ? 2 : KT) * 64 * 64;   // LayerNorm(x) rows (KT tiles of [64][64]); later the two hidden tiles
    constexpr int IT_EL = KT * 64 * 64;          // one stream item: KT tiles of [64][64]
    constexpr int NLD = 2 * KT;                  // loads per loader wave and item: 16 rows of each tile, 8 rows per load
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Ws = lds + A_EL;
    float *b1_s = (float *)(lds + A_EL + ML_NS * IT_EL);   // [Dm]
    float *b2_s = b1_s + ML_MAX_DM;                        // [D]
    float *dump_s = b2_s + D;                              // 64 words nobody reads (target of the L2 warm-up loads)
    float *gb_s = dump_s + 64;                             // LayerNorm gain [D] and shift [D]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave >= 4;
    const int wr = (wave >> 1) & 1, wc = wave & 1, lm = lane & 31, lh = lane >> 5;
    const int Dm = a.Dm;
    const int nch = Dm >> 6;                     // chunks of 64 hidden columns
    const int NQ = 2 * nch;                      // stream items: W1 part and W2 part of every chunk
    const long t0 = (long)blockIdx.x * 64;       // first row of this tile, counted over all blocks

    // Stream order = order of use.  Step h needs W2's slice of chunk h - 2 and W1's rows of chunk h:
    //   q = 0, 1: W1(0), W1(1);   q = 2, 3: W2(0), W1(2);   q = 4, 5: W2(1), W1(3);  ...  ; last two: W2(nch-2), W2(nch-1).
    // Loader wave w loads rows 16w .. 16w + 15 of each of the item's KT tiles, 8 rows (1 KB) per load.  A row's
    // 128 bytes land in lane order; the tile swizzle is applied by permuting the 16-byte pieces on the global side.
    const int lw = wave & 3, lr = lane >> 3;
    auto issue_item = [&](int q) {
        const bool second = q >= 2 && ((q & 1) == 0 || q == NQ - 1);
        const int c = q < 2 ? q : (second ? (q == NQ - 1 ? nch - 1 : (q >> 1) - 1) : (q + 1) >> 1);
        bf16_t *st = Ws + (q % ML_NS) * IT_EL;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int row = lw * 16 + half * 8 + lr;
            const unsigned sw = ((lane & 7) ^ ((row >> 1) & 7)) << 3;
            const unsigned off = second ? (row * Dm + sw) * 2 : (row * D + sw) * 2;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const unsigned dst = __builtin_amdgcn_readfirstlane(lds_addr_of(st + t * 4096 + (lw * 16 + half * 8) * 64));
                if (!second) glds16_s(a.W1t + (size_t)c * 64 * D + t * 64, off, dst);      // tile t: k = 64 t ..
                else glds16_s(a.W2t + (size_t)c * 64 + (size_t)t * 64 * Dm, off, dst);     // tile t: output columns 64 t ..
            }
        }
    };
    // newest item needed in step h
    auto need_at = [&](int h) { return h < 2 ? h : min(2 * h - 1, NQ - 1); };
    // The x rows are requested before anything else: they come from HBM (another kernel has just written them), and
    // whatever is requested first is served first.  The computing waves take them (and the rest of the prologue).
    float *xt = a.x + (size_t)t0 * D;
    f32x4 xv[D / 16];
    f32x4 gbv = {0.f, 0.f, 0.f, 0.f};
    float b1v[ML_MAX_DM / 256], b2v = 0.f;
    if (!loader) {
        ln_load<KT, 4>(xt, (int)min(64L, (long)a.n_out * a.T - t0), 0, tid, xv);   // clamped to the buffer; rows past the true count are never stored
        // gain, shift and biases as well: requested after the weight stream has started they would arrive behind it
        gbv = ln_gb_load<KT>(a.ln_g, a.ln_b, tid);
#pragma unroll
        for (int j = 0; j < ML_MAX_DM / 256; ++j) b1v[j] = a.b1[min(tid + 256 * j, Dm - 1)];   // unconditional: see ln_gb_load
        b2v = a.b2[min(tid, D - 1)];
    }

    const long n_out = a.n_out_dev ? min(*a.n_out_dev, a.n_out) : a.n_out;
    const long nrows = n_out * a.T;
    if (t0 >= nrows) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    const int rows = (int)min(64L, nrows - t0);
    // the weight stream (workgroups past the row count have left without moving data): only the items of steps 0 and 1
    // for now -- the x rows are still on their way and would be slowed down by more; the rest of the ring follows
    // at the barrier below, which the computing waves reach once their loads have arrived
    int last = 1;                                // newest item requested
    if (loader) {
        for (int q = 0; q <= last; ++q) issue_item(q);
        // the rest of both matrices: into L2 now, so that the ring refills below are L2 hits
        l2_warm(a.W1t, (long)Dm * D * 2, lds_addr_of(dump_s), tid - 256, 256);
        l2_warm(a.W2t, (long)Dm * D * 2, lds_addr_of(dump_s), tid - 256, 256);
    } else {
        ln_gb_store<KT>(gbv, gb_s, tid);
#pragma unroll
        for (int j = 0; j < ML_MAX_DM / 256; ++j)
            if (tid + 256 * j < Dm) b1_s[tid + 256 * j] = b1v[j];
        if (tid < D) b2_s[tid] = b2v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");    // gain and shift are in LDS
    if (loader) {
        for (int q = last + 1; q < min(ML_NS, NQ); ++q) issue_item(q);
        last = min(ML_NS, NQ) - 1;
    } else {
        ln_finish<KT, 4>(xv, gb_s, a.eps, As, tid);
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // LayerNorm(x) rows wr*32 + lm as the B operand of the first product
    bf16x8 fa[KT * 4];
    f32x16 y[KT];                                // second product: rows wr*32 + lm, columns wc*32*KT + 32 p + ..
    f32x16 hcur, hnext;                          // first product of chunks h - 1 / h: row lm, columns wc*32 + 8*(e/4) + 4*lh + e%4
    if (!loader) {
#pragma unroll
        for (int kk = 0; kk < KT * 4; ++kk)
            fa[kk] = *(const bf16x8 *)(As + (kk >> 2) * 4096 + tile_off(wr * 32 + lm, 2 * (kk & 3) + lh));
#pragma unroll
        for (int p = 0; p < KT; ++p)
#pragma unroll
            for (int e = 0; e < 16; ++e) y[p][e] = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) hcur[e] = hnext[e] = 0.f;
    }
    // hidden tiles [64 rows][64 columns of a chunk], chunk c in tile c & 1.  As is dead once every wave has its fa:
    // the barrier of step 0 comes before the first write (step 1).
    bf16_t *Hs = As;

    // ---- loader: wait until the items of step h have landed, barrier, refill the ring behind the items that
    // every wave is done with (those of step h - 1 and earlier)
    auto loader_step = [&](int h) {
        const int ahead = last - need_at(h);     // newer items may stay in flight: loads complete in issue order
        if (ahead >= 3) rl_wait_barrier<3 * NLD>();
        else if (ahead == 2) rl_wait_barrier<2 * NLD>();
        else if (ahead == 1) rl_wait_barrier<NLD>();
        else rl_wait_barrier<0>();
        const int upto = min((h >= 1 ? need_at(h - 1) : -1) + ML_NS, NQ - 1);
        for (int q = last + 1; q <= upto; ++q) issue_item(q);
        last = max(last, upto);
    };
    // ---- computing waves, step h: d1: hnext = LayerNorm(x) W1 rows of chunk h; dg: hidden tile of chunk h - 1 =
    // GELU(hcur + b1); d2: y += hidden(chunk h - 2) W2 slice.  MFMA operands are fetched one K step (16) ahead of
    // the MFMAs that use them (LDS latency is a hundred-odd cycles and the compiler on its own keeps only two or
    // three reads in flight); the scheduling barriers pin the order "reads of K step kk + 1, then MFMAs of K step kk
    // with a quarter of the GELU arithmetic between them".
    auto compute_step = [&](auto D1, auto DG, auto D2, int h) {
        constexpr bool d1 = decltype(D1)::value, dg = decltype(DG)::value, d2 = decltype(D2)::value;
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const bf16_t *s2 = Ws + ((h == nch + 1 ? NQ - 1 : 2 * h - 2) % ML_NS) * IT_EL;   // W2(h - 2)
        const bf16_t *s1 = Ws + ((h < 2 ? h : 2 * h - 1) % ML_NS) * IT_EL;               // W1(h)
        const bf16_t *Hr = Hs + (h & 1) * 4096;                                          // chunk h - 2
        bf16_t *Hw = Hs + ((h - 1) & 1) * 4096;                                          // chunk h - 1
        bf16x8 fh[2], f2[2][KT], f1[2][KT];
        f32x4 b[4];
        auto load = [&](int kk, int s) {
            if (d2) {
                fh[s] = *(const bf16x8 *)(Hr + tile_off(wr * 32 + lm, 2 * kk + lh));
#pragma unroll
                for (int p = 0; p < KT; ++p) {
                    const int ncol = wc * 32 * KT + p * 32;   // first of this piece's 32 output columns
                    f2[s][p] = *(const bf16x8 *)(s2 + (ncol >> 6) * 4096 + tile_off((ncol & 63) + lm, 2 * kk + lh));
                }
            }
            if (d1) {
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) f1[s][kt] = *(const bf16x8 *)(s1 + kt * 4096 + tile_off(wc * 32 + lm, 2 * kk + lh));
            }
        };
        if (dg) {
            const float *bp = b1_s + (h - 1) * 64 + wc * 32 + 4 * lh;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) b[g4] = *(const f32x4 *)(bp + 8 * g4);
        }
        load(0, 0);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) load(kk + 1, (kk + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
            if (d2) {
#pragma unroll
                for (int p = 0; p < KT; ++p) y[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[kk & 1][p], fh[kk & 1], y[p], 0, 0, 0);
            }
            if (d1) {
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) hnext = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[kk & 1][kt], fa[kt * 4 + kk], hnext, 0, 0, 0);
            }
            if (dg) {
                const f32x4 v = gelu_poly4(f32x4{hcur[4 * kk], hcur[4 * kk + 1], hcur[4 * kk + 2], hcur[4 * kk + 3]} + b[kk]);
                const bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                *(bf16x4 *)(Hw + tile_off(wr * 32 + lm, 4 * wc + kk) + 4 * lh) = o;
            }
            if ((d1 || d2) && dg) {
                // one MFMA, then a share of the vector work, so that the vector work is issued while an MFMA runs
                constexpr int NM = (d1 ? KT : 0) + (d2 ? KT : 0);
#pragma unroll
                for (int i = 0; i < NM; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, (64 + NM - 1) / NM, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (d1) {
            hcur = hnext;
#pragma unroll
            for (int e = 0; e < 16; ++e) hnext[e] = 0.f;
        }
    };
    using T_ = std::true_type;
    using F_ = std::false_type;

    if (loader) {
        for (int h = 0; h < nch + 2; ++h) loader_step(h);
    } else {
        compute_step(T_{}, F_{}, F_{}, 0);
        compute_step(T_{}, T_{}, F_{}, 1);
        for (int h = 2; h < nch; ++h) compute_step(T_{}, T_{}, T_{}, h);
        compute_step(F_{}, T_{}, T_{}, nch);
        compute_step(F_{}, F_{}, T_{}, nch + 1);
    }

    // ---- y as a row-major fp32 tile [64][D] in LDS (the ring is dead: every item was waited for before the last
    // barrier), then all threads add b2 + x and store full rows
    constexpr int stride = D * 4 + 16;           // bytes; rows start 4 banks apart
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // every wave is done reading the ring and the hidden tiles
    if (!loader) {
        char *prow = (char *)lds + (wr * 32 + lm) * stride + (wc * 32 * KT) * 4 + 16 * lh;
#pragma unroll
        for (int p = 0; p < KT; ++p)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
                *(f32x4 *)(prow + (p * 32 + 8 * g4) * 4) = f32x4{y[p][4 * g4], y[p][4 * g4 + 1], y[p][4 * g4 + 2], y[p][4 * g4 + 3]};
    }
    __syncthreads();
    constexpr int pieces = D / 4;                // 16-byte pieces per row
    const char *P = (const char *)lds;
    for (int idx = tid; idx < rows * pieces; idx += ML_THREADS) {
        const int row = idx / pieces, p = idx - row * pieces;
        const f32x4 v = *(const f32x4 *)(P + row * stride + p * 16) + *(const f32x4 *)(b2_s + 4 * p);
        f32x4 *xp = (f32x4 *)(xt + (size_t)row * D + 4 * p);
        *xp = *xp + v;
    }
}

template <int KT> int launch_mlp_kt(const MlpArgs &a, hipStream_t st)
{
    constexpr int LDS = ((KT < 2 ? 2 : KT) + ML_NS * KT) * 64 * 64 * 2 + (ML_MAX_DM + 64 * KT + 64 + 128 * KT) * 4;
    auto kern = mlp_kernel<KT>;
    if (LDS > 64 * 1024) {
        static bool attr_set = false;   // raising the dynamic LDS limit is a per-kernel, process-wide setting
        if (!attr_set) {
            if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess) return POLY_EHIP;
            attr_set = true;
        }
    }
    const long tiles = ((long)a.n_out * a.T + 63) / 64;
    POLY_LAUNCH_SHMEM(POLY_STAGE_GEMM, kern, dim3((unsigned)tiles), dim3(ML_THREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}

}  // namespace

bool mlp_supported(int D, int Dm)
{
    return (D == 64 || D == 128 || D == 192) && Dm >= 128 && Dm % 64 == 0 && Dm <= ML_MAX_DM;
}

int launch_mlp(const MlpArgs &a, hipStream_t st)
{
    if (a.n_out <= 0 || a.T <= 0) return POLY_OK;
    if (!mlp_supported(a.D, a.Dm) || (long)a.n_out * a.T > 0x3fffffffL) return POLY_EINVAL;
    switch (a.D / 64) {
    case 1: return launch_mlp_kt<1>(a, st);
    case 2: return launch_mlp_kt<2>(a, st);
    default: return launch_mlp_kt<3>(a, st);
    }
}
