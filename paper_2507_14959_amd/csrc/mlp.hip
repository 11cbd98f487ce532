// MLP half of a pre-LN transformer layer for narrow models (D <= 192), on tiles of 64 token rows, in place:
//
//     x <- x + GELU(LayerNorm(x) W1 + b1) W2 + b2
//
// (the feed-forward sub-block of the ViT backbone; no low-rank branch on fc1 / fc2 -- layers that adapt these
// two linears take the separate kernels).  One workgroup owns 64 rows.  LayerNorm(x) is produced once and kept as
// MFMA operand registers; the hidden activation never leaves the chip: it exists one 64-column chunk at a
// time, as a bf16 tile in LDS between the two products.  W1 and W2 stream through a five-stage LDS ring in
// 24 KB items: W1's rows of a chunk, and the 64-wide K slice of W2 that the chunk feeds.
//
// Eight waves = two groups of 2 x 2; group g owns the chunks c with c % 2 == g.  Time is cut into steps separated
// by one barrier.  In step h the group h % 2 is the MFMA group: first product of chunk h (accumulator kept in
// registers) and second product of chunk h - 2 (hidden tile read from LDS).  The other group is the vector
// group: bias + GELU on the accumulator of chunk h - 1, written as the hidden tile.  The two waves that share a
// SIMD belong to different groups, so in every step one of them issues MFMAs and the other plain arithmetic.
#include "poly_dev.h"
#include "rowtile.h"

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
    constexpr int NLD = KT;                      // loads per wave and item
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Ws = lds + A_EL;
    float *b1_s = (float *)(lds + A_EL + ML_NS * IT_EL);   // [Dm]
    float *b2_s = b1_s + ML_MAX_DM;                        // [D]

    const int tiles = (a.T + 63) / 64;
    const int ob = blockIdx.x / tiles, t0 = (blockIdx.x % tiles) * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2, wr = (wave >> 1) & 1, wc = wave & 1, lm = lane & 31, lh = lane >> 5;
    const int Dm = a.Dm;
    const int nch = Dm >> 6;                     // chunks (even: Dm is a multiple of 128)
    const int NQ = 2 * nch;                      // stream items: W1 part and W2 part of every chunk
    const int nsteps = nch + 2;

    // Stream order = order of use.  Step h needs W2's slice of chunk h - 2 and W1's rows of chunk h:
    //   q = 0, 1: W1(0), W1(1);   q = 2, 3: W2(0), W1(2);   q = 4, 5: W2(1), W1(3);  ...  ; last two: W2(nch-2), W2(nch-1).
    // Wave w loads rows 8w .. 8w + 7 of each of the item's KT tiles.
    const int lr = lane >> 3;
    auto issue_item = [&](int q) {
        const bool second = q >= 2 && ((q & 1) == 0 || q == NQ - 1);
        const int c = q < 2 ? q : (second ? (q == NQ - 1 ? nch - 1 : (q >> 1) - 1) : (q + 1) >> 1);
        const int row = wave * 8 + lr;
        const int sw = ((lane & 7) ^ ((row >> 1) & 7)) << 3;
        bf16_t *st = Ws + (q % ML_NS) * IT_EL + wave * 512;
        if (!second) {
            const bf16_t *src = a.W1t + ((size_t)c * 64 + row) * D + sw;               // tile kt: k = 64 kt ..
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) glds16(src + kt * 64, __builtin_amdgcn_readfirstlane(lds_addr_of(st + kt * 4096)));
        } else {
            const bf16_t *src = a.W2t + (size_t)row * Dm + c * 64 + sw;                // tile nt: output columns 64 nt ..
#pragma unroll
            for (int nt = 0; nt < KT; ++nt) glds16(src + (size_t)nt * 64 * Dm, __builtin_amdgcn_readfirstlane(lds_addr_of(st + nt * 4096)));
        }
    };
    // newest item needed in step h
    auto need_at = [&](int h) { return h < 2 ? h : min(2 * h - 1, NQ - 1); };
    int last = min(ML_NS, NQ) - 1;               // newest item requested
    for (int q = 0; q <= last; ++q) issue_item(q);

    const int n_out = a.n_out_dev ? min(*a.n_out_dev, a.n_out) : a.n_out;
    if (ob >= n_out) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    float *xblock = a.x + (size_t)ob * a.T * D;
    ln_rows_to_lds<KT>(xblock, a.T, t0, a.ln_g, a.ln_b, a.eps, As, tid);
    for (int i = tid; i < Dm; i += ML_THREADS) b1_s[i] = a.b1[i];
    if (tid < D) b2_s[tid] = a.b2[tid];
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // LayerNorm(x) rows wr*32 + lm as the B operand of the first product
    bf16x8 fa[KT * 4];
#pragma unroll
    for (int kk = 0; kk < KT * 4; ++kk)
        fa[kk] = *(const bf16x8 *)(As + (kk >> 2) * 4096 + tile_off(wr * 32 + lm, 2 * (kk & 3) + lh));
    bf16_t *Hs = As + grp * 4096;                // this group's hidden tile [64 rows][64 columns of the chunk]; As is dead once
                                                 // every wave has its fa (the barrier of step 0 comes before the first write)

    f32x16 y[KT];                                // second product: rows wr*32 + lm, columns wc*32*KT + 32 p + .., this group's chunks
#pragma unroll
    for (int p = 0; p < KT; ++p)
#pragma unroll
        for (int e = 0; e < 16; ++e) y[p][e] = 0.f;
    f32x16 hacc;                                 // first product of the group's current chunk: row lm, columns wc*32 + 8*(e/4) + 4*lh + e%4
#pragma unroll
    for (int e = 0; e < 16; ++e) hacc[e] = 0.f;

    for (int h = 0; h < nsteps; ++h) {
        // the items of this step must have landed; newer ones stay in flight (loads complete in issue order)
        const int ahead = last - need_at(h);
        if (ahead >= 3) rl_wait_barrier<3 * NLD>();
        else if (ahead == 2) rl_wait_barrier<2 * NLD>();
        else if (ahead == 1) rl_wait_barrier<NLD>();
        else rl_wait_barrier<0>();
        // every wave is past step h - 1, i.e. done with the items up to need_at(h - 1): refill the ring behind them
        const int upto = min((h >= 1 ? need_at(h - 1) : -1) + ML_NS, NQ - 1);
        for (int q = last + 1; q <= upto; ++q) issue_item(q);
        last = max(last, upto);

        if ((h & 1) == grp) {
            // ---- MFMA step: y += hidden(chunk h - 2) W2 slice; hacc = LayerNorm(x) W1 rows of chunk h.  Independent
            // accumulator chains, issued interleaved
            const bool do2 = h >= 2, do1 = h < nch;
            const bf16_t *s2 = Ws + ((2 * h - 2) % ML_NS) * IT_EL;                       // W2(h - 2) is item 2h - 2 (the last chunk's: NQ - 1)
            if (h == nch + 1) s2 = Ws + ((NQ - 1) % ML_NS) * IT_EL;
            const bf16_t *s1 = Ws + ((h < 2 ? h : 2 * h - 1) % ML_NS) * IT_EL;           // W1(h)
            if (do1) {
#pragma unroll
                for (int e = 0; e < 16; ++e) hacc[e] = 0.f;
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                if (do2) {
                    const bf16x8 fh = *(const bf16x8 *)(Hs + tile_off(wr * 32 + lm, 2 * kk + lh));
#pragma unroll
                    for (int p = 0; p < KT; ++p) {
                        const int ncol = wc * 32 * KT + p * 32;   // first of this piece's 32 output columns
                        const bf16x8 fw = *(const bf16x8 *)(s2 + (ncol >> 6) * 4096 + tile_off((ncol & 63) + lm, 2 * kk + lh));
                        y[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fh, y[p], 0, 0, 0);
                    }
                }
                if (do1) {
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt) {
                        const bf16x8 fw = *(const bf16x8 *)(s1 + kt * 4096 + tile_off(wc * 32 + lm, 2 * kk + lh));
                        hacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fa[kt * 4 + kk], hacc, 0, 0, 0);
                    }
                }
            }
        } else if (h >= 1 && h <= nch) {
            // ---- vector step: hidden tile of chunk h - 1 = GELU(hacc + b1), as bf16 in the operand layout of the second product
            const float *bp = b1_s + (h - 1) * 64 + wc * 32 + 4 * lh;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 b = *(const f32x4 *)(bp + 8 * g4);
                bf16x4 o;
#pragma unroll
                for (int z = 0; z < 4; ++z) o[z] = (bf16_t)gelu_poly(hacc[4 * g4 + z] + b[z]);
                *(bf16x4 *)(Hs + tile_off(wr * 32 + lm, 4 * wc + g4) + 4 * lh) = o;
            }
        }
    }

    // ---- the two groups hold partial sums over different chunks: both lay theirs out as a row-major fp32 tile
    // P[grp] = [64][D], then all threads add P[0] + P[1] + b2 + x and store full rows.  The ring is dead
    // (the last wait was vmcnt(0)).
    constexpr int stride = D * 4 + 16;           // bytes; rows start 4 banks apart
    asm volatile("s_barrier" ::: "memory");      // every wave is done reading the ring and the hidden tiles
    {
        char *prow = (char *)lds + grp * (64 * stride) + (wr * 32 + lm) * stride + (wc * 32 * KT) * 4 + 16 * lh;
#pragma unroll
        for (int p = 0; p < KT; ++p)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
                *(f32x4 *)(prow + (p * 32 + 8 * g4) * 4) = f32x4{y[p][4 * g4], y[p][4 * g4 + 1], y[p][4 * g4 + 2], y[p][4 * g4 + 3]};
    }
    __syncthreads();
    constexpr int pieces = D / 4;                // 16-byte pieces per row
    const int rows = min(64, a.T - t0);
    float *xt = xblock + (size_t)t0 * D;
    const char *P0 = (const char *)lds, *P1 = P0 + 64 * stride;
    for (int idx = tid; idx < rows * pieces; idx += ML_THREADS) {
        const int row = idx / pieces, p = idx - row * pieces;
        f32x4 v = *(const f32x4 *)(P0 + row * stride + p * 16) + *(const f32x4 *)(P1 + row * stride + p * 16) + *(const f32x4 *)(b2_s + 4 * p);
        f32x4 *xp = (f32x4 *)(xt + (size_t)row * D + 4 * p);
        *xp = *xp + v;
    }
}

template <int KT> int launch_mlp_kt(const MlpArgs &a, hipStream_t st)
{
    constexpr int LDS = ((KT < 2 ? 2 : KT) + ML_NS * KT) * 64 * 64 * 2 + (ML_MAX_DM + 64 * KT) * 4;
    auto kern = mlp_kernel<KT>;
    if (LDS > 64 * 1024) {
        static bool attr_set = false;   // raising the dynamic LDS limit is a per-kernel, process-wide setting
        if (!attr_set) {
            if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess) return POLY_EHIP;
            attr_set = true;
        }
    }
    const int tiles = (a.T + 63) / 64;
    POLY_LAUNCH_SHMEM(POLY_STAGE_GEMM, kern, dim3((unsigned)(a.n_out * tiles)), dim3(ML_THREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}

}  // namespace

bool mlp_supported(int D, int Dm)
{
    return (D == 64 || D == 128 || D == 192) && Dm >= 128 && Dm % 128 == 0 && Dm <= ML_MAX_DM;
}

int launch_mlp(const MlpArgs &a, hipStream_t st)
{
    if (a.n_out <= 0 || a.T <= 0) return POLY_OK;
    if (!mlp_supported(a.D, a.Dm)) return POLY_EINVAL;
    switch (a.D / 64) {
    case 1: return launch_mlp_kt<1>(a, st);
    case 2: return launch_mlp_kt<2>(a, st);
    default: return launch_mlp_kt<3>(a, st);
    }
}
