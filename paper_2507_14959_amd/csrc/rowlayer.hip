// Everything of a pre-LN transformer layer that works row by row, for narrow models (D <= 192), in one kernel
// on tiles of 64 token rows:
//
//   A (optional)  x' = res + o Wp + bp + s (o Ap_k) Bp_k                 attention output projection, Sec. 3.1 form
//   B             x'' = x' + GELU(LayerNorm2(x') W1 + b1) W2 + b2        feed-forward block (no low-rank branch here)
//   C (optional)  qkv = LayerNorm1'(x'') Wq + bq + s (.. Aq_k) Bq_k      qkv linear of the NEXT layer
//
// Only softmax attention needs whole blocks; with A, B and C in one launch a layer is two kernels instead of
// four, and x', the hidden activation and LayerNorm outputs never leave the chip.  Launch overhead and the cold
// start of every kernel (inputs written by the previous kernel come from HBM) were a quarter of the layer time.
//
// Eight waves.  A wave that issues a load into the saturated L2 path is held at the issue stage, so the weight stream
// has a wave of its own and the waves that compute issue no loads while they compute:
//   waves 0-3 (2 x 2 over a 64 x 64 chunk): the MFMA work of A and C; in B the first product and the GELU;
//   wave 4: the weight stream into a ring of LDS stages (24 KB items; five stages in A and C, four in B);
//   waves 5-7: in B the second product (wave 5 + j owns output columns 64 j .. 64 j + 63 of all 64 rows), each fed from its
//             own tile of the current W2 slice in the fifth stage, which it refills itself as soon as it has copied the
//             tile into registers.  A stage of a shared ring is freed by a workgroup barrier, so what is read in one step can
//             be requested again in the next step at the earliest and the stream runs dry at every barrier; with W2 out
//             of the ring the stream of W1 runs three chunks ahead and the loads of W2 never wait for a barrier;
//   waves 4-7 together: At_k / Bt_k of the block's adapter into LDS, and the residual stream: they hold x' (fp32,
//             16 threads per row) in registers from phase A to the end, do both LayerNorms on it and write x''.
// The loop of B is bound by the number of instructions a wave issues (a wave issues one every five cycles or so,
// whatever the instruction; two waves on a SIMD issue twice as many), which is why its two products sit on
// different waves: the GELU's arithmetic and the second product's operand reads are issued side by side.
// Phase boundaries pass a 64 x D fp32 tile through LDS; it takes the place of ring stages 0-2, so every phase's
// stream starts in stage 3 and at most two items of the next phase are prefetched across a boundary.
#include "poly_dev.h"
#include "rowtile.h"

#include <type_traits>

namespace {

constexpr int LY_NS = 5;            // LDS stages of the weight stream
constexpr int LY_THREADS = 512;
constexpr int LY_MAX_DM = 768;
constexpr int LY_MAX_NQ = 576;      // qkv columns: 9 chunks, their accumulators stay in registers
constexpr int LY_MAXCH = LY_MAX_NQ / 64;
constexpr int LY_AT_STRIDE = 200;   // elements per rank row of At_k in LDS (192 + 8: rows start 4 banks apart)

template <int KT, bool HAS_PROJ, bool HAS_QKV>
__global__ __launch_bounds__(LY_THREADS) void rowlayer_kernel(const RowLayerArgs a)
{
    constexpr int D = 64 * KT;
    constexpr int A_EL = (KT < 2 ? 2 : KT) * 64 * 64;   // activation rows (KT tiles of [64][64]) / Bt_k / the two hidden tiles
    constexpr int IT_EL = KT * 64 * 64;          // one stream item: KT tiles of [64][64]
    constexpr int NLD = 8 * KT;                  // loads per item (all by wave 4): 64 rows of each tile, 8 rows per load
    constexpr int NV = D / 16;                   // 16-byte pieces of fp32 rows per loader thread (four rows, 16 threads per row)
    constexpr int XSTRIDE = D * 4 + 16;          // bytes per row of the fp32 hand-over tile
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Ws = lds + A_EL;
    float *b1_s = (float *)(lds + A_EL + LY_NS * IT_EL);   // [Dm]
    float *bq_s = b1_s + LY_MAX_DM;                        // [3 D]
    float *bp_s = bq_s + LY_MAX_NQ;                        // [D]
    float *b2_s = bp_s + D;                                // [D]
    float *gb2_s = b2_s + D;                               // LayerNorm2 gain [D], shift [D]
    float *gbq_s = gb2_s + 2 * D;                          // LayerNorm1' gain, shift
    bf16_t *at_s = (bf16_t *)(gbq_s + 2 * D);              // At_k of the current phase: [16][LY_AT_STRIDE]
    // Phi table of the GELU (phase B): behind the two hidden tiles in the activation-row area when that has 24 KB, else in
    // a region of its own (narrower models leave LDS to spare)
    float *gelu_s = KT == 3 ? (float *)(As + 2 * 4096) : (float *)(at_s + 16 * LY_AT_STRIDE);

    const int tiles = (a.T + 63) / 64;
    const int ob = blockIdx.x / tiles, t0 = (blockIdx.x % tiles) * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave >= 4;
    const int wr = (wave >> 1) & 1, wc = wave & 1, lm = lane & 31, lh = lane >> 5;
    const int lw = wave & 3, lr = lane >> 3, lt = tid & 255;
    const int Dm = a.Dm, nch = Dm >> 6;
    const int Nq = 3 * D, nchq = (Nq + 63) / 64;
    const int rows = min(64, a.T - t0);

    // ---- the stream.  Items (KT tiles each), in order: phase A: Wp chunk c (stage c); phase B: W1's rows of chunk c, for
    // the first product, in the four stages 0-3 (stage (SB0 + c) % 4; SB0 = 3 when A comes first, whose hand-over tile takes
    // stages 0-2); phase C: Wq chunk c at position PC + c (stage = position % 5, PC = 3 mod 5).  The slices of W2 do not pass
    // through the ring: each wave of the second product keeps its own tile of the current slice in stage 4 and requests the
    // next one itself (see phase B).
    const int NA = HAS_PROJ ? KT : 0;
    constexpr int SB0 = HAS_PROJ ? 3 : 0;
    const int PC = 8;
    const int NI = NA + nch + (HAS_QKV ? nchq : 0);                 // items, numbered in order
    // ring position for the items of A and C; those of B are requested explicitly (never by refill)
    auto pos_of = [&](int i) { return i < NA ? i : (i < NA + nch ? 1 << 20 : PC + (i - NA - nch)); };
    // wave 4 loads each of the item's KT tiles, 8 rows (1 KB) per load; a row's 128 bytes land in lane order, the tile
    // swizzle is applied by permuting the 16-byte pieces on the global side
    auto issue_item = [&](int i) {
        const bf16_t *base;
        int stage;
        if (i < NA) { base = a.Wpt + (size_t)i * 64 * D; stage = i; }
        else if (i < NA + nch) { const int c = i - NA; base = a.W1t + (size_t)c * 64 * D; stage = (SB0 + c) & 3; }
        else { const int c = i - NA - nch; base = a.Wqt + (size_t)c * 64 * D; stage = (PC + c) % LY_NS; }
        bf16_t *st = Ws + stage * IT_EL;
        const int rstride = D, tstride = 64;              // elements between rows / between tiles (tile t: k = 64 t ..)
        // row 8 g + lr of a tile: its 16-byte pieces are permuted by (row >> 1) & 7 = 4 (g & 1) + (lr >> 1).  Every matrix
        // here has a multiple of 64 rows, so no row of a tile is past its end.
        const unsigned rb = rstride * 2;
        const unsigned e0 = lr * rb + ((((lane & 7) ^ (lr >> 1))) << 4), e1 = lr * rb + ((((lane & 7) ^ (4 + (lr >> 1)))) << 4);
        const unsigned lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(st));
#pragma unroll
        for (int t = 0; t < KT; ++t)
            glds16_tile8(base + (size_t)t * tstride, lds0 + t * 8192, e0, e1 + 8 * rb, e0 + 16 * rb, e1 + 24 * rb, e0 + 32 * rb, e1 + 40 * rb,
                         e0 + 48 * rb, e1 + 56 * rb);
    };
    // At_k [r][D] -> at_s, one rank row per load (24 * KT / 3 lanes), rows LY_AT_STRIDE elements apart
    auto issue_at = [&](const bf16_t *At_k, int r) {
        for (int rk = lw; rk < r; rk += 4)
            if (lane < D / 8) glds16(At_k + (size_t)rk * D + lane * 8, __builtin_amdgcn_readfirstlane(lds_addr_of(at_s + rk * LY_AT_STRIDE)));
    };
    // Bt_k [N][r] -> As, as it is
    auto issue_bt = [&](const bf16_t *Bt_k, int N, int r) {
        const int n16 = (N * r) >> 3;
        for (int i0 = lw * 64; i0 < n16; i0 += 256)
            if (i0 + lane < n16) glds16((const char *)Bt_k + (size_t)(i0 + lane) * 16, __builtin_amdgcn_readfirstlane(lds_addr_of(As) + i0 * 16));
    };

    // ---- everything whose address needs no metadata is requested first: it comes from HBM (another kernel has just
    // written it), and whatever is requested first is served first
    bf16x8 pv[D / 32];                           // computing waves: o rows (4 threads per row, pieces part, part + 4, ..)
    f32x4 xr[NV];                                // loader waves: residual rows, then x', then x''
    f32x4 gb2v = {0.f, 0.f, 0.f, 0.f}, gbqv = {0.f, 0.f, 0.f, 0.f};
    float b1v[LY_MAX_DM / 256], bqv[(LY_MAX_NQ + 255) / 256], b2v = 0.f, bpv = 0.f;
    const bool res_early = !HAS_PROJ || a.res_block_of_out == nullptr;
    // Rows of the residual stream in the loader waves: 16 threads per row.  Thread (slot = lt / 16, part = lt % 16) holds, of
    // the four rows slot + 16 k, the 16-byte pieces part + 16 i (i < KT) as xr[k * KT + i]: the 16 lanes of a row read and
    // write 256 contiguous bytes per instruction (whole cache lines), the row statistics are sums over a DPP row, and a
    // thread needs the gains of only KT pieces for its four rows.
    const int xslot = lt >> 4, xpart = lt & 15;
    auto load_res = [&](int rblk) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float *src = (HAS_PROJ ? a.res : a.x_out) + ((size_t)rblk * a.T + min(t0 + xslot + 16 * k, a.T - 1)) * D + 4 * xpart;
#pragma unroll
            for (int i = 0; i < KT; ++i) xr[k * KT + i] = *(const f32x4 *)(src + 64 * i);
        }
    };
    if (!loader) {
        if (HAS_PROJ) {
            const bf16_t *src = a.o + ((size_t)ob * a.T + min(t0 + (tid >> 2), a.T - 1)) * D + 8 * (tid & 3);
#pragma unroll
            for (int i = 0; i < D / 32; ++i) pv[i] = *(const bf16x8 *)(src + 32 * i);
            bpv = a.bp[min(tid, D - 1)];
        }
        gb2v = ln_gb_load<KT>(a.ln2_g, a.ln2_b, tid);
#pragma unroll
        for (int j = 0; j < LY_MAX_DM / 256; ++j) b1v[j] = a.b1[min(tid + 256 * j, Dm - 1)];   // unconditional: see ln_gb_load
        b2v = a.b2[min(tid, D - 1)];
        if (HAS_QKV) {
            gbqv = ln_gb_load<KT>(a.lnq_g, a.lnq_b, tid);
#pragma unroll
            for (int j = 0; j < (LY_MAX_NQ + 255) / 256; ++j) bqv[j] = a.bq[min(tid + 256 * j, Nq - 1)];
        }
    } else if (res_early) {
        load_res(ob);
    }

    const int n_out = a.n_out_dev ? min(*a.n_out_dev, a.n_out) : a.n_out;
    if (ob >= n_out) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    const int k_ad = a.adapter_of_out ? a.adapter_of_out[ob] : -1;
    const bool lora_p = HAS_PROJ && a.Apt && k_ad >= 0, lora_q = HAS_QKV && a.Aqt && k_ad >= 0;

    // ---- loader bookkeeping.  last: newest item requested; cpos: newest ring position every wave is done with.
    // An item may be requested once the item five positions earlier has been consumed, and never beyond `cap`
    // (the positions that a hand-over tile is about to use).
    int last = -1;
    auto refill = [&](int cpos, int cap) {
        while (last + 1 < NI && pos_of(last + 1) <= min(cpos + LY_NS, cap)) {
            ++last;
            if (wave == 4) { issue_item(last); }
        }
    };
    // item `need` has landed; newer ones may stay in flight (loads complete in issue order; the counter holds 63).
    // Waves 5-7 have no part in the stream: whatever else they requested has landed after this.
    auto wait_item = [&](int need) {
        const int ahead = wave == 4 ? last - need : 0;
        if (ahead >= 2) rl_wait_barrier<2 * NLD>();
        else if (ahead == 1) rl_wait_barrier<NLD>();
        else rl_wait_barrier<0>();
    };
    auto issue_next = [&]() {                    // the next item, whatever its position (the caller knows its stage is free)
        ++last;
        if (wave == 4) { issue_item(last); }
    };

    if (loader) {
        if (!res_early) load_res(a.res_block_of_out[ob]);
        // the first items only (all of phase A, or two of B) -- the rows above are still on their way and would be slowed
        // down by more.  At_k first: the wait for the first chunks then covers it (loads complete in issue order).
        if (lora_p) issue_at(a.Apt + (size_t)k_ad * a.r * D, a.r);
        if (HAS_PROJ) refill(-1, KT - 1);
        else { issue_next(); issue_next(); }       // (nch >= 2)
    } else {
        // prologue of the computing waves: what they requested -> LDS
        if (HAS_PROJ) {
#pragma unroll
            for (int i = 0; i < D / 32; ++i) {
                const int k = 8 * (4 * i + (tid & 3));
                *(bf16x8 *)(As + (k >> 6) * 4096 + tile_off(tid >> 2, (k & 63) >> 3)) = pv[i];
            }
            if (tid < D) bp_s[tid] = bpv;
        }
        ln_gb_store<KT>(gb2v, gb2_s, tid);
        if (HAS_QKV) {
            ln_gb_store<KT>(gbqv, gbq_s, tid);
#pragma unroll
            for (int j = 0; j < (LY_MAX_NQ + 255) / 256; ++j)
                if (tid + 256 * j < Nq) bq_s[tid + 256 * j] = bqv[j];
        }
#pragma unroll
        for (int j = 0; j < LY_MAX_DM / 256; ++j)
            if (tid + 256 * j < Dm) b1_s[tid + 256 * j] = b1v[j];
        if (tid < D) b2_s[tid] = b2v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // B0: o rows, biases, gains are in LDS

    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    const bf16x4 zero4 = {0, 0, 0, 0};
    bf16x8 fa[KT * 4];                           // the resident rows wr*32 + lm as the B operand of the transposed product
    auto load_fa = [&]() {
#pragma unroll
        for (int kk = 0; kk < KT * 4; ++kk)
            fa[kk] = *(const bf16x8 *)(As + (kk >> 2) * 4096 + tile_off(wr * 32 + lm, 2 * (kk & 3) + lh));
    };
    // shrink: c[n][m] = sum_k At[n][k] x[m][k] with At_k from at_s; lane (lm, lh) ends up with ranks 4*lh + {0..3} (c[0..3])
    // and 8 + 4*lh + {0..3} (c[4..7]) of row lm -- exactly the 8 contraction slots it must supply to the expand
    auto shrink = [&](int r) {
        f32x16 c;
#pragma unroll
        for (int e = 0; e < 16; ++e) c[e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KT * 4; ++kk) {
            const bf16x8 ft = lm < r ? *(const bf16x8 *)(at_s + min(lm, 15) * LY_AT_STRIDE + kk * 16 + lh * 8) : zero8;
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ft, fa[kk], c, 0, 0, 0);
        }
        bf16x8 fs;
#pragma unroll
        for (int j = 0; j < 8; ++j) fs[j] = (bf16_t)(a.scale * c[j]);
        return fs;
    };
    // expand operand of output column n from Bt_k (in As): ranks 4*lh + {0..3} and 8 + 4*lh + {0..3}; r is a multiple of 4:
    // each half is one 8-byte read at a clamped offset, zeroed where the rank does not exist
    auto bt_frag = [&](int n, int r) {
        const bool lo_ok = 4 * lh + 4 <= r, hi_ok = 8 + 4 * lh + 4 <= r;
        const bf16_t *bt = As + (size_t)n * r;
        const bf16x4 lo = lo_ok ? *(const bf16x4 *)(bt + 4 * lh) : zero4, hi = hi_ok ? *(const bf16x4 *)(bt + 8 + 4 * lh) : zero4;
        return bf16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    };
    // one or two chunks of a plain linear against the resident rows: acc starts from the bias; operands are fetched one
    // K step (16) ahead of the MFMAs that use them (LDS latency is a hundred-odd cycles, and the compiler on its own
    // keeps only two or three reads in flight)
    auto linear_step = [&](f32x16 &acc0, f32x16 &acc1, int c0, int pos0, int N, const float *bias_s, auto PAIR) {
        constexpr bool pair = decltype(PAIR)::value;
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const bf16_t *st0 = Ws + (pos0 % LY_NS) * IT_EL, *st1 = Ws + ((pos0 + 1) % LY_NS) * IT_EL;
        bf16x8 fw0[2][KT], fw1[2][KT];
        auto load = [&](int kk, int sl) {
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                fw0[sl][kt] = *(const bf16x8 *)(st0 + kt * 4096 + tile_off(wc * 32 + lm, 2 * kk + lh));
                if (pair) fw1[sl][kt] = *(const bf16x8 *)(st1 + kt * 4096 + tile_off(wc * 32 + lm, 2 * kk + lh));
            }
        };
        load(0, 0);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 b0 = *(const f32x4 *)(bias_s + min(c0 * 64 + wc * 32 + 8 * g + 4 * lh, N - 4));
#pragma unroll
            for (int z = 0; z < 4; ++z) acc0[4 * g + z] = b0[z];
            if (pair) {
                const f32x4 b1 = *(const f32x4 *)(bias_s + min((c0 + 1) * 64 + wc * 32 + 8 * g + 4 * lh, N - 4));
#pragma unroll
                for (int z = 0; z < 4; ++z) acc1[4 * g + z] = b1[z];
            }
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) load(kk + 1, (kk + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw0[kk & 1][kt], fa[kt * 4 + kk], acc0, 0, 0, 0);
                if (pair) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw1[kk & 1][kt], fa[kt * 4 + kk], acc1, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    char *xtile = (char *)Ws;                    // the fp32 hand-over tile: ring stages 0-2
    // loaders: xr += the tile (the product that the other waves staged)
    auto add_tile = [&]() {
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int i = 0; i < KT; ++i) xr[k * KT + i] += *(const f32x4 *)(xtile + (xslot + 16 * k) * XSTRIDE + (xpart + 16 * i) * 16);
    };
    // loaders: the rows in xr -> LayerNorm (fp32 statistics, centred second moment) -> bf16 tiles at As, gains from gb_s
    auto ln_rows = [&](const float *gb_s) {
        f32x4 gn[KT], sh[KT];
#pragma unroll
        for (int i = 0; i < KT; ++i) { gn[i] = *(const f32x4 *)(gb_s + 4 * (xpart + 16 * i)); sh[i] = *(const f32x4 *)(gb_s + D + 4 * (xpart + 16 * i)); }
        float mean[4], inv[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < KT; ++i) t += xr[k * KT + i][0] + xr[k * KT + i][1] + xr[k * KT + i][2] + xr[k * KT + i][3];
            mean[k] = row16_sum(t) * (1.0f / D);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float q = 0.f;
#pragma unroll
            for (int i = 0; i < KT; ++i)
#pragma unroll
                for (int z = 0; z < 4; ++z) { const float d = xr[k * KT + i][z] - mean[k]; q = fmaf(d, d, q); }
            inv[k] = rsqrtf(row16_sum(q) * (1.0f / D) + a.eps);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float nmi = -mean[k] * inv[k];
            const int row = xslot + 16 * k;
#pragma unroll
            for (int i = 0; i < KT; ++i) {
                const int col = 4 * (xpart + 16 * i);         // first of this piece's 4 elements
                bf16x4 o;
#pragma unroll
                for (int z = 0; z < 4; ++z) o[z] = (bf16_t)fmaf(fmaf(xr[k * KT + i][z], inv[k], nmi), gn[i][z], sh[i][z]);   // ((x - mean) inv) g + b
                *(bf16x4 *)(As + (col >> 6) * 4096 + tile_off(row, (col & 63) >> 3) + (col & 4)) = o;
            }
        }
    };

    // ================================================================ phase A: x' = res + o Wp + bp + lora
    if (HAS_PROJ) {
        constexpr int SA = (KT + 1) / 2;
        if (loader) {
            // (the ring is refilled after each step's barrier, never before it: a loader that is still issuing -- it is held
            // at the issue stage while the L2 path is busy -- would keep every wave waiting at that barrier)
            for (int s = 0; s < SA; ++s) {
                wait_item(min(2 * s + 1, KT - 1));
                if (s == 0 && lora_p) issue_bt(a.Bpt + (size_t)k_ad * D * a.r, D, a.r);     // the computing waves hold their fragments by now
                refill(2 * s - 1, 1 << 20);
                if (s == 0) issue_next();                                           // W1's first rows: stage 3 is free all through A
            }
            wait_item(NA - 1);                                                  // Bf: Bt_k has landed (it is older than the items still in flight)
            asm volatile("s_barrier" ::: "memory");                             // Bs: the tile is complete
            add_tile();
            ln_rows(gb2_s);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");     // Bl: LayerNorm2(x') is in As, the tile is dead
        } else {
            load_fa();
            f32x16 accp[KT + 1];
#pragma unroll
            for (int s = 0; s < SA; ++s) {
                if (2 * s + 1 < KT) linear_step(accp[2 * s], accp[2 * s + 1], 2 * s, 2 * s, D, bp_s, std::true_type{});
                else linear_step(accp[2 * s], accp[2 * s], 2 * s, 2 * s, D, bp_s, std::false_type{});
            }
            bf16x8 fs = zero8;
            if (lora_p) fs = shrink(a.r);                                       // At_k landed before the first chunk did
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");     // Bf
            if (lora_p) {
#pragma unroll
                for (int c = 0; c < KT; ++c) accp[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bt_frag(c * 64 + wc * 32 + lm, a.r), fs, accp[c], 0, 0, 0);
            }
            // the ring positions 0 .. KT - 1 are consumed: the tile takes stages 0-2
            char *trow = xtile + (wr * 32 + lm) * XSTRIDE + (wc * 32 + 4 * lh) * 4;
#pragma unroll
            for (int c = 0; c < KT; ++c)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *(f32x4 *)(trow + (c * 64 + 8 * g) * 4) = f32x4{accp[c][4 * g], accp[c][4 * g + 1], accp[c][4 * g + 2], accp[c][4 * g + 3]};
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");     // Bs
            asm volatile("s_barrier" ::: "memory");                             // Bl
        }
    } else {
        if (loader) {
            ln_rows(gb2_s);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");     // Bl: LayerNorm2(x') is in As
        } else {
            asm volatile("s_barrier" ::: "memory");                             // Bl
        }
    }

    // ================================================================ phase B: y = GELU(LayerNorm2(x') W1 + b1) W2
    // Step h (0 .. nch + 1), one barrier each:
    //   waves 0-3: hb[h & 1] = LayerNorm2(x') W1 rows of chunk h; hidden tile of chunk h - 1 = GELU(hb[(h - 1) & 1] + b1),
    //              a quarter of the GELU's arithmetic between the MFMAs of each K step;
    //   waves 5-7: y += hidden(chunk h - 2) W2 slice;   wave 4: the stream.
    bf16_t *Hs = As;                             // hidden tiles [64 rows][64 columns of a chunk], chunk c in tile c & 1 (As is dead
                                                 // once every wave has its fa: the barrier of step 0 comes before the first write)
    using T_ = std::true_type;
    using F_ = std::false_type;
    if (loader) {
        const int j = wave - 5;                  // waves 5-7: output columns 64 j .. 64 j + 63, rows rt*32 + lm, as y[rt][ct]
        const bool second = j >= 0 && j < KT;
        f32x16 y[2][2];
        if (second) {
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f32x4 b = *(const f32x4 *)(b2_s + 64 * j + ct * 32 + 8 * g4 + 4 * lh);   // the accumulators start from b2
#pragma unroll
                    for (int z = 0; z < 4; ++z) y[0][ct][4 * g4 + z] = y[1][ct][4 * g4 + z] = b[z];
                }
        }
        // this wave's tile of W2's slice c (output columns 64 j .., hidden columns 64 c ..) -> its 8 KB of stage 4
        bf16_t *w2_s = Ws + 4 * IT_EL + (second ? j : 0) * 4096;
        auto issue_w2 = [&](int c) {
            const unsigned rb = Dm * 2;
            const unsigned e0 = lr * rb + ((((lane & 7) ^ (lr >> 1))) << 4), e1 = lr * rb + ((((lane & 7) ^ (4 + (lr >> 1)))) << 4);
            glds16_tile8(a.W2t + (size_t)j * 64 * Dm + (size_t)c * 64, __builtin_amdgcn_readfirstlane(lds_addr_of(w2_s)), e0, e1 + 8 * rb,
                         e0 + 16 * rb, e1 + 24 * rb, e0 + 32 * rb, e1 + 40 * rb, e0 + 48 * rb, e1 + 56 * rb);
        };
        for (int h = 0; h < nch + 2; ++h) {
            // wave 4: W1(h) has landed (later chunks may be in flight).  Waves 5-7 keep their own loads in flight across the
            // barrier and wait for them below.
            if (wave == 4) wait_item(NA + min(h, nch - 1));
            else asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (h == 0) gelu_tab_build(gelu_s, lt, 256);   // every computing wave holds its fragments of LayerNorm2(x') by now; first used in step 1
            // At_k of the qkv linear: at_s is idle since the shrink of phase A, and a request made here does not queue up
            // behind the first chunks of C
            if (h == 1 && lora_q) issue_at(a.Aqt + (size_t)k_ad * a.r * D, a.r);
            // the stream of W1: chunks 1-3 into stages 0-2 once the hand-over tile is dead, then chunk h + 3 into the stage
            // that chunk h - 1 has left; the first chunk of C once W1 is through (stage 3; the second one needs stage 4)
            if (h == 0) { while (last + 1 < NA + min(nch, 4)) issue_next(); }
            else if (last + 1 < NA + nch) issue_next();
            else if (HAS_QKV && h == nch && last + 1 == NA + nch) issue_next();
            if (second && h == 0) issue_w2(0);
            if (second && h >= 2) {
                // The slice of W2 does not pass through the shared ring: this wave's tile of it landed in its own 8 KB (requested
                // one step ago), is copied into registers, and the next slice is requested into the same place at once.
                const bf16_t *Hr = Hs + (h & 1) * 4096;                                                            // chunk h - 2
                bf16x8 fh[2][2], f2[4][2];
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                    for (int t = 0; t < 2; ++t) f2[kk][t] = *(const bf16x8 *)(w2_s + tile_off(t * 32 + lm, 2 * kk + lh));
                auto load = [&](int kk, int s) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) fh[s][t] = *(const bf16x8 *)(Hr + tile_off(t * 32 + lm, 2 * kk + lh));
                };
                load(0, 0);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (h - 1 < nch) issue_w2(h - 1);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    if (kk < 3) load(kk + 1, (kk + 1) & 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                        for (int ct = 0; ct < 2; ++ct)
                            y[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[kk][ct], fh[kk & 1][rt], y[rt][ct], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        wait_item(NA + nch - 1);                                                // Be: every chunk and slice of B is consumed
        refill(HAS_QKV ? PC - 1 : 0, HAS_QKV ? PC + 1 : -1);                    // (the tile still needs stages 0-2)
        if (second) {
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                char *trow = xtile + (rt * 32 + lm) * XSTRIDE + (64 * j + 4 * lh) * 4;
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4)
                        *(f32x4 *)(trow + (ct * 32 + 8 * g4) * 4) = f32x4{y[rt][ct][4 * g4], y[rt][ct][4 * g4 + 1], y[rt][ct][4 * g4 + 2], y[rt][ct][4 * g4 + 3]};
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");         // By: the y tile is complete
        add_tile();                                                             // x'' = x' + y
        if (HAS_QKV) {
            // Bt: the tile is dead.  Chunks 2-4 of C (stages 0-2) are requested now, by a computing wave: requested by a
            // loader after its stores of x'', they would queue up behind those and arrive three thousand cycles into C.
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            last = max(last, NA + nch + min(nchq, 5) - 1);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int row = xslot + 16 * k;
            if (row < rows) {
                float *dst = a.x_out + ((size_t)ob * a.T + t0 + row) * D + 4 * xpart;
#pragma unroll
                for (int i = 0; i < KT; ++i) *(f32x4 *)(dst + 64 * i) = xr[k * KT + i];
            }
        }
        if (HAS_QKV) ln_rows(gbq_s);
    } else {
        load_fa();
        f32x16 hb[2];                            // first product of chunks h / h - 1: row lm, columns wc*32 + 8*(e/4) + 4*lh + e%4
        auto first_step = [&](auto D1, auto DG, auto PAR, int h) {
            constexpr bool d1 = decltype(D1)::value, dg = decltype(DG)::value;
            constexpr int par = decltype(PAR)::value ? 1 : 0;          // h & 1
            f32x16 &hout = hb[par], &hin = hb[par ^ 1];
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const bf16_t *s1 = Ws + ((SB0 + h) & 3) * IT_EL;                                        // W1(h)
            bf16_t *Hw = Hs + ((h - 1) & 1) * 4096;                                                  // chunk h - 1
            bf16x8 f1[2][KT];
            f32x4 b[4];
            auto load = [&](int kk, int s) {
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) f1[s][kt] = *(const bf16x8 *)(s1 + kt * 4096 + tile_off(wc * 32 + lm, 2 * kk + lh));
            };
            if (dg) {
                const float *bp = b1_s + (h - 1) * 64 + wc * 32 + 4 * lh;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) b[g4] = *(const f32x4 *)(bp + 8 * g4);
            }
            if (d1) load(0, 0);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                if (d1 && kk < 3) load(kk + 1, (kk + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                if (d1) {
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt) {
                        const f32x16 z16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        hout = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[kk & 1][kt], fa[kt * 4 + kk], kk == 0 && kt == 0 ? z16 : hout, 0, 0, 0);
                    }
                }
                if (dg) {
                    // a quarter of the chunk's GELU per K step, through the Phi table (fewer instructions than the polynomial)
                    const f32x4 v = gelu_tab4(f32x4{hin[4 * kk], hin[4 * kk + 1], hin[4 * kk + 2], hin[4 * kk + 3]} + b[kk], gelu_s);
                    const bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                    *(bf16x4 *)(Hw + tile_off(wr * 32 + lm, 4 * wc + kk) + 4 * lh) = o;
                }
                if (d1 && dg) {
                    // one MFMA, then a share of the vector work, so that the vector work is issued while an MFMA runs
#pragma unroll
                    for (int i = 0; i < KT; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, (40 + KT - 1) / KT, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        first_step(T_{}, F_{}, F_{}, 0);
        for (int h = 1; h < nch; ++h) {
            if (h & 1) first_step(T_{}, T_{}, T_{}, h);
            else first_step(T_{}, T_{}, F_{}, h);
        }
        if (nch & 1) first_step(F_{}, T_{}, T_{}, nch);
        else first_step(F_{}, T_{}, F_{}, nch);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");         // step nch + 1: the other waves' last product
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");         // Be: the ring positions of B are consumed
        asm volatile("s_barrier" ::: "memory");                                 // By
        if (HAS_QKV) {
            asm volatile("s_barrier" ::: "memory");                             // Bt
            if (wave == 0)
                for (int c = 2; c < min(nchq, 5); ++c) issue_item(NA + nch + c);
        }
    }
    if (!HAS_QKV) return;

    // ================================================================ phase C: qkv = LayerNorm1'(x'') Wq + bq + lora
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");             // Bz: LayerNorm1'(x'') is in As, the tile is dead
    f32x16 acc[LY_MAXCH + 1];                    // acc[c][e]: row wr*32 + lm, column c*64 + wc*32 + 8*(e/4) + 4*lh + e%4
    const int i0q = NA + nch;                    // first item of C
    if (loader) {
        for (int s = 0; 2 * s < nchq; ++s) {
            if (s == 0 && wave == 4) {
                // The first two chunks of C were requested by this wave before it stored its rows of x''; chunks 2-4 are wave 0's
                // (`last` counts them, so wait_item would let two items' worth of this wave's requests stay in flight and
                // guarantee nothing about chunk 1).  What may stay in flight is exactly the stores: KT per group of 16 rows
                // that has a row of this wave's inside the tile -- the stores that are issued whatever the compiler does with
                // the others.
                switch (min(4, (rows + 15) >> 4)) {
                case 4: rl_wait_barrier<4 * KT>(); break;
                case 3: rl_wait_barrier<3 * KT>(); break;
                case 2: rl_wait_barrier<2 * KT>(); break;
                default: rl_wait_barrier<KT>(); break;
                }
            } else {
                wait_item(i0q + min(2 * s + 1, nchq - 1));
            }
            if (s == 0 && lora_q) issue_bt(a.Bqt + (size_t)k_ad * Nq * a.r, Nq, a.r);   // the computing waves hold their fragments by now
            refill(PC + 2 * s - 1, 1 << 30);
        }
        rl_wait_barrier<0>();                                                   // Bf2: Bt_k has landed; the ring is dead
        asm volatile("s_barrier" ::: "memory");                                 // Bg2: expand done, Bt_k is dead
    } else {
        load_fa();
        // the shrink first (At_k has been in LDS since phase B): these waves would only wait for the first chunks otherwise
        bf16x8 fs = zero8;
        if (lora_q) fs = shrink(a.r);
#pragma unroll
        for (int s = 0; s < (LY_MAXCH + 1) / 2; ++s) {
            // chunks 2-4 were requested by wave 0: it waits for its own loads (the other waves have none in flight)
            if (s == 1) {
                if (nchq >= 5) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NLD) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            if (s == 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            // uniform conditions, written as guards (not a break) so that the loop unrolls and acc stays in registers
            if (2 * s + 1 < nchq) linear_step(acc[2 * s], acc[2 * s + 1], 2 * s, PC + 2 * s, Nq, bq_s, std::true_type{});
            else if (2 * s < nchq) linear_step(acc[2 * s], acc[2 * s], 2 * s, PC + 2 * s, Nq, bq_s, std::false_type{});
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");         // Bf2
        if (lora_q) {
            // all operands first, then the MFMAs (one read-then-multiply per chunk would pay the LDS latency nine times)
            bf16x8 fbt[LY_MAXCH];
#pragma unroll
            for (int c = 0; c < LY_MAXCH; ++c) fbt[c] = bt_frag(min(c * 64 + wc * 32 + lm, Nq - 1), a.r);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < LY_MAXCH; ++c)
                if (c < nchq) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fbt[c], fs, acc[c], 0, 0, 0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");         // Bg2
        // A lane owns one row, so storing from registers would touch 32 cache lines per instruction with 8 bytes each:
        // the finished bf16 tile is laid out row-major in LDS and copied out in 16-byte pieces of consecutive threads
        const int qstride = ((Nq * 2 + 255) & ~255) + 16;
        // A lane holds columns 8 g + 4 lh + {0..3} of its row; the two lanes of a row trade halves (lane < 32 gives its piece of
        // group g + 1 for the other's piece of group g) so that each ends up with eight consecutive columns: half as many
        // LDS writes, 16 bytes each (a wave's LDS writes cost the same whatever their width).  Nq is a multiple of 64.
        char *trow = (char *)lds + (wr * 32 + lm) * qstride + (wc * 32 + 8 * lh) * 2;
#pragma unroll
        for (int c = 0; c < LY_MAXCH; ++c) {
            if (c < nchq) {
#pragma unroll
                for (int g = 0; g < 4; g += 2) {
                    const bf16x4 w0 = {(bf16_t)acc[c][4 * g], (bf16_t)acc[c][4 * g + 1], (bf16_t)acc[c][4 * g + 2], (bf16_t)acc[c][4 * g + 3]};
                    const bf16x4 w1 = {(bf16_t)acc[c][4 * g + 4], (bf16_t)acc[c][4 * g + 5], (bf16_t)acc[c][4 * g + 6], (bf16_t)acc[c][4 * g + 7]};
                    *(u32x4 *)(trow + (c * 64 + 8 * g) * 2) = pair_halves(w0, w1);
                }
            }
        }
    }
    __syncthreads();
    {
        const int qstride = ((Nq * 2 + 255) & ~255) + 16, pieces = (Nq * 2) >> 4;
        char *out = (char *)a.qkv_out + ((size_t)ob * a.T + t0) * Nq * 2;
        for (int idx = tid; idx < rows * pieces; idx += LY_THREADS) {
            const int row = idx / pieces, p = idx - row * pieces;
            *(f32x4 *)(out + (size_t)row * Nq * 2 + p * 16) = *(const f32x4 *)((const char *)lds + row * qstride + p * 16);
        }
    }
}

template <int KT, bool HAS_PROJ, bool HAS_QKV> int launch_layer_t(const RowLayerArgs &a, hipStream_t st)
{
    constexpr int D = 64 * KT;
    constexpr int LDS = ((KT < 2 ? 2 : KT) + LY_NS * KT) * 64 * 64 * 2 + (LY_MAX_DM + LY_MAX_NQ + 2 * D + 4 * D) * 4 + 16 * LY_AT_STRIDE * 2 + (KT == 3 ? 0 : GELU_TAB_ENTRIES * 8);
    static_assert(LDS <= 160 * 1024, "LDS budget");
    auto kern = rowlayer_kernel<KT, HAS_PROJ, HAS_QKV>;
    if (LDS > 64 * 1024) {
        static bool attr_set = false;   // raising the dynamic LDS limit is a per-kernel, process-wide setting
        if (!attr_set) {
            if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS) != hipSuccess) return POLY_EHIP;
            attr_set = true;
        }
    }
    const int tiles = (a.T + 63) / 64;
    POLY_LAUNCH_SHMEM(POLY_STAGE_GEMM, kern, dim3((unsigned)(a.n_out * tiles)), dim3(LY_THREADS), LDS, st, a);
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}

template <int KT> int launch_layer_kt(const RowLayerArgs &a, hipStream_t st)
{
    const bool p = a.o != nullptr, q = a.qkv_out != nullptr;
    if (p && q) return launch_layer_t<KT, true, true>(a, st);
    if (p) return launch_layer_t<KT, true, false>(a, st);
    if (q) return launch_layer_t<KT, false, true>(a, st);
    return launch_layer_t<KT, false, false>(a, st);
}

}  // namespace

// D, Dm: model and hidden width; r: adapter rank of the proj / qkv linears that carry adapters (0 = none)
bool rowlayer_supported(int D, int Dm, int r)
{
    if (!((D == 64 || D == 128 || D == 192) && Dm >= 128 && Dm % 64 == 0 && Dm <= LY_MAX_DM)) return false;
    if (r != 0 && !(r >= 4 && r <= 16 && r % 4 == 0)) return false;
    // Bt_k of the qkv linear [3 D][r] takes the place of the activation rows
    return (long)3 * D * r * 2 <= (long)(D / 64 < 2 ? 2 : D / 64) * 64 * 64 * 2;
}

int launch_rowlayer(const RowLayerArgs &a, hipStream_t st)
{
    if (a.n_out <= 0 || a.T <= 0) return POLY_OK;
    const bool lora = (a.o && a.Apt) || (a.qkv_out && a.Aqt);
    if (!rowlayer_supported(a.D, a.Dm, lora ? a.r : 0)) return POLY_EINVAL;
    switch (a.D / 64) {
    case 1: return launch_layer_kt<1>(a, st);
    case 2: return launch_layer_kt<2>(a, st);
    default: return launch_layer_kt<3>(a, st);
    }
}
