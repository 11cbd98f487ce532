// Block-structured linear  y = x W + b  (+ s (x A_k) B_k)  with fused epilogues (Sec. 3.1).
//
// bf16: 128 x BN x 32 tiles, 4 waves in a 2 x 2 grid, v_mfma_f32_32x32x16_bf16, fp32 accumulators.
// The low-rank expand (x A_k) B_k is one more K step of the same MFMA per 16 ranks, fed with the
// shrink output S and the adapter's Bt slab, so W + A_k B_k is never formed and the base product of
// an input block is shared by all the row-blocks that fan out of it.
// fp32: 64 x 64 x 16 tiles on the vector ALUs (reference-precision path).
#include "poly_dev.h"

#include <stdlib.h>

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
__device__ __forceinline__ bool decode_tile(const GemmArgs &g, int id, int BM, int BN, int &xb, int &t0, int &n0, int &ob0, int &ob1)
{
    const int tiles_n = (g.N + BN - 1) / BN, tiles_m = (g.T + BM - 1) / BM;
    const int tn = id % tiles_n; id /= tiles_n;
    const int tm = id % tiles_m; xb = id / tiles_m;
    const int n_in = g.n_in_dev ? min(*g.n_in_dev, g.n_in) : g.n_in;
    if (xb >= n_in) return false;
    ob0 = xb; ob1 = xb + 1;
    if (g.out_off) { ob0 = g.out_off[xb]; ob1 = g.out_off[xb + 1]; }
    t0 = tm * BM; n0 = tn * BN;
    return ob0 < ob1;
}

// ------------------------------------------------------------------ bf16 MFMA, any K % 8 == 0 and any N

template <int BN>
__global__ __launch_bounds__(256) void gemm_bf16_generic_kernel(const GemmArgs g)
{
    constexpr int BM = 128, BK = 32, LS = BK + 8;  // LDS row stride in elements (80 B, 16-byte aligned)
    constexpr int NJ = BN / 64;                     // 32-wide column subtiles per wave
    __shared__ __attribute__((aligned(16))) bf16_t As[BM * LS];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * LS];

    int xb, t0, n0, ob0, ob1;
    if (!decode_tile(g, blockIdx.x, BM, BN, xb, t0, n0, ob0, ob1)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

        const bool has_lora = g.S && g.adapter_of_out;
        const int sb0 = g.set_off ? g.set_off[ob] : ob, sb1 = g.set_off ? g.set_off[ob + 1] : ob + 1;
        for (int sb = sb0; has_lora && sb < sb1; ++sb) {
            const int k_ad = g.adapter_of_out[sb];
            if (k_ad < 0) continue;
            // expand: one more K step per 16 ranks; A operand = S rows, B operand = Bt_k rows
            const bf16_t *S = (const bf16_t *)g.S + (size_t)sb * g.T * g.RP;
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

// ------------------------------------------------------------------ bf16 MFMA, K % 64 == 0 and N % 8 == 0
// 128 x BN x 64 tiles, 4 waves in a 2 x 2 grid, v_mfma_f32_32x32x16_bf16.
//
// Loads: global_load_lds_dwordx4 -- each wave instruction drops 64 x 16 bytes (8 tile rows of 64 elements)
// straight into LDS, so NS - 1 k-tiles are in flight per workgroup without costing registers.  The lane that
// fills position p of row r fetches chunk p ^ ((r >> 1) & 7): a swizzle that keeps 16-byte reads free of bank
// conflicts for 8 or 16 lanes per LDS cycle, without padding.  Waits are counted by hand (vmcnt = loads of
// the k-tiles still allowed in flight) and the barrier is a bare s_barrier, because a fenced barrier would
// drain every outstanding load.
//
// The product is accumulated transposed (Wt fragment as the A operand) so that a lane ends up with four
// consecutive output columns of one row; the epilogue adds the low-rank expand as one more MFMA K step per
// 16 ranks, stages fp32 rows through LDS with 16-byte writes and stores whole 128/256-byte row segments,
// adding bias, residual and position rows with vector loads.
//
// Tile order: workgroup ids are dealt round-robin to the 8 XCDs, so id % 8 picks the XCD.  The tiles, ordered by panel of
// PANEL column tiles, then row tile, then column tile, are cut into eight equal runs, one per XCD: an XCD works on one
// W panel at a time (it stays in that XCD's 4 MB L2 instead of all of W streaming past every row tile) and the XCDs
// finish together (a ninth of a round more on one XCD is a whole round more for the kernel).
#define POLY_GLDS16(gptr, lptr)                                                                          \
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)(gptr),           \
                                     (void __attribute__((address_space(3))) *)(lptr), 16, 0, 0)

template <int N> __device__ __forceinline__ void wait_vm_and_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// (row tile, column tile) of workgroup `bid`; false if this workgroup has nothing to do.  All tiles in the order (panel of
// `panel` column tiles, row tile, column tile inside the panel) are cut into eight equal runs, one per XCD: a run covers one
// or two W panels and a contiguous range of row tiles, and no XCD has more than one tile more than another.
__device__ __forceinline__ bool xcd_tile(int bid, int tiles_mtot, int tiles_n, int panel, int &mt, int &tn)
{
    const int xcd = bid & 7, j = bid >> 3;
    const long total = (long)tiles_mtot * tiles_n;
    const long lo = total * xcd / 8, hi = total * (xcd + 1) / 8;
    const long L = lo + j;
    if (L >= hi) return false;
    const long full = (long)tiles_mtot * panel;            // tiles per full panel
    const int pn = (int)(L / full);
    const int rem = (int)(L - pn * full);
    const int n_lo = pn * panel;
    const int width = min(panel, tiles_n - n_lo);
    mt = rem / width;
    tn = n_lo + rem - mt * width;
    return true;
}

// BM x BN tile, WM x WN waves, each wave (BM/WM) x (BN/WN) = (MI*32) x (NJ*32); NS LDS stages of 64 k-columns.
// EK, the epilogue: 0 = subtile by subtile (fp32 output with residual / position rows, or one column subtile per wave);
// 1, 2 = row-wise for bf16 output (two column subtiles per wave): 2 when the host knows that a wave's region touches at most two
// input blocks and every output block has one low-rank term of at most 16 ranks (all operands of a pass prefetched), 1 otherwise;
// 3 = the same conditions and prefetching as 2 for fp32 output with a residual (no position rows), staged 32 rows at a time.
template <int BM, int BN, int WM, int WN, int NS, int EK>
__global__ __launch_bounds__(64 * WM * WN, (BM * BN >= 256 * 256 || NS * (BM + BN) * 128 > 80 * 1024) ? 1 : 2)
void gemm_bf16_dma_kernel(const GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int BK = 64, NW = WM * WN;
    constexpr int MI = BM / WM / 32, NJ = BN / WN / 32;   // 32 x 32 subtiles per wave
    constexpr int A_EL = BM * BK, B_EL = BN * BK, STAGE_EL = A_EL + B_EL;
    constexpr int NC = NJ * 8;                             // 16-byte chunks per staged fp32 row (NJ*32 columns)
    constexpr int AG = BM / 8 / NW, BG = BN / 8 / NW;      // 8-row groups (1 KB each) per wave and stage
    constexpr int NLD = AG + BG;                           // loads per wave and stage
    constexpr int PANEL = 768 / BN;                        // column tiles per L2 panel (1.2 MB of W at K = 768)
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0 && (NS - 1) * NLD <= 63, "tile / wave layout");
    static_assert(NW * 32 * NC * 16 <= NS * STAGE_EL * 2, "staging must fit in the tile ring");
    extern __shared__ __attribute__((aligned(16))) bf16_t dsmem[];

    int mt, tn;
    if (!xcd_tile(blockIdx.x, g.n_in * tiles_m, tiles_n, PANEL, mt, tn)) return;
    const int xb = mt / tiles_m, t0 = (mt - xb * tiles_m) * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN, lm = lane & 31, lh = lane >> 5;
    const bf16_t *A = (const bf16_t *)g.A + (size_t)xb * g.T * g.K;
    const bf16_t *Wt = (const bf16_t *)g.Wt;

    // rows past the end of the block / of W are clamped: their products land in accumulator rows / columns that
    // are never stored
    const int lr = lane >> 3;   // row inside an 8-row group; lane & 7 = position inside the row
    int ga[AG], gb[BG];
#pragma unroll
    for (int i = 0; i < AG; ++i) {
        const int row = (wave * AG + i) * 8 + lr;
        ga[i] = min(t0 + row, g.T - 1) * g.K + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
    }
#pragma unroll
    for (int i = 0; i < BG; ++i) {
        const int row = (wave * BG + i) * 8 + lr;
        gb[i] = min(n0 + row, g.N - 1) * g.K + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
    }
    auto issue = [&](int kt, int s) {
        bf16_t *st = dsmem + s * STAGE_EL;
#pragma unroll
        for (int i = 0; i < AG; ++i) POLY_GLDS16(A + ga[i] + kt * BK, st + (wave * AG + i) * 512);
#pragma unroll
        for (int i = 0; i < BG; ++i) POLY_GLDS16(Wt + gb[i] + kt * BK, st + A_EL + (wave * BG + i) * 512);
    };

    auto issue_one = [&](int kt, int s, int l) {            // load l (of NLD) of this wave for k-tile kt into stage s
        bf16_t *st = dsmem + s * STAGE_EL;
#pragma unroll
        for (int i = 0; i < AG; ++i) if (l == i) POLY_GLDS16(A + ga[i] + kt * BK, st + (wave * AG + i) * 512);
#pragma unroll
        for (int i = 0; i < BG; ++i) if (l == AG + i) POLY_GLDS16(Wt + gb[i] + kt * BK, st + A_EL + (wave * BG + i) * 512);
    };

    // Row-wise epilogue (two column subtiles per wave, bf16 output): the accumulators start from the bias, so no output block
    // has to add it later.  These loads go out before the tile loads: the in-order load counter then never makes their first
    // use wait for a tile.
    constexpr bool RW = EK > 0;
    static_assert(!RW || NJ == 2, "row-wise epilogue: two column subtiles per wave");
    constexpr bool rowwise = RW;
    f32x4 bias_q[NJ][4];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int bcol = n0 + wn * NJ * 32 + j * 32 + 8 * q + 4 * lh;
            const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
            bias_q[j][q] = (rowwise && g.bias && bcol < g.N) ? *(const f32x4 *)(g.bias + bcol) : z4;
        }

    // The tile loads need nothing but the tile coordinates, so they go out first; the row count, the fan-out
    // offsets and the adapter id are read while they fly.  A tile that turns out to be past the true row count
    // still read inside the caller's buffers (sized for the row bound); it drains its loads and leaves.
    const int nk = g.K / BK;
    const int npro = min(NS, nk);
    for (int s = 0; s < npro; ++s) issue(s, s);
    const bool flat = g.Tb > 0;                            // one run of rows over all blocks: xb = 0, t0 = first row of the tile
    const int n_in = flat ? 1 : (g.n_in_dev ? min(*g.n_in_dev, g.n_in) : g.n_in);
    const int Tlim = flat ? (g.n_in_dev ? min(*g.n_in_dev, g.nb) : g.nb) * g.Tb : g.T;   // rows that exist
    int ob0 = xb, ob1 = xb + 1;
    if (g.out_off && !flat && xb < n_in) { ob0 = g.out_off[xb]; ob1 = g.out_off[xb + 1]; }
    if (xb >= n_in || ob0 >= ob1 || t0 >= Tlim) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = bias_q[j][e >> 2][e & 3];

    // operands of the low-rank expand for ranks [s0, s0 + 16) of output block ob: S rows of this wave's MI row
    // subtiles and Bt rows of its NJ column subtiles (rows past T / columns past N are clamped or zero: they only
    // feed results that are never stored)
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    auto load_fs = [&](bf16x8(&fs)[MI], int ob, int s0) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int t = min(t0 + wm * MI * 32 + i * 32 + lm, g.T - 1);
            fs[i] = *(const bf16x8 *)((const bf16_t *)g.S + ((size_t)ob * g.T + t) * g.RP + s0 + lh * 8);
        }
    };
    auto load_fw = [&](bf16x8(&fw)[NJ], int k_ad, int s0) {
        const bf16_t *Bt = (const bf16_t *)g.Bt + (size_t)k_ad * g.N * g.r;
        const int j0 = s0 + lh * 8;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int bcol = n0 + wn * NJ * 32 + j * 32 + lm;
            bf16x8 f = zero8;
            if (bcol < g.N) {
                const bf16_t *p = Bt + (size_t)bcol * g.r + j0;
                if ((g.r & 7) == 0) {
                    if (j0 + 8 <= g.r) f = *(const bf16x8 *)p;
                } else {
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (j0 + q < g.r) f[q] = p[q];
                }
            }
            fw[j] = f;
        }
    };
    // small tiles have registers to spare: fetch the first output block's expand operands now, so that their
    // latency hides behind the main loop.  They are younger than the prologue's tile loads, so the in-order load
    // counter used below can only over-wait (by these few loads), never under-wait.
    constexpr bool EARLY = MI * NJ <= 4;
    const bool has_lora = g.S && g.adapter_of_out;
    bf16x8 fs0[MI], fw0[NJ];
    int k_ad0 = -1;
    if (EARLY && has_lora && !flat && !g.set_off) {
        k_ad0 = g.adapter_of_out[ob0];
        if (k_ad0 >= 0) { load_fs(fs0, ob0, 0); load_fw(fw0, k_ad0, 0); }
    }

    // Row-wise epilogue: which input blocks this wave's (MI * 32)-row region touches, their fan-out and the adapters of the first
    // two passes.  Every one of these is a chain of dependent loads and each link a full memory round trip under load, so the
    // fan-out offsets are requested here, the adapter ids inside the main loop once the offsets have arrived, and nothing is
    // waited for before the loop has run.
    constexpr int RROWS = MI * 32, RCOLS = NJ * 32;
    static_assert(!RW || NW * RROWS * RCOLS <= NS * STAGE_EL, "bf16 staging must fit in the tile ring");
    int R0 = 0, Rend = 0, Tblk = 1, bbA = 0, bbZ = 0, baseA = 0, tB = 0, oA0 = 0, oA1 = 0, oB0 = 0, oB1 = 0, maxfan = 0;
    int oA0v = 0, oA1v = 0, oB0v = 0, oB1v = 0;               // as loaded (per lane, all lanes equal)
    int kA = -1, kB = -1, kAv = -1, kBv = -1, kAnv = -1, kBnv = -1;   // adapters of the current pass; as loaded: current / next pass
    bool two = true, hasB = false;
    if constexpr (RW) {
        R0 = t0 + wm * RROWS; Rend = min(R0 + RROWS, Tlim);
        if (R0 < Rend) {
            Tblk = flat ? g.Tb : g.T;                         // rows of a block: stride of S and of the output blocks
            bbA = flat ? R0 / Tblk : xb; bbZ = flat ? (Rend - 1) / Tblk : xb;
            baseA = flat ? bbA * Tblk : 0; tB = baseA + Tblk;  // first row (tile coordinates) of blocks bbA and bbA + 1
            two = bbZ - bbA <= 1; hasB = bbZ > bbA;
            // fan-out of the region's first and last input block (with more than two blocks: looked up per block in the epilogue)
            oA0v = g.out_off ? g.out_off[bbA] : bbA; oA1v = g.out_off ? g.out_off[bbA + 1] : bbA + 1;
            oB0v = g.out_off ? g.out_off[bbZ] : bbZ; oB1v = g.out_off ? g.out_off[bbZ + 1] : bbZ + 1;
        }
    }
    auto fanout_arrived = [&]() {
        oA0 = __builtin_amdgcn_readfirstlane(oA0v); oA1 = __builtin_amdgcn_readfirstlane(oA1v);
        oB0 = __builtin_amdgcn_readfirstlane(oB0v); oB1 = __builtin_amdgcn_readfirstlane(oB1v);
        maxfan = R0 < Rend ? max(oA1 - oA0, oB1 - oB0) : 0;
    };
    auto request_ids = [&](int pp, int &kav, int &kbv) {       // adapters of pass pp for blocks A and B (-1: nothing to add)
        kav = kbv = -1;
        if (!has_lora || pp >= maxfan) return;
        if (oA0 + pp < oA1) kav = g.adapter_of_out[oA0 + pp];
        if (hasB && oB0 + pp < oB1) kbv = g.adapter_of_out[oB0 + pp];
    };
    const int it_ids = nk > 1 ? 1 : 0;

    // fragment rows are wm*MI*32 + i*32 + lm and wn*NJ*32 + j*32 + lm: (row >> 1) & 7 == (lm >> 1) & 7 for all
    const int fa0 = (wm * MI * 32 + lm) * BK, fb0 = A_EL + (wn * NJ * 32 + lm) * BK, sw = (lm >> 1) & 7;
    for (int it = 0; it < nk; ++it) {
        // k-tiles issued beyond `it` may stay in flight; everything up to `it` must have landed
        const int last_issued = it == 0 ? npro - 1 : min(nk - 1, it + NS - 2);
        const int ahead = last_issued - it;
        if (NS >= 4 && ahead >= 3) wait_vm_and_barrier<(NS >= 4 ? 3 : 0) * NLD>();
        else if (NS >= 3 && ahead == 2) wait_vm_and_barrier<(NS >= 3 ? 2 : 0) * NLD>();
        else if (ahead == 1) wait_vm_and_barrier<NLD>();
        else wait_vm_and_barrier<0>();
        // every wave is past compute(it - 1): its stage can be refilled
        const bool refill = it >= 1 && it + NS - 1 < nk;
        const int rkt = it + NS - 1, rst = (it + NS - 1) % NS;
        if constexpr (EK >= 2) {
            if (it == it_ids) {                               // (younger than every tile load in flight: the counted waits over-wait at most)
                fanout_arrived();
                request_ids(0, kAv, kBv);
                request_ids(1, kAnv, kBnv);
            }
        }
        const bf16_t *cur = dsmem + (it % NS) * STAGE_EL;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int ko = ((2 * kk + lh) ^ sw) << 3;
            bf16x8 fa[MI], fb[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[i] = *(const bf16x8 *)(cur + fa0 + i * 32 * BK + ko);
#pragma unroll
            for (int j = 0; j < NJ; ++j) fb[j] = *(const bf16x8 *)(cur + fb0 + j * 32 * BK + ko);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    // The refill of the stage that was read in the previous step, spread over this step: PER loads per 16
                    // k-columns, one every GAP MFMAs.  Issued as one burst the loads hold the wave at the issue stage until the
                    // L2 path has taken them, and the MFMAs behind them start that much later.
                    constexpr int NM = MI * NJ, PER = (NLD + 3) / 4;
                    constexpr int GAP = NM / PER > 0 ? NM / PER : 1;
                    const int m = i * NJ + j;
                    if (m % GAP == 0 && m / GAP < PER) {
                        const int l = kk * PER + m / GAP;
                        if (l < NLD) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (refill) issue_one(rkt, rst, l);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
                }
        }
    }
    __syncthreads();   // all loads have landed (vmcnt(0) above) and all waves are done with the tiles

    // ---- row-wise epilogue (bf16 output, two column subtiles per wave).  Per pass p the wave produces, for every row of its
    // (MI * 32) x 64 region, the p-th output block of that row's input block: base product (+ bias, in the accumulators) + the
    // low-rank terms of that output block, GELU, rounding to bf16 -- all in accumulator layout -- then the whole region goes through
    // the wave's own LDS area once (8-byte writes, 16-byte reads, chunks swizzled by row & 7) and leaves as 128-byte row segments,
    // eight rows per store instruction.  A 32-row subtile that straddles two input blocks adds each block's term with the
    // other block's S rows zeroed, so block boundaries cost one more MFMA, not one more trip through LDS.
    if constexpr (RW) {
        bf16_t *stg16 = dsmem + wave * (RROWS * RCOLS);
        if (R0 >= Rend) return;
        if constexpr (EK == 1) {
            fanout_arrived();
            if (!two)
                for (int bb = bbA + 1; bb < bbZ; ++bb) maxfan = max(maxfan, g.out_off ? g.out_off[bb + 1] - g.out_off[bb] : 1);
        }
        const bool gelu = g.mode == EPI_GELU;
        const bf16_t *Sg = (const bf16_t *)g.S;
        const int r8 = lane >> 3, ch = lane & 7;
        const int col = n0 + wn * RCOLS + ch * 8;
        const bool col_ok = col < g.N;

        // one column subtile of results (accumulator layout, fp32) -> GELU -> bf16 -> the wave's staging rows [32 i, 32 i + 32)
        auto stage1 = [&](const f32x16 &cj, int i, int j) {
            const int srow = 32 * i + lm;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 v = {cj[4 * q], cj[4 * q + 1], cj[4 * q + 2], cj[4 * q + 3]};
                if (gelu) v = gelu_poly4(v);
                const bf16x4 w = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                *(bf16x4 *)(stg16 + srow * RCOLS + ((((j * 4 + q) ^ (srow & 7)) << 3) + 4 * lh)) = w;
            }
        };
        // rows of pass p: staging -> global, 8 rows x 128 bytes per instruction
        auto store_rows = [&](int p) {
            const int obA = (two && oA0 + p < oA1) ? oA0 + p : -1, obB = (two && hasB && oB0 + p < oB1) ? oB0 + p : -1;
#pragma unroll 2
            for (int q = 0; q < RROWS / 8; ++q) {
                const int row = 8 * q + r8, t = R0 + row;
                int ob, trow;
                if (EK == 2 || two) {
                    const bool inB = t >= tB;
                    ob = inB ? obB : obA;
                    trow = t - (inB ? tB : baseA);
                } else {                                      // more than two input blocks in the region: looked up per row
                    const int bb = min(t, Rend - 1) / Tblk;
                    trow = t - bb * Tblk;
                    const int o0 = g.out_off ? g.out_off[bb] : bb, o1 = g.out_off ? g.out_off[bb + 1] : bb + 1;
                    ob = o0 + p < o1 ? o0 + p : -1;
                }
                if (t >= Rend || ob < 0 || !col_ok) continue;
                const bf16x8 v = *(const bf16x8 *)(stg16 + row * RCOLS + ((ch ^ r8) << 3));
                *(bf16x8 *)((bf16_t *)g.out + ((long)ob * g.Tout + g.t_off + trow) * g.N + col) = v;
            }
        };

        if constexpr (EK >= 2) {
            // The host has checked: a region touches at most two input blocks, one low-rank term per output block, rank 8 or 16
            // in one 16-rank step.  All operands of a pass -- the Bt fragments of the two adapters, one S fragment per subtile and
            // one more for the subtile that straddles the block boundary -- are requested together, those of pass p + 1 before
            // the rows of pass p are stored and the adapter ids of pass p + 2 with them: a pass never waits for more than what
            // is left of one round trip.  (Bt columns past N and ranks past r are read from clamped addresses: the former
            // feed columns that are never stored, the latter meet the zero padding of S.)
            bf16x8 fwA[NJ], fwB[NJ], fs1[MI], fs2 = zero8;
            auto request_operands = [&](int pp, int ka, int kb) {
                const int j0 = min(lh * 8, g.r - 8);
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const size_t bcol = (size_t)min(n0 + wn * RCOLS + j * 32 + lm, g.N - 1);
                    if (ka >= 0) fwA[j] = *(const bf16x8 *)((const bf16_t *)g.Bt + ((size_t)ka * g.N + bcol) * g.r + j0);
                    if (kb >= 0) fwB[j] = *(const bf16x8 *)((const bf16_t *)g.Bt + ((size_t)kb * g.N + bcol) * g.r + j0);
                }
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int tw = R0 + 32 * i;
                    const bool inB = tw >= tB;                    // the subtile's first block
                    if ((inB ? kb : ka) >= 0 && tw < Rend) {
                        const int trow = min(max(tw + lm - (inB ? tB : baseA), 0), Tblk - 1);
                        fs1[i] = *(const bf16x8 *)(Sg + ((size_t)((inB ? oB0 : oA0) + pp) * Tblk + trow) * 16 + lh * 8);
                    }
                    if (!inB && tw + 32 > tB && tB < Rend && kb >= 0) {   // straddles the boundary: block B's rows of this subtile
                        const int trow = min(max(tw + lm - tB, 0), Tblk - 1);
                        fs2 = *(const bf16x8 *)(Sg + ((size_t)(oB0 + pp) * Tblk + trow) * 16 + lh * 8);
                    }
                }
            };
            kA = __builtin_amdgcn_readfirstlane(kAv); kB = __builtin_amdgcn_readfirstlane(kBv);
            request_operands(0, kA, kB);
            // results of subtile i, column subtile j of the current pass: accumulators + the low-rank term(s)
            auto result = [&](int i, int j, int tw) {
                const bool inB = tw >= tB, both = !inB && tw + 32 > tB && tB < Rend && kB >= 0;
                const bf16x8 f1 = (inB || lm < tB - tw) ? fs1[i] : zero8;   // rows of the other block add nothing
                const bf16x8 f2 = lm >= tB - tw ? fs2 : zero8;
                f32x16 cj = acc[i][j];
                if (inB) {
                    if (kB >= 0) cj = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fwB[j], f1, cj, 0, 0, 0);
                } else {
                    if (kA >= 0) cj = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fwA[j], f1, cj, 0, 0, 0);
                    if (both) cj = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fwB[j], f2, cj, 0, 0, 0);
                }
                return cj;
            };
            if constexpr (EK == 2) {
                for (int p = 0; p < maxfan; ++p) {
#pragma unroll
                    for (int i = 0; i < MI; ++i) {
                        const int tw = R0 + 32 * i;
                        if (tw >= Rend) break;
#pragma unroll
                        for (int j = 0; j < NJ; ++j) stage1(result(i, j, tw), i, j);   // one column subtile at a time: 16 live result registers
                    }
                    kA = __builtin_amdgcn_readfirstlane(kAnv); kB = __builtin_amdgcn_readfirstlane(kBnv);
                    if (p + 1 < maxfan) {
                        request_operands(p + 1, kA, kB);
                        request_ids(p + 2, kAnv, kBnv);
                    }
                    store_rows(p);
                }
            } else {
                // fp32 output with a residual: 32 rows at a time through the wave's 8 KB of LDS (16-byte chunks swizzled by row & 15),
                // whole 256-byte row segments out, 4 rows per store.  The residual rows of a subtile are requested before its MFMAs
                // and without per-lane conditions (rows past the end read a clamped row and are dropped at the store).
                float *stg32 = (float *)dsmem + wave * (32 * RCOLS);
                const int rrow = lane >> 4, rch = lane & 15;
                const int col4 = n0 + wn * RCOLS + rch * 4;
                const bool col4_ok = col4 < g.N;
                const int cfix = col4_ok ? col4 : g.N - 4;
                for (int p = 0; p < maxfan; ++p) {
                    const int obA = oA0 + p < oA1 ? oA0 + p : -1, obB = (hasB && oB0 + p < oB1) ? oB0 + p : -1;
                    const int rbA = (g.res && obA >= 0) ? (g.res_block_of_out ? g.res_block_of_out[obA] : obA) : 0;
                    const int rbB = (g.res && obB >= 0) ? (g.res_block_of_out ? g.res_block_of_out[obB] : obB) : 0;
#pragma unroll
                    for (int i = 0; i < MI; ++i) {
                        const int tw = R0 + 32 * i;
                        if (tw >= Rend) break;
                        f32x4 rv[8];
                        int obq[8];
                        long oq[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const int t = min(tw + 4 * q + rrow, Rend - 1);
                            const bool inB = t >= tB;
                            const int trow = t - (inB ? tB : baseA);
                            obq[q] = (tw + 4 * q + rrow < Rend) ? (inB ? obB : obA) : -1;
                            oq[q] = ((long)max(obq[q], 0) * g.Tout + g.t_off + trow) * g.N;
                            const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
                            rv[q] = g.res ? *(const f32x4 *)(g.res + ((long)(inB ? rbB : rbA) * g.Tout + g.t_off + trow) * g.N + cfix) : z4;
                        }
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            const f32x16 cj = result(i, j, tw);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const f32x4 v = {cj[4 * q], cj[4 * q + 1], cj[4 * q + 2], cj[4 * q + 3]};
                                *(f32x4 *)(stg32 + lm * RCOLS + (((j * 8 + 2 * q + lh) ^ (lm & 15)) << 2)) = v;
                            }
                        }
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const int row = 4 * q + rrow;
                            const f32x4 v = *(const f32x4 *)(stg32 + row * RCOLS + ((rch ^ (row & 15)) << 2)) + rv[q];
                            if (obq[q] >= 0 && col4_ok) *(f32x4 *)((float *)g.out + oq[q] + col4) = v;
                        }
                    }
                    kA = __builtin_amdgcn_readfirstlane(kAnv); kB = __builtin_amdgcn_readfirstlane(kBnv);
                    if (p + 1 < maxfan) {
                        request_operands(p + 1, kA, kB);
                        request_ids(p + 2, kAnv, kBnv);
                    }
                }
            }
        } else {
            for (int p = 0; p < maxfan; ++p) {
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int tw = R0 + 32 * i;
                    if (tw >= Rend) break;
                    f32x16 c[NJ];
#pragma unroll
                    for (int j = 0; j < NJ; ++j) c[j] = acc[i][j];
                    if (has_lora) {
                        const int twe = min(tw + 32, Rend);
                        const int b_lo = flat ? tw / Tblk : xb, b_hi = flat ? (twe - 1) / Tblk : xb;
                        for (int bb = b_lo; bb <= b_hi; ++bb) {
                            const int o0 = g.out_off ? g.out_off[bb] : bb, o1 = g.out_off ? g.out_off[bb + 1] : bb + 1;
                            const int ob = o0 + p;
                            if (ob >= o1) continue;
                            const int rb0 = flat ? bb * Tblk : 0;
                            const int lo = max(rb0 - tw, 0), hi = min(rb0 + Tblk - tw, 32);   // rows [lo, hi) of the subtile lie in block bb
                            const int trow = min(max(tw + lm - rb0, 0), Tblk - 1);
                            const int sb0 = g.set_off ? g.set_off[ob] : ob, sb1 = g.set_off ? g.set_off[ob + 1] : ob + 1;
                            for (int sb = sb0; sb < sb1; ++sb) {
                                const int k_ad = g.adapter_of_out[sb];
                                if (k_ad < 0) continue;
                                for (int s0 = 0; s0 < g.RP; s0 += 16) {
                                    bf16x8 fsb = *(const bf16x8 *)(Sg + ((size_t)sb * Tblk + trow) * g.RP + s0 + lh * 8);
                                    if (lm < lo || lm >= hi) fsb = zero8;
                                    bf16x8 fwb[NJ];
                                    load_fw(fwb, k_ad, s0);
#pragma unroll
                                    for (int j = 0; j < NJ; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fwb[j], fsb, c[j], 0, 0, 0);
                                }
                            }
                        }
                    }
#pragma unroll
                    for (int j = 0; j < NJ; ++j) stage1(c[j], i, j);
                }
                store_rows(p);
            }
        }
        return;
    }

    // ---- epilogue, wave by wave and 32 rows at a time: no workgroup barrier is needed because each wave stages
    // through its own LDS region and the LDS executes one wave's instructions in order.
    // acc[i][j][e] = C[row wm*MI*32 + i*32 + lm][col wn*NJ*32 + j*32 + 8*(e/4) + 4*lh + e%4]
    float *stg = (float *)dsmem + wave * (32 * NC * 4);   // 32 rows x NC chunks of 4 floats; chunk ch of row r at ch ^ swz(r)
    auto swz = [](int r) { return NC == 16 ? (r & 15) : ((r >> 1) & 7); };

    // read-back mapping: NC consecutive lanes cover one row segment; each pass covers 64 / NC rows
    constexpr int RPP = 64 / NC;
    const int rch = lane % NC, rrow = lane / NC;
    const int col = n0 + wn * NJ * 32 + rch * 4;
    const bool col_ok = col < g.N;
    f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
    if (g.bias && col_ok) bias4 = *(const f32x4 *)(g.bias + col);
    const bool gelu = g.mode == EPI_GELU;

    // one 32-row subtile of one output block: c -> LDS -> global.  Row 0 of the subtile is row trow0 of the block (negative
    // when the block starts inside the subtile); rows [lo, hi) of the subtile are stored.
    auto emit = [&](f32x16(&c)[NJ], int ob, int rb, int trow0, int lo, int hi) {
        const long obase = ((long)ob * g.Tout + g.t_off + trow0) * g.N + col;
        const float *res = (g.mode == EPI_RESID && g.res) ? g.res + ((long)rb * g.Tout + g.t_off + trow0) * g.N + col : nullptr;
        const float *pos = (g.mode == EPI_RESID && g.pos) ? g.pos + (long)(g.t_off + trow0) * g.N + col : nullptr;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = j * 8 + 2 * q + lh;
                const f32x4 v = {c[j][4 * q], c[j][4 * q + 1], c[j][4 * q + 2], c[j][4 * q + 3]};
                *(f32x4 *)(stg + lm * (NC * 4) + ((ch ^ swz(lm)) << 2)) = v;
            }
        // LDS -> global
        if (g.mode == EPI_RESID) {
            float *out = (float *)g.out + obase;
#pragma unroll 2
            for (int q = 0; q < 32 / RPP; ++q) {
                const int row = q * RPP + rrow;
                if (row < lo || row >= hi || !col_ok) continue;
                f32x4 v = *(const f32x4 *)(stg + row * (NC * 4) + ((rch ^ swz(row)) << 2)) + bias4;
                if (res) v += *(const f32x4 *)(res + (long)row * g.N);
                if (pos) v += *(const f32x4 *)(pos + (long)row * g.N);
                *(f32x4 *)(out + (long)row * g.N) = v;
            }
        } else {
            bf16_t *out = (bf16_t *)g.out + obase;
#pragma unroll 2
            for (int q = 0; q < 32 / RPP; ++q) {
                const int row = q * RPP + rrow;
                if (row < lo || row >= hi || !col_ok) continue;
                f32x4 v = *(const f32x4 *)(stg + row * (NC * 4) + ((rch ^ swz(row)) << 2)) + bias4;
                if (gelu) {
#pragma unroll
                    for (int z = 0; z < 4; ++z) v[z] = gelu_poly(v[z]);
                }
                const bf16x4 w = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                *(bf16x4 *)(out + (long)row * g.N) = w;
            }
        }
    };

    if (flat) {
        // Row tiles that ignore block boundaries.  The 32 rows of a subtile lie in one block or (a block being at least 32
        // rows, else in several) in consecutive ones: block by block, every row-block that fans out of it gets its own
        // expand, fed with the S rows of that row-block only, and stores its rows of the subtile.
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int tw = t0 + wm * MI * 32 + i * 32;     // first row of this 32-row subtile
            if (tw >= Tlim) break;
            int lo = 0;
            for (int bb = tw / g.Tb; lo < 32 && bb * g.Tb < Tlim; ++bb) {   // (blocks past the true count have no valid ids)
                const int trow0 = tw - bb * g.Tb;
                const int hi = min(32, g.Tb - trow0);                       // rows [lo, hi) of the subtile belong to block bb
                const int o0 = g.out_off ? g.out_off[bb] : bb, o1 = g.out_off ? g.out_off[bb + 1] : bb + 1;
                for (int ob = o0; ob < o1; ++ob) {
                    const int rb = (g.mode == EPI_RESID && g.res) ? (g.res_block_of_out ? g.res_block_of_out[ob] : ob) : 0;
                    f32x16 c[NJ];
#pragma unroll
                    for (int j = 0; j < NJ; ++j) c[j] = acc[i][j];
                    const int sb0 = g.set_off ? g.set_off[ob] : ob, sb1 = g.set_off ? g.set_off[ob + 1] : ob + 1;
                    for (int sb = sb0; has_lora && sb < sb1; ++sb) {     // one low-rank term, or all the terms summed on this block
                        const int k_ad = g.adapter_of_out[sb];
                        if (k_ad < 0) continue;
                        const int t = min(max(trow0 + lm, 0), g.Tb - 1);
                        for (int s0 = 0; s0 < g.RP; s0 += 16) {
                            bf16x8 fsb = *(const bf16x8 *)((const bf16_t *)g.S + ((size_t)sb * g.Tb + t) * g.RP + s0 + lh * 8);
                            if (lm < lo || lm >= hi) fsb = zero8;
                            bf16x8 fwb[NJ];
                            load_fw(fwb, k_ad, s0);
#pragma unroll
                            for (int j = 0; j < NJ; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fwb[j], fsb, c[j], 0, 0, 0);
                        }
                    }
                    emit(c, ob, rb, trow0, lo, hi);
                }
                lo = hi;
            }
        }
        return;
    }

    if (g.set_off) {
        // several low-rank terms summed on one output block: operands fetched term by term, one subtile at a time
        for (int ob = ob0; ob < ob1; ++ob) {
            const int rb = (g.mode == EPI_RESID && g.res) ? (g.res_block_of_out ? g.res_block_of_out[ob] : ob) : 0;
            const int sb0 = g.set_off[ob], sb1 = g.set_off[ob + 1];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int tw = t0 + wm * MI * 32 + i * 32;
                if (tw >= g.T) break;
                f32x16 c[NJ];
#pragma unroll
                for (int j = 0; j < NJ; ++j) c[j] = acc[i][j];
                for (int sb = sb0; has_lora && sb < sb1; ++sb) {
                    const int k_ad = g.adapter_of_out[sb];
                    if (k_ad < 0) continue;
                    const int t = min(tw + lm, g.T - 1);
                    for (int s0 = 0; s0 < g.RP; s0 += 16) {
                        const bf16x8 fsb = *(const bf16x8 *)((const bf16_t *)g.S + ((size_t)sb * g.T + t) * g.RP + s0 + lh * 8);
                        bf16x8 fwb[NJ];
                        load_fw(fwb, k_ad, s0);
#pragma unroll
                        for (int j = 0; j < NJ; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fwb[j], fsb, c[j], 0, 0, 0);
                    }
                }
                emit(c, ob, rb, tw, 0, min(32, g.T - tw));
            }
        }
        return;
    }

    for (int ob = ob0; ob < ob1; ++ob) {
        const int k_ad = has_lora ? g.adapter_of_out[ob] : -1;
        const int rb = (g.mode == EPI_RESID && g.res) ? (g.res_block_of_out ? g.res_block_of_out[ob] : ob) : 0;
        bf16x8 fs[MI], fw[NJ];
        if (k_ad >= 0) {
            if (EARLY && ob == ob0) {
#pragma unroll
                for (int i = 0; i < MI; ++i) fs[i] = fs0[i];
#pragma unroll
                for (int j = 0; j < NJ; ++j) fw[j] = fw0[j];
            } else {
                if (EARLY) { load_fs(fs, ob, 0); load_fw(fw, k_ad, 0); }
            }
        }
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int tw = t0 + wm * MI * 32 + i * 32;     // first row of this 32-row subtile
            if (tw >= g.T) break;
            f32x16 c[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) c[j] = acc[i][j];
            if (k_ad >= 0) {
                // low-rank expand: one more MFMA K step per 16 ranks
                if (!EARLY) {   // large tiles are short of registers: operands are fetched one subtile at a time
                    const int t = min(tw + lm, g.T - 1);
                    fs[i] = *(const bf16x8 *)((const bf16_t *)g.S + ((size_t)ob * g.T + t) * g.RP + lh * 8);
                    load_fw(fw, k_ad, 0);
                }
#pragma unroll
                for (int j = 0; j < NJ; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[j], fs[i], c[j], 0, 0, 0);
                for (int s0 = 16; s0 < g.RP; s0 += 16) {
                    bf16x8 fs2[MI], fw2[NJ];
                    load_fs(fs2, ob, s0);
                    load_fw(fw2, k_ad, s0);
#pragma unroll
                    for (int j = 0; j < NJ; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw2[j], fs2[i], c[j], 0, 0, 0);
                }
            }
            emit(c, ob, rb, tw, 0, min(32, g.T - tw));
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
    if (!decode_tile(g, blockIdx.x, BM, BN, xb, t0, n0, ob0, ob1)) return;

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
        const bool has_lora = g.S && g.adapter_of_out;
        const int sb0 = g.set_off ? g.set_off[ob] : ob, sb1 = g.set_off ? g.set_off[ob + 1] : ob + 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = t0 + ty * 4 + i;
            if (t >= g.T) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = n0 + tx * 4 + j;
                if (col >= g.N) continue;
                float v = acc[i][j];
                for (int sb = sb0; has_lora && sb < sb1; ++sb) {
                    const int k_ad = g.adapter_of_out[sb];
                    if (k_ad < 0) continue;
                    const float *S = (const float *)g.S + ((size_t)sb * g.T + t) * g.RP;
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

template <int BM, int BN, int WM, int WN, int NS> static void launch_dma(const GemmArgs &g, hipStream_t st);

// grid of the XCD order: every XCD gets ceil(tiles / 8) workgroups
static unsigned dma_grid(int tiles_mtot, int tiles_n)
{
    const long total = (long)tiles_mtot * tiles_n;
    return (unsigned)((total + 7) / 8 * 8);
}

template <int BM, int BN, int WM, int WN, int NS, int EK>
static void launch_dma_ek(const GemmArgs &g, hipStream_t st)
{
    constexpr int LDS = NS * (BM + BN) * 64 * 2;
    auto kern = gemm_bf16_dma_kernel<BM, BN, WM, WN, NS, EK>;
    if (LDS > 64 * 1024) {
        static bool attr_set = false;   // raising the dynamic LDS limit is a per-kernel, process-wide setting
        if (!attr_set) {
            (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
            attr_set = true;
        }
    }
    const int tiles_m = (g.T + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    POLY_LAUNCH_SHMEM(POLY_STAGE_GEMM, kern, dim3(dma_grid(g.n_in * tiles_m, tiles_n)), dim3(64 * WM * WN), LDS, st, g, tiles_m, tiles_n);
}

template <int BM, int BN, int WM, int WN, int NS>
static void launch_dma(const GemmArgs &g, hipStream_t st)
{
    if constexpr (BN / WN == 64) {
        // a wave's region of BM / WM rows touches at most two input blocks when a block is at least that long (or when tiles
        // stay inside blocks: Tb == 0)
        const bool two_blocks = g.Tb == 0 || g.Tb >= BM / WM;
        const bool prefetchable = two_blocks && !g.set_off && (!g.S || (g.RP == 16 && g.r % 8 == 0));
        if (g.mode != EPI_RESID) {
            if (prefetchable) launch_dma_ek<BM, BN, WM, WN, NS, 2>(g, st);
            else launch_dma_ek<BM, BN, WM, WN, NS, 1>(g, st);
            return;
        }
        if constexpr (BM / WM <= 64) {   // (with four row subtiles per wave the residual rows in flight do not fit beside the accumulators)
            if (prefetchable && !g.pos) { launch_dma_ek<BM, BN, WM, WN, NS, 3>(g, st); return; }
        }
    }
    launch_dma_ek<BM, BN, WM, WN, NS, 0>(g, st);
}

static int launch_gemm_dma(const GemmArgs &g, hipStream_t st)
{
    // long contractions with many tiles: 256-row tiles cut the L2 -> LDS traffic per flop; short contractions (K = 192)
    // and small batches keep 128-row tiles, whose workgroups are light enough to overlap their load latency and epilogues
    // across a CU
    const long tiles256 = (long)g.n_in * ((g.T + 255) / 256) * ((g.N + 255) / 256);
    const bool big = g.T > 128 && g.K >= 512;
    if (big && g.N % 256 == 0 && tiles256 >= 512) {
        launch_dma<256, 256, 2, 4, 2>(g, st);
    } else if (big && g.N % 128 == 0 && (long)g.n_in * ((g.T + 255) / 256) * ((g.N + 127) / 128) >= 512) {
        launch_dma<256, 128, 4, 2, 3>(g, st);
    } else if (g.N % 128 == 0 || g.N >= 1024) {
        launch_dma<128, 128, 2, 2, 2>(g, st);
    } else if ((long)g.n_in * ((g.T + 127) / 128) * ((g.N + 63) / 64) < 256) {
        // fewer 128 x 64 tiles than CUs (the patch embedding of a small batch): half the rows per tile, twice the workgroups,
        // two of them per CU
        launch_dma<64, 64, 2, 2, 4>(g, st);
    } else {
        launch_dma<128, 64, 2, 2, 2>(g, st);
    }
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}

int launch_gemm(const GemmArgs &g, int dtype, hipStream_t st)
{
    if (g.n_in <= 0 || g.T <= 0) return POLY_OK;
    if (dtype == POLY_BF16) {
        if (g.K % 8 != 0 || (g.S && g.RP % 16 != 0)) return POLY_EINVAL;
        if ((long)g.N * g.K > 0x7fffffffL || (long)g.T * g.K > 0x7fffffffL) return POLY_EINVAL;
        if (g.K % 64 == 0 && g.N % 8 == 0) {
            // input blocks stored back to back and nothing but the output block indexed by the row inside a block: the row
            // tiles run over all input blocks as one (a 197-row block fills only 77 % of a 256-row tile of its own)
            GemmArgs gf = g;
            const long rows = (long)g.n_in * g.T;
            if (g.Tout == g.T && g.t_off == 0 && !g.pos && g.n_in > 1 && g.T % 256 != 0 &&
                rows * g.K <= 0x7fffffffL && rows * g.N <= 0x7fffffffL) {
                gf.Tb = g.T; gf.nb = g.n_in;
                gf.T = (int)rows; gf.n_in = 1;          // (Tout stays the block length: it places the output blocks)
            }
            return launch_gemm_dma(gf, st);
        }
        {
            const int tiles_m = (g.T + 127) / 128;
            const bool wide = g.N % 128 == 0 || g.N >= 1024;
            const long blocks = (long)g.n_in * tiles_m * (wide ? (g.N + 127) / 128 : (g.N + 63) / 64);
            if (blocks > 0x3fffffffL) return POLY_EINVAL;
            if (wide)
                POLY_LAUNCH(POLY_STAGE_GEMM, gemm_bf16_generic_kernel<128>, dim3((unsigned)blocks), dim3(256), st, g);
            else
                POLY_LAUNCH(POLY_STAGE_GEMM, gemm_bf16_generic_kernel<64>, dim3((unsigned)blocks), dim3(256), st, g);
        }
    } else {
        const long blocks = (long)g.n_in * ((g.T + 63) / 64) * ((g.N + 63) / 64);
        if (blocks > 0x7fffffffL) return POLY_EINVAL;
        POLY_LAUNCH(POLY_STAGE_GEMM, gemm_f32_kernel, dim3((unsigned)blocks), dim3(256), st, g);
    }
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}
