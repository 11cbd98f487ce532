// Row-wise and bookkeeping kernels of the forward: CSR validation, patch gathering, LayerNorm,
// LoRA shrink (x A_k), per-adapter heads with sigmoid, and the optional merge to label space.
#include "poly_dev.h"

#include <type_traits>

namespace {

// ------------------------------------------------------------------ CSR check + row maps
// One block.  Validates row_offsets / adapter_ids against (F, R_cap, n_adapters) and builds
// frame_of_row / adapter_of_row.  On any violation nothing downstream runs (meta->R = 0).
__device__ __forceinline__ void prep_block(const int32_t *row_offsets, const int32_t *adapter_ids, int F, int R_cap, int n_adapters,
                                           PolyMeta *meta, int32_t *frame_of_row, int32_t *adapter_of_row, int32_t *dev_status)
{
    __shared__ int bad;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    const int R = row_offsets[F];
    if (row_offsets[0] != 0 || R < 0 || R > R_cap) {
        if (threadIdx.x == 0) bad = 1;
    } else {
        for (int f = threadIdx.x; f < F; f += blockDim.x) {
            const int a = row_offsets[f], b = row_offsets[f + 1];
            if (a > b || a < 0 || b > R) { bad = 1; continue; }
            for (int i = a; i < b; ++i) {
                const int k = adapter_ids[i];
                if (k < 0 || k >= n_adapters) bad = 1;
                frame_of_row[i] = f;
                adapter_of_row[i] = k;
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        meta->R = bad ? 0 : R;
        meta->F_ok = bad ? 0 : F;
        meta->status = bad ? POLY_ERANGE : POLY_OK;
        if (dev_status) *dev_status = meta->status;
    }
}
__global__ void prep_kernel(const int32_t *row_offsets, const int32_t *adapter_ids, int F, int R_cap, int n_adapters,
                            PolyMeta *meta, int32_t *frame_of_row, int32_t *adapter_of_row, int32_t *dev_status)
{
    prep_block(row_offsets, adapter_ids, F, R_cap, n_adapters, meta, frame_of_row, adapter_of_row, dev_status);
}
struct PrepArgs {       // the CSR check as the last block of another launch (row_offsets == nullptr: none)
    const int32_t *row_offsets, *adapter_ids;
    int F, R_cap, n_adapters;
    PolyMeta *meta;
    int32_t *frame_of_row, *adapter_of_row, *dev_status;
};

// ------------------------------------------------------------------ patch gathering
// patches[(f*P + ty*gw + tx)][(i*p + j)*3 + c] = frame[f][ty*p + i][tx*p + j][c]; a run of 3p values
// (fixed i) is contiguous in the NHWC frame.
// VEC elements (16 bytes) per thread when the run length allows it.  The same launch also writes the class-token
// rows x[f][0][:] = cls + pos[0] and clears the merged-score buffer (both are needed much later: two launches less).
template <typename T, int VEC>
__global__ void im2col_kernel(const T *frames, T *patches, int F, int H, int W, int p, float *x, const float *cls, const float *pos,
                              int T_tok, int D, float *merged, size_t n_merged, const PrepArgs pa)
{
    const int nblk = pa.row_offsets ? gridDim.x - 1 : gridDim.x;   // the last block checks the CSR arrays (one launch less)
    if ((int)blockIdx.x == nblk) {
        prep_block(pa.row_offsets, pa.adapter_ids, pa.F, pa.R_cap, pa.n_adapters, pa.meta, pa.frame_of_row, pa.adapter_of_row, pa.dev_status);
        return;
    }
    const int gw = W / p, gh = H / p, run = 3 * p / VEC;         // vectors per contiguous run
    const size_t total = (size_t)F * gh * gw * p * run;
    const size_t gtid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, gsz = (size_t)nblk * blockDim.x;
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    for (size_t idx = gtid; idx < total; idx += gsz) {
        size_t q = idx;
        const int e = q % run; q /= run;
        const int i = q % p; q /= p;
        const int tx = q % gw; q /= gw;
        const int ty = q % gh; const size_t f = q / gh;
        const T *src = frames + ((f * H + (size_t)ty * p + i) * W + (size_t)tx * p) * 3 + (size_t)e * VEC;
        if (VEC == 1) patches[idx] = *src;
        else *(vec_t *)(patches + idx * VEC) = *(const vec_t *)src;
    }
    for (size_t idx = gtid; idx < (size_t)F * D; idx += gsz) {
        const size_t f = idx / D; const int c = idx % D;
        x[f * T_tok * D + c] = cls[c] + pos[c];
    }
    for (size_t idx = gtid; idx < n_merged; idx += gsz) merged[idx] = 0.f;
}

// ------------------------------------------------------------------ LayerNorm
// One wave per row; fp32 statistics (mean, then centred second moment), output in the activation type.
template <typename T>
__global__ __launch_bounds__(256) void layernorm_kernel(const float *x, T *y, const float *gain, const float *shift, int D,
                                                        float eps, int rows_per_block, int n_blocks, const int *n_blocks_dev)
{
    const int nb = n_blocks_dev ? min(*n_blocks_dev, n_blocks) : n_blocks;
    const size_t rows = (size_t)nb * rows_per_block;
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int lane = threadIdx.x & 63;
    const float *xr = x + row * D;
    float s = 0.f;
    for (int k = lane; k < D; k += 64) s += xr[k];
    const float mean = wave_sum(s) / D;
    float v = 0.f;
    for (int k = lane; k < D; k += 64) { const float d = xr[k] - mean; v += d * d; }
    const float inv = rsqrtf(wave_sum(v) / D + eps);
    T *yr = y + row * D;
    for (int k = lane; k < D; k += 64) yr[k] = from_f32<T>((xr[k] - mean) * inv * gain[k] + shift[k]);
}

// D = 256 NV: the row stays in registers (NV 16-byte pieces per lane), read once and written in 8- or 16-byte pieces
template <typename T, int NV>
__global__ __launch_bounds__(256) void layernorm_vec_kernel(const float *x, T *y, const float *gain, const float *shift, float eps,
                                                            int rows_per_block, int n_blocks, const int *n_blocks_dev)
{
    constexpr int D = 256 * NV;
    const int lane = threadIdx.x & 63;
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t rows_cap = (size_t)n_blocks * rows_per_block;
    const float *xr = x + (row < rows_cap ? row : rows_cap - 1) * D + 4 * lane;     // requested before the row count is known
    f32x4 v[NV], g[NV], b[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = *(const f32x4 *)(xr + 256 * i);
#pragma unroll
    for (int i = 0; i < NV; ++i) { g[i] = *(const f32x4 *)(gain + 4 * lane + 256 * i); b[i] = *(const f32x4 *)(shift + 4 * lane + 256 * i); }
    const int nb = n_blocks_dev ? min(*n_blocks_dev, n_blocks) : n_blocks;
    if (row >= (size_t)nb * rows_per_block) return;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += v[i][0] + v[i][1] + v[i][2] + v[i][3];
    const float mean = wave_sum(s) / D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int z = 0; z < 4; ++z) { const float d = v[i][z] - mean; q += d * d; }
    const float inv = rsqrtf(wave_sum(q) / D + eps);
    T *yr = y + row * D + 4 * lane;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        typedef T out4 __attribute__((ext_vector_type(4)));
        out4 o;
#pragma unroll
        for (int z = 0; z < 4; ++z) o[z] = from_f32<T>((v[i][z] - mean) * inv * g[i][z] + b[i][z]);
        *(out4 *)(yr + 256 * i) = o;
    }
}

// ------------------------------------------------------------------ LoRA shrink
// bf16: S = scale * X At_k^T (zero padded to RP columns) with v_mfma_f32_16x16x32_bf16, operands read straight from
// global memory: a lane's 16 bytes are 8 consecutive K elements of one row, four lanes cover 64 contiguous bytes.
//
// The kernel moves few bytes per workgroup, so its time is the length of a workgroup's chain of dependent memory
// round trips and the number of workgroups in flight, not arithmetic.  Hence:
//  - a workgroup covers only 16 * MS = 32 rows of one output block (many workgroups per CU; more rows per workgroup
//    would re-read At_k less often but measured slower) and its four waves split K; the partial sums meet in LDS,
//    where every wave finishes a quarter of the values;
//  - everything that needs only the block index is requested in one go (true count, input block, adapter ids), then
//    -- when output blocks are paired -- the fan-out offsets, then At_k and the rows of a whole batch of K steps at
//    once; the rows of subtile m + 1 are requested before the MFMAs of subtile m.  Rows past T and ranks past r are
//    clamped, not predicated: they feed results that are dropped or zeroed at the store.
// A 16-column MFMA tile is one "group": NG = 2 groups are the two rank halves of an adapter of rank 17-32 or, with
// ranks of at most 16, two adapters: where consecutive output blocks read the same input block (the fan-out of a
// frame into its row-blocks; pair_off = the CSR offsets of the input blocks) the workgroup of the even one does
// both and the input rows are read once instead of twice.
constexpr int SH_NS = 6;    // 32-element K steps whose operands are in flight together

template <int MS, int NG>
__global__ __launch_bounds__(256) void shrink_bf16_kernel(const bf16_t *X, int T, int K, const bf16_t *At, int r, int RP,
                                                          float scale, int n_out, const int *n_out_dev,
                                                          const int *in_block_of_out, const int *adapter_of_out, const int *pair_off,
                                                          bf16_t *S)
{
    constexpr int NV = MS * NG * 4;                              // values per lane and wave
    constexpr int RV = NV < 32 ? NV : 32;                        // values per reduction round
    static_assert(RV % 4 == 0, "reduction rounds");
    __shared__ float red[4][RV][64];
    const int subs = (T + 16 * MS - 1) / (16 * MS);
    const int ob = blockIdx.x / subs, row0 = (blockIdx.x % subs) * (16 * MS);
    const bool paired = NG == 2 && pair_off && in_block_of_out && RP == 16;
    // first round trip: four loads with unconditional addresses, so that they are requested together.  The arrays have
    // n_out entries; those past the true count are read here but never used.
    // (volatile: the compiler would otherwise sink each load below the early exit that precedes its first use)
    const int *pn = n_out_dev ? n_out_dev : adapter_of_out, *pi = in_block_of_out ? in_block_of_out + ob : adapter_of_out + ob;
    const int n_ld = *(const volatile int *)pn, xb_ld = *(const volatile int *)pi;
    const int k1_raw = *(const volatile int *)(adapter_of_out + ob), k2_raw = *(const volatile int *)(adapter_of_out + min(ob + 1, n_out - 1));
    const int n = n_out_dev ? min(n_ld, n_out) : n_out, xb = in_block_of_out ? xb_ld : ob;
    if (ob >= n) return;
    int ob2 = -1;
    if (paired) {                                                // second round trip
        const int p0 = *(const volatile int *)(pair_off + xb), p1 = *(const volatile int *)(pair_off + xb + 1);
        if ((ob - p0) & 1) return;                               // done by the workgroup of ob - 1
        if (ob + 1 < min(p1, n)) ob2 = ob + 1;
    }
    const int k_ad = k1_raw, k_ad2 = ob2 >= 0 ? k2_raw : -1;
    if (k_ad < 0 && k_ad2 < 0) return;
    const int q = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, li = lane & 15, lc = lane >> 4;
    const bf16_t *xblk = X + (size_t)xb * T * K + lc * 8;
    int xoff[MS];                                                // row li of subtile m (the host has checked T * K < 2^31)
#pragma unroll
    for (int m = 0; m < MS; ++m) xoff[m] = min(row0 + 16 * m + li, T - 1) * K;
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    const int steps = K >> 5, per = (steps + 3) / 4;             // full steps; what is left of K (8, 16 or 24) goes to wave 3
    const int s0 = min(q * per, steps), s1 = min(steps, s0 + per);
    for (int j0 = 0; j0 < (paired ? 16 : RP); j0 += 16 * NG) {
        // group g, lane column li: rank `rank` of adapter `ksel`, stored to column `rank` of output block `osel`
        int ksel[NG], osel[NG], rank[NG];
        const bf16_t *ar[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const bool other = paired && g == 1;
            ksel[g] = other ? k_ad2 : k_ad;
            osel[g] = other ? ob2 : ob;
            rank[g] = paired ? li : j0 + 16 * g + li;
            ar[g] = At + ((size_t)max(ksel[g], 0) * r + min(rank[g], r - 1)) * K + lc * 8;
        }
        f32x4 acc[MS][NG];
#pragma unroll
        for (int m = 0; m < MS; ++m)
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[m][g] = f32x4{0.f, 0.f, 0.f, 0.f};
        // NB steps from step st on
        auto batch = [&](auto nb, int st) {
            constexpr int NB = decltype(nb)::value;
            bf16x8 fb[NG][NB], fa[2][NB];
#pragma unroll
            for (int u = 0; u < NB; ++u)
#pragma unroll
                for (int g = 0; g < NG; ++g) fb[g][u] = *(const bf16x8 *)(ar[g] + (st + u) * 32);
#pragma unroll
            for (int u = 0; u < NB; ++u) fa[0][u] = *(const bf16x8 *)(xblk + xoff[0] + (st + u) * 32);
#pragma unroll
            for (int m = 0; m < MS; ++m) {
                if (m + 1 < MS) {
#pragma unroll
                    for (int u = 0; u < NB; ++u) fa[(m + 1) & 1][u] = *(const bf16x8 *)(xblk + xoff[m + 1] + (st + u) * 32);
                }
                __builtin_amdgcn_sched_barrier(0);               // the next rows are requested before these MFMAs wait
#pragma unroll
                for (int u = 0; u < NB; ++u)
#pragma unroll
                    for (int g = 0; g < NG; ++g)
                        acc[m][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[m & 1][u], fb[g][u], acc[m][g], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        int st = s0;                                             // (the counts are the same for the whole wave: scalar branches)
        for (; st + SH_NS <= s1; st += SH_NS) batch(std::integral_constant<int, SH_NS>(), st);
        for (; st + 2 <= s1; st += 2) batch(std::integral_constant<int, 2>(), st);
        for (; st < s1; ++st) batch(std::integral_constant<int, 1>(), st);
        if ((K & 31) && q == 3) {                                // the rest of K: chunks past the end of the row are zero
            const bool in = steps * 32 + lc * 8 + 8 <= K;
            bf16x8 fb[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) fb[g] = in ? *(const bf16x8 *)(ar[g] + steps * 32) : zero8;
#pragma unroll
            for (int m = 0; m < MS; ++m) {
                const bf16x8 fa = in ? *(const bf16x8 *)(xblk + xoff[m] + steps * 32) : zero8;
#pragma unroll
                for (int g = 0; g < NG; ++g) acc[m][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb[g], acc[m][g], 0, 0, 0);
            }
        }
        // value v = (m * NG + g) * 4 + e of a lane: row row0 + 16 m + 4 lc + e, column li of group g.  RV values per round;
        // wave q finishes values [q RV / 4, (q + 1) RV / 4) of the round.
#pragma unroll
        for (int v0 = 0; v0 < NV; v0 += RV) {
            if (v0 || j0) __syncthreads();
#pragma unroll
            for (int v = 0; v < RV; ++v)
                if (v0 + v < NV) red[q][v][lane] = acc[(v0 + v) / (NG * 4)][((v0 + v) / 4) % NG][(v0 + v) & 3];
            __syncthreads();
#pragma unroll
            for (int w = 0; w < RV / 4; ++w) {
                const int vr = q * (RV / 4) + w, v = v0 + vr;    // (q is scalar: the three selections below are uniform)
                const int m = v / (NG * 4), g = (v / 4) % NG, e = v & 3;
                const float sum = red[0][vr][lane] + red[1][vr][lane] + red[2][vr][lane] + red[3][vr][lane];
                const int tt = row0 + 16 * m + 4 * lc + e;
                int ks = ksel[0], os = osel[0], rk = rank[0];
#pragma unroll
                for (int gg = 1; gg < NG; ++gg)
                    if (g == gg) { ks = ksel[gg]; os = osel[gg]; rk = rank[gg]; }
                if (v < NV && tt < T && ks >= 0 && os >= 0 && rk < RP)
                    S[((size_t)os * T + tt) * RP + rk] = rk < r ? (bf16_t)(scale * sum) : (bf16_t)0.f;
            }
        }
    }
}

// fp32: one thread per (row, rank)
__global__ void shrink_f32_kernel(const float *X, int T, int K, const float *At, int r, int RP, float scale, int n_out,
                                  const int *n_out_dev, const int *in_block_of_out, const int *adapter_of_out, float *S)
{
    const int n = n_out_dev ? min(*n_out_dev, n_out) : n_out;
    const size_t total = (size_t)n * T * RP;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int j = idx % RP;
        const size_t row = idx / RP;
        const int ob = row / T, t = row % T;
        const int k_ad = adapter_of_out[ob];
        float acc = 0.f;
        if (k_ad >= 0 && j < r) {
            const int xb = in_block_of_out ? in_block_of_out[ob] : ob;
            const float *xr = X + ((size_t)xb * T + t) * K;
            const float *ar = At + ((size_t)k_ad * r + j) * K;
            for (int k = 0; k < K; ++k) acc = fmaf(xr[k], ar[k], acc);
        }
        S[idx] = scale * acc;
    }
}

// ------------------------------------------------------------------ heads and merge to label space
// One wave per row-block: z = LN(x[src][0][:]); logits = z H_k + hb_k; scores = sigmoid(logits); lane c
// then folds class c into the frame's label vector.  Scores are in (0, 1): the order of positive floats
// is the order of their bit patterns, so an integer atomic max merges overlapping adapters without
// depending on arrival order.
// NX = D/64 values of the row per lane (0: any D, strided loops).  With NX fixed the row, gain, shift and
// the first head row are requested together and each later head row one class ahead of its use.
template <typename T, int NX>
__global__ __launch_bounds__(64) void head_kernel(const float *x, const int *src_block_of_row, int Tn, int D, const float *gain,
                                                  const float *shift, float eps, const T *head_w, const float *head_b, int C,
                                                  const int *adapter_of_row, const int *frame_of_row, const int32_t *class_map,
                                                  int K, const PolyMeta *meta, float *logits, float *scores, float *merged)
{
    const int b = blockIdx.x;
    if (b >= meta->R) return;
    const int lane = threadIdx.x;
    const int src = src_block_of_row ? src_block_of_row[b] : b;
    const int k_ad = adapter_of_row[b];
    const int fr = merged ? frame_of_row[b] : 0;
    const float *xr = x + (size_t)src * Tn * D;
    const int cl = lane < C ? lane : C - 1;
    const float hb = head_b[k_ad * C + cl];
    const int cls = merged ? class_map[k_ad * C + cl] : -1;
    float mine = 0.f;
    if constexpr (NX > 0) {
        float xv[NX], g[NX], sh[NX], hw[NX], hn[NX];
        const T *hk = head_w + (size_t)k_ad * C * D + lane;
#pragma unroll
        for (int i = 0; i < NX; ++i) xv[i] = xr[lane + 64 * i];
#pragma unroll
        for (int i = 0; i < NX; ++i) { g[i] = gain[lane + 64 * i]; sh[i] = shift[lane + 64 * i]; hw[i] = to_f32(hk[64 * i]); }
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NX; ++i) s += xv[i];
        const float mean = wave_sum(s) / D;
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < NX; ++i) { const float d = xv[i] - mean; v += d * d; }
        const float inv = rsqrtf(wave_sum(v) / D + eps);
#pragma unroll
        for (int i = 0; i < NX; ++i) xv[i] = (xv[i] - mean) * inv * g[i] + sh[i];
        for (int c = 0; c < C; ++c) {
            const T *hnext = hk + (size_t)(c + 1 < C ? c + 1 : c) * D;
#pragma unroll
            for (int i = 0; i < NX; ++i) hn[i] = to_f32(hnext[64 * i]);
            float a = 0.f;
#pragma unroll
            for (int i = 0; i < NX; ++i) a = fmaf(xv[i], hw[i], a);
            a = wave_sum(a);
            if (lane == c) mine = a;
#pragma unroll
            for (int i = 0; i < NX; ++i) hw[i] = hn[i];
        }
    } else {
        float s = 0.f;
        for (int k = lane; k < D; k += 64) s += xr[k];
        const float mean = wave_sum(s) / D;
        float v = 0.f;
        for (int k = lane; k < D; k += 64) { const float d = xr[k] - mean; v += d * d; }
        const float inv = rsqrtf(wave_sum(v) / D + eps);
        for (int c = 0; c < C; ++c) {
            const T *hw = head_w + ((size_t)k_ad * C + c) * D;
            float a = 0.f;
            for (int k = lane; k < D; k += 64) a = fmaf((xr[k] - mean) * inv * gain[k] + shift[k], to_f32(hw[k]), a);
            a = wave_sum(a);
            if (lane == c) mine = a;
        }
    }
    if (lane < C) {
        const float lg = mine + hb;
        const float sc = 1.0f / (1.0f + expf(-lg));
        if (logits) logits[(size_t)b * C + lane] = lg;
        scores[(size_t)b * C + lane] = sc;
        if (cls >= 0 && cls < K) atomicMax((int *)(merged + (size_t)fr * K + cls), __float_as_int(sc));
    }
}

}  // namespace

// ------------------------------------------------------------------ launchers

static inline int hip_ok() { return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP; }

int launch_prep(const int32_t *row_offsets, const int32_t *adapter_ids, int F, int R_cap, int n_adapters, PolyMeta *meta,
                int32_t *frame_of_row, int32_t *adapter_of_row, int32_t *dev_status, hipStream_t st)
{
    POLY_LAUNCH(POLY_STAGE_OTHER, prep_kernel, dim3(1), dim3(256), st, row_offsets, adapter_ids, F, R_cap, n_adapters, meta, frame_of_row,
                       adapter_of_row, dev_status);
    return hip_ok();
}

int launch_im2col(const void *frames, void *patches, int F, int H, int W, int p, int dtype, float *x, const float *cls, const float *pos,
                  int T_tok, int D, float *merged, size_t n_merged, const int32_t *row_offsets, const int32_t *adapter_ids, int R_cap,
                  int n_adapters, PolyMeta *meta, int32_t *frame_of_row, int32_t *adapter_of_row, int32_t *dev_status, hipStream_t st)
{
    const PrepArgs pa = {row_offsets, adapter_ids, F, R_cap, n_adapters, meta, frame_of_row, adapter_of_row, dev_status};
    const size_t total = (size_t)F * H * W * 3;
    if (total == 0 && n_merged == 0) {
        if (row_offsets) return launch_prep(row_offsets, adapter_ids, F, R_cap, n_adapters, meta, frame_of_row, adapter_of_row, dev_status, st);
        return POLY_OK;
    }
    // 16-byte vectors when a run of 3p elements is a whole number of them and rows of the frame keep them aligned
    const int vec = dtype == POLY_BF16 ? 8 : 4;
    const bool wide = (3 * p) % vec == 0 && (3 * W) % vec == 0 && ((uintptr_t)frames & 15) == 0 && ((uintptr_t)patches & 15) == 0;
    const size_t work = (wide ? total / vec : total) > n_merged ? (wide ? total / vec : total) : n_merged;
    const unsigned blocks = (unsigned)((work + 255) / 256 > 65536 ? 65536 : (work + 255) / 256 < 1 ? 1 : (work + 255) / 256) + (row_offsets ? 1 : 0);
    if (dtype == POLY_BF16) {
        if (wide) POLY_LAUNCH(POLY_STAGE_OTHER, (im2col_kernel<bf16_t, 8>), dim3(blocks), dim3(256), st, (const bf16_t *)frames, (bf16_t *)patches, F, H, W, p, x, cls, pos, T_tok, D, merged, n_merged, pa);
        else POLY_LAUNCH(POLY_STAGE_OTHER, (im2col_kernel<bf16_t, 1>), dim3(blocks), dim3(256), st, (const bf16_t *)frames, (bf16_t *)patches, F, H, W, p, x, cls, pos, T_tok, D, merged, n_merged, pa);
    } else {
        if (wide) POLY_LAUNCH(POLY_STAGE_OTHER, (im2col_kernel<float, 4>), dim3(blocks), dim3(256), st, (const float *)frames, (float *)patches, F, H, W, p, x, cls, pos, T_tok, D, merged, n_merged, pa);
        else POLY_LAUNCH(POLY_STAGE_OTHER, (im2col_kernel<float, 1>), dim3(blocks), dim3(256), st, (const float *)frames, (float *)patches, F, H, W, p, x, cls, pos, T_tok, D, merged, n_merged, pa);
    }
    return hip_ok();
}

int launch_layernorm(const float *x, void *y, const float *gain, const float *shift, int D, float eps, int T, int n_blocks,
                     const int *n_blocks_dev, int dtype, hipStream_t st)
{
    const size_t rows = (size_t)n_blocks * T;
    if (rows == 0) return POLY_OK;
    const unsigned blocks = (unsigned)((rows + 3) / 4);
    const bool aligned = ((uintptr_t)x & 15) == 0 && ((uintptr_t)y & 15) == 0 && ((uintptr_t)gain & 15) == 0 && ((uintptr_t)shift & 15) == 0;
    if (dtype == POLY_BF16 && aligned && D == 768) {
        POLY_LAUNCH(POLY_STAGE_NORM, (layernorm_vec_kernel<bf16_t, 3>), dim3(blocks), dim3(256), st, x, (bf16_t *)y, gain, shift, eps, T, n_blocks, n_blocks_dev);
    } else if (dtype == POLY_BF16 && aligned && D == 1024) {
        POLY_LAUNCH(POLY_STAGE_NORM, (layernorm_vec_kernel<bf16_t, 4>), dim3(blocks), dim3(256), st, x, (bf16_t *)y, gain, shift, eps, T, n_blocks, n_blocks_dev);
    } else if (dtype == POLY_BF16 && aligned && D == 512) {
        POLY_LAUNCH(POLY_STAGE_NORM, (layernorm_vec_kernel<bf16_t, 2>), dim3(blocks), dim3(256), st, x, (bf16_t *)y, gain, shift, eps, T, n_blocks, n_blocks_dev);
    } else if (dtype == POLY_BF16 && aligned && D == 256) {
        POLY_LAUNCH(POLY_STAGE_NORM, (layernorm_vec_kernel<bf16_t, 1>), dim3(blocks), dim3(256), st, x, (bf16_t *)y, gain, shift, eps, T, n_blocks, n_blocks_dev);
    } else if (dtype == POLY_BF16)
        POLY_LAUNCH(POLY_STAGE_NORM, layernorm_kernel<bf16_t>, dim3(blocks), dim3(256), st, x, (bf16_t *)y, gain, shift, D, eps, T, n_blocks, n_blocks_dev);
    else
        POLY_LAUNCH(POLY_STAGE_NORM, layernorm_kernel<float>, dim3(blocks), dim3(256), st, x, (float *)y, gain, shift, D, eps, T, n_blocks, n_blocks_dev);
    return hip_ok();
}

template <int MS, int NG>
static void launch_shrink_bf16(hipStream_t st, const bf16_t *X, int T, int K, const bf16_t *At, int r, int RP, float scale, int n_out,
                               const int *n_out_dev, const int *in_block_of_out, const int *adapter_of_out, const int *pair_off, bf16_t *S)
{
    const int subs = (T + 16 * MS - 1) / (16 * MS);
    POLY_LAUNCH(POLY_STAGE_SHRINK, (shrink_bf16_kernel<MS, NG>), dim3((unsigned)((size_t)n_out * subs)), dim3(256), st, X, T, K, At, r, RP, scale,
                n_out, n_out_dev, in_block_of_out, adapter_of_out, pair_off, S);
}

int launch_shrink(const void *X, int T, int K, const void *At, int r, int RP, float scale, int n_out, const int *n_out_dev,
                  const int *in_block_of_out, const int *adapter_of_out, const int *pair_off, void *S, int dtype, hipStream_t st)
{
    if (n_out == 0) return POLY_OK;
    if (dtype == POLY_BF16) {
        if (K % 8 != 0 || (long)T * K > 0x7fffffffL) return POLY_EINVAL;
        const bool two_groups = RP > 16 || (pair_off && in_block_of_out);
        if (two_groups)
            launch_shrink_bf16<2, 2>(st, (const bf16_t *)X, T, K, (const bf16_t *)At, r, RP, scale, n_out, n_out_dev, in_block_of_out,
                                     adapter_of_out, pair_off, (bf16_t *)S);
        else
            launch_shrink_bf16<2, 1>(st, (const bf16_t *)X, T, K, (const bf16_t *)At, r, RP, scale, n_out, n_out_dev, in_block_of_out,
                                     adapter_of_out, pair_off, (bf16_t *)S);
    } else {
        const size_t total = (size_t)n_out * T * RP;
        const unsigned blocks = (unsigned)((total + 255) / 256 > 65536 ? 65536 : (total + 255) / 256);
        POLY_LAUNCH(POLY_STAGE_SHRINK, shrink_f32_kernel, dim3(blocks), dim3(256), st, (const float *)X, T, K, (const float *)At, r, RP, scale, n_out,
                           n_out_dev, in_block_of_out, adapter_of_out, (float *)S);
    }
    return hip_ok();
}

template <typename T>
static void launch_head_t(int nx, dim3 grid, hipStream_t st, const float *x, const int *src_block_of_row, int Tn, int D, const float *gain,
                          const float *shift, float eps, const T *head_w, const float *head_b, int C, const int *adapter_of_row,
                          const int *frame_of_row, const int32_t *class_map, int K, const PolyMeta *meta, float *logits, float *scores,
                          float *merged)
{
#define HEAD_CASE(N)                                                                                                             \
    case N:                                                                                                                      \
        POLY_LAUNCH(POLY_STAGE_OTHER, (head_kernel<T, N>), grid, dim3(64), st, x, src_block_of_row, Tn, D, gain, shift, eps, head_w, head_b, \
                    C, adapter_of_row, frame_of_row, class_map, K, meta, logits, scores, merged);                               \
        break;
    switch (nx) {
        HEAD_CASE(1) HEAD_CASE(2) HEAD_CASE(3) HEAD_CASE(4) HEAD_CASE(6) HEAD_CASE(8) HEAD_CASE(12)
        default: HEAD_CASE(0)
    }
#undef HEAD_CASE
}

// ------------------------------------------------------------------ base head of the lagged loop
// Block f: LayerNorm of frame f's class token (row 0 of its block of x) and the K label scores
// sigmoid(z Wb[c] + bb[c]).  The scores go to lag[f + 1] (the selection of frame
// f + 1 reads them there) and to out[f]; block 0 also copies the carried scores of the previous call to lag[0].
template <typename T>
__global__ __launch_bounds__(256) void base_head_kernel(const float *x, int T_tok, int D, const float *gain, const float *shift, float eps,
                                                        const T *Wb, const float *bb, int K, float *lag, float *out, const float *carry)
{
    extern __shared__ float bh_s[];      // z [D], then 8 partial sums
    float *z = bh_s, *part = bh_s + D;
    const int f = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *xr = x + (size_t)f * T_tok * D;
    if (f == 0)
        for (int c = tid; c < K; c += 256) lag[c] = carry ? carry[c] : 0.f;
    float s = 0.f;
    for (int i = tid; i < D; i += 256) s += xr[i];
    s = wave_sum(s);
    if (lane == 0) part[wave] = s;
    __syncthreads();
    const float mean = (part[0] + part[1] + part[2] + part[3]) / D;
    float q = 0.f;
    for (int i = tid; i < D; i += 256) { const float d = xr[i] - mean; q += d * d; }
    q = wave_sum(q);
    if (lane == 0) part[4 + wave] = q;
    __syncthreads();
    const float inv = rsqrtf((part[4] + part[5] + part[6] + part[7]) / D + eps);
    for (int i = tid; i < D; i += 256) z[i] = (xr[i] - mean) * inv * gain[i] + shift[i];
    __syncthreads();
    // eight classes per wave and round: their weight loads are in flight together (one class at a time pays a memory
    // round trip per class), and lane u finishes class c0 + u
    for (int c0 = wave * 8; c0 < K; c0 += 32) {
        float d[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) d[u] = 0.f;
        for (int i = lane; i < D; i += 64) {
            const float zi = z[i];
#pragma unroll
            for (int u = 0; u < 8; ++u) d[u] = fmaf(zi, (float)Wb[(size_t)min(c0 + u, K - 1) * D + i], d[u]);
        }
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float t = wave_sum(d[u]);
            if (lane == u) mine = t;
        }
        const int c = c0 + lane;
        if (lane < 8 && c < K) {
            const float sc = 1.0f / (1.0f + expf(-(mine + bb[c])));
            lag[(size_t)(f + 1) * K + c] = sc;
            if (out) out[(size_t)f * K + c] = sc;
        }
    }
}

// D = 64 ND: no LDS and no workgroup barrier -- every wave normalises the row for itself (lane l holds elements l + 64 j,
// the layout its dot products need), and the weights of the next eight classes are requested before the sums of the
// current eight are reduced, so that a round costs one memory round trip instead of one per K step
template <typename T, int ND>
__global__ __launch_bounds__(256) void base_head_nd_kernel(const float *x, int T_tok, const float *gain, const float *shift, float eps,
                                                           const T *Wb, const float *bb, int K, float *lag, float *out, const float *carry)
{
    constexpr int D = 64 * ND, CW = 8;
    const int f = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *xr = x + (size_t)f * T_tok * D;
    float xv[ND], g[ND], sh[ND];
#pragma unroll
    for (int j = 0; j < ND; ++j) { xv[j] = xr[lane + 64 * j]; g[j] = gain[lane + 64 * j]; sh[j] = shift[lane + 64 * j]; }
    auto loadw = [&](T(&w)[CW][ND], int c0) {
#pragma unroll
        for (int u = 0; u < CW; ++u)
#pragma unroll
            for (int j = 0; j < ND; ++j) w[u][j] = Wb[(size_t)min(c0 + u, K - 1) * D + lane + 64 * j];
    };
    T w0[CW][ND];
    loadw(w0, wave * CW);
    if (f == 0)
        for (int c = tid; c < K; c += 256) lag[c] = carry ? carry[c] : 0.f;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < ND; ++j) s += xv[j];
    const float mean = wave_sum(s) / D;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < ND; ++j) { const float d = xv[j] - mean; q += d * d; }
    const float inv = rsqrtf(wave_sum(q) / D + eps);
    float z[ND];
#pragma unroll
    for (int j = 0; j < ND; ++j) z[j] = (xv[j] - mean) * inv * g[j] + sh[j];
    for (int c0 = wave * CW; c0 < K; c0 += 4 * CW) {
        T w1[CW][ND];
        const bool more = c0 + 4 * CW < K;          // uniform
        if (more) loadw(w1, c0 + 4 * CW);
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < CW; ++u) {
            float d = 0.f;
#pragma unroll
            for (int j = 0; j < ND; ++j) d = fmaf(z[j], (float)w0[u][j], d);
            d = wave_sum(d);
            if (lane == u) mine = d;
        }
        const int c = c0 + lane;
        if (lane < CW && c < K) {
            const float sc = 1.0f / (1.0f + expf(-(mine + bb[c])));
            lag[(size_t)(f + 1) * K + c] = sc;
            if (out) out[(size_t)f * K + c] = sc;
        }
        if (more) {
#pragma unroll
            for (int u = 0; u < CW; ++u)
#pragma unroll
                for (int j = 0; j < ND; ++j) w0[u][j] = w1[u][j];
        }
    }
}

template <typename T>
static bool launch_base_head_nd(int D, int F, hipStream_t st, const float *x, int T_tok, const float *gain, const float *shift, float eps,
                                const T *Wb, const float *bb, int K, float *lag, float *out, const float *carry)
{
    switch (D) {
#define POLY_BH_CASE(ND)                                                                                                            \
    case 64 * ND:                                                                                                                   \
        POLY_LAUNCH(POLY_STAGE_OTHER, (base_head_nd_kernel<T, ND>), dim3(F), dim3(256), st, x, T_tok, gain, shift, eps, Wb, bb, K, lag, out, carry); \
        return true;
        POLY_BH_CASE(1) POLY_BH_CASE(2) POLY_BH_CASE(3) POLY_BH_CASE(4) POLY_BH_CASE(6) POLY_BH_CASE(8) POLY_BH_CASE(12)
#undef POLY_BH_CASE
    default: return false;
    }
}

int launch_base_head(const float *x, int T, int D, const float *gain, const float *shift, float eps, const void *Wb, const float *bb,
                     int K, int F, float *lag, float *out, const float *carry, int dtype, hipStream_t st)
{
    if (F == 0) return POLY_OK;
    if (dtype == POLY_BF16 ? launch_base_head_nd<bf16_t>(D, F, st, x, T, gain, shift, eps, (const bf16_t *)Wb, bb, K, lag, out, carry)
                           : launch_base_head_nd<float>(D, F, st, x, T, gain, shift, eps, (const float *)Wb, bb, K, lag, out, carry))
        return hip_ok();
    const size_t lds = sizeof(float) * (size_t)(D + 8);
    if (dtype == POLY_BF16)
        POLY_LAUNCH_SHMEM(POLY_STAGE_OTHER, base_head_kernel<bf16_t>, dim3(F), dim3(256), lds, st, x, T, D, gain, shift, eps, (const bf16_t *)Wb, bb,
                          K, lag, out, carry);
    else
        POLY_LAUNCH_SHMEM(POLY_STAGE_OTHER, base_head_kernel<float>, dim3(F), dim3(256), lds, st, x, T, D, gain, shift, eps, (const float *)Wb, bb,
                          K, lag, out, carry);
    return hip_ok();
}

// heads, and the merge to the label space when merged is given (zeroed by the caller, F x K)
int launch_head(const float *x, const int *src_block_of_row, int T, int D, const float *gain, const float *shift, float eps,
                const void *head_w, const float *head_b, int C, const int *adapter_of_row, const int *frame_of_row,
                const int32_t *class_map, int K, const PolyMeta *meta, int R_cap, float *logits, float *scores, float *merged, int dtype,
                hipStream_t st)
{
    if (R_cap == 0) return POLY_OK;
    const int nx = D % 64 == 0 ? D / 64 : 0;
    if (dtype == POLY_BF16)
        launch_head_t<bf16_t>(nx, dim3(R_cap), st, x, src_block_of_row, T, D, gain, shift, eps, (const bf16_t *)head_w, head_b, C,
                              adapter_of_row, frame_of_row, class_map, K, meta, logits, scores, merged);
    else
        launch_head_t<float>(nx, dim3(R_cap), st, x, src_block_of_row, T, D, gain, shift, eps, (const float *)head_w, head_b, C,
                             adapter_of_row, frame_of_row, class_map, K, meta, logits, scores, merged);
    return hip_ok();
}
