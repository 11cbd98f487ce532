/*
 * CPU checker for the Polymorph hot path.  TEST INFRASTRUCTURE ONLY: it is
 * what the HIP library is compared against and what the bench times as its
 * CPU baseline.  The product path never calls it, and it shares no code,
 * header, table or helper with the HIP sources.
 *
 * It is the plain definition of what the path computes, written for reading
 * rather than speed: triple loops, double precision everywhere, no blocking,
 * no fusion.  Parameters and frames arrive as float32 (for the bf16 workloads
 * they already hold bf16 values) and are widened to double on use; nothing is
 * rounded in between.
 *
 * Orientation follows the paper (Sec. 3.1): a linear is y = x W + b with
 * W[D_in][D_out]; an adapter is A[D_in][r], B[r][D_out] and the adapted
 * linear is y = x W + b + s (x A) B, computed without ever forming W + A B.
 *
 * What pins each function (tests/test_oracle_*.py):
 *   ora_linear, ora_layernorm, ora_gelu, ora_attention, ora_patch_embed
 *                      -> fp64 library routines on random inputs, and a whole
 *                         forward rebuilt from library routines;
 *   ora_forward        -> zero-B = bare backbone, unmerged = merged (Sec. 3.1),
 *                         position invariance, L0 consistency, Table 2 counts;
 *   ora_forward_sum    -> one adapter per frame = ora_forward (bitwise), equals the forward
 *                         with W + sum_k s A_k B_k merged, a forward rebuilt from library
 *                         routines with the summed weights, order of a frame's ids irrelevant;
 *   ora_build_contexts, ora_intra_coherence, ora_stream_metrics
 *                      -> hand-worked examples, planted groups, a second writing of Alg. 1,
 *                         brute force on small label sets, closed forms (Eq. 6);
 *   ora_select         -> brute force over all context subsets (Eq. 2), the
 *                         closed form on partitions, a second naive writing
 *                         of Alg. 2.
 * Absolute logit values have no printed example in the paper: they are pinned
 * only through the above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define TGT_QKV 1
#define TGT_PROJ 2
#define TGT_FC1 4
#define TGT_FC2 8

typedef struct {
    int32_t H, W, patch, D, heads, L, Dm, L0, targets, r, n_adapters, C;
    double lora_scale, ln_eps;
} ora_model;

typedef struct {
    const float *patch_w, *patch_b, *cls, *pos;                 /* [3pp][D], [D], [D], [T][D] */
    const float *ln1_g, *ln1_b, *qkv_w, *qkv_b, *proj_w, *proj_b; /* stacked over L layers */
    const float *ln2_g, *ln2_b, *fc1_w, *fc1_b, *fc2_w, *fc2_b;
    const float *lnf_g, *lnf_b;
    const float *A[4], *B[4];   /* per target qkv,proj,fc1,fc2: [L-L0][N_ad][D_in][r], [L-L0][N_ad][r][D_out] */
    const float *head_w, *head_b; /* [N_ad][D][C], [N_ad][C] */
    const int32_t *class_map;     /* [N_ad][C] or NULL */
} ora_weights;

/* ------------------------------------------------------------------ stages */

/* y[i][n] = b[n] + sum_k x[i][k] W[k][n]          (x W + b, Sec. 3.1) */
void ora_linear(const double *x, int rows, int din, const float *W, const float *b, int dout, double *y)
{
    for (int i = 0; i < rows; ++i) {
        double *yi = y + (size_t)i * dout;
        for (int n = 0; n < dout; ++n) yi[n] = b ? (double)b[n] : 0.0;
        for (int k = 0; k < din; ++k) {
            const double xk = x[(size_t)i * din + k];
            const float *wk = W + (size_t)k * dout;
            for (int n = 0; n < dout; ++n) yi[n] += xk * (double)wk[n];
        }
    }
}

/* y[i][:] += s * (x[i][:] A) B      (the unmerged low-rank branch x A B, Sec. 3.1) */
void ora_lora_add(const double *x, int rows, int din, const float *A, int r, const float *B, int dout,
                  double s, double *y)
{
    double *sh = (double *)malloc(sizeof(double) * (size_t)r);
    for (int i = 0; i < rows; ++i) {
        for (int j = 0; j < r; ++j) sh[j] = 0.0;
        for (int k = 0; k < din; ++k)
            for (int j = 0; j < r; ++j) sh[j] += x[(size_t)i * din + k] * (double)A[(size_t)k * r + j];
        for (int j = 0; j < r; ++j)
            for (int n = 0; n < dout; ++n) y[(size_t)i * dout + n] += s * sh[j] * (double)B[(size_t)j * dout + n];
    }
    free(sh);
}

/* y = (x - mean) / sqrt(var + eps) * g + b per row, var = mean of squared deviations */
void ora_layernorm(const double *x, int rows, int D, const float *g, const float *b, double eps, double *y)
{
    for (int i = 0; i < rows; ++i) {
        const double *xi = x + (size_t)i * D;
        double mean = 0.0, var = 0.0;
        for (int k = 0; k < D; ++k) mean += xi[k];
        mean /= D;
        for (int k = 0; k < D; ++k) var += (xi[k] - mean) * (xi[k] - mean);
        var /= D;
        const double inv = 1.0 / sqrt(var + eps);
        for (int k = 0; k < D; ++k) y[(size_t)i * D + k] = (xi[k] - mean) * inv * (double)g[k] + (double)b[k];
    }
}

/* exact GELU: x * Phi(x) = x/2 * (1 + erf(x / sqrt 2)) */
void ora_gelu(double *x, size_t n)
{
    for (size_t i = 0; i < n; ++i) x[i] = 0.5 * x[i] * (1.0 + erf(x[i] / sqrt(2.0)));
}

/* Multi-head softmax attention of one token block.  qkv[t] = [q | k | v], each D wide;
 * head j owns columns [j*d, (j+1)*d) of each third, d = D / heads.
 * out[t][j*d + c] = sum_u softmax_u(q_t . k_u / sqrt d) v_u[c]. */
void ora_attention(const double *qkv, int T, int D, int heads, double *out)
{
    const int d = D / heads;
    double *p = (double *)malloc(sizeof(double) * (size_t)T);
    for (int j = 0; j < heads; ++j) {
        for (int t = 0; t < T; ++t) {
            const double *q = qkv + (size_t)t * 3 * D + j * d;
            double mx = -INFINITY;
            for (int u = 0; u < T; ++u) {
                const double *k = qkv + (size_t)u * 3 * D + D + j * d;
                double s = 0.0;
                for (int c = 0; c < d; ++c) s += q[c] * k[c];
                p[u] = s / sqrt((double)d);
                if (p[u] > mx) mx = p[u];
            }
            double den = 0.0;
            for (int u = 0; u < T; ++u) { p[u] = exp(p[u] - mx); den += p[u]; }
            for (int c = 0; c < d; ++c) {
                double o = 0.0;
                for (int u = 0; u < T; ++u) o += p[u] * qkv[(size_t)u * 3 * D + 2 * D + j * d + c];
                out[(size_t)t * D + j * d + c] = o / den;
            }
        }
    }
    free(p);
}

/* Token sequence of one NHWC frame: x[0] = cls + pos[0];
 * x[1 + ty*(W/p) + tx] = patch(ty,tx) W_pe + b_pe + pos[...], the patch vector
 * being indexed (i*p + j)*3 + c for pixel (ty*p + i, tx*p + j), channel c. */
void ora_patch_embed(const float *frame, int H, int W, int p, int D, const float *patch_w,
                     const float *patch_b, const float *cls, const float *pos, double *x)
{
    const int gw = W / p, gh = H / p, pd = 3 * p * p;
    double *v = (double *)malloc(sizeof(double) * (size_t)pd);
    for (int n = 0; n < D; ++n) x[n] = (double)cls[n] + (double)pos[n];
    for (int ty = 0; ty < gh; ++ty)
        for (int tx = 0; tx < gw; ++tx) {
            const int tok = 1 + ty * gw + tx;
            for (int i = 0; i < p; ++i)
                for (int j = 0; j < p; ++j)
                    for (int c = 0; c < 3; ++c)
                        v[(i * p + j) * 3 + c] = (double)frame[((size_t)(ty * p + i) * W + (tx * p + j)) * 3 + c];
            ora_linear(v, 1, pd, patch_w, patch_b, D, x + (size_t)tok * D);
            for (int n = 0; n < D; ++n) x[(size_t)tok * D + n] += (double)pos[(size_t)tok * D + n];
        }
    free(v);
}

/* ------------------------------------------------------------ whole forward */

static int tgt_din(const ora_model *m, int t) { return t == 3 ? m->Dm : m->D; }
static int tgt_dout(const ora_model *m, int t) { return t == 0 ? 3 * m->D : (t == 2 ? m->Dm : m->D); }

/* One linear of layer `layer` (target t: 0 qkv, 1 proj, 2 fc1, 3 fc2) with the adapters ks[0 .. nk) on top (nk = 0: none).
 * merged = 0: y = x W + b + sum_k s (x A_k) B_k   -- "summed on top without merging", Sec. 3.1; one adapter in the branch reading.
 * merged = 1: y = x (W + sum_k s A_k B_k) + b. */
static void adapted_linear(const ora_model *m, const ora_weights *w, int t, int layer, const int32_t *ks, int nk, int merged,
                           const double *x, int rows, const float *W, const float *b, double *y)
{
    const int din = tgt_din(m, t), dout = tgt_dout(m, t), r = m->r;
    const int on = nk > 0 && layer >= m->L0 && (m->targets & (1 << t)) && w->A[t] && w->B[t];
    if (!on) { ora_linear(x, rows, din, W, b, dout, y); return; }
    if (!merged) {
        ora_linear(x, rows, din, W, b, dout, y);
        for (int a = 0; a < nk; ++a) {
            const size_t slot = (size_t)(layer - m->L0) * m->n_adapters + ks[a];
            ora_lora_add(x, rows, din, w->A[t] + slot * din * r, r, w->B[t] + slot * r * dout, dout, m->lora_scale, y);
        }
        return;
    }
    /* W' = W + s sum_k A_k B_k written out, then the plain linear in double */
    double *Wm = (double *)malloc(sizeof(double) * (size_t)din * dout);
    for (size_t i = 0; i < (size_t)din * dout; ++i) Wm[i] = (double)W[i];
    for (int a = 0; a < nk; ++a) {
        const size_t slot = (size_t)(layer - m->L0) * m->n_adapters + ks[a];
        const float *A = w->A[t] + slot * din * r;
        const float *B = w->B[t] + slot * r * dout;
        for (int i = 0; i < din; ++i)
            for (int n = 0; n < dout; ++n) {
                double acc = 0.0;
                for (int j = 0; j < r; ++j) acc += (double)A[(size_t)i * r + j] * (double)B[(size_t)j * dout + n];
                Wm[(size_t)i * dout + n] += m->lora_scale * acc;
            }
    }
    for (int i = 0; i < rows; ++i) {
        double *yi = y + (size_t)i * dout;
        for (int n = 0; n < dout; ++n) yi[n] = (double)b[n];
        for (int kk = 0; kk < din; ++kk)
            for (int n = 0; n < dout; ++n) yi[n] += x[(size_t)i * din + kk] * Wm[(size_t)kk * dout + n];
    }
    free(Wm);
}

/* One pre-LN transformer block in place on x[T][D] with the adapters ks[0 .. nk) on its linears. */
static void block_layer(const ora_model *m, const ora_weights *w, int layer, const int32_t *ks, int nk, int merged, int T, double *x)
{
    const int D = m->D, Dm = m->Dm;
    double *u = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *qkv = (double *)malloc(sizeof(double) * (size_t)T * 3 * D);
    double *o = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *y = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *h = (double *)malloc(sizeof(double) * (size_t)T * Dm);

    ora_layernorm(x, T, D, w->ln1_g + (size_t)layer * D, w->ln1_b + (size_t)layer * D, m->ln_eps, u);
    adapted_linear(m, w, 0, layer, ks, nk, merged, u, T, w->qkv_w + (size_t)layer * D * 3 * D,
                   w->qkv_b + (size_t)layer * 3 * D, qkv);
    ora_attention(qkv, T, D, m->heads, o);
    adapted_linear(m, w, 1, layer, ks, nk, merged, o, T, w->proj_w + (size_t)layer * D * D,
                   w->proj_b + (size_t)layer * D, y);
    for (size_t i = 0; i < (size_t)T * D; ++i) x[i] += y[i];

    ora_layernorm(x, T, D, w->ln2_g + (size_t)layer * D, w->ln2_b + (size_t)layer * D, m->ln_eps, u);
    adapted_linear(m, w, 2, layer, ks, nk, merged, u, T, w->fc1_w + (size_t)layer * D * Dm,
                   w->fc1_b + (size_t)layer * Dm, h);
    ora_gelu(h, (size_t)T * Dm);
    adapted_linear(m, w, 3, layer, ks, nk, merged, h, T, w->fc2_w + (size_t)layer * Dm * D,
                   w->fc2_b + (size_t)layer * D, y);
    for (size_t i = 0; i < (size_t)T * D; ++i) x[i] += y[i];

    free(u); free(qkv); free(o); free(y); free(h);
}

/* Forward of F frames, each with the adapters adapter_ids[row_offsets[f] .. row_offsets[f+1]).
 * Row-block b = (frame f, adapter k) is its own branch: layers [0, L0) run once per frame
 * with no adapter, layers [L0, L) run per row-block with adapter k alone, then the final
 * LayerNorm of the class token and adapter k's head:
 *     logits[b] = LN(x_b[0]) H_k + hb_k,  scores[b] = 1 / (1 + exp(-logits[b])).
 * merged_out (optional, [F][K]): score of class class_map[k][c] taken from row-block (f,k),
 * maximum where adapters overlap, 0 where no active adapter reports the class.
 * x_final (optional, [R][T][D]): residual stream after the last layer, for tests.
 * Returns 0, or -1 on an adapter id out of range / offsets not monotone. */
int ora_forward(const ora_model *m, const ora_weights *w, const float *frames, int F,
                const int32_t *row_offsets, const int32_t *adapter_ids, int merged,
                double *logits, double *scores, double *merged_out, int K, double *x_final)
{
    const int T = 1 + (m->H / m->patch) * (m->W / m->patch), D = m->D, C = m->C;
    const int R = row_offsets[F];
    for (int f = 0; f < F; ++f) if (row_offsets[f + 1] < row_offsets[f]) return -1;
    for (int b = 0; b < R; ++b) if (adapter_ids[b] < 0 || adapter_ids[b] >= m->n_adapters) return -1;

    double *trunk = (double *)malloc(sizeof(double) * (size_t)(F > 0 ? F : 1) * T * D);
#pragma omp parallel for schedule(dynamic, 1)
    for (int f = 0; f < F; ++f) {
        double *x = trunk + (size_t)f * T * D;
        ora_patch_embed(frames + (size_t)f * m->H * m->W * 3, m->H, m->W, m->patch, D, w->patch_w, w->patch_b,
                        w->cls, w->pos, x);
        for (int l = 0; l < m->L0 && l < m->L; ++l) block_layer(m, w, l, NULL, 0, 0, T, x);
    }

    int32_t *frame_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(R > 0 ? R : 1));
    for (int f = 0; f < F; ++f)
        for (int b = row_offsets[f]; b < row_offsets[f + 1]; ++b) frame_of[b] = f;

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < R; ++b) {
        const int k = adapter_ids[b];
        double *x = (double *)malloc(sizeof(double) * (size_t)T * D);
        double *z = (double *)malloc(sizeof(double) * (size_t)D);
        memcpy(x, trunk + (size_t)frame_of[b] * T * D, sizeof(double) * (size_t)T * D);
        for (int l = m->L0; l < m->L; ++l) block_layer(m, w, l, &adapter_ids[b], 1, merged, T, x);
        if (x_final) memcpy(x_final + (size_t)b * T * D, x, sizeof(double) * (size_t)T * D);
        ora_layernorm(x, 1, D, w->lnf_g, w->lnf_b, m->ln_eps, z);
        ora_linear(z, 1, D, w->head_w + (size_t)k * D * C, w->head_b + (size_t)k * C, C, logits + (size_t)b * C);
        for (int c = 0; c < C; ++c)
            scores[(size_t)b * C + c] = 1.0 / (1.0 + exp(-logits[(size_t)b * C + c]));
        free(x); free(z);
    }

    if (merged_out && w->class_map) {
        for (size_t i = 0; i < (size_t)F * K; ++i) merged_out[i] = 0.0;
        for (int b = 0; b < R; ++b)
            for (int c = 0; c < C; ++c) {
                const int cls = w->class_map[(size_t)adapter_ids[b] * C + c];
                if (cls < 0 || cls >= K) continue;
                double *dst = merged_out + (size_t)frame_of[b] * K + cls;
                if (scores[(size_t)b * C + c] > *dst) *dst = scores[(size_t)b * C + c];
            }
    }
    free(trunk); free(frame_of);
    return 0;
}

/* The other reading of Sec. 3.1 for several active adapters: ONE hidden state per frame with all of the frame's
 * adapters summed on top of the shared weights,
 *     linear(x) = x W + b + sum_{k in S_f} s (x A_k) B_k        in layers [L0, L),
 * and then every active adapter's own head on that one state: row b = (f, k) of the CSR arrays gets
 *     logits[b] = LN(x_f[0]) H_k + hb_k,  scores[b] = sigmoid(logits[b]).
 * Arguments and the optional merge to the label space as in ora_forward; x_final is [F][T][D]. */
int ora_forward_sum(const ora_model *m, const ora_weights *w, const float *frames, int F,
                    const int32_t *row_offsets, const int32_t *adapter_ids, int merged,
                    double *logits, double *scores, double *merged_out, int K, double *x_final)
{
    const int T = 1 + (m->H / m->patch) * (m->W / m->patch), D = m->D, C = m->C;
    const int R = row_offsets[F];
    for (int f = 0; f < F; ++f) if (row_offsets[f + 1] < row_offsets[f]) return -1;
    for (int b = 0; b < R; ++b) if (adapter_ids[b] < 0 || adapter_ids[b] >= m->n_adapters) return -1;

#pragma omp parallel for schedule(dynamic, 1)
    for (int f = 0; f < F; ++f) {
        const int32_t *ks = adapter_ids + row_offsets[f];
        const int nk = row_offsets[f + 1] - row_offsets[f];
        double *x = (double *)malloc(sizeof(double) * (size_t)T * D);
        double *z = (double *)malloc(sizeof(double) * (size_t)D);
        ora_patch_embed(frames + (size_t)f * m->H * m->W * 3, m->H, m->W, m->patch, D, w->patch_w, w->patch_b,
                        w->cls, w->pos, x);
        for (int l = 0; l < m->L; ++l) block_layer(m, w, l, ks, l >= m->L0 ? nk : 0, merged, T, x);
        if (x_final) memcpy(x_final + (size_t)f * T * D, x, sizeof(double) * (size_t)T * D);
        ora_layernorm(x, 1, D, w->lnf_g, w->lnf_b, m->ln_eps, z);
        for (int a = 0; a < nk; ++a) {
            const int b = row_offsets[f] + a, k = ks[a];
            ora_linear(z, 1, D, w->head_w + (size_t)k * D * C, w->head_b + (size_t)k * C, C, logits + (size_t)b * C);
            for (int c = 0; c < C; ++c)
                scores[(size_t)b * C + c] = 1.0 / (1.0 + exp(-logits[(size_t)b * C + c]));
        }
        free(x); free(z);
    }

    if (merged_out && w->class_map) {
        for (size_t i = 0; i < (size_t)F * K; ++i) merged_out[i] = 0.0;
        for (int f = 0; f < F; ++f)
            for (int b = row_offsets[f]; b < row_offsets[f + 1]; ++b)
                for (int c = 0; c < C; ++c) {
                    const int cls = w->class_map[(size_t)adapter_ids[b] * C + c];
                    if (cls < 0 || cls >= K) continue;
                    double *dst = merged_out + (size_t)f * K + cls;
                    if (scores[(size_t)b * C + c] > *dst) *dst = scores[(size_t)b * C + c];
                }
    }
    return 0;
}

/* Isolated multi-LoRA linear (Sec. 3.1): row-block b = (X block f, adapter k):
 *     Y[b] = X[f] W + bias + s (X[f] A_k) B_k,   X [n_xblocks][T][Kdim],  Y [R][T][Ndim].
 * Only the row-blocks b in [b_begin, b_end) are computed (Y is indexed from b_begin). */
int ora_lora_linear(const float *X, int n_xblocks, int T, int Kdim, const float *W, const float *bias, int Ndim,
                    const float *A, const float *B, int n_adapters, int r, double s,
                    const int32_t *row_offsets, const int32_t *adapter_ids, int b_begin, int b_end, double *Y)
{
    const int R = row_offsets[n_xblocks];
    if (b_begin < 0 || b_end > R) return -1;
    int32_t *xb_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(R > 0 ? R : 1));
    for (int f = 0; f < n_xblocks; ++f)
        for (int b = row_offsets[f]; b < row_offsets[f + 1]; ++b) xb_of[b] = f;
    for (int b = b_begin; b < b_end; ++b)
        if (adapter_ids[b] < 0 || adapter_ids[b] >= n_adapters) { free(xb_of); return -1; }
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = b_begin; b < b_end; ++b) {
        const int k = adapter_ids[b];
        double *x = (double *)malloc(sizeof(double) * (size_t)T * Kdim);
        const float *xf = X + (size_t)xb_of[b] * T * Kdim;
        for (size_t i = 0; i < (size_t)T * Kdim; ++i) x[i] = (double)xf[i];
        double *y = Y + (size_t)(b - b_begin) * T * Ndim;
        ora_linear(x, T, Kdim, W, bias, Ndim, y);
        ora_lora_add(x, T, Kdim, A + (size_t)k * Kdim * r, r, B + (size_t)k * r * Ndim, Ndim, s, y);
        free(x);
    }
    free(xb_of);
    return 0;
}

/* --------------------------------------------------------------- selection */

typedef struct {
    int32_t valid;        /* 0: no previous frame */
    uint8_t *prev_labels; /* [K]  Y_{t-1} as 0/1 */
    int32_t *prev_set;    /* [M]  S_{t-1} in selection order */
    int32_t prev_count;
} ora_select_state;

/* does context c provide label l?  (l in C and a_{C,l} >= tau; without a table: l in C) */
static int provides(const uint8_t *member, const float *acc, float tau, int K, int c, int l)
{
    if (!member[(size_t)c * K + l]) return 0;
    return acc ? acc[(size_t)c * K + l] >= tau : 1;
}

/* Alg. 2 over a stream of F frames, t ascending.
 *   Y_t = { l : scores[t][l] >= theta }
 *   Y_t == Y_{t-1}                                   -> S_t = S_{t-1}
 *   context_copy and S_{t-1} provides every l in Y_t -> S_t = S_{t-1}
 *   otherwise scan contexts by (|C| ascending, id ascending); take C iff it provides at least one
 *   still-uncovered label; remove those labels; stop when nothing is uncovered.
 * Output CSR: row_offsets[F+1], adapter_ids in selection order.  n_uncovered counts, over all
 * frames, labels of Y_t that no context of S_t provides.  state may be NULL (no previous frame).
 * Returns 0, or -1 if cap is too small (n_rows still holds the needed size). */
int ora_select(const float *scores, int F, int K, const uint8_t *member, int M, float theta, int context_copy,
               const float *acc, float tau, ora_select_state *state,
               int32_t *row_offsets, int32_t *adapter_ids, int cap, int32_t *n_rows, int32_t *n_uncovered)
{
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)M);
    int32_t *size = (int32_t *)malloc(sizeof(int32_t) * (size_t)M);
    for (int c = 0; c < M; ++c) {
        size[c] = 0;
        for (int l = 0; l < K; ++l) size[c] += member[(size_t)c * K + l] ? 1 : 0;
        order[c] = c;
    }
    for (int i = 1; i < M; ++i) { /* insertion sort: stable, so equal sizes stay in id order */
        int c = order[i], j = i - 1;
        while (j >= 0 && size[order[j]] > size[c]) { order[j + 1] = order[j]; --j; }
        order[j + 1] = c;
    }

    uint8_t *Y = (uint8_t *)malloc((size_t)K), *Yprev = (uint8_t *)malloc((size_t)K), *U = (uint8_t *)malloc((size_t)K);
    int32_t *S = (int32_t *)malloc(sizeof(int32_t) * (size_t)M), *Sprev = (int32_t *)malloc(sizeof(int32_t) * (size_t)M);
    int ns = 0, nprev = 0, valid = 0;
    if (state && state->valid) {
        valid = 1; nprev = state->prev_count;
        memcpy(Yprev, state->prev_labels, (size_t)K);
        memcpy(Sprev, state->prev_set, sizeof(int32_t) * (size_t)nprev);
    }

    int total = 0, unc = 0;
    row_offsets[0] = 0;
    for (int t = 0; t < F; ++t) {
        for (int l = 0; l < K; ++l) Y[l] = scores[(size_t)t * K + l] >= theta ? 1 : 0;
        int same = valid, covered = valid && context_copy;
        if (valid) {
            for (int l = 0; l < K; ++l) if (Y[l] != Yprev[l]) same = 0;
            if (context_copy)
                for (int l = 0; l < K; ++l) {
                    if (!Y[l]) continue;
                    int ok = 0;
                    for (int i = 0; i < nprev; ++i) ok |= provides(member, acc, tau, K, Sprev[i], l);
                    if (!ok) covered = 0;
                }
        }
        if (same || covered) {
            ns = nprev;
            memcpy(S, Sprev, sizeof(int32_t) * (size_t)nprev);
        } else {
            ns = 0;
            int left = 0;
            for (int l = 0; l < K; ++l) { U[l] = Y[l]; left += Y[l]; }
            for (int i = 0; i < M && left > 0; ++i) {
                const int c = order[i];
                int got = 0;
                for (int l = 0; l < K; ++l)
                    if (U[l] && provides(member, acc, tau, K, c, l)) { U[l] = 0; ++got; }
                if (got) { S[ns++] = c; left -= got; }
            }
        }
        for (int l = 0; l < K; ++l) {
            if (!Y[l]) continue;
            int ok = 0;
            for (int i = 0; i < ns; ++i) ok |= provides(member, acc, tau, K, S[i], l);
            if (!ok) ++unc;
        }
        for (int i = 0; i < ns; ++i) {
            if (total < cap) adapter_ids[total] = S[i];
            ++total;
        }
        row_offsets[t + 1] = total;
        memcpy(Yprev, Y, (size_t)K);
        memcpy(Sprev, S, sizeof(int32_t) * (size_t)ns);
        nprev = ns; valid = 1;
    }
    if (state && F > 0) {
        state->valid = 1; state->prev_count = nprev;
        memcpy(state->prev_labels, Yprev, (size_t)K);
        memcpy(state->prev_set, Sprev, sizeof(int32_t) * (size_t)nprev);
    }
    *n_rows = total;
    if (n_uncovered) *n_uncovered = unc;
    free(order); free(size); free(Y); free(Yprev); free(U); free(S); free(Sprev);
    return total > cap ? -1 : 0;
}

/* ------------------------------------------- context construction (Alg. 1) */

/* Alg. 1 "BuildContexts" (Sec. 3.4) on a co-occurrence matrix cooc[K][K] (cooc[i][j], i != j: how often labels i
 * and j occur together; cooc[l][l]: how often l occurs at all).  Steps, in the order of the listing:
 *   - a label is valid iff its row has a non-zero entry;
 *   - valid labels are visited by descending frequency cooc[l][l] (ties: lower index first) -- the text builds the
 *     clusters "around frequently occurring labels";
 *   - without overlap a label that is already assigned is skipped;
 *   - the cluster around l is l plus its strongest co-occurring neighbours: up to B - 1 labels j != l with
 *     cooc[l][j] > 0, strongest first (ties: lower index), without overlap only labels not yet assigned;
 *   - the cluster is added iff the same label set is not a context already and fewer than M_max contexts exist;
 *     without overlap its labels become assigned;
 *   - afterwards every valid label that is in no context (same visiting order) is put into the context with
 *     fewer than B labels to which it fits best: largest sum of cooc[l][j] over the context's labels j (ties:
 *     lower context index).  If no context has room the label stays out and is counted in n_unplaced.
 * member[M_max][K] receives the contexts as 0/1 rows in order of creation; returns their number. */
int ora_build_contexts(const float *cooc, int K, int B, int M_max, int allow_overlap, uint8_t *member,
                       int32_t *n_unplaced)
{
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    uint8_t *valid = (uint8_t *)malloc((size_t)K), *assigned = (uint8_t *)calloc((size_t)K, 1);
    uint8_t *cluster = (uint8_t *)malloc((size_t)K);
    int nv = 0, M = 0;
    for (int l = 0; l < K; ++l) {
        valid[l] = 0;
        for (int j = 0; j < K; ++j) if (cooc[(size_t)l * K + j] != 0.f) valid[l] = 1;
        if (valid[l]) order[nv++] = l;
    }
    for (int i = 1; i < nv; ++i) { /* stable insertion sort by descending frequency */
        int l = order[i], j = i - 1;
        while (j >= 0 && cooc[(size_t)order[j] * K + order[j]] < cooc[(size_t)l * K + l]) { order[j + 1] = order[j]; --j; }
        order[j + 1] = l;
    }
    memset(member, 0, (size_t)M_max * K);
    for (int i = 0; i < nv; ++i) {
        const int l = order[i];
        if (!allow_overlap && assigned[l]) continue;
        memset(cluster, 0, (size_t)K);
        cluster[l] = 1;
        for (int n = 1; n < B; ++n) { /* next strongest neighbour that is still free */
            int best = -1;
            for (int j = 0; j < K; ++j) {
                if (cluster[j] || cooc[(size_t)l * K + j] <= 0.f) continue;
                if (!allow_overlap && assigned[j]) continue;
                if (best < 0 || cooc[(size_t)l * K + j] > cooc[(size_t)l * K + best]) best = j;
            }
            if (best < 0) break;
            cluster[best] = 1;
        }
        int unique = 1;
        for (int c = 0; c < M; ++c) if (memcmp(member + (size_t)c * K, cluster, (size_t)K) == 0) unique = 0;
        if (unique && M < M_max) {
            memcpy(member + (size_t)M * K, cluster, (size_t)K);
            ++M;
            if (!allow_overlap) for (int j = 0; j < K; ++j) if (cluster[j]) assigned[j] = 1;
        }
    }
    int unplaced = 0;
    for (int i = 0; i < nv; ++i) {
        const int l = order[i];
        int covered = 0;
        for (int c = 0; c < M; ++c) covered |= member[(size_t)c * K + l];
        if (covered) continue;
        int best = -1;
        double best_fit = 0.0;
        for (int c = 0; c < M; ++c) {
            int size = 0;
            double fit = 0.0;
            for (int j = 0; j < K; ++j)
                if (member[(size_t)c * K + j]) { ++size; fit += (double)cooc[(size_t)l * K + j]; }
            if (size >= B) continue;
            if (best < 0 || fit > best_fit) { best = c; best_fit = fit; }
        }
        if (best >= 0) member[(size_t)best * K + l] = 1; else ++unplaced;
    }
    if (n_unplaced) *n_unplaced = unplaced;
    free(order); free(valid); free(assigned); free(cluster);
    return M;
}

/* IntraCoherence (Eq. 6): mean over the contexts of the mean of co(i, j) over ordered pairs i != j of the context,
 * co(i, j) = cooc[i][j] / norm.  A context with fewer than two labels has no pair and contributes 0. */
double ora_intra_coherence(const float *cooc, int K, double norm, const uint8_t *member, int M)
{
    if (M <= 0) return 0.0;
    double total = 0.0;
    for (int c = 0; c < M; ++c) {
        int size = 0;
        double sum = 0.0;
        for (int i = 0; i < K; ++i) {
            if (!member[(size_t)c * K + i]) continue;
            ++size;
            for (int j = 0; j < K; ++j)
                if (j != i && member[(size_t)c * K + j]) sum += (double)cooc[(size_t)i * K + j] / norm;
        }
        if (size >= 2) total += sum / ((double)size * (size - 1));
    }
    return total / M;
}

/* AvgCoverage = (1/T) sum_t |S_t| and SwitchPenalty = sum_{t >= 2} [S_t != S_{t-1}] (Sec. 3.4) of a stream of
 * context sets given as CSR arrays; sets are compared as sets (the order inside a frame does not matter). */
void ora_stream_metrics(const int32_t *row_offsets, const int32_t *adapter_ids, int F, int M, double *avg_coverage,
                        int64_t *switch_penalty)
{
    uint8_t *cur = (uint8_t *)calloc((size_t)M, 1), *prev = (uint8_t *)calloc((size_t)M, 1);
    int64_t switches = 0;
    for (int t = 0; t < F; ++t) {
        memset(cur, 0, (size_t)M);
        for (int i = row_offsets[t]; i < row_offsets[t + 1]; ++i) cur[adapter_ids[i]] = 1;
        if (t > 0 && memcmp(cur, prev, (size_t)M) != 0) ++switches;
        memcpy(prev, cur, (size_t)M);
    }
    *avg_coverage = F > 0 ? (double)row_offsets[F] / F : 0.0;
    *switch_penalty = switches;
    free(cur); free(prev);
}
