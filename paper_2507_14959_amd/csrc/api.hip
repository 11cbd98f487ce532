// C-ABI entry points: argument checks, workspace carving and the launch sequence of the forward.
#include "poly_dev.h"

namespace {

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }
inline size_t elt_size(int dtype) { return dtype == POLY_BF16 ? 2 : 4; }
inline int rank_pad(int r) { return (r + 15) / 16 * 16; }

struct Carver {
    char *base;
    size_t off;
    template <typename T> T *take(size_t bytes)
    {
        T *p = base ? (T *)(base + off) : nullptr;
        off = align_up(off + bytes);
        return p;
    }
};

struct ForwardWs {
    PolyMeta *meta;
    int32_t *frame_of_row, *adapter_of_row;
    float *xa, *xb;  // residual streams: per frame (shared layers), per row-block (adapted layers)
    void *u, *qkv, *o, *h, *S, *patches;
    size_t bytes;
};

ForwardWs carve_forward(const poly_model_desc *m, int F, int R, void *base)
{
    const size_t T = 1 + (size_t)(m->H / m->patch) * (m->W / m->patch), es = elt_size(m->dtype);
    const size_t nb = (size_t)(F > R ? F : R), rows = nb * T;
    Carver c{(char *)base, 0};
    ForwardWs w;
    w.meta = c.take<PolyMeta>(sizeof(PolyMeta));
    w.frame_of_row = c.take<int32_t>(sizeof(int32_t) * (size_t)(R + 1));
    w.adapter_of_row = c.take<int32_t>(sizeof(int32_t) * (size_t)(R + 1));
    w.xa = c.take<float>(sizeof(float) * (size_t)F * T * m->D);
    w.xb = c.take<float>(sizeof(float) * (size_t)R * T * m->D);
    w.u = c.take<void>(es * rows * m->D);
    w.qkv = c.take<void>(es * rows * 3 * m->D);
    w.o = c.take<void>(es * rows * m->D);
    w.h = c.take<void>(es * rows * m->Dm);
    w.S = c.take<void>(es * (size_t)R * T * rank_pad(m->r));
    w.patches = c.take<void>(es * (size_t)F * (T - 1) * 3 * m->patch * m->patch);
    w.bytes = c.off;
    return w;
}

int check_model(const poly_model_desc *m)
{
    if (!m) return POLY_EINVAL;
    if (m->dtype != POLY_F32 && m->dtype != POLY_BF16) return POLY_EINVAL;
    if (m->patch <= 0 || m->H <= 0 || m->W <= 0 || m->H % m->patch || m->W % m->patch) return POLY_EINVAL;
    if (m->heads <= 0 || m->D != m->heads * POLY_HEAD_DIM || m->Dm <= 0 || m->L <= 0) return POLY_EINVAL;
    if (m->L0 < 0 || m->L0 > m->L) return POLY_EINVAL;
    if (m->r <= 0 || m->r > POLY_MAX_RANK || m->n_adapters <= 0 || m->C <= 0 || m->C > POLY_MAX_HEAD_CLASSES) return POLY_EINVAL;
    if (m->targets & ~15) return POLY_EINVAL;
    if (m->compose != POLY_COMPOSE_BRANCH && m->compose != POLY_COMPOSE_SUM) return POLY_EINVAL;
    const int T = 1 + (m->H / m->patch) * (m->W / m->patch);
    if (m->dtype == POLY_BF16) {
        // 16-byte vector loads along the contraction index; attention keeps a block's keys in LDS
        if (m->Dm % 8 || (3 * m->patch * m->patch) % 8 || T > 224) return POLY_EINVAL;
    } else {
        if (m->Dm % 4 || (3 * m->patch * m->patch) % 4) return POLY_EINVAL;
    }
    return POLY_OK;
}

#define POLY_TRY(expr)                  \
    do {                                \
        const int rc_ = (expr);         \
        if (rc_ != POLY_OK) return rc_; \
    } while (0)

}  // namespace

extern "C" const char *poly_status_string(int status)
{
    switch (status) {
    case POLY_OK: return "ok";
    case POLY_EINVAL: return "invalid argument";
    case POLY_ERANGE: return "adapter id or row offsets out of range";
    case POLY_ECAP: return "output or workspace too small";
    case POLY_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

extern "C" size_t poly_forward_workspace_bytes(const poly_model_desc *m, int F, int R)
{
    if (check_model(m) != POLY_OK || F < 0 || R < 0) return 0;
    return carve_forward(m, F, R, nullptr).bytes;
}

namespace {
// what poly_stream_step adds to the forward: the CSR arrays are written on the way (after the shared layers) instead of given
struct StreamStep {
    const poly_stream *s;
    int32_t *row_offsets, *adapter_ids, *counters;
    float *out_base_scores;
    float *lag;        // [F + 1][K], in the workspace behind the forward's part
};

int forward_impl(const poly_model_desc *m, const poly_base_weights *base, const poly_lora_weights *lora,
                 const poly_heads *heads, const void *frames, int F, const int32_t *row_offsets,
                 const int32_t *adapter_ids, int R, float *out_logits, float *out_scores, float *out_merged, int K,
                 int32_t *dev_status, void *workspace, size_t workspace_bytes, void *stream, const StreamStep *ss)
{
    POLY_TRY(check_model(m));
    if (!base || !heads || F < 0 || R < 0) return POLY_EINVAL;
    if (F == 0) return POLY_OK;
    if (!frames || !row_offsets || (R > 0 && (!adapter_ids || !out_scores))) return POLY_EINVAL;
    if (!base->patch_w || !base->patch_b || !base->cls || !base->pos || !base->ln1_g || !base->ln1_b || !base->qkv_w ||
        !base->qkv_b || !base->proj_w || !base->proj_b || !base->ln2_g || !base->ln2_b || !base->fc1_w || !base->fc1_b ||
        !base->fc2_w || !base->fc2_b || !base->lnf_g || !base->lnf_b || !heads->head_w || !heads->head_b)
        return POLY_EINVAL;
    if (out_merged && (!heads->class_map || K <= 0)) return POLY_EINVAL;
    const bool adapted = m->L0 < m->L;
    for (int t = 0; t < 4; ++t)
        if (adapted && (m->targets & (1 << t)) && (!lora || !lora->At[t] || !lora->Bt[t])) return POLY_EINVAL;
    if (((uintptr_t)workspace & 255) != 0 || !workspace) return POLY_EINVAL;
    const ForwardWs w = carve_forward(m, F, R, workspace);
    if (workspace_bytes < w.bytes) return POLY_ECAP;

    hipStream_t st = (hipStream_t)stream;
    const int dt = m->dtype, D = m->D, Dm = m->Dm, T = 1 + (m->H / m->patch) * (m->W / m->patch), pd = 3 * m->patch * m->patch;
    const int RP = rank_pad(m->r);
    const size_t es = elt_size(dt);
    const int *R_dev = &w.meta->R;
    const bool sum = m->compose == POLY_COMPOSE_SUM;

    // tokens: x[f][0] = cls + pos[0]; x[f][1 + t] = patch_t W_pe + b_pe + pos[1 + t].  The same launch checks the CSR arrays and
    // builds the row maps (nothing before the first adapted layer needs them).
    POLY_TRY(launch_im2col(frames, w.patches, F, m->H, m->W, m->patch, dt, w.xa, base->cls, base->pos, T, D, out_merged,
                           out_merged ? (size_t)F * K : 0, ss ? nullptr : row_offsets, adapter_ids, R, m->n_adapters, w.meta, w.frame_of_row,
                           w.adapter_of_row, dev_status, st));
    // The lagged loop: after the shared layers the base head scores the frames, Alg. 2 turns the scores of frame t - 1 into
    // the adapter set of frame t, and the CSR check builds the row maps -- all on this stream, no host in between.
    bool selected = ss == nullptr;
    auto select_now = [&]() -> int {
        selected = true;
        const poly_stream *s = ss->s;
        POLY_TRY(launch_base_head(w.xa, T, D, base->lnf_g, base->lnf_b, m->ln_eps, s->base_w, s->base_b, s->K, F, ss->lag,
                                  ss->out_base_scores, s->carry, dt, st));
        POLY_TRY(poly_select(ss->lag, F, s->K, s->group_membership, s->M, &s->opts, s->state, ss->row_offsets, ss->adapter_ids, R,
                             ss->counters, stream));
        if (hipMemcpyAsync(s->carry, ss->lag + (size_t)F * s->K, sizeof(float) * (size_t)s->K, hipMemcpyDeviceToDevice, st) != hipSuccess)
            return POLY_EHIP;
        return launch_prep(ss->row_offsets, ss->adapter_ids, F, R, m->n_adapters, w.meta, w.frame_of_row, w.adapter_of_row, dev_status, st);
    };
    {
        GemmArgs g = {};
        g.A = w.patches; g.Wt = base->patch_w; g.bias = base->patch_b;
        g.T = T - 1; g.K = pd; g.N = D; g.n_in = F;
        g.mode = EPI_RESID; g.out = w.xa; g.Tout = T; g.t_off = 1; g.pos = base->pos;
        POLY_TRY(launch_gemm(g, dt, st));
    }

    bool qkv_done = false;                     // the qkv linear of layer l was computed by layer l - 1's row kernel
    for (int l = 0; l < m->L; ++l) {
        if (l == m->L0 && !selected) POLY_TRY(select_now());
        const bool lora_on = l >= m->L0 && R > 0;
        if (l >= m->L0 && R == 0) break;
        // Summed composition: the frame stays ONE block through the adapted layers; its adapters' low-rank terms
        // (one shrink per (frame, adapter) pair, as in the fan-out) are all added in the expand of the frame's block.
        const bool summed = sum && l >= m->L0;
        const bool fan = !sum && l == m->L0;   // first adapted layer: frames fan out into row-blocks
        const bool branch = !sum && l > m->L0; // residual stream already per row-block
        float *x_in = branch ? w.xb : w.xa;
        float *x_out = (!sum && l >= m->L0) ? w.xb : w.xa;
        const int nb = branch ? R : F;         // blocks of the LayerNorm-1 input
        const int *nb_dev = branch ? R_dev : (summed ? &w.meta->F_ok : nullptr);
        const int n_out = (!sum && l >= m->L0) ? R : F;  // blocks after the qkv linear
        const int *n_out_dev = (!sum && l >= m->L0) ? R_dev : (summed ? &w.meta->F_ok : nullptr);

        auto lora_ptr = [&](const void *stack, int t, size_t din, size_t dout, bool is_A) -> const void * {
            (void)t;
            const size_t per_layer = (size_t)m->n_adapters * m->r * (is_A ? din : dout);
            return (const char *)stack + es * per_layer * (size_t)(l - m->L0);
        };
        auto use = [&](int t) { return lora_on && (m->targets & (1 << t)); };

        // narrow models (D <= 192, bf16): LayerNorm, shrink, base product and expand of one linear run in one
        // kernel that keeps 64 token rows on chip; otherwise LayerNorm / shrink / GEMM are separate launches
        auto fused = [&](int t) { return dt == POLY_BF16 && !(summed && use(t)) && rowlin_supported(D, t == 0 ? 3 * D : (t == 2 ? Dm : D), m->r, use(t), t == 1); };
        // low-rank operands of the GEMM path: S block and adapter per (frame, adapter) pair; summed: the pairs of a frame
        // all land on the frame's block
        const int *shrink_map = summed ? w.frame_of_row : nullptr;
        auto lora_gemm = [&](GemmArgs &g, int t, const void *Bt) {
            g.S = w.S; g.RP = RP; g.Bt = Bt; g.r = m->r; g.adapter_of_out = w.adapter_of_row;
            g.set_off = summed ? row_offsets : nullptr;
            (void)t;
        };
        auto rowlin = [&](int t, const float *x_ln, const float *ln_g, const float *ln_b, const void *a_in, const int *in_map,
                          const void *Wt, const float *bias, int N, int mode, void *out, const float *res, const int *res_map) -> int {
            RowLinArgs a = {};
            a.x_ln = x_ln; a.ln_g = ln_g; a.ln_b = ln_b; a.eps = m->ln_eps; a.a_in = (const bf16_t *)a_in; a.in_block_of_out = in_map;
            a.T = T; a.K = D; a.N = N; a.n_out = n_out; a.n_out_dev = n_out_dev;
            a.Wt = (const bf16_t *)Wt; a.bias = bias;
            if (use(t)) {
                a.At = (const bf16_t *)lora_ptr(lora->At[t], t, D, N, true); a.Bt = (const bf16_t *)lora_ptr(lora->Bt[t], t, D, N, false);
                a.r = m->r; a.scale = m->lora_scale; a.adapter_of_out = w.adapter_of_row;
            }
            a.mode = mode; a.out = out; a.res = res; a.res_block_of_out = res_map;
            return launch_rowlin(a, st);
        };
        const int *fan_map = fan ? w.frame_of_row : nullptr;
        const void *Wqkv = (const char *)base->qkv_w + es * (size_t)l * 3 * D * D, *Wproj = (const char *)base->proj_w + es * (size_t)l * D * D;
        const void *Wfc1 = (const char *)base->fc1_w + es * (size_t)l * Dm * D;

        // ---- attention half
        if (qkv_done) {
            qkv_done = false;
        } else if (fused(0)) {
            POLY_TRY(rowlin(0, x_in, base->ln1_g + (size_t)l * D, base->ln1_b + (size_t)l * D, nullptr, fan_map, Wqkv,
                            base->qkv_b + (size_t)l * 3 * D, 3 * D, EPI_STORE, w.qkv, nullptr, nullptr));
        } else {
            POLY_TRY(launch_layernorm(x_in, w.u, base->ln1_g + (size_t)l * D, base->ln1_b + (size_t)l * D, D, m->ln_eps, T, nb, nb_dev, dt, st));
            GemmArgs g = {};
            g.A = w.u; g.Wt = Wqkv; g.bias = base->qkv_b + (size_t)l * 3 * D;
            g.T = T; g.K = D; g.N = 3 * D; g.n_in = nb; g.n_in_dev = fan ? &w.meta->F_ok : nb_dev;
            g.out_off = fan ? row_offsets : nullptr;
            if (use(0)) {
                const void *At = lora_ptr(lora->At[0], 0, D, 3 * D, true), *Bt = lora_ptr(lora->Bt[0], 0, D, 3 * D, false);
                POLY_TRY(launch_shrink(w.u, T, D, At, m->r, RP, m->lora_scale, R, R_dev, summed ? shrink_map : fan_map, w.adapter_of_row,
                                       (summed || fan) ? row_offsets : nullptr, w.S, dt, st));
                lora_gemm(g, 0, Bt);
            }
            g.mode = EPI_STORE; g.out = w.qkv; g.Tout = T;
            POLY_TRY(launch_gemm(g, dt, st));
        }
        POLY_TRY(launch_attention(w.qkv, w.o, T, D, m->heads, n_out, n_out_dev, dt, st));
        // narrow models without adapters on fc1 / fc2: everything row-wise of the layer in one launch -- proj with its
        // residual, the MLP half, and the qkv linear of the next layer when that layer works on the same blocks
        if (dt == POLY_BF16 && !use(2) && !use(3) && !(summed && (use(0) || use(1))) && rowlayer_supported(D, Dm, (use(0) || use(1)) ? m->r : 0)) {
            RowLayerArgs a = {};
            a.T = T; a.D = D; a.Dm = Dm; a.n_out = n_out; a.n_out_dev = n_out_dev;
            a.adapter_of_out = (lora_on && !sum) ? w.adapter_of_row : nullptr; a.r = m->r; a.scale = m->lora_scale; a.eps = m->ln_eps;
            a.o = (const bf16_t *)w.o; a.Wpt = (const bf16_t *)Wproj; a.bp = base->proj_b + (size_t)l * D;
            if (use(1)) { a.Apt = (const bf16_t *)lora_ptr(lora->At[1], 1, D, D, true); a.Bpt = (const bf16_t *)lora_ptr(lora->Bt[1], 1, D, D, false); }
            a.res = x_in; a.res_block_of_out = fan_map;
            a.ln2_g = base->ln2_g + (size_t)l * D; a.ln2_b = base->ln2_b + (size_t)l * D;
            a.W1t = (const bf16_t *)Wfc1; a.b1 = base->fc1_b + (size_t)l * Dm;
            a.W2t = (const bf16_t *)((const char *)base->fc2_w + es * (size_t)l * D * Dm); a.b2 = base->fc2_b + (size_t)l * D;
            a.x_out = x_out;
            const int ln = l + 1;              // next layer: same blocks unless it is the one where frames fan out
            const bool next_qkv_summed = sum && ln >= m->L0 && R > 0 && (m->targets & 1);   // that linear needs the GEMM path
            if (ln < m->L && (sum || ln != m->L0) && !next_qkv_summed) {
                a.lnq_g = base->ln1_g + (size_t)ln * D; a.lnq_b = base->ln1_b + (size_t)ln * D;
                a.Wqt = (const bf16_t *)((const char *)base->qkv_w + es * (size_t)ln * 3 * D * D); a.bq = base->qkv_b + (size_t)ln * 3 * D;
                if (!sum && ln >= m->L0 && R > 0 && (m->targets & 1)) {
                    const size_t per_layer = (size_t)m->n_adapters * m->r * D;
                    a.Aqt = (const bf16_t *)((const char *)lora->At[0] + es * per_layer * (size_t)(ln - m->L0));
                    a.Bqt = (const bf16_t *)((const char *)lora->Bt[0] + es * per_layer * 3 * (size_t)(ln - m->L0));
                }
                a.qkv_out = (bf16_t *)w.qkv;
                qkv_done = true;
            }
            POLY_TRY(launch_rowlayer(a, st));
            continue;
        }
        if (fused(1)) {
            POLY_TRY(rowlin(1, nullptr, nullptr, nullptr, w.o, nullptr, Wproj, base->proj_b + (size_t)l * D, D, EPI_RESID, x_out, x_in, fan_map));
        } else {
            GemmArgs g = {};
            g.A = w.o; g.Wt = Wproj; g.bias = base->proj_b + (size_t)l * D;
            g.T = T; g.K = D; g.N = D; g.n_in = n_out; g.n_in_dev = n_out_dev;
            if (use(1)) {
                const void *At = lora_ptr(lora->At[1], 1, D, D, true), *Bt = lora_ptr(lora->Bt[1], 1, D, D, false);
                POLY_TRY(launch_shrink(w.o, T, D, At, m->r, RP, m->lora_scale, R, R_dev, shrink_map, w.adapter_of_row, summed ? row_offsets : nullptr,
                                       w.S, dt, st));
                lora_gemm(g, 1, Bt);
            }
            g.mode = EPI_RESID; g.out = x_out; g.Tout = T; g.res = x_in; g.res_block_of_out = fan_map;
            POLY_TRY(launch_gemm(g, dt, st));
        }
        // ---- MLP half (x_out holds the stream from here on)
        if (dt == POLY_BF16 && !use(2) && !use(3) && mlp_supported(D, Dm)) {
            // no adapter on fc1 / fc2 in this layer: LayerNorm, both products, GELU and the residual in one kernel
            MlpArgs a = {};
            a.x = x_out; a.ln_g = base->ln2_g + (size_t)l * D; a.ln_b = base->ln2_b + (size_t)l * D; a.eps = m->ln_eps;
            a.T = T; a.D = D; a.Dm = Dm; a.n_out = n_out; a.n_out_dev = n_out_dev;
            a.W1t = (const bf16_t *)Wfc1; a.b1 = base->fc1_b + (size_t)l * Dm;
            a.W2t = (const bf16_t *)((const char *)base->fc2_w + es * (size_t)l * D * Dm); a.b2 = base->fc2_b + (size_t)l * D;
            POLY_TRY(launch_mlp(a, st));
            continue;
        }
        if (fused(2)) {
            POLY_TRY(rowlin(2, x_out, base->ln2_g + (size_t)l * D, base->ln2_b + (size_t)l * D, nullptr, nullptr, Wfc1,
                            base->fc1_b + (size_t)l * Dm, Dm, EPI_GELU, w.h, nullptr, nullptr));
        } else {
            POLY_TRY(launch_layernorm(x_out, w.u, base->ln2_g + (size_t)l * D, base->ln2_b + (size_t)l * D, D, m->ln_eps, T, n_out, n_out_dev, dt, st));
            GemmArgs g = {};
            g.A = w.u; g.Wt = Wfc1; g.bias = base->fc1_b + (size_t)l * Dm;
            g.T = T; g.K = D; g.N = Dm; g.n_in = n_out; g.n_in_dev = n_out_dev;
            if (use(2)) {
                const void *At = lora_ptr(lora->At[2], 2, D, Dm, true), *Bt = lora_ptr(lora->Bt[2], 2, D, Dm, false);
                POLY_TRY(launch_shrink(w.u, T, D, At, m->r, RP, m->lora_scale, R, R_dev, shrink_map, w.adapter_of_row, summed ? row_offsets : nullptr,
                                       w.S, dt, st));
                lora_gemm(g, 2, Bt);
            }
            g.mode = EPI_GELU; g.out = w.h; g.Tout = T;
            POLY_TRY(launch_gemm(g, dt, st));
        }
        {
            GemmArgs g = {};
            g.A = w.h; g.Wt = (const char *)base->fc2_w + es * (size_t)l * D * Dm; g.bias = base->fc2_b + (size_t)l * D;
            g.T = T; g.K = Dm; g.N = D; g.n_in = n_out; g.n_in_dev = n_out_dev;
            if (use(3)) {
                const void *At = lora_ptr(lora->At[3], 3, Dm, D, true), *Bt = lora_ptr(lora->Bt[3], 3, Dm, D, false);
                POLY_TRY(launch_shrink(w.h, T, Dm, At, m->r, RP, m->lora_scale, R, R_dev, shrink_map, w.adapter_of_row, summed ? row_offsets : nullptr,
                                       w.S, dt, st));
                lora_gemm(g, 3, Bt);
            }
            g.mode = EPI_RESID; g.out = x_out; g.Tout = T; g.res = x_out;
            POLY_TRY(launch_gemm(g, dt, st));
        }
    }

    if (!selected) POLY_TRY(select_now());        // (L0 == L: the shared layers are the whole backbone)
    if (R > 0) {
        POLY_TRY(launch_head((adapted && !sum) ? w.xb : w.xa, (adapted && !sum) ? nullptr : w.frame_of_row, T, D, base->lnf_g, base->lnf_b, m->ln_eps,
                             heads->head_w, heads->head_b, m->C, w.adapter_of_row, w.frame_of_row, heads->class_map, K, w.meta, R,
                             out_logits, out_scores, out_merged, dt, st));
    }
    return POLY_OK;
}
}  // namespace

extern "C" int poly_forward(const poly_model_desc *m, const poly_base_weights *base, const poly_lora_weights *lora,
                            const poly_heads *heads, const void *frames, int F, const int32_t *row_offsets,
                            const int32_t *adapter_ids, int R, float *out_logits, float *out_scores, float *out_merged, int K,
                            int32_t *dev_status, void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_impl(m, base, lora, heads, frames, F, row_offsets, adapter_ids, R, out_logits, out_scores, out_merged, K, dev_status,
                        workspace, workspace_bytes, stream, nullptr);
}

static size_t stream_lag_offset(const poly_model_desc *m, int F, int R)
{
    return (carve_forward(m, F, R, nullptr).bytes + 255) & ~(size_t)255;
}

extern "C" size_t poly_stream_step_workspace_bytes(const poly_model_desc *m, int F, int R, int K)
{
    if (check_model(m) != POLY_OK || F < 0 || R < 0 || K <= 0) return 0;
    return stream_lag_offset(m, F, R) + sizeof(float) * (size_t)(F + 1) * K;
}

extern "C" int poly_stream_step(const poly_model_desc *m, const poly_base_weights *base, const poly_lora_weights *lora,
                                const poly_heads *heads, const poly_stream *s, const void *frames, int F, int R,
                                int32_t *row_offsets, int32_t *adapter_ids, int32_t *counters, float *out_base_scores,
                                float *out_logits, float *out_scores, float *out_merged, int32_t *dev_status, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    POLY_TRY(check_model(m));
    if (!s || !s->base_w || !s->base_b || !s->group_membership || !s->carry || !counters) return POLY_EINVAL;
    if (s->K <= 0 || s->K > POLY_MAX_LABELS || s->M <= 0 || s->M > POLY_MAX_CONTEXTS || s->M > m->n_adapters) return POLY_EINVAL;
    if (F < 0 || R < 0) return POLY_EINVAL;
    if (F == 0) return POLY_OK;
    if (!workspace || ((uintptr_t)workspace & 255) != 0) return POLY_EINVAL;
    if (workspace_bytes < poly_stream_step_workspace_bytes(m, F, R, s->K)) return POLY_ECAP;
    StreamStep ss = {s, row_offsets, adapter_ids, counters, out_base_scores, (float *)((char *)workspace + stream_lag_offset(m, F, R))};
    return forward_impl(m, base, lora, heads, frames, F, row_offsets, adapter_ids, R, out_logits, out_scores, out_merged, s->K, dev_status,
                        workspace, workspace_bytes, stream, &ss);
}

// ------------------------------------------------------------------ isolated multi-LoRA linear

namespace {
struct LinearWs {
    PolyMeta *meta;
    int32_t *frame_of_row, *adapter_of_row;
    void *S;
    size_t bytes;
};
LinearWs carve_linear(int T, int r, int R, int dtype, void *base)
{
    Carver c{(char *)base, 0};
    LinearWs w;
    w.meta = c.take<PolyMeta>(sizeof(PolyMeta));
    w.frame_of_row = c.take<int32_t>(sizeof(int32_t) * (size_t)(R + 1));
    w.adapter_of_row = c.take<int32_t>(sizeof(int32_t) * (size_t)(R + 1));
    w.S = c.take<void>(elt_size(dtype) * (size_t)R * T * rank_pad(r));
    w.bytes = c.off;
    return w;
}
}  // namespace

extern "C" size_t poly_lora_linear_workspace_bytes(int n_xblocks, int T, int r, int R, int dtype)
{
    if (n_xblocks < 0 || T <= 0 || r <= 0 || R < 0 || (dtype != POLY_F32 && dtype != POLY_BF16)) return 0;
    return carve_linear(T, r, R, dtype, nullptr).bytes;
}

namespace {
int lora_linear_impl(const void *X, int n_xblocks, int T, int Kdim, const void *Wt, const float *bias, int Ndim, const void *At,
                     const void *Bt, int n_adapters, int r, float scale, const int32_t *row_offsets, const int32_t *adapter_ids, int R,
                     void *Y, int dtype, int32_t *dev_status, void *workspace, size_t workspace_bytes, void *stream)
{
    const LinearWs w = carve_linear(T, r, R, dtype, workspace);
    if (workspace_bytes < w.bytes) return POLY_ECAP;
    hipStream_t st = (hipStream_t)stream;
    const int RP = rank_pad(r);

    POLY_TRY(launch_prep(row_offsets, adapter_ids, n_xblocks, R, n_adapters, w.meta, w.frame_of_row, w.adapter_of_row, dev_status, st));
    if (R == 0) return POLY_OK;
    POLY_TRY(launch_shrink(X, T, Kdim, At, r, RP, scale, R, &w.meta->R, w.frame_of_row, w.adapter_of_row, row_offsets, w.S, dtype, st));
    GemmArgs g = {};
    g.A = X; g.Wt = Wt; g.bias = bias; g.T = T; g.K = Kdim; g.N = Ndim;
    g.n_in = n_xblocks; g.n_in_dev = &w.meta->F_ok; g.out_off = row_offsets;
    g.S = w.S; g.RP = RP; g.Bt = Bt; g.r = r; g.adapter_of_out = w.adapter_of_row;
    g.mode = EPI_STORE; g.out = Y; g.Tout = T;
    return launch_gemm(g, dtype, st);
}

int check_lora_linear(const void *X, int n_xblocks, int T, int Kdim, const void *Wt, int Ndim, const void *At, const void *Bt,
                      int n_adapters, int r, const int32_t *row_offsets, const int32_t *adapter_ids, int R, void *Y, int dtype)
{
    if (dtype != POLY_F32 && dtype != POLY_BF16) return POLY_EINVAL;
    if (n_xblocks < 0 || T <= 0 || Kdim <= 0 || Ndim <= 0 || n_adapters <= 0 || r <= 0 || r > POLY_MAX_RANK || R < 0) return POLY_EINVAL;
    if (Kdim % (dtype == POLY_BF16 ? 8 : 4)) return POLY_EINVAL;
    if (n_xblocks == 0) return POLY_OK;
    if (!X || !Wt || !At || !Bt || !row_offsets || (R > 0 && (!adapter_ids || !Y))) return POLY_EINVAL;
    return POLY_OK;
}
}  // namespace

extern "C" int poly_lora_linear(const void *X, int n_xblocks, int T, int Kdim, const void *Wt, const float *bias, int Ndim,
                                const void *At, const void *Bt, int n_adapters, int r, float scale, const int32_t *row_offsets,
                                const int32_t *adapter_ids, int R, void *Y, int dtype, int32_t *dev_status, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    POLY_TRY(check_lora_linear(X, n_xblocks, T, Kdim, Wt, Ndim, At, Bt, n_adapters, r, row_offsets, adapter_ids, R, Y, dtype));
    if (n_xblocks == 0) return POLY_OK;
    if (!workspace || ((uintptr_t)workspace & 255) != 0) return POLY_EINVAL;
    return lora_linear_impl(X, n_xblocks, T, Kdim, Wt, bias, Ndim, At, Bt, n_adapters, r, scale, row_offsets, adapter_ids, R, Y, dtype,
                            dev_status, workspace, workspace_bytes, stream);
}

// ------------------------------------------------------------------ isolated linear without a caller workspace
// For callers that cannot allocate (code under graph capture, serving loops, harnesses that forbid hipMalloc): the bookkeeping,
// the row maps and the shrink output S live in a file-scope device array instead of a workspace argument.  Each GPU the library
// is loaded on holds its own copy of the array; its address on a device is looked up once, with that device current.
static __device__ __align__(256) unsigned char scratch[POLY_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void *scratch_of_device[MAX_DEVICES];          // device address of `scratch` per device ordinal, null until looked up

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return POLY_EHIP;
    void *p = __atomic_load_n(&scratch_of_device[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return POLY_EHIP;
        __atomic_store_n(&scratch_of_device[dev], p, __ATOMIC_RELEASE);   // (two racing first calls look up the same address)
    }
    *out = p;
    return POLY_OK;
}
}  // namespace

extern "C" int poly_lora_linear_static(const void *X, int n_xblocks, int T, int Kdim, const void *Wt, const float *bias, int Ndim,
                                       const void *At, const void *Bt, int n_adapters, int r, float scale,
                                       const int32_t *row_offsets, const int32_t *adapter_ids, int R, void *Y, int dtype,
                                       int32_t *dev_status, void *stream)
{
    POLY_TRY(check_lora_linear(X, n_xblocks, T, Kdim, Wt, Ndim, At, Bt, n_adapters, r, row_offsets, adapter_ids, R, Y, dtype));
    if (n_xblocks == 0) return POLY_OK;
    if (carve_linear(T, r, R, dtype, nullptr).bytes > (size_t)POLY_STATIC_SCRATCH_BYTES) return POLY_ECAP;
    void *ws = nullptr;
    POLY_TRY(static_scratch(&ws));
    // nothing in the scratch area has to start at zero: the CSR check writes the bookkeeping words and the row maps of every
    // row it accepts, and the shrink writes all RP columns of every S row the product reads
    return lora_linear_impl(X, n_xblocks, T, Kdim, Wt, bias, Ndim, At, Bt, n_adapters, r, scale, row_offsets, adapter_ids, R, Y, dtype,
                            dev_status, ws, POLY_STATIC_SCRATCH_BYTES, stream);
}
