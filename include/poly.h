/*
 * libpoly -- MI355X (gfx950) hot path of Polymorph: per-frame context selection and the
 * forward of a shared ViT backbone whose frames each run their own unmerged LoRA adapters.
 *
 * Conventions
 *   - Plain C ABI.  Every tensor pointer is a DEVICE pointer unless it says "host".
 *     The structs themselves (poly_model_desc, poly_base_weights, ...) live in host memory.
 *   - The caller owns every buffer.  The entry points of this header allocate no device or
 *     host memory and keep no state between calls; scratch memory comes in through
 *     `workspace` (poly_lora_linear_static: the library's own static array).  The measurement
 *     hooks in poly_profile.h are outside this contract.
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  Outputs are valid once the stream has been synchronised.
 *   - Return value: POLY_OK or a negative poly_status.  Conditions that only the device can
 *     see (an adapter id out of range, offsets that are not monotone) are written to the
 *     `dev_status` word by the first kernel; the affected call then computes nothing.
 *   - Matrices are stored with the contraction index fastest.  In the paper's notation a
 *     linear is y = x W + b with W in R^{D_in x D_out} and an adapter is A in R^{D_in x r},
 *     B in R^{r x D_out} (Sec. 3.1); this library takes their column-major images
 *         W -> Wt[D_out][D_in],   A -> At[r][D_in],   B -> Bt[D_out][r].
 *     "elt" below is float for POLY_F32 and bf16 (uint16 bit pattern) for POLY_BF16; vectors
 *     (biases, LayerNorm gains and shifts, cls, pos) are always float.
 *   - Row-block b = (frame f, adapter k): frame f's adapters are
 *     adapter_ids[row_offsets[f] .. row_offsets[f+1]) -- the CSR image of the active context
 *     sets S_t of Sec. 3.3; adapter id = context id.
 */
#ifndef POLY_H
#define POLY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum poly_status {
    POLY_OK = 0,
    POLY_EINVAL = -1, /* null pointer, bad shape, unsupported size or enum */
    POLY_ERANGE = -2, /* adapter id outside [0, n_adapters), offsets not monotone, R above its bound */
    POLY_ECAP = -3,   /* an output or the workspace is too small */
    POLY_EHIP = -4    /* the HIP runtime reported an error */
} poly_status;

enum { POLY_F32 = 0, POLY_BF16 = 1 };
enum { POLY_TGT_QKV = 1, POLY_TGT_PROJ = 2, POLY_TGT_FC1 = 4, POLY_TGT_FC2 = 8 };
/* How a frame's several active adapters are applied (Sec. 3.1 / Fig. 3b leave both readings open):
 *   POLY_COMPOSE_BRANCH  one branch per (frame, adapter): row-block (f, k) runs layers [L0, L) with adapter k alone;
 *   POLY_COMPOSE_SUM     one hidden state per frame with all of its adapters summed on top of the shared weights,
 *                        linear(x) = x W + b + sum_{k in S_f} lora_scale (x A_k) B_k, read by each active adapter's head. */
enum { POLY_COMPOSE_BRANCH = 0, POLY_COMPOSE_SUM = 1 };

/* Limits of this build. */
enum {
    POLY_MAX_CONTEXTS = 64,  /* M: one 64-bit set per frame */
    POLY_MAX_LABELS = 1024,  /* K */
    POLY_MAX_RANK = 64,      /* r */
    POLY_MAX_HEAD_CLASSES = 64,
    POLY_HEAD_DIM = 64       /* D / heads must be 64 */
};

const char *poly_status_string(int status);

/* ------------------------------------------------------------------------------------------
 * poly_select -- context detection for a batch of consecutive frames of one stream
 * (Alg. 2, Sec. 3.5; the cover constraint is Eq. 2).
 *
 *   Y_t = { l : label_scores[t][l] >= theta }                     (the monitor of Sec. 3.2)
 *   Y_t == Y_{t-1}                                    -> S_t = S_{t-1}
 *   context_copy and S_{t-1} provides every l in Y_t  -> S_t = S_{t-1}
 *   else scan the contexts by (size ascending, id ascending) and take a context iff it provides a
 *   label that is still uncovered, until none is left.
 * Context C provides label l iff group_membership[C][l] != 0 and (acc == NULL or acc[C][l] >= tau).
 *
 *   label_scores      [F][K] float.
 *   group_membership  [M][K] uint8, 1 iff label l is in context C_m.  M <= 64, K <= 1024.
 *   opts              host struct below.
 *   state             device buffer of poly_select_state_bytes(K) bytes carrying (Y_{t-1}, S_{t-1})
 *                     between calls; all-zero = "no previous frame"; NULL = stateless call.
 *                     Read and updated by the call.
 *   row_offsets       [F+1] int32 out.
 *   adapter_ids       [cap] int32 out, selection order inside a frame.  Ids past `cap` are dropped.
 *   counters          [2] int32 out: counters[0] = R = total number of (frame, context) rows needed
 *                     (compare with cap: R > cap means adapter_ids is truncated), counters[1] =
 *                     number of (frame, label) pairs of Y_t that no context of S_t provides.
 * Frames are independent unless a state is given or context_copy is set; then a short sequential
 * pass resolves the reuse branches.  Errors: POLY_EINVAL for null/size violations, POLY_EHIP.
 */
typedef struct poly_select_opts {
    float theta;          /* label threshold, >= is active (0.5) */
    int32_t context_copy; /* 0 = the paper's main variant */
    const float *acc;     /* device [M][K] accuracy table a_{C,l}, or NULL */
    float tau;            /* minimum accuracy, used only with acc */
} poly_select_opts;

size_t poly_select_state_bytes(int K);

int poly_select(const float *label_scores, int F, int K, const uint8_t *group_membership, int M,
                const poly_select_opts *opts, void *state, int32_t *row_offsets, int32_t *adapter_ids,
                int cap, int32_t *counters, void *stream);

/* ------------------------------------------------------------------------------------------
 * poly_forward -- forward of F frames through the shared backbone, each (frame, adapter)
 * row-block as its own branch (Sec. 3.1, Fig. 2; inference path of Fig. 3b):
 *   tokens: patch embedding of the NHWC frame (patch vector index (i*patch + j)*3 + c) + class
 *   token + position table; layers [0, L0) once per frame, without adapters; layers [L0, L) per
 *   row-block with adapter k alone,
 *       linear_k(x) = x W + b + lora_scale * (x A_k) B_k      on the linears named in `targets`,
 *   inside the usual pre-LayerNorm block (softmax attention with 64-wide heads, exact-erf GELU
 *   MLP, residuals); then LayerNorm of the class token and adapter k's own head:
 *       logits[b] = LN(x_b[0]) H_k + hb_k,   scores[b] = sigmoid(logits[b]).
 *   W + A_k B_k is never formed.
 *
 *   frames        [F][H][W][3] elt.
 *   row_offsets   [F+1] int32, adapter_ids [>= row_offsets[F]] int32 (device).
 *   R             host upper bound of row_offsets[F]; the kernels read the true value on the device,
 *                 so the output of poly_select can be consumed without a host round trip.
 *   out_logits    [R][C] float, nullable.   out_scores [R][C] float.
 *   out_merged    [F][K] float, nullable (needs heads->class_map): score of class
 *                 class_map[k][c] from row-block (f,k), maximum where adapters overlap, 0 where no
 *                 active adapter reports the class.
 *   dev_status    device int32, nullable: POLY_OK or POLY_ERANGE after the call.
 *   workspace     >= poly_forward_workspace_bytes(m, F, R) bytes, 256-byte aligned.
 * Rows past row_offsets[F] are left untouched.  Results do not depend on where a frame sits in
 * the batch (fixed reduction order, no atomics on floating-point sums).
 * Shape limits (POLY_EINVAL otherwise): D == 64 * heads; 1 <= r <= 64; 1 <= C <= 64; H, W multiples of patch;
 * POLY_BF16: T = 1 + (H/patch)(W/patch) <= 224 tokens (a block's keys stay on chip), Dm % 8 == 0 and
 * (3 * patch * patch) % 8 == 0 (16-byte loads along the contraction index); POLY_F32: both % 4 == 0.
 * With POLY_COMPOSE_SUM the rows of out_logits / out_scores are the same (frame, adapter) pairs in CSR order, each
 * adapter's head reading its frame's one hidden state.
 */
typedef struct poly_model_desc {
    int32_t H, W, patch;  /* frame size and patch edge; H, W multiples of patch */
    int32_t D, heads;     /* model width; D == 64 * heads */
    int32_t L, Dm;        /* layers, MLP width */
    int32_t L0;           /* first adapted layer, 0 <= L0 <= L (L - L0 = final 20 % in the paper) */
    int32_t targets;      /* POLY_TGT_* mask of adapted linears */
    int32_t r;            /* LoRA rank */
    int32_t n_adapters;   /* N_ad */
    int32_t C;            /* classes per adapter head */
    int32_t dtype;        /* POLY_F32 or POLY_BF16 */
    float lora_scale;     /* s */
    float ln_eps;
    int32_t compose;      /* POLY_COMPOSE_BRANCH (0) or POLY_COMPOSE_SUM */
} poly_model_desc;

typedef struct poly_base_weights {
    const void *patch_w;  /* elt [D][3*patch*patch] */
    const float *patch_b; /* [D] */
    const float *cls;     /* [D] */
    const float *pos;     /* [T][D], T = 1 + (H/patch)*(W/patch) */
    /* stacked over the L layers: */
    const float *ln1_g, *ln1_b; /* [L][D] */
    const void *qkv_w;          /* elt [L][3D][D]; output columns ordered q | k | v */
    const float *qkv_b;         /* [L][3D] */
    const void *proj_w;         /* elt [L][D][D] */
    const float *proj_b;        /* [L][D] */
    const float *ln2_g, *ln2_b; /* [L][D] */
    const void *fc1_w;          /* elt [L][Dm][D] */
    const float *fc1_b;         /* [L][Dm] */
    const void *fc2_w;          /* elt [L][D][Dm] */
    const float *fc2_b;         /* [L][D] */
    const float *lnf_g, *lnf_b; /* [D] */
} poly_base_weights;

typedef struct poly_lora_weights {
    /* index 0 qkv, 1 proj, 2 fc1, 3 fc2; NULL for linears not in `targets` */
    const void *At[4]; /* elt [L-L0][N_ad][r][D_in] */
    const void *Bt[4]; /* elt [L-L0][N_ad][D_out][r] */
} poly_lora_weights;

typedef struct poly_heads {
    const void *head_w;       /* elt [N_ad][C][D] */
    const float *head_b;      /* [N_ad][C] */
    const int32_t *class_map; /* [N_ad][C] -> label index in [0, K), nullable */
} poly_heads;

size_t poly_forward_workspace_bytes(const poly_model_desc *m, int F, int R);

int poly_forward(const poly_model_desc *m, const poly_base_weights *base, const poly_lora_weights *lora,
                 const poly_heads *heads, const void *frames, int F, const int32_t *row_offsets,
                 const int32_t *adapter_ids, int R, float *out_logits, float *out_scores,
                 float *out_merged, int K, int32_t *dev_status, void *workspace, size_t workspace_bytes,
                 void *stream);

/* ------------------------------------------------------------------------------------------
 * poly_stream_step -- the inference loop of Fig. 3b on F consecutive frames of one stream, with the
 * one-frame lag of Sec. 3.2 (the adapters of a frame are chosen from the labels seen on the frame
 * before), everything on the device:
 *   layers [0, L0) once per frame;
 *   base head on the class token of their output:
 *       base_scores[t] = sigmoid(LN_f(x_t[0]) base_w^T + base_b)                 [F][K];
 *   Alg. 2 (poly_select, same options and state) on the lagged scores
 *       (carry, base_scores[0], ..., base_scores[F-2])  ->  S_0 .. S_{F-1} as CSR arrays;
 *   layers [L0, L), heads and merge as in poly_forward on those row-blocks;
 *   carry = base_scores[F-1] for the next call.
 * A zeroed carry means "no previous frame": no label is active and the first frame runs without
 * adapters.
 *
 *   s              host struct below; base_w elt [K][D], base_b [K] float, group_membership [M][K]
 *                  uint8, state as in poly_select (nullable), carry device [K] float, in/out.
 *   R              capacity of adapter_ids and of the per-row-block outputs.  If the selection needs
 *                  more rows, counters[0] > R reports it, dev_status becomes POLY_ERANGE and no
 *                  row-block output is written.
 *   row_offsets    [F+1] int32 out, adapter_ids [R] int32 out, counters [2] int32 out (poly_select).
 *   out_base_scores [F][K] float, nullable.  out_logits / out_scores [R][C], out_merged [F][K]
 *                  (label space of the base head; needs heads->class_map) as in poly_forward.
 *   workspace      >= poly_stream_step_workspace_bytes(m, F, R, K) bytes, 256-byte aligned.
 * Errors as poly_forward and poly_select.
 */
typedef struct poly_stream {
    const void *base_w;  /* elt [K][D] */
    const float *base_b; /* [K] */
    int32_t K;           /* labels, <= POLY_MAX_LABELS */
    int32_t M;           /* contexts = adapters that can be selected, <= POLY_MAX_CONTEXTS */
    const uint8_t *group_membership; /* device [M][K] */
    poly_select_opts opts;
    void *state;  /* device, poly_select_state_bytes(K) bytes, or NULL */
    float *carry; /* device [K] */
} poly_stream;

size_t poly_stream_step_workspace_bytes(const poly_model_desc *m, int F, int R, int K);

int poly_stream_step(const poly_model_desc *m, const poly_base_weights *base, const poly_lora_weights *lora,
                     const poly_heads *heads, const poly_stream *s, const void *frames, int F, int R,
                     int32_t *row_offsets, int32_t *adapter_ids, int32_t *counters, float *out_base_scores,
                     float *out_logits, float *out_scores, float *out_merged, int32_t *dev_status,
                     void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * poly_lora_linear -- one multi-adapter linear in isolation (Sec. 3.1: h = xW + xAB with the
 * adapters applied side by side on a shared W).  Row-block b = (X block f, adapter k):
 *       Y[b] = X[f] Wt^T + bias + scale * (X[f] At_k^T) Bt_k^T.
 *   X [n_xblocks][T][Kdim] elt;  Wt [Ndim][Kdim] elt;  bias [Ndim] float, nullable;
 *   At [N_ad][r][Kdim] elt;  Bt [N_ad][Ndim][r] elt;
 *   row_offsets [n_xblocks+1], adapter_ids [R] as in poly_forward (R = host upper bound);
 *   Y [R][T][Ndim] elt.   The base product X[f] Wt^T is computed once per X block and reused by
 *   all row-blocks of that block.
 *   workspace >= poly_lora_linear_workspace_bytes(...) bytes.
 */
size_t poly_lora_linear_workspace_bytes(int n_xblocks, int T, int r, int R, int dtype);

int poly_lora_linear(const void *X, int n_xblocks, int T, int Kdim, const void *Wt, const float *bias,
                     int Ndim, const void *At, const void *Bt, int n_adapters, int r, float scale,
                     const int32_t *row_offsets, const int32_t *adapter_ids, int R, void *Y, int dtype,
                     int32_t *dev_status, void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Offline half of the selector, on HOST memory (no device work, no stream): context construction and the quality
 * metrics of Sec. 3.4.
 *
 * poly_build_contexts -- Alg. 1: label contexts from a co-occurrence matrix.
 *   cooc [K][K] float, host: cooc[i][j] (i != j) = how often labels i and j occur together, cooc[l][l] = how often
 *   l occurs.  A label is valid iff its row has a non-zero entry.  Valid labels are visited by descending
 *   cooc[l][l] (ties: lower id); a visited label (skipped when overlap is off and it is assigned already) forms a
 *   cluster with its up to B - 1 strongest neighbours (cooc[l][j] > 0, ties: lower id; overlap off: unassigned
 *   labels only); the cluster becomes a context iff no equal context exists and fewer than M_max exist.  Valid
 *   labels left in no context are then put, in the same order, into the context with fewer than B labels that
 *   maximises the sum of cooc[l][j] over its labels (ties: lower context id); labels for which no context has room
 *   are counted in n_unplaced (nullable).
 *   group_membership [M_max][K] uint8, host, out (rows past *n_contexts are zero): the layout poly_select reads.
 *   K <= 1024, M_max <= 64, B >= 1.  Errors: POLY_EINVAL.
 *
 * poly_intra_coherence -- Eq. 6: mean over contexts of the mean of co(i, j) = cooc[i][j] / norm over ordered pairs
 *   i != j inside the context; contexts with fewer than two labels contribute 0.
 *
 * poly_stream_metrics -- AvgCoverage = (1/F) sum_t |S_t| and SwitchPenalty = sum_{t >= 1} [S_t != S_{t-1}] (Sec. 3.4)
 *   of the context sets that poly_select wrote (CSR arrays copied to the host); sets compare as sets.
 *   Errors: POLY_EINVAL, POLY_ERANGE (ids outside [0, M), offsets not monotone).
 */
int poly_build_contexts(const float *cooc, int K, int B, int M_max, int allow_overlap, uint8_t *group_membership,
                        int32_t *n_contexts, int32_t *n_unplaced);
int poly_intra_coherence(const float *cooc, int K, double norm, const uint8_t *group_membership, int M, double *out);
int poly_stream_metrics(const int32_t *row_offsets, const int32_t *adapter_ids, int F, int M, double *avg_coverage,
                        int64_t *switch_penalty);

/* ------------------------------------------------------------------------------------------
 * poly_lora_linear_static -- poly_lora_linear for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and same results, but
 * the scratch memory (bookkeeping words, row maps, shrink output S) is a device array of POLY_STATIC_SCRATCH_BYTES
 * bytes inside the library instead of a workspace argument.  Every GPU the library runs on holds that array until the
 * process ends.  The call allocates and frees nothing; the first call on a device looks up the array's address on that
 * device (make that first call outside a graph capture).
 *   Limit: poly_lora_linear_workspace_bytes(n_xblocks, T, r, R, dtype) <= POLY_STATIC_SCRATCH_BYTES, else POLY_ECAP
 *   and nothing is launched (bf16, T = 197, r <= 16: R <= 664 row-blocks).
 *   All calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams or
 *   threads) race on it; calls on one stream are ordered and safe.  The array keeps the last call's contents; nothing
 *   in it needs clearing between calls.
 */
enum { POLY_STATIC_SCRATCH_BYTES = 4 * 1024 * 1024 };

int poly_lora_linear_static(const void *X, int n_xblocks, int T, int Kdim, const void *Wt, const float *bias,
                            int Ndim, const void *At, const void *Bt, int n_adapters, int r, float scale,
                            const int32_t *row_offsets, const int32_t *adapter_ids, int R, void *Y, int dtype,
                            int32_t *dev_status, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* POLY_H */
