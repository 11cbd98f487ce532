// Context detection (Alg. 2, Sec. 3.5): label threshold -> greedy cover by contexts in (size, id)
// order -> CSR adapter sets.  Integer work on 64-bit sets, one workgroup per call: a batch is
// F x K = 64 x 80 scores, so latency, not throughput, is what matters.
//
// Label sets are bitsets built with wave ballots (one 64-label word per ballot, coalesced score
// reads).  Contexts are renumbered by scan position, so a context set is a 64-bit mask whose
// ascending bit order IS the selection order.  Frames are covered in parallel (one thread each);
// the reuse branches of Alg. 2 need the previous frame's result and are resolved by a short
// sequential pass that only runs when a state is carried or context_copy is set.
#include "poly_dev.h"

#include <type_traits>

namespace {

constexpr int CH = 128;  // frames per pass
constexpr int KWMAX = POLY_MAX_LABELS / 64;
constexpr int MMAX = POLY_MAX_CONTEXTS;

struct SelState {       // device image of (Y_{t-1}, S_{t-1})
    int32_t valid, pad;
    uint64_t set_ids;   // S_{t-1} as a mask over context ids
    uint64_t labels[1]; // KW words
};

__global__ __launch_bounds__(256) void select_kernel(const float *scores, int F, int K, const uint8_t *member, int M, float theta,
                                                     int context_copy, const float *acc, float tau, SelState *state,
                                                     int32_t *row_offsets, int32_t *adapter_ids, int cap, int32_t *counters)
{
    __shared__ int size_of[MMAX];
    __shared__ int order[MMAX];                // scan position -> context id
    __shared__ uint64_t cmask[MMAX][KWMAX];    // labels that the context at a scan position provides
    __shared__ uint64_t mem_id[MMAX][KWMAX], prov_id[MMAX][KWMAX];   // member / provided labels by context id
    __shared__ uint64_t Y[CH][KWMAX];          // Y_t
    __shared__ uint64_t S[CH];                 // S_t as a mask over scan positions
    __shared__ int cnt[CH];
    __shared__ int unc[CH];
    __shared__ uint64_t prevY[KWMAX], prevProv[KWMAX];
    __shared__ uint64_t prevS;
    __shared__ int prevValid, total, total_unc, lead_s;
    __shared__ int wtot[4], wunc[4];           // per wave: selected contexts, uncovered labels (scan below)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int KW = (K + 63) / 64;

    // Membership and provided-label bitsets per (context id, 64-label word), one ballot each.  The loads of eight
    // words are requested together (a loop that loads, ballots and stores one word at a time pays a full memory
    // round trip per word), with clamped addresses instead of per-lane conditions.
    for (int w0 = wave * 8; w0 < M * KW; w0 += 32) {
        uint8_t mb[8];
        float ac[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int w = min(w0 + u, M * KW - 1), c = w / KW, l = min((w % KW) * 64 + lane, K - 1);
            mb[u] = member[(size_t)c * K + l];
            ac[u] = acc ? acc[(size_t)c * K + l] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int w = w0 + u;
            if (w < M * KW) {     // uniform
                const bool in = (w % KW) * 64 + lane < K, mem = in && mb[u] != 0;
                const uint64_t mm = __ballot(mem), pm = __ballot(mem && (acc == nullptr || ac[u] >= tau));
                if (lane == 0) { mem_id[w / KW][w % KW] = mm; prov_id[w / KW][w % KW] = pm; }
            }
        }
    }
    __syncthreads();
    // contexts in scan order: size ascending, id ascending
    if (tid < M) {
        int sz = 0;
        for (int j = 0; j < KW; ++j) sz += __popcll(mem_id[tid][j]);
        size_of[tid] = sz;
    }
    __syncthreads();
    if (tid < M) {
        int rank = 0;
        for (int c = 0; c < M; ++c) rank += (size_of[c] < size_of[tid] || (size_of[c] == size_of[tid] && c < tid)) ? 1 : 0;
        order[rank] = tid;
    }
    __syncthreads();
    for (int w = tid; w < M * KW; w += 256) cmask[w / KW][w % KW] = prov_id[order[w / KW]][w % KW];
    if (tid == 0) {
        total = 0; total_unc = 0; prevS = 0; prevValid = 0;
        if (state && state->valid) {
            prevValid = 1;
            uint64_t pos_mask = 0;
            for (int pos = 0; pos < M; ++pos)
                if ((state->set_ids >> order[pos]) & 1ull) pos_mask |= 1ull << pos;
            prevS = pos_mask;
        }
    }
    if (tid < KW) prevY[tid] = (state && state->valid) ? state->labels[tid] : 0ull;
    __syncthreads();
    if (tid < KW) {
        uint64_t pv = 0;
        for (int pos = 0; pos < M; ++pos)
            if ((prevS >> pos) & 1ull) pv |= cmask[pos][tid];
        prevProv[tid] = pv;
    }
    if (tid == 0) row_offsets[0] = 0;
    const bool sequential = state != nullptr || context_copy != 0;

    for (int f0 = 0; f0 < F; f0 += CH) {
        const int n = min(CH, F - f0);
        __syncthreads();
        // Y_t: one ballot per 64 labels, the scores of eight words requested together (see above)
        for (int w0 = wave * 8; w0 < n * KW; w0 += 32) {
            float sv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int w = min(w0 + u, n * KW - 1);
                sv[u] = scores[(size_t)(f0 + w / KW) * K + min((w % KW) * 64 + lane, K - 1)];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int w = w0 + u;
                if (w < n * KW) {     // uniform
                    const uint64_t m = __ballot((w % KW) * 64 + lane < K && sv[u] >= theta);
                    if (lane == 0) Y[w / KW][w % KW] = m;
                }
            }
        }
        __syncthreads();
        // greedy cover, one frame per thread; the uncovered set stays in registers (a round trip through LDS per scan position
        // and word made this the longest phase of the kernel)
        if (tid < n) {
            // NW: compile-time bound of the words per label set (the registers are indexed by unrolled loops)
            auto greedy = [&](auto NWC) {
                constexpr int NW = decltype(NWC)::value;
                uint64_t u[NW];
                bool left = false;
#pragma unroll
                for (int j = 0; j < NW; ++j) {
                    u[j] = j < KW ? Y[tid][j] : 0ull;
                    left |= u[j] != 0;
                }
                uint64_t sel = 0;
                for (int pos = 0; pos < M && left; ++pos) {
                    bool got = false;
#pragma unroll
                    for (int j = 0; j < NW; ++j)
                        if (NW <= 2 || j < KW) got |= (u[j] & cmask[pos][j]) != 0;
                    if (got) {
                        sel |= 1ull << pos;
                        left = false;
#pragma unroll
                        for (int j = 0; j < NW; ++j)
                            if (NW <= 2 || j < KW) { u[j] &= ~cmask[pos][j]; left |= u[j] != 0; }
                    }
                }
                S[tid] = sel;
                int nu = 0;
#pragma unroll
                for (int j = 0; j < NW; ++j) nu += __popcll(u[j]);
                unc[tid] = nu;                   // uncovered labels of the greedy result (recomputed below if a set is reused)
            };
            if (KW <= 2) greedy(std::integral_constant<int, 2>{});       // (cmask words past KW are never read as set: u is 0 there)
            else if (KW <= 4) greedy(std::integral_constant<int, 4>{});
            else greedy(std::integral_constant<int, KWMAX>{});
        }
        __syncthreads();
        // Reuse branches of Alg. 2.  Without context_copy a reused set is the greedy set of the same labels, so only the
        // frames at the head of the call that repeat the carried labels take something else than their own greedy set
        // (the carried one): found in parallel.  With context_copy a kept set need not be greedy: frame order.
        if (sequential && context_copy == 0) {
            if (tid == 0) lead_s = n;
            __syncthreads();
            if (tid < n) {
                bool eq = true;
                for (int j = 0; j < KW; ++j) eq &= Y[tid][j] == (tid ? Y[tid - 1][j] : prevY[j]);
                if (!eq) atomicMin(&lead_s, tid);
            }
            __syncthreads();
            const int lead = prevValid ? lead_s : 0;     // frames [0, lead) repeat the carried labels
            if (tid < lead) S[tid] = prevS;
            __syncthreads();
            if (tid == 0) { prevS = S[n - 1]; prevValid = 1; }
            if (tid < KW) prevY[tid] = Y[n - 1][tid];
        } else if (sequential && tid == 0) {
            for (int t = 0; t < n; ++t) {
                bool same = prevValid != 0, covered = prevValid != 0 && context_copy != 0;
                for (int j = 0; j < KW; ++j) {
                    same &= Y[t][j] == prevY[j];
                    covered &= (Y[t][j] & ~prevProv[j]) == 0;
                }
                if (same || covered) {
                    S[t] = prevS;
                } else if (S[t] != prevS) {
                    prevS = S[t];
                    for (int j = 0; j < KW; ++j) {
                        uint64_t pv = 0;
                        for (int pos = 0; pos < M; ++pos)
                            if ((prevS >> pos) & 1ull) pv |= cmask[pos][j];
                        prevProv[j] = pv;
                    }
                }
                for (int j = 0; j < KW; ++j) prevY[j] = Y[t][j];
                prevValid = 1;
            }
        }
        __syncthreads();
        // sizes; uncovered labels again where the reuse branches may have replaced the set
        if (tid < n) {
            const uint64_t sel = S[tid];
            if (sequential) {
                int u = 0;
                for (int j = 0; j < KW; ++j) {
                    uint64_t pv = 0;
                    for (int pos = 0; pos < M; ++pos)
                        if ((sel >> pos) & 1ull) pv |= cmask[pos][j];
                    u += __popcll(Y[tid][j] & ~pv);
                }
                unc[tid] = u;
            }
            cnt[tid] = __popcll(sel);
        }
        __syncthreads();
        // exclusive scan of at most CH counts: inside each wave by shuffles, then the totals of the waves before
        {
            const int c = tid < n ? cnt[tid] : 0, uu = tid < n ? unc[tid] : 0;
            int inc = c, usum = uu;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_up(inc, o, 64);
                if (lane >= o) inc += v;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) usum += __shfl_xor(usum, o, 64);
            if (lane == 63) { wtot[wave] = inc; wunc[wave] = usum; }
            __syncthreads();
            int before = total, ubefore = total_unc;
            for (int w = 0; w < wave; ++w) before += wtot[w];
            if (tid < n) {
                cnt[tid] = before + inc - c;
                row_offsets[f0 + tid + 1] = before + inc;
            }
            __syncthreads();
            if (tid == 0) {
                int run = total;
                for (int w = 0; w < 4; ++w) { run += wtot[w]; ubefore += wunc[w]; }
                total = run; total_unc = ubefore;
            }
        }
        __syncthreads();
        if (tid < n) {
            uint64_t sel = S[tid];
            int o = cnt[tid];
            while (sel) {
                const int pos = __ffsll((unsigned long long)sel) - 1;
                sel &= sel - 1;
                if (o < cap) adapter_ids[o] = order[pos];
                ++o;
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        counters[0] = total;
        counters[1] = total_unc;
        if (state && F > 0) {
            uint64_t ids = 0;
            for (int pos = 0; pos < M; ++pos)
                if ((prevS >> pos) & 1ull) ids |= 1ull << order[pos];
            state->valid = 1;
            state->set_ids = ids;
        }
    }
    if (state && F > 0 && tid < KW) state->labels[tid] = prevY[tid];
}

}  // namespace

extern "C" size_t poly_select_state_bytes(int K)
{
    if (K <= 0) return 0;
    return 16 + 8 * (size_t)((K + 63) / 64);
}

extern "C" int poly_select(const float *label_scores, int F, int K, const uint8_t *group_membership, int M,
                           const poly_select_opts *opts, void *state, int32_t *row_offsets, int32_t *adapter_ids, int cap,
                           int32_t *counters, void *stream)
{
    if (!opts || !group_membership || !row_offsets || !counters) return POLY_EINVAL;
    if (F < 0 || K <= 0 || K > POLY_MAX_LABELS || M <= 0 || M > POLY_MAX_CONTEXTS || cap < 0) return POLY_EINVAL;
    if ((F > 0 && !label_scores) || (cap > 0 && !adapter_ids)) return POLY_EINVAL;
    POLY_LAUNCH(POLY_STAGE_SELECT, select_kernel, dim3(1), dim3(256), (hipStream_t)stream, label_scores, F, K, group_membership, M, opts->theta,
                       opts->context_copy, opts->acc, opts->tau, (SelState *)state, row_offsets, adapter_ids, cap, counters);
    return hipGetLastError() == hipSuccess ? POLY_OK : POLY_EHIP;
}
