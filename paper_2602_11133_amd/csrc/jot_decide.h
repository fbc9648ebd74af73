// Confidence, spatially adaptive threshold and the finalization decision (Eq. 2 - Eq. 6).
//
// One thread per examined position.  It merges the pieces of its row, forms (p1, p2) and the
// selected confidence signal, evaluates Eq. 3 from a bit image of the step-start mask (bit = 1
// where a position is resolved; bits outside the canvas are 0), and tests Eq. 6.  A finalized
// position gets its token and the step number; the mask itself is updated by the compaction
// kernels afterwards, so every thread of this kernel sees the mask as it was when the step began.
#pragma once
#include "jot_device.h"

// Arrays the decision writes or reads, all in the caller's workspace.
struct JotDecideIO {
    const int32_t* active;      // filled in by the kernel from the frame
    const JotPartial* partials;
    const uint64_t* resolved_bits;
    int32_t* tokens;
    int32_t* commit_step;
    int32_t* last_token;
    float* last_conf;
    float* last_p1;
    float* last_p2;
    float* last_tau;
    uint8_t* last_flags;
    float* last_m1;
    float* last_gap;            // top-2 logit gap m1 - m2 (+inf when only one logit is finite)
    int32_t* last_final;
    int32_t* sample_list;       // NULL unless this step samples its tokens
    int32_t* sample_count;
    unsigned long long* anomalies;
    double* lse;                // per POSITION: log-normalizer m1 + ln S of the last step that examined it
    int32_t* lse_step;          // per position: that step's number, -1 if it had no softmax there
    float* last_kl;             // D(pi_now || pi_prev) per examined entry, NaN where undefined
};

struct JotDecideParams {
    int32_t L, V;
    int32_t conf_mode;
    int32_t D;
    float tau_max, tau_min, eps;
    float wmax;                   // 2 * sum_{d=1..D} gamma^d, summed in float in the order d = 1..D
    int32_t words_per_row;        // 64-bit words of the resolved-bit image per batch row
    int32_t target_items;
    int32_t split_align;          // piece alignment of the vocabulary reduction (elements)
    int32_t do_kl;                // KL stability rule on this step (the partials then carry the cross term)
    float kl_threshold;           // stable iff D(pi_now || pi_prev) <= kl_threshold ...
    float kl_min_prob;            // ... and p1 >= kl_min_prob
    float gpow[JOT_MAX_D + 1];    // gpow[d] = gamma^d
};

// Everything for one examined entry r of the list (pieces = pieces per row this step).
// row_words: the bit image of the entry's batch row if the caller holds a copy of it (all entries
// it passes are then of that row), else NULL and the words are read from io.resolved_bits.
__device__ __forceinline__ void jot_decide_one(const JotDecideParams& prm, const JotDecideIO& io,
                                               int32_t step, int64_t r, int pieces,
                                               const uint64_t* row_words = nullptr)
{
    // ---- merge the pieces of the row, in piece order: S_raw = sum_v exp(l_v - m1), cross on the same scale
    float m1, m2, S_raw, cross;
    int32_t idx;
    jot_merge_pieces(io.partials + r * pieces, pieces, m1, idx, m2, S_raw, cross);

    if (m1 == -INFINITY)
        idx = 0;            // every logit is -inf: all are equal, the smallest index is 0

    // ---- probabilities: p1 = 1/S, p2 = e^(m2-m1)/S
    const float S = fmaxf(S_raw, 1.0f);     // the maximum itself contributes exp(0) = 1: rounding may not go below
    const bool has_softmax = (S_raw >= 0.5f) && (S_raw < INFINITY);            // false for NaN
    const float p1 = 1.0f / S;
    const float p2 = expf(m2 - m1) / S;
    float conf;
    if (prm.conf_mode == 0)
        conf = p1 / (p2 + prm.eps);          // Eq. 2
    else if (prm.conf_mode == 1)
        conf = p1;
    else
        conf = p1 - p2;

    // ---- Eq. 3: neighbours at distance d = 1..D on both sides, from the bit image
    const int pos = io.active[r];
    const int b = pos / prm.L;
    const int i = pos - b * prm.L;
    float phi = 0.0f;
    if (prm.D > 0) {
        const uint64_t* words = row_words ? row_words : io.resolved_bits + (int64_t)b * prm.words_per_row;
        const int wi = i >> 6, bi = i & 63;
        const uint64_t mid = words[wi];
        const uint64_t lo = wi > 0 ? words[wi - 1] : 0ull;
        const uint64_t hi = (wi + 1 < prm.words_per_row) ? words[wi + 1] : 0ull;
        // left: bit 63 = position i, bit 63-d = position i-d
        const uint64_t left = (mid << (63 - bi)) | (bi == 63 ? 0ull : (lo >> (bi + 1)));
        // right: bit 0 = position i, bit d = position i+d
        const uint64_t right = (mid >> bi) | (bi == 0 ? 0ull : (hi << (64 - bi)));
        float w = 0.0f;
        for (int d = 1; d <= prm.D; ++d) {
            const int cnt = (int)((left >> (63 - d)) & 1ull) + (int)((right >> d) & 1ull);
            w += prm.gpow[d] * (float)cnt;
        }
        phi = fminf(1.0f, w / prm.wmax);                        // Eq. 4 (w == wmax exactly when all 2D are resolved)
    }
    const float tau = prm.tau_max - (prm.tau_max - prm.tau_min) * phi;   // Eq. 5

    const bool exit_now = has_softmax && (conf >= tau);         // Eq. 6

    // ---- KL stability rule: needs the log-normalizer this position had in the step just before.
    // D(pi || pi') = A/S - (m1 + ln S) + (m1' + ln S'); A (= cross) and S_raw share their scaling.
    const double nan64 = __longlong_as_double(0x7ff8000000000000ll);
    const double lse = has_softmax ? (double)m1 + log((double)S) : nan64;
    bool stable = false;
    float kl_out = __uint_as_float(0x7fc00000u);
    if (prm.do_kl && has_softmax && io.lse_step[pos] == step - 1) {
        const double kl = (double)cross / (double)S_raw - lse + io.lse[pos];
        kl_out = (float)kl;
        stable = (kl <= (double)prm.kl_threshold) && (p1 >= prm.kl_min_prob);
    }
    io.lse[pos] = lse;
    io.lse_step[pos] = has_softmax ? step : -1;
    io.last_kl[r] = kl_out;

    const bool commit = exit_now || stable;
    if (commit) {
        io.tokens[pos] = idx;
        io.commit_step[pos] = step;
        if (io.sample_list)        // unordered work list for the sampling kernel (rows are independent)
            io.sample_list[atomicAdd(io.sample_count, 1)] = (int32_t)r;
    }
    if (!has_softmax)
        atomicAdd(io.anomalies, 1ull);
    io.last_token[r] = idx;
    io.last_final[r] = idx;            // the sampling kernel, if it runs, overwrites this
    io.last_m1[r] = m1;
    io.last_gap[r] = m1 - m2;
    io.last_flags[r] = (exit_now ? 1 : 0) | (stable ? 8 : 0);
    io.last_conf[r] = has_softmax ? conf : __uint_as_float(0x7fc00000u);
    io.last_p1[r] = p1;
    io.last_p2[r] = p2;
    io.last_tau[r] = tau;
}

// One thread per examined position (used when rows are too long for the per-row kernel).
__global__ __launch_bounds__(JOT_WG) void jot_decide_kernel(JotDecideParams prm, JotDecideIO io, JotFrame frame)
{
    const int half = frame.epoch->parity;
    const int32_t step = frame.epoch->steps_done + 1;
    const int64_t n_active = frame.counters[half]->n_active;
    const int64_t r = (int64_t)blockIdx.x * JOT_WG + threadIdx.x;
    if (r >= n_active)
        return;
    io.active = frame.active[half];
    const JotSplit sp = jot_plan_split(n_active, prm.V, prm.target_items, prm.split_align);
    jot_decide_one(prm, io, step, r, sp.S);
}
