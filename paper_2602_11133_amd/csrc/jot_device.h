// Shared device-side definitions of the finalization pass (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef JOT_WG
#define JOT_WG 256                 // threads per workgroup of every kernel here (4 waves)
#endif
#define JOT_WAVES (JOT_WG / 64)
#define JOT_MAX_D 32

// Partial result of the vocabulary reduction over a contiguous piece of one logit row.
// The exponentials are accumulated in base 2 against an integer-valued reference M:
//   s = sum_v 2^(l_v * log2(e) - M),  so that  sum_v exp(l_v - m1) = s * 2^(M - m1 * log2(e)).
// A piece whose maximum lies outside the range in which that base-2 form is accurate is summed
// a second time directly against its own maximum (`direct` != 0):  s = sum_v exp(l_v - m1).
struct __align__(32) JotPartial {
    float m1;       // largest logit of the piece (-inf if the piece is empty)
    int32_t idx;    // its vocabulary index, smallest index among equal maxima
    float m2;       // second largest logit of the piece as a multiset
    float M;        // reference exponent (integer valued, -inf if nothing finite was seen)
    float s;        // scaled sum of exponentials
    float cross;    // KL variant: sum_v (weight of v, scaled like s) * (l_v - l'_v); else 0
    float direct;   // != 0: s and cross are relative to m1 itself, M is unused
    float pad;
};

struct JotSplit {
    int S;          // pieces per row
    int chunk;      // elements per piece (multiple of the alignment unless S == 1)
};

// How a step with n_active examined rows cuts each row so that the persistent grid has as many
// work items as fit in target_items (= its workgroups): never more, so that no workgroup takes a
// second item while the others have finished (measured: cutting into one piece more than fits, so
// that every workgroup has work, is 5-12 % slower on steps with fewer rows than workgroups).
// `align` = elements one workgroup of the reduction consumes per batch of loads (threads x
// elements per vector x vectors in flight); pieces are whole batches and at least one batch
// long.  Evaluated identically by every kernel of the step.
__host__ __device__ inline JotSplit jot_plan_split(int64_t n_active, int V, int target_items, int align)
{
    JotSplit sp;
    sp.S = 1;
    sp.chunk = V;
    if (n_active <= 0 || n_active >= target_items)
        return sp;
    int64_t want = target_items / n_active;
    int max_s = V / align;
    if (max_s < 1) max_s = 1;
    int s0 = want < max_s ? (int)want : max_s;
    if (s0 <= 1)
        return sp;
    int chunk = (V + s0 - 1) / s0;
    chunk = (chunk + align - 1) / align * align;
    sp.chunk = chunk;
    sp.S = (V + chunk - 1) / chunk;
    return sp;
}

// Device counters, double buffered: step k reads block [cur] and writes block [cur ^ 1].
struct JotCounters {
    int64_t n_active;     // positions the next step examines
    int64_t n_log;        // commit-log triples written so far
    int64_t n_examined;   // positions the last step examined
    int64_t reserved;
};

// Which half of the double buffers is current, and how many steps have been completed, live in
// DEVICE memory: a launch never bakes in a step number or a buffer choice, so the same launch
// sequence (for instance a captured HIP graph) can be replayed step after step.
struct JotEpoch {
    int32_t steps_done;   // completed steps; the running step is steps_done + 1
    int32_t parity;       // half of the double buffers the running step READS
    uint32_t rows_done;   // arrival counter of the last kernel of a step
    int32_t pad;
};

// The double-buffered arrays, handed to every kernel by value.
struct JotFrame {
    JotEpoch* epoch;
    int32_t* active[2];         // examined lists
    JotCounters* counters[2];
    int32_t* row_counts[2];     // per batch row: examined positions of that row
};

// What a kernel needs to know about the running step.  The counters of BOTH halves are requested
// together with the epoch that says which half counts, so a kernel that starts on cold caches
// waits for one memory round trip here, not two.  For kernels that do not write the counters
// before every workgroup has read them.
struct JotNow {
    int half;           // half of the double buffers the running step reads
    int32_t step;       // number of the running step
    int64_t n_active;   // positions it examines
    int64_t n_log;      // commit-log triples written before it
};

__device__ __forceinline__ JotNow jot_now(const JotFrame& f)
{
    const int32_t parity = f.epoch->parity, done = f.epoch->steps_done;
    const int64_t a0 = f.counters[0]->n_active, a1 = f.counters[1]->n_active;
    const int64_t l0 = f.counters[0]->n_log, l1 = f.counters[1]->n_log;
    JotNow n;
    n.half = parity;
    n.step = done + 1;
    n.n_active = parity ? a1 : a0;
    n.n_log = parity ? l1 : l0;
    return n;
}

// Block the last compaction workgroup writes into host-visible pinned memory.
// Written in the order: begin, (fence), everything else, (fence), steps_done -- so a host reader
// that finds begin == steps_done around its reads has a consistent snapshot of that step.
struct JotHostBlock {
    JotCounters c;
    unsigned long long anomalies;
    int32_t steps_done;
    int32_t parity;       // half that the NEXT step reads (= where the current examined list is)
    int32_t begin;        // number of the step whose results are being (or have been) stored
    int32_t pad;
};

#define JOT_LOG2E 1.44269504088896340736f

// Range of a piece's LARGEST logit within which the one-pass base-2 sums are used.  They work on
// l * log2(e); that product is exact to better than one unit only while it stays below 2^23, i.e.
// for |l| < 5.8e6.  A piece whose maximum lies outside +-JOT_LOGIT_LIMIT (no model produces such
// logits, but every finite row has a softmax) is summed a second time, directly against its
// maximum.  Entries far BELOW the range (fill values such as -1e9, -1e30, -FLT_MAX, -inf used to
// mask tokens) are fine in the one-pass form: they contribute 0.
#define JOT_LOGIT_LIMIT 4.0e6f
#define JOT_EXPONENT_FLOOR (-8388608.0f)   // -2^23: lowest reference exponent a lane will take

// Lexicographic merge of two pieces of the same row: larger logit first, then smaller index.
// m2 is the second entry of the merged multiset; the sums are brought to the common reference.
__device__ __forceinline__ void jot_merge(float& m1, int32_t& idx, float& m2, float& M, float& s,
                                          float bm1, int32_t bidx, float bm2, float bM, float bs)
{
    const bool a_wins = (m1 > bm1) || (m1 == bm1 && idx < bidx);
    const float loser = a_wins ? bm1 : m1;
    m2 = fmaxf(fmaxf(m2, bm2), loser);
    idx = a_wins ? idx : bidx;
    m1 = a_wins ? m1 : bm1;
    const float newM = fmaxf(M, bM);
    // references are integer valued, so these scalings are exact powers of two
    const float fa = (M == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(M - newM);
    const float fb = (bM == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(bM - newM);
    s = s * fa + bs * fb;
    M = newM;
}

// Sum of exponentials of a piece relative to the piece's own maximum, sum_v exp(l_v - m1), and the
// factor that brings the piece's scaled sums (s, cross) to that form.
__device__ __forceinline__ float jot_piece_scale(const JotPartial& q)
{
    if (q.direct != 0.0f) return 1.0f;
    if (q.m1 == -INFINITY) return 0.0f;             // nothing but -inf in the piece: it adds nothing (a NaN sum stays NaN)
    return exp2f(fmaf(-q.m1, JOT_LOG2E, q.M));      // 2^(M - m1 log2 e)
}

// Merge of the pieces of one row in piece order, in the form the decision needs: the row's
// (m1, idx, m2), S = sum_v exp(l_v - m1) and the cross term on the same scale.  Larger logit
// first, then smaller index; m2 is the second entry of the merged multiset.
__device__ __forceinline__ void jot_merge_pieces(const JotPartial* q, int pieces, float& m1, int32_t& idx, float& m2,
                                                 float& S, float& cross)
{
    m1 = q[0].m1; idx = q[0].idx; m2 = q[0].m2;
    {
        const float f = jot_piece_scale(q[0]);
        S = q[0].s * f;
        cross = q[0].cross * f;
    }
    for (int j = 1; j < pieces; ++j) {
        const float f = jot_piece_scale(q[j]);
        const float Sj = q[j].s * f, Cj = q[j].cross * f;
        const float bm1 = q[j].m1;
        const bool a_wins = (m1 > bm1) || (m1 == bm1 && idx < q[j].idx);
        const float loser = a_wins ? bm1 : m1;
        m2 = fmaxf(fmaxf(m2, q[j].m2), loser);
        idx = a_wins ? idx : q[j].idx;
        const float top = a_wins ? m1 : bm1;
        // exp(-inf - top) = 0 for an empty piece; equal maxima give factors of exactly 1
        const float fa = (m1 == top) ? 1.0f : expf(m1 - top);
        const float fb = (bm1 == top) ? 1.0f : expf(bm1 - top);
        S = S * fa + Sj * fb;
        cross = cross * fa + Cj * fb;
        m1 = top;
    }
}
