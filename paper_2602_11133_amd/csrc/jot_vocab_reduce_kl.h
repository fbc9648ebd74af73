// Vocabulary reduction with a stability term: the variant of the reduction that a step uses
// when the KL stability rule is on (the per-token rule Section 2 describes: the KL divergence
// between the distributions of consecutive steps marks predictions that have stopped moving).
//
// Besides the argmax, the top-2 logits and the sum of exponentials of the current row l it
// streams the SAME row of the previous step's logits l' and accumulates the cross term
//     A = sum_v exp(l_v - m1) * (l_v - l'_v),
// in base 2 against the same per-lane reference as the exponent sum, so that
//     D(pi || pi') = A / S - (m1 + ln S) + (m1' + ln S'),
// where m1' + ln S' is the log-normalizer the previous step stored for the position.  Both rows
// are fetched exactly once.  An entry whose exponential underflows to 0 contributes nothing,
// whatever l'_v is (0 * log 0 = 0); an entry with positive weight and l'_v = -inf makes A, and
// the divergence, +inf.
//
// Same launch shape as the plain reduction, with fewer vectors of each row in flight per thread
// (two streams share the registers; measured on MI355X, fp32 rows do best with 2 + 2 vectors per
// thread of a 1024-thread workgroup, about 6.9 TB/s over the two tensors).
#pragma once
#include "jot_stability.h"
#include "jot_vocab_reduce.h"

struct JotLaneKL {
    float a0, a1, a2, a3;       // cross-term partial sums, same reference as the lane's s0..s3
};

__device__ __forceinline__ void jot_rereference_kl(JotLane& a, JotLaneKL& c)
{
    const float t = a.m1 * JOT_LOG2E;
    if (t > a.M + 8.0f) {
        const float newM = ceilf(fmaxf(t, JOT_EXPONENT_FLOOR));
        const float f = (a.M == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(a.M - newM);
        a.s0 *= f; a.s1 *= f; a.s2 *= f; a.s3 *= f;
        c.a0 *= f; c.a1 *= f; c.a2 *= f; c.a3 *= f;
        a.M = newM;
    }
}

template <int N>
__device__ __forceinline__ void jot_expsum_kl(JotLane& a, JotLaneKL& c, const float (&x)[N], const float (&y)[N])
{
    const float negM = (a.M == -INFINITY) ? 0.0f : -a.M;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float e = __builtin_amdgcn_exp2f(fmaf(x[k], JOT_LOG2E, negM));
        const float d = (e > 0.0f) ? (x[k] - y[k]) : 0.0f;      // weight 0: no contribution, whatever y is
        if ((k & 3) == 0) { a.s0 += e; c.a0 = fmaf(e, d, c.a0); }
        else if ((k & 3) == 1) { a.s1 += e; c.a1 = fmaf(e, d, c.a1); }
        else if ((k & 3) == 2) { a.s2 += e; c.a2 = fmaf(e, d, c.a2); }
        else { a.s3 += e; c.a3 = fmaf(e, d, c.a3); }
    }
}

#ifndef JOT_F32_KL_UNROLL
#define JOT_F32_KL_UNROLL 2
#endif
#ifndef JOT_F32_KL_WG
#define JOT_F32_KL_WG 1024
#endif
#ifndef JOT_BF16_KL_UNROLL
#define JOT_BF16_KL_UNROLL 2
#endif
#ifndef JOT_BF16_KL_WG
#define JOT_BF16_KL_WG 256
#endif
struct JotF32KL : JotF32 {
    static constexpr int UNROLL = JOT_F32_KL_UNROLL;    // vectors in flight per thread, of EACH row
    static constexpr int WG = JOT_F32_KL_WG;
};
struct JotBF16KL : JotBF16 {
    static constexpr int UNROLL = JOT_BF16_KL_UNROLL;
    static constexpr int WG = JOT_BF16_KL_WG;
};

// T: JotF32KL or JotBF16KL.  prev_logits has the layout (strides, element type) of logits.
template <class T>
__global__ __launch_bounds__(T::WG) void jot_vocab_reduce_kl_kernel(
    const void* __restrict__ logits, const void* __restrict__ prev_logits, int64_t stride_b, int64_t stride_l,
    int L, int V, JotFrame frame, JotPartial* __restrict__ partials, int target_items, float pos_inf)
{
    constexpr int VEC = T::VEC;
    constexpr int U = T::UNROLL;
    constexpr int WG = T::WG;
    constexpr int WAVES = WG / 64;
    const int half = frame.epoch->parity;
    const int32_t* __restrict__ active = frame.active[half];
    const int64_t n_active = frame.counters[half]->n_active;
    const JotSplit sp = jot_plan_split(n_active, V, target_items, WG * VEC * U);
    const int64_t n_items = n_active * sp.S;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    __shared__ JotPartial wave_part[WAVES];

    for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int64_t r = item / sp.S;
        const int piece = (int)(item - r * sp.S);
        const int pos = active[r];
        const int b = pos / L;
        const int i = pos - b * L;
        const int64_t row_off = ((int64_t)b * stride_b + (int64_t)i * stride_l) * T::ESZ;
        const char* row = reinterpret_cast<const char*>(logits) + row_off;
        const char* prow = reinterpret_cast<const char*>(prev_logits) + row_off;
        const int v0 = piece * sp.chunk;
        const int v1 = min(V, v0 + sp.chunk);
        const int nvec = (v1 - v0) / VEC;
        const jot_u32x4* __restrict__ p = reinterpret_cast<const jot_u32x4*>(row + (int64_t)v0 * T::ESZ);
        const jot_u32x4* __restrict__ pp = reinterpret_cast<const jot_u32x4*>(prow + (int64_t)v0 * T::ESZ);

        JotLane a;
        JotLaneKL c;
        jot_lane_init(a);
        c.a0 = c.a1 = c.a2 = c.a3 = 0.0f;

        int base = 0;
        for (; base + U * WG <= nvec; base += U * WG) {
            const int cv = base + tid;
            jot_u32x4 w[U], wp[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                w[u] = __builtin_nontemporal_load(p + cv + u * WG);
                wp[u] = __builtin_nontemporal_load(pp + cv + u * WG);
            }
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                T::unpack(w[u], x[u]);
                jot_top2<VEC>(a, x[u], w[u], cv + u * WG, pos_inf);
            }
            jot_rereference_kl(a, c);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float y[VEC];
                T::unpack(wp[u], y);
                jot_expsum_kl<VEC>(a, c, x[u], y);
            }
        }
        // ragged end: loads beyond the end are not issued past the piece; their current-row words
        // are -inf, so their weight is 0 and the previous-row words do not matter
        if (base < nvec) {
            const int cv = base + tid;
            jot_u32x4 w[U], wp[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int cu = cv + u * WG;
                const bool in = cu < nvec;
                const jot_u32x4 got = __builtin_nontemporal_load(p + (in ? cu : 0));
                wp[u] = __builtin_nontemporal_load(pp + (in ? cu : 0));
                w[u].x = in ? got.x : T::NEG_INF_WORD;
                w[u].y = in ? got.y : T::NEG_INF_WORD;
                w[u].z = in ? got.z : T::NEG_INF_WORD;
                w[u].w = in ? got.w : T::NEG_INF_WORD;
            }
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                T::unpack(w[u], x[u]);
                jot_top2<VEC>(a, x[u], w[u], cv + u * WG, pos_inf);
            }
            jot_rereference_kl(a, c);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float y[VEC];
                T::unpack(wp[u], y);
                jot_expsum_kl<VEC>(a, c, x[u], y);
            }
        }

        int32_t idx = 0x7fffffff;
        if (a.best_vec >= 0) {
            float bx[VEC];
            T::unpack(a.best_raw, bx);
            int k_first = VEC - 1;
#pragma unroll
            for (int k = VEC - 2; k >= 0; --k)
                k_first = (bx[k] == a.m1) ? k : k_first;
            idx = v0 + a.best_vec * VEC + k_first;
        }
        {   // elements after the last whole vector
            const int v = v0 + nvec * VEC + tid;
            if (v < v1) {
                const float xs = T::scalar(row, v);
                a.m2 = __builtin_amdgcn_fmed3f(a.m1, a.m2, xs);
                idx = (xs > a.m1) ? v : idx;
                a.m1 = jot_max_raw(a.m1, xs, pos_inf);
                jot_rereference_kl(a, c);
                const float xa[1] = { xs };
                const float ya[1] = { T::scalar(prow, v) };
                jot_expsum_kl<1>(a, c, xa, ya);
            }
        }

        // lane -> wave -> workgroup, the cross term riding along with the exponent sum
        float s = (a.s0 + a.s1) + (a.s2 + a.s3);
        float ac = (c.a0 + c.a1) + (c.a2 + c.a3);
        float m1 = a.m1, m2 = a.m2, M = a.M;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float bm1 = __shfl_xor(m1, off, 64);
            const int32_t bidx = __shfl_xor(idx, off, 64);
            const float bm2 = __shfl_xor(m2, off, 64);
            const float bM = __shfl_xor(M, off, 64);
            const float bs = __shfl_xor(s, off, 64);
            const float ba = __shfl_xor(ac, off, 64);
            jot_merge_kl(m1, idx, m2, M, s, ac, bm1, bidx, bm2, bM, bs, ba);
        }
        if (lane == 0) {
            JotPartial q;
            q.m1 = m1; q.idx = idx; q.m2 = m2; q.M = M; q.s = s;
            q.pad[0] = ac; q.pad[1] = q.pad[2] = 0.0f;
            wave_part[wave] = q;
        }
        __syncthreads();
        if (tid == 0) {
            JotPartial q = wave_part[0];
#pragma unroll
            for (int k = 1; k < WAVES; ++k) {
                const JotPartial o = wave_part[k];
                jot_merge_kl(q.m1, q.idx, q.m2, q.M, q.s, q.pad[0], o.m1, o.idx, o.m2, o.M, o.s, o.pad[0]);
            }
            partials[item] = q;
        }
        __syncthreads();
    }
}
