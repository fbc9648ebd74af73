// Vocabulary reduction: the one kernel that reads the logits.
//
// For each examined position it produces what Section 4.1 ("Confidence Metric") needs from the
// row l in R^V: the argmax (smallest index among equal maxima), the two largest logits m1 >= m2
// of the multiset, and sum_v exp(l_v - m1) -- hence p1 = 1/S and p2 = exp(m2 - m1)/S -- in ONE
// pass over the row, so the row is fetched from HBM exactly once.
//
// With the KL stability rule on (the per-token rule Section 2 describes: the KL divergence
// between the distributions of consecutive steps marks predictions that have stopped moving) the
// same kernel template also streams the SAME row of the previous step's logits l' and accumulates
//     A = sum_v exp(l_v - m1) * (l_v - l'_v),
// so that D(pi || pi') = A / S - (m1 + ln S) + (m1' + ln S'), where m1' + ln S' is the
// log-normalizer the previous step stored for the position.  Both rows are fetched exactly once.
// An entry whose exponential underflows to 0 contributes nothing, whatever l'_v is
// (0 * log 0 = 0); an entry with positive weight and l'_v = -inf makes A, and the divergence, +inf.
//
// Launch shape: a persistent grid.  Work items are (examined row, piece of the row); workgroup w
// handles items w, w + G, w + 2G, ...  The number of examined rows lives in device memory (it is
// produced by the previous step), so the loop bound is read on the device and the launch itself
// never depends on it.  Each thread streams 16-byte vectors, one workgroup width apart, and
// keeps its running state in registers; a wave-level butterfly and a small LDS exchange
// combine the lane states of the workgroup into one JotPartial.
//
// The sums of exponentials are taken in base 2 against a per-lane integer reference (no rescale
// per element).  That form is accurate while the piece's maximum lies within +-JOT_LOGIT_LIMIT;
// for a piece outside it -- its exact maximum is known after the pass -- the workgroup sums the
// piece a second time directly against that maximum, so every finite row gets its softmax.
#pragma once
#include "jot_device.h"

#ifndef JOT_F32_UNROLL
#define JOT_F32_UNROLL 8
#endif
#ifndef JOT_BF16_UNROLL
#define JOT_BF16_UNROLL 2
#endif
// Workgroup sizes of the reduction, chosen by measurement on MI355X: fp32 rows stream best with
// few, large workgroups (one 1024-thread workgroup per CU, i.e. 256 rows in flight), the bf16
// path does twice the arithmetic per byte and does best with four 256-thread workgroups per CU
// whose threads load the next batch (2 vectors) before they consume the current one.
#ifndef JOT_F32_WG
#define JOT_F32_WG 1024
#endif
#ifndef JOT_BF16_WG
#define JOT_BF16_WG 256
#endif
// With two streams (current and previous logits) sharing the registers, fewer vectors of each
// row are in flight per thread: 2 + 2 measured best for both element types.
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

typedef uint32_t jot_u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte load

// ---- element types -------------------------------------------------------------------------
struct JotF32 {
    static constexpr int VEC = 4;              // elements per 16-byte vector
    static constexpr int ESZ = 4;
    static constexpr int UNROLL = JOT_F32_UNROLL;   // vectors in flight per thread
    static constexpr int WG = JOT_F32_WG;           // threads per workgroup
    static constexpr bool KL = false;               // also stream the previous step's row
    static constexpr bool PIPELINED = false;        // loads of batch k+1 issued before batch k is consumed
    static constexpr int MAX_WG_PER_CU = 16;        // cap on the persistent grid (beyond what fits anyway)
    static constexpr uint32_t NEG_INF_WORD = 0xff800000u;   // one -inf
    __device__ static __forceinline__ void unpack(const jot_u32x4& w, float (&x)[VEC])
    {
        x[0] = __uint_as_float(w.x); x[1] = __uint_as_float(w.y);
        x[2] = __uint_as_float(w.z); x[3] = __uint_as_float(w.w);
    }
    __device__ static __forceinline__ float scalar(const void* row, int v)
    {
        return reinterpret_cast<const float*>(row)[v];
    }
};

struct JotBF16 {
    static constexpr int VEC = 8;
    static constexpr int ESZ = 2;
    static constexpr int UNROLL = JOT_BF16_UNROLL;
    static constexpr int WG = JOT_BF16_WG;
    static constexpr bool KL = false;
    static constexpr bool PIPELINED = true;         // 2 + 2 vectors in flight: +2-4 % on long bf16 steps
    static constexpr int MAX_WG_PER_CU = 4;         // more workgroups fit, but more concurrent rows stream slower
    static constexpr uint32_t NEG_INF_WORD = 0xff80ff80u;   // two -inf
    // a bf16 is the upper half of a binary32: widening is a shift / mask, exact
    __device__ static __forceinline__ void unpack(const jot_u32x4& w, float (&x)[VEC])
    {
        x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xffff0000u);
        x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xffff0000u);
        x[4] = __uint_as_float(w.z << 16); x[5] = __uint_as_float(w.z & 0xffff0000u);
        x[6] = __uint_as_float(w.w << 16); x[7] = __uint_as_float(w.w & 0xffff0000u);
    }
    __device__ static __forceinline__ float scalar(const void* row, int v)
    {
        return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(row)[v] << 16);
    }
};

struct JotF32KL : JotF32 {
    static constexpr int UNROLL = JOT_F32_KL_UNROLL;    // vectors in flight per thread, of EACH row
    static constexpr int WG = JOT_F32_KL_WG;
    static constexpr bool KL = true;
};
struct JotBF16KL : JotBF16 {
    static constexpr int UNROLL = JOT_BF16_KL_UNROLL;
    static constexpr int WG = JOT_BF16_KL_WG;
    static constexpr bool KL = true;
    static constexpr bool PIPELINED = false;
    static constexpr int MAX_WG_PER_CU = 16;
};

// ---- per-lane running state ----------------------------------------------------------------
struct JotLane {
    float m1, m2;
    int32_t best_vec;   // index (within the piece) of the 16-byte vector that first reached m1, -1 = none
    jot_u32x4 best_raw; // that vector's raw contents: the element index is resolved from it at the end
    float M;            // integer-valued reference of the base-2 exponentials, -inf until set
    float s0, s1, s2, s3;
    float a0, a1, a2, a3;   // KL variant: cross-term partial sums on the same reference (else unused)
};

__device__ __forceinline__ void jot_lane_init(JotLane& a)
{
    a.m1 = -INFINITY;
    a.m2 = -INFINITY;
    a.best_vec = -1;
    a.best_raw = (jot_u32x4)(0u);
    a.M = -INFINITY;
    a.s0 = a.s1 = a.s2 = a.s3 = 0.0f;
    a.a0 = a.a1 = a.a2 = a.a3 = 0.0f;
}

// max(a, b) as the median of {a, b, +inf}: one v_med3_f32.  fmaxf() would spend a second
// instruction per element quieting a possible signalling NaN of the freshly loaded value.  With
// a NaN operand v_med3_f32 returns the smallest non-NaN operand, so a NaN logit simply loses;
// it still poisons the sum of exponentials, which is what flags the row.  `pinf` is +inf handed
// in as a kernel argument, so that it lives in a scalar register and the compiler cannot turn
// the median back into the two-instruction maximum.
__device__ __forceinline__ float jot_max_raw(float a, float b, float pinf)
{
    return __builtin_amdgcn_fmed3f(a, b, pinf);
}

// Top-2 of the lane over the N elements of one vector.  The argmax is tracked per VECTOR: if
// some element is strictly larger than the lane maximum so far, remember the vector (index and
// raw bits); which element it was is found once, after the loop.  Strict comparison keeps the
// first of equal maxima, because a lane meets its vectors in ascending index order.
template <int N>
__device__ __forceinline__ void jot_top2(JotLane& a, const float (&x)[N], const jot_u32x4& raw, int vec_index,
                                         float pinf)
{
    const float before = a.m1;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        a.m2 = __builtin_amdgcn_fmed3f(a.m1, a.m2, x[k]);   // second of {m1, m2, x}
        a.m1 = jot_max_raw(a.m1, x[k], pinf);
    }
    const bool better = a.m1 > before;
    a.best_vec = better ? vec_index : a.best_vec;
    a.best_raw.x = better ? raw.x : a.best_raw.x;
    a.best_raw.y = better ? raw.y : a.best_raw.y;
    a.best_raw.z = better ? raw.z : a.best_raw.z;
    a.best_raw.w = better ? raw.w : a.best_raw.w;
}

// Keep every exponent l*log2(e) - M of the lane at or below 8: when the running maximum has
// climbed past that, move the reference to it and rescale the sums (exact: M is an integer).
// Small exponents keep the rounding of the FMA that forms them small (half an ulp of at most 8,
// i.e. 5e-7) for the terms that matter; the branch is rare (the lane maximum of ordinary rows
// settles within the first batch).
template <bool KL>
__device__ __forceinline__ void jot_rereference(JotLane& a)
{
    const float t = a.m1 * JOT_LOG2E;
    if (t > a.M + 8.0f) {
        // a lane that has only seen fill values (-1e9, -1e30 ...) parks its reference at the floor:
        // their terms then underflow to exactly 0 instead of inheriting the rounding of a huge product
        const float newM = ceilf(fmaxf(t, JOT_EXPONENT_FLOOR));
        const float f = (a.M == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(a.M - newM);
        a.s0 *= f; a.s1 *= f; a.s2 *= f; a.s3 *= f;
        if (KL) { a.a0 *= f; a.a1 *= f; a.a2 *= f; a.a3 *= f; }
        a.M = newM;
    }
}

// x: N elements of the current row; y: the same elements of the previous step's row (KL only).
template <bool KL, int N>
__device__ __forceinline__ void jot_expsum(JotLane& a, const float (&x)[N], const float (&y)[N])
{
    const float negM = (a.M == -INFINITY) ? 0.0f : -a.M;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float e = __builtin_amdgcn_exp2f(fmaf(x[k], JOT_LOG2E, negM));
        float d = 0.0f;
        if (KL) d = (e > 0.0f) ? (x[k] - y[k]) : 0.0f;      // weight 0: no contribution, whatever y is
        if ((k & 3) == 0) { a.s0 += e; if (KL) a.a0 = fmaf(e, d, a.a0); }
        else if ((k & 3) == 1) { a.s1 += e; if (KL) a.a1 = fmaf(e, d, a.a1); }
        else if ((k & 3) == 2) { a.s2 += e; if (KL) a.a2 = fmaf(e, d, a.a2); }
        else { a.s3 += e; if (KL) a.a3 = fmaf(e, d, a.a3); }
    }
}

// Lexicographic merge of two partial results of the same piece inside the reduction (lanes,
// waves): larger logit first, then smaller index; m2 is the second entry of the merged multiset;
// the sums are brought to the common reference (integer valued, so the scalings are exact powers
// of two) and the cross term rides along with the exponent sum.
template <bool KL>
__device__ __forceinline__ void jot_merge(float& m1, int32_t& idx, float& m2, float& M, float& s, float& a,
                                          float bm1, int32_t bidx, float bm2, float bM, float bs, float ba)
{
    const bool a_wins = (m1 > bm1) || (m1 == bm1 && idx < bidx);
    const float loser = a_wins ? bm1 : m1;
    m2 = fmaxf(fmaxf(m2, bm2), loser);
    idx = a_wins ? idx : bidx;
    m1 = a_wins ? m1 : bm1;
    const float newM = fmaxf(M, bM);
    const float fa = (M == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(M - newM);
    const float fb = (bM == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(bM - newM);
    s = s * fa + bs * fb;
    if (KL) a = a * fa + ba * fb;
    M = newM;
}

// Sum over a workgroup of (s, c), result in thread 0 (contains barriers; lds: 2 * WAVES floats).
template <int WAVES>
__device__ __forceinline__ void jot_wg_add2(float& s, float& c, float* lds)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        s += __shfl_xor(s, off, 64);
        c += __shfl_xor(c, off, 64);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { lds[2 * wave] = s; lds[2 * wave + 1] = c; }
    __syncthreads();
    if (threadIdx.x == 0) {
        s = lds[0]; c = lds[1];
#pragma unroll
        for (int k = 1; k < WAVES; ++k) { s += lds[2 * k]; c += lds[2 * k + 1]; }
    }
    __syncthreads();
}

// T: JotF32 / JotBF16 (prev_logits unused) or JotF32KL / JotBF16KL (prev_logits has the layout --
// strides, element type -- of logits).
template <class T>
__global__ __launch_bounds__(T::WG) void jot_vocab_reduce_kernel(
    const void* __restrict__ logits, const void* __restrict__ prev_logits, int64_t stride_b, int64_t stride_l,
    int L, int V, JotFrame frame, JotPartial* __restrict__ partials, int target_items, float pos_inf)
{
    constexpr int VEC = T::VEC;
    constexpr int U = T::UNROLL;
    constexpr int WG = T::WG;
    constexpr int WAVES = WG / 64;
    constexpr bool KL = T::KL;
    const JotNow now = jot_now(frame);
    const int32_t* __restrict__ active = frame.active[now.half];
    const int64_t n_active = now.n_active;
    const JotSplit sp = jot_plan_split(n_active, V, target_items, WG * VEC * U);
    const int64_t n_items = n_active * sp.S;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    __shared__ JotPartial wave_part[WAVES];
    __shared__ float redo_max;             // NaN: the piece is done; else: sum it again against this maximum
    __shared__ float redo_sums[2 * WAVES];

    for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int64_t r = item / sp.S;
        const int piece = (int)(item - r * sp.S);
        const int pos = active[r];
        const int b = pos / L;
        const int i = pos - b * L;
        const int64_t row_off = ((int64_t)b * stride_b + (int64_t)i * stride_l) * T::ESZ;
        const char* row = reinterpret_cast<const char*>(logits) + row_off;
        const char* prow = KL ? reinterpret_cast<const char*>(prev_logits) + row_off : row;
        const int v0 = piece * sp.chunk;                       // whole batches: keeps 16-byte alignment
        const int v1 = min(V, v0 + sp.chunk);
        const int nvec = (v1 - v0) / VEC;                      // whole 16-byte vectors
        const jot_u32x4* __restrict__ p = reinterpret_cast<const jot_u32x4*>(row + (int64_t)v0 * T::ESZ);
        const jot_u32x4* __restrict__ pp = reinterpret_cast<const jot_u32x4*>(prow + (int64_t)v0 * T::ESZ);

        JotLane a;
        jot_lane_init(a);

        // Whole batches of U vectors per thread, all loads of a batch issued before any is used;
        // in the pipelined form the loads of the NEXT batch are issued before the current batch
        // (loaded during the previous iteration) is consumed.
        int base = 0;                                          // workgroup-uniform
        constexpr bool PIPE = T::PIPELINED && !KL;
        jot_u32x4 wn[PIPE ? U : 1];
        if (PIPE && U * WG <= nvec) {
#pragma unroll
            for (int u = 0; u < U; ++u) wn[u] = __builtin_nontemporal_load(p + tid + u * WG);
        }
        for (; base + U * WG <= nvec; base += U * WG) {
            const int c = base + tid;
            jot_u32x4 w[U], wp[KL ? U : 1];
            if (PIPE) {
#pragma unroll
                for (int u = 0; u < U; ++u) w[u] = wn[u];
                if (base + 2 * U * WG <= nvec) {               // workgroup-uniform
#pragma unroll
                    for (int u = 0; u < U; ++u) wn[u] = __builtin_nontemporal_load(p + c + U * WG + u * WG);
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    w[u] = __builtin_nontemporal_load(p + c + u * WG);
                    if (KL) wp[u] = __builtin_nontemporal_load(pp + c + u * WG);
                }
            }
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                T::unpack(w[u], x[u]);
                jot_top2<VEC>(a, x[u], w[u], c + u * WG, pos_inf);
            }
            jot_rereference<KL>(a);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float y[VEC];
                if (KL) T::unpack(wp[u], y);
                jot_expsum<KL, VEC>(a, x[u], KL ? y : x[u]);
            }
        }
        // Ragged end of the piece: one more batch, loads beyond the end replaced by -inf (which
        // changes neither the top-2 nor the sum: their weight is 0, so the previous-row words do
        // not matter either).  Workgroup-uniform branch.
        if (base < nvec) {
            const int c = base + tid;
            jot_u32x4 w[U], wp[KL ? U : 1];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int cu = c + u * WG;
                const bool in = cu < nvec;
                const jot_u32x4 got = __builtin_nontemporal_load(p + (in ? cu : 0));
                if (KL) wp[u] = __builtin_nontemporal_load(pp + (in ? cu : 0));
                w[u].x = in ? got.x : T::NEG_INF_WORD;
                w[u].y = in ? got.y : T::NEG_INF_WORD;
                w[u].z = in ? got.z : T::NEG_INF_WORD;
                w[u].w = in ? got.w : T::NEG_INF_WORD;
            }
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                T::unpack(w[u], x[u]);
                jot_top2<VEC>(a, x[u], w[u], c + u * WG, pos_inf);
            }
            jot_rereference<KL>(a);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float y[VEC];
                if (KL) T::unpack(wp[u], y);
                jot_expsum<KL, VEC>(a, x[u], KL ? y : x[u]);
            }
        }

        // Which element of the remembered vector is the lane maximum: the first equal one.
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
        {   // elements after the last whole vector (V not a multiple of VEC; last piece only)
            const int v = v0 + nvec * VEC + tid;
            if (v < v1) {
                const float xs = T::scalar(row, v);
                a.m2 = __builtin_amdgcn_fmed3f(a.m1, a.m2, xs);
                idx = (xs > a.m1) ? v : idx;
                a.m1 = jot_max_raw(a.m1, xs, pos_inf);
                jot_rereference<KL>(a);
                const float xa[1] = { xs };
                const float ya[1] = { KL ? T::scalar(prow, v) : xs };
                jot_expsum<KL, 1>(a, xa, ya);
            }
        }

        // lane -> wave
        float s = (a.s0 + a.s1) + (a.s2 + a.s3);
        float ac = KL ? (a.a0 + a.a1) + (a.a2 + a.a3) : 0.0f;
        float m1 = a.m1, m2 = a.m2, M = a.M;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float bm1 = __shfl_xor(m1, off, 64);
            const int32_t bidx = __shfl_xor(idx, off, 64);
            const float bm2 = __shfl_xor(m2, off, 64);
            const float bM = __shfl_xor(M, off, 64);
            const float bs = __shfl_xor(s, off, 64);
            const float ba = KL ? __shfl_xor(ac, off, 64) : 0.0f;
            jot_merge<KL>(m1, idx, m2, M, s, ac, bm1, bidx, bm2, bM, bs, ba);
        }
        // wave -> workgroup
        if (lane == 0) {
            JotPartial q;
            q.m1 = m1; q.idx = idx; q.m2 = m2; q.M = M; q.s = s;
            q.cross = ac; q.direct = 0.0f; q.pad = 0.0f;
            wave_part[wave] = q;
        }
        __syncthreads();
        if (tid == 0) {
            JotPartial q = wave_part[0];
#pragma unroll
            for (int k = 1; k < WAVES; ++k) {
                const JotPartial o = wave_part[k];
                jot_merge<KL>(q.m1, q.idx, q.m2, q.M, q.s, q.cross, o.m1, o.idx, o.m2, o.M, o.s, o.cross);
            }
            partials[item] = q;
            const float big = fabsf(q.m1);
            redo_max = (big > JOT_LOGIT_LIMIT && big < INFINITY) ? q.m1 : __uint_as_float(0x7fc00000u);
        }
        __syncthreads();

        // A piece whose maximum is outside the range of the base-2 form: its top-2 and argmax above
        // are exact all the same (they never touch the sums); sum it once more, directly against
        // the maximum: exp(l_v - m1) = 2^((l_v - m1) log2 e), accurate at any magnitude.  Rare
        // (no model emits such logits), workgroup-uniform, one vector per thread at a time.
        const float ref = redo_max;
        if (ref == ref) {
            float ds = 0.0f, dc = 0.0f;
            for (int c = tid; c < nvec; c += WG) {
                float x[VEC], y[VEC];
                T::unpack(p[c], x);
                if (KL) T::unpack(pp[c], y);
#pragma unroll
                for (int k = 0; k < VEC; ++k) {
                    const float e = __builtin_amdgcn_exp2f((x[k] - ref) * JOT_LOG2E);
                    ds += e;
                    if (KL) dc = fmaf(e, (e > 0.0f) ? (x[k] - y[k]) : 0.0f, dc);
                }
            }
            {
                const int v = v0 + nvec * VEC + tid;
                if (v < v1) {
                    const float xs = T::scalar(row, v);
                    const float e = __builtin_amdgcn_exp2f((xs - ref) * JOT_LOG2E);
                    ds += e;
                    if (KL) dc = fmaf(e, (e > 0.0f) ? (xs - T::scalar(prow, v)) : 0.0f, dc);
                }
            }
            jot_wg_add2<WAVES>(ds, dc, redo_sums);
            if (tid == 0) {
                JotPartial* q = partials + item;
                q->s = ds;
                q->cross = dc;
                q->direct = 1.0f;
            }
            __syncthreads();            // redo_max is rewritten by the next item
        }
    }
}
