// Vocabulary reduction: the one kernel that reads the logits.
//
// For each examined position it produces what Section 4.1 ("Confidence Metric") needs from the
// row l in R^V: the argmax (smallest index among equal maxima), the two largest logits m1 >= m2
// of the multiset, and sum_v exp(l_v - m1) -- hence p1 = 1/S and p2 = exp(m2 - m1)/S -- in ONE
// pass over the row, so the row is fetched from HBM exactly once.
//
// Launch shape: a persistent grid.  Work items are (examined row, piece of the row); workgroup w
// handles items w, w + G, w + 2G, ...  The number of examined rows lives in device memory (it is
// produced by the previous step), so the loop bound is read on the device and the launch itself
// never depends on it.  Each thread streams 16-byte vectors, one workgroup width apart, and
// keeps its running state in registers; a wave-level butterfly and a small LDS exchange
// combine the lane states of the workgroup into one JotPartial.
#pragma once
#include "jot_device.h"

#ifndef JOT_F32_UNROLL
#define JOT_F32_UNROLL 8
#endif
#ifndef JOT_BF16_UNROLL
#define JOT_BF16_UNROLL 4
#endif
// Workgroup sizes of the reduction, chosen by measurement on MI355X: fp32 rows stream best with
// few, large workgroups (one 1024-thread workgroup per CU, i.e. 256 rows in flight), the bf16
// path does twice the arithmetic per byte and wants more, smaller workgroups to hide it.
#ifndef JOT_F32_WG
#define JOT_F32_WG 1024
#endif
#ifndef JOT_BF16_WG
#define JOT_BF16_WG 256
#endif

typedef uint32_t jot_u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte load

struct JotLane {
    float m1, m2;
    int32_t best_vec;   // index (within the piece) of the 16-byte vector that first reached m1, -1 = none
    jot_u32x4 best_raw; // that vector's raw contents: the element index is resolved from it at the end
    float M;            // integer-valued reference of the base-2 exponentials, -inf until set
    float s0, s1, s2, s3;
};

__device__ __forceinline__ void jot_lane_init(JotLane& a)
{
    a.m1 = -INFINITY;
    a.m2 = -INFINITY;
    a.best_vec = -1;
    a.best_raw = (jot_u32x4)(0u);
    a.M = -INFINITY;
    a.s0 = a.s1 = a.s2 = a.s3 = 0.0f;
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
__device__ __forceinline__ void jot_rereference(JotLane& a)
{
    const float t = a.m1 * JOT_LOG2E;
    if (t > a.M + 8.0f) {
        // a lane that has only seen fill values (-1e9, -1e30 ...) parks its reference at the floor:
        // their terms then underflow to exactly 0 instead of inheriting the rounding of a huge product
        const float newM = ceilf(fmaxf(t, JOT_EXPONENT_FLOOR));
        const float f = (a.M == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(a.M - newM);
        a.s0 *= f; a.s1 *= f; a.s2 *= f; a.s3 *= f;
        a.M = newM;
    }
}

template <int N>
__device__ __forceinline__ void jot_expsum(JotLane& a, const float (&x)[N])
{
    const float negM = (a.M == -INFINITY) ? 0.0f : -a.M;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float e = __builtin_amdgcn_exp2f(fmaf(x[k], JOT_LOG2E, negM));
        if ((k & 3) == 0) a.s0 += e;
        else if ((k & 3) == 1) a.s1 += e;
        else if ((k & 3) == 2) a.s2 += e;
        else a.s3 += e;
    }
}

// ---- element types -------------------------------------------------------------------------
struct JotF32 {
    static constexpr int VEC = 4;              // elements per 16-byte vector
    static constexpr int ESZ = 4;
    static constexpr int UNROLL = JOT_F32_UNROLL;   // vectors in flight per thread
    static constexpr int WG = JOT_F32_WG;           // threads per workgroup
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

template <class T>
__global__ __launch_bounds__(T::WG) void jot_vocab_reduce_kernel(
    const void* __restrict__ logits, int64_t stride_b, int64_t stride_l, int L, int V,
    JotFrame frame, JotPartial* __restrict__ partials, int target_items, float pos_inf)
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
        const char* row = reinterpret_cast<const char*>(logits) +
                          ((int64_t)b * stride_b + (int64_t)i * stride_l) * T::ESZ;
        const int v0 = piece * sp.chunk;                       // whole batches: keeps 16-byte alignment
        const int v1 = min(V, v0 + sp.chunk);
        const int nvec = (v1 - v0) / VEC;                      // whole 16-byte vectors
        const jot_u32x4* __restrict__ p =
            reinterpret_cast<const jot_u32x4*>(row + (int64_t)v0 * T::ESZ);

        JotLane a;
        jot_lane_init(a);

        // Whole batches of U vectors per thread, all loads of a batch issued before any is used.
        int base = 0;                                          // workgroup-uniform
        for (; base + U * WG <= nvec; base += U * WG) {
            const int c = base + tid;
            jot_u32x4 w[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                w[u] = __builtin_nontemporal_load(p + c + u * WG);
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                T::unpack(w[u], x[u]);
                jot_top2<VEC>(a, x[u], w[u], c + u * WG, pos_inf);
            }
            jot_rereference(a);
#pragma unroll
            for (int u = 0; u < U; ++u)
                jot_expsum<VEC>(a, x[u]);
        }
        // Ragged end of the piece: one more batch, loads beyond the end replaced by -inf (which
        // changes neither the top-2 nor the sum).  Workgroup-uniform branch.
        if (base < nvec) {
            const int c = base + tid;
            jot_u32x4 w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int cu = c + u * WG;
                const bool in = cu < nvec;
                const jot_u32x4 got = __builtin_nontemporal_load(p + (in ? cu : 0));
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
            jot_rereference(a);
#pragma unroll
            for (int u = 0; u < U; ++u)
                jot_expsum<VEC>(a, x[u]);
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
                jot_rereference(a);
                const float xa[1] = { xs };
                jot_expsum<1>(a, xa);
            }
        }

        // lane -> wave
        float s = (a.s0 + a.s1) + (a.s2 + a.s3);
        float m1 = a.m1, m2 = a.m2, M = a.M;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float bm1 = __shfl_xor(m1, off, 64);
            const int32_t bidx = __shfl_xor(idx, off, 64);
            const float bm2 = __shfl_xor(m2, off, 64);
            const float bM = __shfl_xor(M, off, 64);
            const float bs = __shfl_xor(s, off, 64);
            jot_merge(m1, idx, m2, M, s, bm1, bidx, bm2, bM, bs);
        }
        // wave -> workgroup
        if (lane == 0) {
            JotPartial q;
            q.m1 = m1; q.idx = idx; q.m2 = m2; q.M = M; q.s = s;
            q.pad[0] = q.pad[1] = q.pad[2] = 0.0f;
            wave_part[wave] = q;
        }
        __syncthreads();
        if (tid == 0) {
            JotPartial q = wave_part[0];
#pragma unroll
            for (int k = 1; k < WAVES; ++k) {
                const JotPartial o = wave_part[k];
                jot_merge(q.m1, q.idx, q.m2, q.M, q.s, o.m1, o.idx, o.m2, o.M, o.s);
            }
            partials[item] = q;
        }
        __syncthreads();
    }
}
