// Sampling-based finalization (Section 4.1, "Early-Exit Decision": the finalized token may be
// sampled from the predicted distribution pi instead of taking its argmax).
//
// Inverse-CDF sampling with one uniform number u per position supplied by the caller: the token
// is the first vocabulary index whose cumulative probability exceeds u, i.e. the first v with
//     sum_{w <= v} exp(l_w - m1)  >  u * S,          S = sum_w exp(l_w - m1)  (from the reduction).
// Only rows that were finalized this step are read again (each position is finalized once per
// decode, so over a whole decode this re-reads every row a few times at most).  The deciding
// kernels append those rows to a work list (in arrival order: rows are independent, the result
// does not depend on it) and this kernel deals the list out to its workgroups.
//
// One workgroup per finalized row.  The exponentials are binary32 (v_exp_f32), every sum is
// accumulated in double, and the threshold u * S uses the kernel's own total S of the same
// terms, so the cumulative probabilities are good to about 1e-7.  Three steps: (1) the total S,
// batch by batch; (2) the batch whose running total first exceeds u * S, from the batch totals
// kept in LDS (rows of more than JOT_SAMPLE_KEPT batches are swept a second time instead, which
// gives bitwise the same totals); (3) inside that batch, an ordered inclusive
// scan over the 16-byte vectors (wave shuffles + LDS offsets) finds the vector, and its owner
// walks the vector's elements.  All running totals are workgroup-uniform, so every branch on
// them is uniform.  If the cumulative sum never exceeds u * S (u within rounding of 1, or a
// number that is not below 1), the token is the last one with a non-zero probability: that is
// where the cumulative probability reaches 1.
#pragma once
#include "jot_device.h"
#include "jot_vocab_reduce.h"

#define JOT_SAMPLE_KEPT 64             // batch totals of a row kept in LDS: rows of up to 524 288 elements

template <class T>
struct JotSampleShape {
    static constexpr int U = (T::VEC == 4) ? 8 : 4;          // vectors per thread per batch
    static constexpr int BATCH_VEC = JOT_WG * U;             // vectors per batch
};

__device__ __forceinline__ double jot_wg_total(double v, double* lds)   // every thread gets the sum
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = lds[0];
#pragma unroll
    for (int k = 1; k < JOT_WAVES; ++k) r += lds[k];
    __syncthreads();
    return r;
}

template <class T>
__global__ __launch_bounds__(JOT_WG) void jot_sample_kernel(
    const void* __restrict__ logits, int64_t stride_b, int64_t stride_l, int L, int V,
    JotFrame frame, const int32_t* __restrict__ sample_list,
    const int32_t* __restrict__ sample_count, const float* __restrict__ last_m1,
    const float* __restrict__ uniforms, int32_t* __restrict__ tokens, int32_t* __restrict__ last_final,
    int compact)        // != 0: logits holds one row per examined entry, row r at r * stride_l
{
    constexpr int VEC = T::VEC;
    constexpr int U = JotSampleShape<T>::U;
    constexpr int BATCH_VEC = JotSampleShape<T>::BATCH_VEC;
    __shared__ double lds[JOT_WAVES];
    __shared__ double wave_tot[JOT_WAVES];
    __shared__ double kept[JOT_SAMPLE_KEPT];
    __shared__ int found_token;
    const int32_t* __restrict__ active = frame.active[frame.epoch->parity];
    const int n_items = *sample_count;            // rows finalized this step, listed by the kernels before
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int r = sample_list[item];
        const int pos = active[r];
        const int b = pos / L, i = pos - b * L;
        const int64_t row_off = compact ? (int64_t)r * stride_l : (int64_t)b * stride_b + (int64_t)i * stride_l;
        const char* row = reinterpret_cast<const char*>(logits) + row_off * T::ESZ;
        const jot_u32x4* __restrict__ p = reinterpret_cast<const jot_u32x4*>(row);
        const float top = last_m1[r];                             // exp(l - m1) = 2^((l - m1) log2 e), any magnitude
        const int nvec = V / VEC;
        if (tid == 0) found_token = -1;
        __syncthreads();

        // sum of one batch of vectors, identical arithmetic in sweeps 1 and 2
        auto batch_total = [&](int base) -> double {
            double part = 0.0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = base + u * JOT_WG + tid;
                if (c < nvec) {
                    float x[VEC];
                    T::unpack(p[c], x);
                    float vs = 0.0f;
#pragma unroll
                    for (int k = 0; k < VEC; ++k)
                        vs += __builtin_amdgcn_exp2f((x[k] - top) * JOT_LOG2E);
                    part += (double)vs;
                }
            }
            return jot_wg_total(part, lds);
        };
        auto tail_term = [&](int v) -> double {
            return (double)__builtin_amdgcn_exp2f((T::scalar(row, v) - top) * JOT_LOG2E);
        };

        // (1) total; the batch totals are kept if the row has few enough batches
        const bool keep = (nvec + BATCH_VEC - 1) / BATCH_VEC <= JOT_SAMPLE_KEPT;
        double S = 0.0;
        for (int base = 0, k = 0; base < nvec; base += BATCH_VEC, ++k) {
            const double total = batch_total(base);
            if (keep && tid == 0) kept[k] = total;
            S += total;
        }
        for (int v = nvec * VEC; v < V; ++v) S += tail_term(v);
        __syncthreads();                                          // kept[] is complete
        const float u01 = uniforms[pos];
        const double thresh = (u01 < 1.0f) ? (double)u01 * S : (double)INFINITY;   // u >= 1: nothing exceeds it

        // (2) the batch in which the running total first exceeds thresh
        double running = 0.0;
        int cross = -1;
        for (int base = 0, k = 0; base < nvec; base += BATCH_VEC, ++k) {
            const double total = keep ? kept[k] : batch_total(base);
            if (running + total > thresh) {
                cross = base;
                break;
            }
            running += total;
        }

        if (cross >= 0) {
            // (3) ordered scan from the start of the crossing batch, one sub-row of JOT_WG vectors at a
            // time.  The scan sums in another order than the batch totals, so a crossing that lies
            // within rounding of the batch's end may only show up in the sub-rows after it: keep
            // going to the end of the row if need be.
            for (int sub = cross; sub < nvec; sub += JOT_WG) {
                const int c = sub + tid;
                float x[VEC];
                float vs = 0.0f;
                if (c < nvec) {
                    T::unpack(p[c], x);
#pragma unroll
                    for (int k = 0; k < VEC; ++k) {
                        x[k] = __builtin_amdgcn_exp2f((x[k] - top) * JOT_LOG2E);
                        vs += x[k];
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < VEC; ++k) x[k] = 0.0f;
                }
                // inclusive scan over the lanes of the wave
                double incl = (double)vs;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const double up = __shfl_up(incl, off, 64);
                    if (lane >= off) incl += up;
                }
                if (lane == 63) wave_tot[wave] = incl;
                __syncthreads();
                double wave_off = 0.0, sub_total = 0.0;
#pragma unroll
                for (int w = 0; w < JOT_WAVES; ++w) {
                    if (w == wave) wave_off = sub_total;
                    sub_total += wave_tot[w];
                }
                const double prev = __shfl_up(incl, 1, 64);
                const double lo = running + ((lane == 0) ? wave_off : wave_off + prev);
                const double hi = running + (wave_off + incl);
                if (!(lo > thresh) && hi > thresh && c < nvec) {      // exactly one thread
                    int kk = VEC - 1;
#pragma unroll
                    for (int k = VEC - 1; k >= 0; --k) {
                        double ck = lo;                               // cumulative through element k
#pragma unroll
                        for (int q = 0; q <= k; ++q) ck += (double)x[q];
                        kk = (ck > thresh) ? k : kk;
                    }
                    found_token = c * VEC + kk;
                }
                __syncthreads();
                if (found_token >= 0)
                    break;                                        // uniform: read after the barrier
                running += sub_total;
            }
        }
        // (found_token is latched into a register, with a barrier before anyone writes it again, so
        // that the branches on it are uniform)
        bool none = found_token < 0;
        __syncthreads();
        if (none && nvec * VEC < V) {
            // crossing not in any whole vector: the few trailing elements, in order
            if (tid == 0) {
                double cum = running;
                for (int v = nvec * VEC; v < V; ++v) {
                    cum += tail_term(v);
                    if (cum > thresh) { found_token = v; break; }
                }
            }
            __syncthreads();
        }
        none = found_token < 0;
        __syncthreads();
        if (none) {
            // The cumulative sum never exceeds u * S: u is within rounding of 1 (or not below 1).  The
            // cumulative probability reaches 1 at the last token with a non-zero probability: take it.
            int last_nz = -1;
            for (int c = tid; c < nvec; c += JOT_WG) {
                float x[VEC];
                T::unpack(p[c], x);
#pragma unroll
                for (int k = 0; k < VEC; ++k)
                    if (__builtin_amdgcn_exp2f((x[k] - top) * JOT_LOG2E) > 0.0f) last_nz = c * VEC + k;
            }
            for (int v = nvec * VEC + tid; v < V; v += JOT_WG)
                if (tail_term(v) > 0.0) last_nz = v;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) last_nz = max(last_nz, __shfl_xor(last_nz, off, 64));
            if (lane == 0) atomicMax(&found_token, last_nz);
            __syncthreads();
        }
        if (tid == 0) {
            const int tok = found_token;
            if (tok >= 0) {
                tokens[pos] = tok;
                last_final[r] = tok;
            }
        }
        __syncthreads();
    }
}
