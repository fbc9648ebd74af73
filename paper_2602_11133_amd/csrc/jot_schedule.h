// Transfer schedule on top of the early exit (Section 3.2 "Iterative Sampling"; Section 4.2
// "Interaction with transfer schedules" / "Implementation details": the decoder's schedule
// reveals the k most confident of the masked positions, confidence = max_v pi_v, and the
// early-exit mask is OR-ed on top, uncapped).
//
// One workgroup per batch row.  Among the positions the row examined this step it selects the
// k with the largest p1 (equal p1: lower position first) and finalizes those that Eq. 6 has not
// finalized already.  Selection is exact and order-deterministic: a radix descent over the
// binary32 patterns of p1 (positive floats order like unsigned integers), one byte per pass,
// finds the k-th largest value T from histograms in LDS; everything above T is taken, and of the
// values equal to T the first k - #(> T) in position order, by a ballot prefix scan.
#pragma once
#include "jot_device.h"

#define JOT_SCHED_CACHE 8          // keys per thread held in registers (rows up to 2048 examined)

struct JotScheduleParams {
    int32_t B, L;
    float transfer_frac;
    int32_t do_schedule;        // transfer schedule requested this step
    int32_t do_rowwide;         // row-wide early commit requested this step
    float global_gap;           // its threshold on the mean top-2 logit gap
};

__device__ __forceinline__ int jot_wg_sum(int v, int* lds)      // v already summed per wave in lane 0
{
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = 0;
#pragma unroll
    for (int k = 0; k < JOT_WAVES; ++k) r += lds[k];
    __syncthreads();
    return r;
}

// Arrays of the schedule pass, all in the caller's workspace.
struct JotScheduleIO {
    const int32_t* n_transfer;      // [B] device, or NULL
    const int32_t* active;          // filled in by the kernel from the frame
    const float* last_p1;
    const float* last_conf;
    const float* last_gap;
    const int32_t* last_token;
    uint8_t* last_flags;
    int32_t* tokens;
    int32_t* commit_step;
    int32_t* sample_list;           // NULL unless this step samples its tokens
    int32_t* sample_count;
};

// The schedule of batch row b, whose examined entries are [base, base + n) of the list.
// Called by every thread of the workgroup (it contains barriers); lds / wave_eq: JOT_WAVES ints each.
__device__ __forceinline__ void jot_schedule_row(const JotScheduleParams& prm, const JotScheduleIO& io,
                                                 int32_t step, int b, int64_t base, int n, int* lds, int* wave_eq)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (n == 0)
        return;

    // key of entry j: bit pattern of p1, or 0 for a row without a softmax (conf is NaN there)
    auto load_key = [&](int j) -> uint32_t {
        const float c = io.last_conf[base + j];
        return (c == c) ? __float_as_uint(io.last_p1[base + j]) : 0u;
    };
    // Rows of up to JOT_SCHED_CACHE * 256 examined positions keep their keys in registers
    // (thread t holds entries t, t + 256, ...); longer rows re-read them from memory each pass.
    constexpr int CACHE = JOT_SCHED_CACHE;
    const bool cached = n <= CACHE * JOT_WG;
    uint32_t kreg[CACHE];
#pragma unroll
    for (int c = 0; c < CACHE; ++c) {
        const int j = c * JOT_WG + threadIdx.x;
        kreg[c] = (cached && j < n) ? load_key(j) : 0u;
    }
    // number of entries with key >= lo (lo >= 1), counted with wave ballots; result in every thread
    auto count_ge = [&](uint32_t lo) -> int {
        int c = 0;
        if (cached) {
#pragma unroll
            for (int q = 0; q < CACHE; ++q)
                if (q * JOT_WG < n)
                    c += __popcll(__ballot(kreg[q] >= lo)) * (lane == 0);
        } else {
            for (int j0 = 0; j0 < n; j0 += JOT_WG) {
                const int j = j0 + threadIdx.x;
                c += __popcll(__ballot(j < n && load_key(j) >= lo)) * (lane == 0);
            }
        }
        return jot_wg_sum(c, lds);
    };

    // how many to reveal
    const int n_valid = count_ge(1u);
    long long want = (io.n_transfer ? (long long)io.n_transfer[b] : 0ll) +
                     (long long)floor((double)prm.transfer_frac * (double)n);
    if (want > n_valid) want = n_valid;
    if (want <= 0)
        return;
    const int k = (int)want;

    // T = k-th largest key, one byte of it per pass, most significant first: a histogram of that
    // byte over the keys that agree with the bytes fixed so far (LDS atomics; counts do not depend
    // on their order), suffix sums over the 256 bins, and the bin in which the k-th largest lies.
    // need_eq = how many of the keys equal to T are still to be taken after everything above it.
    // When everything with a softmax is taken, T stays 0 (all their keys are >= 1 > T).
    static_assert(JOT_WG == 256, "one histogram bin per thread");
    uint32_t T = 0u;
    int need_eq = 0;
    if (k < n_valid) {
        __shared__ int hist[256];
        __shared__ int wave_sum[JOT_WAVES];
        __shared__ int pick[2];                         // the chosen bin, and the keys in the bins above it
        uint32_t fixed = 0u;                            // mask of the bytes of T fixed so far
        int k_rem = k;                                  // rank of T among the keys that agree with them
        for (int shift = 24; shift >= 0; shift -= 8) {
            hist[threadIdx.x] = 0;
            __syncthreads();
            auto count = [&](uint32_t key) {
                if (key != 0u && (key & fixed) == T)
                    atomicAdd(&hist[(key >> shift) & 255u], 1);
            };
            if (cached) {
#pragma unroll
                for (int q = 0; q < CACHE; ++q)
                    if (q * JOT_WG < n) count(kreg[q]);
            } else {
                for (int j = threadIdx.x; j < n; j += JOT_WG) count(load_key(j));
            }
            __syncthreads();
            // keys in bins >= t: suffix sum inside the wave, then the waves above
            const int h = hist[threadIdx.x];
            int s = h;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int v = __shfl_down(s, off, 64);
                if (lane + off < 64) s += v;
            }
            if (lane == 0) wave_sum[wave] = s;
            __syncthreads();
            int higher = 0;
#pragma unroll
            for (int w = 0; w < JOT_WAVES; ++w)
                if (w > wave) higher += wave_sum[w];
            const int at_least = s + higher, above_bin = at_least - h;
            if (at_least >= k_rem && above_bin < k_rem) {     // exactly one bin
                pick[0] = threadIdx.x;
                pick[1] = above_bin;
            }
            __syncthreads();
            T |= (uint32_t)pick[0] << shift;
            fixed |= 255u << shift;
            k_rem -= pick[1];
            __syncthreads();                            // before the bins and the pick are written again
        }
        need_eq = k_rem;
    }

    // take: key > T, and the first need_eq entries with key == T
    int run_eq = 0;
    for (int j0 = 0; j0 < n; j0 += JOT_WG) {
        const int j = j0 + threadIdx.x;
        const bool in = j < n;
        uint32_t key = 0u;
        if (cached) {
#pragma unroll
            for (int q = 0; q < CACHE; ++q)
                key = (j0 == q * JOT_WG) ? kreg[q] : key;
        } else if (in) {
            key = load_key(j);
        }
        const bool above = in && key > T;
        const bool equal = in && key != 0u && key == T;
        const uint64_t m_eq = __ballot(equal);
        const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        if (lane == 0) wave_eq[wave] = __popcll(m_eq);
        __syncthreads();
        int off = run_eq, tot = 0;
#pragma unroll
        for (int w = 0; w < JOT_WAVES; ++w) {
            if (w < wave) off += wave_eq[w];
            tot += wave_eq[w];
        }
        const bool take = above || (equal && off + __popcll(m_eq & below) < need_eq);
        if (take) {
            const int64_t r = base + j;
            const int pos = io.active[r];
            io.last_flags[r] |= 2;
            if (io.commit_step[pos] != step) {          // not already finalized by the early exit
                io.tokens[pos] = io.last_token[r];
                io.commit_step[pos] = step;
                if (io.sample_list)
                    io.sample_list[atomicAdd(io.sample_count, 1)] = (int32_t)r;
            }
        }
        run_eq += tot;
        __syncthreads();
    }
}

// Row-wide early commit (the global rule of Section 2: once the top-2 gap clears a threshold,
// every remaining masked position is finalized at once).  Per batch row: if the mean of the
// top-2 LOGIT gaps m1 - m2 over the row's examined positions that have a softmax reaches
// global_gap, all of them are finalized.  The mean is accumulated in double in a fixed order.
// Called by every thread of the workgroup; dlds: JOT_WAVES doubles, lds: JOT_WAVES ints.
__device__ __forceinline__ void jot_rowwide_row(const JotScheduleParams& prm, const JotScheduleIO& io,
                                                int32_t step, int64_t base, int n, double* dlds, int* lds)
{
    double part = 0.0;
    int cnt = 0;
    for (int j = threadIdx.x; j < n; j += JOT_WG) {
        const float c = io.last_conf[base + j];
        if (c == c) {                       // rows without a softmax carry a NaN confidence
            part += (double)io.last_gap[base + j];
            cnt += 1;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        part += __shfl_xor(part, off, 64);
        cnt += __shfl_xor(cnt, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        dlds[threadIdx.x >> 6] = part;
        lds[threadIdx.x >> 6] = cnt;
    }
    __syncthreads();
    double sum = 0.0;
    int total = 0;
#pragma unroll
    for (int k = 0; k < JOT_WAVES; ++k) {
        sum += dlds[k];
        total += lds[k];
    }
    __syncthreads();
    if (total == 0 || !(sum / (double)total >= (double)prm.global_gap))
        return;
    for (int j = threadIdx.x; j < n; j += JOT_WG) {
        const int64_t r = base + j;
        const float c = io.last_conf[r];
        if (c == c) {
            const int pos = io.active[r];
            io.last_flags[r] |= 4;
            if (io.commit_step[pos] != step) {
                io.tokens[pos] = io.last_token[r];
                io.commit_step[pos] = step;
                if (io.sample_list)
                    io.sample_list[atomicAdd(io.sample_count, 1)] = (int32_t)r;
            }
        }
    }
}

// Sum over the batch rows before b of the per-row examined counts = start of row b's slice.
__device__ __forceinline__ int64_t jot_row_base(const int32_t* __restrict__ row_n_active, int b, int* lds)
{
    int pa = 0;
    for (int k = threadIdx.x; k < b; k += JOT_WG) pa += row_n_active[k];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) pa += __shfl_xor(pa, off, 64);
    return jot_wg_sum(pa, lds);
}

// Stand-alone launch of the per-row rules (used when rows are too long for the per-row kernel).
__global__ __launch_bounds__(JOT_WG) void jot_row_rules_kernel(JotScheduleParams prm, JotScheduleIO io, JotFrame frame)
{
    __shared__ int lds[JOT_WAVES];
    __shared__ int wave_eq[JOT_WAVES];
    __shared__ double dlds[JOT_WAVES];
    const int half = frame.epoch->parity;
    const int32_t step = frame.epoch->steps_done + 1;
    const int32_t* row_n_active = frame.row_counts[half];
    io.active = frame.active[half];
    const int b = blockIdx.x;
    const int64_t base = jot_row_base(row_n_active, b, lds);
    const int n = row_n_active[b];
    if (prm.do_schedule) {
        jot_schedule_row(prm, io, step, b, base, n, lds, wave_eq);
        __syncthreads();
    }
    if (prm.do_rowwide)
        jot_rowwide_row(prm, io, step, base, n, dlds, lds);
}
