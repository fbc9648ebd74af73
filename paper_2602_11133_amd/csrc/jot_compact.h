// Mask maintenance and ordered stream compaction (Algorithm 1: M_{n+1} = positions still [M]).
//
// After the decisions of step n, two small kernels -- one workgroup per batch row -- turn
// "commit_step == n" into: the updated byte mask, the bit image of resolved positions that the
// next step's Eq. 3 reads, the next list of examined positions (ascending b*L+i) and the
// commit-log entries of this step (ascending b*L+i).  Order is fixed by construction (wave
// ballots and prefix counts), never by the arrival order of atomics.
//
// Block mode (semi-autoregressive decoding): a row's examined positions are the masked
// positions of the block that holds its lowest masked position; blocks have block_size
// positions and are counted from gen_start.
#pragma once
#include "jot_device.h"

struct JotCompactParams {
    int32_t B, L;
    int32_t gen_start, block_size;
    int32_t words_per_row;
};

__device__ __forceinline__ int jot_floor_div(int a, int b)   // b > 0
{
    int q = a / b;
    return (a % b < 0) ? q - 1 : q;
}

__device__ __forceinline__ int jot_block_reduce_min(int v, int* lds)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v = min(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = lds[0];
#pragma unroll
    for (int k = 1; k < JOT_WAVES; ++k) r = min(r, lds[k]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ int jot_block_reduce_sum(int v, int* lds)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = 0;
#pragma unroll
    for (int k = 0; k < JOT_WAVES; ++k) r += lds[k];
    __syncthreads();
    return r;
}

// Pass 1: per batch row, the block currently being decoded and the two counts.
// Called by every thread of the workgroup that owns row b (contains barriers); lds: JOT_WAVES ints.
struct JotRowCounts {
    int blk;        // block being decoded (0 outside block mode)
    int n_act;      // positions of the row the next step examines
    int n_com;      // positions of the row finalized in this step
};

// The block a row is decoding: the one that holds its lowest still-masked position (0 outside
// block mode, where no pass over the row is needed).  Contains barriers.
__device__ __forceinline__ int jot_row_block(const JotCompactParams& prm, int32_t step, int b,
                                             const uint8_t* masked, const int32_t* commit_step, int* lds)
{
    if (prm.block_size <= 0)
        return 0;
    const int64_t base = (int64_t)b * prm.L;
    int first = 0x7fffffff;
    for (int i = threadIdx.x; i < prm.L; i += JOT_WG) {
        const bool still = masked[base + i] && commit_step[base + i] != step;
        if (still) first = min(first, i);
    }
    first = jot_block_reduce_min(first, lds);
    return first != 0x7fffffff ? jot_floor_div(first - prm.gen_start, prm.block_size) : 0;
}

__device__ __forceinline__ JotRowCounts jot_row_count(const JotCompactParams& prm, int32_t step, int b,
                                                      const uint8_t* masked, const int32_t* commit_step,
                                                      int32_t* __restrict__ row_block,
                                                      int32_t* __restrict__ row_n_active,
                                                      int32_t* __restrict__ row_n_commit, int* lds)
{
    const int64_t base = (int64_t)b * prm.L;
    const int blk = jot_row_block(prm, step, b, masked, commit_step, lds);
    int n_act = 0, n_com = 0;
    for (int i = threadIdx.x; i < prm.L; i += JOT_WG) {
        const bool was = masked[base + i] != 0;
        const bool com = was && commit_step[base + i] == step;
        const bool still = was && !com;
        const bool elig = still &&
            (prm.block_size <= 0 || jot_floor_div(i - prm.gen_start, prm.block_size) == blk);
        n_act += elig ? 1 : 0;
        n_com += com ? 1 : 0;
    }
    n_act = jot_block_reduce_sum(n_act, lds);
    n_com = jot_block_reduce_sum(n_com, lds);
    if (threadIdx.x == 0) {
        row_block[b] = blk;
        row_n_active[b] = n_act;
        row_n_commit[b] = n_com;
    }
    JotRowCounts out;
    out.blk = blk; out.n_act = n_act; out.n_com = n_com;
    return out;         // the same in every thread of the workgroup
}

// `creating`: the pass that builds the first examined list when a state is created; it matches
// no commit (step -1) and does not count as a step.
__global__ __launch_bounds__(JOT_WG) void jot_row_count_kernel(
    JotCompactParams prm, JotFrame frame, int creating, const uint8_t* __restrict__ masked,
    const int32_t* __restrict__ commit_step, int32_t* __restrict__ row_block,
    int32_t* __restrict__ row_n_commit)
{
    __shared__ int lds[JOT_WAVES];
    const int half = frame.epoch->parity;
    const int32_t step = creating ? -1 : frame.epoch->steps_done + 1;
    (void)jot_row_count(prm, step, blockIdx.x, masked, commit_step, row_block, frame.row_counts[half ^ 1], row_n_commit, lds);
}

// Arrays of the write pass, all in the caller's workspace (host_out: mapped pinned host memory).
struct JotWriteIO {
    uint8_t* masked;
    const int32_t* commit_step;
    const int32_t* tokens;
    int32_t* commit_log;
    uint64_t* resolved_bits;
    const unsigned long long* anomalies;
    JotHostBlock* host_out;
    int32_t* sample_count;
};

// Pass 2 for batch row b, given where its slices start: act_base = examined positions of the rows
// before it (next step's list), log_base = commit-log entries before its own, blk = its block.
// Called by every thread of the workgroup (contains barriers); wave_act / wave_com: JOT_WAVES ints.
// Returns the row's counts (n_act, n_com; the same in every thread).
__device__ __forceinline__ JotRowCounts jot_row_write(const JotCompactParams& prm, int32_t* __restrict__ active_out,
                                                      int32_t step, const JotWriteIO& io, int b, int64_t act_base,
                                                      int64_t log_base, int blk, int* wave_act, int* wave_com)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = (int64_t)b * prm.L;

    int run_act = 0, run_com = 0;
    for (int c0 = 0; c0 < prm.L; c0 += JOT_WG) {
        const int i = c0 + threadIdx.x;
        const bool in = i < prm.L;
        const bool was = in && io.masked[base + i] != 0;
        const bool com = was && io.commit_step[base + i] == step;
        const bool still = was && !com;
        const bool elig = still &&
            (prm.block_size <= 0 || jot_floor_div(i - prm.gen_start, prm.block_size) == blk);
        const uint64_t m_act = __ballot(elig);
        const uint64_t m_com = __ballot(com);
        const uint64_t m_res = __ballot(in && !still);
        const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        if (lane == 0) {
            wave_act[wave] = __popcll(m_act);
            wave_com[wave] = __popcll(m_com);
            if (c0 + wave * 64 < prm.words_per_row * 64)
                io.resolved_bits[(int64_t)b * prm.words_per_row + ((c0 + wave * 64) >> 6)] = m_res;
        }
        __syncthreads();
        int off_act = run_act, off_com = run_com, tot_act = 0, tot_com = 0;
#pragma unroll
        for (int k = 0; k < JOT_WAVES; ++k) {
            if (k < wave) { off_act += wave_act[k]; off_com += wave_com[k]; }
            tot_act += wave_act[k];
            tot_com += wave_com[k];
        }
        if (elig)
            active_out[act_base + off_act + __popcll(m_act & below)] = (int32_t)(base + i);
        if (com) {
            int32_t* e = io.commit_log + 3 * (log_base + off_com + __popcll(m_com & below));
            e[0] = step;
            e[1] = (int32_t)(base + i);
            e[2] = io.tokens[base + i];
            io.masked[base + i] = 0;
        }
        run_act += tot_act;
        run_com += tot_com;
        __syncthreads();
    }
    JotRowCounts out;
    out.blk = blk; out.n_act = run_act; out.n_com = run_com;
    return out;
}

// End of a step, called by every thread of every workgroup of the step's last kernel after its
// row's write pass: `half` / `done` = the half the step read and the number of completed steps
// once it is closed; n_examined = positions the step examined; the row's list ended at
// n_active_end, its log entries at n_log_end.  The workgroup of the last row stores the new
// counters; the workgroup that arrives last closes the step: every other workgroup has finished
// reading the epoch by then.  It flips the double buffers, counts the step, and stores the new
// counters straight into pinned host memory (the host reads them after synchronising).
// A canvas of one row has one workgroup: nothing to count in, nothing of another workgroup's
// to make visible, and the counters are the values this thread has just stored.
__device__ __forceinline__ void jot_close_step(const JotCompactParams& prm, const JotFrame& frame, int half,
                                               int32_t done, const JotWriteIO& io, int b, int64_t n_examined,
                                               int64_t n_active_end, int64_t n_log_end)
{
    JotCounters* cnt_out = frame.counters[half ^ 1];
    if (b == prm.B - 1 && threadIdx.x == 0) {
        cnt_out->n_active = n_active_end;
        cnt_out->n_log = n_log_end;
        cnt_out->n_examined = n_examined;
        cnt_out->reserved = 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        bool last = true;
        int64_t n_active_new = n_active_end, n_log_new = n_log_end, n_examined_new = n_examined;
        if (prm.B > 1) {
            __threadfence();
            const uint32_t arrived = atomicAdd(&frame.epoch->rows_done, 1u);
            last = arrived == (uint32_t)prm.B - 1u;
            if (last) {
                __threadfence();
                // device-scope loads: the numbers were written by the workgroup of the last row
                n_active_new = __hip_atomic_load(&cnt_out->n_active, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                n_log_new = __hip_atomic_load(&cnt_out->n_log, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                n_examined_new = __hip_atomic_load(&cnt_out->n_examined, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (last) {
            const unsigned long long anomalies = __hip_atomic_load(io.anomalies, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            io.host_out->begin = done;
            __threadfence_system();
            io.host_out->c.n_active = n_active_new;
            io.host_out->c.n_log = n_log_new;
            io.host_out->c.n_examined = n_examined_new;
            io.host_out->c.reserved = 0;
            io.host_out->anomalies = anomalies;
            io.host_out->parity = half ^ 1;
            __threadfence_system();
            io.host_out->steps_done = done;
            *io.sample_count = 0;         // the sampling work list of this step has been consumed
            frame.epoch->rows_done = 0u;
            frame.epoch->steps_done = done;
            frame.epoch->parity = half ^ 1;
        }
    }
}

// Pass 2 as a launch of its own: exclusive prefix over the rows' counts, then the ordered writes.
__global__ __launch_bounds__(JOT_WG) void jot_row_write_kernel(
    JotCompactParams prm, JotFrame frame, int creating, JotWriteIO io,
    const int32_t* __restrict__ row_block, const int32_t* __restrict__ row_n_commit)
{
    const int half = frame.epoch->parity;
    const int32_t steps_done = frame.epoch->steps_done;
    const int64_t n_examined = frame.counters[half]->n_active;
    const int64_t n_log = frame.counters[half]->n_log;
    const int32_t* __restrict__ row_n_active = frame.row_counts[half ^ 1];
    __shared__ int lds[JOT_WAVES];
    __shared__ int wave_act[JOT_WAVES], wave_com[JOT_WAVES];
    const int b = blockIdx.x;
    int pa = 0, pc = 0;
    for (int k = threadIdx.x; k < b; k += JOT_WG) {
        pa += row_n_active[k];
        pc += row_n_commit[k];
    }
    const int64_t act_base = jot_block_reduce_sum(pa, lds);
    const int64_t log_base = n_log + jot_block_reduce_sum(pc, lds);
    const JotRowCounts rc = jot_row_write(prm, frame.active[half ^ 1], creating ? -1 : steps_done + 1, io, b,
                                          act_base, log_base, row_block[b], wave_act, wave_com);
    jot_close_step(prm, frame, half, steps_done + (creating ? 0 : 1), io, b, n_examined,
                   act_base + rc.n_act, log_base + rc.n_com);
}

// Copy of the caller's initial canvas into the workspace.
__global__ __launch_bounds__(JOT_WG) void jot_init_copy_kernel(
    int64_t n, const int32_t* __restrict__ tokens_in, const uint8_t* __restrict__ masked_in,
    int32_t* __restrict__ tokens, uint8_t* __restrict__ masked, int32_t* __restrict__ commit_step,
    JotCounters* __restrict__ cnt0, unsigned long long* __restrict__ anomalies, JotEpoch* __restrict__ epoch,
    int32_t* __restrict__ lse_step, int32_t* __restrict__ identity)
{
    const int64_t k = (int64_t)blockIdx.x * JOT_WG + threadIdx.x;
    if (k < n) {
        identity[k] = (int32_t)k;      // "row r is entry r": the examined list of a compact logits tensor
        tokens[k] = tokens_in[k];
        masked[k] = masked_in[k] ? 1 : 0;
        commit_step[k] = 0;
        lse_step[k] = -1;              // no position has a previous distribution yet
    }
    if (k == 0) {
        cnt0->n_active = 0;
        cnt0->n_log = 0;
        cnt0->n_examined = 0;
        cnt0->reserved = 0;
        *anomalies = 0ull;
        epoch->steps_done = 0;
        epoch->parity = 0;
        epoch->rows_done = 0u;
        epoch->pad = 0;
    }
}
