// Per-row step kernel: for canvases whose rows examine at most a couple of thousand positions
// per step (every workload of the paper's shape) the decision (Eq. 2 - Eq. 6), the optional
// transfer schedule, the optional row-wide early commit and the per-row counting pass of the
// compaction run in ONE launch, one workgroup per batch row, instead of three.  Nothing crosses
// rows here: a row's slice of the examined list is found from the per-row counts of the
// previous step, and the counts for the next step go to the other half of a double buffer (a
// workgroup that starts late must still see the old counts of the rows before it).
#pragma once
#include "jot_compact.h"
#include "jot_decide.h"
#include "jot_schedule.h"

#define JOT_ROW_WORDS_LDS 512              // rows of up to 32 768 positions keep their bit image in LDS

// With a single batch row (the setting of the paper's experiments) nothing is left for a second
// launch to wait for, and the same workgroup goes on to the write pass of the compaction
// (`write_too`; the host asks for it only when B == 1 and the step does not sample its tokens,
// because the sampling kernel runs between the two passes).
__global__ __launch_bounds__(JOT_WG) void jot_row_step_kernel(
    JotDecideParams dprm, JotDecideIO dio, JotScheduleParams sprm, JotScheduleIO sio,
    JotCompactParams cprm, JotFrame frame, JotWriteIO wio,
    int32_t* __restrict__ row_block, int32_t* __restrict__ row_n_commit, int write_too)
{
    __shared__ int lds[JOT_WAVES];
    __shared__ int wave_eq[JOT_WAVES];
    __shared__ int wave_com[JOT_WAVES];
    __shared__ double dlds[JOT_WAVES];
    __shared__ uint64_t row_words[JOT_ROW_WORDS_LDS];
    const int b = blockIdx.x;
    // Requested before anything else so that they travel together with the epoch and counters
    // below instead of one round trip after the other: the row's words of the bit image (into
    // LDS, for Eq. 3), and one element of every cache line of the row's mask and commit steps,
    // which the compaction reads once the decisions are made.
    const bool words_in_lds = dprm.words_per_row <= JOT_ROW_WORDS_LDS;
    if (words_in_lds)
        for (int w = threadIdx.x; w < dprm.words_per_row; w += JOT_WG)
            row_words[w] = dio.resolved_bits[(int64_t)b * dprm.words_per_row + w];
    int warm = 0;
    {
        const int64_t row0 = (int64_t)b * cprm.L;
        for (int k = threadIdx.x * 32; k < cprm.L; k += JOT_WG * 32) warm += dio.commit_step[row0 + k];
        for (int k = threadIdx.x * 128; k < cprm.L; k += JOT_WG * 128) warm += wio.masked[row0 + k];
    }
    const JotNow now = jot_now(frame);
    const int half = now.half;
    const int32_t step = now.step;
    const int32_t* row_n_active_in = frame.row_counts[half];
    dio.active = frame.active[half];
    sio.active = frame.active[half];
    __syncthreads();                       // row_words is filled
    // a canvas of one row: its slice is the whole list, no look-up of per-row counts
    const int64_t base = cprm.B == 1 ? 0 : jot_row_base(row_n_active_in, b, lds);
    const int n = cprm.B == 1 ? (int)now.n_active : row_n_active_in[b];
    const JotSplit sp = jot_plan_split(now.n_active, dprm.V, dprm.target_items, dprm.split_align);

    for (int j = threadIdx.x; j < n; j += JOT_WG)
        jot_decide_one(dprm, dio, step, base + j, sp.S, words_in_lds ? row_words : nullptr);
    asm volatile("" :: "v"(warm));         // keeps the early loads of the row's mask lines alive
    __syncthreads();                       // this row's results are visible to the whole workgroup
    if (sprm.do_schedule) {
        jot_schedule_row(sprm, sio, step, b, base, n, lds, wave_eq);
        __syncthreads();
    }
    if (sprm.do_rowwide) {
        jot_rowwide_row(sprm, sio, step, base, n, dlds, lds);
        __syncthreads();
    }
    if (!write_too) {
        (void)jot_row_count(cprm, step, b, wio.masked, dio.commit_step, row_block, frame.row_counts[half ^ 1],
                            row_n_commit, lds);
        return;
    }
    // B == 1: this row's slices start where the lists start, and the write pass counts as it goes
    const int blk = jot_row_block(cprm, step, b, wio.masked, dio.commit_step, lds);
    const JotRowCounts rc = jot_row_write(cprm, frame.active[half ^ 1], step, wio, b, 0, now.n_log, blk,
                                          wave_eq, wave_com);
    if (threadIdx.x == 0) {
        row_block[b] = blk;
        frame.row_counts[half ^ 1][b] = rc.n_act;
        row_n_commit[b] = rc.n_com;
    }
    jot_close_step(cprm, frame, half, step, wio, b, now.n_active, rc.n_act, now.n_log + rc.n_com);
}
