// Per-row step kernel: for canvases whose rows examine at most a couple of thousand positions
// per step (every workload of the paper's shape) the decision (Eq. 2 - Eq. 6), the optional
// transfer schedule, the optional row-wide early commit and the per-row counting pass of the compaction run in ONE launch, one
// workgroup per batch row, instead of three.  Nothing crosses rows here: a row's slice of the
// examined list is found from the per-row counts of the previous step, and the counts for the
// next step go to the other half of a double buffer (a workgroup that starts late must still
// see the old counts of the rows before it).
#pragma once
#include "jot_compact.h"
#include "jot_decide.h"
#include "jot_schedule.h"

//
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
    const int half = frame.epoch->parity;
    const int32_t step = frame.epoch->steps_done + 1;
    const int32_t* row_n_active_in = frame.row_counts[half];
    dio.active = frame.active[half];
    sio.active = frame.active[half];
    const int b = blockIdx.x;
    const int64_t base = jot_row_base(row_n_active_in, b, lds);
    const int n = row_n_active_in[b];
    const JotSplit sp = jot_plan_split(frame.counters[half]->n_active, dprm.V, dprm.target_items, dprm.split_align);

    for (int j = threadIdx.x; j < n; j += JOT_WG)
        jot_decide_one(dprm, dio, step, base + j, sp.S);
    __syncthreads();                       // this row's results are visible to the whole workgroup
    if (sprm.do_schedule) {
        jot_schedule_row(sprm, sio, step, b, base, n, lds, wave_eq);
        __syncthreads();
    }
    if (sprm.do_rowwide) {
        jot_rowwide_row(sprm, sio, step, base, n, dlds, lds);
        __syncthreads();
    }
    const JotRowCounts rc = jot_row_count(cprm, step, b, wio.masked, dio.commit_step, row_block,
                                          frame.row_counts[half ^ 1], row_n_commit, lds);
    if (write_too) {        // B == 1: this row's slices start where the lists start
        __syncthreads();
        jot_row_write(cprm, frame, /*creating=*/0, wio, b, 0, frame.counters[half]->n_log, rc.blk, wave_eq, wave_com);
    }
}
