// Host side of the C ABI declared in include/jot.h: argument validation, workspace layout and
// the per-step launch sequence.  No device memory is allocated here; the only host resources
// are the state object, one small pinned buffer for counter read-back and a few events.
#include "../../include/jot.h"

#include <hip/hip_runtime.h>
#include <chrono>
#include <math.h>
#include <mutex>
#include <new>
#include <string.h>

#include "jot_compact.h"
#include "jot_decide.h"
#include "jot_device.h"
#include "jot_row_step.h"
#include "jot_sample.h"
#include "jot_schedule.h"
#include "jot_vocab_reduce.h"

// Working memory of jot_step_static() (see below): one fixed array per GPU.
static __device__ __align__(256) unsigned char scratch[JOT_STATIC_MAX_WORKSPACE];

namespace {

constexpr int64_t kAlign = 256;

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Persistent grid of the vocabulary reduction: workgroups per compute unit, and how many work
// items a step aims for (rows are split into pieces when fewer rows than that are examined).
constexpr int kDefaultWgPerCu = 4;
constexpr int kMaxWgPerCu = 16;
constexpr int kFallbackCus = 256;
// Work items a step aims for per workgroup of the grid.  Measured over whole decode loops on
// MI355X: 1 is best (each item costs a lane-state exchange; 2 and 4 lose 1-5 %).
#ifndef JOT_ITEMS_PER_WG
#define JOT_ITEMS_PER_WG 1
#endif
constexpr int kItemsPerWg = JOT_ITEMS_PER_WG;
constexpr int kPollMicroseconds = 300;   // how long a wait polls the pinned step counter before it blocks on the event
constexpr int kPerRowStepMax = 2048;   // longest per-row examined list handled by the one-launch row kernel

struct Layout {
    int64_t tokens, masked, commit_step, resolved_bits, active0, active1, counters, epoch, anomalies,
        partials, last_token, last_conf, last_p1, last_p2, last_tau, last_flags, last_m1, last_gap, last_final, lse, lse_step, last_kl, identity, sample_list, sample_count, row_block, row_n_active0, row_n_active1,
        row_n_commit, commit_log, host_block, total;
    int64_t n_partials;
    int32_t words_per_row;
};

int validate(const jot_params* p)
{
    if (!p) return JOT_ERR_NULL_POINTER;
    if (p->dtype != JOT_F32 && p->dtype != JOT_BF16) return JOT_ERR_UNSUPPORTED_DTYPE;
    if (p->B < 1 || p->L < 1 || p->V < 2) return JOT_ERR_INVALID_ARG;
    if ((int64_t)p->B * p->L >= (int64_t)1 << 30) return JOT_ERR_INVALID_ARG;
    if (p->conf_mode < JOT_CONF_RATIO || p->conf_mode > JOT_CONF_PROBGAP) return JOT_ERR_INVALID_ARG;
    if (!(p->tau_min <= p->tau_max) || !isfinite(p->tau_min) || !isfinite(p->tau_max))
        return JOT_ERR_INVALID_ARG;
    if (!(p->gamma > 0.0f && p->gamma <= 1.0f)) return JOT_ERR_INVALID_ARG;
    if (p->D < 0 || p->D > JOT_MAX_D) return JOT_ERR_INVALID_ARG;
    if (!(p->eps >= 0.0f) || !isfinite(p->eps)) return JOT_ERR_INVALID_ARG;
    if (p->gen_start < 0 || p->gen_start > p->L) return JOT_ERR_INVALID_ARG;
    if (p->block_size < 0) return JOT_ERR_INVALID_ARG;
    return JOT_OK;
}

int max_target_items() { return 2048 * kMaxWgPerCu * kItemsPerWg; }   // bound used for sizing only

Layout make_layout(const jot_params* p, int target_items)
{
    Layout l;
    const int64_t n = (int64_t)p->B * p->L;
    l.words_per_row = (p->L + 63) / 64;
    l.n_partials = n + target_items;     // n_active * pieces <= n_active + target_items
    int64_t off = 0;
    auto take = [&](int64_t bytes) { int64_t o = off; off = round_up(off + bytes, kAlign); return o; };
    l.tokens = take(n * 4);
    l.masked = take(n);
    l.commit_step = take(n * 4);
    l.resolved_bits = take((int64_t)p->B * l.words_per_row * 8);
    l.active0 = take(n * 4);
    l.active1 = take(n * 4);
    l.counters = take(2 * sizeof(JotCounters));
    l.epoch = take(sizeof(JotEpoch));
    l.anomalies = take(8);
    l.partials = take(l.n_partials * (int64_t)sizeof(JotPartial));
    l.last_token = take(n * 4);
    l.last_conf = take(n * 4);
    l.last_p1 = take(n * 4);
    l.last_p2 = take(n * 4);
    l.last_tau = take(n * 4);
    l.last_flags = take(n);
    l.last_m1 = take(n * 4);
    l.last_gap = take(n * 4);
    l.last_final = take(n * 4);
    l.lse = take(n * 8);
    l.lse_step = take(n * 4);
    l.last_kl = take(n * 4);
    l.identity = take(n * 4);
    l.sample_list = take(n * 4);
    l.sample_count = take(4);
    l.row_block = take((int64_t)p->B * 4);
    l.row_n_active0 = take((int64_t)p->B * 4);
    l.row_n_active1 = take((int64_t)p->B * 4);
    l.row_n_commit = take((int64_t)p->B * 4);
    l.commit_log = take(n * 12);
    l.host_block = take(sizeof(JotHostBlock));   // where a state without pinned host memory sends its counters
    l.total = off;
    return l;
}

using HostCounters = JotHostBlock;

}  // namespace

struct jot_state {
    jot_params p;
    int device;                 // HIP device the state lives on
    Layout lay;
    char* ws;
    JotFrame frame;             // device pointers of the double buffers and the epoch
    bool sync_device;           // the last step was enqueued under stream capture: wait = device sync
    int32_t step;
    int grid_reduce;
    int grid_reduce_kl, target_items_kl;
    int grid_sample;
    int target_items;
    JotDecideParams decide;
    JotCompactParams compact;
    HostCounters* host;         // pinned, mapped into the device address space
    HostCounters* host_dev;     // the device-side address of the same block
    hipEvent_t done;
    bool have_done;
    bool per_row_step;          // decision + schedule + row counts in one per-row launch
    bool host_counts_steps;     // every step so far was enqueued eagerly: s->step is what the device will count to
    bool host_resources;        // owns pinned host counters and events (false: a transient state on the caller's stack)
    bool profile;
    hipEvent_t prof0[JOT_PROFILE_RING], prof1[JOT_PROFILE_RING];
    int32_t prof_step[JOT_PROFILE_RING];    // step recorded in each ring slot, 0 = none

    template <class T> T* at(int64_t off) const { return reinterpret_cast<T*>(ws + off); }
    int32_t* active(int which) const { return at<int32_t>(which ? lay.active1 : lay.active0); }
    JotCounters* counters(int which) const { return at<JotCounters>(lay.counters) + which; }
    int32_t* row_counts(int which) const { return at<int32_t>(which ? lay.row_n_active1 : lay.row_n_active0); }
};

namespace {

bool stream_is_capturing(hipStream_t st)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &status) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return status != hipStreamCaptureStatusNone;
}

// Second half of the compaction (and, if `count_rows`, the first half too): ordered writes of the
// next examined list, the commit log, the mask and its bit image, the counters; its last
// workgroup closes the step (flips the double buffers in the device-side epoch).
JotWriteIO write_io(jot_state* s)
{
    JotWriteIO w;
    w.masked = s->at<uint8_t>(s->lay.masked);
    w.commit_step = s->at<int32_t>(s->lay.commit_step);
    w.tokens = s->at<int32_t>(s->lay.tokens);
    w.commit_log = s->at<int32_t>(s->lay.commit_log);
    w.resolved_bits = s->at<uint64_t>(s->lay.resolved_bits);
    w.anomalies = s->at<unsigned long long>(s->lay.anomalies);
    w.host_out = s->host_dev;
    w.sample_count = s->at<int32_t>(s->lay.sample_count);
    return w;
}

// count_rows / write_rows: which of the two compaction passes still have to be launched (a step's
// per-row kernel may have done the first, or both).
int enqueue_compaction(jot_state* s, bool creating, hipStream_t st, bool count_rows, bool write_rows = true)
{
    if (count_rows)
        hipLaunchKernelGGL(jot_row_count_kernel, dim3(s->p.B), dim3(JOT_WG), 0, st, s->compact, s->frame,
                           creating ? 1 : 0, s->at<uint8_t>(s->lay.masked), s->at<int32_t>(s->lay.commit_step),
                           s->at<int32_t>(s->lay.row_block), s->at<int32_t>(s->lay.row_n_commit));
    if (write_rows)
        hipLaunchKernelGGL(jot_row_write_kernel, dim3(s->p.B), dim3(JOT_WG), 0, st, s->compact, s->frame,
                           creating ? 1 : 0, write_io(s), s->at<int32_t>(s->lay.row_block),
                           s->at<int32_t>(s->lay.row_n_commit));
    if (hipGetLastError() != hipSuccess) return JOT_ERR_HIP;
    // The kernel above also wrote the new counters into pinned host memory.  Outside stream
    // capture the host waits on an event recorded here; a captured step may be replayed any number
    // of times later, so after one the host waits for the whole device instead.
    if (!s->host_resources) {
        // transient state: nothing on the host waits for it
    } else if (stream_is_capturing(st)) {
        s->sync_device = true;
        s->host_counts_steps = false;       // a captured step runs when (and as often as) its graph is replayed
    } else {
        if (hipEventRecord(s->done, st) != hipSuccess) return JOT_ERR_HIP;
        s->have_done = true;
        s->sync_device = false;
    }
    return JOT_OK;
}

// Waits until the results of every step enqueued so far can be read.  The last kernel of a step
// stores its step number into pinned host memory after everything else it writes, so short steps
// are awaited by polling that number for a bounded time (a few microseconds of latency instead of
// an event wait); long steps, and states whose steps are replayed from a graph (the host cannot
// count those), fall back to the event / the device.
int wait_done(jot_state* s)
{
    if (!s) return JOT_ERR_NULL_POINTER;
    if (s->sync_device) {
        if (hipDeviceSynchronize() != hipSuccess) return JOT_ERR_HIP;
        return JOT_OK;
    }
    if (!s->have_done) return JOT_OK;
    if (s->host_counts_steps) {
        const volatile int32_t* done = &s->host->steps_done;
        const auto t0 = std::chrono::steady_clock::now();
        for (int spins = 0; *done < s->step; ++spins) {
            if ((spins & 63) == 63 &&
                std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(kPollMicroseconds))
                break;
#if defined(__x86_64__)
            __builtin_ia32_pause();
#endif
        }
        if (*done >= s->step) {
            __atomic_thread_fence(__ATOMIC_ACQUIRE);
            return JOT_OK;
        }
    }
    return hipEventSynchronize(s->done) == hipSuccess ? JOT_OK : JOT_ERR_HIP;
}

// Working memory of jot_step_static(): one fixed array per GPU, held until the process ends.
// In host code the array's name is only a handle; its address on a device comes from
// hipGetSymbolAddress, asked once per device with that device current.
constexpr int64_t kStaticScratchBytes = JOT_STATIC_MAX_WORKSPACE;
void* g_scratch_ptr[64];
std::mutex g_scratch_mutex;

int scratch_address(int dev, char** out)
{
    if (dev < 0 || dev >= 64) return JOT_ERR_NO_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return JOT_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = static_cast<char*>(g_scratch_ptr[dev]);
    return JOT_OK;
}

// Results of a transient state, copied from its workspace into the caller's arrays.
__global__ __launch_bounds__(JOT_WG) void jot_copy_out_kernel(
    int64_t n, JotFrame frame, const int32_t* __restrict__ tokens, const uint8_t* __restrict__ masked,
    int32_t* __restrict__ tokens_out, uint8_t* __restrict__ masked_out, int32_t* __restrict__ active_out,
    int64_t* __restrict__ n_active_out)
{
    const int half = frame.epoch->parity;                 // the half the NEXT step would read
    const int64_t n_active = frame.counters[half]->n_active;
    const int32_t* __restrict__ active = frame.active[half];
    for (int64_t k = (int64_t)blockIdx.x * JOT_WG + threadIdx.x; k < n; k += (int64_t)gridDim.x * JOT_WG) {
        tokens_out[k] = tokens[k];
        masked_out[k] = masked[k];
        if (k < n_active) active_out[k] = active[k];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_active_out = n_active;
}

// Launch shapes of a device, queried once per device and logit type.
struct DeviceShape {
    bool known;
    int cus;
    int occ[2], occ_kl[2];      // resident workgroups per CU of the two reductions, by jot_dtype
};
constexpr int kMaxDevices = 64;
DeviceShape g_shape[kMaxDevices];
std::mutex g_shape_mutex;

int occupancy_of(const void* kernel, int wg, int cap)
{
    int occ = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, wg, 0) != hipSuccess || occ < 1) {
        (void)hipGetLastError();
        occ = kDefaultWgPerCu;
    }
    if (occ > cap) occ = cap;
    return occ > kMaxWgPerCu ? kMaxWgPerCu : occ;
}

DeviceShape shape_of(int dev)
{
    std::lock_guard<std::mutex> lock(g_shape_mutex);
    DeviceShape local;
    DeviceShape& d = (dev >= 0 && dev < kMaxDevices) ? g_shape[dev] : local;
    if (dev < 0 || dev >= kMaxDevices) d.known = false;
    if (!d.known) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = kFallbackCus;
        d.cus = cus > 2048 ? 2048 : cus;
        // persistent grids = exactly the workgroups that can be resident at once
        d.occ[JOT_F32] = occupancy_of(reinterpret_cast<const void*>(jot_vocab_reduce_kernel<JotF32>), JotF32::WG, JotF32::MAX_WG_PER_CU);
        d.occ[JOT_BF16] = occupancy_of(reinterpret_cast<const void*>(jot_vocab_reduce_kernel<JotBF16>), JotBF16::WG, JotBF16::MAX_WG_PER_CU);
        // the reduction with the stability term has its own register footprint, hence its own grid
        d.occ_kl[JOT_F32] = occupancy_of(reinterpret_cast<const void*>(jot_vocab_reduce_kernel<JotF32KL>), JotF32KL::WG, JotF32KL::MAX_WG_PER_CU);
        d.occ_kl[JOT_BF16] = occupancy_of(reinterpret_cast<const void*>(jot_vocab_reduce_kernel<JotBF16KL>), JotBF16KL::WG, JotBF16KL::MAX_WG_PER_CU);
        d.known = true;
    }
    return d;
}

// Everything of a state that follows from the parameters, the device and the workspace address.
void configure(jot_state* s, const jot_params* p, int dev, char* ws)
{
    const DeviceShape shape = shape_of(dev);
    s->p = *p;
    s->device = dev;
    s->ws = ws;
    s->grid_reduce = shape.cus * shape.occ[p->dtype];
    s->grid_reduce_kl = shape.cus * shape.occ_kl[p->dtype];
    s->target_items_kl = s->grid_reduce_kl * kItemsPerWg;
    if (s->target_items_kl > max_target_items()) s->target_items_kl = max_target_items();
    s->grid_sample = shape.cus * 4;
    s->target_items = s->grid_reduce * kItemsPerWg;
    if (s->target_items > max_target_items()) s->target_items = max_target_items();
    s->lay = make_layout(p, max_target_items());
    s->step = 0;
    s->sync_device = false;
    s->frame.epoch = s->at<JotEpoch>(s->lay.epoch);
    for (int h = 0; h < 2; ++h) {
        s->frame.active[h] = s->active(h);
        s->frame.counters[h] = s->counters(h);
        s->frame.row_counts[h] = s->row_counts(h);
    }
    {   // rows examine at most this many positions per step
        const int per_row = (p->block_size > 0 && p->block_size < p->L) ? p->block_size : p->L;
        s->per_row_step = per_row <= kPerRowStepMax;
    }
    s->have_done = false;
    s->profile = false;
    s->host_counts_steps = true;
    s->host_resources = false;
    s->host = nullptr;
    s->host_dev = s->at<HostCounters>(s->lay.host_block);     // replaced by pinned host memory if the state owns some

    JotDecideParams& d = s->decide;
    memset(&d, 0, sizeof d);
    d.L = p->L; d.V = p->V; d.conf_mode = p->conf_mode; d.D = p->D;
    d.tau_max = p->tau_max; d.tau_min = p->tau_min; d.eps = p->eps;
    d.words_per_row = s->lay.words_per_row;
    d.target_items = s->target_items;
    d.split_align = p->dtype == JOT_F32 ? JotF32::WG * JotF32::VEC * JotF32::UNROLL
                                        : JotBF16::WG * JotBF16::VEC * JotBF16::UNROLL;
    float wmax = 0.0f;
    for (int k = 0; k <= JOT_MAX_D; ++k) d.gpow[k] = 0.0f;
    for (int k = 1; k <= p->D; ++k) {
        d.gpow[k] = (float)pow((double)p->gamma, (double)k);
        wmax += d.gpow[k] * 2.0f;
    }
    d.wmax = p->D > 0 ? wmax : 1.0f;
    s->compact.B = p->B; s->compact.L = p->L;
    s->compact.gen_start = p->gen_start; s->compact.block_size = p->block_size;
    s->compact.words_per_row = s->lay.words_per_row;
}

// Copies the caller's canvas into the workspace and builds the first examined list.
int enqueue_init(jot_state* s, const int32_t* tokens_dev, const uint8_t* masked_dev, hipStream_t st)
{
    const int64_t n = (int64_t)s->p.B * s->p.L;
    hipLaunchKernelGGL(jot_init_copy_kernel, dim3((unsigned)((n + JOT_WG - 1) / JOT_WG)), dim3(JOT_WG), 0, st,
                       n, tokens_dev, masked_dev, s->at<int32_t>(s->lay.tokens),
                       s->at<uint8_t>(s->lay.masked), s->at<int32_t>(s->lay.commit_step),
                       s->counters(0), s->at<unsigned long long>(s->lay.anomalies), s->frame.epoch,
                       s->at<int32_t>(s->lay.lse_step), s->at<int32_t>(s->lay.identity));
    if (hipGetLastError() != hipSuccess) return JOT_ERR_HIP;
    return enqueue_compaction(s, /*creating=*/true, st, true);
}

// Host-side checks of one step's arguments (no device work).
int validate_step(const jot_params& p, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                  const jot_step_options* opt)
{
    const int32_t* n_transfer_dev = opt->n_transfer_dev;
    const float transfer_frac = opt->transfer_frac;
    const float* uniforms_dev = opt->uniforms_dev;
    const bool do_rowwide = opt->enable_global_gap != 0;
    const bool do_kl = opt->enable_kl != 0;
    const bool compact = opt->logits_compact != 0;
    if (!logits_dev) return JOT_ERR_NULL_POINTER;
    if (compact && do_kl) return JOT_ERR_INVALID_ARG;     // the previous step's rows are in another order
    if (do_kl) {
        if (!opt->prev_logits_dev) return JOT_ERR_NULL_POINTER;
        if (reinterpret_cast<uintptr_t>(opt->prev_logits_dev) % 16) return JOT_ERR_MISALIGNED;
        if (!(opt->kl_threshold >= 0.0f) || !isfinite(opt->kl_threshold)) return JOT_ERR_INVALID_ARG;
        if (!(opt->kl_min_prob >= 0.0f && opt->kl_min_prob <= 1.0f)) return JOT_ERR_INVALID_ARG;
    }
    if (do_rowwide && !isfinite(opt->global_gap)) return JOT_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(uniforms_dev) % 4) return JOT_ERR_MISALIGNED;
    if (!(transfer_frac >= 0.0f && transfer_frac <= 1.0f)) return JOT_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(n_transfer_dev) % 4) return JOT_ERR_MISALIGNED;
    const int64_t esz = p.dtype == JOT_F32 ? 4 : 2;
    if (stride_l < p.V) return JOT_ERR_INVALID_ARG;
    if (!compact) {
        if (p.B > 1 && stride_b < (int64_t)(p.L - 1) * stride_l + p.V) return JOT_ERR_INVALID_ARG;
        if (stride_b < 0) return JOT_ERR_INVALID_ARG;
    }
    if (reinterpret_cast<uintptr_t>(logits_dev) % 16 || (stride_l * esz) % 16 ||
        (!compact && p.B > 1 && (stride_b * esz) % 16))
        return JOT_ERR_MISALIGNED;
    return JOT_OK;
}

// The launch sequence of one step; arguments already validated.
int enqueue_step(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                 const jot_step_options* opt, hipStream_t st)
{
    const jot_params& p = s->p;
    const int32_t* n_transfer_dev = opt->n_transfer_dev;
    const float transfer_frac = opt->transfer_frac;
    const float* uniforms_dev = opt->uniforms_dev;
    const bool do_rowwide = opt->enable_global_gap != 0;
    const bool do_kl = opt->enable_kl != 0;
    const bool compact = opt->logits_compact != 0;
    // A compact tensor has one row per examined entry.  The reduction is handed the identity list
    // and a canvas length no position reaches, so that "position" r resolves to row r of batch 0.
    JotFrame reduce_frame = s->frame;
    int reduce_L = p.L;
    if (compact) {
        reduce_frame.active[0] = reduce_frame.active[1] = s->at<int32_t>(s->lay.identity);
        reduce_L = 0x7fffffff;
    }

    const int32_t step = s->step + 1;           // host-side call count; the kernels use the device epoch
    const int64_t n = (int64_t)p.B * p.L;
    const bool capturing = stream_is_capturing(st);

    const int slot = step % JOT_PROFILE_RING;
    if (s->profile && !capturing) {
        s->prof_step[slot] = 0;
        if (hipEventRecord(s->prof0[slot], st) != hipSuccess) return JOT_ERR_HIP;
    }
    if (do_kl && p.dtype == JOT_F32)
        hipLaunchKernelGGL(jot_vocab_reduce_kernel<JotF32KL>, dim3(s->grid_reduce_kl), dim3(JotF32KL::WG), 0, st,
                           logits_dev, opt->prev_logits_dev, stride_b, stride_l, p.L, p.V, s->frame,
                           s->at<JotPartial>(s->lay.partials), s->target_items_kl, INFINITY);
    else if (do_kl)
        hipLaunchKernelGGL(jot_vocab_reduce_kernel<JotBF16KL>, dim3(s->grid_reduce_kl), dim3(JotBF16KL::WG), 0, st,
                           logits_dev, opt->prev_logits_dev, stride_b, stride_l, p.L, p.V, s->frame,
                           s->at<JotPartial>(s->lay.partials), s->target_items_kl, INFINITY);
    else if (p.dtype == JOT_F32)
        hipLaunchKernelGGL(jot_vocab_reduce_kernel<JotF32>, dim3(s->grid_reduce), dim3(JotF32::WG), 0, st,
                           logits_dev, nullptr, stride_b, stride_l, reduce_L, p.V, reduce_frame,
                           s->at<JotPartial>(s->lay.partials), s->target_items, INFINITY);
    else
        hipLaunchKernelGGL(jot_vocab_reduce_kernel<JotBF16>, dim3(s->grid_reduce), dim3(JotBF16::WG), 0, st,
                           logits_dev, nullptr, stride_b, stride_l, reduce_L, p.V, reduce_frame,
                           s->at<JotPartial>(s->lay.partials), s->target_items, INFINITY);
    if (hipGetLastError() != hipSuccess) return JOT_ERR_HIP;
    if (s->profile && !capturing) {
        if (hipEventRecord(s->prof1[slot], st) != hipSuccess) return JOT_ERR_HIP;
        s->prof_step[slot] = step;
    }

    JotDecideIO dio;
    dio.active = nullptr;       // taken from the frame on the device
    dio.partials = s->at<JotPartial>(s->lay.partials);
    dio.resolved_bits = s->at<uint64_t>(s->lay.resolved_bits);
    dio.tokens = s->at<int32_t>(s->lay.tokens);
    dio.commit_step = s->at<int32_t>(s->lay.commit_step);
    dio.last_token = s->at<int32_t>(s->lay.last_token);
    dio.last_conf = s->at<float>(s->lay.last_conf);
    dio.last_p1 = s->at<float>(s->lay.last_p1);
    dio.last_p2 = s->at<float>(s->lay.last_p2);
    dio.last_tau = s->at<float>(s->lay.last_tau);
    dio.last_flags = s->at<uint8_t>(s->lay.last_flags);
    dio.last_m1 = s->at<float>(s->lay.last_m1);
    dio.last_gap = s->at<float>(s->lay.last_gap);
    dio.last_final = s->at<int32_t>(s->lay.last_final);
    dio.sample_list = uniforms_dev ? s->at<int32_t>(s->lay.sample_list) : nullptr;
    dio.sample_count = s->at<int32_t>(s->lay.sample_count);
    dio.anomalies = s->at<unsigned long long>(s->lay.anomalies);
    dio.lse = s->at<double>(s->lay.lse);
    dio.lse_step = s->at<int32_t>(s->lay.lse_step);
    dio.last_kl = s->at<float>(s->lay.last_kl);
    JotDecideParams dprm = s->decide;
    if (do_kl) {
        dprm.do_kl = 1;
        dprm.kl_threshold = opt->kl_threshold;
        dprm.kl_min_prob = opt->kl_min_prob;
        dprm.target_items = s->target_items_kl;
        dprm.split_align = p.dtype == JOT_F32 ? JotF32KL::WG * JotF32KL::VEC * JotF32KL::UNROLL
                                              : JotBF16KL::WG * JotBF16KL::VEC * JotBF16KL::UNROLL;
    }
    const bool do_schedule = n_transfer_dev || transfer_frac > 0.0f;
    JotScheduleParams sprm;
    sprm.B = p.B; sprm.L = p.L; sprm.transfer_frac = transfer_frac;
    sprm.do_schedule = do_schedule ? 1 : 0;
    sprm.do_rowwide = do_rowwide ? 1 : 0;
    sprm.global_gap = do_rowwide ? opt->global_gap : 0.0f;
    JotScheduleIO sio;
    sio.n_transfer = n_transfer_dev;
    sio.active = dio.active;
    sio.last_p1 = dio.last_p1;
    sio.last_conf = dio.last_conf;
    sio.last_gap = dio.last_gap;
    sio.last_token = dio.last_token;
    sio.last_flags = dio.last_flags;
    sio.tokens = dio.tokens;
    sio.commit_step = dio.commit_step;
    sio.sample_list = dio.sample_list;
    sio.sample_count = dio.sample_count;

    // a single batch row without sampling: the per-row kernel also does the write pass
    const bool one_launch = s->per_row_step && p.B == 1 && !uniforms_dev;
    if (s->per_row_step) {
        hipLaunchKernelGGL(jot_row_step_kernel, dim3(p.B), dim3(JOT_WG), 0, st, dprm, dio, sprm, sio,
                           s->compact, s->frame, write_io(s),
                           s->at<int32_t>(s->lay.row_block), s->at<int32_t>(s->lay.row_n_commit),
                           one_launch ? 1 : 0);
        if (hipGetLastError() != hipSuccess) return JOT_ERR_HIP;
    } else {
        hipLaunchKernelGGL(jot_decide_kernel, dim3((unsigned)((n + JOT_WG - 1) / JOT_WG)), dim3(JOT_WG), 0, st,
                           dprm, dio, s->frame);
        if (hipGetLastError() != hipSuccess) return JOT_ERR_HIP;
        if (do_schedule || do_rowwide) {
            hipLaunchKernelGGL(jot_row_rules_kernel, dim3(p.B), dim3(JOT_WG), 0, st, sprm, sio, s->frame);
            if (hipGetLastError() != hipSuccess) return JOT_ERR_HIP;
        }
    }
    if (uniforms_dev) {
        const int grid = s->grid_sample;
        if (p.dtype == JOT_F32)
            hipLaunchKernelGGL(jot_sample_kernel<JotF32>, dim3(grid), dim3(JOT_WG), 0, st, logits_dev, stride_b,
                               stride_l, p.L, p.V, s->frame, s->at<int32_t>(s->lay.sample_list),
                               s->at<int32_t>(s->lay.sample_count), s->at<float>(s->lay.last_m1), uniforms_dev,
                               s->at<int32_t>(s->lay.tokens), s->at<int32_t>(s->lay.last_final), compact ? 1 : 0);
        else
            hipLaunchKernelGGL(jot_sample_kernel<JotBF16>, dim3(grid), dim3(JOT_WG), 0, st, logits_dev, stride_b,
                               stride_l, p.L, p.V, s->frame, s->at<int32_t>(s->lay.sample_list),
                               s->at<int32_t>(s->lay.sample_count), s->at<float>(s->lay.last_m1), uniforms_dev,
                               s->at<int32_t>(s->lay.tokens), s->at<int32_t>(s->lay.last_final), compact ? 1 : 0);
        if (hipGetLastError() != hipSuccess) return JOT_ERR_HIP;
    }
    s->step = step;
    return enqueue_compaction(s, /*creating=*/false, st, /*count_rows=*/!s->per_row_step, /*write_rows=*/!one_launch);
}

}  // namespace

extern "C" {

int64_t jot_workspace_bytes(const jot_params* p)
{
    const int rc = validate(p);
    if (rc != JOT_OK) return rc;
    return make_layout(p, max_target_items()).total;
}

int jot_init_state(jot_state** out, const jot_params* p, void* workspace_dev, int64_t workspace_bytes,
                   const int32_t* tokens_dev, const uint8_t* masked_dev, void* stream)
{
    if (!out) return JOT_ERR_NULL_POINTER;
    *out = nullptr;
    const int rc = validate(p);
    if (rc != JOT_OK) return rc;
    if (!workspace_dev || !tokens_dev || !masked_dev) return JOT_ERR_NULL_POINTER;
    if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign) return JOT_ERR_MISALIGNED;
    if (reinterpret_cast<uintptr_t>(tokens_dev) % 4) return JOT_ERR_MISALIGNED;
    if (workspace_bytes < make_layout(p, max_target_items()).total) return JOT_ERR_WORKSPACE_TOO_SMALL;

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return JOT_ERR_NO_DEVICE;

    jot_state* s = new (std::nothrow) jot_state();
    if (!s) return JOT_ERR_NO_MEMORY;
    configure(s, p, dev, static_cast<char*>(workspace_dev));
    s->host_resources = true;

    if (hipHostMalloc(reinterpret_cast<void**>(&s->host), sizeof(HostCounters), hipHostMallocMapped) != hipSuccess) {
        delete s;
        return JOT_ERR_HIP;
    }
    memset(s->host, 0, sizeof(HostCounters));
    if (hipHostGetDevicePointer(reinterpret_cast<void**>(&s->host_dev), s->host, 0) != hipSuccess) {
        (void)hipHostFree(s->host);
        delete s;
        return JOT_ERR_HIP;
    }
    if (hipEventCreateWithFlags(&s->done, hipEventDisableTiming) != hipSuccess) {
        (void)hipHostFree(s->host);
        delete s;
        return JOT_ERR_HIP;
    }

    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc2 = enqueue_init(s, tokens_dev, masked_dev, st);
    if (rc2 == JOT_OK && hipStreamSynchronize(st) != hipSuccess) rc2 = JOT_ERR_HIP;
    if (rc2 != JOT_OK) {
        jot_release(s);
        return rc2;
    }
    *out = s;
    return JOT_OK;
}

int jot_step(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l, void* stream)
{
    return jot_step_scheduled(s, logits_dev, stride_b, stride_l, nullptr, 0.0f, stream);
}

int jot_step_scheduled(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                       const int32_t* n_transfer_dev, float transfer_frac, void* stream)
{
    return jot_step_sampled(s, logits_dev, stride_b, stride_l, n_transfer_dev, transfer_frac, nullptr, stream);
}

int jot_step_sampled(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                     const int32_t* n_transfer_dev, float transfer_frac, const float* uniforms_dev,
                     void* stream)
{
    jot_step_options opt;
    memset(&opt, 0, sizeof opt);
    opt.n_transfer_dev = n_transfer_dev;
    opt.transfer_frac = transfer_frac;
    opt.uniforms_dev = uniforms_dev;
    return jot_step_ex(s, logits_dev, stride_b, stride_l, &opt, stream);
}

int jot_step_ex(jot_state* s, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                const jot_step_options* opt, void* stream)
{
    jot_step_options none;
    memset(&none, 0, sizeof none);
    if (!opt) opt = &none;
    if (!s) return JOT_ERR_NULL_POINTER;
    const int rc = validate_step(s->p, logits_dev, stride_b, stride_l, opt);
    if (rc != JOT_OK) return rc;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return JOT_ERR_NO_DEVICE;
    if (dev != s->device) return JOT_ERR_WRONG_DEVICE;
    return enqueue_step(s, logits_dev, stride_b, stride_l, opt, static_cast<hipStream_t>(stream));
}

int jot_step_static(const jot_params* p, const void* logits_dev, int64_t stride_b, int64_t stride_l,
                    int32_t* tokens_dev, uint8_t* masked_dev, int32_t* active_out_dev, int64_t* n_active_out_dev,
                    void* stream)
{
    const int rc = validate(p);
    if (rc != JOT_OK) return rc;
    if (!tokens_dev || !masked_dev || !active_out_dev || !n_active_out_dev) return JOT_ERR_NULL_POINTER;
    if (reinterpret_cast<uintptr_t>(tokens_dev) % 4 || reinterpret_cast<uintptr_t>(active_out_dev) % 4 ||
        reinterpret_cast<uintptr_t>(n_active_out_dev) % 8)
        return JOT_ERR_MISALIGNED;
    jot_step_options none;
    memset(&none, 0, sizeof none);
    const int rc1 = validate_step(*p, logits_dev, stride_b, stride_l, &none);
    if (rc1 != JOT_OK) return rc1;
    if (make_layout(p, max_target_items()).total > kStaticScratchBytes) return JOT_ERR_TOO_LARGE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return JOT_ERR_NO_DEVICE;
    char* ws = nullptr;
    const int rc2 = scratch_address(dev, &ws);
    if (rc2 != JOT_OK) return rc2;

    jot_state t;                      // transient: lives for this call only, owns nothing
    configure(&t, p, dev, ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc3 = enqueue_init(&t, tokens_dev, masked_dev, st);
    if (rc3 == JOT_OK) rc3 = enqueue_step(&t, logits_dev, stride_b, stride_l, &none, st);
    if (rc3 != JOT_OK) return rc3;
    const int64_t n = (int64_t)p->B * p->L;
    const unsigned grid = (unsigned)((n + JOT_WG - 1) / JOT_WG);
    hipLaunchKernelGGL(jot_copy_out_kernel, dim3(grid), dim3(JOT_WG), 0, st, n, t.frame,
                       t.at<int32_t>(t.lay.tokens), t.at<uint8_t>(t.lay.masked), tokens_dev, masked_dev,
                       active_out_dev, n_active_out_dev);
    return hipGetLastError() == hipSuccess ? JOT_OK : JOT_ERR_HIP;
}

int64_t jot_active_count(jot_state* s)
{
    const int rc = wait_done(s);
    return rc != JOT_OK ? rc : s->host->c.n_active;
}

int32_t jot_step_index(jot_state* s)
{
    const int rc = wait_done(s);
    return rc != JOT_OK ? rc : s->host->steps_done;     // counted on the device: right under graph replay too
}

int64_t jot_active_count_poll(const jot_state* s, int32_t* steps_done)
{
    if (!s) return JOT_ERR_NULL_POINTER;
    // The closing workgroup of a step stores `begin`, then the counters, then `steps_done`, with
    // system-scope fences between: a snapshot is consistent if steps_done (read first) equals
    // begin (read last).  Otherwise a store is in flight: try again.
    const volatile HostCounters* h = s->host;
    for (int tries = 0; tries < 100000; ++tries) {
        const int32_t end = h->steps_done;
        __atomic_thread_fence(__ATOMIC_ACQUIRE);
        const int64_t n = h->c.n_active;
        __atomic_thread_fence(__ATOMIC_ACQUIRE);
        if (h->begin == end) {
            if (steps_done) *steps_done = end;
            return n;
        }
    }
    return JOT_ERR_HIP;
}

int jot_wait_on_stream(jot_state* s, void* stream)
{
    if (!s) return JOT_ERR_NULL_POINTER;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (stream_is_capturing(st)) return JOT_ERR_INVALID_ARG;
    if (hipEventRecord(s->done, st) != hipSuccess) return JOT_ERR_HIP;
    s->have_done = true;
    s->sync_device = false;
    return JOT_OK;
}

int64_t jot_anomaly_count(jot_state* s)
{
    const int rc = wait_done(s);
    return rc != JOT_OK ? rc : (int64_t)s->host->anomalies;
}

const int32_t* jot_tokens(const jot_state* s) { return s ? s->at<int32_t>(s->lay.tokens) : nullptr; }
const uint8_t* jot_masked(const jot_state* s) { return s ? s->at<uint8_t>(s->lay.masked) : nullptr; }
const int32_t* jot_commit_step(const jot_state* s) { return s ? s->at<int32_t>(s->lay.commit_step) : nullptr; }
const int32_t* jot_active_list(jot_state* s)
{
    if (!s || wait_done(s) != JOT_OK) return nullptr;
    return s->active(s->host->parity);
}

const int32_t* jot_commit_log(jot_state* s, int64_t* n)
{
    if (!s || !n || wait_done(s) != JOT_OK) return nullptr;
    *n = s->host->c.n_log;
    return s->at<int32_t>(s->lay.commit_log);
}

const int32_t* jot_examined_list(jot_state* s, int64_t* n)
{
    if (!s || !n || wait_done(s) != JOT_OK) return nullptr;
    *n = s->host->c.n_examined;
    return s->active(s->host->parity ^ 1);
}

const int32_t* jot_last_token(const jot_state* s) { return s ? s->at<int32_t>(s->lay.last_token) : nullptr; }
const int32_t* jot_last_final_token(const jot_state* s) { return s ? s->at<int32_t>(s->lay.last_final) : nullptr; }
const float* jot_last_conf(const jot_state* s) { return s ? s->at<float>(s->lay.last_conf) : nullptr; }
const float* jot_last_p1(const jot_state* s) { return s ? s->at<float>(s->lay.last_p1) : nullptr; }
const float* jot_last_p2(const jot_state* s) { return s ? s->at<float>(s->lay.last_p2) : nullptr; }
const float* jot_last_tau(const jot_state* s) { return s ? s->at<float>(s->lay.last_tau) : nullptr; }
const uint8_t* jot_last_flags(const jot_state* s) { return s ? s->at<uint8_t>(s->lay.last_flags) : nullptr; }
const float* jot_last_gap(const jot_state* s) { return s ? s->at<float>(s->lay.last_gap) : nullptr; }
const float* jot_last_kl(const jot_state* s) { return s ? s->at<float>(s->lay.last_kl) : nullptr; }

int jot_profile_enable(jot_state* s, int on)
{
    if (!s) return JOT_ERR_NULL_POINTER;
    if (on && !s->profile) {
        int made = 0;                       // events created so far (prof0[k] before prof1[k])
        for (int k = 0; k < JOT_PROFILE_RING; ++k) {
            s->prof_step[k] = 0;
            if (hipEventCreate(&s->prof0[k]) != hipSuccess) break;
            ++made;
            if (hipEventCreate(&s->prof1[k]) != hipSuccess) break;
            ++made;
        }
        if (made != 2 * JOT_PROFILE_RING) {     // give back what was created
            for (int k = 0; k < made; ++k)
                (void)hipEventDestroy((k & 1) ? s->prof1[k >> 1] : s->prof0[k >> 1]);
            (void)hipGetLastError();
            return JOT_ERR_HIP;
        }
        s->profile = true;
    } else if (!on && s->profile) {
        for (int k = 0; k < JOT_PROFILE_RING; ++k) {
            (void)hipEventDestroy(s->prof0[k]);
            (void)hipEventDestroy(s->prof1[k]);
        }
        s->profile = false;
    }
    return JOT_OK;
}

int jot_profile_read(jot_state* s, int32_t step, float* vocab_reduce_ms)
{
    if (!s || !vocab_reduce_ms) return JOT_ERR_NULL_POINTER;
    if (!s->profile || step < 1) return JOT_ERR_INVALID_ARG;
    const int slot = step % JOT_PROFILE_RING;
    if (s->prof_step[slot] != step) return JOT_ERR_INVALID_ARG;
    if (hipEventSynchronize(s->prof1[slot]) != hipSuccess) return JOT_ERR_HIP;
    if (hipEventElapsedTime(vocab_reduce_ms, s->prof0[slot], s->prof1[slot]) != hipSuccess) return JOT_ERR_HIP;
    return JOT_OK;
}

void jot_release(jot_state* s)
{
    if (!s) return;
    (void)wait_done(s);       // the last step's final kernel writes into the pinned block freed below
    if (s->profile) (void)jot_profile_enable(s, 0);
    (void)hipEventDestroy(s->done);
    if (s->host) (void)hipHostFree(s->host);
    delete s;
}

const char* jot_strerror(int code)
{
    switch (code) {
    case JOT_OK: return "success";
    case JOT_ERR_INVALID_ARG: return "invalid argument";
    case JOT_ERR_NULL_POINTER: return "null pointer";
    case JOT_ERR_UNSUPPORTED_DTYPE: return "unsupported logit dtype";
    case JOT_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case JOT_ERR_MISALIGNED: return "misaligned pointer or stride";
    case JOT_ERR_HIP: return "HIP runtime error";
    case JOT_ERR_NO_DEVICE: return "no HIP device";
    case JOT_ERR_NO_MEMORY: return "out of host memory";
    case JOT_ERR_WRONG_DEVICE: return "state belongs to another HIP device";
    case JOT_ERR_TOO_LARGE: return "problem needs more working memory than the library's fixed scratch array holds";
    default: return "unknown error";
    }
}

}  // extern "C"
