/*
 * A plain C client of include/jot.h (no Python, no C++): reads a small problem from raw files,
 * runs a few finalization steps through the C ABI and writes the results back as raw files.
 * tests/test_gpu_c_client.py builds it with gcc, runs it and compares with the CPU oracle.
 *
 * usage: c_abi_client <dir> B L V dtype conf_mode tau_max tau_min gamma D gen_start block_size n_steps
 *   <dir>/tokens.i32 [B*L], <dir>/masked.u8 [B*L], <dir>/logits_<n>.bin [B*L*V] for n = 1..n_steps
 *   writes <dir>/out_tokens.i32, <dir>/out_masked.u8, <dir>/out_log.i32 (triples), <dir>/out_counts.i64
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "jot.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); return 3; } } while (0)
#define CHECK_JOT(x) do { int r_ = (x); if (r_ < 0) { \
    fprintf(stderr, "jot error %d (%s) at %s:%d\n", r_, jot_strerror(r_), __FILE__, __LINE__); return 4; } } while (0)

static void *slurp(const char *dir, const char *name, size_t bytes)
{
    char path[1024];
    snprintf(path, sizeof path, "%s/%s", dir, name);
    FILE *f = fopen(path, "rb");
    if (!f) { perror(path); exit(2); }
    void *buf = malloc(bytes ? bytes : 1);
    if (fread(buf, 1, bytes, f) != bytes) { fprintf(stderr, "short read: %s\n", path); exit(2); }
    fclose(f);
    return buf;
}

static void dump(const char *dir, const char *name, const void *buf, size_t bytes)
{
    char path[1024];
    snprintf(path, sizeof path, "%s/%s", dir, name);
    FILE *f = fopen(path, "wb");
    if (!f) { perror(path); exit(2); }
    fwrite(buf, 1, bytes, f);
    fclose(f);
}

int main(int argc, char **argv)
{
    if (argc != 14) { fprintf(stderr, "wrong number of arguments\n"); return 1; }
    const char *dir = argv[1];
    jot_params p;
    memset(&p, 0, sizeof p);
    p.B = atoi(argv[2]); p.L = atoi(argv[3]); p.V = atoi(argv[4]);
    p.dtype = atoi(argv[5]); p.conf_mode = atoi(argv[6]);
    p.tau_max = (float)atof(argv[7]); p.tau_min = (float)atof(argv[8]); p.gamma = (float)atof(argv[9]);
    p.D = atoi(argv[10]); p.eps = 1e-12f; p.gen_start = atoi(argv[11]); p.block_size = atoi(argv[12]);
    const int n_steps = atoi(argv[13]);
    const size_t n = (size_t)p.B * p.L, esz = p.dtype == JOT_F32 ? 4 : 2;
    /* rows must start on 16-byte boundaries: pad the row stride of the device tensor */
    const size_t stride_l = ((size_t)p.V + 7) & ~(size_t)7;

    const int64_t ws_bytes = jot_workspace_bytes(&p);
    CHECK_JOT((int)(ws_bytes < 0 ? ws_bytes : 0));

    int32_t *tokens = slurp(dir, "tokens.i32", n * 4);
    uint8_t *masked = slurp(dir, "masked.u8", n);
    void *ws_dev, *tokens_dev, *masked_dev, *logits_dev;
    CHECK_HIP(hipMalloc(&ws_dev, (size_t)ws_bytes));
    CHECK_HIP(hipMalloc(&tokens_dev, n * 4));
    CHECK_HIP(hipMalloc(&masked_dev, n));
    CHECK_HIP(hipMalloc(&logits_dev, n * stride_l * esz));
    CHECK_HIP(hipMemcpy(tokens_dev, tokens, n * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(masked_dev, masked, n, hipMemcpyHostToDevice));

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    jot_state *st = NULL;
    CHECK_JOT(jot_init_state(&st, &p, ws_dev, ws_bytes, tokens_dev, masked_dev, stream));

    int64_t counts[64];
    int steps_run = 0;
    for (int s = 1; s <= n_steps && s < 64; s++) {
        if (jot_active_count(st) == 0)
            break;                                   /* Algorithm 1: leave the loop when nothing is masked */
        char name[64];
        snprintf(name, sizeof name, "logits_%d.bin", s);
        void *lg = slurp(dir, name, n * p.V * esz);
        CHECK_HIP(hipMemcpy2DAsync(logits_dev, stride_l * esz, lg, (size_t)p.V * esz, (size_t)p.V * esz, n,
                                   hipMemcpyHostToDevice, stream));
        CHECK_JOT(jot_step(st, logits_dev, (int64_t)(p.L * stride_l), (int64_t)stride_l, stream));
        /* the non-blocking form: poll until the step has closed, then the blocking call must agree */
        int64_t polled = -1;
        for (long spins = 0; spins < 200000000L; spins++) {
            int32_t done = -1;
            polled = jot_active_count_poll(st, &done);
            if (polled < 0) { fprintf(stderr, "poll failed: %s\n", jot_strerror((int)polled)); return 6; }
            if (done >= steps_run + 1)
                break;
            polled = -1;
        }
        counts[steps_run++] = jot_active_count(st);  /* also makes it safe to free the host copy */
        if (polled != counts[steps_run - 1]) { fprintf(stderr, "polled count %lld differs from %lld\n",
                                                      (long long)polled, (long long)counts[steps_run - 1]); return 6; }
        free(lg);
    }
    if (jot_step_index(st) != steps_run) { fprintf(stderr, "step index mismatch\n"); return 5; }

    int64_t n_log = 0;
    const int32_t *log_dev = jot_commit_log(st, &n_log);
    int32_t *log = malloc((size_t)(n_log ? n_log : 1) * 12);
    CHECK_HIP(hipMemcpy(tokens, jot_tokens(st), n * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(masked, jot_masked(st), n, hipMemcpyDeviceToHost));
    if (n_log)
        CHECK_HIP(hipMemcpy(log, log_dev, (size_t)n_log * 12, hipMemcpyDeviceToHost));
    dump(dir, "out_tokens.i32", tokens, n * 4);
    dump(dir, "out_masked.u8", masked, n);
    dump(dir, "out_log.i32", log, (size_t)n_log * 12);
    dump(dir, "out_counts.i64", counts, (size_t)steps_run * 8);

    jot_release(st);
    CHECK_HIP(hipStreamDestroy(stream));
    CHECK_HIP(hipFree(ws_dev)); CHECK_HIP(hipFree(tokens_dev)); CHECK_HIP(hipFree(masked_dev)); CHECK_HIP(hipFree(logits_dev));
    free(tokens); free(masked); free(log);
    printf("ok: %d steps, %lld finalized\n", steps_run, (long long)n_log);
    return 0;
}
