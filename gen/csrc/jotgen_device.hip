// Synthetic logit rows, device implementation (gfx950).  Byte-for-byte the same function of
// (seed, step, position, vocabulary index) as jotgen_host.c: Philox4x32-10 counter RNG
// (Salmon et al., SC'11), inverse-CDF table with linear interpolation, planted target / rival
// logits.  Every floating-point step is one correctly rounded binary32 operation (explicit
// __fmul_rn / __fadd_rn / __fsub_rn, so nothing is contracted into an FMA).
// Input generation only: no softmax, threshold or decision here.
#include <hip/hip_runtime.h>
#include <stdint.h>

#define GEN_TABLE_LEN 1666
#define GEN_WG 256

__device__ __forceinline__ void philox4x32_10(uint32_t (&c)[4], uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
        const uint32_t n0 = hi1 ^ c[1] ^ k0, n1 = lo1, n2 = hi0 ^ c[3] ^ k1, n3 = lo0;
        c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
}

__device__ __forceinline__ float noise_from_bits(uint32_t u, const float* tab)
{
    const uint32_t k = u & 0x7FFFFFFFu;
    uint32_t idx;
    float frac;
    if (k < 128u) {
        idx = k;
        frac = 0.0f;
    } else {
        const int len = 32 - __clz((int)k);
        const int sh = len - 7;
        idx = 64u + 64u * (uint32_t)sh + ((k >> sh) - 64u);
        const uint32_t rem = k & ((1u << sh) - 1u);
        const float scale = __uint_as_float((uint32_t)(127 - sh) << 23);
        frac = __fmul_rn(__uint2float_rn(rem), scale);
    }
    const float t0 = tab[idx], t1 = tab[idx + 1];
    const float v = __fadd_rn(t0, __fmul_rn(frac, __fsub_rn(t1, t0)));
    return (u >> 31) ? -v : v;
}

__device__ __forceinline__ uint32_t to_bf16(float x)
{
    const uint32_t b = __float_as_uint(x);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// One thread makes 8 consecutive vocabulary entries (two counter blocks) of one row.
// Row k of the launch is canvas position pos[k]; it is written at out + b*stride_b + i*stride_l.
template <int DTYPE>
__global__ __launch_bounds__(GEN_WG) void jotgen_rows_kernel(
    void* __restrict__ out, int64_t stride_b, int64_t stride_l, int L, int V,
    const int32_t* __restrict__ pos, const int64_t* __restrict__ n_rows_dev, int64_t n_rows,
    uint32_t step, uint32_t k0, uint32_t k1, uint32_t stream_id, const float* __restrict__ table,
    const int32_t* __restrict__ target, const float* __restrict__ T,
    const int32_t* __restrict__ rival, const float* __restrict__ R, int groups_per_row)
{
    __shared__ float tab[GEN_TABLE_LEN];
    for (int k = threadIdx.x; k < GEN_TABLE_LEN; k += GEN_WG)
        tab[k] = table[k];
    __syncthreads();
    const int64_t rows = n_rows_dev ? min(*n_rows_dev, n_rows) : n_rows;
    const int64_t gid = (int64_t)blockIdx.x * GEN_WG + threadIdx.x;
    const int64_t r = gid / groups_per_row;
    if (r >= rows)
        return;
    const int g8 = (int)(gid - r * groups_per_row);       // group of 8 elements
    const int v0 = g8 * 8;
    if (v0 >= V)
        return;
    const int p = pos[r];
    const int b = p / L, i = p - b * L;
    const int tg = target[p], rv = rival[p];
    float x[8];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t c[4] = { (uint32_t)(2 * g8 + h), (uint32_t)p, step, stream_id };
        philox4x32_10(c, k0, k1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int v = v0 + 4 * h + j;
            float val = noise_from_bits(c[j], tab);
            if (v == tg) val = __fadd_rn(val, T[p]);
            if (v == rv) val = __fadd_rn(val, R[p]);
            x[4 * h + j] = val;
        }
    }
    const int64_t row_off = (int64_t)b * stride_b + (int64_t)i * stride_l;
    if (DTYPE == 0) {
        float* o = reinterpret_cast<float*>(out) + row_off + v0;
        if (v0 + 8 <= V) {
            reinterpret_cast<float4*>(o)[0] = make_float4(x[0], x[1], x[2], x[3]);
            reinterpret_cast<float4*>(o)[1] = make_float4(x[4], x[5], x[6], x[7]);
        } else {
            for (int j = 0; j < 8 && v0 + j < V; ++j) o[j] = x[j];
        }
    } else {
        uint16_t* o = reinterpret_cast<uint16_t*>(out) + row_off + v0;
        if (v0 + 8 <= V) {
            uint4 w;
            w.x = to_bf16(x[0]) | (to_bf16(x[1]) << 16);
            w.y = to_bf16(x[2]) | (to_bf16(x[3]) << 16);
            w.z = to_bf16(x[4]) | (to_bf16(x[5]) << 16);
            w.w = to_bf16(x[6]) | (to_bf16(x[7]) << 16);
            *reinterpret_cast<uint4*>(o) = w;
        } else {
            for (int j = 0; j < 8 && v0 + j < V; ++j) o[j] = (uint16_t)to_bf16(x[j]);
        }
    }
}

// Fill `count` 32-bit words with a pattern (used to poison logits that must never be read).
__global__ __launch_bounds__(GEN_WG) void jotgen_fill_kernel(uint32_t* p, int64_t count, uint32_t value)
{
    const int64_t stride = (int64_t)gridDim.x * GEN_WG;
    for (int64_t k = (int64_t)blockIdx.x * GEN_WG + threadIdx.x; k < count; k += stride)
        p[k] = value;
}

extern "C" {

// All pointers are device pointers except none; rows must be 16-byte aligned (out, strides).
// n_rows_dev (optional, may be NULL): device int64 with the actual number of rows (<= n_rows).
// Returns 0 or the hipError_t of the launch.
int jotgen_rows_device(void* out_dev, int dtype, int64_t stride_b, int64_t stride_l, int32_t L,
                       int32_t V, const int32_t* pos_dev, const int64_t* n_rows_dev, int64_t n_rows,
                       uint32_t step, uint64_t seed, uint32_t stream_id, const float* table_dev,
                       const int32_t* target_dev, const float* T_dev, const int32_t* rival_dev,
                       const float* R_dev, void* stream)
{
    if (n_rows <= 0) return 0;
    const int groups = (V + 7) / 8;
    const int64_t threads = n_rows * groups;
    const int64_t blocks = (threads + GEN_WG - 1) / GEN_WG;
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    if (dtype == 0)
        hipLaunchKernelGGL(jotgen_rows_kernel<0>, dim3((unsigned)blocks), dim3(GEN_WG), 0, st, out_dev,
                           stride_b, stride_l, L, V, pos_dev, n_rows_dev, n_rows, step, k0, k1, stream_id,
                           table_dev, target_dev, T_dev, rival_dev, R_dev, groups);
    else
        hipLaunchKernelGGL(jotgen_rows_kernel<1>, dim3((unsigned)blocks), dim3(GEN_WG), 0, st, out_dev,
                           stride_b, stride_l, L, V, pos_dev, n_rows_dev, n_rows, step, k0, k1, stream_id,
                           table_dev, target_dev, T_dev, rival_dev, R_dev, groups);
    return (int)hipGetLastError();
}

int jotgen_fill_device(void* p_dev, int64_t n_words, uint32_t value, void* stream)
{
    if (n_words <= 0) return 0;
    hipLaunchKernelGGL(jotgen_fill_kernel, dim3(8192), dim3(GEN_WG), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<uint32_t*>(p_dev), n_words, value);
    return (int)hipGetLastError();
}

}  // extern "C"
