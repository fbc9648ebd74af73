/*
 * Synthetic logit rows, host implementation.
 *
 * A row is a pure function of (seed, step, flattened position, vocabulary index):
 *
 *   bits  = Philox4x32-10( counter = (v / 4, position, step, stream), key = seed )[v % 4]
 *           (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11)
 *   noise = inverse-CDF table lookup of the 31 low bits, linearly interpolated, sign from bit 31
 *   logit = noise (+ T[position] if v == target[position]) (+ R[position] if v == rival[position])
 *
 * The table is built once on the host in double (see tables.py) and handed to this file and to
 * the device implementation as the same bytes; every floating-point step here is a single
 * IEEE-754 binary32 operation (compile with -ffp-contract=off), so the device implementation
 * produces identical bytes.  There is no softmax, threshold or decision in this file.
 */
#include <stdint.h>
#include <string.h>

enum { GEN_F32 = 0, GEN_BF16 = 1 };
#define GEN_TABLE_LEN 1666   /* 64 direct + 25 octaves x 64 segments + closing entry + pad */

static void philox4x32_10(uint32_t c[4], uint32_t k0, uint32_t k1)
{
    for (int r = 0; r < 10; r++) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
}

void jotgen_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c[4] = { ctr[0], ctr[1], ctr[2], ctr[3] };
    philox4x32_10(c, key[0], key[1]);
    memcpy(out, c, sizeof c);
}

/* 31 bits -> table segment and position inside it.
 * k < 128: one entry per value.  Otherwise the top 7 bits of k pick one of 64 segments in k's
 * octave and the remaining bits (at most 24, so exact in binary32) give the fraction. */
static float noise_from_bits(uint32_t u, const float *tab)
{
    uint32_t k = u & 0x7FFFFFFFu;
    uint32_t idx;
    float frac;
    if (k < 128u) {
        idx = k;
        frac = 0.0f;
    } else {
        int len = 32 - __builtin_clz(k);           /* 8..31 */
        int sh = len - 7;                          /* 1..24 */
        idx = 64u + 64u * (uint32_t)sh + ((k >> sh) - 64u);
        uint32_t rem = k & ((1u << sh) - 1u);
        uint32_t scale_bits = (uint32_t)(127 - sh) << 23;   /* 2^-sh */
        float scale;
        memcpy(&scale, &scale_bits, sizeof scale);
        frac = (float)rem * scale;
    }
    float t0 = tab[idx], t1 = tab[idx + 1];
    float d = t1 - t0;
    float m = frac * d;
    float v = t0 + m;
    return (u >> 31) ? -v : v;
}

static uint16_t to_bf16(float x)
{
    uint32_t b;
    memcpy(&b, &x, sizeof b);
    return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

/*
 * out        : n_rows rows of V elements, row k at element offset k*out_row_stride
 * pos        : [n_rows] flattened canvas position b*L+i of each row
 * target/T   : per flattened position (arrays over the whole canvas); target < 0 = none
 * rival/R    : same for the optional second planted token
 * table      : GEN_TABLE_LEN floats
 */
void jotgen_rows_host(void *out, int dtype, int64_t n_rows, int32_t V, int64_t out_row_stride,
                      const int64_t *pos, uint32_t step, uint64_t seed, uint32_t stream,
                      const float *table, const int32_t *target, const float *T,
                      const int32_t *rival, const float *R, int threads)
{
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
#endif
    for (int64_t r = 0; r < n_rows; r++) {
        const int64_t p = pos[r];
        const int32_t tg = target[p], rv = rival[p];
        for (int32_t g = 0; g * 4 < V; g++) {
            uint32_t c[4] = { (uint32_t)g, (uint32_t)p, step, stream };
            philox4x32_10(c, k0, k1);
            for (int j = 0; j < 4; j++) {
                int32_t v = g * 4 + j;
                if (v >= V)
                    break;
                float x = noise_from_bits(c[j], table);
                if (v == tg)
                    x = x + T[p];
                if (v == rv)
                    x = x + R[p];
                if (dtype == GEN_F32)
                    ((float *)out)[r * out_row_stride + v] = x;
                else
                    ((uint16_t *)out)[r * out_row_stride + v] = to_bf16(x);
            }
        }
    }
}
