// The A-operand table of the dense large kernel's matrix path (esc_dense.hip), entry by entry:
// shared by the small kernel that builds it and by the estimator launch, which builds it on the
// side when a dense call has an estimator to run (one launch less).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace esc {

typedef unsigned dw_u32x4 __attribute__((ext_vector_type(4)));

// fp32 -> bf16, round to nearest even, NaN kept quiet
__device__ __forceinline__ uint16_t dw_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// a value as three bf16 terms by truncation (the top eight mantissa bits, the next eight, the
// rest): exact (but for values within 2^24 of the smallest normal number)
__device__ __forceinline__ void dw_split3(float v, uint16_t (&t)[3])
{
    const uint32_t hb = __float_as_uint(v) & 0xffff0000u;
    const float r1 = v - __uint_as_float(hb);
    const uint32_t mb = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(mb);
    t[0] = (uint16_t)(hb >> 16), t[1] = (uint16_t)(mb >> 16), t[2] = (uint16_t)(__float_as_uint(r2) >> 16);
}

// entries of the table: one per (pair of tap columns, kernel row, lane)
__host__ __device__ inline int dense_table_entries(int Kse) { return (Kse + 1) / 2 * Kse * 64; }

// wa[pair of columns jp][kernel row i][term][lane l][8 bf16]: lane l holds output channel l % 16,
// tap (i, 2 jp + l / 32), input channels 8 ((l / 16) % 2) .. + 7 - the A operand of the
// instruction; zero beyond the kernel (the last pair's second column) and beyond C_a.  Terms:
// nw == 2: hi = bf16(w), lo = bf16(w - hi) (bf16 storage); nw == 3: the exact split (fp32 storage).
// Entry idx = (jp * Kse + i) * 64 + l, all its terms.
__device__ __forceinline__ void dense_table_entry(const float *lk, int Ca, int Ks, int Kse, int nw, uint32_t *wa, int idx)
{
    const int q = idx >> 6, l = idx & 63, co = l & 15, kg = l >> 4, off = (Kse - Ks) / 2;
    const int jp = q / Kse, i = q - jp * Kse - off, j = 2 * jp + (kg >> 1) - off;
    uint32_t term[3][4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint16_t t2[2][3];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int ci = 8 * (kg & 1) + 2 * w + s;
            const bool in = co < Ca && ci < Ca && i >= 0 && i < Ks && j >= 0 && j < Ks;
            const float v = in ? lk[(((size_t)co * Ca + ci) * Ks + i) * Ks + j] : 0.f;
            if (nw == 3) {
                dw_split3(v, t2[s]);
            } else {
                t2[s][0] = dw_f32_to_bf16(v);
                t2[s][1] = dw_f32_to_bf16(v - __uint_as_float((uint32_t)t2[s][0] << 16));
                t2[s][2] = 0;
            }
        }
#pragma unroll
        for (int t = 0; t < 3; ++t) term[t][w] = (uint32_t)t2[0][t] | ((uint32_t)t2[1][t] << 16);
    }
    dw_u32x4 *dst = reinterpret_cast<dw_u32x4 *>(wa) + (size_t)q * nw * 64 + l;
    for (int t = 0; t < nw; ++t) dst[t * 64] = dw_u32x4{term[t][0], term[t][1], term[t][2], term[t][3]};
}

}  // namespace esc
