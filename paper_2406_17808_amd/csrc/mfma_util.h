// Device helpers of the bf16 MFMA attention kernel: fragment types, packed conversion, the
// cross-half reduction of the S^T layout and the iterator over the key tiles of a segment list.
//
// MFMA used: v_mfma_f32_32x32x16_bf16, D[m][n] += sum_k A[m][k] B[k][n] with, for lane l,
//   A: row m = l%32, k = 8*(l/32) .. +7        B: column n = l%32, k = 8*(l/32) .. +7
//   D: column n = l%32, rows 8*(j/4) + 4*(l/32) + j%4 for accumulator register j = 0..15.
//
// Attention computes S^T = K Q^T (keys are rows, queries are columns), so one lane owns one
// query: row max and row sum are in-lane reductions plus one exchange with lane l^32, and the
// probabilities sit in the accumulators exactly as the B operand of O^T = V^T P^T needs them
// (the contraction index runs over keys in the accumulator's own order; the V^T tile in LDS is
// stored in that same order).
#pragma once

#include "launch.h"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

union Frag {
    bf16x8_t v;
    u32x4_t u;
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

// two floats -> packed bf16 pair (v_cvt_pk_bf16_f32, round to nearest even)
__device__ inline uint32_t cvt_pk_bf16(float lo, float hi)
{
    const f32x2_t x = {lo, hi};
    const bf16x2_t y = __builtin_convertvector(x, bf16x2_t);
    return __builtin_bit_cast(uint32_t, y);
}

// max over the two lanes l and l^32 (they hold the two halves of one query's keys)
__device__ inline float max_xor32(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

constexpr int kBN = 64;               // keys per tile
constexpr int kScorePadRows = 64;     // the score kernel reads query rows in stages of this many: offsets exist for that many rows behind the chunk
constexpr float kRescaleLog2 = 8.f;   // the running maximum is only raised when it grew by 2^8
constexpr float kBoundLog2 = 90.f;    // exponents proven to stay this close to the running maximum need no tracking (2^90 x 2^17 keys < 2^127)

// Iterates over the 64-key tiles of all segments.  All fields are workgroup-uniform.
struct TileIter {
    int si, t0, len;
    Seg sg;
    __device__ void load(const SegList& sl, int wg_imax)
    {
        sg = sl.s[si];
        len = sg.chunk ? min(sg.len, wg_imax + 1) : sg.len;   // chunk keys after the last row are never visible
    }
    __device__ bool valid(const SegList& sl) const { return si < sl.n; }
    __device__ void first(const SegList& sl, int wg_imax)
    {
        si = 0; t0 = 0;
        if (valid(sl)) load(sl, wg_imax);
    }
    __device__ void next(const SegList& sl, int wg_imax)
    {
        t0 += kBN;
        if (t0 >= len) {
            ++si; t0 = 0;
            if (valid(sl)) load(sl, wg_imax);
        }
    }
};

}  // namespace ckv
