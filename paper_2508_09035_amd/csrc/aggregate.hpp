// Aggregation of token-importance scores over attention layers and heads
// (paper Section 4.4: several layers take part in the selection, their weight
// distributions differ in magnitude, and the choice of layers is left open).
//
//   out[h, j] (+)= sum_l w_l * scores[l, h, j]              (per head row)
//   out[0, j] (+)= sum_l w_l * sum_h scores[l, h, j]        (heads reduced)
//
// Streaming, HBM bound: every score is read once, every output written once
// (read first when accumulating).  One thread per 4 consecutive tokens
// (16-byte accesses); layers then heads are added in ascending order in fp32,
// so results are deterministic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdd {

typedef float agg_f32x4 __attribute__((ext_vector_type(4)));

struct AggParams {
    const float *scores;     // [n_layers, n_heads, total_k], layer stride in elements
    const float *weights;    // [n_layers] or nullptr (= 1)
    float *out;              // [n_heads or 1, total_k]
    int64_t layer_stride;
    int32_t n_layers, n_heads, total_k, reduce_heads, accumulate;
};

template <int VEC>
__global__ __launch_bounds__(256) void aggregate_scores_kernel(const AggParams p)
{
    const int64_t j0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (j0 >= p.total_k) return;
    const int row = blockIdx.y;                       // output row
    const int h_lo = p.reduce_heads ? 0 : row, h_hi = p.reduce_heads ? p.n_heads : row + 1;
    float acc[VEC];
    float *op = p.out + (int64_t)row * p.total_k + j0;
    if (p.accumulate) {
        if constexpr (VEC == 4) { const agg_f32x4 t = *(const agg_f32x4 *)op; acc[0] = t.x; acc[1] = t.y; acc[2] = t.z; acc[3] = t.w; }
        else acc[0] = *op;
    } else {
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
    }
    for (int l = 0; l < p.n_layers; ++l) {
        const float w = p.weights ? p.weights[l] : 1.f;
        const float *sp = p.scores + (int64_t)l * p.layer_stride + (int64_t)h_lo * p.total_k + j0;
        float part[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) part[c] = 0.f;
        for (int h = h_lo; h < h_hi; ++h, sp += p.total_k) {
            if constexpr (VEC == 4) {
                const agg_f32x4 t = __builtin_nontemporal_load((const agg_f32x4 *)sp);
                part[0] += t.x; part[1] += t.y; part[2] += t.z; part[3] += t.w;
            } else {
                part[0] += *sp;
            }
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] = fmaf(w, part[c], acc[c]);
    }
    if constexpr (VEC == 4) { const agg_f32x4 t = {acc[0], acc[1], acc[2], acc[3]}; *(agg_f32x4 *)op = t; }
    else *op = acc[0];
}

}  // namespace pdd
