// Selection mask -> bit stream (paper Section 3.2: the mask tensor, 1 at
// position i = token i selected, is treated as a bit stream before it is
// compressed for transmission).  Per (head row, sequence) the stream starts at
// a byte boundary; byte j holds tokens 8j .. 8j+7, first token in the most
// significant bit; the tail of the last byte is zero.
//
// A wave reads 64 consecutive mask bytes (coalesced), one ballot turns them into
// a 64-bit word, and eight lanes write the eight output bytes.  HBM traffic: 1 B
// read per token, 1/8 B written.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdd {

struct PackParams {
    const uint8_t *mask;      // [rows, total_k]
    uint8_t *bits;            // [rows, total_bytes]
    const int32_t *cu_k;      // [B+1]
    const int32_t *cu_bytes;  // [B+1], cu_bytes[b+1] - cu_bytes[b] >= ceil(Nk_b / 8)
    int32_t rows, B, total_k, total_bytes;
};

constexpr int kPackThreads = 256;

__global__ __launch_bounds__(kPackThreads) void pack_mask_kernel(const PackParams p)
{
    const int b = blockIdx.y, r = blockIdx.z;
    const int ks = min(max(p.cu_k[b], 0), p.total_k);
    const int ke = min(max(p.cu_k[b + 1], ks), p.total_k);
    const int nk = ke - ks;
    const int b0 = min(max(p.cu_bytes[b], 0), p.total_bytes);
    const int b1 = min(max(p.cu_bytes[b + 1], b0), p.total_bytes);
    const int nbytes = b1 - b0;                       // bytes reserved for this sequence
    const int lane = threadIdx.x & 63;
    const int tok0 = (blockIdx.x * kPackThreads + (threadIdx.x & ~63));   // first token of this wave
    if (tok0 >= 8 * nbytes) return;
    const int tok = tok0 + lane;
    const uint8_t m = tok < nk ? p.mask[(int64_t)r * p.total_k + ks + tok] : 0;
    const uint64_t w = __ballot(m != 0);              // bit i = token tok0 + i
    // byte j of the stream = tokens 8j..8j+7, first token in the MSB
    const int byte_idx = (tok0 >> 3) + lane;
    if (lane < 8 && byte_idx < nbytes) {
        const uint32_t eight = (uint32_t)(w >> (8 * lane)) & 0xffu;       // token 8j+t at bit t
        p.bits[(int64_t)r * p.total_bytes + b0 + byte_idx] = (uint8_t)(__brev(eight) >> 24);
    }
}

}  // namespace pdd
