// Selection mask -> bit stream (paper Section 3.2: the mask tensor, 1 at
// position i = token i selected, is treated as a bit stream before it is
// compressed for transmission).  Per (head row, sequence) the stream starts at
// a byte boundary; byte j holds tokens 8j .. 8j+7, first token in the most
// significant bit; the tail of the last byte is zero.
//
// One thread makes one output byte from eight mask bytes: a single 8-byte load
// when the sequence's first token is 8-byte aligned in memory (byte loads
// otherwise and for the ragged tail), the non-zero flags of the eight bytes are
// gathered into one byte with a multiply.  Loads of 512 B and stores of 64 B per
// wave, both contiguous.  HBM traffic: 1 B read per token, 1/8 B written.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdd {

struct PackParams {
    const uint8_t *mask;      // [rows, total_k]
    uint8_t *bits;            // [rows, total_bytes]
    const int32_t *cu_k;      // [B+1]
    const int32_t *cu_bytes;  // [B+1] byte offsets of the sequences' streams inside a row
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
    const int nbytes = min(b1 - b0, (nk + 7) / 8);    // bytes written: what the sequence needs, inside its span
    const int j = blockIdx.x * kPackThreads + threadIdx.x;       // output byte = tokens 8j .. 8j+7
    if (j >= nbytes) return;
    const uint8_t *src = p.mask + (int64_t)r * p.total_k + ks;
    const int t0 = 8 * j;
    uint64_t w = 0;                                   // token t0 + t in byte t
    if (t0 + 8 <= nk && (((uintptr_t)src) & 7) == 0) {
        w = *(const uint64_t *)(src + t0);
    } else {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (t0 + t < nk) w |= (uint64_t)src[t0 + t] << (8 * t);
    }
    // non-zero flag of every byte in its bit 0 ...
    w |= w >> 4;  w |= w >> 2;  w |= w >> 1;
    w &= 0x0101010101010101ull;
    // ... gathered, first token in the most significant bit: flag t moves from bit 8t to
    // bit 63 - t of the product (no two partial products meet, so there are no carries)
    p.bits[(int64_t)r * p.total_bytes + b0 + j] = (uint8_t)((w * 0x8040201008040201ull) >> 56);
}

}  // namespace pdd
