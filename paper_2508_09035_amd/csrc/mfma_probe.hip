// Measurement helper (not part of the method): what the bf16 matrix pipe of this
// GPU sustains on its own, as a reference point beside the published peak.
//
// Every wave runs nothing but v_mfma_f32_32x32x16_bf16 on four independent
// accumulators, two waves per SIMD, one workgroup of 8 waves per compute unit
// and round.  Two operand regimes:
//   constant  every MFMA reads the same A and B fragment (little switching
//             activity in the multipliers);
//   varying   eight different A and B fragments taken from a caller-supplied
//             buffer (random bf16 patterns) are cycled, so consecutive MFMAs
//             see unrelated operands, as in a real contraction.
// The loop is bound by the matrix pipe alone (32 cycles per MFMA and SIMD), so
// cycles needed / duration bounds the clock the run had from below.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int kThreads = 512;
constexpr int kFrags = 8;

template <bool VARYING>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void mfma_probe_kernel(const uint16_t *operands, int iters, float *sink)
{
#if defined(__HIP_DEVICE_COMPILE__)
    bf16x8 a[kFrags], b[kFrags];
    if (VARYING) {
        // 2 * kFrags fragments of 16 bytes per lane: 16 KiB per wave, 128 KiB per workgroup
        const bf16x8 *src = (const bf16x8 *)operands + (size_t)threadIdx.x * 2 * kFrags;
#pragma unroll
        for (int i = 0; i < kFrags; ++i) { a[i] = src[i]; b[i] = src[kFrags + i]; }
    } else {
#pragma unroll
        for (int i = 0; i < kFrags; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) { a[i][e] = (__bf16)1.0f; b[i][e] = (__bf16)0.5f; }
    }
    f32x16 c[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) c[r][e] = 0.f;

    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kFrags; ++i)
            c[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], c[i & 3], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += c[r][e];
    sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = s;
#else
    (void)operands; (void)iters; (void)sink;
#endif
}

}  // namespace

extern "C" {

// Bytes of `operands` the varying mode reads (random bf16 patterns with finite values).
int pdd_probe_operand_bytes(void) { return kThreads * 2 * kFrags * 16; }

// MFMA flops one launch executes.
double pdd_probe_mfma_flops(int blocks, int iters)
{
    return (double)blocks * (kThreads / 64) * (double)iters * kFrags * 2.0 * 32 * 32 * 16;
}

// Enqueue one probe launch on `stream`.  All pointers are DEVICE memory owned by the
// caller: operands (pdd_probe_operand_bytes() bytes, read only when varying != 0),
// sink float[blocks * 512].  Returns 0, or the hipError_t of a failed launch.
int pdd_probe_mfma(int varying, int blocks, int iters, const void *operands, void *sink, void *stream)
{
    if (blocks < 1 || iters < 1 || !sink || (varying && !operands)) return (int)hipErrorInvalidValue;
    if (varying)
        hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream,
                           (const uint16_t *)operands, iters, (float *)sink);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream,
                           (const uint16_t *)operands, iters, (float *)sink);
    return (int)hipGetLastError();
}

}  // extern "C"
