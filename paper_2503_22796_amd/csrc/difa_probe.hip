// Measurement hook: the rate at which this GPU sustains v_mfma_f32_32x32x16_bf16 on given operand data.
//
// The attention kernel is priced against the published dense bf16 MFMA peak.  What the matrix cores
// sustain for longer than a few milliseconds depends on the operand bits: with all-zero operands an
// MI355X holds its full clock, with N(0,1) operands it reaches its power limit and lowers the clock.
// This probe runs nothing but independent MFMAs (one or two wavefronts per SIMD, every compute unit)
// on operands taken from a caller's buffer, so that bench.py can report that ceiling beside the
// attention kernel's rate.  It is not part of the operator.
#include <hip/hip_runtime.h>

#include "difa.h"

namespace difa {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

template <int NT>
__global__ __launch_bounds__(NT, 1) void mfma_rate_kernel(const __bf16* data, long long n_vec, int rounds, float* sink) {
    // eight A and eight B operands per lane, 16 bytes each, from consecutive 16-byte vectors of `data`
    probe_bf16x8 a[8], b[8];
    const long long first = ((long long)blockIdx.x * NT + threadIdx.x) * 16;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = *(const probe_bf16x8*)(data + 8 * ((first + i) % n_vec));
        b[i] = *(const probe_bf16x8*)(data + 8 * ((first + 8 + i) % n_vec));
    }
    probe_floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    // 64 MFMAs per round, every A paired with every B; four accumulators, so no MFMA waits for the one before it
    for (int it = 0; it < rounds; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[(i + r) & 7], acc[i & 3], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[i][r];
    if (sum == 123.456f) *sink = sum;      // keeps the accumulators alive; practically never true
}

}  // namespace difa

extern "C" difa_status_t difa_probe_mfma_rate(const void* data, int64_t n_elems, int32_t waves_per_simd,
                                              int32_t rounds, void* scratch4, void* stream_v,
                                              double* tflops_out, double* ms_out) {
    if (!data || !scratch4 || !tflops_out || n_elems < 8 || rounds < 1 || rounds > (1 << 22) ||
        (waves_per_simd != 1 && waves_per_simd != 2))
        return DIFA_ERR_INVALID_ARG;
    if (((uintptr_t)data & 15) != 0) return DIFA_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_v;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return DIFA_ERR_HIP;
    const int n_wg = prop.multiProcessorCount;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return DIFA_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return DIFA_ERR_HIP; }
    const long long n_vec = n_elems / 8;
    auto launch = [&](int r) {
        if (waves_per_simd == 1)
            hipLaunchKernelGGL(difa::mfma_rate_kernel<256>, dim3(n_wg), dim3(256), 0, stream, (const __bf16*)data, n_vec, r, (float*)scratch4);
        else
            hipLaunchKernelGGL(difa::mfma_rate_kernel<512>, dim3(n_wg), dim3(512), 0, stream, (const __bf16*)data, n_vec, r, (float*)scratch4);
    };
    launch(rounds / 8 > 0 ? rounds / 8 : 1);     // untimed: code load, clocks up
    hipError_t e = hipEventRecord(e0, stream);
    launch(rounds);
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return DIFA_ERR_HIP;
    // 32 x 32 x 16 multiply-adds per MFMA, 64 MFMAs per round and wavefront, 4 * waves_per_simd wavefronts per workgroup
    const double flops = 2.0 * 32 * 32 * 16 * 64.0 * rounds * 4.0 * waves_per_simd * n_wg;
    *tflops_out = flops / (ms * 1e-3) * 1e-12;
    if (ms_out) *ms_out = ms;
    return DIFA_OK;
}
