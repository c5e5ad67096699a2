// Per-head influence metric of the plan search (Sec. 3.4.1, Eq. 1, as Alg. 1 applies it per head):
//   I[h] = sum (y_m - y_o)^2 / sum (y_o - mean(y_o))^2   over the batch entries, tokens and features of head h.
// Two launches: rse_partial_kernel streams both tensors once (HBM bound: 2 * B * H * N * D * elem bytes)
// and leaves three fp64 sums per (batch, head, chunk); rse_final_kernel adds them in a fixed order and divides.
// The spread of y_o is accumulated about a pivot (the head's first element) and corrected by the pivot's
// distance to the mean at the end, var * n = S2 - S1^2 / n, so a large common offset costs no digits.
#include "difa_internal.h"

namespace difa {

typedef float rse_floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int rse_uintx4 __attribute__((ext_vector_type(4)));

// eight bf16 values (or four fp32 values) of one 16-byte vector, widened to fp32
template <typename T> struct RseVec;
template <> struct RseVec<__bf16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void widen(const rse_uintx4& raw, float (&x)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __builtin_bit_cast(float, raw[i] << 16);             // a bf16 is the upper half of an fp32
            x[2 * i + 1] = __builtin_bit_cast(float, raw[i] & 0xffff0000u);
        }
    }
};
template <> struct RseVec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void widen(const rse_uintx4& raw, float (&x)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned u = raw[i];      // copied to a scalar first: a bit_cast applied directly to a vector element reads element 0
            x[i] = __builtin_bit_cast(float, u);
        }
    }
};

__device__ __forceinline__ double rse_wave_sum(double x) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) x += __shfl_xor(x, s, 64);
    return x;
}

template <typename T>
__global__ __launch_bounds__(256) void rse_partial_kernel(RseArgs a) {
    constexpr int NV = RseVec<T>::N;
    const int chunk = blockIdx.x, bh = blockIdx.y, b = bh / a.heads, h = bh - b * a.heads;
    const T* ym = (const T*)a.y_m + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const T* yo = (const T*)a.y_o + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const float pivot = (float)((const T*)a.y_o)[(int64_t)h * a.stride_h];   // one pivot per head, batch entry 0
    const int vpr = a.head_dim / NV;                  // 16-byte vectors per token row
    const int rows_per_pass = 256 / vpr;
    const int rows_per_chunk = (a.n_tokens + (int)gridDim.x - 1) / (int)gridDim.x;
    const int r0 = chunk * rows_per_chunk;
    const int r1 = r0 + rows_per_chunk < a.n_tokens ? r0 + rows_per_chunk : a.n_tokens;
    const int col = ((int)threadIdx.x % vpr) * NV;
    double s_err = 0.0, s_1 = 0.0, s_2 = 0.0;
    auto add = [&](const rse_uintx4& rm, const rse_uintx4& ro) {
        float m[NV], o[NV];
        RseVec<T>::widen(rm, m);
        RseVec<T>::widen(ro, o);
        float e = 0.f, t1 = 0.f, t2 = 0.f;         // fp32 over one vector, fp64 across vectors
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const float d = m[i] - o[i], c = o[i] - pivot;
            e = fmaf(d, d, e);
            t1 += c;
            t2 = fmaf(c, c, t2);
        }
        s_err += (double)e;
        s_1 += (double)t1;
        s_2 += (double)t2;
    };
    int r = r0 + (int)threadIdx.x / vpr;
    // four rows in flight per thread and tensor
    for (; r + 3 * rows_per_pass < r1; r += 4 * rows_per_pass) {
        rse_uintx4 vm[4], vo[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t off = (int64_t)(r + u * rows_per_pass) * a.stride_n + col;
            vm[u] = *(const rse_uintx4*)(ym + off);
            vo[u] = *(const rse_uintx4*)(yo + off);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) add(vm[u], vo[u]);
    }
    for (; r < r1; r += rows_per_pass) {
        const int64_t off = (int64_t)r * a.stride_n + col;
        add(*(const rse_uintx4*)(ym + off), *(const rse_uintx4*)(yo + off));
    }
    __shared__ double red[4][3];
    s_err = rse_wave_sum(s_err);
    s_1 = rse_wave_sum(s_1);
    s_2 = rse_wave_sum(s_2);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { red[wave][0] = s_err; red[wave][1] = s_1; red[wave][2] = s_2; }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int k = threadIdx.x;
        a.partial[((int64_t)bh * gridDim.x + chunk) * 3 + k] = (red[0][k] + red[1][k]) + (red[2][k] + red[3][k]);
    }
}

// One wavefront per head: lane c adds chunk c of every batch entry, the lanes are combined by a butterfly
// (a fixed order: the result does not depend on timing), lane 0 divides.
static_assert(kRseChunks == 64, "one lane per chunk");
__global__ __launch_bounds__(64) void rse_final_kernel(RseArgs a) {
    const int h = blockIdx.x, c = threadIdx.x;
    double s_err = 0.0, s_1 = 0.0, s_2 = 0.0;
    for (int b = 0; b < a.batch; ++b) {
        const double* p = a.partial + ((int64_t)(b * a.heads + h) * kRseChunks + c) * 3;
        s_err += p[0];
        s_1 += p[1];
        s_2 += p[2];
    }
    s_err = rse_wave_sum(s_err);
    s_1 = rse_wave_sum(s_1);
    s_2 = rse_wave_sum(s_2);
    if (c == 0) {
        const double n = (double)a.batch * a.n_tokens * a.head_dim;
        const double spread = s_2 - s_1 * s_1 / n;          // sum (y_o - mean)^2
        a.out[h] = (float)(s_err / spread);
    }
}

hipError_t launch_head_rse(const RseArgs& a, int dtype, hipStream_t stream) {
    const dim3 grid(kRseChunks, (unsigned)(a.batch * a.heads));
    if (dtype == DIFA_DTYPE_BF16) hipLaunchKernelGGL(rse_partial_kernel<__bf16>, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(rse_partial_kernel<float>, grid, dim3(256), 0, stream, a);
    hipLaunchKernelGGL(rse_final_kernel, dim3((unsigned)a.heads), dim3(64), 0, stream, a);
    return hipGetLastError();
}

}  // namespace difa
