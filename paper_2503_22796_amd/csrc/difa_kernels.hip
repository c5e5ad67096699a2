// gfx950 kernels of the head-wise joint-attention operator (Sec. 3.3 of the paper):
//   attn_bf16_kernel  -- full / arrow heads, bf16 MFMA with fp32 accumulation
//   attn_f32_kernel   -- the same result in plain fp32 arithmetic (slow debug path)
//   cache_copy_kernel -- cached heads: out[b,h] = cache[b,h] (Alg. 1, last statement)
#include "difa_internal.h"

namespace difa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Exchange between lane l and lane l^32 (the two halves of a wavefront).
__device__ __forceinline__ float xchg32(float x) {
    return __shfl_xor(x, 32, 64);
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA attention.
//
// One workgroup = 4 wavefronts = one 128-row query tile of one (batch, head); wavefront w owns
// rows 32w..32w+31.  Key/value tiles of 64 keys are staged through LDS and visited in the order
// the host-compiled work record lists them (text tiles, then the band tiles), so a tile with no
// allowed pair is never loaded (Sec. 3.1 / 3.3: block-sparse band).
//
// Scores are produced transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then holds
// 16 keys of ONE query (column = lane % 32), so the softmax row statistics are per-lane scalars
// and need one exchange between the wavefront halves.  The same register layout is exactly the
// B operand of O^T = V^T P^T, so P never goes through LDS.
// ------------------------------------------------------------------------------------------
template <int D>
struct TileCfg {
    static constexpr int KSTR = D + 8;      // bf16 per K row in LDS (+16 B: conflict-free 16 B reads)
    static constexpr int VSTR = kBN + 4;    // bf16 per V^T row in LDS (+8 B: conflict-free 8 B reads)
};

template <int D>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnArgs a) {
    constexpr int KS = D / 16;        // MFMA k-steps of S^T = K Q^T
    constexpr int DB = D / 32;        // 32-row blocks of O^T
    constexpr int KSTR = TileCfg<D>::KSTR, VSTR = TileCfg<D>::VSTR;
    constexpr int CPR = D / 8;        // 16-byte chunks per K/V row
    constexpr int LOADS = kBN * CPR / 256;  // 16-byte loads per thread per tensor per tile

    __shared__ __attribute__((aligned(16))) __bf16 Ks[kBN * KSTR];
    __shared__ __attribute__((aligned(16))) __bf16 Vt[D * VSTR];

    const difa_work_item_t it = a.items[blockIdx.x];
    if (it.q_tile < 0) return;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int N = a.n_tokens, n_text = a.n_text;
    const int b = it.bh / a.heads, h = it.bh - b * a.heads;
    const int64_t base = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const __bf16* __restrict__ qg = (const __bf16*)a.q + base;
    const __bf16* __restrict__ kg = (const __bf16*)a.k + base;
    const __bf16* __restrict__ vg = (const __bf16*)a.v + base;
    __bf16* __restrict__ og = (__bf16*)a.out + base;

    const int row0 = it.q_tile * kBM + wave * 32;           // first query row of this wavefront
    const int i_raw = row0 + l32;
    const int i = i_raw < N ? i_raw : N - 1;                // rows past the end recompute row N-1
    const float c = a.scale * 1.44269504088896340736f;      // scores are kept in the log2 domain

    // allowed keys of this lane's query: [0, n_text) and [lo, hi]
    int lo, hi;
    if (it.window < 0 || i < n_text) { lo = 0; hi = N - 1; }
    else { lo = i - it.window; hi = i + it.window < N - 1 ? i + it.window : N - 1; }
    const unsigned span = (unsigned)(hi - lo);              // key j is in the band iff (unsigned)(j - lo) <= span

    // Q operand (B of S^T = K Q^T): column = query l32, k-slots 8*half..8*half+7 of each 16-wide step
    bf16x8 qf[KS];
    {
        const __bf16* qrow = qg + (int64_t)i * a.stride_n + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(qrow + 16 * ks);
    }

    floatx16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m = -1.0e30f;   // running maximum (log2 domain); finite so that exp2(-inf - m) is 0, not NaN
    float l = 0.f;        // running sum of this lane's half of the keys

    const int n_iter = it.kv0_end + (it.kv1_end - it.kv1_begin);
    bf16x8 kreg[LOADS], vreg[LOADS];

    auto tile_of = [&](int idx) { return idx < it.kv0_end ? idx : it.kv1_begin + (idx - it.kv0_end); };
    auto load_tile = [&](int t) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            const int ch = tid + 256 * u;
            const int r = ch / CPR, cc = ch - r * CPR;
            int j = t * kBN + r;
            j = j < N ? j : N - 1;                          // tail keys are masked later
            const int64_t off = (int64_t)j * a.stride_n + 8 * cc;
            kreg[u] = *(const bf16x8*)(kg + off);
            vreg[u] = *(const bf16x8*)(vg + off);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            const int ch = tid + 256 * u;
            const int r = ch / CPR, cc = ch - r * CPR;
            *(bf16x8*)&Ks[r * KSTR + 8 * cc] = kreg[u];
#pragma unroll
            for (int e = 0; e < 8; ++e) Vt[(8 * cc + e) * VSTR + r] = vreg[u][e];   // transpose
        }
    };

    if (n_iter > 0) {
        load_tile(tile_of(0));
        store_tile();
    }
    __syncthreads();

    for (int idx = 0; idx < n_iter; ++idx) {
        const int t = tile_of(idx);
        const bool more = idx + 1 < n_iter;
        if (more) load_tile(tile_of(idx + 1));              // global loads overlap the math below

        const bool masked = idx < it.kv0_end ? (t >= it.nm0_end) : (t < it.nm1_begin || t >= it.nm1_end);
        const int j0 = t * kBN;
        // A masked tile may hold no allowed pair for this wavefront's 32 rows: skip its math.
        bool active = true;
        if (masked && it.window >= 0) {
            const int r_first = row0 < N ? row0 : N - 1;
            const int r_last = row0 + 31 < N ? row0 + 31 : N - 1;
            const int j_last = (j0 + kBN < N ? j0 + kBN : N) - 1;
            active = (r_first < n_text) || (j0 < n_text) ||
                     (j0 <= r_last + it.window && j_last >= r_first - it.window);
        }

        if (active) {
            // ---- S^T = K Q^T : two 32-key blocks
            floatx16 s[2];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[jb][r] = 0.f;
                const __bf16* krow = &Ks[(32 * jb + l32) * KSTR + 8 * half];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 ka = *(const bf16x8*)(krow + 16 * ks);
                    s[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[ks], s[jb], 0, 0, 0);
                }
            }
            // register r of block jb holds key j0 + 32*jb + 8*(r/4) + 4*half + r%4
            if (masked) {
#pragma unroll
                for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int j = j0 + 32 * jb + 8 * (r >> 2) + 4 * half + (r & 3);
                        // branch-free on purpose: one unsigned range test per segment
                        const bool ok = ((unsigned)j < (unsigned)n_text) | ((unsigned)(j - lo) <= span);
                        s[jb][r] = ok ? s[jb][r] : -INFINITY;
                    }
            }
            // ---- online softmax (per-lane row statistics)
            float tmax = -INFINITY;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[jb][r]);
            tmax = fmaxf(tmax, xchg32(tmax));
            const float m_new = fmaxf(m, tmax * c);
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            bf16x8 pb[2][2];
            float psum = 0.f;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pf = __builtin_amdgcn_exp2f(fmaf(s[jb][r], c, -m_new));
                    const __bf16 pr = (__bf16)pf;           // the weight that enters P V ...
                    pb[jb][r >> 3][r & 7] = pr;
                    psum += (float)pr;                       // ... is also the one that is summed
                }
            l = l * alpha + psum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
            // ---- O^T += V^T P^T
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const __bf16* vrow = &Vt[(32 * db + l32) * VSTR + 4 * half];
#pragma unroll
                for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt) {
                        // k-slot e of this lane is key 32*jb + 16*tt + 4*half + (e<4 ? e : e+4)
                        const bf16x4 v0 = *(const bf16x4*)(vrow + 32 * jb + 16 * tt);
                        const bf16x4 v1 = *(const bf16x4*)(vrow + 32 * jb + 16 * tt + 8);
                        const bf16x8 va = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[jb][tt], o[db], 0, 0, 0);
                    }
            }
        }
        __syncthreads();                  // every wavefront is done reading this tile
        if (more) store_tile();
        __syncthreads();
    }

    // ---- epilogue: O^T register r of block db is feature d = 32*db + 8*(r/4) + 4*half + r%4
    const float l_tot = l + xchg32(l);
    const float inv = 1.0f / l_tot;
    if (i_raw < N) {
        __bf16* orow = og + (int64_t)i_raw * a.stride_n;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 w4;
#pragma unroll
                for (int e = 0; e < 4; ++e) w4[e] = (__bf16)(o[db][4 * g + e] * inv);
                *(bf16x4*)(orow + 32 * db + 8 * g + 4 * half) = w4;
            }
    }
}

hipError_t launch_attn_bf16(const AttnArgs& a, int head_dim, int n_items, hipStream_t stream) {
    if (n_items <= 0) return hipSuccess;
    if (head_dim == 128)
        hipLaunchKernelGGL(attn_bf16_kernel<128>, dim3(n_items), dim3(256), 0, stream, a);
    else if (head_dim == 64)
        hipLaunchKernelGGL(attn_bf16_kernel<64>, dim3(n_items), dim3(256), 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// fp32 debug path: one wavefront per query row, lanes stride over the allowed keys; the row is
// evaluated exactly as defined -- maximum, exponentials, sum, weighted mean -- with fp32 data,
// the accurate expf and fp32 value accumulation; only the score dot products run in fp64.  It shares only the work record's (batch, head, query tile) with the fast path.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_max(double x) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) x = fmax(x, __shfl_xor(x, s, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) x += __shfl_xor(x, s, 64);
    return x;
}

template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a) {
    const difa_work_item_t it = a.items[blockIdx.x];
    if (it.q_tile < 0) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int N = a.n_tokens, n_text = a.n_text;
    const int b = it.bh / a.heads, h = it.bh - b * a.heads;
    const int64_t base = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const float* __restrict__ qg = (const float*)a.q + base;
    const float* __restrict__ kg = (const float*)a.k + base;
    const float* __restrict__ vg = (const float*)a.v + base;
    float* __restrict__ og = (float*)a.out + base;

    for (int r = 0; r < 32; ++r) {
        const int i = it.q_tile * kBM + wave * 32 + r;
        if (i >= N) break;                                   // uniform over the wavefront
        // allowed keys: [0, seg0_end) and [lo, hi]
        int seg0_end, lo, hi;
        if (it.window < 0 || i < n_text) { seg0_end = 0; lo = 0; hi = N - 1; }
        else {
            seg0_end = n_text;
            lo = i - it.window > n_text ? i - it.window : n_text;
            hi = i + it.window < N - 1 ? i + it.window : N - 1;
        }
        float qv[D];
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const floatx4 t4 = *(const floatx4*)(qg + (int64_t)i * a.stride_n + d);
            qv[d] = t4[0]; qv[d + 1] = t4[1]; qv[d + 2] = t4[2]; qv[d + 3] = t4[3];
        }
        // Scores are accumulated in fp64: with logits of magnitude ~10 an fp32 dot product alone
        // costs a few 1e-6 in every weight, which is the whole error budget of this path.
        auto score = [&](int j) {
            const float* kr = kg + (int64_t)j * a.stride_n;
            double s = 0.0;
#pragma unroll
            for (int d = 0; d < D; d += 4) {
                const floatx4 t4 = *(const floatx4*)(kr + d);
                s = fma((double)qv[d], (double)t4[0], s); s = fma((double)qv[d + 1], (double)t4[1], s);
                s = fma((double)qv[d + 2], (double)t4[2], s); s = fma((double)qv[d + 3], (double)t4[3], s);
            }
            return s * (double)a.scale;
        };
        // pass 1: row maximum
        double m = -INFINITY;
        for (int j = lane; j < seg0_end; j += 64) m = fmax(m, score(j));
        for (int j = lo + lane; j <= hi; j += 64) m = fmax(m, score(j));
        m = wave_max(m);
        // pass 2: weights, their sum, and the weighted sum of value rows
        float acc[D];
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] = 0.f;
        float l = 0.f;
        auto accumulate = [&](int j) {
            const float p = expf((float)(score(j) - m));
            l += p;
            const float* vr = vg + (int64_t)j * a.stride_n;
#pragma unroll
            for (int d = 0; d < D; d += 4) {
                const floatx4 t4 = *(const floatx4*)(vr + d);
                acc[d] = fmaf(p, t4[0], acc[d]); acc[d + 1] = fmaf(p, t4[1], acc[d + 1]);
                acc[d + 2] = fmaf(p, t4[2], acc[d + 2]); acc[d + 3] = fmaf(p, t4[3], acc[d + 3]);
            }
        };
        for (int j = lane; j < seg0_end; j += 64) accumulate(j);
        for (int j = lo + lane; j <= hi; j += 64) accumulate(j);
        l = wave_sum(l);
        float mine = 0.f;                                    // lane d%64 keeps feature d
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const float tot = wave_sum(acc[d]);
            if ((d & 63) == lane) mine = tot / l;
            if ((d & 63) == 63) og[(int64_t)i * a.stride_n + (d - 63) + lane] = mine;
        }
    }
}

hipError_t launch_attn_f32(const AttnArgs& a, int head_dim, int n_items, hipStream_t stream) {
    if (n_items <= 0) return hipSuccess;
    if (head_dim == 128)
        hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(n_items), dim3(256), 0, stream, a);
    else if (head_dim == 64)
        hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(n_items), dim3(256), 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Cached heads: a 16-byte-per-lane copy of the head's rows, four vectors in flight per thread.
// HBM bound: 2 * N * D * elem bytes per (batch entry, cached head).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cache_copy_kernel(CopyArgs c) {
    const int64_t per_head = (int64_t)c.n_tokens * c.vec_per_row;
    const int64_t total = per_head * c.n_copy * c.batch;
    const int64_t stride = (int64_t)gridDim.x * 256;
    const char* __restrict__ src = (const char*)c.src;
    char* __restrict__ dst = (char*)c.dst;
    auto offset_of = [&](int64_t idx) {
        const int64_t hh = idx / per_head, rem = idx - hh * per_head;
        const int bb = (int)(hh / c.n_copy), ch = (int)(hh - (int64_t)bb * c.n_copy);
        const int head = c.copy_heads[ch];
        const int64_t n = rem / c.vec_per_row, vc = rem - n * c.vec_per_row;
        return (int64_t)bb * c.stride_b + (int64_t)head * c.stride_h + n * c.stride_n + vc * 16;
    };
    int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; idx + 3 * stride < total; idx += 4 * stride) {
        const int64_t o0 = offset_of(idx), o1 = offset_of(idx + stride);
        const int64_t o2 = offset_of(idx + 2 * stride), o3 = offset_of(idx + 3 * stride);
        const uint4 v0 = *(const uint4*)(src + o0);
        const uint4 v1 = *(const uint4*)(src + o1);
        const uint4 v2 = *(const uint4*)(src + o2);
        const uint4 v3 = *(const uint4*)(src + o3);
        *(uint4*)(dst + o0) = v0;
        *(uint4*)(dst + o1) = v1;
        *(uint4*)(dst + o2) = v2;
        *(uint4*)(dst + o3) = v3;
    }
    for (; idx < total; idx += stride) {
        const int64_t o0 = offset_of(idx);
        *(uint4*)(dst + o0) = *(const uint4*)(src + o0);
    }
}

hipError_t launch_cache_copy(const CopyArgs& c, hipStream_t stream) {
    const int64_t total = (int64_t)c.n_tokens * c.vec_per_row * c.n_copy * c.batch;
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 256 * 4 - 1) / (256 * 4);
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(cache_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, c);
    return hipGetLastError();
}

}  // namespace difa
