// gfx950 kernels of the head-wise joint-attention operator (Sec. 3.3 of the paper):
//   attn_bf16_kernel  -- full / arrow heads, bf16 MFMA with fp32 accumulation
//   attn_f32_kernel   -- the same result in plain fp32 arithmetic (slow debug path)
//   cache_copy_kernel -- cached heads: out[b,h] = cache[b,h] (Alg. 1, last statement)
#include <type_traits>

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
// One workgroup = 4 wavefronts (one per SIMD) = one 256-row query tile of one (batch, head);
// wavefront w owns rows 64w..64w+63 as two 32-row blocks.  Key/value tiles of 64 keys go through
// a 3-stage LDS ring and are visited in the order the host-compiled work record lists them
// (text tiles, then the band tiles), so a tile with no allowed pair is never loaded
// (Sec. 3.1 / 3.3: block-sparse band).
//
// Why 64 rows per wavefront: LDS delivers 128 B/clk/CU, i.e. one 16-byte-per-lane operand read
// per MFMA issue slot of the CU.  With 32 rows per wavefront every MFMA needs a fresh K or V
// operand from LDS and the LDS port, not the matrix core, sets the pace; with 64 rows each
// operand read feeds two MFMAs.
//
// Scores are produced transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then holds
// 16 keys of ONE query (column = lane % 32), so the softmax row statistics are per-lane scalars
// and need one exchange between the wavefront halves.  The same register layout is exactly the
// B operand of O^T = V^T P^T, so P never goes through LDS.  V stays row-major [key][feature] in
// LDS and its transposed operand comes from ds_read_b64_tr_b16.
//
// Software pipeline inside a wavefront: S^T of tile t+1 (MFMA) is issued in the same basic block
// as the softmax of tile t (VALU), so the two pipes overlap without a second wavefront.
// ------------------------------------------------------------------------------------------
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// LDS transpose read: within each group of 16 lanes, lane i receives element (i % 4) of the four
// 8-byte rows that lanes (i/4), 4+(i/4), 8+(i/4), 12+(i/4) of the group point at.
__device__ __forceinline__ bf16x4 lds_read_tr16(const __bf16* p) {
    const shortx4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (shortx4 __attribute__((address_space(3)))*)(p));
    return __builtin_bit_cast(bf16x4, r);
}

struct RowState {
    float m;       // reference maximum (log2 domain) the weights are expressed against
    float l;       // running sum of this lane's half of the keys
    int lo;        // band of allowed image keys is [lo, lo + span]; text keys [0, n_text) always allowed
    unsigned span;
};

template <int D>
__global__ __launch_bounds__(256, 1) void attn_bf16_kernel(AttnArgs a) {
    constexpr int KS = D / 16;              // MFMA k-steps of S^T = K Q^T
    constexpr int DB = D / 32;              // 32-row blocks of O^T
    constexpr int CPR = D / 8;              // 16-byte chunks per K/V row
    constexpr int LOADS = kBN * CPR / 256;  // 16-byte loads per thread per tensor per tile
    constexpr int TILE = kBN * D;           // elements of one K or V tile
    constexpr int NSK = 3;                  // LDS ring depth for K tiles
    constexpr int NSV = 4;                  // ... and for V tiles (P V trails S^T by one more block)
    constexpr float kBump = 8.0f;           // the reference maximum moves only when exceeded by 2^8

    // K rows: 16-byte chunk c of row r is stored at chunk c ^ (r % CPR)       (conflict-free b128 reads)
    // V rows: chunk c of row r is stored at chunk c ^ (2 * (r % 4))          (conflict-free transpose reads)
    __shared__ __attribute__((aligned(16))) __bf16 Ksm[NSK * TILE];
    __shared__ __attribute__((aligned(16))) __bf16 Vsm[NSV * TILE];

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

    const int row0 = it.q_tile * kBM + wave * 64;           // first query row of this wavefront
    const float c = a.scale * 1.44269504088896340736f;      // scores are kept in the log2 domain

    // ---- per-lane query rows (two: one per 32-row block), their allowed key ranges, Q operands
    RowState rs[2];
    bf16x8 qf[2][KS];
    int i_raw[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        i_raw[qb] = row0 + 32 * qb + l32;
        const int i = i_raw[qb] < N ? i_raw[qb] : N - 1;    // rows past the end recompute row N-1
        int lo, hi;
        if (it.window < 0 || i < n_text) { lo = 0; hi = N - 1; }
        else { lo = i - it.window; hi = i + it.window < N - 1 ? i + it.window : N - 1; }
        rs[qb].lo = lo;
        rs[qb].span = (unsigned)(hi - lo);                  // key j is in the band iff (unsigned)(j-lo) <= span
        rs[qb].m = -1.0e30f;                                // finite: exp2(-inf - m) must be 0, not NaN
        rs[qb].l = 0.f;
        // B operand of S^T = K Q^T: column = query l32, k-slots 8*half..8*half+7 of each 16-wide step
        const __bf16* qrow = qg + (int64_t)i * a.stride_n + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *(const bf16x8*)(qrow + 16 * ks);
    }

    // ---- per-lane LDS offsets (elements, within one stage)
    int koff[KS];                                           // A operand of S^T: row l32, chunk 2*ks+half
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = l32 * D + 8 * ((2 * ks + half) ^ (l32 & (CPR - 1)));
    int voff[DB];                                           // transpose read: row 4*half + s/4, 4 features
    {
        const int blk = lane >> 4, s16 = lane & 15;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * (blk & 1) + ((s16 & 3) >> 1);
            voff[db] = (4 * half + (s16 >> 2)) * D + 8 * (chunk ^ (2 * (s16 >> 2))) + 4 * (s16 & 1);
        }
    }

    floatx16 o[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;

    const int n_iter = it.kv0_end + (it.kv1_end - it.kv1_begin);
    auto tile_of = [&](int idx) {
        idx = idx < n_iter ? idx : n_iter - 1;              // past the end: reload the last tile (unused)
        return idx < it.kv0_end ? idx : it.kv1_begin + (idx - it.kv0_end);
    };
    auto tile_masked = [&](int idx) {
        const int t = tile_of(idx);
        return idx < it.kv0_end ? (t >= it.nm0_end) : (t < it.nm1_begin || t >= it.nm1_end);
    };
    // ---- global -> registers -> LDS staging of one K/V tile.  Buffer loads: one descriptor per
    // tensor for this (batch, head), a per-thread byte offset that is constant over the loop plus the
    // tile's byte offset; rows past the last token read as zero (they are masked later).
    const unsigned head_bytes = (unsigned)(((int64_t)(N - 1) * a.stride_n + D) * 2);
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kg, 0, head_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)vg, 0, head_bytes, 0x00020000);
    unsigned goff[LOADS];
#pragma unroll
    for (int u = 0; u < LOADS; ++u) {
        const int ch = tid + 256 * u;
        const int r = ch / CPR, cc = ch - r * CPR;
        goff[u] = (unsigned)(r * (int)a.stride_n + 8 * cc) * 2u;
    }
    const unsigned tile_bytes = (unsigned)(kBN * (int)a.stride_n) * 2u;
    uintx4 kreg[LOADS], vreg[LOADS];
    auto load_tile = [&](int t) {
        const unsigned tb = (unsigned)t * tile_bytes;
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            kreg[u] = __builtin_amdgcn_raw_buffer_load_b128(krsrc, goff[u] + tb, 0, 0);
            vreg[u] = __builtin_amdgcn_raw_buffer_load_b128(vrsrc, goff[u] + tb, 0, 0);
        }
    };
    auto store_tile = [&](int idx) {
        const int ks = idx % NSK, vs = idx % NSV;
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            const int ch = tid + 256 * u;
            const int r = ch / CPR, cc = ch - r * CPR;
            *(uintx4*)&Ksm[ks * TILE + r * D + 8 * (cc ^ (r & (CPR - 1)))] = kreg[u];
            *(uintx4*)&Vsm[vs * TILE + r * D + 8 * (cc ^ (2 * (r & 3)))] = vreg[u];
        }
    };

    // ---- S^T = K Q^T for one 32-key block jb of a tile: s[qb], register r = key 32*jb + 8*(r/4) + 4*half + r%4
    auto qk_block = [&](int idx, int jb, floatx16 (&s)[2]) {
        const __bf16* kst = &Ksm[(idx % NSK) * TILE + 32 * jb * D];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[qb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ka = *(const bf16x8*)(kst + koff[ks]);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
                s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[qb][ks], s[qb], 0, 0, 0);
        }
    };
    auto mask_block = [&](int j0, floatx16 (&s)[2]) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j0 + 8 * (r >> 2) + 4 * half + (r & 3);
                // branch-free on purpose: one unsigned range test per segment
                const bool ok = ((unsigned)j < (unsigned)n_text) | ((unsigned)(j - rs[qb].lo) <= rs[qb].span);
                s[qb][r] = ok ? s[qb][r] : -INFINITY;
            }
    };
    // ---- softmax of one 32-key block, split in three pieces so that they can be laid between MFMAs.
    //   sm_read : copy 8 scores of the block out of the accumulation registers, fold them into the
    //             running block maximum
    //   sm_stats: finish the block maximum across the two wavefront halves, move the reference
    //             maximum if needed, produce the rescale factors
    //   sm_exp  : weights of `cnt` consecutive score pairs as bf16 B operands + their sum
    // The online-softmax state advances once per block.
    auto sm_read = [&](const floatx16 (&s)[2], float (&sv)[2][16], float (&tmax)[2], int part) {
        const int qb = part >> 1, r0 = (part & 1) * 8;
#pragma unroll
        for (int r = 0; r < 8; ++r) sv[qb][r0 + r] = s[qb][r0 + r];
#pragma unroll
        for (int r = 0; r < 8; r += 2) tmax[qb] = fmaxf(tmax[qb], fmaxf(sv[qb][r0 + r], sv[qb][r0 + r + 1]));
    };
    auto sm_stats = [&](float (&tmax)[2], float (&mneg)[2], float (&alpha)[2]) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float t = fmaxf(tmax[qb], xchg32(tmax[qb])) * c;
            // The reference maximum only moves when it is exceeded by more than 2^kBump: weights
            // stay <= 2^kBump (harmless in fp32 / bf16) and O is rescaled rarely.
            const float m_old = rs[qb].m;
            const float m_new = t > m_old + kBump ? t : m_old;
            alpha[qb] = __builtin_amdgcn_exp2f(m_old - m_new);
            rs[qb].m = m_new;
            rs[qb].l *= alpha[qb];
            mneg[qb] = -m_new;
        }
    };
    auto sm_exp = [&](const float (&sv)[2][16], const float (&mneg)[2], bf16x8 (&pw)[2][2], int first_pair, int cnt) {
        bf16x2 ones;
        ones[0] = (__bf16)1.0f;
        ones[1] = (__bf16)1.0f;
#pragma unroll
        for (int pi = first_pair; pi < first_pair + cnt; ++pi) {   // pair pi: row block qb = pi/8, scores 2*(pi%8), +1
            const int qb = pi >> 3, r = 2 * (pi & 7);
            floatx2 pf;
            pf[0] = __builtin_amdgcn_exp2f(fmaf(sv[qb][r], c, mneg[qb]));
            pf[1] = __builtin_amdgcn_exp2f(fmaf(sv[qb][r + 1], c, mneg[qb]));
            bf16x2 pr = __builtin_convertvector(pf, bf16x2);             // the weights that enter P V ...
            {   // keep the computation in this slot: without the pin it is sunk to the block that uses it
                unsigned bits = __builtin_bit_cast(unsigned, pr);
                asm volatile("" : "+v"(bits));
                pr = __builtin_bit_cast(bf16x2, bits);
            }
            pw[qb][r >> 3][r & 7] = pr[0];
            pw[qb][r >> 3][(r & 7) + 1] = pr[1];
            rs[qb].l = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs[qb].l, false);   // ... are the ones summed
        }
    };
    auto rescale = [&](const float (&alpha)[2]) {
        // Uniform over the wavefront and rare: taken only when some row moved its reference maximum.
        // The accumulators live in accumulation registers; they are scaled in place there so that the
        // hot path never has to move them.  The waits cover MFMA results still in flight.
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(alpha[0] != 1.0f || alpha[1] != 1.0f) != 0, 0)) {
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float e = o[db][qb][r], t;
                        asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                                     : "+a"(e), "=&v"(t) : "v"(alpha[qb]));
                        o[db][qb][r] = e;
                    }
            asm volatile("s_nop 7" ::: "memory");
        }
    };
    // ---- O^T += V^T P^T: k-slot e of a lane is key 32*jb + 16*tt + 4*half + (e<4 ? e : e+4)
    // ---- operand fetches from LDS
    auto k_operand = [&](const __bf16* kst, int ks) { return *(const bf16x8*)(kst + koff[ks]); };
    auto v_operand = [&](const __bf16* vst, int i) {          // operand i = 2*db + tt
        const __bf16* vp = vst + 16 * (i & 1) * D + voff[i >> 1];
        const bf16x4 v0 = lds_read_tr16(vp);
        const bf16x4 v1 = lds_read_tr16(vp + 8 * D);
        return (bf16x8)__builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto k_block_ptr = [&](int idx, int jb) { return &Ksm[(idx % NSK) * TILE + 32 * jb * D]; };
    auto v_block_ptr = [&](int idx, int jb) { return &Vsm[(idx % NSV) * TILE + 32 * jb * D]; };

    // ---- prologue: tiles 0 and 1 into the ring, S^T of block (tile 0, jb 0)
    load_tile(tile_of(0));
    store_tile(0);
    load_tile(tile_of(1));
    store_tile(1);
    __syncthreads();

    // The pipeline advances by 32-key blocks g = 2*tile + jb.  One half-step for block g is
    //   part 1:  P V of block g-1 (16 MFMA)  next to  the maximum / statistics of block g (VALU)
    //   side  :  rescale of O if some row moved its reference maximum (rare)
    //   part 2:  S^T of block g+1 (16 MFMA)  next to  the exponentials of block g (VALU)
    //   side  :  element mask of the scores of block g+1 (edge tiles only)
    // Every part is cut into 8 slots of 2 MFMAs that share one LDS operand; operands are fetched
    // four slots ahead, and the slots are fenced so that the order written here is the order issued.
    // K tiles live in a 3-deep ring, V tiles in a 4-deep ring because P V of a tile's second block
    // runs one iteration after its S^T.  In the last iteration block g+1 is a reload of the last
    // tile whose scores are never used.
    constexpr int NOP = D / 16;             // LDS operands (= MFMA pairs) per part: 8 at D=128, 4 at D=64
    constexpr int AHEAD = 4;                // operands fetched this many slots ahead
    floatx16 s0[2], s1[2];                  // scores of the even / odd block in flight
    bf16x8 pa[2][2], pb[2][2];              // weights of the even / odd block in flight
    bf16x8 kq[NOP], vq[NOP];                // LDS operands in flight (slot i uses entry i)

    auto half_step = [&](floatx16 (&s_cur)[2], floatx16 (&s_nxt)[2], const bf16x8 (&p_prev)[2][2],
                         bf16x8 (&p_cur)[2][2], const __bf16* kst_nxt, const __bf16* vst_prev,
                         const __bf16* vst_cur, bool with_pv, bool mask_nxt,
                         int j0_nxt) __attribute__((always_inline)) {
        float sv[2][16], tmax[2] = {-INFINITY, -INFINITY}, mneg[2], alpha[2];
        // ---- part 1 (vq[0..AHEAD) were fetched by the previous half-step)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (with_pv && i < NOP) {
                if (i + AHEAD < NOP) vq[i + AHEAD] = v_operand(vst_prev, i + AHEAD);
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
                    o[i >> 1][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[i], p_prev[qb][i & 1], o[i >> 1][qb], 0, 0, 0);
            }
            if (i >= 8 - AHEAD) kq[i - (8 - AHEAD)] = k_operand(kst_nxt, i - (8 - AHEAD));
            if (i < 4) sm_read(s_cur, sv, tmax, i);
            if (i == 4) sm_stats(tmax, mneg, alpha);
            if (i == 6) sm_exp(sv, mneg, p_cur, 0, 2);
            if (i == 7) sm_exp(sv, mneg, p_cur, 2, 2);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (with_pv) rescale(alpha);
        // ---- part 2
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s_nxt[qb][r] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i < NOP) {
                if (i + AHEAD < NOP) kq[i + AHEAD] = k_operand(kst_nxt, i + AHEAD);
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
                    s_nxt[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kq[i], qf[qb][i], s_nxt[qb], 0, 0, 0);
            }
            if (i >= 8 - AHEAD) vq[i - (8 - AHEAD)] = v_operand(vst_cur, i - (8 - AHEAD));
            if (i < 4) sm_exp(sv, mneg, p_cur, 4 + 2 * i, 2); else sm_exp(sv, mneg, p_cur, 8 + i, 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (__builtin_expect(mask_nxt, 0)) mask_block(j0_nxt, s_nxt);
    };
    static_assert(NOP == 8 || NOP == 4, "slot layout assumes head_dim 128 or 64");
    static_assert(AHEAD <= NOP, "operands are fetched at most one part ahead");

    qk_block(0, 0, s0);
    if (tile_masked(0)) mask_block(tile_of(0) * kBN, s0);

    // first tile: its even block has no predecessor whose P V would be due
    load_tile(tile_of(2));
    half_step(s0, s1, pb, pa, k_block_ptr(0, 1), v_block_ptr(0, 0), v_block_ptr(0, 0), false,
              tile_masked(0), tile_of(0) * kBN + 32);
    half_step(s1, s0, pa, pb, k_block_ptr(1, 0), v_block_ptr(0, 0), v_block_ptr(0, 1), true,
              tile_masked(1), tile_of(1) * kBN);
    store_tile(2);

    for (int idx = 1; idx < n_iter; ++idx) {
        __syncthreads();    // tile idx+1 is in LDS for everyone; the stages of tile idx+2 are no longer read
        load_tile(tile_of(idx + 2));
        half_step(s0, s1, pb, pa, k_block_ptr(idx, 1), v_block_ptr(idx - 1, 1), v_block_ptr(idx, 0), true,
                  tile_masked(idx), tile_of(idx) * kBN + 32);
        half_step(s1, s0, pa, pb, k_block_ptr(idx + 1, 0), v_block_ptr(idx, 0), v_block_ptr(idx, 1), true,
                  tile_masked(idx + 1), tile_of(idx + 1) * kBN);
        store_tile(idx + 2);
    }
    // P V of the very last block (its operands 0..AHEAD-1 are already in flight)
    {
        const __bf16* vst = v_block_ptr(n_iter - 1, 1);
#pragma unroll
        for (int i = 0; i < NOP; ++i) {
            if (i + AHEAD < NOP) vq[i + AHEAD] = v_operand(vst, i + AHEAD);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
                o[i >> 1][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[i], pb[qb][i & 1], o[i >> 1][qb], 0, 0, 0);
        }
    }

    // ---- epilogue: O^T register r of block db is feature d = 32*db + 8*(r/4) + 4*half + r%4
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l_tot = rs[qb].l + xchg32(rs[qb].l);
        const float inv = 1.0f / l_tot;
        if (i_raw[qb] < N) {
            __bf16* orow = og + (int64_t)i_raw[qb] * a.stride_n;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 w4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w4[e] = (__bf16)(o[db][qb][4 * g + e] * inv);
                    *(bf16x4*)(orow + 32 * db + 8 * g + 4 * half) = w4;
                }
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

    for (int r = 0; r < kBM / 4; ++r) {
        const int i = it.q_tile * kBM + wave * (kBM / 4) + r;
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
