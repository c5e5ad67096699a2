// gfx950 kernels of the head-wise joint-attention operator (Sec. 3.3 of the paper):
//   attn_bf16_kernel  -- the whole layer in one launch: full / arrow heads with bf16 MFMA and fp32
//                        accumulation, then the cached heads, out[b,h] = cache[b,h] (the cache fill that
//                        ends Alg. 1), copied by whichever workgroups have finished their attention work
//   attn_f32_kernel   -- full / arrow heads in plain fp32 arithmetic (slow debug path)
//   cache_copy_kernel -- cached heads of the debug path, and of a bf16 layer with every head cached
#include <mutex>
#include <type_traits>

#include "difa_internal.h"

namespace difa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Maximum / sum of a value over the two halves of a wavefront (lanes l and l^32).
// v_permlane32_swap is a VALU instruction: unlike ds_bpermute it does not queue behind the LDS
// reads in flight.  With both operands equal it returns {low half, low half} and {high half, high half}.
__device__ __forceinline__ float halves_max(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned lo = r[0], hi = r[1];    // copied to scalars first: a bit_cast applied directly to a vector element reads element 0
    return fmaxf(__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi));
}
__device__ __forceinline__ float halves_sum(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned lo = r[0], hi = r[1];
    return __builtin_bit_cast(float, lo) + __builtin_bit_cast(float, hi);
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA attention.
//
// A workgroup is 8 / QB wavefronts (QB = 32-row blocks per wavefront; 1 in the shipped build, so eight
// wavefronts, two per SIMD) and stays resident: it walks the list of segments the host scheduler gave
// it.  A segment is a 256-row query tile of one (batch, head) together with a
// run of that record's key/value tiles (the whole run for most records; a few records are cut so
// that every workgroup ends at the same time, and their pieces leave fp32 partial results that the
// piece finishing last folds into its own).  Wavefront w owns rows 32*QB*w .. 32*QB*(w+1)-1 as QB 32-row blocks.
// Key/value tiles of 64 keys are written into 4-stage LDS rings by the buffer-load-to-LDS DMA, K three
// tiles and V two tiles ahead of their use, in the order the work record lists them (text tiles,
// then the band tiles), so a tile with no allowed pair is never loaded (Sec. 3.1 / 3.3:
// block-sparse band).  The first tiles and the Q rows of the next segment are requested before
// the current segment's epilogue.
//
// Rows per wavefront: with 64 rows (QB = 2) every 16-byte-per-lane LDS operand read feeds two MFMAs,
// but the whole register file goes to one wavefront per SIMD, and a single wavefront does not overlap
// its own vector arithmetic with its own MFMAs: measured, the clocks of the two simply add.  With 32
// rows (QB = 1) a wavefront fits in half the register file, two share a SIMD, and one's softmax runs
// under the other's MFMAs; LDS (twice the operand reads) is busy about a third of the time.
//
// Scores are produced transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then holds
// 16 keys of ONE query (column = lane % 32), so the softmax row statistics are per-lane scalars
// and need one exchange between the wavefront halves.  The same register layout is exactly the
// B operand of O^T = V^T P^T, so P never goes through LDS.  V stays row-major [key][feature] in
// LDS and its transposed operand comes from ds_read_b64_tr_b16.
//
// Software pipeline inside a wavefront: a wavefront issues in order, so the loop body is laid
// out by hand as 8 * QB slots per 32-key half-step, each slot one MFMA (S^T of the next block, or
// P V of the previous one) followed by the few vector instructions of the softmax of the block
// in between, an LDS operand read or a DMA request; the vector work runs while the matrix core
// is busy with the slot's MFMA.
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

// S^T = K Q^T MFMAs are written as assembly so that the register classes are fixed: the scores
// accumulate in ordinary vector registers, where the softmax arithmetic reads them directly (the
// compiler's own choice for a kernel this size is accumulation registers plus one copy per score),
// and the Q operand sits in accumulation registers, which only matrix instructions read.
// The hardware does not interlock a vector instruction that reads a matrix result too early and the
// compiler does not see through the assembly, so every reader is either a full half-step away or
// preceded by an explicit wait (mfma_results_visible).
__device__ __forceinline__ void mfma_s_first(floatx16& d, const bf16x8& k, const bf16x8& q) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_s_acc(floatx16& d, const bf16x8& k, const bf16x8& q) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_results_visible() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }
// (the same wait, tied to the registers it is for: no read of them can be moved ahead of it)
__device__ __forceinline__ void mfma_results_visible(floatx16& d) { asm volatile("s_nop 15\n\ts_nop 15" : "+v"(d) :: "memory"); }

// Cache-policy operand of the buffer load/store builtins: device scope ("sc1").
constexpr int kDeviceCoherent = 16;
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

struct RowState {
    float m;       // reference maximum (log2 domain) the weights are expressed against
    float l;       // running sum of this lane's half of the keys
    int lo;        // band of allowed image keys is [lo, lo + span]; text keys are always allowed
    unsigned span;
};

template <int D, int QB>
__global__ __launch_bounds__(512 / QB, 1) void attn_bf16_kernel(AttnArgs a) {
    constexpr int NW = 8 / QB;              // wavefronts per workgroup; each owns 32*QB query rows
    constexpr int RW = 32 * QB;
    constexpr int KS = D / 16;              // MFMA k-steps of S^T = K Q^T
    constexpr int DB = D / 32;              // 32-row blocks of O^T
    constexpr int CPR = D / 8;              // 16-byte chunks per K/V row
    constexpr int TILE = kBN * D;           // elements of one K or V tile
    constexpr int NS = 4;                   // LDS ring depth, K and V alike: tile p lives in stage p % 4
    constexpr float kTrip = 0x1p40f;        // a block row sum beyond this sends the wavefront to the renormalising side path
    constexpr float kBump = 16.0f;          // ... where a row's reference moves if its block maximum exceeds it by 2^16

    // LDS moves 256 bytes per clock over 64 banks of 4 bytes: a b128 read is served 16 lanes at a time
    // (16 consecutive key rows, one 16-byte chunk each), a transpose read 32 lanes at a time (4 key rows
    // x 8 pieces of 8 bytes out of one group of 4 chunks).  A 256-byte row (D = 128) covers every bank
    // once, a 128-byte row (D = 64) half of them, alternating with the row's parity.  The 16-byte chunk c
    // of row r is therefore stored at chunk c ^ kswz(r) (K) or c ^ vswz(r) (V), chosen so that the
    // lanes served together land in different banks:
    //   K: 16 rows x 1 chunk:  D = 128: r % 16;        D = 64: (r / 2) % 8 (rows of one parity share banks)
    //   V: 4 rows x 4 chunks:  D = 128: 4 * (r % 4);   D = 64: 2 * (r % 4) (the group moves for r % 4 >= 2, the parity does the rest)
    auto kswz = [](int r) { return CPR == 16 ? (r & 15) : ((r >> 1) & 7); };
    auto vswz = [](int r) { return CPR == 16 ? 4 * (r & 3) : 2 * (r & 3); };
    __shared__ __attribute__((aligned(16))) __bf16 Ksm[NS * TILE];
    __shared__ __attribute__((aligned(16))) __bf16 Vsm[NS * TILE];
    __shared__ int ctl_sm[4];                // [0]: a ticket, handed from thread 0 to the workgroup; [2..3]: thread 0's start time
    // The arguments that only the rare paths use (merging a cut record, the cached-head copy) are read
    // from the kernel-argument block where they are needed: named through `a` they would be fetched at
    // kernel entry and held in scalar registers for the whole key loop, which has none to spare.
    auto cold_args = []() __attribute__((always_inline)) {
        unsigned long long kp = (unsigned long long)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(kp));
        return (const AttnArgs*)kp;
    };

    const int tid = threadIdx.x, wave = tid >> 6;
    // How long the workgroup runs is reported to the host, which learns from it how fast each accelerator
    // die is going (their clocks differ by a few percent under load) and shares out later work accordingly.
    // The start time waits in LDS (ctl_sm[2..3]): no register is held for it across the kernel.
    int l32, half;                                          // lane % 32, lane / 32 (set by lane_offsets below)
    const int N = a.n_tokens, n_text = a.n_text;
    // text tokens are [text_begin, text_begin + n_text), image tokens [img0, img1) (the text block sits
    // before or after the image block); a record's key-tile position u is tile (u + tile_rot) % n_kv_tiles
    const int text_begin = a.text_begin;
    const int img0 = text_begin == 0 ? n_text : 0, img1 = text_begin == 0 ? N : text_begin;
    auto tile_at = [&](int u) { const int t = u + a.tile_rot; return t >= a.n_kv_tiles ? t - a.n_kv_tiles : t; };
    const float c = a.scale * 1.44269504088896340736f;      // scores are kept in the log2 domain

    // ---- per-lane offsets: LDS operand reads (elements, within one stage) and the lane's place in a tile load
    int koff[KS];                                           // A operand of S^T: row l32, chunk 2*ks+half
    int voff[DB];                                           // transpose read: row 4*half + s/4, 4 features

    // ---- global -> LDS: K/V tiles are written into the ring by the load itself
    // (buffer_load_dwordx4 ... lds: lane l of a wavefront deposits its 16 bytes at M0 + 16*l), so a
    // tile never occupies registers and needs no ds_write.  One instruction fills RPI consecutive
    // tile rows; the XOR swizzle of the LDS layout is applied by permuting which 16-byte chunk of the
    // row each lane fetches.  One buffer descriptor per tensor for the segment's (batch, head): rows
    // past the last token read as zero (they are masked later).  The loads are outside the compiler's
    // view, so the wait for them is explicit (dma_wait) and sits just before the barrier that
    // publishes the tile.
    constexpr int RPI = 64 / CPR;                           // tile rows per load instruction
    constexpr int NDMA = kBN / RPI / NW;                     // load instructions per wavefront, tensor and tile
    const unsigned head_bytes = (unsigned)(((int64_t)(N - 1) * a.stride_n + D) * 2);
    uintx4 krsrc, vrsrc;                                    // descriptors of the head whose tiles are being loaded
    const unsigned wave_u = __builtin_amdgcn_readfirstlane(wave);
    unsigned gk[NDMA], gv[NDMA];                            // per-lane byte offsets inside a tile
    // These sixteen-odd registers are derived from the lane number again at the start of every segment,
    // through a copy the compiler cannot see through.  Held for the whole kernel instead, they would be
    // live across the rare, register-hungry paths between segments (merging a cut record, the cached-head
    // copy), and the register allocator would answer by parking some of them in accumulation registers
    // and fetching them back inside the key loop.
    auto lane_offsets = [&]() __attribute__((always_inline)) {
        int lane = tid & 63;
        asm volatile("" : "+v"(lane));
        l32 = lane & 31;
        half = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) koff[ks] = l32 * D + 8 * ((2 * ks + half) ^ kswz(l32));
        const int blk = lane >> 4, s16 = lane & 15;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int chunk = 4 * db + 2 * (blk & 1) + ((s16 & 3) >> 1);
            voff[db] = (4 * half + (s16 >> 2)) * D + 8 * (chunk ^ vswz(s16 >> 2)) + 4 * (s16 & 1);
        }
#pragma unroll
        for (int u = 0; u < NDMA; ++u) {
            const int r = (wave * NDMA + u) * RPI + lane / CPR, pc = lane % CPR;   // tile row, chunk slot in LDS
            gk[u] = (unsigned)(r * (int)a.stride_n + 8 * (pc ^ kswz(r))) * 2u;
            gv[u] = (unsigned)(r * (int)a.stride_n + 8 * (pc ^ vswz(r))) * 2u;
        }
    };
    const unsigned tile_bytes = (unsigned)(kBN * (int)a.stride_n) * 2u;
    const unsigned k_lds = (unsigned)(unsigned long long)(__attribute__((address_space(3))) __bf16*)Ksm;
    const unsigned v_lds = (unsigned)(unsigned long long)(__attribute__((address_space(3))) __bf16*)Vsm;
    // One load instruction: part u (0..NDMA-1) of a K (tensor 0) or V (tensor 1) tile.  `tb` is the tile's
    // byte offset inside the head, or an offset beyond the buffer for positions past the end of the
    // segment (those fetch nothing and deposit zeros); `dst` is this wavefront's LDS byte address inside
    // the ring stage.  All per-tile scalars are computed once per iteration by the caller.
    auto dma_part = [&](int tensor, int u, unsigned tb, unsigned dst) __attribute__((always_inline)) {
        if (tensor == 0)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :: "s"(dst + (unsigned)(u * RPI * D * 2)), "v"(gk[u] + tb), "s"(krsrc) : "m0");
        else
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                         :: "s"(dst + (unsigned)(u * RPI * D * 2)), "v"(gv[u] + tb), "s"(vrsrc) : "m0");
    };
    const unsigned wave_lds = wave_u * (unsigned)(NDMA * RPI * D * 2);     // this wavefront's rows inside a stage
    // all loads done / all but the 2*NDMA youngest (= the tiles issued during the current iteration) done
    auto dma_wait_all = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    auto dma_wait_older = [] { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * NDMA) : "memory"); };

    // What a segment needs before its first block: its K tiles 0..2 and V tiles 0, 1 in the ring (the
    // segment's tile p goes to stage (sb + p) % 4) and its query rows in the Q operand registers.
    // Requested ahead of time: for the first segment at once, for every other one by its predecessor,
    // between the end of its own key loop and its epilogue.
    bf16x8 qf[QB][KS];
    auto first_tiles = [&](const difa_segment_t& sg, int sb) __attribute__((always_inline)) {
        const int b = sg.bh / a.heads, h = sg.bh - b * a.heads;
        const int64_t base = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
        const unsigned long long ka = (unsigned long long)((const __bf16*)a.k + base);
        const unsigned long long va = (unsigned long long)((const __bf16*)a.v + base);
        krsrc[0] = (unsigned)ka; krsrc[1] = (unsigned)(ka >> 32) & 0xffffu; krsrc[2] = head_bytes; krsrc[3] = 0x00020000u;
        vrsrc[0] = (unsigned)va; vrsrc[1] = (unsigned)(va >> 32) & 0xffffu; vrsrc[2] = head_bytes; vrsrc[3] = 0x00020000u;
        const int n = sg.pos_end - sg.pos_begin;
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const int p = sg.pos_begin + t;
            const int tile = tile_at(p < sg.kv0_end ? p : sg.kv1_begin + (p - sg.kv0_end));
            const unsigned tb = t < n ? (unsigned)tile * tile_bytes : 0x80000000u;
            const unsigned st = (unsigned)(((sb + t) & 3) * TILE * 2) + wave_lds;
#pragma unroll
            for (int u = 0; u < NDMA; ++u) {
                dma_part(0, u, tb, k_lds + st);
                if (t < 2) dma_part(1, u, tb, v_lds + st);
            }
        }
    };
    constexpr int kFirstTileLoads = 5 * NDMA;               // load instructions first_tiles issues
    auto query_rows = [&](const difa_segment_t& sg) __attribute__((always_inline)) {
        const int b = sg.bh / a.heads, h = sg.bh - b * a.heads;
        const int64_t base = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
        const __bf16* qg = (const __bf16*)a.q + base;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int i_r = sg.q_tile * kBM + wave * RW + 32 * qb + l32;
            const int i = i_r < N ? i_r : N - 1;            // rows past the end recompute row N-1
            // B operand of S^T = K Q^T: column = query l32, k-slots 8*half..8*half+7 of each 16-wide step
            const __bf16* qrow = qg + (int64_t)i * a.stride_n + 8 * half;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *(const bf16x8*)(qrow + 16 * ks);
        }
    };
    auto first_loads = [&](const difa_segment_t& sg, int sb) __attribute__((always_inline)) {
        first_tiles(sg, sb);
        query_rows(sg);
    };

    // Persistent workgroup: one per compute unit, walking the segments the host scheduled for it.
    // The record of the following segment is fetched while the current one runs.
    const int seg_end = __builtin_amdgcn_readfirstlane(a.wg_begin[blockIdx.x + 1]);
    const int seg_first = __builtin_amdgcn_readfirstlane(a.wg_begin[blockIdx.x]);
    // ---- cached heads (Sec. 3.2; the cache fill that ends Alg. 1): out[b, h] = cache[b, h], bit for bit.
    // HBM-bound work that needs no matrix core.  It is cut into chunks of kCopyVecs 16-byte vectors of one
    // (batch entry, cached head); workgroup p takes chunks p, p + gridDim.x, ... and moves one after each of
    // its attention segments, when it waits for the next segment's first tiles anyway, so the copy is
    // spread over the launch and runs in the shadow of the other workgroups' arithmetic.
    auto copy_chunk = [&](int chunk) __attribute__((always_inline)) {
        constexpr int PER = kCopyVecs / (NW * 64);          // vectors per thread and chunk, all in flight together
        const AttnArgs* ca = cold_args();
        const int per_head = ca->copy_chunks_per_head, n_copy = ca->n_copy, shift = ca->copy_vec_shift;
        const int head_vecs = ca->copy_head_vecs;
        const unsigned row_bytes = (unsigned)ca->copy_stride_n;     // (a head spans less than 2 GiB)
        const int hh = chunk / per_head, cc = chunk - hh * per_head;
        const int bb = hh / n_copy, head = ca->copy_heads[hh - bb * n_copy];
        const int64_t base = (int64_t)bb * ca->copy_stride_b + (int64_t)head * ca->copy_stride_h;
        const char* __restrict__ src = (const char*)ca->copy_src + base;
        char* __restrict__ dst = (char*)ca->out + base;
        uintx4 val[PER];
        unsigned off[PER];
        bool live[PER];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            int vi = cc * kCopyVecs + u * (NW * 64) + tid;                // vector inside the head
            live[u] = vi < head_vecs;
            vi = live[u] ? vi : head_vecs - 1;                            // past the end: reread the last one, store nothing
            off[u] = (unsigned)(vi >> shift) * row_bytes + (unsigned)(vi & ((1 << shift) - 1)) * 16u;
        }
#pragma unroll
        for (int u = 0; u < PER; ++u) val[u] = *(const uintx4*)(src + off[u]);
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (live[u]) *(uintx4*)(dst + off[u]) = val[u];
    };
    int next_chunk = (int)blockIdx.x;

    difa_segment_t seg_next{};
    int sbase = 0;                                          // ring stage of the current segment's tile 0
    if (seg_first < seg_end) {
        seg_next = a.segs[seg_first];
        lane_offsets();
        first_loads(seg_next, sbase);
        // (the clock is read here, a few hundred clocks into the kernel, rather than on entry: at this point it
        // costs no register that the key loop needs)
        if (tid == 0) {
            const unsigned long long t = wall_clock64();
            ctl_sm[2] = (int)(unsigned)t;
            ctl_sm[3] = (int)(unsigned)(t >> 32);
        }
    }
    for (int seg_idx = seg_first; seg_idx < seg_end; ++seg_idx) {
    lane_offsets();
    // (the record was read with vector loads; moving its fields to scalar registers tells the compiler
    // that everything derived from them is uniform over the wavefront)
    difa_segment_t it;
    it.bh = __builtin_amdgcn_readfirstlane(seg_next.bh);
    it.q_tile = __builtin_amdgcn_readfirstlane(seg_next.q_tile);
    it.kv0_end = __builtin_amdgcn_readfirstlane(seg_next.kv0_end);
    it.nm0_end = __builtin_amdgcn_readfirstlane(seg_next.nm0_end);
    it.kv1_begin = __builtin_amdgcn_readfirstlane(seg_next.kv1_begin);
    it.kv1_end = __builtin_amdgcn_readfirstlane(seg_next.kv1_end);
    it.nm1_begin = __builtin_amdgcn_readfirstlane(seg_next.nm1_begin);
    it.nm1_end = __builtin_amdgcn_readfirstlane(seg_next.nm1_end);
    it.window = __builtin_amdgcn_readfirstlane(seg_next.window);
    it.pos_begin = __builtin_amdgcn_readfirstlane(seg_next.pos_begin);
    it.pos_end = __builtin_amdgcn_readfirstlane(seg_next.pos_end);
    it.part_slot = __builtin_amdgcn_readfirstlane(seg_next.part_slot);
    it.merge_idx = __builtin_amdgcn_readfirstlane(seg_next.merge_idx);
    it.n_parts = __builtin_amdgcn_readfirstlane(seg_next.n_parts);
    it.first_slot = __builtin_amdgcn_readfirstlane(seg_next.first_slot);
    it.flags = __builtin_amdgcn_readfirstlane(seg_next.flags);

    const int b = it.bh / a.heads, h = it.bh - b * a.heads;
    __bf16* __restrict__ og = (__bf16*)a.out + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const int row0 = it.q_tile * kBM + wave * RW;           // first query row of this wavefront

    // ---- per-lane query rows (two: one per 32-row block) and their allowed key ranges
    RowState rs[QB];
    int i_raw[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        i_raw[qb] = row0 + 32 * qb + l32;
        const int i = i_raw[qb] < N ? i_raw[qb] : N - 1;
        int lo, hi;
        if (it.window < 0 || (unsigned)(i - text_begin) < (unsigned)n_text) { lo = 0; hi = N - 1; }
        else { lo = i - it.window; hi = i + it.window < N - 1 ? i + it.window : N - 1; }
        rs[qb].lo = lo;
        rs[qb].span = (unsigned)(hi - lo);                  // key j is in the band iff (unsigned)(j-lo) <= span
        rs[qb].m = -1.0e30f;                                // finite: exp2(-inf - m) must be 0, not NaN
        rs[qb].l = 0.f;
    }

    floatx16 o[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][qb][r] = 0.f;

    // The segment covers positions [pos_begin, pos_end) of the record's visiting order; idx counts from
    // the segment's first position.
    const int n_iter = it.pos_end - it.pos_begin;
    auto upos_of = [&](int idx) {                           // key-tile position in the record's rotated order
        const int p = it.pos_begin + (idx < n_iter ? idx : n_iter - 1);   // past the end: reload the last tile (unused)
        return p < it.kv0_end ? p : it.kv1_begin + (p - it.kv0_end);
    };
    auto tile_of = [&](int idx) { return tile_at(upos_of(idx)); };
    auto tile_masked = [&](int idx) {
        const int t = upos_of(idx);
        return it.pos_begin + idx < it.kv0_end ? (t >= it.nm0_end) : (t < it.nm1_begin || t >= it.nm1_end);
    };
    auto tile_offset = [&](int idx) {                       // byte offset of the tile at position idx
        return idx < n_iter ? (unsigned)tile_of(idx) * tile_bytes : 0x80000000u;
    };

    // ---- S^T = K Q^T for one 32-key block jb of a tile: s[qb], register r = key 32*jb + 8*(r/4) + 4*half + r%4
    auto qk_block = [&](int idx, int jb, floatx16 (&s)[QB]) {
        const __bf16* kst = &Ksm[((idx + sbase) & 3) * TILE + 32 * jb * D];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 ka = *(const bf16x8*)(kst + koff[ks]);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                if (ks == 0) mfma_s_first(s[qb], ka, qf[qb][ks]);
                else mfma_s_acc(s[qb], ka, qf[qb][ks]);
            }
        }
        mfma_results_visible();
    };
    // Element mask of one 32-key block whose first key is j0.  The host marks a tile as masked when any
    // of the workgroup's 256 rows has a forbidden key in it; for the rows of one wavefront most such
    // blocks lie entirely inside the band, or are cut by one band edge only.  That is decided here from
    // scalars, so that the common cases cost nothing or two plain integer instructions per score.
    const int row_first = it.q_tile * kBM + (int)wave_u * RW;              // this wavefront's rows (uniform)
    const int row_last = row_first + RW - 1 < N - 1 ? row_first + RW - 1 : N - 1;
    auto mask_block = [&](int j0, floatx16 (&s)[QB]) {
        const bool plain = j0 >= img0 && j0 + 31 < img1 && row_first >= img0 && row_last < img1 && it.window >= 0;
        // image rows, image keys, no tail: row i allows keys [i - w, i + w]
        const bool low = row_last - it.window > j0;                        // some row's band starts after j0
        const bool high = row_first + it.window < j0 + 31;                 // some row's band ends before the block does
        if (plain && !low && !high) return;
        const unsigned ninf = 0xff800000u;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            // bit r of `gone` says that register r holds the score of a forbidden key
            unsigned gone = 0;
            if (plain) {
                // Register r of a lane holds the key at offset 8*(r/4) + r%4 (+ 4*half) of the block, increasing
                // with r, so the keys below the band's start are the lane's first k registers and the keys beyond
                // its end the last ones.  The count k comes from the lane's edge with a handful of integer
                // instructions.
                auto below = [](int e) {                                    // registers whose key offset is < e
                    const int ec = e < 0 ? 0 : (e > 32 ? 32 : e);
                    const int rem = ec & 7;
                    return 4 * (ec >> 3) + (rem < 4 ? rem : 4);
                };
                if (low) gone = (1u << below(rs[qb].lo - j0 - 4 * half)) - 1u;
                if (high) gone |= ~((1u << below(rs[qb].lo + (int)rs[qb].span - j0 - 4 * half + 1)) - 1u);
            } else {
                // text keys or rows, or the tail of the sequence, in the block: one unsigned range test per segment and key
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + 8 * (r >> 2) + 4 * half + (r & 3);
                    const bool ok = ((unsigned)(j - text_begin) < (unsigned)n_text) | ((unsigned)(j - rs[qb].lo) <= rs[qb].span);
                    gone |= ok ? 0u : 1u << r;
                }
            }
            // Each score then costs a signed one-bit extract (all ones or zero) and a bit-select between the score
            // and -inf, in place.  No compare writes a lane mask that the next instruction would have to wait for
            // (a compare and a select that reads its result cost 20 clocks a pair on this chip, four ordinary
            // instructions 16), and the sixteen registers are not rebuilt elsewhere (a select per score into a
            // fresh set of registers makes the compiler copy all sixteen over and back on every path through
            // here, the one that changes nothing included).
            // (one statement for the block's sixteen scores, written out so that the compiler neither turns
            // the bit-select back into a compare and a select nor pads every score with a wait state)
            float x[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) x[r] = s[qb][r];
            unsigned t0, t1;
            asm volatile("v_bfe_i32 %16, %18, 0, 1\n\tv_bfe_i32 %17, %18, 1, 1\n\tv_bfi_b32 %0, %16, %19, %0\n\tv_bfi_b32 %1, %17, %19, %1\n\tv_bfe_i32 %16, %18, 2, 1\n\tv_bfe_i32 %17, %18, 3, 1\n\tv_bfi_b32 %2, %16, %19, %2\n\tv_bfi_b32 %3, %17, %19, %3\n\tv_bfe_i32 %16, %18, 4, 1\n\tv_bfe_i32 %17, %18, 5, 1\n\tv_bfi_b32 %4, %16, %19, %4\n\tv_bfi_b32 %5, %17, %19, %5\n\tv_bfe_i32 %16, %18, 6, 1\n\tv_bfe_i32 %17, %18, 7, 1\n\tv_bfi_b32 %6, %16, %19, %6\n\tv_bfi_b32 %7, %17, %19, %7\n\tv_bfe_i32 %16, %18, 8, 1\n\tv_bfe_i32 %17, %18, 9, 1\n\tv_bfi_b32 %8, %16, %19, %8\n\tv_bfi_b32 %9, %17, %19, %9\n\tv_bfe_i32 %16, %18, 10, 1\n\tv_bfe_i32 %17, %18, 11, 1\n\tv_bfi_b32 %10, %16, %19, %10\n\tv_bfi_b32 %11, %17, %19, %11\n\tv_bfe_i32 %16, %18, 12, 1\n\tv_bfe_i32 %17, %18, 13, 1\n\tv_bfi_b32 %12, %16, %19, %12\n\tv_bfi_b32 %13, %17, %19, %13\n\tv_bfe_i32 %16, %18, 14, 1\n\tv_bfe_i32 %17, %18, 15, 1\n\tv_bfi_b32 %14, %16, %19, %14\n\tv_bfi_b32 %15, %17, %19, %15"
                         : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]),
                           "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13]), "+v"(x[14]), "+v"(x[15]),
                           "=&v"(t0), "=&v"(t1)
                         : "v"(gone), "v"(ninf));
#pragma unroll
            for (int r = 0; r < 16; ++r) s[qb][r] = x[r];
        }
    };
    // ---- softmax of one 32-key block, cut into 16 pieces of six VALU instructions, one per slot, each
    // split in two halves that sit behind the slot's two MFMAs (a wavefront issues in order:
    // whatever is not behind an MFMA delays the next one; the steady state spends nothing on a running
    // maximum).
    //   piece s: scores 2*(s&7), 2*(s&7)+1 of row block s>>3 -> two weights 2^(score*c - reference) as
    //   bf16 B operands, added to the block's row sum
    // The reference of a row is NOT the running maximum: it is set from the first block that holds an
    // allowed key and afterwards moves only when a weight outgrows 2^kTrip.  That is detected after
    // the fact, from the block's row sum, and repaired on a rare side path (renormalise() below), so
    // the hot path needs no maximum at all.  Weights are at most 2^kTrip * 16: bf16 has fp32's exponent
    // range, the row sum and O stay below 2^kTrip * N * max|v| < 2^70, far inside fp32, and the
    // common factor cancels in O / l.
    // Each piece ends in an empty volatile asm on its results: that keeps it in its slot (otherwise the
    // optimizer sinks the arithmetic to the block that uses it).
    auto pin = [](float& x) { asm volatile("" : "+v"(x)); };
    auto softmax_a = [&](int s, const floatx16 (&sc)[QB], const float (&mneg)[QB], float (&x)[2]) __attribute__((always_inline)) {
        const int qb = s >> 3, r = 2 * (s & 7);
        x[0] = __builtin_amdgcn_exp2f(fmaf(sc[qb][r], c, mneg[qb]));
        x[1] = fmaf(sc[qb][r + 1], c, mneg[qb]);
        pin(x[0]);
        pin(x[1]);
    };
    // (the row-sum update of a pair trails its conversion by one slot: a dot product issued right after
    // the conversion it reads costs a wait state, as does a conversion right after its exponential)
    auto softmax_b = [&](int s, float (&x)[2], float (&lb)[QB], bf16x8 (&pw)[QB][2], unsigned& held) __attribute__((always_inline)) {
        const int qb = s >> 3, r = 2 * (s & 7);
        bf16x2 ones;
        ones[0] = (__bf16)1.0f;
        ones[1] = (__bf16)1.0f;
        floatx2 pf;
        pf[0] = x[0];
        pf[1] = __builtin_amdgcn_exp2f(x[1]);
        if (s > 0) {                                                  // the weights that entered P V are the ones summed
            const int qp = (s - 1) >> 3;
            lb[qp] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, held), ones, ((s - 1) & 7) ? lb[qp] : 0.f, false);
            pin(lb[qp]);
        }
        bf16x2 pr = __builtin_convertvector(pf, bf16x2);
        unsigned bits = __builtin_bit_cast(unsigned, pr);
        asm volatile("" : "+v"(bits));
        pr = __builtin_bit_cast(bf16x2, bits);
        pw[qb][r >> 3][r & 7] = pr[0];
        pw[qb][r >> 3][(r & 7) + 1] = pr[1];
        held = bits;
    };
    // Rare side path, uniform over the wavefront: some row of block g produced a weight beyond 2^kTrip
    // (always the case for the first block, whose rows still carry the initial reference).  Every row
    // whose block maximum exceeds its reference by more than 2^kBump takes that maximum as its new
    // reference; the block's weights and row sums are recomputed, the running sums and O are scaled.
    // The accumulators live in accumulation registers and are scaled in place there; the waits cover
    // MFMA results still in flight.
    auto renormalise = [&](const floatx16 (&sc)[QB], float (&mneg)[QB], float (&lb)[QB], bf16x8 (&pw)[QB][2], bool rescale_o) __attribute__((always_inline)) {
        float alpha[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float tmax = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sc[qb][r]);
            const float t = halves_max(tmax) * c;
            const float m_old = rs[qb].m;
            const float m_new = t > m_old + kBump ? t : m_old;
            alpha[qb] = __builtin_amdgcn_exp2f(m_old - m_new);
            rs[qb].m = m_new;
            rs[qb].l *= alpha[qb];
            mneg[qb] = -m_new;
            lb[qb] = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                bf16x2 ones;
                ones[0] = (__bf16)1.0f;
                ones[1] = (__bf16)1.0f;
                floatx2 pf;
                pf[0] = __builtin_amdgcn_exp2f(fmaf(sc[qb][r], c, mneg[qb]));
                pf[1] = __builtin_amdgcn_exp2f(fmaf(sc[qb][r + 1], c, mneg[qb]));
                const bf16x2 pr = __builtin_convertvector(pf, bf16x2);
                pw[qb][r >> 3][r & 7] = pr[0];
                pw[qb][r >> 3][(r & 7) + 1] = pr[1];
                lb[qb] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lb[qb], false);
            }
        }
        if (!rescale_o) return;     // nothing has been accumulated yet
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float e = o[db][qb][r], t;
                    asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                                 : "+a"(e), "=&v"(t) : "v"(alpha[qb]));
                    o[db][qb][r] = e;
                }
        asm volatile("s_nop 7" ::: "memory");
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

    // ---- prologue: tiles 0 and 1 into the ring, S^T of block (tile 0, jb 0)
    dma_wait_all();     // the segment's first tiles and query rows, requested ahead of time
    // The assembly MFMAs read Q from accumulation registers.  If the compiler holds the loaded rows in
    // ordinary registers, this is where it has to move them over: a vector write needs two wait states
    // before a matrix instruction reads it, and only here are those guaranteed.
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[qb][ks]));
    asm volatile("s_nop 1" ::: "memory");
    __syncthreads();

    // The pipeline advances by 32-key blocks g = 2*tile + jb.  One half-step for block g is one basic
    // block of 8 * QB slots; slot s issues
    //     MFMA s of S^T of block g+1   | two pieces of the softmax of block g |   MFMA s of P V of block g-1
    // so that consecutive MFMAs never depend on each other and every MFMA has a few VALU
    // instructions behind it.  LDS operands are fetched three operands ahead, across half-step
    // boundaries.  Two rare side blocks follow and modify registers in place: the rescale of O by the
    // factors the softmax just produced (after P V of block g-1, before P V of block g) and the
    // element mask of the scores of block g+1.  In the last iteration block g+1 is a reload of the
    // last tile whose scores are never used.
    constexpr int NOP = D / 16;             // LDS operands per MFMA stream per half-step: 8 at D=128, 4 at D=64
    constexpr int NMF = QB * NOP;           // MFMAs per stream per half-step
    constexpr int NSLOT = 8 * QB;           // slots per half-step: one per pair of scores of a lane
    constexpr int AHEAD = 3;                // operands in flight per stream
    static_assert(NOP == 8 || NOP == 4, "slot layout assumes head_dim 128 or 64");
    floatx16 s0[QB], s1[QB];                  // scores of the even / odd block in flight
    bf16x8 pa[QB][2], pb[QB][2];              // weights of the even / odd block in flight
    bf16x8 kq[NOP], vq[NOP];                // LDS operands (entry j = operand j of the stream)

    auto half_step = [&](const floatx16 (&s_cur)[QB], floatx16 (&s_nxt)[QB], const bf16x8 (&p_prev)[QB][2],
                         bf16x8 (&p_cur)[QB][2], const __bf16* kst_nxt, const __bf16* kst_after,
                         const __bf16* vst_prev, const __bf16* vst_cur, bool with_pv, bool mask_nxt,
                         int blk_nxt, int dma_tensor, unsigned dma_tb, unsigned dma_dst) __attribute__((always_inline)) {
        float mneg[QB], lb[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mneg[qb] = -rs[qb].m;
        unsigned held = 0;
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            const int j = s / QB, qb = s % QB, jn = j + AHEAD;    // operand jn is fetched while operand j is used
            float x[2];
            if (s < NMF) {
                if (j == 0) mfma_s_first(s_nxt[qb], kq[j], qf[qb][j]);
                else mfma_s_acc(s_nxt[qb], kq[j], qf[qb][j]);
                if (qb == 0) {
                    if (jn < NOP) kq[jn] = k_operand(kst_nxt, jn);
                    else kq[jn - NOP] = k_operand(kst_after, jn - NOP);
                }
            }
            softmax_a(s, s_cur, mneg, x);
            __builtin_amdgcn_sched_barrier(0);
            if (s < NMF) {
                if (with_pv)
                    o[j >> 1][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[j], p_prev[qb][j & 1], o[j >> 1][qb], 0, 0, 0);
                if (qb == 0) {
                    if (jn < NOP) { if (with_pv) vq[jn] = v_operand(vst_prev, jn); }
                    else vq[jn - NOP] = v_operand(vst_cur, jn - NOP);
                }
            }
            softmax_b(s, x, lb, p_cur, held);
            // the loads of a later tile are spread over the slots (a burst of them right after the
            // barrier stalls all wavefronts on the one memory pipe)
            if ((s & 3) == 1 && (s >> 2) < NDMA) dma_part(dma_tensor, s >> 2, dma_tb, dma_dst);
            __builtin_amdgcn_sched_barrier(0);
        }
        {
            bf16x2 ones;
            ones[0] = (__bf16)1.0f;
            ones[1] = (__bf16)1.0f;
            lb[QB - 1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, held), ones, lb[QB - 1], false);
        }
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(fmaxf(lb[0], lb[QB - 1]) > kTrip) != 0, 0))
            renormalise(s_cur, mneg, lb, p_cur, with_pv);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) rs[qb].l += lb[qb];
        // block number blk_nxt = 2*position + jb; its first key is only needed on this rare path
        if (__builtin_expect(mask_nxt, 0)) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) mfma_results_visible(s_nxt[qb]);
            mask_block(tile_of(blk_nxt >> 1) * kBN + 32 * (blk_nxt & 1), s_nxt);
        }
    };

    seg_next = a.segs[seg_idx + 1 < seg_end ? seg_idx + 1 : seg_idx];   // has the whole key loop to arrive
    qk_block(0, 0, s0);
    if (tile_masked(0)) mask_block(tile_of(0) * kBN, s0);   // (before the loop-carried flags exist)

    // Loop-carried scalars (all uniform over the wavefront), advanced once per iteration instead of
    // being recomputed from the position: ring stages of the tiles in use, mask flags, load target.
    // A wavefront issues in order and scalar work delays its next MFMA, so there is as little of it as possible.
    const int m0e = (it.nm0_end < it.kv0_end ? it.nm0_end : it.kv0_end) - it.pos_begin;   // idx in [.., m0e) and
    const int m1b = it.kv0_end + (it.nm1_begin > it.kv1_begin ? it.nm1_begin - it.kv1_begin : 0) - it.pos_begin;
    const int m1e = it.kv0_end + ((it.nm1_end < it.kv1_end ? it.nm1_end : it.kv1_end) - it.kv1_begin) - it.pos_begin;
    auto pos_masked = [&](int idx) { return !(idx < m0e || (idx >= m1b && idx < m1e)); };   // [m1b, m1e) are mask-free
    auto bump = [](int& off) { off = (off + TILE) & (NS * TILE - 1); };          // next ring stage (element offset)
    auto kptr = [&](int off, int jb) { return &Ksm[off + 32 * jb * D]; };
    auto vptr = [&](int off, int jb) { return &Vsm[off + 32 * jb * D]; };
    // ring stages as element offsets: K stages of positions idx, idx+1, idx+3, V stages of idx-1, idx, idx+2
    int k_cur = (sbase & 3) * TILE, k_nxt = ((sbase + 1) & 3) * TILE, k_ld = ((sbase + 3) & 3) * TILE;
    int v_prv = k_cur, v_cur = k_cur, v_ld = ((sbase + 2) & 3) * TILE;
    bool msk_cur = pos_masked(0), msk_nxt = pos_masked(1);
    unsigned tb_k = tile_offset(3), tb_v = tile_offset(2);  // tiles whose K / V loads the coming iteration issues

    // first tile: its even block has no predecessor whose P V would be due
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) kq[j] = k_operand(kptr(k_cur, 1), j);
    half_step(s0, s1, pb, pa, kptr(k_cur, 1), kptr(k_nxt, 0), vptr(v_cur, 0), vptr(v_cur, 0), false,
              msk_cur, 1, 0, tb_k, k_lds + (unsigned)(k_ld * 2) + wave_lds);
    if (QB == 1) mfma_results_visible();    // no P V MFMA separated this block's last S^T MFMA from its first reader
    half_step(s1, s0, pa, pb, kptr(k_nxt, 0), kptr(k_nxt, 1), vptr(v_cur, 0), vptr(v_cur, 1), true,
              msk_nxt, 2, 1, tb_v, v_lds + (unsigned)(v_ld * 2) + wave_lds);
    dma_wait_older();

    // Iteration idx works on tiles idx-1 (P V), idx and idx+1 (S^T), issues the loads of K tile idx+3 and
    // V tile idx+2 and, before the next barrier, waits for the loads issued one iteration earlier
    // (K tile idx+2, V tile idx+1).  K tile p is last read in the first half of iteration p, V tile p in
    // the first half of iteration p+1, so both rings are four stages deep.
    // The loop body exists four times, once per ring stage the current tile can sit in: with the stage a
    // compile-time constant the ring offsets become immediate operands of the LDS reads, which saves the
    // two dozen address additions a tile costs when the stage is a run-time value, and the stage
    // bookkeeping itself.  The loop is entered at the copy the segment's second tile needs.
    auto iteration = [&](auto stage_c, int idx) __attribute__((always_inline)) {
        constexpr int P = decltype(stage_c)::value;         // ring stage of tile idx
        constexpr int KC = P * TILE, KN = ((P + 1) & 3) * TILE, KL = ((P + 3) & 3) * TILE;
        constexpr int VP = ((P + 3) & 3) * TILE, VC = P * TILE, VL = ((P + 2) & 3) * TILE;
        msk_cur = msk_nxt;
        msk_nxt = pos_masked(idx + 1);
        tb_v = tb_k;
        tb_k = tile_offset(idx + 3);
        __syncthreads();    // the tiles waited for last are in LDS for everyone; the stages loaded next are no longer read
        half_step(s0, s1, pb, pa, kptr(KC, 1), kptr(KN, 0), vptr(VP, 1), vptr(VC, 0), true,
                  msk_cur, 2 * idx + 1, 0, tb_k, k_lds + (unsigned)(KL * 2) + wave_lds);
        half_step(s1, s0, pa, pb, kptr(KN, 0), kptr(KN, 1), vptr(VC, 0), vptr(VC, 1), true,
                  msk_nxt, 2 * idx + 2, 1, tb_v, v_lds + (unsigned)(VL * 2) + wave_lds);
        dma_wait_older();
    };
    {
        int idx = 1;
        int phase = (sbase + 1) & 3;
        while (idx < n_iter) {
            switch (phase) {
                case 0:
                    iteration(std::integral_constant<int, 0>(), idx);
                    if (++idx >= n_iter) break;
                    [[fallthrough]];
                case 1:
                    iteration(std::integral_constant<int, 1>(), idx);
                    if (++idx >= n_iter) break;
                    [[fallthrough]];
                case 2:
                    iteration(std::integral_constant<int, 2>(), idx);
                    if (++idx >= n_iter) break;
                    [[fallthrough]];
                default:
                    iteration(std::integral_constant<int, 3>(), idx);
                    ++idx;
            }
            phase = 0;
        }
        v_cur = ((sbase + n_iter - 1) & 3) * TILE;          // stage of the last tile, for its second block's P V
    }
    // The key loop is over: the K stages and all V stages but the last tile's are free.  Loads past the
    // segment's end may still be depositing zeros, and other wavefronts may still be reading: wait for
    // both, then request what the next segment needs first, so that it arrives during the epilogue.
    dma_wait_all();
    __syncthreads();
    const int sbase_next = (sbase + n_iter) & 3;            // keeps clear of the stage the last P V still reads
    if (seg_idx + 1 < seg_end && it.part_slot < 0) first_loads(seg_next, sbase_next);   // (a piece: after its slot stores)
    // P V of the very last block (its first operands are already in flight)
    {
        const __bf16* vst = vptr(v_cur, 1);
#pragma unroll
        for (int i = 0; i < NOP; ++i) {
            if (i + AHEAD < NOP) vq[i + AHEAD] = v_operand(vst, i + AHEAD);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                o[i >> 1][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[i], pb[qb][i & 1], o[i >> 1][qb], 0, 0, 0);
        }
    }

    // ---- epilogue: O^T register r of block db is feature d = 32*db + 8*(r/4) + 4*half + r%4
    float l_fin[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_fin[qb] = halves_sum(rs[qb].l);
    bool writes_rows = it.part_slot < 0;
    if (it.part_slot >= 0) {
        // A piece of a cut record.  Its unnormalised fp32 accumulators, row reference (log2 domain) and row
        // sum go to the piece's scratch slot; then it takes a ticket of the record.  The piece that draws
        // the last ticket folds the other pieces' slots into its own accumulators,
        //     O = sum_p O_p 2^(m_p - M),  l = sum_p l_p 2^(m_p - M),  M = max_p m_p,
        // in the register layout it already holds them in, writes the record's rows like a whole record
        // and puts the ticket counter back to zero for the next launch.
        // The slot stores and loads are device-coherent ("sc1": written through and read around a stale L2
        // line): another piece may run on another accelerator die, with an L2 of its own, and ordinary
        // accesses would need a device-wide release and acquire, i.e. writing back and invalidating a die's
        // whole L2, the K/V tiles its workgroups share included.
        const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(a.part_o, 0, 0x7fffffff, 0x00020000);
        const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(a.part_ml, 0, 0x7fffffff, 0x00020000);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int rl = it.part_slot * kBM + wave * RW + 32 * qb + l32;       // row inside the scratch
            if (i_raw[qb] < N) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        floatx4 w4;
#pragma unroll
                        for (int e = 0; e < 4; ++e) w4[e] = o[db][qb][4 * g + e];
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, w4), ro,
                                                               (rl * D + 32 * db + 8 * g + 4 * half) * 4, 0, kDeviceCoherent);
                    }
                if (half == 0) {
                    floatx2 ml;
                    ml[0] = rs[qb].m;
                    ml[1] = l_fin[qb];
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(uintx2, ml), rm, rl * 8, 0, kDeviceCoherent);
                }
            }
        }
        // The slot has to be written before the ticket is taken.  The next segment's query rows and first
        // tiles are requested behind the slot stores, and the tiles are not waited for: memory operations
        // complete in the order they were issued, so "all but the youngest kFirstTileLoads" covers the
        // stores.  (The empty statements keep the compiler from moving a memory operation across them, so
        // that no store is issued among the tile loads; anything it adds there only makes the wait stricter.)
        if (seg_idx + 1 < seg_end) {
            asm volatile("" ::: "memory");
            query_rows(seg_next);
            asm volatile("" ::: "memory");
            first_tiles(seg_next, sbase_next);
            asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kFirstTileLoads) : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        __syncthreads();                                     // ... by every wavefront
        if (tid == 0) ctl_sm[0] = atomicAdd(cold_args()->tickets + it.merge_idx, 1);
        __syncthreads();
        if (ctl_sm[0] == it.n_parts - 1) {
#pragma unroll 1
            for (int p = 0; p < it.n_parts; ++p) {
                const int slot = it.first_slot + p;
                if (slot == it.part_slot) continue;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const int rl = slot * kBM + wave * RW + 32 * qb + l32;
                    // (whole vectors are reinterpreted: a bit_cast applied to one vector element reads element 0)
                    const floatx2 ml = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(rm, rl * 8, 0, kDeviceCoherent));
                    floatx4 x[DB][4];
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int g = 0; g < 4; ++g)
                            x[db][g] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                ro, (rl * D + 32 * db + 8 * g + 4 * half) * 4, 0, kDeviceCoherent));
                    const float m_new = fmaxf(rs[qb].m, ml[0]);
                    const float w_mine = __builtin_amdgcn_exp2f(rs[qb].m - m_new), w_other = __builtin_amdgcn_exp2f(ml[0] - m_new);
                    rs[qb].m = m_new;
                    l_fin[qb] = fmaf(ml[1], w_other, l_fin[qb] * w_mine);
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int g = 0; g < 4; ++g)
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                o[db][qb][4 * g + e] = fmaf(x[db][g][e], w_other, o[db][qb][4 * g + e] * w_mine);
                }
            }
            if (tid == 0) atomicExch(cold_args()->tickets + it.merge_idx, 0);
            writes_rows = true;
        }
    }
    if (writes_rows) {
        // A lane holds features 8g + 4*half + (0..3) of its row for g = 0..3 in each block db.  The two
        // halves of the wavefront exchange one quad per pair (g, g+1), after which the lower half holds
        // features 8g..8g+7 and the upper half 8(g+1)..8(g+1)+7: 16-byte stores, half as many of them (with
        // the next segment's loads already in flight, more memory instructions than the 63 the counter
        // can track would stall the wavefront until loads return).
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float inv = 1.0f / l_fin[qb];
            const int64_t row_off = (int64_t)(i_raw[qb] < N ? i_raw[qb] : N - 1) * a.stride_n;
            __bf16* orow = og + row_off;
            if (it.flags & DIFA_ITEM_ADD_RESIDUAL) {
                // arrow attention with residual sharing: the head's kept difference is added to the
                // normalised result before it is rounded (the lane's features: four in a row per (db, g))
                const __bf16* rrow = (const __bf16*)cold_args()->residual + (og - (__bf16*)a.out) + row_off;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const bf16x4 rv = *(const bf16x4*)(rrow + 32 * db + 8 * g + 4 * half);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            o[db][qb][4 * g + e] = fmaf(o[db][qb][4 * g + e], inv, (float)rv[e]);
                    }
                inv = 1.0f;
            }
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) {
                    unsigned w[2][2];                        // [g - 2*gp][pair of features]
#pragma unroll
                    for (int gg = 0; gg < 2; ++gg)
#pragma unroll
                        for (int e2 = 0; e2 < 2; ++e2) {
                            floatx2 f;
                            f[0] = o[db][qb][4 * (2 * gp + gg) + 2 * e2] * inv;
                            f[1] = o[db][qb][4 * (2 * gp + gg) + 2 * e2 + 1] * inv;
                            w[gg][e2] = __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
                        }
                    uintx4 q4;
#pragma unroll
                    for (int e2 = 0; e2 < 2; ++e2) {
                        // lower half keeps its quad of g and receives the upper half's; the upper half receives
                        // the lower half's quad of g+1 and keeps its own
                        const auto r = __builtin_amdgcn_permlane32_swap(w[0][e2], w[1][e2], false, false);
                        const unsigned first = r[0], second = r[1];
                        q4[e2] = first;
                        q4[2 + e2] = second;
                    }
                    if (i_raw[qb] < N) *(uintx4*)(orow + 32 * db + 16 * gp + 8 * half) = q4;
                }
        }
    }
    sbase = sbase_next;
    // one chunk of the cached-head copy, while the next segment's first tiles are on their way
    if (next_chunk < cold_args()->copy_chunks) {
        copy_chunk(next_chunk);
        next_chunk += (int)gridDim.x;
    }
    }
    // whatever is left of this workgroup's share of the copy (a layer with every head cached goes to cache_copy_kernel instead)
    {
        const int copy_chunks = cold_args()->copy_chunks;
        for (; next_chunk < copy_chunks; next_chunk += (int)gridDim.x) copy_chunk(next_chunk);
    }
    if (tid == 0) {
        const AttnArgs* ca = cold_args();
        if (ca->wg_times) {
            // (read through a pointer the compiler cannot trace back to the store, or it would carry the value
            // in registers from one end of the kernel to the other)
            const int* ts = ctl_sm;
            asm volatile("" : "+v"(ts));
            const unsigned long long t0 = (unsigned long long)(unsigned)ts[2] | ((unsigned long long)(unsigned)ts[3] << 32);
            const unsigned long long ran = seg_first < seg_end ? wall_clock64() - t0 : 0;   // (no segments: no start time)
            ca->wg_times[blockIdx.x] = ((unsigned long long)ca->launch_tag << 32) | (ran < 0xffffffffull ? ran : 0xffffffffull);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Scratch of difa_joint_attention_static, the entry point for callers that must not allocate: the
// partial results of cut records (what part_o / part_ml point at) live in this file-scope array
// instead of a buffer the plan object allocated.  512 pieces of 256 rows at head_dim 128:
// 512 * 256 * (128 + 2) floats = 68 157 440 bytes, held by every GPU the library runs on until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the device
// address is looked up once per device and is what the kernels receive as an argument.
// ------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchFloats = (size_t)512 * kBM * (128 + 2);
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices];      // device address of `scratch` per device ordinal
static std::mutex g_scratch_mutex;

hipError_t static_scratch_init(int device) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return hipSuccess;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));   // of the current device's copy
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = (float*)ptr;
    return hipSuccess;
}

float* static_scratch(int device, size_t* bytes) {
    if (bytes) *bytes = kStaticScratchFloats * sizeof(float);
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return g_scratch_ptr[device];
}

// 32-row blocks per wavefront (the kernel's QB).  1: eight wavefronts per workgroup, two per SIMD, so that
// one wavefront's softmax arithmetic runs while the other's MFMA occupies the matrix core; 2: four
// wavefronts, one per SIMD, each LDS operand read feeding two MFMAs.  Measured on one MI355X, 1 against 2:
// 16 % fewer clocks per key tile, and at the 1K layers, head_dim 64 and narrow windows 5-19 % less time;
// at the long 2K layers the time is the same, because there the chip runs at its power limit and
// lowers its clock by as much as the schedule got tighter.
constexpr int kRowBlocks = 1;

hipError_t launch_attn_bf16(const AttnArgs& a, int head_dim, int n_wg, hipStream_t stream) {
    if (n_wg <= 0) return hipSuccess;
    if (head_dim == 128)
        hipLaunchKernelGGL((attn_bf16_kernel<128, kRowBlocks>), dim3(n_wg), dim3(512 / kRowBlocks), 0, stream, a);
    else if (head_dim == 64)
        hipLaunchKernelGGL((attn_bf16_kernel<64, kRowBlocks>), dim3(n_wg), dim3(512 / kRowBlocks), 0, stream, a);
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
        // allowed keys: the text keys [seg0_begin, seg0_end) and the image keys [lo, hi]
        const int tb = a.text_begin, img0 = tb == 0 ? n_text : 0, img1 = tb == 0 ? N : tb;
        int seg0_begin, seg0_end, lo, hi;
        if (it.window < 0 || (unsigned)(i - tb) < (unsigned)n_text) { seg0_begin = seg0_end = 0; lo = 0; hi = N - 1; }
        else {
            seg0_begin = tb;
            seg0_end = tb + n_text;
            lo = i - it.window > img0 ? i - it.window : img0;
            hi = i + it.window < img1 - 1 ? i + it.window : img1 - 1;
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
        for (int j = seg0_begin + lane; j < seg0_end; j += 64) m = fmax(m, score(j));
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
        for (int j = seg0_begin + lane; j < seg0_end; j += 64) accumulate(j);
        for (int j = lo + lane; j <= hi; j += 64) accumulate(j);
        l = wave_sum(l);
        float mine = 0.f;                                    // lane d%64 keeps feature d
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const float tot = wave_sum(acc[d]);
            if ((d & 63) == lane) mine = tot / l;
            if ((d & 63) == 63) {
                const int64_t e = (int64_t)i * a.stride_n + (d - 63) + lane;
                if (it.flags & DIFA_ITEM_ADD_RESIDUAL) mine += ((const float*)a.residual)[base + e];   // + kept difference
                og[e] = mine;
            }
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
// Cached heads (Sec. 3.2) by a kernel of their own: on the fp32 debug path, and for a bf16 layer that computes
// no head at all.  A 16-byte-per-lane copy of the heads' rows; beyond 32768 workgroups a thread takes
// several vectors, four in flight.  HBM bound: 2 * N * D * elem bytes per (batch entry, cached head).
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

// ------------------------------------------------------------------------------------------
// Residual sharing, refresh step: residual = o_full - o_arrow, element by element, rounded once to the
// element type.  HBM bound: three tensors pass once.
// ------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void residual_store_kernel(const void* o_full, const void* o_arrow, void* residual,
                                                              int64_t n_vec) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride) {
        if (BF16) {
            const bf16x8 a = ((const bf16x8*)o_full)[i], b = ((const bf16x8*)o_arrow)[i];
            bf16x8 r;
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = (__bf16)((float)a[e] - (float)b[e]);   // the difference of two bf16 values is exact in fp32
            ((bf16x8*)residual)[i] = r;
        } else {
            const floatx4 a = ((const floatx4*)o_full)[i], b = ((const floatx4*)o_arrow)[i];
            ((floatx4*)residual)[i] = a - b;
        }
    }
}

hipError_t launch_residual_store(const void* o_full, const void* o_arrow, void* residual, int64_t n_elems, int dtype,
                                 hipStream_t stream) {
    if (n_elems <= 0) return hipSuccess;
    const bool bf16 = dtype == DIFA_DTYPE_BF16;
    const int64_t n_vec = n_elems / (bf16 ? 8 : 4);          // (head_dim is a multiple of 64: no remainder)
    int64_t blocks = (n_vec + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (bf16) hipLaunchKernelGGL(residual_store_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, o_full, o_arrow, residual, n_vec);
    else hipLaunchKernelGGL(residual_store_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, o_full, o_arrow, residual, n_vec);
    return hipGetLastError();
}

hipError_t launch_cache_copy(const CopyArgs& c, hipStream_t stream) {
    const int64_t total = (int64_t)c.n_tokens * c.vec_per_row * c.n_copy * c.batch;
    if (total <= 0) return hipSuccess;
    // (measured on a 2K layer with every head cached: one vector per thread and as many small workgroups as
    // that takes moves 6.4 TB/s, four per thread in a quarter of the workgroups 5.9)
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 128) blocks = 256 * 128;
    hipLaunchKernelGGL(cache_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, c);
    return hipGetLastError();
}

}  // namespace difa
