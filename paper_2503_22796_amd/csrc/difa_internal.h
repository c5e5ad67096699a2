// Internal declarations shared by the host API and the kernel translation unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "difa.h"

namespace difa {

constexpr int kBM = 256;  // query rows per workgroup (8 wavefronts x 32 rows)
constexpr int kBN = 64;   // keys per K/V tile
constexpr int kCopyVecs = 8192;  // 16-byte vectors per chunk of the cached-head copy (128 KiB)

// Arguments common to the attention kernels.  Strides are in elements.
struct AttnArgs {
    const void* q;
    const void* k;
    const void* v;
    void* out;
    const difa_work_item_t* items;  // device: one record per workgroup (fp32 debug kernel)
    const difa_segment_t* segs;     // device: segments grouped by workgroup (bf16 kernel)
    const int32_t* wg_begin;        // device: first segment of each workgroup, n_wg + 1 entries
    const difa_merge_item_t* merges;  // device: records cut into pieces
    float* part_o;                  // device scratch: [slot][kBM][head_dim] unnormalised accumulators
    float* part_ml;                 // device scratch: [slot][kBM][2] row reference (log2 domain), row sum
    int32_t* tickets;               // device, one per cut record, zero between launches: pieces finished so far
    const void* residual;           // device, shaped like out: kept differences of the residual-sharing heads (or NULL)
    // cached heads (bf16 kernel): out[b, h] = copy_src[b, h] for the heads listed in copy_heads
    const void* copy_src;
    const int32_t* copy_heads;      // device, n_copy entries
    int64_t copy_stride_b, copy_stride_h, copy_stride_n;   // in bytes
    int32_t n_copy;
    int32_t copy_chunks;            // batch * n_copy * copy_chunks_per_head; 0: nothing to copy
    int32_t copy_chunks_per_head;
    int32_t copy_head_vecs;         // 16-byte vectors per (batch entry, head): n_tokens << copy_vec_shift
    int32_t copy_vec_shift;         // log2(16-byte vectors per token row)
    int64_t stride_b, stride_h, stride_n;
    int32_t heads, n_tokens, n_text;
    int32_t text_begin;  // first text token: 0, or n_img when the image tokens come first
    int32_t tile_rot;    // key-tile position u of a record is tile (u + tile_rot) % n_kv_tiles
    int32_t n_kv_tiles;
    float scale;  // softmax scale (natural-log domain)
    // bf16 kernel, optional: workgroup p leaves (launch_tag << 32 | its running time in ticks of the
    // constant-rate 100 MHz counter) in wg_times[p] when it ends (host memory mapped into the device; NULL: off)
    unsigned long long* wg_times;
    uint32_t launch_tag;
};

struct CopyArgs {
    const void* src;
    void* dst;
    const int32_t* copy_heads;  // device, n_copy entries
    int64_t stride_b, stride_h, stride_n;  // in bytes
    int32_t batch, n_copy, n_tokens, vec_per_row;  // 16-byte vectors per token row
};

// Arguments of the influence-metric kernels.  Strides are in elements.
constexpr int kRseChunks = 64;  // workgroups per (batch, head) of the streaming pass
struct RseArgs {
    const void* y_m;
    const void* y_o;
    double* partial;  // device scratch: [batch * heads][kRseChunks][3]
    float* out;       // device: heads values
    int64_t stride_b, stride_h, stride_n;
    int32_t batch, heads, n_tokens, head_dim;
};

// Launchers (defined in difa_kernels.hip and difa_rse.hip).  All enqueue on `stream` and return the launch status.
hipError_t launch_attn_bf16(const AttnArgs& a, int head_dim, int n_wg, hipStream_t stream);
hipError_t launch_attn_f32(const AttnArgs& a, int head_dim, int n_items, hipStream_t stream);
hipError_t launch_cache_copy(const CopyArgs& a, hipStream_t stream);
hipError_t launch_head_rse(const RseArgs& a, int dtype, hipStream_t stream);
hipError_t launch_residual_store(const void* o_full, const void* o_arrow, void* residual, int64_t n_elems, int dtype,
                                 hipStream_t stream);

// File-scope device scratch of difa_joint_attention_static (defined beside the kernels that use it).
// static_scratch_init: looks up the array's address on `device`, which must be the current device; once per
// device, later calls return at once.  static_scratch: that address (NULL before init) and the array's size.
hipError_t static_scratch_init(int device);
float* static_scratch(int device, size_t* bytes);

}  // namespace difa
