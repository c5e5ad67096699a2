// Host side of the C ABI: argument checking, the per-plan memo of compiled work lists, and
// the launches.  The operator is Sec. 3.3 of the paper (per-head full / arrow / cached
// output, cached heads filled as in the last statement of Alg. 1).
#include <limits.h>
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "difa_internal.h"
#include "difa_schedule.h"

namespace {

constexpr int kSlots = 8;      // distinct (head plan, n_text, n_img) schedules kept resident on the device
constexpr int kStagings = 16;  // pinned host buffers the schedules are uploaded from, used in turn
constexpr int kXcd = 8;        // accelerator dies of an MI355X: workgroup p runs on die p % 8

constexpr int kMaxDies = 16;
constexpr int kRecent = 64;

struct Slot {
    void* d_buf = nullptr;  // device: CACHE-head indices, then the schedule (or the debug path's work records)
    int32_t n_items = 0, n_copy = 0, n_merges = 0, n_slots = 0;
    size_t wg_off = 0, segs_off = 0, merges_off = 0, items_off = 0;  // byte offsets inside the buffer
    bool valid = false;
    uint64_t stamp = 0;
    int64_t die_span[kMaxDies] = {};    // predicted finishing time of each die, in the scheduler's cost units
    // The schedule exists in two versions: dies alike (0), or work in proportion to the measured die speeds (1).
    // Which one is faster is measured, not assumed: the one made first runs until three launches of it have
    // been timed, then the other one, then the faster of the two stays.
    int version = 0;                    // the one in the buffer
    int trial = 0;                      // 0: first version on trial, 1: second version on trial, 2: settled
    uint32_t sched_id = 0;              // names this compilation (run-time reports are credited to it)
    double ticks[2] = {0.0, 0.0};       // measured launch times per version, summed
    int timed[2] = {0, 0};
};

struct Staging {
    void* h_buf = nullptr;        // pinned host memory
    hipEvent_t copied = nullptr;  // recorded behind the host-to-device copy that reads h_buf
    bool pending = false;         // such a copy has been issued
};

struct TimingPair {
    hipEvent_t start, stop;
    int kind;  // 0 attention, 1 copy, 2 influence metric
};

}  // namespace

struct difa_plan {
    difa_plan_desc_t desc;
    float scale;
    int32_t bm, bn;
    int32_t item_capacity;
    int32_t n_wg, n_xcd;           // persistent workgroups (one per compute unit), accelerator dies
    size_t buf_bytes, heads_bytes; // schedule buffer: cached-head list, then the schedule
    float* part_o = nullptr;       // device scratch for records cut into pieces: 2 * n_wg slots
    float* part_ml = nullptr;
    int32_t* ctl = nullptr;        // device: one ticket per cut record; zero between launches
    // Die speeds (bf16 path).  Every workgroup of a launch reports how long it ran into pinned host memory;
    // before the next schedule is made, the host turns the reports of the latest finished launch into
    // relative speeds of the accelerator dies (predicted cost of a die's slowest workgroup / its measured
    // time) and keeps a running average.  Nothing waits for a report: one that has not arrived is not used.
    unsigned long long* h_times = nullptr;   // pinned, n_wg entries: launch tag << 32 | ticks
    unsigned long long* d_times = nullptr;   // the same memory as the device addresses it
    double die_speed[kMaxDies];              // mean 1
    int speed_samples = 0, retunes = 0, reports_seen = 0;
    uint32_t launch_tag = 0, harvested_tag = 0;
    struct Launch { uint32_t tag = 0; int64_t span[kMaxDies] = {}; int slot = -1; uint32_t sched_id = 0; };
    uint32_t next_sched_id = 0;
    Launch recent[kRecent];                  // the latest launches, by tag % kRecent: what each die was predicted to take
    double* rse_part = nullptr;    // device scratch of difa_head_rse: batch * heads * kRseChunks * 3 sums
    // Everything the object enqueues is kept in one order, whatever streams the calls name: the scratch
    // buffers, the counters and the schedule buffers are shared by all of them.  While the calls stay on
    // one stream that costs nothing; when the stream changes, the new one waits for an event recorded
    // on the old one at that moment.
    hipStream_t cur_stream = nullptr;
    hipEvent_t order_ev = nullptr;
    bool launched = false;
    std::vector<difa_work_item_t> recs; // host scratch of the work-list compiler
    std::vector<int32_t> keys;          // memo keys: kSlots rows of 2 * heads + 2, then one row for the call's own
    Slot slots[kSlots];
    Staging stagings[kStagings];
    int next_staging = 0;
    uint64_t clock = 0;
    std::string err;
    bool timing = false;
    std::vector<TimingPair> pending, pool;
    double attn_ms = 0, copy_ms = 0, rse_ms = 0;
    int64_t launches = 0, rse_launches = 0;
};

namespace {

thread_local std::string g_create_err;

// (Keeping the message is best effort: running out of host memory while recording an error must not
// turn into an exception that crosses the C boundary.)
difa_status_t fail(difa_plan* p, difa_status_t st, const std::string& msg) noexcept {
    try {
        if (p) p->err = msg; else g_create_err = msg;
    } catch (...) {
    }
    return st;
}
difa_status_t fail(difa_plan* p, difa_status_t st, const char* msg) noexcept {
    try {
        if (p) p->err = msg; else g_create_err = msg;
    } catch (...) {
    }
    return st;
}

// Runs the body of an entry point; nothing it throws leaves the library.
template <class F>
difa_status_t guarded(difa_plan* p, F&& body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(p, DIFA_ERR_ALLOC, "out of host memory");
    } catch (...) {
        return fail(p, DIFA_ERR_HIP, "unexpected C++ exception");
    }
}

std::string hip_msg(const char* what, hipError_t e) noexcept {
    try {
        return std::string(what) + ": " + hipGetErrorString(e);
    } catch (...) {
        return std::string();
    }
}

size_t elem_size(int dtype) { return dtype == DIFA_DTYPE_BF16 ? 2 : 4; }

void free_buffers(difa_plan* p) {
    for (Slot& s : p->slots) {
        if (s.d_buf) (void)hipFree(s.d_buf);
        s = Slot();
    }
    for (Staging& g : p->stagings) {
        if (g.h_buf) (void)hipHostFree(g.h_buf);
        if (g.copied) (void)hipEventDestroy(g.copied);
        g = Staging();
    }
    if (p->h_times) (void)hipHostFree(p->h_times);
    p->h_times = p->d_times = nullptr;
    if (p->part_o) (void)hipFree(p->part_o);
    if (p->part_ml) (void)hipFree(p->part_ml);
    if (p->ctl) (void)hipFree(p->ctl);
    if (p->rse_part) (void)hipFree(p->rse_part);
    if (p->order_ev) (void)hipEventDestroy(p->order_ev);
    p->part_o = p->part_ml = nullptr;
    p->ctl = nullptr;
    p->rse_part = nullptr;
    p->order_ev = nullptr;
}

constexpr int kMaxDevices = 64;
struct DeviceSpeeds { double speed[kMaxDies]; int n_dies = 0; };
DeviceSpeeds g_device_speeds[kMaxDevices];
std::mutex g_speed_mutex;

// Turns the run-time reports into die speeds when they are all from one launch (its workgroups have all ended
// and no workgroup of a later launch has) and that launch is still remembered.
void harvest_die_speeds(difa_plan* p) {
    if (!p->h_times) return;
    const int n_xcd = p->n_xcd;
    unsigned long long ticks[kMaxDies] = {};
    const volatile unsigned long long* t = p->h_times;
    const uint32_t tag = (uint32_t)(t[0] >> 32);
    if (tag == 0 || tag == p->harvested_tag) return;
    const difa_plan::Launch& l = p->recent[tag % kRecent];
    if (l.tag != tag) return;                                         // too long ago
    for (int w = 0; w < p->n_wg; ++w) {
        const unsigned long long v = t[w];
        if ((uint32_t)(v >> 32) != tag) return;                       // two launches' reports side by side: not now
        const unsigned long long ran = v & 0xffffffffull;
        if (ran > ticks[w % n_xcd]) ticks[w % n_xcd] = ran;
    }
    p->harvested_tag = tag;
    if (l.slot >= 0 && l.slot < kSlots) {                             // the launch's own time, for its schedule's trial
        Slot& sl = p->slots[l.slot];
        unsigned long long longest = 0;
        for (int x = 0; x < n_xcd; ++x) longest = std::max(longest, ticks[x]);
        if (sl.valid && sl.sched_id == l.sched_id && sl.trial < 2 && longest > 0) {
            if (p->reports_seen > 0) {                                // (the process's very first launch runs on a cold chip)
                sl.ticks[sl.version] += (double)longest;
                ++sl.timed[sl.version];
            }
        }
    }
    ++p->reports_seen;
    double rate[kMaxDies], mean = 0.0;
    for (int x = 0; x < n_xcd; ++x) {
        // (only launches that keep every die busy for a few dozen key-tile iterations say anything)
        if (l.span[x] < 256 || ticks[x] < 1000) return;
        rate[x] = (double)l.span[x] / (double)ticks[x];
        mean += rate[x] / n_xcd;
    }
    for (int x = 0; x < n_xcd; ++x) {
        double sp = rate[x] / mean;
        sp = sp < 0.85 ? 0.85 : (sp > 1.15 ? 1.15 : sp);
        p->die_speed[x] = p->speed_samples == 0 ? sp : 0.7 * p->die_speed[x] + 0.3 * sp;
    }
    ++p->speed_samples;
    // (what one plan object has learnt is where the next one on this device starts)
    if (p->desc.device >= 0 && p->desc.device < kMaxDevices) {
        std::lock_guard<std::mutex> lock(g_speed_mutex);
        DeviceSpeeds& g = g_device_speeds[p->desc.device];
        for (int x = 0; x < n_xcd; ++x) g.speed[x] = p->die_speed[x];
        g.n_dies = n_xcd;
    }
}

// Puts what is about to be enqueued on `stream` behind everything this object enqueued before.
hipError_t order_behind_earlier_calls(difa_plan* p, hipStream_t stream) {
    if (p->launched && p->cur_stream != stream) {
        hipError_t e = hipEventRecord(p->order_ev, p->cur_stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(stream, p->order_ev, 0);
        if (e != hipSuccess) {
            // (the earlier stream may have been destroyed by its owner: fall back to the whole device)
            (void)hipGetLastError();
            e = hipDeviceSynchronize();
            if (e != hipSuccess) return e;
        }
    }
    p->cur_stream = stream;
    p->launched = true;
    return hipSuccess;
}

// Switches to the plan's device for the scope of a call and back afterwards.
struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    hipError_t enter(int dev) {
        hipError_t e = hipGetDevice(&prev);
        if (e != hipSuccess) return e;
        if (prev != dev) {
            e = hipSetDevice(dev);
            if (e != hipSuccess) return e;
            switched = true;
        }
        return hipSuccess;
    }
    ~DeviceGuard() {
        if (switched) (void)hipSetDevice(prev);
    }
};

hipError_t timing_begin(difa_plan* p, hipStream_t stream, int kind, TimingPair* out) {
    TimingPair tp{};
    if (!p->pool.empty()) {
        tp = p->pool.back();
        p->pool.pop_back();
    } else {
        hipError_t e = hipEventCreate(&tp.start);
        if (e != hipSuccess) return e;
        e = hipEventCreate(&tp.stop);
        if (e != hipSuccess) { (void)hipEventDestroy(tp.start); return e; }
    }
    tp.kind = kind;
    *out = tp;
    return hipEventRecord(tp.start, stream);
}

hipError_t timing_flush(difa_plan* p) {
    hipError_t first = hipSuccess;
    for (TimingPair& tp : p->pending) {
        hipError_t e = hipEventSynchronize(tp.stop);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, tp.start, tp.stop);
        if (e == hipSuccess) {
            if (tp.kind == 0) { p->attn_ms += ms; p->launches += 1; }
            else if (tp.kind == 1) p->copy_ms += ms;
            else { p->rse_ms += ms; p->rse_launches += 1; }
        } else if (first == hipSuccess) {
            first = e;
        }
        p->pool.push_back(tp);
    }
    p->pending.clear();
    return first;
}

}  // namespace

extern "C" const char* difa_status_string(difa_status_t st) {
    switch (st) {
        case DIFA_OK: return "ok";
        case DIFA_ERR_INVALID_ARG: return "invalid argument";
        case DIFA_ERR_UNSUPPORTED: return "unsupported configuration";
        case DIFA_ERR_ALLOC: return "allocation failed";
        case DIFA_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char* difa_last_error(const difa_plan_t* plan) {
    return plan ? plan->err.c_str() : g_create_err.c_str();
}

extern "C" difa_status_t difa_plan_create(const difa_plan_desc_t* desc, difa_plan_t** plan_out) {
    return guarded(nullptr, [&]() -> difa_status_t {
    if (plan_out) *plan_out = nullptr;
    if (!desc || !plan_out) return fail(nullptr, DIFA_ERR_INVALID_ARG, "desc and plan_out must not be NULL");
    if (desc->batch < 1 || desc->heads < 1 || desc->max_tokens < 1 ||
        (desc->flags & ~(uint32_t)(DIFA_FLAG_BLOCK_BAND | DIFA_FLAG_IMAGE_FIRST)) != 0 || desc->device < 0)
        return fail(nullptr, DIFA_ERR_INVALID_ARG, "batch, heads, max_tokens must be >= 1, device >= 0, no unknown flag bits");
    if (!(desc->softmax_scale >= 0.f) || isinf(desc->softmax_scale))
        return fail(nullptr, DIFA_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0 (0 = 1/sqrt(head_dim))");
    if (desc->head_dim != 64 && desc->head_dim != 128)
        return fail(nullptr, DIFA_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
    if (desc->dtype != DIFA_DTYPE_BF16 && desc->dtype != DIFA_DTYPE_F32)
        return fail(nullptr, DIFA_ERR_UNSUPPORTED, "dtype must be DIFA_DTYPE_BF16 or DIFA_DTYPE_F32");
    if (desc->dtype == DIFA_DTYPE_F32 && (desc->flags & DIFA_FLAG_BLOCK_BAND))
        return fail(nullptr, DIFA_ERR_UNSUPPORTED, "the fp32 debug path evaluates the exact band only (no DIFA_FLAG_BLOCK_BAND)");
    if (desc->layout != DIFA_LAYOUT_BHND && desc->layout != DIFA_LAYOUT_BNHD)
        return fail(nullptr, DIFA_ERR_UNSUPPORTED, "layout must be DIFA_LAYOUT_BHND or DIFA_LAYOUT_BNHD");

    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess) return fail(nullptr, DIFA_ERR_HIP, hip_msg("hipGetDeviceCount", e));
    if (desc->device >= n_dev) return fail(nullptr, DIFA_ERR_INVALID_ARG, "device ordinal out of range");
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, desc->device);
    if (e != hipSuccess) return fail(nullptr, DIFA_ERR_HIP, hip_msg("hipGetDeviceProperties", e));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(nullptr, DIFA_ERR_UNSUPPORTED, std::string("device is ") + prop.gcnArchName + ", kernels are built for gfx950 only");

    difa_plan* p = new (std::nothrow) difa_plan();
    if (!p) return fail(nullptr, DIFA_ERR_ALLOC, "out of host memory");
    p->desc = *desc;
    for (double& sp : p->die_speed) sp = 1.0;
    p->scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)desc->head_dim);
    difa_tile_shape(desc->head_dim, desc->dtype, &p->bm, &p->bn);
    const int64_t q_tiles = ((int64_t)desc->max_tokens + p->bm - 1) / p->bm;
    const int64_t cap = (int64_t)desc->batch * desc->heads * q_tiles;
    if (cap > (int64_t)1 << 24) {
        delete p;
        return fail(nullptr, DIFA_ERR_UNSUPPORTED, "batch*heads*query tiles exceeds the work-list limit");
    }
    p->item_capacity = (int32_t)cap;
    p->n_wg = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    p->n_xcd = p->n_wg % kXcd == 0 ? kXcd : 1;
    p->heads_bytes = ((size_t)desc->heads * sizeof(int32_t) + 63) / 64 * 64;
    // worst case: every record whole plus two pieces per workgroup, one merge entry per workgroup
    p->buf_bytes = p->heads_bytes + ((size_t)p->n_wg + 1) * sizeof(int32_t) + 64 +
                   ((size_t)cap + 2 * (size_t)p->n_wg) * sizeof(difa_segment_t) + 64 +
                   2 * (size_t)p->n_wg * sizeof(difa_merge_item_t) + 64 + (size_t)cap * sizeof(difa_work_item_t);
    try {
        p->recs.resize((size_t)cap);
        p->keys.assign((size_t)(kSlots + 1) * (2 * (size_t)desc->heads + 2), 0);
    } catch (const std::bad_alloc&) {
        delete p;
        return fail(nullptr, DIFA_ERR_ALLOC, "out of host memory");
    }

    DeviceGuard guard;
    e = guard.enter(desc->device);
    if (e != hipSuccess) { delete p; return fail(nullptr, DIFA_ERR_HIP, hip_msg("hipSetDevice", e)); }
    const char* what = "hipGetSymbolAddress(static scratch)";
    e = difa::static_scratch_init(desc->device);   // device address of the file-scope scratch, once per device
    if (e == hipSuccess && desc->dtype == DIFA_DTYPE_BF16) {
        what = "allocating the scratch for cut records";
        const size_t slots = 2 * (size_t)p->n_wg;
        e = hipMalloc((void**)&p->part_o, slots * (size_t)p->bm * desc->head_dim * sizeof(float));
        if (e == hipSuccess) e = hipMalloc((void**)&p->part_ml, slots * (size_t)p->bm * 2 * sizeof(float));
        const size_t ctl_bytes = slots * sizeof(int32_t);
        if (e == hipSuccess) e = hipMalloc((void**)&p->ctl, ctl_bytes);
        if (e == hipSuccess) e = hipMemset(p->ctl, 0, ctl_bytes);      // (synchronous; the kernels leave them at zero)
        if (e == hipSuccess && p->n_xcd > 1 && p->n_xcd <= kMaxDies) {
            what = "allocating the run-time reports";
            e = hipHostMalloc((void**)&p->h_times, (size_t)p->n_wg * sizeof(unsigned long long), hipHostMallocMapped);
            if (e == hipSuccess) {
                memset(p->h_times, 0, (size_t)p->n_wg * sizeof(unsigned long long));
                e = hipHostGetDevicePointer((void**)&p->d_times, p->h_times, 0);
            }
            if (e == hipSuccess && desc->device >= 0 && desc->device < kMaxDevices) {
                std::lock_guard<std::mutex> lock(g_speed_mutex);
                const DeviceSpeeds& g = g_device_speeds[desc->device];
                if (g.n_dies == p->n_xcd) {
                    for (int x = 0; x < p->n_xcd; ++x) p->die_speed[x] = g.speed[x];
                    p->speed_samples = 3;                             // (counts as known)
                }
            }
        }
    }
    if (e == hipSuccess) {
        what = "allocating work-list buffers";
        e = hipEventCreateWithFlags(&p->order_ev, hipEventDisableTiming);
        for (int s = 0; s < kSlots && e == hipSuccess; ++s) e = hipMalloc(&p->slots[s].d_buf, p->buf_bytes);
        for (int s = 0; s < kStagings && e == hipSuccess; ++s) {
            e = hipHostMalloc(&p->stagings[s].h_buf, p->buf_bytes, hipHostMallocDefault);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&p->stagings[s].copied, hipEventDisableTiming);
        }
    }
    if (e == hipSuccess) {
        what = "allocating the influence-metric scratch";
        e = hipMalloc((void**)&p->rse_part, (size_t)desc->batch * desc->heads * difa::kRseChunks * 3 * sizeof(double));
    }
    if (e != hipSuccess) {
        const difa_status_t st = e == hipErrorOutOfMemory ? DIFA_ERR_ALLOC : DIFA_ERR_HIP;
        const std::string msg = hip_msg(what, e);
        free_buffers(p);
        delete p;
        return fail(nullptr, st, msg);
    }
    *plan_out = p;
    return DIFA_OK;
    });
}

extern "C" difa_status_t difa_plan_destroy(difa_plan_t* p) {
    if (!p) return DIFA_OK;
    DeviceGuard guard;
    (void)guard.enter(p->desc.device);
    (void)timing_flush(p);
    // everything the object enqueued is in one order, so the stream of its last call has seen it all
    if (p->launched && hipStreamSynchronize(p->cur_stream) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipDeviceSynchronize();
    }
    for (TimingPair& tp : p->pool) { (void)hipEventDestroy(tp.start); (void)hipEventDestroy(tp.stop); }
    free_buffers(p);
    delete p;
    return DIFA_OK;
}

extern "C" difa_status_t difa_device_info(int32_t device, int32_t* compute_units, int32_t* clock_khz,
                                          int32_t* memory_clock_khz, int32_t* l2_bytes, char* arch, int32_t arch_len) {
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return DIFA_ERR_INVALID_ARG;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return DIFA_ERR_HIP;
    if (compute_units) *compute_units = prop.multiProcessorCount;
    if (clock_khz) *clock_khz = prop.clockRate;
    if (memory_clock_khz) *memory_clock_khz = prop.memoryClockRate;
    if (l2_bytes) *l2_bytes = prop.l2CacheSize;
    if (arch && arch_len > 0) {
        strncpy(arch, prop.gcnArchName, (size_t)arch_len - 1);
        arch[arch_len - 1] = 0;
    }
    return DIFA_OK;
}

extern "C" difa_status_t difa_plan_timing_enable(difa_plan_t* p, int32_t enable) {
    if (!p) return DIFA_ERR_INVALID_ARG;
    p->timing = enable != 0;
    return DIFA_OK;
}

extern "C" difa_status_t difa_plan_timing_read(difa_plan_t* p, double* attn_ms, double* copy_ms,
                                               int64_t* launches, int32_t reset) {
    return guarded(p, [&]() -> difa_status_t {
    if (!p) return DIFA_ERR_INVALID_ARG;
    DeviceGuard guard;
    hipError_t e = guard.enter(p->desc.device);
    if (e == hipSuccess) e = timing_flush(p);
    if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("reading kernel timing events", e));
    if (attn_ms) *attn_ms = p->attn_ms;
    if (copy_ms) *copy_ms = p->copy_ms;
    if (launches) *launches = p->launches;
    if (reset) { p->attn_ms = 0; p->copy_ms = 0; p->launches = 0; }
    return DIFA_OK;
    });
}

extern "C" difa_status_t difa_plan_die_speeds(difa_plan_t* p, double* speeds, int32_t capacity, int32_t* n_dies,
                                              int32_t* samples, int32_t* retunes) {
    if (!p) return DIFA_ERR_INVALID_ARG;
    const int n = p->h_times ? p->n_xcd : 1;
    if (n_dies) *n_dies = n;
    if (samples) *samples = p->speed_samples;
    if (retunes) *retunes = p->retunes;
    if (speeds) {
        if (capacity < n) return fail(p, DIFA_ERR_INVALID_ARG, "difa_plan_die_speeds: capacity below the number of dies");
        harvest_die_speeds(p);
        if (samples) *samples = p->speed_samples;
        for (int x = 0; x < n; ++x) speeds[x] = p->h_times ? p->die_speed[x] : 1.0;
    }
    return DIFA_OK;
}

extern "C" difa_status_t difa_plan_timing_read_head_rse(difa_plan_t* p, double* rse_ms, int64_t* launches, int32_t reset) {
    return guarded(p, [&]() -> difa_status_t {
    if (!p) return DIFA_ERR_INVALID_ARG;
    DeviceGuard guard;
    hipError_t e = guard.enter(p->desc.device);
    if (e == hipSuccess) e = timing_flush(p);
    if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("reading kernel timing events", e));
    if (rse_ms) *rse_ms = p->rse_ms;
    if (launches) *launches = p->rse_launches;
    if (reset) { p->rse_ms = 0; p->rse_launches = 0; }
    return DIFA_OK;
    });
}

namespace {

// The body of both attention entry points.  static_scratch: partial results of cut records go to the
// library's file-scope device array instead of the plan's own buffer.
difa_status_t joint_attention_impl(difa_plan_t* p, const void* q, const void* k, const void* v,
                                   void* out, const void* cache, const int32_t* head_plan,
                                   int32_t n_text, int32_t n_img, const int32_t* window,
                                   void* stream_v, bool static_scratch, const void* residual = nullptr,
                                   bool residual_entry = false) {
    if (!p) return DIFA_ERR_INVALID_ARG;
    if (!q || !k || !v || !out || !head_plan)
        return fail(p, DIFA_ERR_INVALID_ARG, "q, k, v, out and head_plan must not be NULL");
    if (n_text < 0 || n_img < 0) return fail(p, DIFA_ERR_INVALID_ARG, "n_text and n_img must be >= 0");
    const int64_t n64 = (int64_t)n_text + n_img;
    if (n64 < 1 || n64 > p->desc.max_tokens)
        return fail(p, DIFA_ERR_INVALID_ARG, "n_text + n_img must be in [1, max_tokens]");
    if (out == q || out == k || out == v) return fail(p, DIFA_ERR_INVALID_ARG, "out must not alias q, k or v");
    const int H = p->desc.heads, B = p->desc.batch, D = p->desc.head_dim, N = (int)n64;
    bool any_cache = false, any_residual = false;
    for (int h = 0; h < H; ++h) {
        const int mode = head_plan[h];
        const bool banded = mode == DIFA_HEAD_ARROW || mode == DIFA_HEAD_ARROW_RESIDUAL;
        if (mode == DIFA_HEAD_ARROW_RESIDUAL && !residual_entry)
            return fail(p, DIFA_ERR_INVALID_ARG, "DIFA_HEAD_ARROW_RESIDUAL needs difa_joint_attention_residual");
        if (mode != DIFA_HEAD_FULL && !banded && mode != DIFA_HEAD_CACHE)
            return fail(p, DIFA_ERR_INVALID_ARG, "head_plan entries must be DIFA_HEAD_FULL, _ARROW, _CACHE or _ARROW_RESIDUAL");
        if (banded && !window)
            return fail(p, DIFA_ERR_INVALID_ARG, "window must not be NULL when a head is ARROW");
        if (banded && window[h] < 0)
            return fail(p, DIFA_ERR_INVALID_ARG, "window of an ARROW head must be >= 0");
        any_cache |= (mode == DIFA_HEAD_CACHE);
        any_residual |= (mode == DIFA_HEAD_ARROW_RESIDUAL);
    }
    if (any_cache && !cache) return fail(p, DIFA_ERR_INVALID_ARG, "cache must not be NULL when a head is CACHE");
    if (any_residual && !residual)
        return fail(p, DIFA_ERR_INVALID_ARG, "residual must not be NULL when a head is ARROW_RESIDUAL");
    if (any_residual && residual == out) return fail(p, DIFA_ERR_INVALID_ARG, "residual must not alias out");
    if (p->desc.dtype == DIFA_DTYPE_BF16) {
        // the bf16 kernel addresses a head's K and V through 32-bit byte offsets (and uses offset 2^31 to
        // mean "no tile"): the distance from a head's first to its last element must stay below 2 GiB
        const int64_t row = p->desc.layout == DIFA_LAYOUT_BHND ? D : (int64_t)H * D;
        if (((n64 - 1) * row + D) * 2 >= ((int64_t)1 << 31))
            return fail(p, DIFA_ERR_UNSUPPORTED, "one head's K/V spans 2 GiB or more in this layout: too many tokens");
    }
    hipStream_t stream = (hipStream_t)stream_v;

    DeviceGuard guard;
    hipError_t e = guard.enter(p->desc.device);
    if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("hipSetDevice", e));

    e = order_behind_earlier_calls(p, stream);
    if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("ordering the call behind earlier ones", e));

    // ---- memo lookup: key = effective per-head (mode, window) + token counts
    const size_t key_len = 2 * (size_t)H + 2;
    int32_t* key = p->keys.data() + (size_t)kSlots * key_len;
    for (int h = 0; h < H; ++h) {
        key[2 * h] = head_plan[h];
        key[2 * h + 1] = head_plan[h] == DIFA_HEAD_ARROW || head_plan[h] == DIFA_HEAD_ARROW_RESIDUAL ? window[h] : 0;
    }
    key[2 * H] = n_text;
    key[2 * H + 1] = n_img;
    harvest_die_speeds(p);
    const bool speeds_known = p->h_times && p->speed_samples >= 3;
    Slot* slot = nullptr;
    int victim = -1, want_version = -1;
    for (int s = 0; s < kSlots; ++s)
        if (p->slots[s].valid && memcmp(p->keys.data() + (size_t)s * key_len, key, key_len * sizeof(int32_t)) == 0) {
            slot = &p->slots[s];
            // The trial of the schedule's two versions (see Slot): made again at most twice in its life.
            if (p->h_times && slot->n_items > 0 && slot->trial < 2 && slot->timed[slot->version] >= 3) {
                const int other = 1 - slot->version;
                if (slot->trial == 0) {
                    if (other == 0 || speeds_known) { want_version = other; slot->trial = 1; }
                } else {
                    const double mine = slot->ticks[slot->version] / slot->timed[slot->version];
                    const double theirs = slot->timed[other] > 0 ? slot->ticks[other] / slot->timed[other] : 1e300;
                    if (theirs < mine * 0.997) want_version = other;  // the earlier version was faster after all
                    slot->trial = 2;
                }
                if (want_version >= 0) { victim = s; slot = nullptr; }
            }
            break;
        }
    if (!slot) {
        const bool retune = victim >= 0;
        if (!retune) {
            victim = 0;
            for (int s = 0; s < kSlots; ++s) {
                if (!p->slots[s].valid) { victim = s; break; }
                if (p->slots[s].stamp < p->slots[victim].stamp) victim = s;
            }
        }
        Slot* lru = &p->slots[victim];
        if (retune) {
            ++p->retunes;
            lru->version = want_version;
        } else {
            lru->version = speeds_known ? 1 : 0;
            lru->trial = 0;
            lru->ticks[0] = lru->ticks[1] = 0.0;
            lru->timed[0] = lru->timed[1] = 0;
        }
        lru->sched_id = ++p->next_sched_id;
        // The device buffer may still be read by launches enqueued earlier: the copy below goes on `stream`,
        // behind all of them.  The pinned buffer it is written into on the host may still be the source of a
        // copy issued kStagings distinct plans ago that the device has not reached yet: only then the host waits.
        Staging& stg = p->stagings[p->next_staging];
        if (stg.pending && hipEventQuery(stg.copied) != hipSuccess) {
            (void)hipGetLastError();
            e = hipEventSynchronize(stg.copied);
            if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("waiting for an earlier work-list upload", e));
        }
        stg.pending = false;
        lru->valid = false;
        int32_t n_items = 0, n_copy = 0, n_segs = 0, n_merges = 0, n_slots = 0;
        char* hb = (char*)stg.h_buf;
        difa_status_t st = difa_worklist_build(B, H, head_plan, window, n_text, n_img, p->bm, p->bn, 1, p->desc.flags,
                                               p->recs.data(), p->item_capacity, &n_items, (int32_t*)hb, &n_copy);
        if (st != DIFA_OK) return fail(p, st, "work-list compilation failed");
        size_t used = p->heads_bytes;
        lru->wg_off = lru->segs_off = lru->merges_off = lru->items_off = used;
        if (p->desc.dtype == DIFA_DTYPE_BF16) {
            lru->wg_off = used;
            lru->segs_off = (lru->wg_off + ((size_t)p->n_wg + 1) * sizeof(int32_t) + 63) / 64 * 64;
            const int32_t seg_cap = n_items + 2 * p->n_wg;
            lru->merges_off = (lru->segs_off + (size_t)seg_cap * sizeof(difa_segment_t) + 63) / 64 * 64;
            const bool dies = p->h_times != nullptr;
            st = difa::schedule_for_dies(p->recs.data(), n_items, p->n_wg, p->n_xcd, dies && lru->version == 1 ? p->die_speed : nullptr,
                                         dies ? lru->die_span : nullptr, (difa_segment_t*)(hb + lru->segs_off),
                                         seg_cap, (int32_t*)(hb + lru->wg_off), &n_segs,
                                         (difa_merge_item_t*)(hb + lru->merges_off), 2 * p->n_wg, &n_merges, &n_slots);
            if (st != DIFA_OK) return fail(p, st, "scheduling the work list failed");
            used = lru->merges_off + (size_t)n_merges * sizeof(difa_merge_item_t);
        } else {
            lru->items_off = used;
            memcpy(hb + used, p->recs.data(), (size_t)n_items * sizeof(difa_work_item_t));
            used += (size_t)n_items * sizeof(difa_work_item_t);
        }
        e = hipMemcpyAsync(lru->d_buf, stg.h_buf, used, hipMemcpyHostToDevice, stream);   // only the part in use
        if (e == hipSuccess) e = hipEventRecord(stg.copied, stream);
        stg.pending = true;
        p->next_staging = (p->next_staging + 1) % kStagings;
        if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("uploading the work list", e));
        lru->n_merges = n_merges;
        lru->n_slots = n_slots;
        lru->n_items = n_items;
        lru->n_copy = n_copy;
        memcpy(p->keys.data() + (size_t)victim * key_len, key, key_len * sizeof(int32_t));
        lru->valid = true;
        slot = lru;
    }
    slot->stamp = ++p->clock;

    const size_t es = elem_size(p->desc.dtype);
    int64_t sb, sh, sn;  // strides in elements
    if (p->desc.layout == DIFA_LAYOUT_BHND) {
        sn = D; sh = (int64_t)N * D; sb = (int64_t)H * N * D;
    } else {
        sh = D; sn = (int64_t)H * D; sb = (int64_t)N * H * D;
    }
    const bool fast = p->desc.dtype == DIFA_DTYPE_BF16;
    const bool copies = slot->n_copy > 0 && cache != out;   // cached heads (Sec. 3.2): out[b, h] = cache[b, h]

    // ---- cached heads by a copy kernel of their own: on the fp32 debug path, and for a bf16 layer that computes no
    // head at all (the copy kernel fills the chip with many small workgroups and moves a fifth more bytes per second
    // than the layer kernel's one workgroup per compute unit; it is then the call's one launch)
    const bool copy_only = fast && copies && slot->n_items == 0;
    if (copies && (!fast || copy_only)) {
        difa::CopyArgs c{};
        c.src = cache;
        c.dst = out;
        c.copy_heads = (const int32_t*)slot->d_buf;
        c.stride_b = sb * (int64_t)es; c.stride_h = sh * (int64_t)es; c.stride_n = sn * (int64_t)es;
        c.batch = B; c.n_copy = slot->n_copy; c.n_tokens = N;
        c.vec_per_row = (int32_t)(D * es / 16);
        TimingPair tp{};
        if (p->timing && (e = timing_begin(p, stream, copy_only ? 0 : 1, &tp)) != hipSuccess)
            return fail(p, DIFA_ERR_HIP, hip_msg("hipEventRecord", e));
        e = difa::launch_cache_copy(c, stream);
        if (p->timing) { (void)hipEventRecord(tp.stop, stream); p->pending.push_back(tp); }
        if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("cache-copy launch", e));
    }

    // ---- one launch: the computed heads and, on the bf16 path, the cached heads as well
    if (slot->n_items > 0) {
        const char* db = (const char*)slot->d_buf;
        difa::AttnArgs a{};
        a.q = q; a.k = k; a.v = v; a.out = out;
        a.residual = residual;
        a.items = (const difa_work_item_t*)(db + slot->items_off);
        a.segs = (const difa_segment_t*)(db + slot->segs_off);
        a.wg_begin = (const int32_t*)(db + slot->wg_off);
        a.merges = (const difa_merge_item_t*)(db + slot->merges_off);
        a.part_o = p->part_o;
        a.part_ml = p->part_ml;
        if (static_scratch && fast && slot->n_slots > 0) {
            // [n_slots][bm][head_dim] accumulators, then [n_slots][bm][2] row references and sums
            size_t cap = 0;
            float* base = difa::static_scratch(p->desc.device, &cap);
            const size_t o_floats = (size_t)slot->n_slots * p->bm * D, ml_floats = (size_t)slot->n_slots * p->bm * 2;
            if (!base)
                return fail(p, DIFA_ERR_HIP, "the static scratch array has no address on this device (set up in difa_plan_create)");
            if ((o_floats + ml_floats) * sizeof(float) > cap) {
                char msg[200];
                snprintf(msg, sizeof msg, "difa_joint_attention_static: this call needs %zu bytes of scratch for %d cut-record "
                         "pieces, the static array holds %zu", (o_floats + ml_floats) * sizeof(float), slot->n_slots, cap);
                return fail(p, DIFA_ERR_UNSUPPORTED, msg);
            }
            a.part_o = base;
            a.part_ml = base + o_floats;
        }
        a.stride_b = sb; a.stride_h = sh; a.stride_n = sn;
        a.heads = H; a.n_tokens = N; a.n_text = n_text;
        const bool image_first = (p->desc.flags & DIFA_FLAG_IMAGE_FIRST) != 0;
        a.text_begin = image_first ? n_img : 0;
        a.n_kv_tiles = (N + p->bn - 1) / p->bn;
        a.tile_rot = image_first && n_text > 0 && n_img > 0 ? n_img / p->bn : 0;   // as difa_worklist_build numbers the tiles
        a.scale = p->scale;
        if (fast) {
            a.tickets = p->ctl;
            if (p->h_times && slot->n_items > 0) {
                if (++p->launch_tag == 0) p->launch_tag = 1;
                a.wg_times = p->d_times;
                a.launch_tag = p->launch_tag;
                difa_plan::Launch& l = p->recent[p->launch_tag % kRecent];
                l.tag = p->launch_tag;
                l.slot = (int)(slot - p->slots);
                l.sched_id = slot->sched_id;
                memcpy(l.span, slot->die_span, sizeof l.span);
            }
            if (copies) {
                const int vec_per_row = (int)(D * es / 16);                 // 8 or 16: a power of two
                int shift = 0;
                while ((1 << shift) < vec_per_row) ++shift;
                a.copy_src = cache;
                a.copy_heads = (const int32_t*)slot->d_buf;
                a.copy_stride_b = sb * (int64_t)es; a.copy_stride_h = sh * (int64_t)es; a.copy_stride_n = sn * (int64_t)es;
                a.n_copy = slot->n_copy;
                a.copy_vec_shift = shift;
                a.copy_head_vecs = N << shift;
                a.copy_chunks_per_head = (a.copy_head_vecs + difa::kCopyVecs - 1) / difa::kCopyVecs;
                const int64_t chunks = (int64_t)B * slot->n_copy * a.copy_chunks_per_head;
                if (chunks > INT32_MAX) return fail(p, DIFA_ERR_UNSUPPORTED, "too many cached-head chunks");
                a.copy_chunks = (int32_t)chunks;
            }
        }
        TimingPair tp{};
        if (p->timing && (e = timing_begin(p, stream, 0, &tp)) != hipSuccess)
            return fail(p, DIFA_ERR_HIP, hip_msg("hipEventRecord", e));
        e = fast ? difa::launch_attn_bf16(a, D, p->n_wg, stream)
                 : difa::launch_attn_f32(a, D, slot->n_items, stream);
        if (p->timing) { (void)hipEventRecord(tp.stop, stream); p->pending.push_back(tp); }
        if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("attention launch", e));
    }
    if (p->timing && p->pending.size() > 512) (void)timing_flush(p);
    return DIFA_OK;
}

}  // namespace

extern "C" difa_status_t difa_joint_attention(difa_plan_t* p, const void* q, const void* k, const void* v,
                                              void* out, const void* cache, const int32_t* head_plan,
                                              int32_t n_text, int32_t n_img, const int32_t* window,
                                              void* stream) {
    return guarded(p, [&]() { return joint_attention_impl(p, q, k, v, out, cache, head_plan, n_text, n_img, window, stream, false); });
}

extern "C" difa_status_t difa_joint_attention_static(difa_plan_t* p, const void* q, const void* k, const void* v,
                                                     void* out, const void* cache, const int32_t* head_plan,
                                                     int32_t n_text, int32_t n_img, const int32_t* window,
                                                     void* stream) {
    return guarded(p, [&]() { return joint_attention_impl(p, q, k, v, out, cache, head_plan, n_text, n_img, window, stream, true); });
}

extern "C" difa_status_t difa_joint_attention_residual(difa_plan_t* p, const void* q, const void* k, const void* v,
                                                       void* out, const void* cache, const void* residual,
                                                       const int32_t* head_plan, int32_t n_text, int32_t n_img,
                                                       const int32_t* window, void* stream) {
    return guarded(p, [&]() {
        return joint_attention_impl(p, q, k, v, out, cache, head_plan, n_text, n_img, window, stream, false, residual, true);
    });
}

extern "C" difa_status_t difa_residual_store(difa_plan_t* p, const void* o_full, const void* o_arrow, void* residual,
                                             int32_t n_tokens, void* stream_v) {
    return guarded(p, [&]() -> difa_status_t {
        if (!p) return DIFA_ERR_INVALID_ARG;
        if (!o_full || !o_arrow || !residual) return fail(p, DIFA_ERR_INVALID_ARG, "o_full, o_arrow and residual must not be NULL");
        if (residual == o_full || residual == o_arrow) return fail(p, DIFA_ERR_INVALID_ARG, "residual must not alias an input");
        if (n_tokens < 1 || n_tokens > p->desc.max_tokens)
            return fail(p, DIFA_ERR_INVALID_ARG, "n_tokens must be in [1, max_tokens]");
        if ((((uintptr_t)o_full | (uintptr_t)o_arrow | (uintptr_t)residual) & 15) != 0)
            return fail(p, DIFA_ERR_INVALID_ARG, "o_full, o_arrow and residual must be 16-byte aligned");
        DeviceGuard guard;
        hipError_t e = guard.enter(p->desc.device);
        if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("hipSetDevice", e));
        const int64_t n = (int64_t)p->desc.batch * p->desc.heads * n_tokens * p->desc.head_dim;
        e = difa::launch_residual_store(o_full, o_arrow, residual, n, p->desc.dtype, (hipStream_t)stream_v);
        if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("residual-store launch", e));
        return DIFA_OK;
    });
}

// Influence[h] = RSE(O[h], O'[h]) of Alg. 1 (Sec. 3.4.1, Eq. 1): one streaming pass over both tensors.
extern "C" difa_status_t difa_head_rse(difa_plan_t* p, const void* y_m, const void* y_o, int32_t n_tokens,
                                       float* rse_out, void* stream_v) {
    return guarded(p, [&]() -> difa_status_t {
    if (!p) return DIFA_ERR_INVALID_ARG;
    if (!y_m || !y_o || !rse_out) return fail(p, DIFA_ERR_INVALID_ARG, "y_m, y_o and rse_out must not be NULL");
    if (n_tokens < 1 || n_tokens > p->desc.max_tokens)
        return fail(p, DIFA_ERR_INVALID_ARG, "n_tokens must be in [1, max_tokens]");
    if ((((uintptr_t)y_m | (uintptr_t)y_o) & 15) != 0)
        return fail(p, DIFA_ERR_INVALID_ARG, "y_m and y_o must be 16-byte aligned");
    hipStream_t stream = (hipStream_t)stream_v;
    DeviceGuard guard;
    hipError_t e = guard.enter(p->desc.device);
    if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("hipSetDevice", e));
    const int64_t D = p->desc.head_dim, H = p->desc.heads, N = n_tokens;
    difa::RseArgs a{};
    a.y_m = y_m; a.y_o = y_o; a.partial = p->rse_part; a.out = rse_out;
    if (p->desc.layout == DIFA_LAYOUT_BHND) { a.stride_n = D; a.stride_h = N * D; a.stride_b = H * N * D; }
    else { a.stride_h = D; a.stride_n = H * D; a.stride_b = N * H * D; }
    a.batch = p->desc.batch; a.heads = p->desc.heads; a.n_tokens = n_tokens; a.head_dim = p->desc.head_dim;
    // the partial sums live in one scratch per plan object
    e = order_behind_earlier_calls(p, stream);
    if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("ordering the call behind earlier ones", e));
    TimingPair tp{};
    if (p->timing && (e = timing_begin(p, stream, 2, &tp)) != hipSuccess)
        return fail(p, DIFA_ERR_HIP, hip_msg("hipEventRecord", e));
    e = difa::launch_head_rse(a, p->desc.dtype, stream);
    if (p->timing) { (void)hipEventRecord(tp.stop, stream); p->pending.push_back(tp); }
    if (e != hipSuccess) return fail(p, DIFA_ERR_HIP, hip_msg("influence-metric launch", e));
    return DIFA_OK;
    });
}
