// C ABI of libetsattn (see include/etsattn.h) and the kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "advance_kernel.hpp"
#include "bench_kernels.hpp"
#include "etsattn.h"
#include "merge_kernel.hpp"
#include "plan.h"
#include "prefill_attn_kernel.hpp"
#include "prefill_plan.h"
#include "selector.h"
#include "stream_kernel.hpp"
#include "tree_attn_kernel.hpp"

using namespace ets;

struct ets_ctx {
    ets_shape shape{};
    float scale = 0.f;
    int device = -1;
    PlanOptions opt;
    // variants: pools of E4M3 codes with one scale each; bf16 output
    int kv_format = ETS_KV_NATIVE;
    HeadScales k_scales{}, v_scales{};  // per kv head; all ones for native pools
    bool out_bf16 = false;
    Plan plan;
    // device copies of the plan's index arrays, carved out of one allocation
    char* d_buf = nullptr;
    size_t d_cap = 0;
    Run* d_runs = nullptr;
    StreamItem* d_stream = nullptr;
    UnitSlot* d_units = nullptr;     // the matrix-core kernel's start table, in launch order
    CascadeItem* d_wide = nullptr;
    int32_t* d_ent_order = nullptr;
    int32_t* d_part_base = nullptr;
    int32_t* d_ent_base = nullptr;   // part_base of ent_order[i]
    AdvEntry* d_adv = nullptr;       // decode-step advance: tails to extend
    int32_t* d_adv_src = nullptr;    // per growing node: leaf query that supplies its new token
    int32_t* d_adv_slots = nullptr;  // slots of the start table to refresh after an advance
    int64_t* d_adv_last_row = nullptr;  // per growing node: newest pool row at plan time
    int32_t* d_arrived = nullptr;    // merge inside the attention launch: [leaf][kv head] counters
    // step prefill: its own plan and device tables
    PrefillPlan prefill;
    char* d_pre_buf = nullptr;
    size_t d_pre_cap = 0;
    Run* d_pre_runs = nullptr;
    PrefillItem* d_pre_items = nullptr;
    hipStream_t last_stream = nullptr;
    bool stream_used = false;
    void* static_scratch = nullptr;  // this device's copy of `scratch` (null: host-only context)
    // kernel timing (benchmarks only): five events per recorded call
    bool profile = false;
    std::vector<hipEvent_t> events;
    size_t calls_recorded = 0;
};

// Partial results of ets_tree_decode_attn_static: part of the device image, so that the call
// needs no allocation.  In host code the array's name only stands for the symbol; its
// device address is looked up per GPU (scratch_on_device) and that pointer is what the
// kernels receive.
static __device__ __align__(256) unsigned char scratch[ETS_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // the array's address on every device seen so far

// Address of `scratch` on `device`, which has to be current.  Looked up once per device.
void* scratch_on_device(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[device] = ptr;
    }
    return g_scratch_ptr[device];
}

// Makes the context's device current for the scope of a call.
struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) {
            ok = false;
            return;
        }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
        target = dev;
    }
    ~DeviceGuard() {
        if (ok && prev != target) (void)hipSetDevice(prev);
    }
    int target = -1;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool shape_supported(const ets_shape& s) {
    if (s.n_kv_heads <= 0 || s.n_q_heads <= 0) return false;
    if (s.head_dim != 64 && s.head_dim != 128) return false;
    if (s.dtype != ETS_F32 && s.dtype != ETS_BF16) return false;
    if (s.n_q_heads % s.n_kv_heads != 0) return false;
    const int g = s.n_q_heads / s.n_kv_heads;
    return g == 1 || g == 2 || g == 4 || g == 8;
}

ets_status upload_plan_unguarded(ets_ctx* c);

// Copies the plan's index arrays to the device.  Nothing may throw across the C boundary:
// a failed host allocation of the staging copy becomes a status code.
ets_status upload_plan(ets_ctx* c) {
    try {
        return upload_plan_unguarded(c);
    } catch (const std::bad_alloc&) {
        return ETS_ERR_NOMEM;
    }
}

ets_status upload_plan_unguarded(ets_ctx* c) {
    const Plan& p = c->plan;
    const size_t b_runs = align_up(p.runs.size() * sizeof(Run), 256);
    const size_t b_stream = align_up(p.stream_items.size() * sizeof(StreamItem), 256);
    const size_t b_units = align_up(p.units.size() * sizeof(UnitSlot), 256);
    const size_t b_wide = align_up(p.wide_items.size() * sizeof(CascadeItem), 256);
    // Both per-entry tables end in kEntryPadding zero entries (leaf query 0, slot 0): a
    // wave's 16-entry scalar load may run past the item's last entry (check_plan replays
    // how far).
    const size_t b_ent =
        align_up((p.ent_order.size() + kEntryPadding) * sizeof(int32_t), 256);
    const size_t b_base = align_up(p.part_base.size() * sizeof(int32_t), 256);
    const size_t b_adv = align_up(p.adv.size() * sizeof(AdvEntry), 256);
    const size_t b_asrc = align_up(p.adv_src.size() * sizeof(int32_t), 256);
    const size_t b_aslot = align_up(p.adv_slots.size() * sizeof(int32_t), 256);
    const size_t b_arow = align_up(p.adv_last_row.size() * sizeof(int64_t), 256);
    // arrival counters of the merge inside the attention launch: zero here, and put back
    // to zero by the kernel itself at the end of every call
    const size_t b_arrived =
        p.fused ? align_up((size_t)p.stats.n_leaves * c->shape.n_kv_heads * sizeof(int32_t), 256) : 0;
    const size_t total = b_runs + b_stream + b_units + b_wide + 2 * b_ent + b_base + b_adv +
                         b_asrc + b_aslot + b_arow + b_arrived + 256;

    std::vector<char> stage(total, 0);
    size_t off = 0;
    auto put = [&](const void* src, size_t bytes, size_t padded) {
        if (bytes) std::memcpy(stage.data() + off, src, bytes);
        const size_t at = off;
        off += padded;
        return at;
    };
    const size_t o_runs = put(p.runs.data(), p.runs.size() * sizeof(Run), b_runs);
    const size_t o_stream =
        put(p.stream_items.data(), p.stream_items.size() * sizeof(StreamItem), b_stream);
    const size_t o_units = put(p.units.data(), p.units.size() * sizeof(UnitSlot), b_units);
    const size_t o_wide =
        put(p.wide_items.data(), p.wide_items.size() * sizeof(CascadeItem), b_wide);
    const size_t o_ent = put(p.ent_order.data(), p.ent_order.size() * sizeof(int32_t), b_ent);
    const size_t o_base = put(p.part_base.data(), p.part_base.size() * sizeof(int32_t), b_base);
    const size_t o_ebase = put(p.ent_base.data(), p.ent_base.size() * sizeof(int32_t), b_ent);
    const size_t o_adv = put(p.adv.data(), p.adv.size() * sizeof(AdvEntry), b_adv);
    const size_t o_asrc = put(p.adv_src.data(), p.adv_src.size() * sizeof(int32_t), b_asrc);
    const size_t o_aslot = put(p.adv_slots.data(), p.adv_slots.size() * sizeof(int32_t), b_aslot);
    const size_t o_arow = put(p.adv_last_row.data(), p.adv_last_row.size() * sizeof(int64_t), b_arow);
    const size_t o_arrived = put(nullptr, 0, b_arrived);

    DeviceGuard guard(c->device);
    if (!guard.ok) return ETS_ERR_HIP;
    if (c->stream_used && hipStreamSynchronize(c->last_stream) != hipSuccess) return ETS_ERR_HIP;
    if (total > c->d_cap) {
        if (c->d_buf) (void)hipFree(c->d_buf);
        c->d_buf = nullptr;
        c->d_cap = 0;
        const size_t want = align_up(total + total / 2, 4096);
        if (hipMalloc(reinterpret_cast<void**>(&c->d_buf), want) != hipSuccess) {
            (void)hipGetLastError();
            return ETS_ERR_HIP;
        }
        c->d_cap = want;
    }
    if (hipMemcpy(c->d_buf, stage.data(), total, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return ETS_ERR_HIP;
    }
    c->d_runs = reinterpret_cast<Run*>(c->d_buf + o_runs);
    c->d_stream = reinterpret_cast<StreamItem*>(c->d_buf + o_stream);
    c->d_units = reinterpret_cast<UnitSlot*>(c->d_buf + o_units);
    c->d_wide = reinterpret_cast<CascadeItem*>(c->d_buf + o_wide);
    c->d_ent_order = reinterpret_cast<int32_t*>(c->d_buf + o_ent);
    c->d_part_base = reinterpret_cast<int32_t*>(c->d_buf + o_base);
    c->d_ent_base = reinterpret_cast<int32_t*>(c->d_buf + o_ebase);
    c->d_adv = reinterpret_cast<AdvEntry*>(c->d_buf + o_adv);
    c->d_adv_src = reinterpret_cast<int32_t*>(c->d_buf + o_asrc);
    c->d_adv_slots = reinterpret_cast<int32_t*>(c->d_buf + o_aslot);
    c->d_adv_last_row = reinterpret_cast<int64_t*>(c->d_buf + o_arow);
    c->d_arrived = reinterpret_cast<int32_t*>(c->d_buf + o_arrived);
    return ETS_OK;
}

struct LaunchArgs {
    const void *k, *v, *q;
    int64_t pool_tokens;
    void* out;
    float* lse;
    float* ws_o;
    float2* ws_ml;
    hipStream_t stream;
};

template <typename T, int D, int G>
void launch_stream(const ets_ctx* c, const LaunchArgs& a) {
    constexpr int U = (G >= 8) ? 2 : 4;
    const int64_t n_items = (int64_t)c->plan.stream_items.size();
    if (n_items == 0) return;
    const unsigned grid = (unsigned)(n_items * c->shape.n_kv_heads);
    hipLaunchKernelGGL((stream_attn_kernel<T, D, G, U>), dim3(grid), dim3(64), 0, a.stream,
                       static_cast<const T*>(a.k), static_cast<const T*>(a.v), a.pool_tokens,
                       static_cast<const T*>(a.q), c->d_runs, c->d_stream, c->shape.n_kv_heads,
                       c->scale * 1.4426950408889634f, a.ws_o, a.ws_ml);
}

template <typename T, int D>
void launch_stream_g(const ets_ctx* c, const LaunchArgs& a) {
    switch (c->shape.n_q_heads / c->shape.n_kv_heads) {
        case 1: launch_stream<T, D, 1>(c, a); break;
        case 2: launch_stream<T, D, 2>(c, a); break;
        case 4: launch_stream<T, D, 4>(c, a); break;
        default: launch_stream<T, D, 8>(c, a); break;
    }
}

// Segments shared by many leaf queries: the step-prefill kernel in its decode mode, 256 query
// rows per workgroup, partial results into the same workspace slots.
void launch_wide_attn(const ets_ctx* c, const LaunchArgs& a) {
    const int64_t n_items = (int64_t)c->plan.wide_items.size();
    if (n_items <= 0) return;
    const int g = c->shape.n_q_heads / c->shape.n_kv_heads;
    const int g_shift = g == 1 ? 0 : g == 2 ? 1 : g == 4 ? 2 : 3;
    for (int64_t y0 = 0; y0 < n_items; y0 += 65535) {
        const unsigned ny = (unsigned)std::min<int64_t>(65535, n_items - y0);
        if (c->kv_format == ETS_KV_FP8_E4M3)
            hipLaunchKernelGGL((prefill_attn_kernel<true, true>),
                               dim3((unsigned)c->shape.n_kv_heads, ny), dim3(512), 0, a.stream, a.k,
                               a.v, a.pool_tokens, static_cast<const bf16_t*>(a.q), c->d_runs,
                               c->d_wide, (int)y0, g_shift, c->scale * 1.4426950408889634f,
                               c->k_scales, c->v_scales, a.ws_o, nullptr, c->d_ent_order,
                               c->d_ent_base, a.ws_ml);
        else
            hipLaunchKernelGGL((prefill_attn_kernel<false, true>),
                               dim3((unsigned)c->shape.n_kv_heads, ny), dim3(512), 0, a.stream, a.k,
                               a.v, a.pool_tokens, static_cast<const bf16_t*>(a.q), c->d_runs,
                               c->d_wide, (int)y0, g_shift, c->scale * 1.4426950408889634f,
                               c->k_scales, c->v_scales, a.ws_o, nullptr, c->d_ent_order,
                               c->d_ent_base, a.ws_ml);
    }
}

void launch_tree_attn(const ets_ctx* c, const LaunchArgs& a) {
    const int64_t n_items = (int64_t)c->plan.cascade_items.size();
    if (n_items <= 0) return;
    const int g = c->shape.n_q_heads / c->shape.n_kv_heads;
    const int g_shift = g == 1 ? 0 : g == 2 ? 1 : g == 4 ? 2 : 3;
    // grid: x = kv head, y = workgroup (at most 65535 per launch): first the items that
    // take a workgroup each, then the small ones, four to a workgroup
    const int64_t n_wgs = (int64_t)c->plan.wg_map.size();
    MergeTail tail{};
    if (c->plan.fused) {
        tail.part_base = c->d_part_base;
        tail.arrived = c->d_arrived;
        tail.n_ws_rows = c->plan.stats.n_partials * c->shape.n_q_heads;
        tail.out = a.out;
        tail.lse = a.lse;
        tail.out_bf16 = c->out_bf16 ? 1 : 0;
        tail.v_scales = c->v_scales;
    }
    for (int64_t y0 = 0; y0 < n_wgs; y0 += 65535) {
        const unsigned ny = (unsigned)std::min<int64_t>(65535, n_wgs - y0);
        const bool fp8 = c->kv_format == ETS_KV_FP8_E4M3;
        auto kernel =
            c->shape.head_dim == 64
                ? (c->plan.fused ? (fp8 ? tree_attn_kernel<true, true, 64> : tree_attn_kernel<false, true, 64>)
                                 : (fp8 ? tree_attn_kernel<true, false, 64> : tree_attn_kernel<false, false, 64>))
                : (c->plan.fused ? (fp8 ? tree_attn_kernel<true, true> : tree_attn_kernel<false, true>)
                                 : (fp8 ? tree_attn_kernel<true, false> : tree_attn_kernel<false, false>));
        hipLaunchKernelGGL(kernel, dim3((unsigned)c->shape.n_kv_heads, ny), dim3(256), 0, a.stream,
                           a.k, a.v, a.pool_tokens, static_cast<const bf16_t*>(a.q), c->d_runs,
                           c->d_units, (int)y0,
                           c->d_ent_order, c->d_ent_base, g_shift, c->scale * 1.4426950408889634f,
                           c->k_scales, a.ws_o, a.ws_ml, tail);
    }
}

ets_status upload_prefill_plan_unguarded(ets_ctx* c);

ets_status upload_prefill_plan(ets_ctx* c) {
    try {
        return upload_prefill_plan_unguarded(c);
    } catch (const std::bad_alloc&) {
        return ETS_ERR_NOMEM;
    }
}

ets_status upload_prefill_plan_unguarded(ets_ctx* c) {
    const PrefillPlan& p = c->prefill;
    // the kernel's prologue reads a whole descriptor per thread only below n_runs, but
    // keep the table padded so that a wide scalar load near its end stays inside
    const size_t b_runs = align_up((p.runs.size() + 4) * sizeof(Run), 256);
    const size_t b_items = align_up(p.items.size() * sizeof(PrefillItem), 256);
    const size_t total = b_runs + b_items + 256;
    std::vector<char> stage(total, 0);
    if (!p.runs.empty()) std::memcpy(stage.data(), p.runs.data(), p.runs.size() * sizeof(Run));
    if (!p.items.empty())
        std::memcpy(stage.data() + b_runs, p.items.data(), p.items.size() * sizeof(PrefillItem));
    DeviceGuard guard(c->device);
    if (!guard.ok) return ETS_ERR_HIP;
    if (c->stream_used && hipStreamSynchronize(c->last_stream) != hipSuccess) return ETS_ERR_HIP;
    if (total > c->d_pre_cap) {
        if (c->d_pre_buf) (void)hipFree(c->d_pre_buf);
        c->d_pre_buf = nullptr;
        c->d_pre_cap = 0;
        const size_t want = align_up(total + total / 2, 4096);
        if (hipMalloc(reinterpret_cast<void**>(&c->d_pre_buf), want) != hipSuccess) {
            (void)hipGetLastError();
            return ETS_ERR_HIP;
        }
        c->d_pre_cap = want;
    }
    if (hipMemcpy(c->d_pre_buf, stage.data(), total, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return ETS_ERR_HIP;
    }
    c->d_pre_runs = reinterpret_cast<Run*>(c->d_pre_buf);
    c->d_pre_items = reinterpret_cast<PrefillItem*>(c->d_pre_buf + b_runs);
    return ETS_OK;
}

constexpr size_t kMaxProfiledCalls = 8192;

// Event `which` (0..4) of the call being recorded, created on first use.
void mark(ets_ctx* c, int which, hipStream_t stream) {
    if (!c->profile || c->calls_recorded >= kMaxProfiledCalls) return;
    const size_t idx = c->calls_recorded * 5 + (size_t)which;
    while (c->events.size() <= idx) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) {
            (void)hipGetLastError();
            c->profile = false;
            return;
        }
        try {
            c->events.push_back(e);
        } catch (const std::bad_alloc&) {
            (void)hipEventDestroy(e);
            c->profile = false;
            return;
        }
    }
    (void)hipEventRecord(c->events[idx], stream);
}

template <int D, int G>
void launch_merge_dg(ets_ctx* c, const LaunchArgs& a) {
    const int n_leaves = (int)c->plan.stats.n_leaves;
    const int64_t pairs = (int64_t)n_leaves * c->shape.n_kv_heads;  // one wave each
    const unsigned grid = (unsigned)((pairs + 3) / 4);
    hipLaunchKernelGGL((merge_kernel<D, G>), dim3(grid), dim3(256), 0, a.stream, c->d_part_base,
                       n_leaves, c->shape.n_kv_heads, a.ws_o, a.ws_ml, a.out, c->out_bf16 ? 1 : 0,
                       a.lse, c->v_scales);
}

template <int D>
void launch_merge_d(ets_ctx* c, const LaunchArgs& a) {
    switch (c->shape.n_q_heads / c->shape.n_kv_heads) {
        case 1: launch_merge_dg<D, 1>(c, a); break;
        case 2: launch_merge_dg<D, 2>(c, a); break;
        case 4: launch_merge_dg<D, 4>(c, a); break;
        default: launch_merge_dg<D, 8>(c, a); break;
    }
}

void launch_merge(ets_ctx* c, const LaunchArgs& a) {
    if (c->shape.head_dim == 128) launch_merge_d<128>(c, a);
    else launch_merge_d<64>(c, a);
}

// `timed`: bracket the kernels with events when the "profile" option is on (may allocate)
void launch_all(ets_ctx* c, const LaunchArgs& a, bool timed) {
    const bool bf = c->shape.dtype == ETS_BF16;
    const bool was_profiling = c->profile;
    if (!timed) c->profile = false;
    mark(c, 0, a.stream);
    if (c->shape.head_dim == 128) {
        if (bf) launch_stream_g<bf16_t, 128>(c, a);
        else launch_stream_g<float, 128>(c, a);
    } else {
        if (bf) launch_stream_g<bf16_t, 64>(c, a);
        else launch_stream_g<float, 64>(c, a);
    }
    mark(c, 1, a.stream);
    launch_wide_attn(c, a);
    mark(c, 2, a.stream);
    launch_tree_attn(c, a);
    mark(c, 3, a.stream);
    if (!c->plan.fused) launch_merge(c, a);
    mark(c, 4, a.stream);
    if (c->profile && c->calls_recorded < kMaxProfiledCalls) c->calls_recorded += 1;
    if (!timed) c->profile = was_profiling;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Argument checks and launches shared by the two decode entry points.
ets_status decode_call(ets_ctx* ctx, const void* k_pool, const void* v_pool, int64_t pool_tokens,
                       const void* q, void* out, float* lse, void* workspace,
                       int64_t workspace_bytes, void* hip_stream, bool timed) {
    if (!ctx) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    if (ctx->device < 0) return ETS_ERR_HIP;
    const ets_stats& st = ctx->plan.stats;
    if (st.n_leaves == 0) return ETS_OK;
    if (!q || !out || !lse || pool_tokens < 0 || workspace_bytes < 0) return ETS_ERR_INVALID_ARG;
    if (st.unique_tokens > 0 && (!k_pool || !v_pool)) return ETS_ERR_INVALID_ARG;
    if (pool_tokens < st.min_pool_tokens) return ETS_ERR_BAD_TREE;
    // E4M3 pools are read by the matrix-core kernel only
    if (ctx->kv_format == ETS_KV_FP8_E4M3 && !ctx->plan.stream_items.empty())
        return ETS_ERR_UNSUPPORTED;
    if (workspace_bytes < st.workspace_bytes || (st.workspace_bytes > 0 && !workspace))
        return ETS_ERR_WORKSPACE;
    if (misaligned(k_pool) || misaligned(v_pool) || misaligned(q) || misaligned(out) ||
        misaligned(workspace) || (reinterpret_cast<uintptr_t>(lse) & 3u))
        return ETS_ERR_INVALID_ARG;

    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ETS_ERR_HIP;
    LaunchArgs a;
    a.k = k_pool;
    a.v = v_pool;
    a.q = q;
    a.pool_tokens = pool_tokens;
    a.out = out;
    a.lse = lse;
    a.ws_o = static_cast<float*>(workspace);
    a.ws_ml = reinterpret_cast<float2*>(a.ws_o + st.n_partials * ctx->shape.n_q_heads *
                                                     (int64_t)ctx->shape.head_dim);
    a.stream = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    launch_all(ctx, a, timed);
    ctx->last_stream = a.stream;
    ctx->stream_used = true;
    if (hipGetLastError() != hipSuccess) return ETS_ERR_HIP;
    return ETS_OK;
}

}  // namespace

extern "C" {

ets_status ets_create(ets_ctx** out, const ets_shape* shape, int hip_device) {
    if (!out || !shape) return ETS_ERR_INVALID_ARG;
    if (!shape_supported(*shape)) return ETS_ERR_UNSUPPORTED;
    if (hip_device >= 0) {
        int n = 0;
        if (hipGetDeviceCount(&n) != hipSuccess) {
            (void)hipGetLastError();
            return ETS_ERR_HIP;
        }
        if (hip_device >= n) return ETS_ERR_INVALID_ARG;
    }
    ets_ctx* c = new (std::nothrow) ets_ctx();
    if (!c) return ETS_ERR_NOMEM;
    c->shape = *shape;
    c->scale = shape->sm_scale > 0.f ? shape->sm_scale : 1.0f / std::sqrt((float)shape->head_dim);
    c->device = hip_device < 0 ? -1 : hip_device;
    for (int h = 0; h < kMaxScaledHeads; ++h) c->k_scales.s[h] = c->v_scales.s[h] = 1.f;
    if (c->device >= 0) {
        // set-up is the place for the symbol look-up: ets_tree_decode_attn_static must not
        // do anything that could allocate
        DeviceGuard guard(c->device);
        c->static_scratch = guard.ok ? scratch_on_device(c->device) : nullptr;
        if (!c->static_scratch) {
            delete c;
            return ETS_ERR_HIP;
        }
    }
    *out = c;
    return ETS_OK;
}

void ets_destroy(ets_ctx* ctx) {
    if (!ctx) return;
    if (ctx->d_buf || ctx->d_pre_buf) {
        DeviceGuard guard(ctx->device);
        if (guard.ok) {
            if (ctx->stream_used) (void)hipStreamSynchronize(ctx->last_stream);
            if (ctx->d_buf) (void)hipFree(ctx->d_buf);
            if (ctx->d_pre_buf) (void)hipFree(ctx->d_pre_buf);
        }
    }
    if (!ctx->events.empty()) {
        DeviceGuard guard(ctx->device);
        for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
    }
    delete ctx;
}

ets_status ets_set_option(ets_ctx* ctx, const char* key, int64_t value) {
    if (!ctx || !key) return ETS_ERR_INVALID_ARG;
    if (!std::strcmp(key, "wide_rows") && value == -1) {
        ctx->opt.wide_rows = -1;
        return ETS_OK;
    }
    if (!std::strcmp(key, "fuse_merge") && value == -1) {
        ctx->opt.fuse_merge = -1;
        return ETS_OK;
    }
    if (value < 0) return ETS_ERR_INVALID_ARG;
    if (!std::strcmp(key, "stream_chunk")) ctx->opt.stream_chunk = value;
    else if (!std::strcmp(key, "cascade_chunk")) ctx->opt.cascade_chunk = value;
    else if (!std::strcmp(key, "cascade_min_leaves")) ctx->opt.cascade_min_leaves = value;
    else if (!std::strcmp(key, "cascade_rows")) {
        if (value != 16 && value != 32 && value != 64) return ETS_ERR_INVALID_ARG;
        ctx->opt.cascade_rows = value;
    } else if (!std::strcmp(key, "wave_items")) ctx->opt.wave_items = value;
    else if (!std::strcmp(key, "interleave")) ctx->opt.interleave = value != 0;
    else if (!std::strcmp(key, "wide_rows")) ctx->opt.wide_rows = value;
    else if (!std::strcmp(key, "fuse_merge")) ctx->opt.fuse_merge = value != 0;
    else if (!std::strcmp(key, "mfma")) ctx->opt.mfma = value;
    else if (!std::strcmp(key, "require_sharing")) ctx->opt.require_sharing = value != 0;
    else if (!std::strcmp(key, "out_bf16")) ctx->out_bf16 = value != 0;
    else if (!std::strcmp(key, "profile")) {
        if (value != 0 && ctx->device < 0) return ETS_ERR_HIP;
        ctx->profile = value != 0;
    }
    else return ETS_ERR_INVALID_ARG;
    return ETS_OK;
}

ets_status ets_set_kv_format(ets_ctx* ctx, int kv_format, float k_scale, float v_scale) {
    if (!ctx) return ETS_ERR_INVALID_ARG;
    if (kv_format != ETS_KV_NATIVE && kv_format != ETS_KV_FP8_E4M3) return ETS_ERR_INVALID_ARG;
    if (kv_format == ETS_KV_FP8_E4M3) {
        if (!(k_scale > 0.f) || !(v_scale > 0.f) || !std::isfinite(k_scale) ||
            !std::isfinite(v_scale))
            return ETS_ERR_INVALID_ARG;
        if (ctx->shape.dtype != ETS_BF16) return ETS_ERR_UNSUPPORTED;
    }
    ctx->kv_format = kv_format;
    for (int h = 0; h < kMaxScaledHeads; ++h) {
        ctx->k_scales.s[h] = kv_format == ETS_KV_FP8_E4M3 ? k_scale : 1.f;
        ctx->v_scales.s[h] = kv_format == ETS_KV_FP8_E4M3 ? v_scale : 1.f;
    }
    ctx->opt.kv_elem_bytes = kv_format == ETS_KV_FP8_E4M3 ? 1 : 0;
    // byte counts and item sizes of a plan depend on the element size
    ctx->plan.valid = false;
    ctx->prefill.valid = false;
    return ETS_OK;
}

ets_status ets_set_kv_head_scales(ets_ctx* ctx, const float* k_scales, const float* v_scales) {
    if (!ctx || !k_scales || !v_scales) return ETS_ERR_INVALID_ARG;
    if (ctx->kv_format != ETS_KV_FP8_E4M3) return ETS_ERR_INVALID_ARG;
    const int n = ctx->shape.n_kv_heads;
    if (n > kMaxScaledHeads) return ETS_ERR_UNSUPPORTED;
    for (int h = 0; h < n; ++h)
        if (!(k_scales[h] > 0.f) || !(v_scales[h] > 0.f) || !std::isfinite(k_scales[h]) ||
            !std::isfinite(v_scales[h]))
            return ETS_ERR_INVALID_ARG;
    for (int h = 0; h < n; ++h) {
        ctx->k_scales.s[h] = k_scales[h];
        ctx->v_scales.s[h] = v_scales[h];
    }
    return ETS_OK;
}

ets_status ets_plan(ets_ctx* ctx, const ets_tree* tree, int mode) {
    if (!ctx || !tree) return ETS_ERR_INVALID_ARG;
    ets_status s = build_plan(ctx->shape, ctx->opt, *tree, mode, ctx->plan);
    if (s != ETS_OK) return s;
    if (ctx->device >= 0) {
        s = upload_plan(ctx);
        if (s != ETS_OK) ctx->plan.valid = false;
    }
    return s;
}

ets_status ets_plan_advance(ets_ctx* ctx, void* hip_stream, int32_t* replanned) {
    if (!ctx) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    if (replanned) *replanned = 0;
    Plan& p = ctx->plan;
    const int advances_before = p.advances;
    if (advance_in_place(p)) {
        if (ctx->device >= 0 && !p.adv.empty()) {
            DeviceGuard guard(ctx->device);
            if (!guard.ok) return ETS_ERR_HIP;
            hipStream_t stream = static_cast<hipStream_t>(hip_stream);
            const int n = (int)p.adv.size();
            hipLaunchKernelGGL(advance_runs_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                               stream, ctx->d_runs, ctx->d_adv, n, (int)p.piece, advances_before);
            const int n_slots = (int)p.adv_slots.size();
            if (n_slots > 0)
                hipLaunchKernelGGL(refresh_units_kernel, dim3((unsigned)((n_slots + 255) / 256)),
                                   dim3(256), 0, stream, ctx->d_units, ctx->d_adv_slots, n_slots,
                                   ctx->d_runs);
            if (hipGetLastError() != hipSuccess) return ETS_ERR_HIP;
            ctx->last_stream = stream;
            ctx->stream_used = true;
        }
        return ETS_OK;
    }
    // no room left in the step lists: plan again from the grown copy of the tree
    try {
        advance_tree(p);
        const std::vector<int32_t> parent = p.parent, n_tokens = p.n_tokens, leaf_node = p.leaf_node;
        const std::vector<int64_t> tok_offset = p.tok_offset;
        const ets_tree t{(int32_t)parent.size(), parent.data(),        tok_offset.data(),
                         n_tokens.data(),        (int32_t)leaf_node.size(), leaf_node.data()};
        ets_status s = build_plan(ctx->shape, ctx->opt, t, p.mode, p);
        if (s != ETS_OK) return s;
        if (ctx->device >= 0) {
            s = upload_plan(ctx);
            if (s != ETS_OK) {
                p.valid = false;
                return s;
            }
        }
    } catch (const std::bad_alloc&) {
        p.valid = false;
        return ETS_ERR_NOMEM;
    }
    if (replanned) *replanned = 1;
    return ETS_OK;
}

ets_status ets_kv_append(ets_ctx* ctx, void* k_pool, void* v_pool, int64_t pool_tokens,
                         const void* k_new, const void* v_new, void* hip_stream) {
    if (!ctx) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    if (ctx->device < 0) return ETS_ERR_HIP;
    const Plan& p = ctx->plan;
    const int n = (int)p.adv_node.size();
    if (n == 0) return ETS_OK;
    if (!k_pool || !v_pool || !k_new || !v_new) return ETS_ERR_INVALID_ARG;
    // the newest row of every growing node has to exist in the pool
    int64_t last_row = -1;
    for (const int64_t r0 : p.adv_last_row) last_row = std::max(last_row, r0 + p.advances);
    if (last_row >= pool_tokens) return ETS_ERR_INVALID_ARG;
    if (last_row < 0) return ETS_OK;  // no growing node has a row
    const int64_t esz =
        ctx->kv_format == ETS_KV_FP8_E4M3 ? 1 : ctx->shape.dtype == ETS_F32 ? 4 : 2;
    const int head_bytes = (int)(ctx->shape.head_dim * esz);
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ETS_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)n), dim3(256), 0, stream,
                       static_cast<char*>(k_pool), static_cast<char*>(v_pool),
                       static_cast<const char*>(k_new), static_cast<const char*>(v_new),
                       ctx->d_adv_src, ctx->d_adv_last_row, (int)p.advances, ctx->shape.n_kv_heads,
                       head_bytes, pool_tokens);
    if (hipGetLastError() != hipSuccess) return ETS_ERR_HIP;
    ctx->last_stream = stream;
    ctx->stream_used = true;
    return ETS_OK;
}

ets_status ets_plan_check(const ets_ctx* ctx, ets_plan_check_report* report) {
    if (!ctx) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid && !ctx->prefill.valid) return ETS_ERR_NO_PLAN;
    ets_plan_check_report rep{};
    rep.max_entry_index = rep.max_pool_row = rep.max_partial_row = -1;
    bool ok = true;
    if (ctx->plan.valid) {
        PlanCheck c;
        ok = check_plan(ctx->plan, ctx->shape, c) && ok;
        rep.decode_items = c.items;
        rep.entry_table_entries = c.entry_table_entries;
        rep.max_entry_index = c.max_entry_index;
        rep.max_entry_overreach = c.max_entry_overreach;
        rep.max_pool_row = c.max_pool_row;
        rep.max_partial_row = c.max_partial_row;
        rep.violations += c.violations;
    }
    if (ctx->prefill.valid) {
        PlanCheck c;
        ok = check_prefill_plan(ctx->prefill, ctx->shape, c) && ok;
        rep.prefill_items = c.items;
        rep.max_pool_row = std::max(rep.max_pool_row, c.max_pool_row);
        rep.violations += c.violations;
    }
    if (report) *report = rep;
    return ok ? ETS_OK : ETS_ERR_BAD_TREE;
}

ets_status ets_plan_append_rows(const ets_ctx* ctx, int64_t* rows) {
    if (!ctx || !rows) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    const Plan& p = ctx->plan;
    for (int64_t l = 0; l < p.stats.n_leaves; ++l) rows[l] = -1;
    for (size_t i = 0; i < p.adv_node.size(); ++i) {
        const int64_t row = p.adv_last_row[i] + p.advances;
        rows[p.adv_src[i]] = row < 0 ? -1 : row;
    }
    return ETS_OK;
}

ets_status ets_plan_stats(const ets_ctx* ctx, ets_stats* out) {
    if (!ctx || !out) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    *out = ctx->plan.stats;
    return ETS_OK;
}

ets_status ets_plan_paths(const ets_ctx* ctx, int64_t* path_ptr, int32_t* path_nodes, int64_t cap,
                          int64_t* n_path_nodes) {
    if (!ctx || !path_ptr || cap < 0 || (cap > 0 && !path_nodes)) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    const Plan& p = ctx->plan;
    const int32_t L = (int32_t)p.stats.n_leaves;
    try {
        std::vector<int32_t> all;
        std::vector<int64_t> ptr((size_t)L + 1, 0);
        for (int32_t l = 0; l < L; ++l) {
            chain_of(p, l, all);
            ptr[l + 1] = (int64_t)all.size();
        }
        if (n_path_nodes) *n_path_nodes = (int64_t)all.size();
        if ((int64_t)all.size() > cap) return ETS_ERR_INVALID_ARG;
        std::memcpy(path_ptr, ptr.data(), ptr.size() * sizeof(int64_t));
        if (!all.empty()) std::memcpy(path_nodes, all.data(), all.size() * sizeof(int32_t));
    } catch (const std::bad_alloc&) {
        return ETS_ERR_NOMEM;
    }
    return ETS_OK;
}

ets_status ets_plan_leaf_counts(const ets_ctx* ctx, int64_t* leaf_count) {
    if (!ctx || !leaf_count) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    const Plan& p = ctx->plan;
    if (!p.leaf_count.empty())
        std::memcpy(leaf_count, p.leaf_count.data(), p.leaf_count.size() * sizeof(int64_t));
    return ETS_OK;
}

ets_status ets_plan_leaf_cover(const ets_ctx* ctx, int32_t leaf, int64_t* rows, int64_t cap,
                               int64_t* n_rows, int32_t* n_partials) {
    if (!ctx || cap < 0 || (cap > 0 && !rows)) return ETS_ERR_INVALID_ARG;
    if (!ctx->plan.valid) return ETS_ERR_NO_PLAN;
    if (leaf < 0 || leaf >= ctx->plan.stats.n_leaves) return ETS_ERR_BAD_LEAF;
    try {
        std::vector<int64_t> r;
        int32_t np = 0;
        const bool ok = leaf_cover(ctx->plan, leaf, r, np);
        if (n_rows) *n_rows = (int64_t)r.size();
        if (n_partials) *n_partials = np;
        if (!ok) return ETS_ERR_BAD_TREE;
        if ((int64_t)r.size() > cap) return ETS_ERR_INVALID_ARG;
        if (!r.empty()) std::memcpy(rows, r.data(), r.size() * sizeof(int64_t));
    } catch (const std::bad_alloc&) {
        return ETS_ERR_NOMEM;
    }
    return ETS_OK;
}

ets_status ets_tree_decode_attn(ets_ctx* ctx, const void* k_pool, const void* v_pool,
                                int64_t pool_tokens, const void* q, void* out, float* lse,
                                void* workspace, int64_t workspace_bytes, void* hip_stream) {
    return decode_call(ctx, k_pool, v_pool, pool_tokens, q, out, lse, workspace, workspace_bytes,
                       hip_stream, true);
}

ets_status ets_tree_decode_attn_static(ets_ctx* ctx, const void* k_pool, const void* v_pool,
                                       int64_t pool_tokens, const void* q, void* out, float* lse,
                                       void* hip_stream) {
    if (!ctx) return ETS_ERR_INVALID_ARG;
    if (ctx->device < 0) return ETS_ERR_HIP;
    // ctx->static_scratch is the device address found at ets_create, never the symbol itself
    return decode_call(ctx, k_pool, v_pool, pool_tokens, q, out, lse, ctx->static_scratch,
                       ETS_STATIC_SCRATCH_BYTES, hip_stream, false);
}

ets_status ets_plan_prefill(ets_ctx* ctx, const ets_tree* tree) {
    if (!ctx || !tree) return ETS_ERR_INVALID_ARG;
    if (ctx->shape.dtype != ETS_BF16 || ctx->shape.head_dim != 128) return ETS_ERR_UNSUPPORTED;
    ets_status s = build_prefill_plan(ctx->shape, *tree, ctx->prefill,
                                      ctx->kv_format == ETS_KV_FP8_E4M3 ? 1 : 2);
    if (s != ETS_OK) return s;
    if (ctx->device >= 0) {
        s = upload_prefill_plan(ctx);
        if (s != ETS_OK) ctx->prefill.valid = false;
    }
    return s;
}

ets_status ets_prefill_plan_stats(const ets_ctx* ctx, ets_prefill_stats* out) {
    if (!ctx || !out) return ETS_ERR_INVALID_ARG;
    if (!ctx->prefill.valid) return ETS_ERR_NO_PLAN;
    *out = ctx->prefill.stats;
    return ETS_OK;
}

ets_status ets_prefill_q_ptr(const ets_ctx* ctx, int64_t* q_ptr) {
    if (!ctx || !q_ptr) return ETS_ERR_INVALID_ARG;
    if (!ctx->prefill.valid) return ETS_ERR_NO_PLAN;
    std::memcpy(q_ptr, ctx->prefill.q_ptr.data(), ctx->prefill.q_ptr.size() * sizeof(int64_t));
    return ETS_OK;
}

ets_status ets_prefill_cover(const ets_ctx* ctx, int32_t leaf, int32_t tok, int64_t* rows,
                             int64_t cap, int64_t* n_rows) {
    if (!ctx || cap < 0 || (cap > 0 && !rows)) return ETS_ERR_INVALID_ARG;
    if (!ctx->prefill.valid) return ETS_ERR_NO_PLAN;
    const PrefillPlan& p = ctx->prefill;
    if (leaf < 0 || leaf >= p.stats.n_leaves) return ETS_ERR_BAD_LEAF;
    if (tok < 0 || tok >= p.n_tokens[p.leaf_node[leaf]]) return ETS_ERR_INVALID_ARG;
    try {
        std::vector<int64_t> r;
        const bool ok = prefill_cover(p, leaf, tok, r);
        if (n_rows) *n_rows = (int64_t)r.size();
        if (!ok) return ETS_ERR_BAD_TREE;
        if ((int64_t)r.size() > cap) return ETS_ERR_INVALID_ARG;
        if (!r.empty()) std::memcpy(rows, r.data(), r.size() * sizeof(int64_t));
    } catch (const std::bad_alloc&) {
        return ETS_ERR_NOMEM;
    }
    return ETS_OK;
}

ets_status ets_tree_prefill_attn(ets_ctx* ctx, const void* k_pool, const void* v_pool,
                                 int64_t pool_tokens, const void* q, float* out, float* lse,
                                 void* hip_stream) {
    if (!ctx) return ETS_ERR_INVALID_ARG;
    if (!ctx->prefill.valid) return ETS_ERR_NO_PLAN;
    if (ctx->device < 0) return ETS_ERR_HIP;
    const ets_prefill_stats& st = ctx->prefill.stats;
    if (st.n_q_rows == 0) return ETS_OK;
    if (!q || !out || !lse || !k_pool || !v_pool || pool_tokens < 0) return ETS_ERR_INVALID_ARG;
    if (pool_tokens < st.min_pool_tokens) return ETS_ERR_BAD_TREE;
    if (misaligned(k_pool) || misaligned(v_pool) || misaligned(q) || misaligned(out) ||
        (reinterpret_cast<uintptr_t>(lse) & 3u))
        return ETS_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ETS_ERR_HIP;
    const int g = ctx->shape.n_q_heads / ctx->shape.n_kv_heads;
    const int g_shift = g == 1 ? 0 : g == 2 ? 1 : g == 4 ? 2 : 3;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    // grid: x = kv head, y = item, at most 65535 items per launch
    for (int64_t y0 = 0; y0 < st.n_items; y0 += 65535) {
        const unsigned ny = (unsigned)std::min<int64_t>(65535, st.n_items - y0);
        if (ctx->kv_format == ETS_KV_FP8_E4M3)
            hipLaunchKernelGGL((prefill_attn_kernel<true, false>), dim3((unsigned)ctx->shape.n_kv_heads, ny),
                               dim3(512), 0, stream, k_pool, v_pool, pool_tokens,
                               static_cast<const bf16_t*>(q), ctx->d_pre_runs, ctx->d_pre_items,
                               (int)y0, g_shift, ctx->scale * 1.4426950408889634f, ctx->k_scales,
                               ctx->v_scales, out, lse, nullptr, nullptr, nullptr);
        else
            hipLaunchKernelGGL((prefill_attn_kernel<false, false>), dim3((unsigned)ctx->shape.n_kv_heads, ny),
                               dim3(512), 0, stream, k_pool, v_pool, pool_tokens,
                               static_cast<const bf16_t*>(q), ctx->d_pre_runs, ctx->d_pre_items,
                               (int)y0, g_shift, ctx->scale * 1.4426950408889634f, ctx->k_scales,
                               ctx->v_scales, out, lse, nullptr, nullptr, nullptr);
    }
    ctx->last_stream = stream;
    ctx->stream_used = true;
    if (hipGetLastError() != hipSuccess) return ETS_ERR_HIP;
    return ETS_OK;
}

ets_status ets_rebase_weights(int32_t n, const double* rewards, int32_t budget,
                              double temperature, int32_t* weights) {
    if (n < 0 || budget < 0 || !(temperature > 0.0)) return ETS_ERR_INVALID_ARG;
    if (n > 0 && (!rewards || !weights)) return ETS_ERR_INVALID_ARG;
    try {
        rebase_weights(n, rewards, budget, temperature, weights);
    } catch (const std::bad_alloc&) {
        return ETS_ERR_NOMEM;
    }
    return ETS_OK;
}

ets_status ets_select_leaves(const ets_tree* tree, const int32_t* weights, const int32_t* cluster,
                             double lambda_b, double lambda_d, int64_t node_limit, uint8_t* keep,
                             ets_select_info* info) {
    if (!tree || !keep) return ETS_ERR_INVALID_ARG;
    SelectResult r;
    const ets_status s = select_leaves(*tree, weights, cluster, lambda_b, lambda_d, node_limit, r);
    if (s != ETS_OK) return s;
    std::memcpy(keep, r.keep.data(), r.keep.size());
    if (info) {
        info->objective = r.objective;
        info->kept_nodes = r.kept_nodes;
        info->live_nodes = r.live_nodes;
        info->kept_clusters = r.kept_clusters;
        info->clusters = r.clusters;
        info->bb_nodes = r.bb_nodes;
        info->optimal = r.optimal ? 1 : 0;
        info->pad = 0;
    }
    return ETS_OK;
}

ets_status ets_bench_read_stream(int hip_device, const void* buf, int64_t bytes, int nontemporal,
                                 void* sink, int64_t sink_bytes, void* hip_stream) {
    if (hip_device < 0 || !buf || !sink || bytes < 0 || misaligned(buf) ||
        (reinterpret_cast<uintptr_t>(sink) & 3u))
        return ETS_ERR_INVALID_ARG;
    DeviceGuard guard(hip_device);
    if (!guard.ok) return ETS_ERR_HIP;
    // enough workgroups to fill every compute unit several times over, each with many spans
    const int64_t spans = bytes / 16 / (256 * 8);
    const int64_t grid = std::max<int64_t>(1, std::min<int64_t>(spans, 256 * 16));
    if (sink_bytes < grid * 4) return ETS_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    if (nontemporal)
        hipLaunchKernelGGL(read_stream_kernel<true>, dim3((unsigned)grid), dim3(256), 0, stream,
                           static_cast<const bench_u32x4_t*>(buf), bytes / 16,
                           static_cast<uint32_t*>(sink));
    else
        hipLaunchKernelGGL(read_stream_kernel<false>, dim3((unsigned)grid), dim3(256), 0, stream,
                           static_cast<const bench_u32x4_t*>(buf), bytes / 16,
                           static_cast<uint32_t*>(sink));
    if (hipGetLastError() != hipSuccess) return ETS_ERR_HIP;
    return ETS_OK;
}

ets_status ets_profile_read(ets_ctx* ctx, ets_profile* out) {
    if (!ctx || !out) return ETS_ERR_INVALID_ARG;
    *out = ets_profile{};
    if (ctx->device < 0) return ETS_ERR_HIP;
    if (ctx->calls_recorded == 0) return ETS_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ETS_ERR_HIP;
    const size_t n = ctx->calls_recorded;
    ctx->calls_recorded = 0;
    if (hipEventSynchronize(ctx->events[n * 5 - 1]) != hipSuccess) return ETS_ERR_HIP;
    for (size_t i = 0; i < n; ++i) {
        float ms[4] = {0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < 4; ++k)
            if (hipEventElapsedTime(&ms[k], ctx->events[i * 5 + k], ctx->events[i * 5 + k + 1]) !=
                hipSuccess) {
                (void)hipGetLastError();
                return ETS_ERR_HIP;
            }
        out->stream_ms += ms[0];
        out->wide_ms += ms[1];
        out->cascade_ms += ms[2];
        out->merge_ms += ms[3];
    }
    out->calls = (int64_t)n;
    return ETS_OK;
}

const char* ets_strerror(int status) {
    switch (status) {
        case ETS_OK: return "ok";
        case ETS_ERR_INVALID_ARG: return "invalid argument";
        case ETS_ERR_BAD_TREE: return "malformed tree";
        case ETS_ERR_BAD_LEAF: return "leaf node id out of range";
        case ETS_ERR_UNSUPPORTED: return "unsupported shape";
        case ETS_ERR_WORKSPACE: return "workspace too small";
        case ETS_ERR_NO_PLAN: return "no plan";
        case ETS_ERR_HIP: return "HIP runtime error or host-only context";
        case ETS_ERR_NOMEM: return "out of host memory";
        default: return "unknown status";
    }
}

}  // extern "C"
