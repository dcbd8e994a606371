// C ABI of kvprefetch: argument validation, error reporting, partition planning and
// kernel dispatch.  Host code only; the kernels live in the other sources.
#include "../../include/kvprefetch.h"
#include "attn_device.h"

#include <cmath>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <vector>

// Split-KV scratch of kv_decode_attn_noalloc: a fixed array in the library's own device image instead of memory
// somebody allocated.  Every device the library runs on holds its own copy at its own address for the life of the
// process; the name below is a host-side handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[KV_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// Per-device state, under g_state_mutex.  The registered workspace is handed out in slices, one per stream that
// has called: calls on one stream run in stream order and may share a slice, calls on different streams may
// overlap in time and must not.  A slice is carved from the end of what is in use the first time a stream calls
// (or when it needs more than it has; its old slice is then abandoned until the workspace is registered again),
// so a call finds its slice with a short search and nothing is ever waited for.  Each slot also owns the side
// stream and the two events of the layer stack's cross-layer touch, created when first needed.
struct StreamSlot {
    hipStream_t stream = nullptr;
    size_t offset = 0, bytes = 0;
    hipStream_t side = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
};
struct DeviceState {
    void* ws_ptr = nullptr;
    size_t ws_bytes = 0, ws_used = 0;
    std::vector<StreamSlot> slots;
    void* scratch_ptr = nullptr;        // device address of g_static_scratch on this device, once resolved
};
std::mutex g_state_mutex;
DeviceState g_dev[kvp::kMaxDevices];
void* g_trace_ptr = nullptr;         // optional per-worker timestamps (under g_state_mutex)
size_t g_trace_bytes = 0;
std::atomic<int> g_waves_per_cu{0};  // 0 = automatic
std::atomic<int> g_variant{KV_VARIANT_ONE_PASS};   // kernel form of kv_decode_attn on 16-bit caches
std::atomic<int> g_l2_touch{0};      // tiles per group of the L2 touch wave (0 = none); calls with prefetch_distance 0 only
std::atomic<int> g_plain_fetch{0};   // comparison mode: KV fetches and dense-layer weight loads without the non-temporal hint
std::atomic<int> g_xcd_skew{10};     // per 1024: even workers get 1024 + 10 parts of the tile space, odd ones 1024 - 10
using kvp::kMaxDevices;
std::atomic<int> g_num_cus[kMaxDevices];   // compute units per device ordinal, read once each (0 = not read yet)

constexpr int kLdsBytesPerCU = 160 * 1024;
constexpr int kMaxWavesPerCU = 16;

int num_cus() {     // of the current device
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    int n = g_num_cus[dev].load();
    if (n > 0) return n;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return -1;
    n = prop.multiProcessorCount;
    g_num_cus[dev].store(n);
    return n;
}

// Persistent waves per compute unit of the attention kernel: what the caller asked for, else a count chosen
// for the bytes it puts in flight.  The kernel runs fastest with about 32-48 KB of KV requested per compute
// unit at any time; beyond that throughput falls again (measured: 64-96 KB in flight costs 4-8 %).  A wave
// keeps max(1, distance) tile pairs of 8 KB (head_dim 128) or 4 KB (head_dim 64) in flight, so deep look-ahead
// wants few waves and no look-ahead wants many; head_dim 64 needs at least four waves to keep up with the
// arithmetic of its smaller tiles.  An 8-bit cache has tile pairs of the same bytes (32 tokens) and twice the
// arithmetic per byte: two waves cannot keep up (115 us on the Llama-3-8B-shaped batch), three with a look-ahead of
// one can (85 us, and a merge over 768 workers: step 90.5 us), six without look-ahead come close (87 us, step
// 96 us with the merge over 1536 workers); head_dim 64: eight waves at every distance (step 55.0 us at distance
// 1, 58.1 at 0; twelve at distance 0: 66.6).  Above four, an odd count (uneven over the four SIMDs) is 40 % slower
// than the even count below it.  The two-phase variant moves one tile per step where the one-pass kernel moves a pair, so it wants
// twice the waves for the same bytes in flight (measured best: 12 / 6 / 4 at distance 0 / 1 / 2).  Always capped
// by the LDS the rings (and the two-phase variant's logits buffer) need.
int waves_per_cu(int prefetch_distance, int d, bool kv8, int two_phase_group = 0) {
    const int lds_limit = kLdsBytesPerCU / (two_phase_group ? kvp::twophase_worker_lds_bytes(prefetch_distance, d, two_phase_group)
                                            : kv8         ? kvp::kv8_worker_lds_bytes(prefetch_distance, d)
                                                            : kvp::mfma_worker_lds_bytes(prefetch_distance, d));
    int w = g_waves_per_cu.load();
    if (w <= 0) {
        if (two_phase_group) w = prefetch_distance == 0 ? 12 : prefetch_distance == 1 ? 6 : 4;
        else if (kv8) w = d == 128 ? (prefetch_distance == 0 ? 6 : 3) : 8;
        else if (d == 128) w = prefetch_distance <= 1 ? 6 : 2;
        else w = prefetch_distance <= 1 ? 8 : 4;
    }
    const bool automatic = g_waves_per_cu.load() <= 0;
    w = w < lds_limit ? w : lds_limit;
    w = w < kMaxWavesPerCU ? w : kMaxWavesPerCU;
    if (kv8 && automatic && w > 4 && (w & 1)) --w;     // above four an odd count is uneven over the four SIMDs (measured 40 % slower)
    return w;
}

// Workspace layout: the dense layer's ticket words, the attention partials (two pieces of G rows per worker,
// sized for the largest launch), then the dense layer's partial tiles (layer stack with weights in operand
// order only).
size_t attn_partial_region(int Hq, int d) {
    return kvp::mfma_partial_bytes(kvp::kMaxMfmaWorkers, Hq < 16 ? Hq : 16, d);
}
size_t workspace_bytes(int Hq, int d) {
    return kvp::kGemmTicketBytes + attn_partial_region(Hq, d);
}

bool dense_tile(const kv_tensor* t) {   // [NBLK, Hkv, bs, d] with the [bs, d] tile contiguous
    return t->stride[3] == 1 && t->stride[2] == t->shape[3];
}

struct Resolved {
    kvp::AttnParams p;
    int elem, d, bs;
    bool kv8, two_phase;
    size_t partial_bytes;       // split-KV scratch the launch writes and the merge kernel reads
};

int resolve(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
            const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
            float scale, int num_kv_heads, int block_size, int prefetch_distance, Resolved* r,
            bool kv8 = false, float k_scale = 1.0f, float v_scale = 1.0f) {
    if (!q || !k_cache || !v_cache || !block_tables || !context_lens || !out)
        return fail(KV_ERR_INVALID, "kv_decode_attn: null tensor descriptor");
    if (!q->data || !k_cache->data || !v_cache->data || !block_tables->data || !context_lens->data || !out->data)
        return fail(KV_ERR_INVALID, "kv_decode_attn: null data pointer");
    if (q->ndim != 3 || out->ndim != 3 || k_cache->ndim != 4 || v_cache->ndim != 4 ||
        block_tables->ndim != 2 || context_lens->ndim != 1)
        return fail(KV_ERR_INVALID, "kv_decode_attn: wrong rank (q,out 3; caches 4; block_tables 2; context_lens 1)");
    if (q->dtype != KV_F16 && q->dtype != KV_BF16)
        return fail(KV_ERR_UNSUPPORTED, "kv_decode_attn: q dtype %d is not f16/bf16", q->dtype);
    if (kv8) {
        if (k_cache->dtype != KV_FP8_E4M3 || v_cache->dtype != KV_FP8_E4M3 || out->dtype != q->dtype)
            return fail(KV_ERR_INVALID, "kv_decode_attn_kv8: caches must be FP8 E4M3, out of q's dtype");
        if (!(k_scale > 0.0f) || !(v_scale > 0.0f) || !std::isfinite(k_scale) || !std::isfinite(v_scale))
            return fail(KV_ERR_INVALID, "kv_decode_attn_kv8: k_scale and v_scale must be positive and finite");
    } else if (k_cache->dtype != q->dtype || v_cache->dtype != q->dtype || out->dtype != q->dtype) {
        return fail(KV_ERR_INVALID, "kv_decode_attn: q, k_cache, v_cache and out must share one dtype");
    }
    if (block_tables->dtype != KV_I32 || context_lens->dtype != KV_I32)
        return fail(KV_ERR_INVALID, "kv_decode_attn: block_tables and context_lens must be int32");
    const int64_t B = q->shape[0], Hq = q->shape[1], d = q->shape[2];
    if (B <= 0 || Hq <= 0) return fail(KV_ERR_INVALID, "kv_decode_attn: empty batch or head count");
    if (B > 65535) return fail(KV_ERR_UNSUPPORTED, "kv_decode_attn: batch %lld exceeds 65535", (long long)B);
    if (num_kv_heads <= 0 || Hq % num_kv_heads != 0)
        return fail(KV_ERR_INVALID, "kv_decode_attn: %lld query heads not divisible by %d kv heads", (long long)Hq, num_kv_heads);
    if (out->shape[0] != B || out->shape[1] != Hq || out->shape[2] != d)
        return fail(KV_ERR_INVALID, "kv_decode_attn: out shape differs from q");
    for (int i = 0; i < 4; ++i)
        if (k_cache->shape[i] != v_cache->shape[i])
            return fail(KV_ERR_INVALID, "kv_decode_attn: k_cache and v_cache shapes differ");
    if (k_cache->shape[1] != num_kv_heads || k_cache->shape[2] != block_size || k_cache->shape[3] != d)
        return fail(KV_ERR_INVALID, "kv_decode_attn: cache shape [%lld,%lld,%lld,%lld] does not match num_kv_heads %d, block_size %d, head_dim %lld",
                    (long long)k_cache->shape[0], (long long)k_cache->shape[1], (long long)k_cache->shape[2],
                    (long long)k_cache->shape[3], num_kv_heads, block_size, (long long)d);
    if (k_cache->shape[0] <= 0 || k_cache->shape[0] > INT32_MAX)
        return fail(KV_ERR_INVALID, "kv_decode_attn: cache must hold between 1 and 2^31-1 blocks");
    if (block_tables->shape[0] != B || context_lens->shape[0] != B)
        return fail(KV_ERR_INVALID, "kv_decode_attn: block_tables / context_lens batch differs from q");
    if (block_tables->shape[1] <= 0 || block_tables->shape[1] > (1 << 24))
        return fail(KV_ERR_INVALID, "kv_decode_attn: block table width out of range");
    if (q->stride[1] < 0 || q->stride[1] * 2 * 15 + 512 > INT32_MAX)
        return fail(KV_ERR_UNSUPPORTED, "kv_decode_attn: query head stride %lld out of range", (long long)q->stride[1]);
    if (q->stride[2] != 1 || out->stride[2] != 1 || block_tables->stride[1] != 1 || context_lens->stride[0] != 1)
        return fail(KV_ERR_INVALID, "kv_decode_attn: innermost stride must be 1");
    if (!dense_tile(k_cache) || !dense_tile(v_cache))
        return fail(KV_ERR_INVALID, "kv_decode_attn: the [block_size, head_dim] tile of a cache block must be dense");
    if (d != 64 && d != 128) return fail(KV_ERR_UNSUPPORTED, "kv_decode_attn: head_dim %lld not in {64,128}", (long long)d);
    if (block_size != 16 && block_size != 32)
        return fail(KV_ERR_UNSUPPORTED, "kv_decode_attn: block_size %d not in {16,32}", block_size);
    const int G = (int)(Hq / num_kv_heads);
    if (G > 16) return fail(KV_ERR_UNSUPPORTED, "kv_decode_attn: %d query heads per kv head exceeds 16", G);
    // KV_PREFETCH_AUTO: the distance measured best for the cache type, at the occupancy that goes with it (16-bit
    // caches: two tiles ahead with two waves per compute unit; 8-bit caches: one tile ahead with three, eight at
    // head_dim 64: see waves_per_cu)
    if (prefetch_distance == KV_PREFETCH_AUTO) prefetch_distance = kv8 ? 1 : 2;
    if (prefetch_distance < 0 || prefetch_distance > KV_MAX_PREFETCH_DISTANCE)
        return fail(KV_ERR_INVALID, "kv_decode_attn: prefetch_distance %d outside 0..%d (or KV_PREFETCH_AUTO)", prefetch_distance, KV_MAX_PREFETCH_DISTANCE);
    // 128-bit loads need 16-byte aligned rows
    auto aligned = [](const kv_tensor* t, int nstr, int elems_per_16_bytes) {
        if (((uintptr_t)t->data) % 16) return false;
        for (int i = 0; i < nstr; ++i) if (t->stride[i] % elems_per_16_bytes) return false;
        return true;
    };
    const int cache_elems = kv8 ? 16 : 8;
    if (!aligned(q, 2, 8) || !aligned(k_cache, 2, cache_elems) || !aligned(v_cache, 2, cache_elems) || !aligned(out, 2, 8))
        return fail(KV_ERR_INVALID, "kv_decode_attn: data pointers and outer strides must be 16-byte aligned");

    const int64_t MB = block_tables->shape[1];
    kvp::AttnParams& p = r->p;
    p.q = q->data; p.k_cache = k_cache->data; p.v_cache = v_cache->data;
    p.block_tables = (const int32_t*)block_tables->data;
    p.context_lens = (const int32_t*)context_lens->data;
    p.out = out->data;
    p.q_stride_b = q->stride[0]; p.q_stride_h = q->stride[1];
    p.kv_stride_blk = k_cache->stride[0]; p.kv_stride_h = k_cache->stride[1];
    p.v_stride_blk = v_cache->stride[0]; p.v_stride_h = v_cache->stride[1];
    p.out_stride_b = out->stride[0]; p.out_stride_h = out->stride[1];
    p.bt_stride_b = block_tables->stride[0];
    p.B = (int)B; p.Hq = (int)Hq; p.Hkv = num_kv_heads; p.G = G;
    p.MB = (int)MB; p.NBLK = (int)k_cache->shape[0];
    p.prefetch_distance = prefetch_distance;
    p.tile_shift = kv8 ? 5 : 4;
    p.scale_log2e = scale * kvp::kLog2e * (kv8 ? k_scale : 1.0f);
    p.out_scale = kv8 ? v_scale : 1.0f;
    r->elem = q->dtype; r->d = (int)d; r->bs = block_size; r->kv8 = kv8;
    r->two_phase = !kv8 && g_variant.load() == KV_VARIANT_TWO_PHASE;
    const int cus = num_cus();
    if (cus <= 0) return fail(KV_ERR_HIP, "kv_decode_attn: cannot read the device's compute unit count");
    const int nw = cus * waves_per_cu(prefetch_distance, (int)d, kv8, r->two_phase ? G : 0);
    p.num_workers = nw < kvp::kMaxMfmaWorkers ? nw : kvp::kMaxMfmaWorkers;
    p.xcd_skew = g_xcd_skew.load();
    p.plain_fetch = (!kv8 && !r->two_phase) ? g_plain_fetch.load() : 0;
    p.rescale_slack = kvp::kRescaleSlack;
    p.l2_touch = (!kv8 && !r->two_phase && prefetch_distance == 0 && !p.plain_fetch) ? g_l2_touch.load() : 0;
    r->partial_bytes = kvp::mfma_partial_bytes(p.num_workers, G, (int)d);
    p.partials = nullptr;           // bound by bind_registered / bind_static
    p.worker_trace = nullptr;
    return KV_OK;
}

int current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

// The slice of the current device's registered workspace that calls on `stream` use, at least `need` bytes.
// Caller holds g_state_mutex.
int acquire_slice(DeviceState& ds, hipStream_t stream, size_t need, const char* who, StreamSlot** out) {
    if (!ds.ws_ptr) return fail(KV_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, none registered on this device", who, need);
    StreamSlot* slot = nullptr;
    for (StreamSlot& sl : ds.slots)
        if (sl.stream == stream) { slot = &sl; break; }
    if (slot && slot->bytes >= need) { *out = slot; return KV_OK; }
    if (slot && slot->bytes > 0 && slot->offset + slot->bytes == ds.ws_used && slot->offset + need <= ds.ws_bytes) {
        slot->bytes = need;                 // the slice at the end of what is in use grows in place
        ds.ws_used = slot->offset + need;
        *out = slot;
        return KV_OK;
    }
    const size_t offset = (ds.ws_used + 255) & ~(size_t)255;
    if (offset + need > ds.ws_bytes)
        return fail(KV_ERR_WORKSPACE, "%s: workspace of %zu bytes needed for this stream, %zu registered of which %zu are in use "
                    "by %zu stream(s); register a larger one (registering again also releases every stream's slice)",
                    who, need, ds.ws_bytes, ds.ws_used, ds.slots.size());
    if (!slot) {
        ds.slots.emplace_back();
        slot = &ds.slots.back();
        slot->stream = stream;
    }
    slot->offset = offset;
    slot->bytes = need;
    ds.ws_used = offset + need;
    *out = slot;
    return KV_OK;
}

// Points a resolved call at the static scratch array of the current device.  The array's address is looked up once
// per device, at the first such call there; afterwards this is a table read.  No allocation on any path.
int bind_static(Resolved& r) {
    const int dev = current_device();
    if (dev < 0) return fail(KV_ERR_HIP, "kv_decode_attn_noalloc: cannot read the current device");
    if (r.partial_bytes > (size_t)KV_NOALLOC_SCRATCH_BYTES)
        return fail(KV_ERR_WORKSPACE, "kv_decode_attn_noalloc: the launch needs %zu bytes of split-KV scratch (%d workers x 2 pieces x %d "
                    "query heads per kv head), the static array holds %zu; use fewer waves per compute unit or kv_decode_attn",
                    r.partial_bytes, r.p.num_workers, r.p.G, (size_t)KV_NOALLOC_SCRATCH_BYTES);
    std::lock_guard<std::mutex> lock(g_state_mutex);
    DeviceState& ds = g_dev[dev];
    if (!ds.scratch_ptr) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(KV_ERR_HIP, "kv_decode_attn_noalloc: address of the static scratch array: %s", hipGetErrorString(e));
        ds.scratch_ptr = ptr;
    }
    r.p.partials = (float*)ds.scratch_ptr;
    r.p.worker_trace = nullptr;
    return KV_OK;
}

// Points a resolved call at its stream's slice of the registered workspace: [ticket words][attention partials].
int bind_registered(Resolved& r, hipStream_t stream, const char* who) {
    const int dev = current_device();
    if (dev < 0) return fail(KV_ERR_HIP, "%s: cannot read the current device", who);
    std::lock_guard<std::mutex> lock(g_state_mutex);
    StreamSlot* slot = nullptr;
    if (int rc = acquire_slice(g_dev[dev], stream, kvp::kGemmTicketBytes + r.partial_bytes, who, &slot)) return rc;
    r.p.partials = (float*)((unsigned char*)g_dev[dev].ws_ptr + slot->offset + kvp::kGemmTicketBytes);
    r.p.worker_trace = g_trace_bytes >= (size_t)r.p.num_workers * 32 ? (unsigned long long*)g_trace_ptr : nullptr;
    return KV_OK;
}

// Optional per-call timing: two events per call, one on each side of the main attention kernel, recorded on
// the call's stream (the merge kernel that follows is outside the bracket).
std::mutex g_prof_mutex;
std::vector<hipEvent_t> g_prof_events;
int g_prof_capacity = 0, g_prof_calls = 0, g_prof_every = 1, g_prof_seen = 0;

hipEvent_t prof_event(int call, int which) { return g_prof_events[(size_t)call * 2 + which]; }

constexpr int kTouchTiles = 4;          // leading 16-token tiles of every worker's range that the cross-layer touch reads

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KV_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return KV_OK;
}

int run_attn(const Resolved& r, hipStream_t stream) {
    std::unique_lock<std::mutex> prof_lock(g_prof_mutex);
    int slot = -1;
    if (g_prof_capacity > 0 && g_prof_calls < g_prof_capacity && (g_prof_seen++ % g_prof_every) == 0) slot = g_prof_calls++;
    prof_lock.unlock();
    if (slot >= 0) (void)hipEventRecord(prof_event(slot, 0), stream);
    const int launched = r.kv8          ? kvp::launch_attn_kv8(r.p, r.elem, r.d, r.bs, stream)
                         : r.two_phase  ? kvp::launch_attn_twophase(r.p, r.elem, r.d, r.bs, stream)
                         : r.p.l2_touch ? kvp::launch_attn_l2_touch(r.p, r.elem, r.d, r.bs, stream)
                                        : kvp::launch_attn_mfma(r.p, r.elem, r.d, r.bs, stream);
    if (launched != 0)
        return fail(KV_ERR_UNSUPPORTED, "kv_decode_attn: no kernel for head_dim %d, block_size %d, group %d%s", r.d, r.bs, r.p.G,
                    r.p.plain_fetch ? " under KV_FETCH_PLAIN (bf16, head_dim 128, distance 0 or 2 only)" : "");
    if (int rc = check_launch("kv_decode_attn main kernel")) return rc;
    if (slot >= 0) (void)hipEventRecord(prof_event(slot, 1), stream);
    kvp::launch_finalize_mfma(r.p, r.elem, r.d, r.bs, stream);
    if (int rc = check_launch("kv_decode_attn merge kernel")) return rc;
    return KV_OK;
}

}  // namespace

extern "C" {

int kv_decode_attn(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                   const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                   float scale, int num_kv_heads, int block_size, int prefetch_distance, void* stream) {
    Resolved r;
    if (int rc = resolve(q, k_cache, v_cache, block_tables, context_lens, out, scale, num_kv_heads,
                         block_size, prefetch_distance, &r))
        return rc;
    if (int rc = bind_registered(r, (hipStream_t)stream, "kv_decode_attn")) return rc;
    return run_attn(r, (hipStream_t)stream);
}

int kv_decode_attn_noalloc(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                           const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                           float scale, int num_kv_heads, int block_size, int prefetch_distance, void* stream) {
    Resolved r;
    if (int rc = resolve(q, k_cache, v_cache, block_tables, context_lens, out, scale, num_kv_heads,
                         block_size, prefetch_distance, &r))
        return rc;
    if (int rc = bind_static(r)) return rc;
    return run_attn(r, (hipStream_t)stream);
}

int kv_decode_fetch_probe(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                          const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                          float scale, int num_kv_heads, int block_size, int prefetch_distance, void* stream) {
    Resolved r;
    if (int rc = resolve(q, k_cache, v_cache, block_tables, context_lens, out, scale, num_kv_heads,
                         block_size, prefetch_distance, &r))
        return rc;
    if (int rc = bind_registered(r, (hipStream_t)stream, "kv_decode_fetch_probe")) return rc;
    std::unique_lock<std::mutex> prof_lock(g_prof_mutex);
    int slot = -1;
    if (g_prof_capacity > 0 && g_prof_calls < g_prof_capacity && (g_prof_seen++ % g_prof_every) == 0) slot = g_prof_calls++;
    prof_lock.unlock();
    r.p.worker_trace = nullptr;
    if (slot >= 0) (void)hipEventRecord(prof_event(slot, 0), (hipStream_t)stream);
    if (kvp::launch_fetch_probe(r.p, r.d, r.bs, (hipStream_t)stream) != 0)
        return fail(KV_ERR_UNSUPPORTED, "kv_decode_fetch_probe: no kernel for head_dim %d, block_size %d", r.d, r.bs);
    if (int rc = check_launch("kv_decode_fetch_probe")) return rc;
    if (slot >= 0) (void)hipEventRecord(prof_event(slot, 1), (hipStream_t)stream);
    return KV_OK;
}

int kv_decode_attn_kv8(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                       const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                       float scale, float k_scale, float v_scale, int num_kv_heads, int block_size,
                       int prefetch_distance, void* stream) {
    Resolved r;
    if (int rc = resolve(q, k_cache, v_cache, block_tables, context_lens, out, scale, num_kv_heads,
                         block_size, prefetch_distance, &r, true, k_scale, v_scale))
        return rc;
    if (int rc = bind_registered(r, (hipStream_t)stream, "kv_decode_attn_kv8")) return rc;
    return run_attn(r, (hipStream_t)stream);
}

int kv_decode_layerstack(int num_layers, const kv_tensor* x, const kv_tensor* const* weights,
                         kv_tensor* gemm_out, const kv_tensor* const* q,
                         const kv_tensor* const* k_caches, const kv_tensor* const* v_caches,
                         const kv_tensor* block_tables, const kv_tensor* context_lens,
                         kv_tensor* const* outs, float scale, int num_kv_heads, int block_size,
                         int prefetch_distance, int cross_layer_prefetch, void* stream) {
    if (num_layers < 1 || num_layers > 4096) return fail(KV_ERR_INVALID, "kv_decode_layerstack: %d layers", num_layers);
    if (!x || !weights || !gemm_out || !k_caches || !v_caches || !outs || !block_tables || !context_lens)
        return fail(KV_ERR_INVALID, "kv_decode_layerstack: null argument");
    if (!x->data || !gemm_out->data) return fail(KV_ERR_INVALID, "kv_decode_layerstack: null data pointer");
    if (x->ndim != 2 || gemm_out->ndim != 2) return fail(KV_ERR_INVALID, "kv_decode_layerstack: x and gemm_out must have rank 2");
    if (x->dtype != KV_BF16 || gemm_out->dtype != KV_BF16)
        return fail(KV_ERR_UNSUPPORTED, "kv_decode_layerstack: x and gemm_out must be bf16");
    if (x->stride[1] != 1 || gemm_out->stride[1] != 1) return fail(KV_ERR_INVALID, "kv_decode_layerstack: innermost stride must be 1");
    const int64_t M = x->shape[0], K = x->shape[1], N = gemm_out->shape[1];
    if (gemm_out->shape[0] != M) return fail(KV_ERR_INVALID, "kv_decode_layerstack: gemm_out rows differ from x");
    if (((uintptr_t)x->data) % 16 || ((uintptr_t)gemm_out->data) % 16 || x->stride[0] % 8 || gemm_out->stride[0] % 8)
        return fail(KV_ERR_INVALID, "kv_decode_layerstack: x and gemm_out rows must be 16-byte aligned");
    for (int l = 0; l < num_layers; ++l) {
        const kv_tensor* w = weights[l];
        if (!w || !w->data || !k_caches[l] || !v_caches[l] || !outs[l] || (q && !q[l]))
            return fail(KV_ERR_INVALID, "kv_decode_layerstack: null tensor in layer %d", l);
        const bool row_major = w->ndim == 2 && w->shape[0] == K && w->shape[1] == N && w->stride[1] == 1 && w->stride[0] % 8 == 0;
        const bool packed = w->ndim == 3 && w->shape[0] * 128 == N && w->shape[1] == K && w->shape[2] == 128 &&
                            w->stride[2] == 1 && w->stride[1] % 8 == 0 && w->stride[0] % 8 == 0;
        // operand order [N/64][K/32][4][64][8], contiguous
        const bool operand = w->ndim == 5 && w->shape[0] * 64 == N && w->shape[1] * 32 == K && w->shape[2] == 4 &&
                             w->shape[3] == 64 && w->shape[4] == 8 && w->stride[4] == 1 && w->stride[3] == 8 &&
                             w->stride[2] == 512 && w->stride[1] == 2048 && w->stride[0] == 2048 * w->shape[1];
        if (w->dtype != KV_BF16 || ((uintptr_t)w->data) % 16 || !(row_major || packed || operand))
            return fail(KV_ERR_INVALID, "kv_decode_layerstack: weights[%d] must be bf16 [%lld, %lld] row-major, [%lld, %lld, 128] tile-packed "
                        "or [%lld, %lld, 4, 64, 8] in operand order",
                        l, (long long)K, (long long)N, (long long)(N / 128), (long long)K, (long long)(N / 64), (long long)(K / 32));
        if (operand && K != 1024 && K != 2048 && K != 4096 && K != 8192)
            return fail(KV_ERR_UNSUPPORTED, "kv_decode_layerstack: weights in operand order need K of 1024, 2048, 4096 or 8192, not %lld",
                        (long long)K);
        if (outs[l]->ndim != 3) return fail(KV_ERR_INVALID, "kv_decode_layerstack: outs[%d] must have rank 3", l);
    }
    const int64_t B = outs[0]->shape[0], Hq = outs[0]->shape[1], d = outs[0]->shape[2];
    if (B != M) return fail(KV_ERR_INVALID, "kv_decode_layerstack: outs batch %lld differs from x rows %lld", (long long)B, (long long)M);
    if (!q && N < Hq * d) return fail(KV_ERR_INVALID, "kv_decode_layerstack: gemm_out has %lld columns, queries need %lld", (long long)N, (long long)(Hq * d));
    if (M > 128 || K % 128 || K < 128 || N % 128 || N < 128)
        return fail(KV_ERR_UNSUPPORTED, "kv_decode_layerstack: GEMM shape [%lld x %lld] . [%lld x %lld] not covered (rows <= 128, K %% 128 == 0, N %% 128 == 0)",
                    (long long)M, (long long)K, (long long)K, (long long)N);
    hipStream_t main_stream = (hipStream_t)stream;

    // queries of layer l: the caller's tensor, or the leading Hq*d columns of the GEMM output viewed [B, Hq, d]
    kv_tensor qview;
    qview.data = gemm_out->data; qview.dtype = KV_BF16; qview.ndim = 3;
    qview.shape[0] = B; qview.shape[1] = Hq; qview.shape[2] = d;
    qview.stride[0] = gemm_out->stride[0]; qview.stride[1] = d; qview.stride[2] = 1;

    // every layer's attention call is checked before anything is enqueued
    std::vector<Resolved> layers((size_t)num_layers);
    size_t attn_bytes = 0;
    for (int l = 0; l < num_layers; ++l) {
        if (int rc = resolve(q ? q[l] : &qview, k_caches[l], v_caches[l], block_tables, context_lens, outs[l], scale,
                             num_kv_heads, block_size, prefetch_distance, &layers[(size_t)l]))
            return rc;
        attn_bytes = layers[(size_t)l].partial_bytes > attn_bytes ? layers[(size_t)l].partial_bytes : attn_bytes;
    }

    // this stream's slice of the workspace: [ticket words][attention partials][partial tiles of the dense layer].
    // With weights in operand order the dense layer splits K over two workgroups per column tile, which meet
    // through the ticket words and the partial tiles.
    bool any_operand = false;
    for (int l = 0; l < num_layers; ++l) any_operand = any_operand || weights[l]->ndim == 5;
    const size_t attn_region = (attn_bytes + 255) & ~(size_t)255;
    const size_t need = kvp::kGemmTicketBytes + attn_region + (any_operand ? kvp::layer_gemm_packed_partial_bytes((int)N) : 0);
    const bool touch = cross_layer_prefetch != 0;
    const int dev = current_device();
    if (dev < 0) return fail(KV_ERR_HIP, "kv_decode_layerstack: cannot read the current device");
    unsigned char* slice = nullptr;
    unsigned long long* trace = nullptr;
    hipStream_t side = nullptr;
    hipEvent_t fork_event = nullptr, join_event = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_state_mutex);
        StreamSlot* slot = nullptr;
        if (int rc = acquire_slice(g_dev[dev], main_stream, need, "kv_decode_layerstack", &slot)) return rc;
        slice = (unsigned char*)g_dev[dev].ws_ptr + slot->offset;
        trace = g_trace_bytes >= (size_t)layers[0].p.num_workers * 32 ? (unsigned long long*)g_trace_ptr : nullptr;
        if (touch && !slot->side) {        // side stream (default priority) and the fork / join events of this stream's calls
            hipError_t e = hipStreamCreateWithFlags(&slot->side, hipStreamNonBlocking);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&slot->fork, hipEventDisableTiming);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&slot->join, hipEventDisableTiming);
            if (e != hipSuccess) {
                if (slot->side) (void)hipStreamDestroy(slot->side);
                if (slot->fork) (void)hipEventDestroy(slot->fork);
                slot->side = nullptr; slot->fork = nullptr; slot->join = nullptr;
                return fail(KV_ERR_HIP, "kv_decode_layerstack: side stream: %s", hipGetErrorString(e));
            }
        }
        side = slot->side; fork_event = slot->fork; join_event = slot->join;
    }
    int* gemm_tickets = (int*)slice;
    float* attn_partials = (float*)(slice + kvp::kGemmTicketBytes);
    float* gemm_partials = (float*)(slice + kvp::kGemmTicketBytes + attn_region);
    // the ticket words must be zero when the first dense layer starts (every launch leaves them zero again);
    // a fill kernel rather than a memset, so that the call can be captured into a graph
    if (any_operand) kvp::launch_zero_words(gemm_tickets, (int)(kvp::kGemmTicketBytes / sizeof(int)), main_stream);

    for (int l = 0; l < num_layers; ++l) {
        Resolved& r = layers[(size_t)l];
        r.p.partials = attn_partials;
        r.p.worker_trace = trace;
        if (touch) {        // fork: touch this layer's leading KV tiles while the dense layer in front of its attention runs
            (void)hipEventRecord(fork_event, main_stream);
            (void)hipStreamWaitEvent(side, fork_event, 0);
            kvp::launch_touch_mfma(r.p, r.d, r.bs, kTouchTiles, (uint32_t*)r.p.partials, side);
            (void)hipEventRecord(join_event, side);
        }
        const kv_tensor* wl = weights[l];
        int grc;
        if (wl->ndim == 5) {
            grc = kvp::launch_layer_gemm_packed(x->data, wl->data, gemm_out->data, (int)M, (int)K, (int)N, x->stride[0],
                                                gemm_out->stride[0], gemm_tickets, gemm_partials, g_plain_fetch.load() != 0,
                                                main_stream);
        } else {
            const int64_t ldw = wl->ndim == 2 ? wl->stride[0] : wl->stride[1];
            const int64_t w_tile_stride = wl->ndim == 2 ? 128 : wl->stride[0];
            grc = kvp::launch_layer_gemm(x->data, wl->data, gemm_out->data, (int)M, (int)K, (int)N, x->stride[0], ldw,
                                         w_tile_stride, gemm_out->stride[0], main_stream);
        }
        if (grc == -2) return fail(KV_ERR_HIP, "kv_decode_layerstack: could not raise the dynamic LDS limit of the GEMM kernel");
        if (grc != 0) return fail(KV_ERR_UNSUPPORTED, "kv_decode_layerstack: GEMM shape not covered");
        if (int rc = check_launch("kv_decode_layerstack GEMM kernel")) return rc;
        if (touch) (void)hipStreamWaitEvent(main_stream, join_event, 0);
        if (int rc = run_attn(r, main_stream)) return rc;
    }
    return KV_OK;
}

size_t kv_decode_workspace_bytes(int B, int Hq, int d, int max_context, int block_size) {
    if (B <= 0 || Hq <= 0 || (d != 64 && d != 128) || max_context <= 0 || block_size <= 0) return 0;
    return workspace_bytes(Hq, d);
}

size_t kv_layerstack_workspace_bytes(int Hq, int d, int gemm_n) {
    if (Hq <= 0 || (d != 64 && d != 128) || gemm_n < 128 || gemm_n % 128) return 0;
    return workspace_bytes(Hq, d) + kvp::layer_gemm_packed_partial_bytes(gemm_n);
}

int kv_decode_set_workspace(void* dev_ptr, size_t bytes) {
    if ((dev_ptr == nullptr) != (bytes == 0))
        return fail(KV_ERR_INVALID, "kv_decode_set_workspace: pointer and size must both be set or both be zero");
    if (((uintptr_t)dev_ptr) % 16) return fail(KV_ERR_INVALID, "kv_decode_set_workspace: pointer must be 16-byte aligned");
    const int dev = current_device();
    if (dev < 0) {
        if (!dev_ptr) return KV_OK;          // no device: nothing can be registered, so nothing is left to unregister
        return fail(KV_ERR_HIP, "kv_decode_set_workspace: cannot read the current device");
    }
    std::lock_guard<std::mutex> lock(g_state_mutex);
    DeviceState& ds = g_dev[dev];
    ds.ws_ptr = dev_ptr;
    ds.ws_bytes = bytes;
    ds.ws_used = 0;
    for (StreamSlot& sl : ds.slots) { sl.offset = 0; sl.bytes = 0; }    // every stream takes a new slice at its next call
    return KV_OK;
}

int kv_validate_inputs(const kv_tensor* block_tables, const kv_tensor* context_lens, int num_blocks, int block_size, void* stream) {
    if (!block_tables || !context_lens || !block_tables->data || !context_lens->data)
        return fail(KV_ERR_INVALID, "kv_validate_inputs: null tensor");
    if (block_tables->ndim != 2 || context_lens->ndim != 1 || block_tables->dtype != KV_I32 || context_lens->dtype != KV_I32 ||
        block_tables->stride[1] != 1 || context_lens->stride[0] != 1 || block_tables->shape[0] != context_lens->shape[0] ||
        block_tables->shape[0] <= 0 || block_tables->shape[1] <= 0 || block_tables->stride[0] < block_tables->shape[1])
        return fail(KV_ERR_INVALID, "kv_validate_inputs: block_tables must be int32 [B, MB] with dense rows, context_lens int32 [B], dense");
    if (num_blocks <= 0 || (block_size != 16 && block_size != 32))
        return fail(KV_ERR_INVALID, "kv_validate_inputs: num_blocks %d, block_size %d", num_blocks, block_size);
    const int64_t B = block_tables->shape[0], MB = block_tables->shape[1], ld = block_tables->stride[0];
    std::vector<int32_t> lens((size_t)B), table((size_t)((B - 1) * ld + MB));
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess) e = hipMemcpy(lens.data(), context_lens->data, lens.size() * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(table.data(), block_tables->data, table.size() * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(KV_ERR_HIP, "kv_validate_inputs: %s", hipGetErrorString(e));
    for (int64_t b = 0; b < B; ++b) {
        const int64_t n = lens[(size_t)b];
        if (n < 0 || n > MB * block_size)
            return fail(KV_ERR_INVALID, "kv_validate_inputs: context_lens[%lld] = %lld outside 0..%lld (table width x block size)",
                        (long long)b, (long long)n, (long long)(MB * block_size));
        const int64_t used = (n + block_size - 1) / block_size;
        for (int64_t i = 0; i < used; ++i) {
            const int32_t id = table[(size_t)(b * ld + i)];
            if (id < 0 || id >= num_blocks)
                return fail(KV_ERR_INVALID, "kv_validate_inputs: block_tables[%lld, %lld] = %d outside 0..%d", (long long)b, (long long)i,
                            id, num_blocks - 1);
        }
    }
    return KV_OK;
}

int kv_decode_set_worker_trace(void* dev_ptr, size_t bytes) {
    if ((dev_ptr == nullptr) != (bytes == 0))
        return fail(KV_ERR_INVALID, "kv_decode_set_worker_trace: pointer and size must both be set or both be zero");
    if (((uintptr_t)dev_ptr) % 8) return fail(KV_ERR_INVALID, "kv_decode_set_worker_trace: pointer must be 8-byte aligned");
    std::lock_guard<std::mutex> lock(g_state_mutex);
    g_trace_ptr = dev_ptr;
    g_trace_bytes = bytes;
    return KV_OK;
}

int kv_decode_set_waves_per_cu(int waves) {
    if (waves < 0 || waves > kMaxWavesPerCU)
        return fail(KV_ERR_INVALID, "kv_decode_set_waves_per_cu: %d outside 0..%d", waves, kMaxWavesPerCU);
    g_waves_per_cu.store(waves);
    return KV_OK;
}

int kv_decode_set_variant(int variant) {
    if (variant != KV_VARIANT_ONE_PASS && variant != KV_VARIANT_TWO_PHASE)
        return fail(KV_ERR_INVALID, "kv_decode_set_variant: unknown variant %d", variant);
    g_variant.store(variant);
    return KV_OK;
}

int kv_decode_set_l2_touch(int tiles) {
    if (tiles < 0 || tiles > 8) return fail(KV_ERR_INVALID, "kv_decode_set_l2_touch: %d outside 0..8", tiles);
    g_l2_touch.store(tiles);
    return KV_OK;
}

int kv_decode_set_fetch_policy(int policy) {
    if (policy != KV_FETCH_NON_TEMPORAL && policy != KV_FETCH_PLAIN)
        return fail(KV_ERR_INVALID, "kv_decode_set_fetch_policy: unknown policy %d", policy);
    g_plain_fetch.store(policy == KV_FETCH_PLAIN ? 1 : 0);
    return KV_OK;
}

int kv_decode_set_xcd_skew(int per_1024) {
    if (per_1024 < 0 || per_1024 > 256)
        return fail(KV_ERR_INVALID, "kv_decode_set_xcd_skew: %d outside 0..256", per_1024);
    g_xcd_skew.store(per_1024);
    return KV_OK;
}

int kv_decode_get_waves_per_cu(int prefetch_distance, int head_dim) {
    if (prefetch_distance < 0 || prefetch_distance > KV_MAX_PREFETCH_DISTANCE || (head_dim != 64 && head_dim != 128)) return 0;
    // (two-phase variant: for the widest group of query heads, 16, whose logits buffer is the largest)
    return waves_per_cu(prefetch_distance, head_dim, false, g_variant.load() == KV_VARIANT_TWO_PHASE ? 16 : 0);
}

int kv_decode_get_waves_per_cu_for(int prefetch_distance, int head_dim, int q_heads_per_kv_head) {
    if (prefetch_distance < 0 || prefetch_distance > KV_MAX_PREFETCH_DISTANCE || (head_dim != 64 && head_dim != 128) ||
        q_heads_per_kv_head < 1 || q_heads_per_kv_head > 16)
        return 0;
    return waves_per_cu(prefetch_distance, head_dim, false, g_variant.load() == KV_VARIANT_TWO_PHASE ? q_heads_per_kv_head : 0);
}

int kv_decode_get_waves_per_cu_kv8(int prefetch_distance, int head_dim) {
    if (prefetch_distance < 0 || prefetch_distance > KV_MAX_PREFETCH_DISTANCE || (head_dim != 64 && head_dim != 128)) return 0;
    return waves_per_cu(prefetch_distance, head_dim, true);
}

int kv_profile_enable(int max_calls, int every) {
    if (max_calls < 0 || max_calls > 100000) return fail(KV_ERR_INVALID, "kv_profile_enable: max_calls %d outside 0..100000", max_calls);
    if (every < 1) return fail(KV_ERR_INVALID, "kv_profile_enable: every %d must be at least 1", every);
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    for (hipEvent_t ev : g_prof_events) (void)hipEventDestroy(ev);
    g_prof_events.clear();
    g_prof_capacity = 0;
    g_prof_calls = 0;
    g_prof_seen = 0;
    g_prof_every = every;
    for (int i = 0; i < 2 * max_calls; ++i) {
        hipEvent_t ev;
        hipError_t e = hipEventCreate(&ev);
        if (e != hipSuccess) {
            for (hipEvent_t x : g_prof_events) (void)hipEventDestroy(x);
            g_prof_events.clear();
            return fail(KV_ERR_HIP, "kv_profile_enable: %s", hipGetErrorString(e));
        }
        g_prof_events.push_back(ev);
    }
    g_prof_capacity = max_calls;
    return KV_OK;
}

int kv_profile_read(double* main_ms_sum, int* calls) {
    if (!main_ms_sum || !calls) return fail(KV_ERR_INVALID, "kv_profile_read: null output");
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    *main_ms_sum = 0;
    *calls = g_prof_calls;
    for (int i = 0; i < g_prof_calls; ++i) {
        hipError_t e = hipEventSynchronize(prof_event(i, 1));
        float a = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&a, prof_event(i, 0), prof_event(i, 1));
        if (e != hipSuccess) return fail(KV_ERR_HIP, "kv_profile_read: %s", hipGetErrorString(e));
        *main_ms_sum += a;
    }
    g_prof_calls = 0;
    g_prof_seen = 0;
    return KV_OK;
}

int kv_profile_read_each(float* main_ms, int capacity, int* calls) {
    if (!main_ms || !calls || capacity < 0) return fail(KV_ERR_INVALID, "kv_profile_read_each: null output or negative capacity");
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (g_prof_calls > capacity)
        return fail(KV_ERR_INVALID, "kv_profile_read_each: %d samples recorded, room for %d", g_prof_calls, capacity);
    *calls = g_prof_calls;
    for (int i = 0; i < g_prof_calls; ++i) {
        hipError_t e = hipEventSynchronize(prof_event(i, 1));
        if (e == hipSuccess) e = hipEventElapsedTime(&main_ms[i], prof_event(i, 0), prof_event(i, 1));
        if (e != hipSuccess) return fail(KV_ERR_HIP, "kv_profile_read_each: %s", hipGetErrorString(e));
    }
    g_prof_calls = 0;
    g_prof_seen = 0;
    return KV_OK;
}

const char* kv_last_error(void) { return g_err; }

int kv_version(void) { return 100; }

int kv_worker_range(int64_t tiles, int workers, int xcd_skew, int worker, int64_t* first, int64_t* end) {
    if (tiles < 1 || tiles > ((int64_t)1 << 40) || workers < 1 || workers > kvp::kMaxMfmaWorkers || xcd_skew < 0 ||
        xcd_skew > 256 || !first || !end)
        return fail(KV_ERR_INVALID, "kv_worker_range: invalid argument");
    const int nw = tiles < workers ? (int)tiles : workers;
    if (worker < 0 || worker >= nw) return fail(KV_ERR_INVALID, "kv_worker_range: worker %d of %d", worker, nw);
    const int skew = kvp::effective_skew(tiles, nw, xcd_skew);
    *first = kvp::range_start(worker, tiles, nw, skew);
    *end = kvp::range_start(worker + 1, tiles, nw, skew);
    return KV_OK;
}

int kv_worker_of_tile(int64_t tiles, int workers, int xcd_skew, int64_t tile) {
    if (tiles < 1 || tiles > ((int64_t)1 << 40) || workers < 1 || workers > kvp::kMaxMfmaWorkers || xcd_skew < 0 ||
        xcd_skew > 256 || tile < 0 || tile >= tiles)
        return -1;
    const int nw = tiles < workers ? (int)tiles : workers;
    return kvp::range_owner(tile, tiles, nw, kvp::effective_skew(tiles, nw, xcd_skew));
}

size_t kv_block_bytes(int elem_bytes, int head_dim, int block_size) {
    if (elem_bytes <= 0 || head_dim <= 0 || block_size <= 0) return 0;
    return (size_t)elem_bytes * head_dim * block_size;
}

size_t kv_iter_working_set_bytes(size_t block_bytes, int units_per_wg, int H, int B) {
    if (units_per_wg <= 0 || H <= 0 || B <= 0) return 0;
    return block_bytes * (size_t)units_per_wg * H * B;
}

}  // extern "C"
