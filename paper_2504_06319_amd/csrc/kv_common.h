// Shared declarations of the kvprefetch HIP sources: launch parameters and small
// device helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace kvp {

constexpr int kWaveSize = 64;
constexpr float kNegBig = -1.0e30f;       // "no token seen yet" running maximum (finite on purpose)
// log2 units a head's running maximum may grow before the accumulators are rescaled (AttnParams::rescale_slack).
// Swept at run time over 0, 1, 2, 4, 8 on the three benchmark batches: 2 is best or within 0.3 % of best on each
// (against 0: +0.8 %, +0.1 %, +2.3 %); larger values cost the batch of few long sequences 1 %.
constexpr float kRescaleSlack = 2.0f;
constexpr float kLog2e = 1.4426950408889634f;

// One attention call, resolved by the host.  Strides in elements.
struct AttnParams {
    const void* q;
    const void* k_cache;
    const void* v_cache;
    const int32_t* block_tables;
    const int32_t* context_lens;
    void* out;
    float* partials;          // split-KV scratch: unnormalised acc, running max (log2 domain), sum per piece
    unsigned long long* worker_trace;   // optional: 4 words per worker (clock at entry, after the scan, at exit; tiles); may be null
    int64_t q_stride_b, q_stride_h;
    int64_t kv_stride_blk, kv_stride_h;
    int64_t v_stride_blk, v_stride_h;
    int64_t out_stride_b, out_stride_h;
    int64_t bt_stride_b;
    int32_t B, Hq, Hkv, G;
    int32_t MB;               // table width (max blocks per sequence)
    int32_t NBLK;             // physical blocks in the cache
    int32_t prefetch_distance;
    int32_t num_workers;      // persistent waves (workers) of the launch
    int32_t tile_shift;       // log2 of the tokens per tile of the flat tile space: 4 (16-bit caches) or 5 (8-bit)
    int32_t l2_touch;         // > 0 with prefetch_distance 0: a second wave per worker touches this many tiles per group into L2
    int32_t xcd_skew;         // per-1024 skew of the range sizes between even and odd workers (XCDs)
    int32_t plain_fetch;      // comparison mode: KV fetches without the non-temporal hint (benchmark shapes only)
    float scale_log2e;        // scale * log2(e) (* k_scale for an 8-bit cache): logits live in the base-2 domain
    float out_scale;          // multiplies every output row: 1, or v_scale for an 8-bit cache
    float rescale_slack;      // log2 units a head's running maximum may grow before the accumulators are rescaled
};

enum class Elem : int { F16 = 0, BF16 = 1 };

// float -> 16-bit pattern, round to nearest even.
template <Elem E>
__device__ __forceinline__ uint16_t pack1(float f) {
    if constexpr (E == Elem::BF16) {
        return __builtin_bit_cast(uint16_t, (__bf16)f);
    } else {
        return __builtin_bit_cast(uint16_t, (_Float16)f);
    }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

int launch_attn_mfma(const AttnParams& p, int elem, int d, int bs, hipStream_t stream);
int launch_attn_twophase(const AttnParams& p, int elem, int d, int bs, hipStream_t stream);
int twophase_worker_lds_bytes(int prefetch_distance, int d, int G);
int launch_attn_l2_touch(const AttnParams& p, int elem, int d, int bs, hipStream_t stream);
int launch_fetch_probe(const AttnParams& p, int d, int bs, hipStream_t stream);
int launch_attn_kv8(const AttnParams& p, int elem, int d, int bs, hipStream_t stream);
int launch_finalize_mfma(const AttnParams& p, int elem, int d, int bs, hipStream_t stream);
int launch_touch_mfma(const AttnParams& p, int d, int bs, int tiles, uint32_t* sink, hipStream_t stream);
int launch_layer_gemm(const void* x, const void* w, void* y, int M, int K, int N, int64_t ldx, int64_t ldw,
                      int64_t w_tile_stride, int64_t ldy, hipStream_t stream);
int launch_layer_gemm_packed(const void* x, const void* wp, void* y, int M, int K, int N, int64_t ldx, int64_t ldy,
                             int* tickets, float* partials, bool plain_fetch, hipStream_t stream);
size_t layer_gemm_packed_partial_bytes(int N);
void launch_zero_words(int* p, int n, hipStream_t stream);
constexpr size_t kGemmTicketBytes = 4096;      // head of the workspace: one ticket word per 128-column tile of the dense layer
int mfma_worker_lds_bytes(int prefetch_distance, int d);
int kv8_worker_lds_bytes(int prefetch_distance, int d);
size_t mfma_partial_bytes(int num_workers, int G, int d);
constexpr int kMaxMfmaWorkers = 4096;
constexpr int kMaxDevices = 64;                // device ordinals the library keeps state for

// Dynamic-LDS limit of one kernel: raised to the kernel's own maximum, once per device (the attribute belongs to
// the device's copy of the function).  Threads that race set the same value.
struct LdsLimit {
    std::atomic<int> done[kMaxDevices] = {};
    // 0, or -2 when HIP refuses
    int raise(const void* kern, int max_bytes) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -2;
        if (done[dev].load(std::memory_order_acquire)) return 0;
        if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, max_bytes) != hipSuccess) return -2;
        done[dev].store(1, std::memory_order_release);
        return 0;
    }
};

}  // namespace kvp
