// Shared declarations of the kvprefetch HIP sources: launch parameters and small
// device helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvp {

constexpr int kWaveSize = 64;
constexpr int kWavesPerWG = 4;            // waves of one attention workgroup
constexpr float kNegBig = -1.0e30f;       // "no token seen yet" running maximum (finite on purpose)
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
    int64_t q_stride_b, q_stride_h;
    int64_t kv_stride_blk, kv_stride_h;
    int64_t v_stride_blk, v_stride_h;
    int64_t out_stride_b, out_stride_h;
    int64_t bt_stride_b;
    int32_t B, Hq, Hkv, G;
    int32_t MB;               // table width (max blocks per sequence)
    int32_t NBLK;             // physical blocks in the cache
    int32_t part_blocks;      // KV blocks per partition
    int32_t NP;               // partitions per sequence in the launch grid
    int32_t prefetch_distance;
    int32_t num_workers;      // persistent waves of the head_dim-128 kernel
    float scale_log2e;        // scale * log2(e): logits live in the base-2 domain
};

enum class Elem : int { F16 = 0, BF16 = 1 };

// 16-bit pair in one dword -> two floats.
template <Elem E>
__device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    if constexpr (E == Elem::BF16) {
        lo = __uint_as_float(w << 16);
        hi = __uint_as_float(w & 0xffff0000u);
    } else {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        h2 v = __builtin_bit_cast(h2, w);
        lo = (float)v.x;
        hi = (float)v.y;
    }
}

// float -> 16-bit pattern, round to nearest even.
template <Elem E>
__device__ __forceinline__ uint16_t pack1(float f) {
    if constexpr (E == Elem::BF16) {
        return __builtin_bit_cast(uint16_t, (__bf16)f);
    } else {
        return __builtin_bit_cast(uint16_t, (_Float16)f);
    }
}

template <Elem E>
__device__ __forceinline__ float load1(const void* base, int64_t idx) {
    uint16_t bits = reinterpret_cast<const uint16_t*>(base)[idx];
    float lo, hi;
    unpack2<E>((uint32_t)bits, lo, hi);
    return lo;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// DPP lane exchanges inside a row of 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// Sum over the aligned group of N lanes (N = 8 or 16) a lane belongs to; every lane gets it.
template <int N>
__device__ __forceinline__ float group_sum(float x) {
    x += dpp_move<kDppQuadXor1>(x);
    x += dpp_move<kDppQuadXor2>(x);
    x += dpp_move<kDppRowHalfMirror>(x);
    if constexpr (N == 16) x += dpp_move<kDppRowMirror>(x);
    return x;
}

int launch_attn_valu(const AttnParams& p, int elem, int d, int bs, hipStream_t stream);
int launch_attn_mfma(const AttnParams& p, int elem, int bs, hipStream_t stream);
int launch_finalize_mfma(const AttnParams& p, int elem, int bs, hipStream_t stream);
int launch_touch_mfma(const AttnParams& p, int bs, int tiles, uint32_t* sink, hipStream_t stream);
int launch_layer_gemm(const void* x, const void* w, void* y, int M, int K, int N, int64_t ldx, int64_t ldw,
                      int64_t w_tile_stride, int64_t ldy, hipStream_t stream);
int mfma_worker_lds_bytes(int prefetch_distance);
size_t mfma_partial_bytes(int num_workers, int G);
constexpr int kMaxMfmaWorkers = 4096;
int launch_reduce(const AttnParams& p, int elem, int d, int bs, hipStream_t stream);

}  // namespace kvp
