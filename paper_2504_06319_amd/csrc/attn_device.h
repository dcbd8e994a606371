// Device-side pieces shared by the attention kernels: operand types and MFMA wrappers, lane-swap reductions,
// counted waits, the flat tile space (lengths scan, worker ranges, cursor) and the FP8 widening.
#pragma once
#include "kv_common.h"

namespace kvp {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define KVP_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define KVP_GLOBAL(p) ((const __attribute__((address_space(1))) void*)(p))

template <Elem E>
__device__ __forceinline__ float4v mfma_k32(u32x4 a, u32x4 b, float4v c) {
    if constexpr (E == Elem::BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

template <Elem E>
__device__ __forceinline__ float4v mfma_k16(u32x2 a, u32x2 b, float4v c) {
    if constexpr (E == Elem::BF16)
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(short4v, a), __builtin_bit_cast(short4v, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4, a), __builtin_bit_cast(half4, b), c, 0, 0, 0);
}

typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

// Two floats -> two 16-bit patterns in one dword (lo in bits 15:0), round to nearest even; one packed convert.
template <Elem E>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const float2v f = {lo, hi};
    if constexpr (E == Elem::BF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
    else return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, half2v));
}

// The values of the lanes 16 and 32 away (lane ^ 16, lane ^ 32), by the lane-swap instructions: a register-file
// operation, where a shuffle would be a round trip through the LDS crossbar on the critical path of every tile.
// v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of its second,
// v_permlane32_swap the upper half of the first with the lower half of the second; fed the same value twice, the
// two results hold, for every lane, its own value and the partner's, in some order.
struct LanePair { float a, b; };
__device__ __forceinline__ LanePair swap16(float v) {
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const uint32_t r0 = r[0], r1 = r[1];        // copies: a bit_cast applied to a vector element reads element 0
    return {__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}
__device__ __forceinline__ LanePair swap32(float v) {
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const uint32_t r0 = r[0], r1 = r[1];        // copies: a bit_cast applied to a vector element reads element 0
    return {__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}
// max / sum over the four lanes {lr, lr + 16, lr + 32, lr + 48}
__device__ __forceinline__ float group_max(float v) {
    LanePair p = swap16(v);
    v = fmaxf(p.a, p.b);
    p = swap32(v);
    return fmaxf(p.a, p.b);
}
__device__ __forceinline__ float group_sum(float v) {
    LanePair p = swap16(v);
    v = p.a + p.b;
    p = swap32(v);
    return p.a + p.b;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    // gfx9 encoding of s_waitcnt: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14; expcnt and lgkmcnt left at max
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | 0x0f70);
}

// four FP8 E4M3 codes of a dword -> four 16-bit values of type E in two dwords (exact: both 16-bit types hold every
// E4M3 value)
template <Elem E>
__device__ __forceinline__ u32x2 widen_fp8x4(uint32_t w) {
    if constexpr (E == Elem::BF16) {
        return u32x2{__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false)),
                     __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true))};
    } else {
        return u32x2{__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false)),
                     __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true))};
    }
}

constexpr int kAuxNonTemporal = 2;                   // cache-policy operand of global_load_lds: nt

// Position of a worker inside the flat tile space; every field is wave-uniform.
struct Cursor {
    int b;        // sequence
    int kvh;      // kv head
    int j;        // tile index inside the sequence
    int ntiles;   // tiles of sequence b
    int n;        // clamped context length of sequence b
};

typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;   // uniform loads become scalar loads

__device__ __forceinline__ int clamp_len(int n, int max_len) { return min(max(n, 0), max_len); }
// tiles of 2^shift tokens that n tokens occupy (16-token tiles for 16-bit caches, 32-token tiles for 8-bit ones)
__device__ __forceinline__ int tiles_of(int n, int shift) { return (n + (1 << shift) - 1) >> shift; }

__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// scan_total: per-kv-head tile total of the batch.  scan_locate: for a flat position `target`, the sequence
// that holds it, i.e. the last b whose first flat tile Hkv * cum[b] is <= target, that cum[b] and the sequence's
// clamped length (handed back from the scan's registers: one dependent memory round trip less at the start).

__device__ __forceinline__ int scan_total(const_i32_ptr cl, int B, int max_len, int lane, int shift) {
    int total = 0;
    for (int base = 0; base < B; base += kWaveSize) {
        const int idx = base + lane;
        const int t = idx < B ? tiles_of(clamp_len(cl[idx], max_len), shift) : 0;
        total += wave_sum_i32(t);
    }
    return __builtin_amdgcn_readfirstlane(total);   // every lane holds the sum: make it a scalar for the compiler too
}

__device__ __forceinline__ void scan_locate(const_i32_ptr cl, int B, int max_len, int lane, int shift, int Hkv,
                                            int64_t target, int& b_out, int& cum_out, int& n_out) {
    int cum = 0, found_b = 0, found_cum = 0, found_n = 0;
    for (int base = 0; base < B; base += kWaveSize) {
        const int idx = base + lane;
        const int n = idx < B ? clamp_len(cl[idx], max_len) : 0;
        const int t = tiles_of(n, shift);
        int incl = t;
#pragma unroll
        for (int off = 1; off < kWaveSize; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        const int excl = cum + incl - t;
        const bool pred = idx < B && (int64_t)Hkv * excl <= target;
        const int cnt = __builtin_popcountll(__builtin_amdgcn_ballot_w64(pred));
        if (cnt == 0) break;                       // the predicate is monotone: nothing further matches
        found_b = base + cnt - 1;
        found_cum = __builtin_amdgcn_readlane(excl, cnt - 1);
        found_n = __builtin_amdgcn_readlane(n, cnt - 1);
        cum += __builtin_amdgcn_readlane(incl, kWaveSize - 1);
        if (cnt < kWaveSize) break;
    }
    b_out = found_b;
    cum_out = found_cum;
    n_out = found_n;
}

// Range boundaries of the flat tile space.  Worker w's share is proportional to 1024 + skew for even w and
// 1024 - skew for odd w: workgroups go to the eight XCDs round-robin, and under load the odd XCD of every XCD
// pair delivers 3-4 % less bandwidth than the even one (per-worker exit times, grouped by XCC_ID), so
// equal shares would leave the even XCDs idle at the end.  The cumulative weight of workers [0, w) is
// 1024 w + skew (w & 1).  Ranges of fewer than 16 tiles are not skewed.
__host__ __device__ __forceinline__ int effective_skew(int64_t T, int num_workers, int skew) {
    return T >= 16 * (int64_t)num_workers ? skew : 0;
}
// floor(num / den) for 0 <= num < 2^62, 0 < den, quotient below 2^31: a double-precision estimate (error below one)
// and one exact correction step; an emulated 64-bit integer division costs several times as much.
__host__ __device__ __forceinline__ int64_t floor_div(int64_t num, int64_t den) {
    int64_t q = (int64_t)((double)num / (double)den);
    const int64_t r = num - q * den;
    if (r < 0) --q;
    else if (r >= den) ++q;
    return q;
}
__host__ __device__ __forceinline__ int64_t range_weight(int worker, int skew) { return 1024 * (int64_t)worker + skew * (worker & 1); }
__host__ __device__ __forceinline__ int64_t range_start(int worker, int64_t T, int num_workers, int skew) {
    return floor_div(T * range_weight(worker, skew), range_weight(num_workers, skew));
}
// Last worker whose range starts at or before flat tile x (0 <= x < T): range_start(w) <= x exactly when
// T weight(w) < (x + 1) total, i.e. weight(w) <= floor(((x + 1) total - 1) / T).
__host__ __device__ __forceinline__ int range_owner(int64_t x, int64_t T, int num_workers, int skew) {
    const int64_t limit = floor_div((x + 1) * range_weight(num_workers, skew) - 1, T);
    int w = (int)(limit >> 10);
    if (range_weight(w, skew) > limit) --w;
    return w < num_workers - 1 ? w : num_workers - 1;
}
// Whether range_start(worker) < x, without a division.
__host__ __device__ __forceinline__ bool range_starts_before(int worker, int64_t x, int64_t T, int num_workers, int skew) {
    return T * range_weight(worker, skew) < x * range_weight(num_workers, skew);
}
// XCC_ID field (bits 3:0) of hardware register 20: the XCD this wave runs on.
__device__ __forceinline__ int xcc_id() { return (int)__builtin_amdgcn_s_getreg((3 << 11) | 20); }

// ---- 16-bit tiles: LDS operand reads and the per-head_dim geometry (shared by the 16-bit attention kernels)

// LDS reads of the ring are written as inline assembly on purpose.  The compiler knows
// that global_load_lds writes LDS and, unable to tell ring stages apart, would put a
// wait for ALL outstanding fetches in front of every LDS read it can see, which would
// serialise the look-ahead.  The fetch completion is tracked by hand instead (vmcnt),
// and so is the completion of these reads (lgkmcnt, LDS returns data in order).
__device__ __forceinline__ void lds_read_b128_x4(u32x4& r0, u32x4& r1, u32x4& r2, u32x4& r3,
                                                 uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3) {
    asm volatile(
        "ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7"
        : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
        : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
        : "memory");
}

__device__ __forceinline__ void lds_read_tr16_x4(u32x2& r0, u32x2& r1, u32x2& r2, u32x2& r3,
                                                 uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3) {
    asm volatile(
        "ds_read_b64_tr_b16 %0, %4\n\tds_read_b64_tr_b16 %1, %5\n\tds_read_b64_tr_b16 %2, %6\n\tds_read_b64_tr_b16 %3, %7"
        : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
        : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
        : "memory");
}

__device__ __forceinline__ void lds_read_b128_x2(u32x4& r0, u32x4& r1, uint32_t a0, uint32_t a1) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3" : "=&v"(r0), "=&v"(r1) : "v"(a0), "v"(a1) : "memory");
}

// Wait until at most N of this wave's LDS operations are outstanding; the registers are
// passed through so that no use of them can be scheduled above the wait.
template <int N>
__device__ __forceinline__ void lds_wait_k(u32x4& r0, u32x4& r1, u32x4& r2, u32x4& r3) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_wait_k(u32x4& r0, u32x4& r1) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(r0), "+v"(r1) : "n"(N) : "memory");
}
__device__ __forceinline__ void lds_wait_v(u32x2 (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) : : "memory");
}
__device__ __forceinline__ void lds_wait_v(u32x2 (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 :
                 : "memory");
}


constexpr int kTileTokens = 16;
constexpr int kTileShift = 4;

// Per-head_dim geometry of a 16-token tile.
template <int D>
struct Geo {
    static constexpr int kRowBytes = D * 2;                        // one token's row of K (or V)
    static constexpr int kTileBytes = kTileTokens * kRowBytes;     // 4 KB (d 128) / 2 KB (d 64) for K, the same for V
    static constexpr int kStageBytes = 2 * kTileBytes;
    static constexpr int kQueryBytes = kTileBytes;                 // a unit's query rows, laid out like a K tile (16 rows)
    static constexpr int kChunks = D / 8;                          // 16-byte chunks per row
    static constexpr int kRowsPerLoad = kWaveSize / kChunks;       // rows one wave-wide 1 KB fetch lands
    static constexpr int kLoadsPerTile = kTileTokens / kRowsPerLoad;
    static constexpr int kSwzShift = 16 / kChunks;                 // rows that share a swizzle value
    static constexpr int kKSteps = D / 32;                         // MFMAs of the logits
    static constexpr int kColBlocks = D / 16;                      // 16-column blocks of the output
    static constexpr int kPartialStride = D + 4;                   // floats per partial row: acc, max, sum, 2 pad (16-byte rows)
    __host__ __device__ static constexpr int swz_k(int row) { return (row / kSwzShift) % kChunks; }
    // V swizzle of the 16-byte chunk index: even, so that it moves the 32-byte block a transpose read takes
    __host__ __device__ static constexpr int swz_v(int row) { return 2 * ((row / kSwzShift) % (kChunks / 2)); }
};

}  // namespace kvp
