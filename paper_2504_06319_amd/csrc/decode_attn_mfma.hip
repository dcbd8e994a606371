// Paged decode attention for head_dim 128 on the matrix cores, with an LDS ring that
// holds the KV tiles a wave will consume next.
//
// Work mapping (paper Section 3.1, re-mapped so that a KV byte is fetched once for all
// grouped query heads): one workgroup per (sequence, kv head, partition [s, e) of the
// block range); each wave owns one 16-token tile per iteration and walks the range with
// a stride of the wave count, the walk of Algorithm 1.
//
// Prefetch (Algorithm 1 generalised to distance PD): a wave owns PD + 1 LDS stages.
// Per iteration it waits for the current tile, issues the asynchronous global->LDS
// fetch of the tile it will consume PD iterations later (guarded by the range end),
// and only then computes on the current tile, so PD tiles per wave are in flight under
// the compute.  PD = 0 is the baseline flow: fetch, wait, compute.  gfx950 has no
// prefetch-to-cache instruction; the LDS-direct load (no VGPR landing zone) is its
// closest asynchronous fetch.
//
// Tile math, all on MFMA with fp32 accumulation:
//   S^T[t, g]  = sum_c K[t, c] Q[g, c]     4 x v_mfma_f32_16x16x32 (A = K tile, B = Q^T)
//   P^T[t, g]  = 2^(S^T - m[g])            online softmax; max over tokens by lane permutes
//   O^T[c, g] += sum_t V[t, c] P^T[t, g]   8 x v_mfma_f32_16x16x16 (A = V^T via LDS transpose read)
// Computing the transposed products keeps the head index on lane % 16 from the logits to
// the output accumulators, so the softmax rescale is a per-lane multiply.
//
// LDS layout of a stage: K tile then V tile, each 16 rows x 256 B, written by
// global_load_lds_dwordx4 (lane i of load r lands at r*1024 + i*16).  Bank conflicts are
// avoided by permuting which 16-byte chunk of a row each lane fetches: K rows are stored
// with chunk index XOR row, V rows with chunk index XOR 2*(row % 8).
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

template <Elem E>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)pack1<E>(lo) | ((uint32_t)pack1<E>(hi) << 16);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    // gfx9 encoding of s_waitcnt: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14; expcnt and lgkmcnt left at max
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | 0x0f70);
}

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

// Wait until at most N of this wave's LDS operations are outstanding; the registers are
// passed through so that no use of them can be scheduled above the wait.
template <int N>
__device__ __forceinline__ void lds_wait_k(u32x4& r0, u32x4& r1, u32x4& r2, u32x4& r3) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3) : "n"(N) : "memory");
}
__device__ __forceinline__ void lds_wait_v(u32x2 (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 :
                 : "memory");
}

constexpr int kTileTokens = 16;
constexpr int kRowBytes = 256;                       // 128 x 16-bit
constexpr int kTileBytes = kTileTokens * kRowBytes;  // 4 KB for K, the same for V
constexpr int kStageBytes = 2 * kTileBytes;

template <Elem E, int BS, int PD, int W>
__global__ __launch_bounds__(W* kWaveSize) void attn_mfma_kernel(AttnParams p) {
    constexpr int D = 128;
    constexpr int NS = PD + 1;                  // LDS stages per wave
    constexpr int TPB = BS / kTileTokens;       // 16-token tiles per KV block
    constexpr int LOADS = 8;                    // wave-wide 1 KB loads per tile pair (4 K + 4 V)
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int part = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWaveSize);
    const int lane = tid % kWaveSize;
    const int lq = lane / 16, lr = lane % 16;   // lane group (0..3) and index in the group

    int n = p.context_lens[b];
    n = min(max(n, 0), p.MB * BS);
    const int ntiles_seq = (n + kTileTokens - 1) / kTileTokens;
    const int part_tiles = p.part_blocks * TPB;
    const int s = part * part_tiles;
    const bool direct = (p.NP == 1);
    if (s >= ntiles_seq && !(direct && part == 0)) return;
    const int e = min(ntiles_seq, s + part_tiles);
    const int G = p.G;

    // ---- Q^T operand: lane (g = lr, lq) holds Q[g][(4j + lq) * 8 .. +8] for j = 0..3, zero rows for g >= G
    u32x4 qb[4];
    {
        const uint16_t* qrow = reinterpret_cast<const uint16_t*>(p.q) + (int64_t)b * p.q_stride_b +
                               (int64_t)(kvh * G + min(lr, G - 1)) * p.q_stride_h;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(qrow + (4 * j + lq) * 8);
            qb[j] = lr < G ? v : u32x4{0, 0, 0, 0};
        }
    }

    // ---- per-lane byte offsets, loop invariant
    // fetch r (0..3) of a tile lands rows 4r..4r+3; this lane lands row t = 4r + lq at LDS slot lr, so it
    // fetches chunk (lr ^ swizzle(t)) of row t
    uint32_t koff[4], voff[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int t = 4 * r + lq;
        koff[r] = t * kRowBytes + ((lr ^ t) << 4);
        voff[r] = t * kRowBytes + ((lr ^ (2 * (t % 8))) << 4);
    }
    // K read for MFMA j: row lr, logical chunk 4j + lq  ->  stored chunk (4j + lq) ^ lr
    uint32_t kread[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) kread[j] = lr * kRowBytes + (((4 * j + lq) ^ lr) << 4);
    // V transpose read for column block cb: row lane/4, logical byte 32 cb + 8 (lane % 4)
    const int vt = lane / 4;
    uint32_t vread[8];
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) vread[cb] = kTileBytes + vt * kRowBytes + ((cb ^ (vt % 8)) << 5) + ((lane % 4) << 3);

    unsigned char* ring = smem + wave * (NS * kStageBytes);
    const uint32_t ring_addr = (uint32_t)(uintptr_t)KVP_LDS(ring);      // LDS byte address of the wave's ring
    // read through the constant address space: the table is never written while the kernel runs, and a
    // uniform constant load becomes a scalar load whose wait does not involve the KV fetches in flight
    const __attribute__((address_space(4))) int32_t* bt =
        (const __attribute__((address_space(4))) int32_t*)(p.block_tables + (int64_t)b * p.bt_stride_b);
    const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k_cache) + (int64_t)kvh * p.kv_stride_h * 2;
    const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v_cache) + (int64_t)kvh * p.v_stride_h * 2;

    auto issue = [&](int tile, int stage) {       // asynchronous fetch of one K tile and one V tile into a stage
        int phys = bt[tile / TPB];
        phys = min(max(phys, 0), p.NBLK - 1);
        const int sub = (tile % TPB) * kTileBytes;
        const unsigned char* kt = kbase + (int64_t)phys * p.kv_stride_blk * 2 + sub;
        const unsigned char* vt_ = vbase + (int64_t)phys * p.v_stride_blk * 2 + sub;
        unsigned char* dst = ring + stage * kStageBytes;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GLOBAL(kt + koff[r]), KVP_LDS(dst + r * 1024), 16, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GLOBAL(vt_ + voff[r]), KVP_LDS(dst + kTileBytes + r * 1024), 16, 0, 0);
    };

    float4v o[8];
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) o[cb] = float4v{0.f, 0.f, 0.f, 0.f};
    float m = kNegBig, l = 0.f;

    // ---- prologue: fill the ring
    const int first = s + wave;
    if constexpr (PD > 0) {
#pragma unroll
        for (int k = 0; k < PD; ++k)
            if (first + k * W < e) issue(first + k * W, k);
    }

    int stage = 0;
    for (int tile = first; tile < e; tile += W) {
        if constexpr (PD == 0) {
            issue(tile, 0);
            wait_vmcnt<0>();
        } else {
            // Algorithm 1 order: current tile is on its way; issue the look-ahead fetch, then compute
            const int ahead = tile + PD * W;
            int ahead_stage = stage + PD; if (ahead_stage >= NS) ahead_stage -= NS;
            if (ahead < e) {
                issue(ahead, ahead_stage);
                wait_vmcnt<LOADS * PD>();          // everything older than the PD newest tiles has landed
            } else {
                wait_vmcnt<0>();
            }
        }
        asm volatile("" ::: "memory");
        const uint32_t st = ring_addr + stage * kStageBytes;

        // ---- issue every LDS read of the tile: 4 K operands, then 8 transposed V operands
        u32x4 ka[4];
        u32x2 va[8];
        lds_read_b128_x4(ka[0], ka[1], ka[2], ka[3], st + kread[0], st + kread[1], st + kread[2], st + kread[3]);
        lds_read_tr16_x4(va[0], va[1], va[2], va[3], st + vread[0], st + vread[1], st + vread[2], st + vread[3]);
        lds_read_tr16_x4(va[4], va[5], va[6], va[7], st + vread[4], st + vread[5], st + vread[6], st + vread[7]);

        // ---- S^T = K Q^T once the K operands are back (the 8 V reads may still be outstanding)
        lds_wait_k<8>(ka[0], ka[1], ka[2], ka[3]);
        float4v sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) sacc = mfma_k32<E>(ka[j], qb[j], sacc);
        lds_wait_v(va);

        // ---- online softmax over this tile's 16 tokens (lane holds tokens 4 lq + i of head lr)
        float sc[4];
        const int tok0 = tile * kTileTokens + 4 * lq;
        const bool tail = (tile + 1) * kTileTokens > n;        // wave-uniform
#pragma unroll
        for (int i = 0; i < 4; ++i) sc[i] = sacc[i] * p.scale_log2e;
        if (tail) {
#pragma unroll
            for (int i = 0; i < 4; ++i) sc[i] = (tok0 + i < n) ? sc[i] : -INFINITY;    // select, not multiply
            // masked tokens: zero their V values so garbage (NaN) cannot reach the accumulators
            const uint32_t m01 = ((tok0 + 0 < n) ? 0x0000ffffu : 0u) | ((tok0 + 1 < n) ? 0xffff0000u : 0u);
            const uint32_t m23 = ((tok0 + 2 < n) ? 0x0000ffffu : 0u) | ((tok0 + 3 < n) ? 0xffff0000u : 0u);
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) { va[cb][0] &= m01; va[cb][1] &= m23; }
        }
        float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx);
        if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {      // some head's maximum moved: rescale
            const float alpha = fast_exp2(m - m_new);
            l *= alpha;
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) o[cb] *= alpha;
            m = m_new;
        }
        float pr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pr[i] = fast_exp2(sc[i] - m);
        l += (pr[0] + pr[1]) + (pr[2] + pr[3]);
        const u32x2 pb = {pack2<E>(pr[0], pr[1]), pack2<E>(pr[2], pr[3])};

        // ---- O^T += V^T P^T
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) o[cb] = mfma_k16<E>(va[cb], pb, o[cb]);

        if constexpr (PD > 0) { stage = stage + 1 == NS ? 0 : stage + 1; }
    }

    // ---- merge the waves through LDS (the rings are idle: every wave has consumed all it fetched)
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);               // [W][G][D + 2]
    if (lr < G) {
        float* dst = red + (wave * G + lr) * (D + 2);
#pragma unroll
        for (int cb = 0; cb < 8; ++cb)
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[16 * cb + 4 * lq + i] = o[cb][i];
        if (lq == 0) { dst[D] = m; dst[D + 1] = l; }
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += W * kWaveSize) {
        const int g = idx / D, c = idx % D;
        float ms = kNegBig;
#pragma unroll
        for (int w = 0; w < W; ++w) ms = fmaxf(ms, red[(w * G + g) * (D + 2) + D]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const float* src = red + (w * G + g) * (D + 2);
            const float wgt = fast_exp2(src[D] - ms);
            num += wgt * src[c];
            den += wgt * src[D + 1];
        }
        const int h = kvh * G + g;
        if (direct) {
            const float ov = den > 0.f ? num / den : 0.f;
            reinterpret_cast<uint16_t*>(p.out)[(int64_t)b * p.out_stride_b + (int64_t)h * p.out_stride_h + c] = pack1<E>(ov);
        } else {
            float* dst = p.partials + (((int64_t)b * p.Hq + h) * p.NP + part) * (D + 2);
            dst[c] = num;
            if (c == 0) { dst[D] = ms; dst[D + 1] = den; }
        }
    }
}

template <Elem E, int BS, int PD, int W>
static int launch_one(const AttnParams& p, hipStream_t stream) {
    const size_t ring = (size_t)W * (PD + 1) * kStageBytes;
    const size_t merge = (size_t)W * p.G * (128 + 2) * sizeof(float);
    const size_t lds = ring > merge ? ring : merge;
    auto kern = attn_mfma_kernel<E, BS, PD, W>;
    static bool attr_set = false;       // raising the dynamic LDS limit once per instantiation
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return -2;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(p.NP, p.Hkv, p.B), dim3(W * kWaveSize), lds, stream, p);
    return 0;
}

template <Elem E, int BS>
static int launch_pd(const AttnParams& p, hipStream_t stream) {
    switch (p.prefetch_distance) {
        case 0: return launch_one<E, BS, 0, 4>(p, stream);
        case 1: return launch_one<E, BS, 1, 4>(p, stream);
        case 2: return launch_one<E, BS, 2, 4>(p, stream);
        case 3: return launch_one<E, BS, 3, 4>(p, stream);
        case 4: return launch_one<E, BS, 4, 4>(p, stream);
        default: return -1;
    }
}

// head_dim 128 only.  Returns 0, -1 (no such instantiation) or -2 (HIP refused the LDS size).
int launch_attn_mfma(const AttnParams& p, int elem, int bs, hipStream_t stream) {
    if (elem == (int)Elem::F16) return bs == 16 ? launch_pd<Elem::F16, 16>(p, stream) : launch_pd<Elem::F16, 32>(p, stream);
    return bs == 16 ? launch_pd<Elem::BF16, 16>(p, stream) : launch_pd<Elem::BF16, 32>(p, stream);
}

}  // namespace kvp
