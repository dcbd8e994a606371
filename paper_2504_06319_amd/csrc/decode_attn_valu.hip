// Paged decode attention, vector-ALU formulation.
//
// Work mapping (paper Section 3.1 re-mapped for GQA grouping): one workgroup per
// (sequence, kv head, partition of the block range); its 4 waves each own one KV
// block per iteration and walk the partition's range [s, e) with stride 4, exactly
// the walk of Algorithm 1.  All G query heads of the kv head are served from the
// same K/V registers, so every KV byte is fetched once.
//
// Inside a wave one 128-bit load per lane covers 64/LPR token rows (LPR = d/8 lanes
// per row); logits are reduced over the LPR lanes of a row with DPP, and every row
// group keeps its own running (max, sum, acc), merged once after the loop.
#include "kv_common.h"

namespace kvp {

template <Elem E, int D, int G, int BS>
__global__ __launch_bounds__(kWavesPerWG* kWaveSize) void attn_valu_kernel(AttnParams p) {
    constexpr int LPR = D / 8;               // lanes per token row
    constexpr int ROWS = kWaveSize / LPR;    // token rows per wave-wide load
    constexpr int LOADS = BS / ROWS;         // wave-wide loads per K (or V) tile
    constexpr int W = kWavesPerWG;

    const int part = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid / kWaveSize, lane = tid % kWaveSize;
    const int row = lane / LPR, cc = lane % LPR;

    int n = p.context_lens[b];
    n = min(max(n, 0), p.MB * BS);
    const int nblocks = (n + BS - 1) / BS;
    const int s = part * p.part_blocks;
    const bool direct = (p.NP == 1);
    if (s >= nblocks && !(direct && part == 0)) return;   // nothing to do; the combine kernel skips it
    const int e = min(nblocks, s + p.part_blocks);

    __shared__ float red_acc[W][G][D];
    __shared__ float red_m[W][G];
    __shared__ float red_l[W][G];

    float qf[G][8], acc[G][8], m[G], l[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int64_t qoff = (int64_t)b * p.q_stride_b + (int64_t)(kvh * G + g) * p.q_stride_h + cc * 8;
        const uint4 raw = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(p.q) + qoff);
        const uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float lo, hi;
            unpack2<E>(w4[i], lo, hi);
            qf[g][2 * i] = lo * p.scale_log2e;
            qf[g][2 * i + 1] = hi * p.scale_log2e;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;
        m[g] = kNegBig;
        l[g] = 0.f;
    }

    const int32_t* bt = p.block_tables + (int64_t)b * p.bt_stride_b;
    const uint16_t* kbase = reinterpret_cast<const uint16_t*>(p.k_cache) + (int64_t)kvh * p.kv_stride_h;
    const uint16_t* vbase = reinterpret_cast<const uint16_t*>(p.v_cache) + (int64_t)kvh * p.v_stride_h;
    const bool lookahead = p.prefetch_distance > 0;

    uint4 kr[LOADS], vr[LOADS], kn[LOADS], vn[LOADS];
    auto fetch = [&](int blk, uint4* kd, uint4* vd) {
        int phys = bt[blk];
        phys = min(max(phys, 0), p.NBLK - 1);
        const uint4* kp = reinterpret_cast<const uint4*>(kbase + (int64_t)phys * p.kv_stride_blk) + lane;
        const uint4* vp = reinterpret_cast<const uint4*>(vbase + (int64_t)phys * p.v_stride_blk) + lane;
#pragma unroll
        for (int r = 0; r < LOADS; ++r) kd[r] = kp[r * kWaveSize];
#pragma unroll
        for (int r = 0; r < LOADS; ++r) vd[r] = vp[r * kWaveSize];
    };

    int blk = s + wave;
    if (lookahead && blk < e) fetch(blk, kn, vn);
    for (; blk < e; blk += W) {
        if (lookahead) {
            // Algorithm 1 order: take the current tile, issue the next one (guarded by < e), compute.
#pragma unroll
            for (int r = 0; r < LOADS; ++r) { kr[r] = kn[r]; vr[r] = vn[r]; }
            if (blk + W < e) fetch(blk + W, kn, vn);
        } else {
            fetch(blk, kr, vr);
        }
        const bool tail = (blk + 1) * BS > n;
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            const int t = blk * BS + r * ROWS + row;
            const bool valid = t < n;
            uint4 vraw = vr[r];
            if (tail && !valid) vraw = make_uint4(0, 0, 0, 0);   // select, never multiply by zero
            float kf[8], vf[8];
            const uint32_t kw[4] = {kr[r].x, kr[r].y, kr[r].z, kr[r].w};
            const uint32_t vw[4] = {vraw.x, vraw.y, vraw.z, vraw.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                unpack2<E>(kw[i], kf[2 * i], kf[2 * i + 1]);
                unpack2<E>(vw[i], vf[2 * i], vf[2 * i + 1]);
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) dot = fmaf(qf[g][i], kf[i], dot);
                dot = group_sum<LPR>(dot);
                const float sc = valid ? dot : -INFINITY;
                const float m_new = fmaxf(m[g], sc);
                const float alpha = fast_exp2(m[g] - m_new);
                const float pr = fast_exp2(sc - m_new);
                l[g] = l[g] * alpha + pr;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[g][i] = fmaf(pr, vf[i], acc[g][i] * alpha);
                m[g] = m_new;
            }
        }
    }

    // merge the row groups of the wave (log-sum-exp merge), then the waves through LDS
#pragma unroll
    for (int off = LPR; off < kWaveSize; off *= 2) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m_o = __shfl_xor(m[g], off);
            const float l_o = __shfl_xor(l[g], off);
            const float m_new = fmaxf(m[g], m_o);
            const float a = fast_exp2(m[g] - m_new), c = fast_exp2(m_o - m_new);
            l[g] = l[g] * a + l_o * c;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g][i] = acc[g][i] * a + __shfl_xor(acc[g][i], off) * c;
            m[g] = m_new;
        }
    }
    if (row == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int i = 0; i < 8; ++i) red_acc[wave][g][cc * 8 + i] = acc[g][i];
            if (cc == 0) { red_m[wave][g] = m[g]; red_l[wave][g] = l[g]; }
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += W * kWaveSize) {
        const int g = idx / D, c = idx % D;
        float ms = red_m[0][g];
#pragma unroll
        for (int w = 1; w < W; ++w) ms = fmaxf(ms, red_m[w][g]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const float wgt = fast_exp2(red_m[w][g] - ms);
            num += wgt * red_acc[w][g][c];
            den += wgt * red_l[w][g];
        }
        const int h = kvh * G + g;
        if (direct) {
            const float o = den > 0.f ? num / den : 0.f;
            reinterpret_cast<uint16_t*>(p.out)[(int64_t)b * p.out_stride_b + (int64_t)h * p.out_stride_h + c] = pack1<E>(o);
        } else {
            float* dst = p.partials + (((int64_t)b * p.Hq + h) * p.NP + part) * (D + 2);
            dst[c] = num;
            if (c == 0) { dst[D] = ms; dst[D + 1] = den; }
        }
    }
}

template <Elem E, int D, int BS>
static int launch_g(const AttnParams& p, hipStream_t stream) {
    dim3 grid(p.NP, p.Hkv, p.B), block(kWavesPerWG * kWaveSize);
    switch (p.G) {
#define KVP_CASE(GV) case GV: hipLaunchKernelGGL((attn_valu_kernel<E, D, GV, BS>), grid, block, 0, stream, p); return 0;
        KVP_CASE(1) KVP_CASE(2) KVP_CASE(3) KVP_CASE(4) KVP_CASE(5) KVP_CASE(6) KVP_CASE(7) KVP_CASE(8)
#undef KVP_CASE
        default: return -1;
    }
}

template <Elem E>
static int launch_e(const AttnParams& p, int d, int bs, hipStream_t stream) {
    if (d == 128 && bs == 16) return launch_g<E, 128, 16>(p, stream);
    if (d == 128 && bs == 32) return launch_g<E, 128, 32>(p, stream);
    if (d == 64 && bs == 16) return launch_g<E, 64, 16>(p, stream);
    if (d == 64 && bs == 32) return launch_g<E, 64, 32>(p, stream);
    return -1;
}

int launch_attn_valu(const AttnParams& p, int elem, int d, int bs, hipStream_t stream) {
    return elem == (int)Elem::F16 ? launch_e<Elem::F16>(p, d, bs, stream)
                                  : launch_e<Elem::BF16>(p, d, bs, stream);
}

}  // namespace kvp
