// Paged decode attention in the two-phase form of the kernel the paper patches (Sections 3.1 and 3.2):
// first the logits of a run of tokens against all their K blocks, kept in shared memory, then the
// softmax weights applied to the V blocks; the next K block is prefetched while the current one is
// multiplied, and the next V block while the current one is accumulated.  A comparison variant of the
// one-pass kernel in decode_attn_mfma.hip: same work mapping (flat tile space, one contiguous range per
// persistent wave), same MFMA tile math, same partial pieces and finalize kernel, same results up to
// rounding.
//
// A wave cuts its range into chunks of up to 32 tiles (512 tokens, the partition of the two-phase
// kernels the paper builds on) that stay inside one (sequence, kv head) unit.  Per chunk:
//   phase 1   for every K tile: S^T = K Q^T, scaled, masked, written to the chunk's logits buffer in
//             LDS; running maximum of the chunk;
//   between   m_new = max(m, chunk maximum); accumulators and sum rescaled by 2^(m - m_new);
//   phase 2   for every V tile: logits back from LDS, P = 2^(S - m_new), O^T += V^T P^T, sum += P.
// Chunks of one unit are chained by the usual running (m, l, O) recurrence.
//
// Fetch stream: the tiles in consumption order (K tiles of a chunk, V tiles of the chunk, next
// chunk ...) go through a ring of 2 PD + 1 single-tile LDS stages; the fetch cursor runs 2 PD tiles
// ahead of the consumer, across phase and chunk boundaries, so the bytes in flight are those of the
// one-pass kernel at the same prefetch distance.  PD = 0: fetch, wait, compute.
#include "attn_device.h"

namespace kvp {

namespace {

constexpr int kChunkTiles = 32;

__device__ __forceinline__ void lds_write_b128(uint32_t a, float4v v) {
    asm volatile("ds_write_b128 %0, %1" : : "v"(a), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_read_b128(float4v& r, uint32_t a) {
    asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(a) : "memory");
}
__device__ __forceinline__ void lds_wait_all(float4v& s, u32x2 (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(s), "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) : : "memory");
}
__device__ __forceinline__ void lds_wait_all(float4v& s, u32x2 (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(s), "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 :
                 : "memory");
}

// Position in the consumption order of a worker's range: chunk, phase, tile within the chunk.
struct Stream {
    Cursor chunk0;      // first tile of the chunk
    Cursor cur;         // tile `k` of the chunk
    int64_t r_chunk;    // flat index of the chunk's first tile
    int c;              // tiles of the chunk
    int k;              // tile within the chunk
    bool v;             // false: K tiles (phase 1), true: V tiles (phase 2)
    bool done;          // past the end of the range
};

template <Elem E, int D, int BS, int PD>
__global__ __launch_bounds__(kWaveSize) void attn_twophase_kernel(AttnParams p) {
    using G_ = Geo<D>;
    constexpr int LA = 2 * PD;                  // look-ahead in single-tile stages
    constexpr int NS = LA + 1;
    constexpr int TPB = BS / kTileTokens;
    constexpr int KJ = G_::kKSteps, CB = G_::kColBlocks;
    constexpr int kRowBytes = G_::kRowBytes, kTileBytes = G_::kTileBytes;
    constexpr int LPT = kTileBytes / 1024;      // wave-wide 1 KB fetches per tile
    constexpr int kRing = NS * kTileBytes;      // the logits buffer follows the ring
    constexpr int kPartialStride = G_::kPartialStride;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int worker = blockIdx.x;
    const int lane = threadIdx.x;
    const int lq = lane / 16, lr = lane % 16;
    const int G = p.G, Hkv = p.Hkv;
    const int max_len = p.MB * BS;
    const_i32_ptr cl = (const_i32_ptr)p.context_lens;
    const_i32_ptr bt = (const_i32_ptr)p.block_tables;

    // ---- this worker's range of the flat tile space
    const int total = scan_total(cl, p.B, max_len, lane, kTileShift);
    const int64_t T = (int64_t)total * Hkv;
    const int nw = T < p.num_workers ? (int)T : p.num_workers;
    if (worker >= nw) return;
    const int skew = effective_skew(T, nw, p.xcd_skew);
    const int64_t r0 = range_start(worker, T, nw, skew);
    const int64_t r1 = range_start(worker + 1, T, nw, skew);
    Cursor first;
    {
        int b0, cum0, n0;
        scan_locate(cl, p.B, max_len, lane, kTileShift, Hkv, r0, b0, cum0, n0);
        first.b = b0;
        first.n = n0;
        first.ntiles = tiles_of(n0, kTileShift);
        const int rem = (int)(r0 - (int64_t)Hkv * cum0);
        first.kvh = rem / first.ntiles;
        first.j = rem - first.kvh * first.ntiles;
    }
    auto advance = [&](Cursor& c) {              // step to the next flat tile; the caller knows one exists
        if (++c.j < c.ntiles) return;
        c.j = 0;
        if (++c.kvh < Hkv) return;
        c.kvh = 0;
        do {
            ++c.b;
            c.n = clamp_len(cl[c.b], max_len);
            c.ntiles = tiles_of(c.n, kTileShift);
        } while (c.ntiles == 0 && c.b + 1 < p.B);
    };
    auto chunk_tiles = [&](const Cursor& c, int64_t r) {     // chunk that starts at tile c (flat index r)
        const int in_unit = c.ntiles - c.j;
        const int64_t in_range = r1 - r;
        int n = in_unit < kChunkTiles ? in_unit : kChunkTiles;
        return in_range < n ? (int)in_range : n;
    };
    auto start_stream = [&](Stream& s) {
        s.chunk0 = first; s.cur = first; s.r_chunk = r0; s.c = chunk_tiles(first, r0); s.k = 0; s.v = false; s.done = false;
    };
    auto next = [&](Stream& s) {                 // one step in consumption order
        if (++s.k < s.c) { ++s.cur.j; return; }  // the next tile of the chunk lies in the same unit
        s.k = 0;
        if (!s.v) { s.v = true; s.cur = s.chunk0; return; }
        s.v = false;
        s.r_chunk += s.c;
        if (s.r_chunk >= r1) { s.done = true; return; }
        advance(s.cur);                          // from the chunk's last tile to the first tile of the next chunk
        s.chunk0 = s.cur;
        s.c = chunk_tiles(s.cur, s.r_chunk);
    };

    // ---- Q^T operand of a unit
    u32x4 qb[KJ];
    auto load_q = [&](int b, int kvh) {
        const uint16_t* qrow = reinterpret_cast<const uint16_t*>(p.q) + (int64_t)b * p.q_stride_b +
                               (int64_t)(kvh * G + min(lr, G - 1)) * p.q_stride_h;
#pragma unroll
        for (int j = 0; j < KJ; ++j) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(qrow + (4 * j + lq) * 8);
            qb[j] = lr < G ? v : u32x4{0, 0, 0, 0};
        }
    };
    load_q(first.b, first.kvh);

    // ---- per-lane byte offsets (as in the one-pass kernel; a stage holds one tile)
    uint32_t koff[LPT], voff[LPT];
#pragma unroll
    for (int r = 0; r < LPT; ++r) {
        const int t = r * G_::kRowsPerLoad + lane / G_::kChunks, stored = lane % G_::kChunks;
        koff[r] = t * kRowBytes + ((stored ^ G_::swz_k(t)) << 4);
        voff[r] = t * kRowBytes + ((stored ^ G_::swz_v(t)) << 4);
    }
    uint32_t kread[KJ];
#pragma unroll
    for (int j = 0; j < KJ; ++j) kread[j] = lr * kRowBytes + (((4 * j + lq) ^ G_::swz_k(lr)) << 4);
    const int vt = lane / 4;
    uint32_t vread[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
        vread[cb] = vt * kRowBytes + (((2 * cb + (lane % 4) / 2) ^ G_::swz_v(vt)) << 4) + ((lane % 2) << 3);
    // logits of tile k of the chunk: G heads x 16 tokens of fp32; this lane owns tokens 4 lq .. + 4 of head lr
    // (lanes of the padding heads lr >= G keep theirs in no buffer: they compute on zeros and write nothing)
    const uint32_t ring_addr = (uint32_t)(uintptr_t)KVP_LDS(smem);
    const uint32_t logit_addr = ring_addr + kRing + (lr * 16 + 4 * lq) * 4;
    const uint32_t logit_tile = G * 64;           // bytes of one tile's logits

    const unsigned char* kcache = reinterpret_cast<const unsigned char*>(p.k_cache);
    const unsigned char* vcache = reinterpret_cast<const unsigned char*>(p.v_cache);
    auto issue = [&](const Stream& s, int stage) {   // asynchronous fetch of the K or the V tile the stream points at
        int phys = bt[(int64_t)s.cur.b * p.bt_stride_b + s.cur.j / TPB];
        phys = __builtin_amdgcn_readfirstlane(min(max(phys, 0), p.NBLK - 1));
        const int sub = (s.cur.j % TPB) * kTileBytes;
        const unsigned char* tile = s.v ? vcache + ((int64_t)phys * p.v_stride_blk + (int64_t)s.cur.kvh * p.v_stride_h) * 2 + sub
                                        : kcache + ((int64_t)phys * p.kv_stride_blk + (int64_t)s.cur.kvh * p.kv_stride_h) * 2 + sub;
        unsigned char* dst = smem + stage * kTileBytes;
#pragma unroll
        for (int r = 0; r < LPT; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GLOBAL(tile + (s.v ? voff[r] : koff[r])), KVP_LDS(dst + r * 1024), 16, 0, kAuxNonTemporal);
    };

    float4v o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) o[cb] = float4v{0.f, 0.f, 0.f, 0.f};
    float m = kNegBig, l = 0.f, m_chunk = kNegBig;

    // ---- prologue: the fetch stream runs LA tiles ahead of the consumer
    Stream fs, cs;
    start_stream(fs);
    start_stream(cs);
    if constexpr (LA > 0) {
#pragma unroll
        for (int k = 0; k < LA; ++k)
            if (!fs.done) { issue(fs, k); next(fs); }
    }

    int stage = 0;
    int piece_first_j = first.j;                  // where the current piece of the current unit began
    bool piece_at_range_start = true;
    while (!cs.done) {
        if constexpr (LA == 0) {
            issue(fs, 0);
            next(fs);
            wait_vmcnt<0>();
        } else {
            int ahead_stage = stage + LA; if (ahead_stage >= NS) ahead_stage -= NS;
            if (!fs.done) {
                issue(fs, ahead_stage);
                next(fs);
                wait_vmcnt<LPT * LA>();            // everything older than the LA newest tiles has landed
            } else {
                wait_vmcnt<0>();
            }
        }
        asm volatile("" ::: "memory");
        const uint32_t st = ring_addr + stage * kTileBytes;
        const int n = cs.cur.n;
        const int tok0 = cs.cur.j * kTileTokens + 4 * lq;
        const bool tail = (cs.cur.j + 1) * kTileTokens > n;    // wave-uniform

        if (!cs.v) {
            // ---- phase 1: logits of this K tile into the chunk's buffer
            u32x4 ka[KJ];
            if constexpr (KJ == 4) {
                lds_read_b128_x4(ka[0], ka[1], ka[2], ka[3], st + kread[0], st + kread[1], st + kread[2], st + kread[3]);
                lds_wait_k<0>(ka[0], ka[1], ka[2], ka[3]);
            } else {
                lds_read_b128_x2(ka[0], ka[1], st + kread[0], st + kread[1]);
                lds_wait_k<0>(ka[0], ka[1]);
            }
            float4v sacc = mfma_k32<E>(ka[0], qb[0], float4v{0.f, 0.f, 0.f, 0.f});
            float4v sacc1 = mfma_k32<E>(ka[1], qb[1], float4v{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int j = 2; j < KJ; j += 2) {
                sacc = mfma_k32<E>(ka[j], qb[j], sacc);
                sacc1 = mfma_k32<E>(ka[j + 1], qb[j + 1], sacc1);
            }
            sacc += sacc1;
            float4v sc;
#pragma unroll
            for (int i = 0; i < 4; ++i) sc[i] = sacc[i] * p.scale_log2e;
            if (tail) {
#pragma unroll
                for (int i = 0; i < 4; ++i) sc[i] = (tok0 + i < n) ? sc[i] : -INFINITY;    // select, not multiply
            }
            m_chunk = fmaxf(m_chunk, group_max(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]))));
            if (lr < G) lds_write_b128(logit_addr + cs.k * logit_tile, sc);
            if (cs.k + 1 == cs.c) {                // the chunk's logits are complete: move the running maximum
                const float m_new = fmaxf(m, m_chunk);
                const float alpha = fast_exp2(m - m_new);
                l *= alpha;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) o[cb] *= alpha;
                m = m_new;
                m_chunk = kNegBig;
            }
        } else {
            // ---- phase 2: weights of this tile's tokens from the buffer, applied to the V tile
            u32x2 va[CB];
            float4v sc;
#pragma unroll
            for (int c4 = 0; c4 < CB; c4 += 4)
                lds_read_tr16_x4(va[c4], va[c4 + 1], va[c4 + 2], va[c4 + 3], st + vread[c4], st + vread[c4 + 1], st + vread[c4 + 2], st + vread[c4 + 3]);
            sc = float4v{0.f, 0.f, 0.f, 0.f};
            if (lr < G) lds_read_b128(sc, logit_addr + cs.k * logit_tile);
            lds_wait_all(sc, va);
            if (tail) {
                // masked tokens: zero their V values so garbage (NaN) cannot reach the accumulators
                const uint32_t m01 = ((tok0 + 0 < n) ? 0x0000ffffu : 0u) | ((tok0 + 1 < n) ? 0xffff0000u : 0u);
                const uint32_t m23 = ((tok0 + 2 < n) ? 0x0000ffffu : 0u) | ((tok0 + 3 < n) ? 0xffff0000u : 0u);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) { va[cb][0] &= m01; va[cb][1] &= m23; }
            }
            float pr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pr[i] = fast_exp2(sc[i] - m);
            l += (pr[0] + pr[1]) + (pr[2] + pr[3]);
            const u32x2 pb = {pack2<E>(pr[0], pr[1]), pack2<E>(pr[2], pr[3])};
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) o[cb] = mfma_k16<E>(va[cb], pb, o[cb]);
        }

        if constexpr (LA > 0) { stage = stage + 1 == NS ? 0 : stage + 1; }

        // ---- end of a chunk's phase 2: end of this unit's piece?
        const bool chunk_end = cs.v && cs.k + 1 == cs.c;
        const Cursor at = cs.cur;                  // the tile just consumed
        const bool range_end = chunk_end && cs.r_chunk + cs.c == r1;
        const bool unit_end = chunk_end && at.j + 1 == at.ntiles;
        if (unit_end || range_end) {
            const float lt = group_sum(l);
            if (lr < G) {
                if (piece_first_j == 0 && unit_end) {           // the whole unit was ours: final rows
                    const float inv = p.out_scale / lt;
                    uint16_t* orow = reinterpret_cast<uint16_t*>(p.out) + (int64_t)at.b * p.out_stride_b +
                                     (int64_t)(at.kvh * G + lr) * p.out_stride_h + 4 * lq;
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        const u32x2 w = {pack2<E>(o[cb][0] * inv, o[cb][1] * inv), pack2<E>(o[cb][2] * inv, o[cb][3] * inv)};
                        *reinterpret_cast<u32x2*>(orow + 16 * cb) = w;
                    }
                } else {                                        // a cut unit: unnormalised partial for the finalize kernel
                    const int slot = piece_at_range_start ? 0 : 1;
                    float* dst = p.partials + ((int64_t)(worker * 2 + slot) * G + lr) * kPartialStride;
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) *reinterpret_cast<float4v*>(dst + 16 * cb + 4 * lq) = o[cb];
                    if (lq == 0) { dst[D] = m; dst[D + 1] = lt; }
                }
            }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) o[cb] = float4v{0.f, 0.f, 0.f, 0.f};
            m = kNegBig;
            l = 0.f;
            piece_at_range_start = false;
        }
        next(cs);
        if (unit_end && !cs.done) {
            piece_first_j = 0;
            load_q(cs.cur.b, cs.cur.kvh);
        }
    }
}

template <Elem E, int D, int BS, int PD>
int launch_one(const AttnParams& p, hipStream_t stream) {
    auto kern = attn_twophase_kernel<E, D, BS, PD>;
    const int lds = twophase_worker_lds_bytes(PD, D, p.G);
    // beyond the default limit of dynamic LDS the limit is raised, once, to what the widest group of query heads
    // needs: the size of a launch depends on the call's group size, the limit must cover every later call
    constexpr int kMaxGroup = 16;
    const int lds_max = twophase_worker_lds_bytes(PD, D, kMaxGroup);
    if (p.G > kMaxGroup) return -1;
    if (lds_max > 64 * 1024) {
        static LdsLimit limit;
        if (limit.raise(reinterpret_cast<const void*>(kern), lds_max) != 0) return -1;
    }
    hipLaunchKernelGGL(kern, dim3(p.num_workers), dim3(kWaveSize), (size_t)lds, stream, p);
    return 0;
}

template <Elem E, int D, int BS>
int launch_pd(const AttnParams& p, hipStream_t stream) {
    switch (p.prefetch_distance) {
        case 0: return launch_one<E, D, BS, 0>(p, stream);
        case 1: return launch_one<E, D, BS, 1>(p, stream);
        case 2: return launch_one<E, D, BS, 2>(p, stream);
        case 3: return launch_one<E, D, BS, 3>(p, stream);
        case 4: return launch_one<E, D, BS, 4>(p, stream);
        default: return -1;
    }
}

template <Elem E>
int launch_shape(const AttnParams& p, int d, int bs, hipStream_t stream) {
    if (d == 128) return bs == 16 ? launch_pd<E, 128, 16>(p, stream) : launch_pd<E, 128, 32>(p, stream);
    return bs == 16 ? launch_pd<E, 64, 16>(p, stream) : launch_pd<E, 64, 32>(p, stream);
}

}  // namespace

// LDS bytes one worker holds: 2 PD + 1 single-tile stages and the logits of a chunk (32 tiles x G heads x 16
// tokens of fp32).
int twophase_worker_lds_bytes(int prefetch_distance, int d, int G) {
    const int tile = d == 128 ? Geo<128>::kTileBytes : Geo<64>::kTileBytes;
    return (2 * prefetch_distance + 1) * tile + kChunkTiles * G * 64;
}

// Returns 0 or -1 (no such instantiation).
int launch_attn_twophase(const AttnParams& p, int elem, int d, int bs, hipStream_t stream) {
    if (p.num_workers < 1 || p.num_workers > kMaxMfmaWorkers || p.tile_shift != kTileShift) return -1;
    if (d != 64 && d != 128) return -1;
    if (bs != 16 && bs != 32) return -1;
    return elem == (int)Elem::F16 ? launch_shape<Elem::F16>(p, d, bs, stream) : launch_shape<Elem::BF16>(p, d, bs, stream);
}

}  // namespace kvp
