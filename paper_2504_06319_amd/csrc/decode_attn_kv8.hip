// Paged decode attention over an 8-bit (FP8 E4M3) KV cache, q and out in a 16-bit type.
//
// The same persistent-worker scheme as the 16-bit kernel (flat tile space cut into one contiguous range per
// wave, LDS ring of PD + 1 stages filled by asynchronous global->LDS fetches that run PD tiles ahead of the
// compute: Algorithm 1 of the paper at distance PD), with tiles of 32 tokens: a K (or V) tile of 32 rows of d
// one-byte codes has the bytes of a 16-bit tile of 16 rows, so stages, fetch counts and the look-ahead in
// bytes are those of the 16-bit kernel, and the per-tile bookkeeping is paid once per 32 tokens.
//
// The ring holds the raw codes as they are in HBM.  Widening to the query's 16-bit type happens in registers
// (v_cvt_scalef32_pk_*_fp8, exact: both 16-bit types hold every E4M3 value), so the products are the 16-bit
// MFMAs of the 16-bit kernel:
//   S^T[t, g]  = sum_c K[t, c] Q[g, c]     2 row blocks x d/32 v_mfma_f32_16x16x32; A = eight codes of a K row,
//                                          read with ds_read_b64 and widened
//   O^T[c, g] += sum_t V[t, c] P^T[t, g]   d/16 v_mfma_f32_16x16x32 over the 32 tokens; A = V^T, eight tokens of
//                                          one column per lane, read with the 8-bit transpose read
//                                          (ds_read_b64_tr_b8) and widened
// Row r of S row block rb is token 8 (r / 4) + 4 rb + r % 4 of the tile, so that lane group lq ends up holding
// the logits of tokens 8 lq .. 8 lq + 7: the eight tokens whose V values the transpose read gives that group.
//
// ds_read_b64_tr_b8, per group of 16 lanes: lanes 2k and 2k + 1 read the two 8-byte halves of a 16-byte row k
// (k = 0..7); lane c of the group receives byte c of rows 0..7.  Here row k of group lq is token 8 lq + k and
// the 16 bytes are columns 16 cb .. + 16.
//
// LDS layout of a stage: K tile then V tile, each 32 rows of d bytes, written by global_load_lds_dwordx4 (lane
// i of load r lands at 1024 r + 16 i).  The 16-byte chunk a lane fetches is permuted (chunk index XOR a function
// of the row) so that the 16 rows an operand read touches in one pass fall into different banks.
#include "attn_device.h"

namespace kvp {

namespace {

constexpr int kTileShift8 = 5;
constexpr int kTileTokens8 = 32;

template <int D>
struct Geo8 {
    static constexpr int kTileBytes = kTileTokens8 * D;           // 4 KB (d 128) / 2 KB (d 64) for K, the same for V
    static constexpr int kStageBytes = 2 * kTileBytes;
    static constexpr int kChunks = D / 16;                        // 16-byte chunks per row
    static constexpr int kRowsPerLoad = kWaveSize / kChunks;      // rows one wave-wide 1 KB fetch lands: 8 / 16
    static constexpr int kKSteps = D / 32;
    static constexpr int kColBlocks = D / 16;
    static constexpr int kPartialStride = D + 4;                  // as in the 16-bit kernel: the finalize kernel is shared
    // An operand read of K takes, per pass, 16 bytes of each of the rows {0..3, 8..11, 16..19, 24..27} (+ 4 for the
    // second row block); a transpose read of V 16 bytes of rows 0..15 (or 16..31).  256 / d rows share a 256-byte
    // bank line; the swizzle gives the rows of a pass that share a line position different chunk positions.
    __host__ __device__ static constexpr int swz_k(int row) {
        return D == 128 ? (((row >> 1) & 1) | (((row >> 3) & 3) << 1)) : ((row >> 3) & 3);
    }
    __host__ __device__ static constexpr int swz_v(int row) { return D == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
};

__device__ __forceinline__ void lds_read_b64(u32x2& r, uint32_t a) {
    asm volatile("ds_read_b64 %0, %1" : "=v"(r) : "v"(a) : "memory");
}
__device__ __forceinline__ void lds_read_tr8(u32x2& r, uint32_t a) {
    asm volatile("ds_read_b64_tr_b8 %0, %1" : "=v"(r) : "v"(a) : "memory");
}
// Wait until at most N of this wave's LDS operations are outstanding; the registers are passed through so that
// no use of them can be scheduled above the wait.
template <int N>
__device__ __forceinline__ void lds_wait(u32x2 (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_wait(u32x2 (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 : "n"(N)
                 : "memory");
}

// eight codes (two dwords) -> eight 16-bit values, the k-operand of one lane of a 16x16x32 MFMA
template <Elem E>
__device__ __forceinline__ u32x4 widen8(u32x2 raw) {
    const uint32_t w0 = raw[0], w1 = raw[1];
    const u32x2 e0 = widen_fp8x4<E>(w0), e1 = widen_fp8x4<E>(w1);
    const uint32_t a0 = e0[0], a1 = e0[1], a2 = e1[0], a3 = e1[1];
    return u32x4{a0, a1, a2, a3};
}

template <Elem E, int D, int BS, int PD>
__global__ __launch_bounds__(kWaveSize) void attn_kv8_kernel(AttnParams p) {
    using G_ = Geo8<D>;
    constexpr int NS = PD + 1;                      // LDS stages of the wave
    constexpr int BPT = kTileTokens8 / BS;          // KV blocks a tile spans: 2 (block_size 16) or 1
    constexpr int KJ = G_::kKSteps, CB = G_::kColBlocks;
    constexpr int kTileBytes = G_::kTileBytes, kStageBytes = G_::kStageBytes;
    constexpr int LPT = kTileBytes / 1024;          // wave-wide 1 KB fetches per K (or V) tile
    constexpr int LOADS = 2 * LPT;
    constexpr int kPartialStride = G_::kPartialStride;
    static_assert(BPT == 1 || BPT == 2, "block_size 16 or 32");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int worker = blockIdx.x;
    const int lane = threadIdx.x;
    const int lq = lane / 16, lr = lane % 16;
    const int G = p.G, Hkv = p.Hkv;
    const bool traced = p.worker_trace != nullptr;
    const unsigned long long t_entry = traced ? wall_clock64() : 0;
    const int max_len = p.MB * BS;
    const_i32_ptr cl = (const_i32_ptr)p.context_lens;
    const_i32_ptr bt = (const_i32_ptr)p.block_tables;

    // ---- this worker's range of the flat tile space (32-token tiles)
    const int total = scan_total(cl, p.B, max_len, lane, kTileShift8);
    const int64_t T = (int64_t)total * Hkv;
    const int nw = T < p.num_workers ? (int)T : p.num_workers;
    if (worker >= nw) return;
    const int skew = effective_skew(T, nw, p.xcd_skew);
    const int64_t r0 = range_start(worker, T, nw, skew);
    const int64_t r1 = range_start(worker + 1, T, nw, skew);
    Cursor ca;
    {
        int b0, cum0, n0;
        scan_locate(cl, p.B, max_len, lane, kTileShift8, Hkv, r0, b0, cum0, n0);
        ca.b = b0;
        ca.n = n0;
        ca.ntiles = tiles_of(ca.n, kTileShift8);
        const int rem = (int)(r0 - (int64_t)Hkv * cum0);
        ca.kvh = rem / ca.ntiles;
        ca.j = rem - ca.kvh * ca.ntiles;
    }
    auto advance = [&](Cursor& c) {              // step to the next flat tile (the caller knows one exists); true when it belongs to another unit
        if (++c.j < c.ntiles) return false;
        c.j = 0;
        if (++c.kvh < Hkv) return true;
        c.kvh = 0;
        do {
            ++c.b;
            c.n = clamp_len(cl[c.b], max_len);
            c.ntiles = tiles_of(c.n, kTileShift8);
        } while (c.ntiles == 0 && c.b + 1 < p.B);
        return true;
    };

    // ---- Q^T operand of a unit: lane (g = lr, lq) holds Q[g][(4j + lq) * 8 .. +8], zero rows for g >= G.  As in the
    // 16-bit kernel the unit's query rows are fetched by global_load_lds into a ring of PD + 1 query images (16 rows of
    // 16-bit values, laid out and read like that kernel's K tile) just ahead of the unit's first tile, so that no
    // ordinary load at a unit boundary makes the wave wait for everything it has in flight.
    using GQ = Geo<D>;
    constexpr int kQBytes = GQ::kQueryBytes;
    constexpr int QL = kQBytes / 1024;             // wave-wide 1 KB fetches per query image
    u32x4 qb[KJ];
    uint32_t qoff[QL], qread[KJ];
#pragma unroll
    for (int r = 0; r < QL; ++r) {
        const int t = r * GQ::kRowsPerLoad + lane / GQ::kChunks, stored = lane % GQ::kChunks;
        qoff[r] = (uint32_t)((int64_t)min(t, G - 1) * p.q_stride_h * 2 + ((stored ^ GQ::swz_k(t)) << 4));
    }
#pragma unroll
    for (int j = 0; j < KJ; ++j) qread[j] = lr * GQ::kRowBytes + (((4 * j + lq) ^ GQ::swz_k(lr)) << 4);
    const unsigned long long t_scan = traced ? wall_clock64() : 0;

    // ---- per-lane byte offsets, loop invariant
    // fetch r of a tile lands rows r * kRowsPerLoad ..; this lane lands row t at stored chunk lane % kChunks, so it
    // fetches chunk (stored ^ swizzle(t)) of row t.  Row t is row t % BS of KV block t / BS of the tile.
    uint32_t koff[LPT], voff[LPT];
#pragma unroll
    for (int r = 0; r < LPT; ++r) {
        const int t = r * G_::kRowsPerLoad + lane / G_::kChunks, stored = lane % G_::kChunks;
        koff[r] = (t % BS) * D + ((stored ^ G_::swz_k(t)) << 4);
        voff[r] = (t % BS) * D + ((stored ^ G_::swz_v(t)) << 4);
    }
    // K operand of row block rb, step j: row 8 (lr / 4) + 4 rb + lr % 4, bytes 32 j + 8 lq .. + 8
    uint32_t kread[2][KJ];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int row = 8 * (lr / 4) + 4 * rb + lr % 4;
#pragma unroll
        for (int j = 0; j < KJ; ++j)
            kread[rb][j] = row * D + (((2 * j + lq / 2) ^ G_::swz_k(row)) << 4) + ((lq % 2) << 3);
    }
    // V transpose read of column block cb: row 8 lq + lr / 2, half lr % 2 of chunk cb
    uint32_t vread[CB];
    {
        const int row = 8 * lq + lr / 2;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
            vread[cb] = kTileBytes + row * D + ((cb ^ G_::swz_v(row)) << 4) + ((lr % 2) << 3);
    }

    const uint32_t ring_addr = (uint32_t)(uintptr_t)KVP_LDS(smem);
    unsigned char* qring = smem + NS * kStageBytes;                     // query images behind the stages
    const uint32_t qring_addr = ring_addr + NS * kStageBytes;
    auto issue_q = [&](const Cursor& c, int slot) {
        const unsigned char* qrow = reinterpret_cast<const unsigned char*>(p.q) +
                                    ((int64_t)c.b * p.q_stride_b + (int64_t)c.kvh * G * p.q_stride_h) * 2;
#pragma unroll
        for (int r = 0; r < QL; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GLOBAL(qrow + qoff[r]), KVP_LDS(qring + slot * kQBytes + r * 1024), 16, 0, 0);
    };
    const unsigned char* kcache = reinterpret_cast<const unsigned char*>(p.k_cache);
    const unsigned char* vcache = reinterpret_cast<const unsigned char*>(p.v_cache);

    auto issue = [&](const Cursor& c, int stage) {   // asynchronous fetch of one K tile and one V tile into a stage
        // block table entries of the tile; the second half of a tile that ends inside its first block repeats the
        // first block (its tokens are masked), so that no entry beyond the context is ever dereferenced
        const unsigned char* kb[BPT];
        const unsigned char* vb[BPT];
#pragma unroll
        for (int h = 0; h < BPT; ++h) {
            const int blk = BPT * c.j + ((h == 0 || (BPT * c.j + h) * BS < c.n) ? h : 0);
            int phys = bt[(int64_t)c.b * p.bt_stride_b + blk];
            phys = __builtin_amdgcn_readfirstlane(min(max(phys, 0), p.NBLK - 1));
            kb[h] = kcache + (int64_t)phys * p.kv_stride_blk + (int64_t)c.kvh * p.kv_stride_h;
            vb[h] = vcache + (int64_t)phys * p.v_stride_blk + (int64_t)c.kvh * p.v_stride_h;
        }
        unsigned char* dst = smem + stage * kStageBytes;
        // every KV byte is used once: non-temporal fetches (the paper's eviction-priority remark, Section 3.3)
#pragma unroll
        for (int r = 0; r < LPT; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GLOBAL(kb[(r * G_::kRowsPerLoad) / BS] + koff[r]), KVP_LDS(dst + r * 1024), 16, 0, kAuxNonTemporal);
#pragma unroll
        for (int r = 0; r < LPT; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GLOBAL(vb[(r * G_::kRowsPerLoad) / BS] + voff[r]), KVP_LDS(dst + kTileBytes + r * 1024), 16, 0, kAuxNonTemporal);
    };

    float4v o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) o[cb] = float4v{0.f, 0.f, 0.f, 0.f};
    float m = kNegBig, l = 0.f;

    // ---- prologue: the prefetch cursor runs PD tiles ahead of the consume cursor
    Cursor cp = ca;
    int64_t rp = r0;
    bool cp_new_unit = true;                      // cp stands on the first tile of a unit's piece: its queries go first
    int q_issue = 0, q_read = 0;
    auto issue_next = [&](int stage) {
        if (cp_new_unit) {
            issue_q(cp, q_issue);
            q_issue = q_issue + 1 == NS ? 0 : q_issue + 1;
        }
        issue(cp, stage);
        cp_new_unit = ++rp < r1 ? advance(cp) : false;
    };
    if constexpr (PD > 0) {
#pragma unroll
        for (int k = 0; k < PD; ++k)
            if (rp < r1) issue_next(k);
    }

    int stage = 0;
    int piece_first_j = ca.j;
    bool piece_at_range_start = true;
    bool ca_new_unit = true;
    for (int64_t r = r0; r < r1; ++r) {
        if constexpr (PD == 0) {
            issue_next(0);
            wait_vmcnt<0>();
        } else {
            int ahead_stage = stage + PD; if (ahead_stage >= NS) ahead_stage -= NS;
            if (rp < r1) {
                issue_next(ahead_stage);
                wait_vmcnt<LOADS * PD>();          // everything older than the PD newest tiles has landed
            } else {
                wait_vmcnt<0>();
            }
        }
        asm volatile("" ::: "memory");
        if (ca_new_unit) {      // the unit's queries landed before its first tile did: into registers, rows past G zeroed
            const uint32_t qa = qring_addr + q_read * kQBytes;
            if constexpr (KJ == 4) {
                lds_read_b128_x4(qb[0], qb[1], qb[2], qb[3], qa + qread[0], qa + qread[1], qa + qread[2], qa + qread[3]);
                lds_wait_k<0>(qb[0], qb[1], qb[2], qb[3]);
            } else {
                lds_read_b128_x2(qb[0], qb[1], qa + qread[0], qa + qread[1]);
                lds_wait_k<0>(qb[0], qb[1]);
            }
#pragma unroll
            for (int j = 0; j < KJ; ++j) qb[j] = lr < G ? qb[j] : u32x4{0, 0, 0, 0};
            q_read = q_read + 1 == NS ? 0 : q_read + 1;
            ca_new_unit = false;
        }
        const uint32_t st = ring_addr + stage * kStageBytes;

        // ---- every LDS read of the tile: raw K operands of both row blocks, then the transposed raw V operands
        u32x2 kr[2 * KJ];
        u32x2 vr[CB];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int j = 0; j < KJ; ++j) lds_read_b64(kr[rb * KJ + j], st + kread[rb][j]);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) lds_read_tr8(vr[cb], st + vread[cb]);
        lds_wait<CB>(kr);

        // ---- S^T = K Q^T for the two row blocks: two independent accumulation chains
        float4v s0 = float4v{0.f, 0.f, 0.f, 0.f}, s1 = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KJ; ++j) {
            s0 = mfma_k32<E>(widen8<E>(kr[j]), qb[j], s0);
            s1 = mfma_k32<E>(widen8<E>(kr[KJ + j]), qb[j], s1);
        }
        lds_wait<0>(vr);

        // ---- online softmax over the tile's 32 tokens: this lane holds tokens 8 lq + i (s0) and 8 lq + 4 + i (s1)
        float sc[8];
        const int n = ca.n;
        const int tok0 = ca.j * kTileTokens8 + 8 * lq;
        const bool tail = (ca.j + 1) * kTileTokens8 > n;       // wave-uniform
#pragma unroll
        for (int i = 0; i < 4; ++i) { sc[i] = s0[i] * p.scale_log2e; sc[4 + i] = s1[i] * p.scale_log2e; }
        if (tail) {
            uint32_t keep[2] = {0u, 0u};           // byte masks of the eight tokens' V codes
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool valid = tok0 + i < n;
                sc[i] = valid ? sc[i] : -INFINITY;                 // select, not multiply
                keep[i / 4] |= valid ? (0xffu << (8 * (i % 4))) : 0u;
            }
            // masked tokens: zero their V codes (+0) so garbage (NaN) cannot reach the accumulators
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) { vr[cb][0] &= keep[0]; vr[cb][1] &= keep[1]; }
        }
        const float mx = group_max(fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])),
                                         fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7]))));
        const float m_new = fmaxf(m, mx);
        // The running maximum is only a reference point: any m with s - m small enough not to overflow gives the
        // same sums after the final division.  So it is moved (and the accumulators rescaled: 4 d / 16 + 2
        // multiplications and an exponential on the critical path of a lone wave) only when some head's maximum has
        // grown by more than p.rescale_slack; weights then reach at most 2^slack.  A unit's maxima move on most of
        // its first tiles and seldom by much, so this removes most of the 15 to 25 rescales per unit.
        if (__builtin_amdgcn_ballot_w64(m_new > m + p.rescale_slack) != 0) {
            const float alpha = fast_exp2(m - m_new);
            l *= alpha;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) o[cb] *= alpha;
            m = m_new;
        }
        float pr[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) pr[i] = fast_exp2(sc[i] - m);
        l += ((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7]));
        const u32x4 pb = {pack2<E>(pr[0], pr[1]), pack2<E>(pr[2], pr[3]), pack2<E>(pr[4], pr[5]), pack2<E>(pr[6], pr[7])};

        // ---- O^T += V^T P^T over the 32 tokens
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) o[cb] = mfma_k32<E>(widen8<E>(vr[cb]), pb, o[cb]);

        if constexpr (PD > 0) { stage = stage + 1 == NS ? 0 : stage + 1; }

        // ---- end of this unit's piece: write it out and start the next one
        const bool unit_end = ca.j + 1 == ca.ntiles;
        const bool range_end = r + 1 == r1;
        if (unit_end || range_end) {
            const float lt = group_sum(l);
            if (lr < G) {
                if (piece_first_j == 0 && unit_end) {           // the whole unit was ours: final rows
                    const float inv = p.out_scale / lt;         // lt > 0: a unit has at least one valid token
                    uint16_t* orow = reinterpret_cast<uint16_t*>(p.out) + (int64_t)ca.b * p.out_stride_b +
                                     (int64_t)(ca.kvh * G + lr) * p.out_stride_h + 4 * lq;
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
        if (!range_end) {
            ca_new_unit = advance(ca);
            if (ca_new_unit) piece_first_j = 0;
        }
    }
    if (traced && lane == 0) {
        unsigned long long* t = p.worker_trace + (int64_t)worker * 4;
        t[0] = t_entry; t[1] = t_scan; t[2] = wall_clock64();
        t[3] = (unsigned long long)(r1 - r0) | ((unsigned long long)xcc_id() << 32);
    }
}

template <Elem E, int D, int BS, int PD>
int launch_one(const AttnParams& p, hipStream_t stream) {
    const size_t lds = (size_t)kv8_worker_lds_bytes(PD, D);
    auto kern = attn_kv8_kernel<E, D, BS, PD>;
    hipLaunchKernelGGL(kern, dim3(p.num_workers), dim3(kWaveSize), lds, stream, p);
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

// LDS bytes one worker (wave) holds: its ring of fetched tile pairs (32 tokens each) and as many query images.
int kv8_worker_lds_bytes(int prefetch_distance, int d) {
    return (prefetch_distance + 1) * (d == 128 ? Geo8<128>::kStageBytes + Geo<128>::kQueryBytes : Geo8<64>::kStageBytes + Geo<64>::kQueryBytes);
}

// Returns 0 or -1 (no such instantiation).  elem is the type of q and out.
int launch_attn_kv8(const AttnParams& p, int elem, int d, int bs, hipStream_t stream) {
    if (p.num_workers < 1 || p.num_workers > kMaxMfmaWorkers) return -1;
    if (d != 64 && d != 128) return -1;
    if (bs != 16 && bs != 32) return -1;
    if (p.tile_shift != kTileShift8) return -1;
    return elem == (int)Elem::F16 ? launch_shape<Elem::F16>(p, d, bs, stream) : launch_shape<Elem::BF16>(p, d, bs, stream);
}

}  // namespace kvp
