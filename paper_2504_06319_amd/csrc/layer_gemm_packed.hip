// Dense layer of the layer-stack harness for weights stored in MFMA operand order:
// y[M, N] = x[M, K] . W[K, N], bf16 in, fp32 accumulate, bf16 out, M <= 128.
//
// What bounds this layer on the chip, measured with variants of this kernel: streaming W (117 MB at
// 4096 x 14336) from HBM once is the floor (18 us at 6.5 TB/s); a skinny GEMM also re-reads x (1 MB)
// once per column tile, and a compute unit takes in only about 64 bytes per clock, so the tile must
// be wide and x must be fetched once per workgroup, not once per wave.
//
// Design.
//  * W is stored so that one 16-byte load per lane IS the B operand of v_mfma_f32_16x16x32_bf16
//    (lane l holds k = 8 (l / 16) .. + 7 of column l % 16), and goes from HBM straight into
//    registers: no LDS hop, no transpose.
//        Wp[t][ks][nb][l][j] = W[32 ks + 8 (l / 16) + j][64 t + 16 nb + l % 16]
//        t < N / 64, ks < K / 32 (k-step), nb < 4, l < 64, j < 8
//  * A workgroup owns all 128 rows of a 128-column tile over HALF of K; its four waves split the
//    columns (32 each), so the x slab of a k-step ([128 m][32 k], 8 KB) is fetched once per
//    workgroup, by global_load_lds into a ring of LDS stages shared by the waves (each wave
//    fetches a quarter of every slab), and read by all of them as the A operand.  One s_barrier
//    per k-step.  Bytes taken in per compute unit: 0.5 MB of W + 0.5 MB of x.
//  * The two workgroups of a column tile (lower and upper half of K; block ids 8 apart) each
//    write their fp32 partial tile with device-scope stores and then take a ticket with a
//    device-scope atomic; the one that draws the second ticket adds the other's partial to its
//    registers and writes y.  Nobody waits for anybody, so no workgroup can hang on another.
//    The ticket word is reset by its last user (zero before the first launch and after every one).
//
// A wave's loads complete in issue order, so x (from L2) and W (from HBM) get the same look-ahead.
// Every memory operation of a wave is issued in program order by volatile statements, so the
// number of operations younger than a given one is known at compile time: the main loop is fully
// unrolled (the k-step count is a template parameter) and each wait is an exact s_waitcnt vmcnt(n)
// computed from a model of that schedule.
#include "kv_common.h"

#include <type_traits>
#include <utility>

namespace kvp {

typedef __bf16 pk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f4 __attribute__((ext_vector_type(4)));
typedef uint32_t pk_u4 __attribute__((ext_vector_type(4)));

constexpr int kPkBN = 128;                // output columns per workgroup
constexpr int kPkBM = 128;                // output rows per workgroup (all of them)
constexpr int kPkBK = 32;                 // k per step
// look-ahead: measured flat from 4 / 3 to 16 / 15 stages (32.6 - 33.8 us); the middle is used
constexpr int kPkXS = 8;                  // LDS stages of x per workgroup
constexpr int kPkWD = 7;                  // register slots (k-steps) of W per wave
constexpr int kPkXTile = kPkBM * kPkBK * 2;            // 8 KB
constexpr int kPkXOwn = 2;                             // wave-wide 1 KB fetches of a slab issued by each wave
constexpr int kPkWOwn = 2;                             // 1 KB fetches of W per wave and k-step (two 16-column blocks)
constexpr int kPkLds = kPkXS * kPkXTile;               // 64 KB

#define KVP_PK_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define KVP_PK_GLOBAL(p) ((const __attribute__((address_space(1))) void*)(p))

// ---- compile-time model of the order in which a wave issues its memory operations.
// Prologue: its parts of x(0) .. x(XS-1), then W(0) .. W(WD-1).  Step s: its parts of x(s + XS) if that
// slab exists, then, after the MFMAs of each 16-column block nb, that block's W(s + WD) if it exists.
struct PkSchedule {
    static constexpr int imin(int a, int b) { return a < b ? a : b; }
    static constexpr int prologue_x(int steps) { return imin(kPkXS, steps) * kPkXOwn; }
    static constexpr int prologue(int steps) { return prologue_x(steps) + imin(kPkWD, steps) * kPkWOwn; }
    // operations issued before step s fetches x
    static constexpr int before_step(int steps, int s) {
        int n = prologue(steps);
        for (int t = 0; t < s; ++t) {
            if (t + kPkXS < steps) n += kPkXOwn;
            if (t + kPkWD < steps) n += kPkWOwn;
        }
        return n;
    }
    // operations issued up to and including this wave's last fetch of x(j)
    static constexpr int end_of_x(int steps, int j) {
        return j < kPkXS ? (j + 1) * kPkXOwn : before_step(steps, j - kPkXS) + kPkXOwn;
    }
    // operations issued up to and including fetch nb of W(j)
    static constexpr int end_of_w(int steps, int j, int nb) {
        if (j < kPkWD) return prologue_x(steps) + j * kPkWOwn + nb + 1;
        const int t = j - kPkWD;                        // issued during step t, after that step's x fetch
        return before_step(steps, t) + (t + kPkXS < steps ? kPkXOwn : 0) + nb + 1;
    }
    static constexpr int clamp(int y) { return y > 63 ? 63 : y; }
    // at the top of step s: operations younger than this wave's last fetch of x(s + 1)
    static constexpr int younger_than_next_x(int steps, int s) {
        return clamp(before_step(steps, s) - end_of_x(steps, s + 1));
    }
    // at step s, block nb (fetches 0 .. nb-1 of W(s + WD) already issued): younger than fetch nb of W(s)
    static constexpr int younger_than_w(int steps, int s, int nb) {
        const int now = before_step(steps, s) + (s + kPkXS < steps ? kPkXOwn : 0) + (s + kPkWD < steps ? nb : 0);
        return clamp(now - end_of_w(steps, s, nb));
    }
};

// 16 bytes per lane from (wave-uniform base in scalar registers) + (lane byte offset) + OFF; non-temporal: W is
// read once per pass
// (PLAIN: without the hint, the "before" of the cache-policy comparison)
template <int OFF, bool PLAIN>
__device__ __forceinline__ void pk_load_w(pk_u4& dst, const unsigned char* base, uint32_t lane_off) {
    if constexpr (PLAIN)
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(dst) : "v"(lane_off), "s"(base), "n"(OFF) : "memory");
    else
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 nt" : "=v"(dst) : "v"(lane_off), "s"(base), "n"(OFF) : "memory");
}

template <class F, int... I>
__device__ __forceinline__ void pk_static_for(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}

template <int N>
__device__ __forceinline__ void pk_wait_w(pk_u4& r) {          // the register passes through: no use can move above the wait
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(N) : "memory");
}

template <int N>
__device__ __forceinline__ void pk_wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

__device__ __forceinline__ void pk_read_a(pk_u4 (&a)[8], uint32_t base) {
    asm volatile(
        "ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:1024\n\tds_read_b128 %2, %8 offset:2048\n\t"
        "ds_read_b128 %3, %8 offset:3072\n\tds_read_b128 %4, %8 offset:4096\n\tds_read_b128 %5, %8 offset:5120\n\t"
        "ds_read_b128 %6, %8 offset:6144\n\tds_read_b128 %7, %8 offset:7168"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(a[4]), "=&v"(a[5]), "=&v"(a[6]), "=&v"(a[7])
        : "v"(base)
        : "memory");
}

__device__ __forceinline__ void pk_wait_a(pk_u4 (&a)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
                 :
                 : "memory");
}

// STEPS = k-steps per workgroup: K = 2 halves * STEPS * 32.
// tickets: one word per column tile, zero before the first launch; partials: per column tile two fp32 tiles of
// 128 x 128 in register order.
template <int STEPS, bool PLAIN = false>
__global__ __launch_bounds__(256) void layer_gemm_packed_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wp,
                                                                uint16_t* __restrict__ y, int M, int N, int64_t ldx,
                                                                int64_t ldy, int* tickets, float* partials) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWaveSize);
    const int lane = tid % kWaveSize;
    const int lq = lane / 16, lr = lane % 16;
    // block id -> (column tile, half of K): ids i and i + 8 take the two halves of one column tile
    const int bid = blockIdx.x;
    const int tile = (bid / 16) * 8 + bid % 8, khalf = (bid / 8) % 2;
    if (tile >= N / kPkBN) return;              // both halves of a tile past the end leave together
    constexpr int KS = 2 * STEPS;               // k-steps of the whole K

    const uint32_t ring_addr = (uint32_t)(uintptr_t)KVP_PK_LDS(smem);

    // x fetch r (0..7) of a slab fills the 1 KB of m-block r; this wave issues r = 2 wave and 2 wave + 1.  A lane
    // lands position lane / 4 (0..15) of the m-block at stored chunk lane % 4.  Position p holds matrix row
    // 2 (p % 8) + p / 8 of the m-block (even rows first, then odd rows) and stored chunk c holds the row's logical
    // chunk c ^ f(p), f(p) = 2 (p / 4 % 2) + p / 8: a ds_read_b128 is served 16 lanes at a time, and both for
    // 16 consecutive lanes and for every other lane of a half wave (what the conflict counter points to: with rows
    // in natural order it read 4 conflict cycles in every 8) those 16 lanes then cover all 64 banks.  Rows >= M
    // re-read row M - 1 (their products are never stored)
    auto swz = [](int pos) { return 2 * ((pos / 4) % 2) + pos / 8; };
    uint32_t xoff[kPkXOwn];
#pragma unroll
    for (int i = 0; i < kPkXOwn; ++i) {
        const int pos = lane / 4;
        const int row = 16 * (kPkXOwn * wave + i) + 2 * (pos % 8) + pos / 8;
        const int logical = (lane % 4) ^ swz(pos);
        xoff[i] = (uint32_t)(min(row, M - 1) * ldx * 2 + logical * 16);
    }
    const unsigned char* xg = reinterpret_cast<const unsigned char*>(x) + (int64_t)khalf * STEPS * kPkBK * 2;
    // this wave's run of W: 64-column tile 2 tile + wave / 2, 16-column blocks 2 (wave % 2) and + 1 (2 KB of every
    // 4 KB k-step), k-steps khalf * STEPS .. + STEPS
    const unsigned char* wg = reinterpret_cast<const unsigned char*>(wp) +
                              ((int64_t)(2 * tile + wave / 2) * KS + (int64_t)khalf * STEPS) * 4096 + (wave % 2) * 2048;
    const uint32_t w_lane = lane * 16;
    auto load_w = [&](pk_u4 (&slot)[kPkWOwn], int kstep, auto nb_tag) {
        constexpr int nb = decltype(nb_tag)::value;
        pk_load_w<nb * 1024, PLAIN>(slot[nb], wg + (int64_t)kstep * 4096, w_lane);
    };
    // A operand of m-block mb: row 16 mb + lr sits at position lr / 2 + 8 (lr % 2), its logical chunk lq at stored
    // chunk lq ^ f(position); + 1024 per m-block
    const int a_pos = lr / 2 + 8 * (lr % 2);
    const uint32_t a_off = a_pos * 64 + ((lq ^ swz(a_pos)) << 4);

    auto issue_x = [&](int step) {
        const unsigned char* xt = xg + (int64_t)step * (kPkBK * 2);
        unsigned char* dst = smem + (step % kPkXS) * kPkXTile + (kPkXOwn * wave) * 1024;
#pragma unroll
        for (int i = 0; i < kPkXOwn; ++i)
            __builtin_amdgcn_global_load_lds(KVP_PK_GLOBAL(xt + xoff[i]), KVP_PK_LDS(dst + i * 1024), 16, 0, 0);
    };

    pk_f4 acc[8][kPkWOwn];
#pragma unroll
    for (int mb = 0; mb < 8; ++mb)
#pragma unroll
        for (int nb = 0; nb < kPkWOwn; ++nb) acc[mb][nb] = pk_f4{0.f, 0.f, 0.f, 0.f};

    pk_u4 wr[kPkWD][kPkWOwn];         // W ring: slot s % WD holds k-step s
    pk_u4 a[2][8];                    // A operands of the current and of the next k-step

    // ---- prologue (order matters: the schedule model above mirrors it)
#pragma unroll
    for (int s = 0; s < kPkXS; ++s)
        if (s < STEPS) issue_x(s);
#pragma unroll
    for (int s = 0; s < kPkWD; ++s)
        if (s < STEPS)
            pk_static_for([&](auto nb) { load_w(wr[s], s, nb); }, std::make_integer_sequence<int, kPkWOwn>{});
    {
        // x(0): everything issued after this wave's last fetch of it is younger
        constexpr int y = PkSchedule::prologue(STEPS) - kPkXOwn;
        pk_wait_vm<PkSchedule::clamp(y)>();
        __builtin_amdgcn_s_barrier();                        // every wave's quarter of x(0) has landed
        pk_read_a(a[0], ring_addr + a_off);
    }

    auto step = [&](auto tag) {
        constexpr int s = decltype(tag)::value;
        constexpr int cur = s % 2, nxt = (s + 1) % 2, slot = s % kPkWD;
        pk_wait_a(a[cur]);                                   // A(s) is in registers
        if constexpr (s + 1 < STEPS) pk_wait_vm<PkSchedule::younger_than_next_x(STEPS, s)>();   // own quarter of x(s + 1)
        // after the barrier: x(s + 1) is complete in LDS, and nobody reads stage s % XS any more
        if constexpr (s + 1 < STEPS) __builtin_amdgcn_s_barrier();
        if constexpr (s + kPkXS < STEPS) issue_x(s + kPkXS);
        if constexpr (s + 1 < STEPS) pk_read_a(a[nxt], ring_addr + ((s + 1) % kPkXS) * kPkXTile + a_off);
        pk_static_for([&](auto nb_tag) {
            constexpr int nb = decltype(nb_tag)::value;
            pk_wait_w<PkSchedule::younger_than_w(STEPS, s, nb)>(wr[slot][nb]);       // exact wait for fetch nb of W(s)
            const pk_bf16x8 bv = __builtin_bit_cast(pk_bf16x8, wr[slot][nb]);
#pragma unroll
            for (int mb = 0; mb < 8; ++mb)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(pk_bf16x8, a[cur][mb]), bv, acc[mb][nb], 0, 0, 0);
            // the slot's registers have been read by the MFMAs above: refill them with k-step s + WD
            if constexpr (s + kPkWD < STEPS) load_w(wr[slot], s + kPkWD, nb_tag);
        }, std::make_integer_sequence<int, kPkWOwn>{});
    };
    pk_static_for(step, std::make_integer_sequence<int, STEPS>{});

    // ---- exchange with the workgroup that holds the other half of K.  Element e = (mb, nb, i) of lane `lane` of
    // wave `wave` lives at part[((wave * 64 + e) * 64) + lane]: every store and load is a 256-byte run per wave.
    float* mine = partials + ((int64_t)tile * 2 + khalf) * (kPkBM * kPkBN);
    const float* other = partials + ((int64_t)tile * 2 + (1 - khalf)) * (kPkBM * kPkBN);
    const int base = wave * 64 * 64 + lane;
#pragma unroll
    for (int mb = 0; mb < 8; ++mb)
#pragma unroll
        for (int nb = 0; nb < kPkWOwn; ++nb)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __hip_atomic_store(mine + base + ((mb * kPkWOwn + nb) * 4 + i) * 64, acc[mb][nb][i], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
    // Publication, ordered by what the instructions guarantee rather than by a release / acquire pair: the partial
    // values are device-scope stores (written through to the level all XCDs share), s_waitcnt vmcnt(0) returns when
    // they have been acknowledged there, the barrier collects the whole workgroup, and only then does thread 0 draw the
    // ticket, a device-scope read-modify-write at that same level.  The workgroup that draws the second ticket reads
    // the other tile with device-scope loads (which bypass the caches that are not coherent between XCDs) issued after
    // its ticket has returned.  The same exchange with an acquire-release ticket was measured: the compiler brackets it
    // with a write-back and an invalidate of the whole L2 (buffer_wbl2 / buffer_inv), 38.2 us per launch against
    // 32.9 us, for lines that never were in a non-coherent cache.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // this thread's partial values are written
    __builtin_amdgcn_s_barrier();                            // ... and so are the whole workgroup's
    int ticket = 0;
    if (tid == 0) ticket = __hip_atomic_fetch_add(tickets + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // broadcast through LDS (the x ring is no longer read: every wave is past its last k-step)
    int* flag = reinterpret_cast<int*>(smem);
    if (tid == 0) *flag = ticket;
    __syncthreads();
    ticket = *flag;
    if (ticket == 0) return;                                 // first to arrive: the other workgroup finishes the tile
    if (tid == 0) tickets[tile] = 0;                         // last user of the ticket word: leave it zero

    const int n0 = tile * kPkBN + 32 * wave;
    // every load first, so that they are all in flight together; then the sums and the stores
    float o[8][kPkWOwn][4];
#pragma unroll
    for (int mb = 0; mb < 8; ++mb)
#pragma unroll
        for (int nb = 0; nb < kPkWOwn; ++nb)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                o[mb][nb][i] = __hip_atomic_load(other + base + ((mb * kPkWOwn + nb) * 4 + i) * 64, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int mb = 0; mb < 8; ++mb)
#pragma unroll
        for (int nb = 0; nb < kPkWOwn; ++nb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 16 * mb + 4 * lq + i;
                const float v = acc[mb][nb][i] + o[mb][nb][i];        // one fp32 add: the same value whoever arrived last
                if (row < M) y[(int64_t)row * ldy + n0 + 16 * nb + lr] = pack1<Elem::BF16>(v);
            }
}

template <int STEPS, bool PLAIN = false>
static int launch_packed(const void* x, const void* wp, void* y, int M, int N, int64_t ldx, int64_t ldy, int* tickets,
                         float* partials, hipStream_t stream) {
    auto kern = layer_gemm_packed_kernel<STEPS, PLAIN>;
    static LdsLimit limit;
    if (limit.raise(reinterpret_cast<const void*>(kern), kPkLds) != 0) return -2;
    const int tiles = N / kPkBN;
    const int grid = ((tiles + 7) / 8) * 16;        // two workgroups per column tile, ids paired 8 apart
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), kPkLds, stream, reinterpret_cast<const uint16_t*>(x),
                       reinterpret_cast<const uint16_t*>(wp), reinterpret_cast<uint16_t*>(y), M, N, ldx, ldy,
                       tickets, partials);
    return 0;
}

__global__ void zero_words_kernel(int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

void launch_zero_words(int* p, int n, hipStream_t stream) {
    hipLaunchKernelGGL(zero_words_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
}

// Bytes of partial-tile scratch the kernel needs for N columns: two fp32 tiles per column tile.
size_t layer_gemm_packed_partial_bytes(int N) {
    return (size_t)(N / kPkBN) * 2 * kPkBM * kPkBN * sizeof(float);
}

// Weights in operand order, [N/64][K/32][4][64][8] contiguous.  `tickets` holds kGemmTicketBytes that were zero
// before the first launch, `partials` layer_gemm_packed_partial_bytes(N).  Returns 0, -1 (shape not covered: K must
// be 1024, 2048, 4096 or 8192, N a multiple of 128 up to 128 * 1024) or -2 (HIP refused the LDS size).
int launch_layer_gemm_packed(const void* x, const void* wp, void* y, int M, int K, int N, int64_t ldx, int64_t ldy,
                             int* tickets, float* partials, bool plain_fetch, hipStream_t stream) {
    if (M < 1 || M > kPkBM || N < kPkBN || N % kPkBN || N / kPkBN > (int)(kGemmTicketBytes / sizeof(int))) return -1;
    if ((int64_t)kPkBM * ldx * 2 + 64 > 0x7fffffffLL) return -1;      // x byte offsets are kept in 32 bits
    if (plain_fetch)            // comparison mode: the benchmark's K only
        return K == 4096 ? launch_packed<64, true>(x, wp, y, M, N, ldx, ldy, tickets, partials, stream) : -1;
    switch (K) {
        case 1024: return launch_packed<16>(x, wp, y, M, N, ldx, ldy, tickets, partials, stream);
        case 2048: return launch_packed<32>(x, wp, y, M, N, ldx, ldy, tickets, partials, stream);
        case 4096: return launch_packed<64>(x, wp, y, M, N, ldx, ldy, tickets, partials, stream);
        case 8192: return launch_packed<128>(x, wp, y, M, N, ldx, ldy, tickets, partials, stream);
        default: return -1;
    }
}

}  // namespace kvp
