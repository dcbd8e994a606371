// Stand-in dense layer of the layer-stack harness: y[M, N] = x[M, K] . W[K, N], bf16 in,
// fp32 accumulate on MFMA, bf16 out, M <= 128 (one decode batch), W row-major (N contiguous).
//
// The shape is skinny (M = 128), so the kernel is bound by streaming W from HBM once
// (K*N*2 bytes; 117 MB for 4096 x 14336).  A workgroup owns a 64-row x 128-column tile of y;
// its four waves split K four ways (no barrier in the main loop) and add their partial tiles
// through LDS at the end.  Every operand travels global -> LDS by asynchronous
// global_load_lds into a per-wave ring of three stages, so two k-steps are in flight under
// the MFMAs of the current one; x (1 MB, L2 resident) takes the same route so that all
// fetches of a wave form one in-order stream that is counted by hand.
//
// The two workgroups that share a column tile (upper and lower 64 rows) read the same W bytes.
// They are given block ids 8 apart, which the dispatcher places on the same XCD, so the second
// reader finds the lines in that XCD's L2 while both walk K in step.  Splitting M this way makes
// a stage 8 KB of W for 4 KB of x (a 128-row tile of 64 columns would be the reverse), which
// doubles the HBM bytes a compute unit keeps in flight for the same LDS.
//
// k-step = 32 rows of W.  Stage = W tile [32 k][128 n] (8 KB, 256 B rows) + x tile
// [64 m][32 k] (4 KB, 64 B rows).  The B operand of v_mfma_f32_16x16x32_bf16 needs 8
// consecutive k for one n per lane, i.e. a transposed read of the row-major W tile:
// ds_read_b64_tr_b16, two per operand.  Bank conflicts are avoided by XOR-swizzling which
// 16-byte chunk of a row each lane fetches (W: chunk ^ 2*(k%8), x: chunk ^ (m/4)%4).
#include "kv_common.h"

namespace kvp {

typedef __bf16 gemm_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gemm_f4 __attribute__((ext_vector_type(4)));
typedef uint32_t gemm_u4 __attribute__((ext_vector_type(4)));
typedef uint32_t gemm_u2 __attribute__((ext_vector_type(2)));

constexpr int kGemmBN = 128;              // output columns per workgroup
constexpr int kGemmBM = 64;               // output rows per workgroup
constexpr int kGemmBK = 32;               // k per step
constexpr int kGemmM = 128;               // rows of x the kernel covers (two workgroups per column tile)
constexpr int kGemmStages = 3;
constexpr int kGemmWTile = kGemmBK * kGemmBN * 2;       // 8 KB
constexpr int kGemmXTile = kGemmBM * kGemmBK * 2;       // 4 KB
constexpr int kGemmStage = kGemmWTile + kGemmXTile;     // 12 KB
constexpr int kGemmLoads = 12;                          // wave-wide 1 KB fetches per stage
constexpr int kGemmLds = 4 * kGemmStages * kGemmStage;  // 144 KB

#define KVP_GEMM_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define KVP_GEMM_GLOBAL(p) ((const __attribute__((address_space(1))) void*)(p))

template <int N>
__device__ __forceinline__ void gemm_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | 0x0f70);
}

// The ring is read with inline assembly: the compiler cannot tell ring stages apart and would wait
// for every outstanding fetch before any LDS read it can see.
__device__ __forceinline__ void gemm_read_a(gemm_u4 (&a)[4], uint32_t base) {
    asm volatile(
        "ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:1024\n\tds_read_b128 %2, %4 offset:2048\n\t"
        "ds_read_b128 %3, %4 offset:3072"
        : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3])
        : "v"(base)
        : "memory");
}
__device__ __forceinline__ void gemm_read_b(gemm_u2& lo, gemm_u2& hi, uint32_t addr_lo, uint32_t addr_hi) {
    asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %3"
                 : "=&v"(lo), "=&v"(hi)
                 : "v"(addr_lo), "v"(addr_hi)
                 : "memory");
}
__device__ __forceinline__ void gemm_wait_lds(gemm_u4 (&a)[4], gemm_u2 (&b)[16]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]),
                   "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7]),
                   "+v"(b[8]), "+v"(b[9]), "+v"(b[10]), "+v"(b[11]), "+v"(b[12]), "+v"(b[13]), "+v"(b[14]), "+v"(b[15])
                 :
                 : "memory");
}

__global__ __launch_bounds__(256) void layer_gemm_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                                         uint16_t* __restrict__ y, int M, int K, int N,
                                                         int64_t ldx, int64_t ldw, int64_t w_tile_stride, int64_t ldy) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWaveSize);
    const int lane = tid % kWaveSize;
    const int lq = lane / 16, lr = lane % 16;
    // block id -> (column tile, row half): ids i and i + 8 (same XCD) take the two halves of one column tile
    const int bid = blockIdx.x;
    const int tile = (bid / 16) * 8 + bid % 8, half = (bid / 8) % 2;
    if (tile >= N / kGemmBN) return;
    const int n0 = tile * kGemmBN, m0 = half * kGemmBM;
    if (m0 >= M) return;
    const int ksteps = K / (4 * kGemmBK);                    // k-steps of this wave
    const int kbase = wave * ksteps * kGemmBK;

    unsigned char* ring = smem + wave * (kGemmStages * kGemmStage);
    const uint32_t ring_addr = (uint32_t)(uintptr_t)KVP_GEMM_LDS(ring);

    // ---- fetch offsets (bytes), loop invariant
    // W fetch r (0..7): lane lands row 4r + lane/16 at stored chunk lane%16; it fetches logical chunk stored ^ fW(row)
    uint32_t woff[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int row = 4 * r + lane / 16;
        const int logical = (lane % 16) ^ (2 * (row % 8));
        woff[r] = (uint32_t)(row * ldw * 2 + logical * 16);
    }
    // x fetch r (0..3): lane lands row 16r + lane/4 at stored chunk lane%4; logical chunk stored ^ fx(row); rows >= M
    // re-read row M-1 (their products are never stored)
    uint32_t xoff[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 16 * r + lane / 4;
        const int logical = (lane % 4) ^ ((row / 4) % 4);
        xoff[r] = (uint32_t)(min(m0 + row, M - 1) * ldx * 2 + logical * 16);
    }
    // column tile t of W starts at w + t * w_tile_stride: 128 for a row-major [K, N] matrix (rows ldw apart),
    // K * 128 for the tile-packed [N/128, K, 128] form (rows 128 apart, one contiguous 1 MB run per tile)
    const unsigned char* wg = reinterpret_cast<const unsigned char*>(w) + (int64_t)tile * w_tile_stride * 2;
    const unsigned char* xg = reinterpret_cast<const unsigned char*>(x);

    auto issue = [&](int step, int stage) {
        const int k0 = kbase + step * kGemmBK;
        const unsigned char* wt = wg + (int64_t)k0 * ldw * 2;
        const unsigned char* xt = xg + (int64_t)k0 * 2;
        unsigned char* dst = ring + stage * kGemmStage;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GEMM_GLOBAL(wt + woff[r]), KVP_GEMM_LDS(dst + r * 1024), 16, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            __builtin_amdgcn_global_load_lds(KVP_GEMM_GLOBAL(xt + xoff[r]), KVP_GEMM_LDS(dst + kGemmWTile + r * 1024), 16, 0, 0);
    };

    // ---- LDS read addresses inside a stage
    // A (x) operand of m-block mb: row 16mb + lr, logical chunk lq -> stored lq ^ (lr/4)%4; +1024 per m-block
    const uint32_t a_off = kGemmWTile + lr * 64 + ((lq ^ ((lr / 4) % 4)) << 4);
    // B (W) operand of n-block nb, half h: row 8lq + 4h + lr/4, logical byte 32nb + 8(lr%4); n-block nb moves the
    // logical chunk by 2nb, which an XOR with nb << 5 applies to the swizzled address (2(row%8) is even)
    uint32_t b_off[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int row = 8 * lq + 4 * h + lr / 4;
        b_off[h] = row * 256 + (((row % 8)) << 5) + ((lr % 4) << 3);
    }

    gemm_f4 acc[4][8];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) acc[mb][nb] = gemm_f4{0.f, 0.f, 0.f, 0.f};

    constexpr int PD = kGemmStages - 1;
#pragma unroll
    for (int s = 0; s < PD; ++s)
        if (s < ksteps) issue(s, s);

    int stage = 0;
    for (int step = 0; step < ksteps; ++step) {
        int ahead_stage = stage + PD; if (ahead_stage >= kGemmStages) ahead_stage -= kGemmStages;
        if (step + PD < ksteps) {
            issue(step + PD, ahead_stage);
            gemm_wait_vmcnt<kGemmLoads * PD>();
        } else {
            gemm_wait_vmcnt<0>();
        }
        asm volatile("" ::: "memory");
        const uint32_t st = ring_addr + stage * kGemmStage;
        gemm_u4 a[4];
        gemm_u2 b[16];
        gemm_read_a(a, st + a_off);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb)
            gemm_read_b(b[2 * nb], b[2 * nb + 1], st + (b_off[0] ^ (nb << 5)), st + (b_off[1] ^ (nb << 5)));
        gemm_wait_lds(a, b);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
            const gemm_u4 bv = {b[2 * nb][0], b[2 * nb][1], b[2 * nb + 1][0], b[2 * nb + 1][1]};
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(gemm_bf16x8, a[mb]),
                                                                       __builtin_bit_cast(gemm_bf16x8, bv), acc[mb][nb], 0, 0, 0);
        }
        stage = stage + 1 == kGemmStages ? 0 : stage + 1;
    }

    // ---- add the four k-quarters through LDS (every wave has consumed all it fetched), write bf16
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem) + wave * (kGemmBM * kGemmBN);
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 8; ++nb)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[(16 * mb + 4 * lq + i) * kGemmBN + 16 * nb + lr] = acc[mb][nb][i];
    __syncthreads();
    const float* all = reinterpret_cast<const float*>(smem);
    constexpr int TS = kGemmBM * kGemmBN;
    for (int i = 0; i < 16; ++i) {
        const int row = 16 * wave + i;
        if (m0 + row >= M) break;
#pragma unroll
        for (int cpart = 0; cpart < 2; ++cpart) {
            const int idx = row * kGemmBN + cpart * kWaveSize + lane;
            const float v = (all[idx] + all[idx + TS]) + (all[idx + 2 * TS] + all[idx + 3 * TS]);
            y[(int64_t)(m0 + row) * ldy + n0 + cpart * kWaveSize + lane] = pack1<Elem::BF16>(v);
        }
    }
}

// Returns 0, -1 (shape not covered) or -2 (HIP refused the LDS size).
int launch_layer_gemm(const void* x, const void* w, void* y, int M, int K, int N, int64_t ldx, int64_t ldw,
                      int64_t w_tile_stride, int64_t ldy, hipStream_t stream) {
    if (M < 1 || M > kGemmM || K < 4 * kGemmBK || K % (4 * kGemmBK) || N < kGemmBN || N % kGemmBN) return -1;
    // byte offsets inside a k-step are kept in 32 bits
    if ((int64_t)kGemmBK * ldw * 2 + 256 > 0x7fffffffLL || (int64_t)kGemmM * ldx * 2 + 64 > 0x7fffffffLL) return -1;
    static LdsLimit limit;
    if (limit.raise(reinterpret_cast<const void*>(layer_gemm_kernel), kGemmLds) != 0) return -2;
    // two workgroups (row halves) per column tile, ids paired 8 apart: round the tile count up to a multiple of 8
    const int tiles = N / kGemmBN;
    const int grid = ((tiles + 7) / 8) * 16;
    hipLaunchKernelGGL(layer_gemm_kernel, dim3(grid), dim3(256), kGemmLds, stream,
                       reinterpret_cast<const uint16_t*>(x), reinterpret_cast<const uint16_t*>(w),
                       reinterpret_cast<uint16_t*>(y), M, K, N, ldx, ldw, w_tile_stride, ldy);
    return 0;
}

}  // namespace kvp
