// Combine of split-KV partitions: out = sum_p 2^(m_p - m*) acc_p / sum_p 2^(m_p - m*) l_p.
// One workgroup per (query head, sequence), one thread per output column.
#include "kv_common.h"

namespace kvp {

template <Elem E, int D>
__global__ __launch_bounds__(D) void reduce_kernel(AttnParams p, int bs) {
    const int h = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
    int n = p.context_lens[b];
    n = min(max(n, 0), p.MB * bs);
    const int nblocks = (n + bs - 1) / bs;
    const int np = (nblocks + p.part_blocks - 1) / p.part_blocks;   // partitions that wrote a partial
    const float* src = p.partials + ((int64_t)b * p.Hq + h) * p.NP * (D + 2);
    float ms = kNegBig;
    for (int i = 0; i < np; ++i) ms = fmaxf(ms, src[(int64_t)i * (D + 2) + D]);
    float num = 0.f, den = 0.f;
    for (int i = 0; i < np; ++i) {
        const float* row = src + (int64_t)i * (D + 2);
        const float wgt = fast_exp2(row[D] - ms);
        num += wgt * row[c];
        den += wgt * row[D + 1];
    }
    const float o = den > 0.f ? num / den : 0.f;
    reinterpret_cast<uint16_t*>(p.out)[(int64_t)b * p.out_stride_b + (int64_t)h * p.out_stride_h + c] = pack1<E>(o);
}

int launch_reduce(const AttnParams& p, int elem, int d, int bs, hipStream_t stream) {
    dim3 grid(p.Hq, p.B);
    if (elem == (int)Elem::F16) {
        if (d == 128) hipLaunchKernelGGL((reduce_kernel<Elem::F16, 128>), grid, dim3(128), 0, stream, p, bs);
        else hipLaunchKernelGGL((reduce_kernel<Elem::F16, 64>), grid, dim3(64), 0, stream, p, bs);
    } else {
        if (d == 128) hipLaunchKernelGGL((reduce_kernel<Elem::BF16, 128>), grid, dim3(128), 0, stream, p, bs);
        else hipLaunchKernelGGL((reduce_kernel<Elem::BF16, 64>), grid, dim3(64), 0, stream, p, bs);
    }
    return 0;
}

}  // namespace kvp
