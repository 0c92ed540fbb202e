// Split-K across workgroups (Sec. II-D: K-splitting extracts parallelism along
// K for the smaller GEMM shapes): when a problem has too few output tiles to
// fill the chip, each tile's K range is cut into `splits` parts computed by
// different workgroups, which leave fp32 partial results in a workspace; this
// file holds the plan and the second launch that sums the parts in a fixed
// order and rounds to bf16 once.
#include <hip/hip_runtime.h>

#include "w2_internal.h"

namespace w2 {

int splitk_plan(int64_t wgs, int64_t n_kt, int64_t min_tiles, int64_t M, int64_t N, int64_t cap, int64_t max_bytes)
{
    // enough parts for about 1.5 workgroups per CU; a part spans at least min_tiles 256-k tiles (below
    // that the partial results and the second launch cost more than the idle CUs); at most 16 parts
    // and at most max_bytes (16 MiB unless the caller says otherwise) of partial results (the second launch
    // reads them all)
    if (wgs >= 192 || cap < 2) return 1;
    int64_t s = (384 + wgs - 1) / wgs;
    s = min(s, n_kt / min_tiles);
    s = min(s, (int64_t)16);
    s = min(s, max_bytes / (M * N * (int64_t)sizeof(float)));
    s = min(s, cap);
    return s < 2 ? 1 : (int)s;
}

// Sum over the parts of eight adjacent columns, part 0 first.  All SMAX loads are issued before the
// first addition (a loop with a run-time trip count would wait for each part's round trip in turn);
// slots past the last part re-read it and are left out of the sum.
template <int SMAX>
__device__ __forceinline__ void sum8(const float* __restrict__ part, int splits, int64_t M, int64_t N, int64_t m,
                                     int64_t n, float (&acc)[8])
{
    float4 a[SMAX], b[SMAX];
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
        const int se = s < splits ? s : splits - 1;
        const float4* p = reinterpret_cast<const float4*>(part + ((int64_t)se * M + m) * N + n);
        a[s] = p[0];
        b[s] = p[1];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
        if (s < splits) {
            acc[0] += a[s].x; acc[1] += a[s].y; acc[2] += a[s].z; acc[3] += a[s].w;
            acc[4] += b[s].x; acc[5] += b[s].y; acc[6] += b[s].z; acc[7] += b[s].w;
        }
    }
}

// One thread per eight adjacent output columns.  The fused epilogue is applied here, after the sum:
// bias, SiLU, or (gated) silu(gate block) * (up block) for the pairs of adjacent 16-column blocks.
template <int SMAX>
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float* __restrict__ part, int splits, int64_t M, int64_t N, uint16_t* __restrict__ Y,
                     int64_t ldy, Epilogue epi)
{
    const bool gated = epi.act == ACT_SILU_MUL;
    const int64_t n_out = gated ? N / 2 : N;
    const int64_t n8 = n_out / 8;                            // N % 8 == 0 (gated: N % 32 == 0)
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= M * n8) return;
    const int64_t m = i / n8, no = (i - m * n8) * 8;
    float acc[8];
    if (!gated) {
        sum8<SMAX>(part, splits, M, N, m, no, acc);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (epi.bias) acc[e] += __uint_as_float((uint32_t)epi.bias[no + e] << 16);
            if (epi.act == ACT_SILU) acc[e] = acc[e] / (1.0f + __expf(-acc[e]));
        }
    } else {
        const int64_t ng = (no / 16) * 32 + (no % 16);       // the gate columns of these outputs; up: 16 further
        float up[8];
        sum8<SMAX>(part, splits, M, N, m, ng, acc);
        sum8<SMAX>(part, splits, M, N, m, ng + 16, up);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (epi.bias) {
                acc[e] += __uint_as_float((uint32_t)epi.bias[ng + e] << 16);
                up[e] += __uint_as_float((uint32_t)epi.bias[ng + 16 + e] << 16);
            }
            acc[e] = acc[e] / (1.0f + __expf(-acc[e])) * up[e];
        }
    }
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        uint32_t lo = __float_as_uint(acc[2 * e]), hi = __float_as_uint(acc[2 * e + 1]);
        lo += 0x7fffu + ((lo >> 16) & 1u);                   // round to nearest even
        hi += 0x7fffu + ((hi >> 16) & 1u);
        o[e] = (lo >> 16) | (hi & 0xffff0000u);
    }
    *reinterpret_cast<uint4*>(Y + m * ldy + no) = make_uint4(o[0], o[1], o[2], o[3]);
}

int launch_splitk_reduce(const float* part, int splits, int64_t M, int64_t N, uint16_t* Y, int64_t ldy,
                         const Epilogue& epi, hipStream_t stream)
{
    const int64_t items = M * ((epi.act == ACT_SILU_MUL ? N / 2 : N) / 8);
    const dim3 grid((unsigned)((items + 255) / 256)), block(256);
    if (splits < 1 || splits > 16) { set_error("split-K reduce: %d parts", splits); return W2_ERR_INVALID_ARG; }
    if (splits <= 4) hipLaunchKernelGGL(splitk_reduce_kernel<4>, grid, block, 0, stream, part, splits, M, N, Y, ldy, epi);
    else if (splits <= 8) hipLaunchKernelGGL(splitk_reduce_kernel<8>, grid, block, 0, stream, part, splits, M, N, Y, ldy, epi);
    else hipLaunchKernelGGL(splitk_reduce_kernel<16>, grid, block, 0, stream, part, splits, M, N, Y, ldy, epi);
    return check_launch("split-K reduce");
}

}  // namespace w2
