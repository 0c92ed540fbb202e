// Comparator kernels for the benchmark (not part of the method): the paper
// reads its 2-bit GEMV against an int8-weight GEMV of the same shape, the
// "attainable roofline" with no up-convert and a quarter of the arithmetic
// intensity (Sec. III-B, III-C).  This is that kernel for CDNA4: int8 weights
// [N][K] row-major, int8 activations, exact int32 results; a wave streams
// four rows at a time with 16-byte loads and v_dot4_i32_i8.
#include <hip/hip_runtime.h>

#include "w2_internal.h"

namespace w2 {

constexpr int CMP_ROWS = 4;            // rows per wave
constexpr int CMP_SPAN = 4096;         // k per wave pass: 64 lanes x 4 x 16 bytes

__global__ void __launch_bounds__(256)
int8_gemv_kernel(const int8_t* __restrict__ W8, const int8_t* __restrict__ xq, int32_t* __restrict__ out,
                 int64_t K, int64_t N, int kpad)
{
    extern __shared__ __align__(16) int8_t xs[];             // kpad bytes: the activations, zero-padded
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid * 16; i < kpad; i += 256 * 16) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (i < K) v = *reinterpret_cast<const uint4*>(xq + i);
        *reinterpret_cast<uint4*>(xs + i) = v;
    }
    __syncthreads();
    const int64_t n0 = ((int64_t)blockIdx.x * 4 + wave) * CMP_ROWS;
    const int8_t* rowp[CMP_ROWS];
#pragma unroll
    for (int r = 0; r < CMP_ROWS; ++r) rowp[r] = W8 + min(n0 + r, N - 1) * K;
    int acc[CMP_ROWS] = {};
    for (int64_t k0 = 0; k0 < K; k0 += CMP_SPAN) {
        uint4 wv[CMP_ROWS][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t k = k0 + u * 1024 + lane * 16;
            const int64_t kc = k < K ? k : K - 16;           // past the end: any valid address, x is zero there
#pragma unroll
            for (int r = 0; r < CMP_ROWS; ++r) wv[r][u] = *reinterpret_cast<const uint4*>(rowp[r] + kc);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint4 xv = *reinterpret_cast<const uint4*>(xs + k0 + u * 1024 + lane * 16);
#pragma unroll
            for (int r = 0; r < CMP_ROWS; ++r) {
                acc[r] = __builtin_amdgcn_sdot4((int)wv[r][u].x, (int)xv.x, acc[r], false);
                acc[r] = __builtin_amdgcn_sdot4((int)wv[r][u].y, (int)xv.y, acc[r], false);
                acc[r] = __builtin_amdgcn_sdot4((int)wv[r][u].z, (int)xv.z, acc[r], false);
                acc[r] = __builtin_amdgcn_sdot4((int)wv[r][u].w, (int)xv.w, acc[r], false);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < CMP_ROWS; ++r) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc[r] += __shfl_xor(acc[r], off);
        if (lane == 0 && n0 + r < N) out[n0 + r] = acc[r];
    }
}

int launch_int8_gemv(const int8_t* W8, const int8_t* xq, int32_t* out, int64_t K, int64_t N, hipStream_t stream)
{
    const int kpad = (int)((K + CMP_SPAN - 1) / CMP_SPAN * CMP_SPAN);
    const dim3 grid((unsigned)((N + 4 * CMP_ROWS - 1) / (4 * CMP_ROWS))), block(256);
    hipLaunchKernelGGL(int8_gemv_kernel, grid, block, kpad, stream, W8, xq, out, K, N, kpad);
    return check_launch("w2_debug_int8_gemv");
}

}  // namespace w2
