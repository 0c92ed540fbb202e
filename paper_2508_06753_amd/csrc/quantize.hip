// Per-token int8 quantisation of the activations (Sec. II-B; Sec. II-D: the
// abs-max of the quantisation granularity gives the scale, entries are
// multiplied by the inverse of the scale and converted to int8).  One scale
// per row.  Every operation is a single IEEE binary32 operation (correctly
// rounded divide, one multiply, round-half-even), so the int8 codes are
// reproducible bit for bit.
#include <hip/hip_runtime.h>

#include "w2_internal.h"

namespace w2 {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

template <bool BF16>
struct RowLoader;

template <>
struct RowLoader<false> {                 // fp32: 4 elements per thread per step
    static constexpr int EPT = 4;
    __device__ static void load(const void* row, int64_t k, float (&v)[4])
    {
        const float4 f = *reinterpret_cast<const float4*>((const float*)row + k);
        v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
    }
};

template <>
struct RowLoader<true> {                  // bf16: 8 elements per thread per step
    static constexpr int EPT = 8;
    __device__ static void load(const void* row, int64_t k, float (&v)[8])
    {
        const uint4 u = *reinterpret_cast<const uint4*>((const uint16_t*)row + k);
        v[0] = bf16_lo(u.x); v[1] = bf16_hi(u.x); v[2] = bf16_lo(u.y); v[3] = bf16_hi(u.y);
        v[4] = bf16_lo(u.z); v[5] = bf16_hi(u.z); v[6] = bf16_lo(u.w); v[7] = bf16_hi(u.w);
    }
};

__device__ __forceinline__ int quant1(float x, float inv)
{
    float t = x * inv;                        // one rounded multiply
    float r = __builtin_rintf(t);             // v_rndne_f32: half to even
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// One workgroup per row.  Pass 1: abs-max (wave shuffles + LDS).  Pass 2: quantise and store packed
// int8.  The first CR vectors of a thread stay in registers between the passes (with 1024 threads
// that is a whole row of up to 16384 fp32 or 32768 bf16 values: one trip to memory instead of two);
// longer rows re-read the rest (L2-resident).
constexpr int CR = 4;

template <bool BF16>
__global__ void __launch_bounds__(1024)
quantize_rows_kernel(const void* __restrict__ X, int64_t K, int64_t ldx, int G,
                     int8_t* __restrict__ xq, float* __restrict__ sx, int32_t* __restrict__ gsum)
{
    using L = RowLoader<BF16>;
    constexpr int EPT = L::EPT;
    const int64_t m = blockIdx.x;
    const void* row = BF16 ? (const void*)((const uint16_t*)X + m * ldx)
                           : (const void*)((const float*)X + m * ldx);
    __shared__ float s_red[16];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t step = (int64_t)blockDim.x * EPT;

    float cache[CR][EPT];
#pragma unroll
    for (int c = 0; c < CR; ++c) {
        const int64_t k = (int64_t)threadIdx.x * EPT + c * step;
#pragma unroll
        for (int i = 0; i < EPT; ++i) cache[c][i] = 0.0f;
        if (k < K) L::load(row, k, cache[c]);
    }
    if (threadIdx.x < 16) s_red[threadIdx.x] = 0.0f;         // slots of waves that do not exist stay 0
    __syncthreads();

    float amax = 0.0f;
#pragma unroll
    for (int c = 0; c < CR; ++c)
#pragma unroll
        for (int i = 0; i < EPT; ++i) amax = fmaxf(amax, fabsf(cache[c][i]));
    for (int64_t k = (int64_t)threadIdx.x * EPT + CR * step; k < K; k += step) {
        float v[EPT];
        L::load(row, k, v);
#pragma unroll
        for (int i = 0; i < EPT; ++i) amax = fmaxf(amax, fabsf(v[i]));
    }
    amax = wave_max_f32(amax);
    if (lane == 0) s_red[wave] = amax;
    __syncthreads();
    amax = s_red[lane & 15];                                 // every wave reduces the (at most 16) partial maxima itself
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    float inv = 0.0f, s = 0.0f;
    if (amax > 0.0f) {
        inv = __fdiv_rn(127.0f, amax);
        s = __fdiv_rn(amax, 127.0f);
    }
    if (threadIdx.x == 0) sx[m] = s;

    const int lanes_per_group = G / EPT;      // 8..32, a power of two, divides 64
    auto emit = [&](int64_t k, const float (&v)[EPT]) {
        int q[EPT];
        int sum = 0;
#pragma unroll
        for (int i = 0; i < EPT; ++i) { q[i] = quant1(v[i], inv); sum += q[i]; }
        uint32_t p0 = (q[0] & 0xff) | ((q[1] & 0xff) << 8) | ((q[2] & 0xff) << 16) |
                      ((uint32_t)(q[3] & 0xff) << 24);
        if constexpr (EPT == 4) {
            *reinterpret_cast<uint32_t*>(xq + m * K + k) = p0;
        } else {
            uint32_t p1 = (q[4] & 0xff) | ((q[5] & 0xff) << 8) | ((q[6] & 0xff) << 16) |
                          ((uint32_t)(q[7] & 0xff) << 24);
            *reinterpret_cast<uint2*>(xq + m * K + k) = make_uint2(p0, p1);
        }
        if (gsum) {
            // Each group occupies lanes_per_group (at most 32) consecutive, aligned lanes, and K % 256 == 0
            // makes the active lanes of a wave a whole number of such runs (a bf16 row of 256 values fills
            // half a wave: lanes 0..31): a lane only ever reads lanes of its own, fully active, run.
            for (int off = 1; off < lanes_per_group; off <<= 1) sum += __shfl_xor(sum, off);
            if ((lane & (lanes_per_group - 1)) == 0) gsum[m * (K / G) + k / G] = sum;
        }
    };
#pragma unroll
    for (int c = 0; c < CR; ++c) {
        const int64_t k = (int64_t)threadIdx.x * EPT + c * step;
        if (k < K) emit(k, cache[c]);                        // whole groups of lanes (K % 256 == 0)
    }
    for (int64_t k = (int64_t)threadIdx.x * EPT + CR * step; k < K; k += step) {
        float v[EPT];
        L::load(row, k, v);
        emit(k, v);
    }
}

int launch_quantize(const void* X, int x_is_bf16, int64_t M, int64_t K, int64_t ldx, int G,
                    int8_t* xq, float* sx, int32_t* gsum, hipStream_t stream)
{
    if (M == 0) return 0;
    // Few rows (decode): one wide workgroup per row to shorten the serial chain.
    // Many rows (prefill): 256 threads, several rows per CU.
    const int ept = x_is_bf16 ? 8 : 4;
    int threads = M <= 64 ? 1024 : 256;
    while (threads > 64 && (int64_t)threads * ept > K) threads >>= 1;
    if (x_is_bf16)
        hipLaunchKernelGGL(quantize_rows_kernel<true>, dim3((unsigned)M), dim3(threads), 0, stream,
                           X, K, ldx, G, xq, sx, gsum);
    else
        hipLaunchKernelGGL(quantize_rows_kernel<false>, dim3((unsigned)M), dim3(threads), 0,
                           stream, X, K, ldx, G, xq, sx, gsum);
    return check_launch("w2_quantize_rows");
}

}  // namespace w2
