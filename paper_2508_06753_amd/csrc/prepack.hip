// Off-line weight pre-formatting (Sec. II-B: the 2-bit tensor is re-laid-out
// ahead of time because inference weights are frozen) and its inverse, used
// by the round-trip test.  Neither is on the timed path.
#include <hip/hip_runtime.h>

#include "w2_internal.h"

namespace w2 {

// One thread builds one packed dword: 16 weights of one column.
__global__ void __launch_bounds__(256)
prepack_codes_kernel(const uint8_t* __restrict__ codes, int64_t K, int64_t N, int64_t n_kt,
                     int64_t n_dwords, int codec, uint32_t* __restrict__ out,
                     int32_t* __restrict__ bad_codes)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= n_dwords) return;
    const int t = (int)(id & 3);
    const int lane = (int)((id >> 2) & 63);
    const int64_t tile = id >> 8;
    const int64_t kt = tile % n_kt;
    const int64_t cb = tile / n_kt;
    const int64_t n = cb * TILE_N + (lane & 15);
    const int64_t k0 = kt * TILE_K + t * 64 + (lane >> 4) * 16;
    const int z = codec == 0 ? 2 : 1;
    const int top = codec == 0 ? 3 : 2;
    uint32_t w = 0;
    int bad = 0;
    if (n < N) {
        for (int j = 0; j < 4; ++j) {
            for (int b = 0; b < 4; ++b) {
                const int64_t k = k0 + 4 * j + b;
                if (k >= K) continue;
                const int c = codes[k * N + n];
                if (c > top) { ++bad; continue; }          // stored as value 0
                w |= (uint32_t)((c - z) & 3) << (8 * b + 2 * j);
            }
        }
    }
    out[id] = w;
    if (bad && bad_codes) atomicAdd(bad_codes, bad);
}

// One thread per stored scale.
__global__ void __launch_bounds__(256)
prepack_scales_kernel(const uint16_t* __restrict__ scales, int64_t K, int64_t N, int G,
                      int64_t n_kt, int gpt, int64_t n_scales, uint16_t* __restrict__ out)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= n_scales) return;
    const int gi = (int)(id % gpt);
    const int nl = (int)((id / gpt) % TILE_N);
    const int64_t tile = id / (gpt * TILE_N);
    const int64_t kt = tile % n_kt;
    const int64_t cb = tile / n_kt;
    const int64_t n = cb * TILE_N + nl;
    const int64_t g = kt * gpt + gi;
    uint16_t s = 0;
    if (n < N && g < K / G) s = scales[g * N + n];
    out[id] = s;
}

// Inverse: one thread per canonical code.
__global__ void __launch_bounds__(256)
unpack_codes_kernel(const uint32_t* __restrict__ packed, int64_t K, int64_t N, int64_t n_kt,
                    int codec, uint8_t* __restrict__ codes)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= K * N) return;
    const int64_t k = id / N, n = id % N;
    const int64_t cb = n / TILE_N, kt = k / TILE_K;
    const int kk = (int)(k % TILE_K);
    const int t = kk / 64, qb = (kk % 64) / 16, j = (kk % 16) / 4, b = kk % 4;
    const int lane = qb * 16 + (int)(n % TILE_N);
    const uint32_t w = packed[((cb * n_kt + kt) * 64 + lane) * 4 + t];
    int x = (w >> (8 * b + 2 * j)) & 3;
    int q = x >= 2 ? x - 4 : x;
    codes[id] = (uint8_t)(q + (codec == 0 ? 2 : 1));
}

__global__ void __launch_bounds__(256)
unpack_scales_kernel(const uint16_t* __restrict__ pscales, int64_t K, int64_t N, int G,
                     int64_t n_kt, int gpt, uint16_t* __restrict__ scales)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t Kg = K / G;
    if (id >= Kg * N) return;
    const int64_t g = id / N, n = id % N;
    const int64_t cb = n / TILE_N, kt = g / gpt;
    scales[id] = pscales[((cb * n_kt + kt) * TILE_N + (n % TILE_N)) * gpt + (g % gpt)];
}

int launch_prepack(const uint8_t* codes, const uint16_t* scales, const Layout& L, int codec,
                   void* packed, int32_t* bad_codes, hipStream_t stream)
{
    const int64_t n_dwords = (int64_t)(L.codes_bytes / 4);
    const int64_t n_scales = (int64_t)(L.scales_bytes / 2);
    hipLaunchKernelGGL(prepack_codes_kernel, dim3((unsigned)((n_dwords + 255) / 256)), dim3(256), 0,
                       stream, codes, L.K, L.N, L.n_kt, n_dwords, codec, (uint32_t*)packed,
                       bad_codes);
    hipLaunchKernelGGL(prepack_scales_kernel, dim3((unsigned)((n_scales + 255) / 256)), dim3(256),
                       0, stream, scales, L.K, L.N, L.G, L.n_kt, L.gpt, n_scales,
                       (uint16_t*)((char*)packed + L.codes_bytes));
    return check_launch("w2_prepack");
}

int launch_unpack(const void* packed, const Layout& L, int codec, uint8_t* codes,
                  uint16_t* scales, hipStream_t stream)
{
    const int64_t n_codes = L.K * L.N;
    const int64_t n_scales = (L.K / L.G) * L.N;
    hipLaunchKernelGGL(unpack_codes_kernel, dim3((unsigned)((n_codes + 255) / 256)), dim3(256), 0,
                       stream, (const uint32_t*)packed, L.K, L.N, L.n_kt, codec, codes);
    hipLaunchKernelGGL(unpack_scales_kernel, dim3((unsigned)((n_scales + 255) / 256)), dim3(256), 0,
                       stream, (const uint16_t*)((const char*)packed + L.codes_bytes), L.K, L.N,
                       L.G, L.n_kt, L.gpt, scales);
    return check_launch("w2_debug_unpack");
}

}  // namespace w2
