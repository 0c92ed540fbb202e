// Internal declarations shared by the translation units of libw2mm.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../include/w2mm.h"
#include "w2_layout.h"

namespace w2 {

// Maximum of a value over the 64 lanes of a wave, the same in every lane.  Cross-lane moves inside a row of 16
// lanes ride on the vector instruction itself (DPP), the four rows meet through scalar registers: no trip
// through local memory per step, which is what a generic lane shuffle costs here.  fmaxf semantics (a NaN
// operand is ignored).
template <int CTRL>
__device__ __forceinline__ float dpp_move_f32(float v)      // lanes with no source read 0
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

__device__ __forceinline__ float wave_max_f32(float m)
{
    m = fmaxf(m, dpp_move_f32<0xB1>(m));                     // quad_perm [1,0,3,2]
    m = fmaxf(m, dpp_move_f32<0x4E>(m));                     // quad_perm [2,3,0,1]
    m = fmaxf(m, dpp_move_f32<0x141>(m));                    // row_half_mirror
    m = fmaxf(m, dpp_move_f32<0x140>(m));                    // row_mirror: every lane holds its row's maximum
    const int b = __float_as_int(m);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// Records `what` + the HIP error string as this thread's last error if the
// preceding launches failed; returns a w2_status_t.
int check_launch(const char* what);
void set_error(const char* fmt, ...);

int launch_prepack(const uint8_t* codes, const uint16_t* scales, const Layout& L, int codec,
                   void* packed, int32_t* bad_codes, hipStream_t stream);
int launch_unpack(const void* packed, const Layout& L, int codec, uint8_t* codes,
                  uint16_t* scales, hipStream_t stream);
int launch_quantize(const void* X, int x_is_bf16, int64_t M, int64_t K, int64_t ldx, int G,
                    int8_t* xq, float* sx, int32_t* gsum, hipStream_t stream);
int launch_stream_read(const void* src, size_t bytes, uint32_t* sink, const w2_tuning_t& tune, hipStream_t stream);

// Work fused into the store of the result (Sec. II-D: bias addition and post-GEMM activation
// functions are applied while the outputs are still in registers).  z = fp32 result + bias[n];
// act 0: Y = bf16(z); 1: Y = bf16(silu(z)); 2: the 16-column blocks of the matrix alternate
// gate, up, gate, up ... and Y[m][16 b + l] = bf16(silu(z[m][32 b + l]) * z[m][32 b + 16 + l])
// (N / 2 output columns).
struct Epilogue {
    const uint16_t* bias = nullptr;     // bf16 [N], or nullptr
    int act = 0;
};
constexpr int ACT_NONE = 0, ACT_SILU = 1, ACT_SILU_MUL = 2;

// Arguments common to the w2a8 kernels.  acc_out != nullptr selects the debug
// mode that stores the int32 group accumulators and skips Y.
struct A8Args {
    const uint32_t* codes;
    const uint16_t* scales;
    const int8_t* xq;
    const float* sx;
    uint16_t* Y;
    int32_t* acc_out;
    int64_t M, K, N, ldy;
    int64_t n_cb, n_kt;
    int G;
    // split-K across workgroups (tiled and mid-M kernels): fp32 partial results [splits][M][N] in a caller's
    // workspace, summed and rounded by a second launch; nullptr / 0 = not available
    float* part = nullptr;
    size_t part_bytes = 0;
    Epilogue epi;
    w2_tuning_t tune = {};      // overrides from the caller (all 0: the library's rules)
};

bool a8_dot4_supports(const A8Args& a);
int launch_a8_dot4(const A8Args& a, hipStream_t stream);
bool a8_smallm_supports(const A8Args& a);
int launch_a8_smallm(const A8Args& a, hipStream_t stream);
bool a8_midm_supports(const A8Args& a);
int launch_a8_midm(const A8Args& a, hipStream_t stream);
int launch_a8_tiled(const A8Args& a, hipStream_t stream);
bool a8_tiled128_supports(const A8Args& a);
int launch_a8_tiled128(const A8Args& a, int splits, hipStream_t stream);
int a8_tiled128_splits(int64_t M, int64_t N, int64_t n_kt, int64_t cap, const w2_tuning_t& tune);

// The decode kernel (M <= 32; rows quantised in the kernel: M <= 4): xt 0 = int8 rows (a.xq / a.sx), 1 = fp32 rows,
// 2 = bf16 rows quantised in the kernel.
bool a8_gemv_supports(int64_t M);
int launch_a8_gemv(const A8Args& a, const void* X, int xt, int64_t ldx, hipStream_t stream);


struct A16Args {
    const uint32_t* codes;
    const uint16_t* scales;
    const uint16_t* X;
    uint16_t* Y;
    int64_t M, K, N, ldx, ldy;
    int64_t n_cb, n_kt;
    int G;
    int fold;       // build the weights as sw*q (scale folded in): no zero-point term, no dequant step
    float* part = nullptr;      // split-K workspace, as in A8Args (scale-folded tiled kernel and mid-M kernel)
    size_t part_bytes = 0;
    Epilogue epi;
    w2_tuning_t tune = {};
};

bool a16_smallm_supports(const A16Args& a);
int launch_a16_smallm(const A16Args& a, hipStream_t stream);
int launch_a16_tiled(const A16Args& a, hipStream_t stream);
int launch_a16_fold_tiled(const A16Args& a, hipStream_t stream);
// w2a16 through the decode kernel (bf16 rows as they are, M <= 4, rows that fit one workgroup)
bool a16_gemv_supports(const A16Args& a);
int launch_a16_gemv(const A16Args& a, hipStream_t stream);
bool a16_midm_supports(const A16Args& a);
int launch_a16_midm(const A16Args& a, hipStream_t stream);

// Split-K across workgroups for shapes whose output tiles are too few to fill the chip (Sec. II-D,
// K-splitting for smaller GEMM shapes).  splitk_plan: number of K ranges for `wgs` output tiles of a
// kernel whose K loop has `n_kt` 256-k tiles (a part spans at least `min_tiles` of them), given room
// for `cap` fp32 copies of the M x N output.
int splitk_plan(int64_t wgs, int64_t n_kt, int64_t min_tiles, int64_t M, int64_t N, int64_t cap,
                int64_t max_bytes = (int64_t)16 << 20);
// Bytes of workspace with which the tiled kernels would split K for this problem (0: they would not).
size_t a8_tiled_splitk_bytes(int64_t M, int64_t N, int64_t n_kt, int G, const w2_tuning_t& tune);
size_t a8_midm_splitk_bytes(int64_t M, int64_t N, int64_t n_cb, int64_t n_kt, const w2_tuning_t& tune);
// The mid-M kernels' launch shape (both activation types): column blocks per workgroup and K ranges.
struct MidmPlan { int cbw, splits; };
MidmPlan midm_plan(int64_t M, int64_t n_cb, int64_t n_kt, int64_t cap, const w2_tuning_t& tune);
size_t a16_fold_splitk_bytes(int64_t M, int64_t N, int64_t n_kt, const w2_tuning_t& tune);
size_t a16_midm_splitk_bytes(int64_t M, int64_t N, int64_t n_cb, int64_t n_kt, const w2_tuning_t& tune);
// Y[m][n] = bf16(sum_s part[s][m][n]), a fixed order of summation
int launch_splitk_reduce(const float* part, int splits, int64_t M, int64_t N, uint16_t* Y, int64_t ldy,
                         const Epilogue& epi, hipStream_t stream);

int launch_int8_gemv(const int8_t* W8, const int8_t* xq, int32_t* out, int64_t K, int64_t N, hipStream_t stream);

// Opts a kernel in to more than 64 KiB of dynamic LDS.  The library remembers, per kernel and device,
// the largest size it has asked for: the attribute is set when a launch needs more than any earlier
// one did, not on every launch (host-side bookkeeping only; no device state).
int ensure_dynamic_lds(const void* kern, size_t bytes, const char* what);

}  // namespace w2
