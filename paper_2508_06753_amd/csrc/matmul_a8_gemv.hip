// w2a8 for one to four rows (decode): the memory-bound regime, where time
// tracks the bytes of weight streamed (Sec. I, II-A) and the job of the kernel
// is to keep the vector work per streamed code word below what the memory
// system delivers (Sec. II-E: effective bandwidth = min(beta, B / gamma)).
// One kernel serves both entry points:
//   - int8 rows in (w2_matmul_a8, after w2_quantize_rows);
//   - fp32 / bf16 rows in, quantised in the kernel (w2_matmul_a8_fused; Sec.
//     II-D: on a GPU the separate quantise -> GEMM -> dequantise sequence costs
//     launches and passes, so the abs-max is computed per workgroup,
//     redundantly, kept in local memory, the rows are quantised in the kernel
//     and the result is dequantised before the store; Sec. III-C: fusing wins
//     for matrix-vector shapes).  The arithmetic is that of w2_quantize_rows
//     value for value (one rounded multiply by 127/amax, round half to even),
//     so both routes give the same bits.
//
// "Up-convert and compute" (Sec. II-C): a lane reads 128 bits of packed 2-bit
// weights, one shift + one mask per four weights make int8 operands, and
// v_mfma_i32_16x16x64_i8 multiplies them with the (at most four live) rows.
//
// Schedule.  A wave owns one 16-column block and a CONTIGUOUS run of its 256-k
// tiles (K is split across the waves of a workgroup, Sec. II-D; partial sums
// meet in LDS in a fixed order).  The tiles of the run pass through a rolling
// window of W register slots: the load of tile i+W is issued the moment tile i
// has been consumed, so the arithmetic of a tile runs while the following ones
// are in flight and what remains after the last byte has arrived is one tile's
// work.  Every load is unconditional, so the compiler can count the loads in
// flight and waits for exactly the slot it needs; they are buffer loads whose
// resource spans exactly the wave's run (the row, for the activations): a slot
// past the end is out of range, which the hardware answers with zeros without
// touching memory (measured: dummy loads aimed at one shared line instead cost
// a microsecond, every wave of the grid queueing on it).  Addresses are
// "resource + lane offset + tile offset", one vector add per load (the range
// check covers the vector offset only), and no division.
#include <hip/hip_runtime.h>

#include "w2_small_common.h"

// Timeline probe for instrumented builds (a working build defines it to record a timestamp per wave);
// expands to nothing in the library.
#ifndef W2_GEMV_MARK
#define W2_GEMV_MARK(i)
#define W2_GEMV_MARK_DECL
#endif

namespace w2 {

namespace gemv {

constexpr int HDR = 512;          // LDS: abs-max partials [16 waves][4 rows] fp32, the rows' scales, padding
constexpr int SX_SLOT = 64;       // ... the scales' first float
// most 16-byte pieces of the activation rows a thread holds in registers: 8 for up to four rows (workgroups of
// up to 16 waves, 128 registers a lane), 32 for the wide form (up to 8 waves, 256 registers)
// (bf16 rows left unquantised, XT 3: 16 slots, up to 8 waves of up to 256 registers; bf16 rows quantised in the wide
// form: 16, a piece is eight values in flight through the quantiser and 32 slots spilled)
constexpr int xslots(int RL, int XT = 0) { return RL > 4 ? (XT == 2 ? 16 : 32) : XT == 3 ? 16 : 8; }
constexpr int max_waves(int RL, int XT = 0) { return RL > 4 || XT == 3 ? 8 : 16; }

// ---- w2a16 in the same kernel (XT 3; Sec. II-D, "Alternative implementation": the activations stay bf16, the
// weights become 16-bit values in registers and go to the 16-bit matrix instruction, fp32 accumulation).
// The up-convert is the one of the other w2a16 kernels: XOR 0xAAAAAAAA turns every field into s = q + 2, OR-ing a
// field into the mantissa of the bf16 constant 128 gives 130 + q, two weights per (shift, and-or); the matrix
// instruction then sums x * (130 + q) and a group's accumulator STARTS from -130 * (sum of the group's x), which
// the staging pass leaves in local memory, so that the group ends as sum x * q and the dequant is one fma.
// Operand dwords 0..3 take their two weights from bytes 0 and 2 of the code word (even k of the lane's 16-k
// block), dwords 4..7 from bytes 1 and 3 (odd k); the rows are staged de-interleaved the same way.
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
constexpr float ZP16 = 130.0f;
struct Bf16Consts { uint32_t mask, base; };
__device__ __forceinline__ Bf16Consts bf16_consts()
{
    Bf16Consts c = {0x00030003u, 0x43004300u};
    asm volatile("" : "+v"(c.mask), "+v"(c.base));           // in vector registers: (x & mask) | base is one instruction
    return c;
}
__device__ __forceinline__ void upconvert_bf16(uint32_t w, const Bf16Consts& c, v4i& b0, v4i& b1)
{
    const uint32_t x = w ^ 0xAAAAAAAAu;
    b0[0] = (int)((x & c.mask) | c.base);
    b0[1] = (int)(((x >> 2) & c.mask) | c.base);
    b0[2] = (int)(((x >> 4) & c.mask) | c.base);
    b0[3] = (int)(((x >> 6) & c.mask) | c.base);
    b1[0] = (int)(((x >> 8) & c.mask) | c.base);
    b1[1] = (int)(((x >> 10) & c.mask) | c.base);
    b1[2] = (int)(((x >> 12) & c.mask) | c.base);
    b1[3] = (int)(((x >> 14) & c.mask) | c.base);
}
__device__ __forceinline__ v4f mfma_bf16(const v4i& a, const v4i& b, const v4f& c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

struct Args {
    // What a wave needs before it can issue its first loads comes first, 64 bytes that one scalar load fetches:
    // the kernel's first memory request waits for these and for nothing else.
    const void* X;                // XT 0: int8 [M][K] dense; 1: fp32 rows; 2: bf16 rows (row stride ldx elements)
    int64_t ldx;
    const uint32_t* codes;
    const uint16_t* scales;
    int K, M, n_cb, n_kt;
    int cbw_rcp, cbw;             // waves of a workgroup = cbw column blocks x ks k-ranges (cbw: any number up to 16);
                                  // cbw_rcp = ceil(256 / cbw): wave / cbw = (wave * cbw_rcp) >> 8, exact for waves below 16
    int t_lo, t_rem;              // tiles per k-range: t_lo, and one more for the first t_rem ranges
    // ... the rest
    int ks;
    int outs_magic;               // ceil(2^20 / outputs per row of a workgroup): item / outputs for items below 4096
    int red_off;                  // LDS offset of the reduction scratch
    int sc_off;                   // LDS offset of the waves' scale slices
    int xg_off;                   // XT 3: LDS offset of -130 * (group sums of the rows), [K / G][4 rows] fp32
    const float* sx;              // XT 0: activation scales [M]
    uint16_t* Y;
    int32_t* acc_out;             // debug export (XT 0)
    int64_t ldy, N;
    Epilogue epi;
};

constexpr int MAX_RUN = 16;       // most tiles in a wave's run: their scales are fetched in one go

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Raw buffer resource over [base, base + bytes): loads at or past `bytes` return zeros and move nothing.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

constexpr int AUX_NT = 2;         // non-temporal: the weights are streamed once

__device__ __forceinline__ u32x4 load_tile(__amdgpu_buffer_rsrc_t wr, int w_lane, int i)
{
    // the tile's offset goes into the vector offset: the range check covers that one, not the scalar offset
    return __builtin_amdgcn_raw_buffer_load_b128(wr, w_lane + i * TILE_BYTES, 0, AUX_NT);
}

// x * inv, one rounding, then round half to even by adding 1.5 * 2^23 (one more rounding: exact for
// |t| < 2^22): the low byte of the sum's bit pattern is the int8 code.  |x * inv| never exceeds
// 127.00001 for finite inputs (|x| <= amax, inv = RN(127 / amax)), so the clamp of the definition
// never acts and is left out.
__device__ __forceinline__ uint32_t quant_bits(float x, float inv)
{
#pragma clang fp contract(off)                               // two roundings, as defined: never one fused multiply-add
    const float t = x * inv;
    return __float_as_uint(t + 12582912.0f);
}

__device__ __forceinline__ uint32_t pack4(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    // low bytes of a, b, c, d -> one dword
    const uint32_t lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);   // {a.b0, b.b0, 0, 0}
    const uint32_t hi = __builtin_amdgcn_perm(d, c, 0x04000c0cu);   // {0, 0, c.b0, d.b0}
    return lo | hi;
}

// RL: rows staged (M <= RL).  Up to four rows sit in accumulator rows 0..3, which the lanes of the first
// quarter of a wave hold (one, two or four values each); the wide form (RL = 8, 16 or 32 for int8 rows, 8 or 16 for unquantised bf16 rows)
// uses every accumulator row: lane (q, l) holds rows 4q..4q+3 of column l, for one row tile or, at RL = 32,
// two (the up-converted operand then feeds two matrix instructions).
// NP: 16-byte pieces per row and thread (a launch-time choice: the row's pieces / the workgroup's threads, rounded up)
// The kernel takes the head of Args as scalar parameters, fourteen dwords, and the rest as a structure: the
// first fourteen dwords of scalar kernel arguments can be handed to a wave in registers at its launch (the build
// asks for that, for this file only), so the first loads wait for no argument fetch at all; where the machine
// does not preload, the compiled entry fetches them with one scalar load as before.
struct ArgsRest {
    int outs_magic, red_off, sc_off, xg_off;
    const float* sx;
    uint16_t* Y;
    int32_t* acc_out;
    int64_t ldy, N;
    Epilogue epi;
};

template <int G, int RL, int XT, int W, int NP, bool DBG>
__global__ void __launch_bounds__(64 * max_waves(RL, XT))
a8_gemv_kernel(const void* p_X, int64_t p_ldx, const uint32_t* p_codes, const uint16_t* p_scales, int p_K, int p_M,
               int p_n_cb, int p_n_kt, int p_cbw_rcp, int p_shape, ArgsRest rest)
{
    Args a;
    a.X = p_X; a.ldx = p_ldx; a.codes = p_codes; a.scales = p_scales; a.K = p_K; a.M = p_M; a.n_cb = p_n_cb;
    a.n_kt = p_n_kt; a.cbw_rcp = p_cbw_rcp;
    // fourteen dwords fit the registers: the workgroup's shape and the K ranges travel in one of them
    a.cbw = p_shape & 0xff; a.ks = (p_shape >> 8) & 0xff; a.t_lo = (p_shape >> 16) & 0xff;
    a.t_rem = (p_shape >> 24) & 0xff;
    a.outs_magic = rest.outs_magic; a.red_off = rest.red_off; a.sc_off = rest.sc_off; a.xg_off = rest.xg_off;
    a.sx = rest.sx; a.Y = rest.Y; a.acc_out = rest.acc_out; a.ldy = rest.ldy; a.N = rest.N; a.epi = rest.epi;
    constexpr bool WIDE = RL > 4;
    constexpr bool A16 = XT == 3;                            // bf16 rows, bf16 matrix instruction
    static_assert(!A16 || (RL <= 16 && !DBG), "the w2a16 form: up to sixteen rows");
    constexpr int RA = WIDE ? 4 : RL;                        // accumulator rows a lane folds into y
    constexpr int RT = RL > 16 ? RL / 16 : 1;                // 16-row tiles
    static_assert(!WIDE || XT == 0 || XT == 3 || RL == 8, "the wide form: rows quantised in the kernel up to eight");
    constexpr int XGS = WIDE ? 16 : 4;                       // w2a16: rows per group in the table of group sums
    extern __shared__ __align__(16) int8_t smem[];
    constexpr int GPT = TILE_K / G;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_waves = a.cbw * a.ks;                        // = blockDim.x / 64
    const int threads = n_waves * 64;
    const int ksi = (wave * a.cbw_rcp) >> 8, cbi = wave - ksi * a.cbw;
    const int q = lane >> 4, l16 = lane & 15;
    const int cb = (int)blockIdx.x * a.cbw + cbi;
    const bool cb_ok = cb < a.n_cb;
    const int cbc = cb_ok ? cb : a.n_cb - 1;                 // clamp: keeps loads in bounds
    const int kt_b = ksi * a.t_lo + min(ksi, a.t_rem);       // this wave's run of tiles
    const int T = a.t_lo + (ksi < a.t_rem ? 1 : 0);
    const int row_stride = a.K * (A16 ? 2 : 1) + XS_PAD;
    float* s_red = reinterpret_cast<float*>(smem);           // [16 waves][4 rows]
    int8_t* xs = smem + HDR;                                 // int8 rows

    W2_GEMV_MARK_DECL;
    W2_GEMV_MARK(0);
    // ---- 1. the activation rows: unconditional vector loads, issued before the weight loads
    constexpr int ES = XT == 1 ? 4 : XT >= 2 ? 2 : 1;        // bytes per source element
    constexpr int PR = NP;                                   // register slots per row
    static_assert(NP * RL <= xslots(RL, XT), "too many register slots");
    const int ppr = a.K * ES / 16;                           // 16-byte pieces per row
    uint4 pc[RL][PR];
#pragma unroll
    for (int r = 0; r < RL; ++r) {
        const int rr = r < a.M ? r : a.M - 1;
        const __amdgpu_buffer_rsrc_t xr =
            make_rsrc(reinterpret_cast<const char*>(a.X) + (int64_t)rr * a.ldx * ES, r < a.M ? (uint32_t)a.K * ES : 0u);   // rows past M: nothing to fetch
#pragma unroll
        for (int j = 0; j < PR; ++j) {                       // pieces past the end of the row: out of range, zeros
            const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(xr, (tid + j * threads) * 16, 0, 0);
            pc[r][j] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    }

    // The rows' scales for the epilogue.  One or two rows: in registers (scalar loads).  More: the scale of
    // row `tid`, parked in LDS below; unconditional like every load here (past M it is out of range).
    constexpr bool SX_IN_REGS = RL <= 2;
    float sxv[SX_IN_REGS ? RL : 1] = {};
    float sx_mine = 0.f;
    if constexpr (XT == 0 && !DBG) {
        if constexpr (SX_IN_REGS) {
#pragma unroll
            for (int r = 0; r < RL; ++r) sxv[r] = a.sx[r < a.M ? r : a.M - 1];
        } else {
            sx_mine = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(make_rsrc(a.sx, (uint32_t)a.M * 4u), tid * 4, 0, 0));
        }
    }

    // ---- 2. the first W tiles of the weight stream
    const int64_t tile0 = (int64_t)cbc * a.n_kt + kt_b;
    const __amdgpu_buffer_rsrc_t wr =                        // exactly this wave's run: tiles [0, T)
        make_rsrc(reinterpret_cast<const char*>(a.codes) + tile0 * TILE_BYTES, (uint32_t)T * TILE_BYTES);
    // The scales of the whole run, [T][16 columns][GPT] bf16, are contiguous: one 16-byte load per lane
    // (two for G = 64) fetches up to 16 tiles' worth, parked in this wave's LDS slice and read back per tile
    // (measured: one small scale load per tile, a second memory request per KiB of codes, cost 0.4 to 0.9 us
    // on 4096 x 28672).
    constexpr int SPT = TILE_N * GPT * 2;                    // bytes of scales per tile: 64 or 128
    constexpr int NSL = MAX_RUN * SPT / 1024;                // 16-byte loads per lane: 1 or 2
    const __amdgpu_buffer_rsrc_t sr =
        make_rsrc(reinterpret_cast<const char*>(a.scales) + tile0 * SPT, (uint32_t)T * SPT);
    const int w_lane = lane * 16;
    u32x4 tr[W];
    auto issue = [&](int i, u32x4& dst) {                    // i: tile of the run (uniform); past the end: zeros, no traffic
        dst = load_tile(wr, w_lane, i);
    };
    u32x4 sc_regs[NSL];
#pragma unroll
    for (int j = 0; j < NSL; ++j) sc_regs[j] = __builtin_amdgcn_raw_buffer_load_b128(sr, w_lane + j * 1024, 0, 0);
#pragma unroll
    for (int u = 0; u < W; ++u) issue(u, tr[u]);
    W2_GEMV_MARK(1);
    // The rest of the arguments, fetched here, under the latency of the loads just issued: left to the compiler
    // their scalar loads sit right in front of the first barrier and in the epilogue, where a wave waits them out.
    asm volatile("" ::"s"(a.red_off), "s"(a.sc_off), "s"(a.xg_off), "s"(a.outs_magic), "s"(a.sx), "s"(a.Y), "s"(a.acc_out),
                 "s"(a.ldy), "s"(a.N), "s"(a.epi.bias), "s"(a.epi.act));

    // ---- 3. quantise (or copy) the rows into LDS
    if constexpr (XT == 0) {
#pragma unroll
        for (int r = 0; r < RL; ++r)
#pragma unroll
            for (int j = 0; j < PR; ++j) {
                const int i = tid + j * threads;
                if (i < ppr && r < a.M) *reinterpret_cast<uint4*>(xs + r * row_stride + i * 16) = pc[r][j];
            }
        // (here, not at the load: a store right behind it would hold up the weight loads)
        if (!DBG && !SX_IN_REGS && tid < a.M) s_red[SX_SLOT + tid] = sx_mine;
    } else if constexpr (A16) {
        // bf16 rows as they are, de-interleaved per 16-k block ([8 even k | 8 odd k]: the two matrix operands of
        // a lane are then one 16-byte read each), and -130 x the sum of every group of every row.  A piece
        // is 8 values; the G / 8 pieces of a group sit in consecutive lanes of one row of 16 lanes.
        constexpr int PPG = G / 8;
        float* xg = reinterpret_cast<float*>(smem + a.xg_off);
#pragma unroll
        for (int r = 0; r < RL; ++r)
#pragma unroll
            for (int j = 0; j < PR; ++j) {
                const int i = tid + j * threads;
                const uint32_t d[4] = {pc[r][j].x, pc[r][j].y, pc[r][j].z, pc[r][j].w};
                float sum = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) sum += __uint_as_float(d[e] << 16) + __uint_as_float(d[e] & 0xffff0000u);
                sum += dpp_move_f32<0xB1>(sum);              // pairs, quads, eights, (sixteen) lanes: every lane
                sum += dpp_move_f32<0x4E>(sum);              // ends with its group's sum, added in one fixed order
                sum += dpp_move_f32<0x141>(sum);
                if constexpr (PPG == 16) sum += dpp_move_f32<0x140>(sum);
                if (i < ppr && r < a.M) {
                    const uint2 ev = make_uint2(__builtin_amdgcn_perm(d[1], d[0], 0x05040100u), __builtin_amdgcn_perm(d[3], d[2], 0x05040100u));
                    const uint2 od = make_uint2(__builtin_amdgcn_perm(d[1], d[0], 0x07060302u), __builtin_amdgcn_perm(d[3], d[2], 0x07060302u));
                    int8_t* blk = xs + r * row_stride + (i >> 1) * 32 + (i & 1) * 8;
                    *reinterpret_cast<uint2*>(blk) = ev;
                    *reinterpret_cast<uint2*>(blk + 16) = od;
                    if ((i & (PPG - 1)) == 0) xg[(i / PPG) * XGS + r] = -ZP16 * sum;
                }
            }
        // no activation scale: the epilogue's sx * 2^-6 is exactly 1
        if constexpr (SX_IN_REGS) {
#pragma unroll
            for (int r = 0; r < RL; ++r) sxv[r] = 64.0f;
        } else if (tid < (WIDE ? RL : 4)) s_red[SX_SLOT + tid] = 64.0f;
    } else {
        float amax[RL];
#pragma unroll
        for (int r = 0; r < RL; ++r) {
            float m = 0.f;
#pragma unroll
            for (int j = 0; j < PR; ++j) {
                const uint32_t d[4] = {pc[r][j].x, pc[r][j].y, pc[r][j].z, pc[r][j].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if constexpr (XT == 2) {
                        m = fmaxf(m, fabsf(__uint_as_float(d[e] << 16)));
                        m = fmaxf(m, fabsf(__uint_as_float(d[e] & 0xffff0000u)));
                    } else {
                        m = fmaxf(m, fabsf(__uint_as_float(d[e])));
                    }
                }
            }
            amax[r] = wave_max_f32(m);
        }
        W2_GEMV_MARK(8);
        // the waves' partial maxima: [wave][4] floats in the header; the wide form's [wave][RL] in the scratch of
        // the final reduction, which nothing touches before the stream is over
        float* s_max = WIDE ? reinterpret_cast<float*>(smem + a.red_off) : s_red;
        constexpr int MS = WIDE ? RL : 4;
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < RL; ++r) s_max[wave * MS + r] = amax[r];
        }
        __syncthreads();
        W2_GEMV_MARK(9);
        // The rows' maxima: one read per wave brings all its rows' partial maxima.  Only 127 / amax stands between a
        // wave and its quantising; the row's scale amax / 127, the other correctly rounded division, is wanted in the
        // epilogue only: for one or two rows the threads that store results divide there (sxv holds amax until
        // then), for more the first threads of the workgroup do it here, one row each, the other waves pass by.
        float inv[RL], mrow[RL];
#pragma unroll
        for (int r = 0; r < RL; ++r) mrow[r] = 0.f;
        for (int w = 0; w < n_waves; ++w) {
            typedef float vrow __attribute__((ext_vector_type(RL == 3 || WIDE ? 4 : RL)));
            if constexpr (RL == 1) {
                mrow[0] = fmaxf(mrow[0], s_red[w * 4]);
            } else if constexpr (WIDE) {
#pragma unroll
                for (int r4 = 0; r4 < RL / 4; ++r4) {
                    const v4f v = *reinterpret_cast<const v4f*>(s_max + w * MS + 4 * r4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) mrow[4 * r4 + e] = fmaxf(mrow[4 * r4 + e], v[e]);
                }
            } else {
                const vrow v = *reinterpret_cast<const vrow*>(s_red + w * 4);
#pragma unroll
                for (int r = 0; r < RL; ++r) mrow[r] = fmaxf(mrow[r], v[r]);
            }
        }
        if constexpr (RL == 1) {
            inv[0] = mrow[0] > 0.f ? __fdiv_rn(127.0f, mrow[0]) : 0.f;
        } else {
            // one division for all rows: lane r divides for row r, the quotients come back through scalar registers
            float mm = mrow[0];
#pragma unroll
            for (int r = 1; r < RL; ++r) mm = lane == r ? mrow[r] : mm;
            const float iv = mm > 0.f ? __fdiv_rn(127.0f, mm) : 0.f;
#pragma unroll
            for (int r = 0; r < RL; ++r) inv[r] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(iv), r));
        }
        if constexpr (SX_IN_REGS) {
#pragma unroll
            for (int r = 0; r < RL; ++r) sxv[r] = mrow[r];
        }
        if constexpr (!SX_IN_REGS) {
            // (LDS: another slot of the header than the partial maxima being read)
            if (tid < RL) {
                float m = mrow[0];
#pragma unroll
                for (int r = 1; r < RL; ++r) m = tid == r ? mrow[r] : m;
                s_red[SX_SLOT + tid] = m > 0.f ? __fdiv_rn(m, 127.0f) : 0.f;
            }
        }
        W2_GEMV_MARK(10);
#pragma unroll
        for (int r = 0; r < RL; ++r)
#pragma unroll
            for (int j = 0; j < PR; ++j) {
                const int i = tid + j * threads;
                if (i < ppr && r < a.M) {
                    const uint32_t d[4] = {pc[r][j].x, pc[r][j].y, pc[r][j].z, pc[r][j].w};
                    if constexpr (XT == 2) {
                        uint32_t b[8];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            b[2 * e] = quant_bits(__uint_as_float(d[e] << 16), inv[r]);
                            b[2 * e + 1] = quant_bits(__uint_as_float(d[e] & 0xffff0000u), inv[r]);
                        }
                        *reinterpret_cast<uint2*>(xs + r * row_stride + i * 8) =
                            make_uint2(pack4(b[0], b[1], b[2], b[3]), pack4(b[4], b[5], b[6], b[7]));
                    } else {
                        *reinterpret_cast<uint32_t*>(xs + r * row_stride + i * 4) =
                            pack4(quant_bits(__uint_as_float(d[0]), inv[r]), quant_bits(__uint_as_float(d[1]), inv[r]),
                                  quant_bits(__uint_as_float(d[2]), inv[r]), quant_bits(__uint_as_float(d[3]), inv[r]));
                    }
                }
            }
    }
    // this wave's scales -> its LDS slice (read back by the same wave only: LDS operations of a wave complete in order)
    int8_t* sc_lds = smem + a.sc_off + wave * (MAX_RUN * SPT);
#pragma unroll
    for (int j = 0; j < NSL; ++j) *reinterpret_cast<u32x4*>(sc_lds + j * 1024 + w_lane) = sc_regs[j];
    __syncthreads();
    W2_GEMV_MARK(2);

    // ---- 4. the stream: up-convert and compute
    float y[RT][RA];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int r = 0; r < RA; ++r) y[rt][r] = 0.f;
    // Two accumulators alternate between groups; a finished group is dequantised after the next
    // group's first matrix instruction has been issued, so its int -> float conversion does not wait
    // for the matrix pipe.
    v4i acc[2][RT];
    v4f accf[2] = {v4f{0.f, 0.f, 0.f, 0.f}, v4f{0.f, 0.f, 0.f, 0.f}};      // the w2a16 form's
    const Bf16Consts kc = bf16_consts();
    (void)kc; (void)accf;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[0][rt] = acc[1][rt] = v4i{0, 0, 0, 0};
    float pend_sw = 0.f;                                     // scale of the group waiting in acc[1]: none yet
    int pend_g = -1;                                         // its index (debug export)
    auto dequant = [&](int b) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int r = 0; r < RA; ++r) {
                if constexpr (DBG) {
                    const int64_t n = (int64_t)cb * TILE_N + l16;
                    const int row = WIDE ? rt * 16 + 4 * q + r : r;
                    if (pend_g >= 0 && (WIDE || q == 0) && cb_ok && n < a.N && row < a.M)
                        a.acc_out[((int64_t)row * (a.K / G) + pend_g) * a.N + n] = acc[b][rt][r] >> 6;
                }
                if constexpr (A16) y[rt][r] = fmaf(pend_sw, accf[b][r], y[rt][r]);
                else y[rt][r] = fmaf(pend_sw, (float)acc[b][rt][r], y[rt][r]);
            }
    };
    // LDS address of this lane's A operand: row (lane & 15, padded rows repeat the last), 16-byte piece lane >> 4
    uint32_t a_lane[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int arow = rt * 16 + l16 < a.M ? rt * 16 + l16 : a.M - 1;
        a_lane[rt] = (uint32_t)(HDR + arow * row_stride + q * (A16 ? 32 : 16));
    }
    constexpr int NA = A16 ? 8 : 4;                          // A operands per tile and row tile
    auto read_aop = [&](int kt, v4i (&aop)[RT][NA]) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int8_t* p = smem + a_lane[rt] + (uint32_t)kt * (TILE_K * (A16 ? 2 : 1));
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if constexpr (A16) {
                    aop[rt][2 * t] = *reinterpret_cast<const v4i*>(p + t * 128);            // even k of the lane's block
                    aop[rt][2 * t + 1] = *reinterpret_cast<const v4i*>(p + t * 128 + 16);   // odd k
                } else {
                    aop[rt][t] = *reinterpret_cast<const v4i*>(p + t * 64);
                }
            }
        }
    };
    // w2a16: what a group's accumulator starts from, the lane's four rows of the tile's groups (rows 0..3 in
    // every lane; the wide form: rows 4q..4q+3)
    auto read_cinit = [&](int kt, v4f (&ci)[GPT]) {
        if constexpr (A16) {
            const float* xg = reinterpret_cast<const float*>(smem + a.xg_off) + kt * (GPT * XGS) + (WIDE ? 4 * q : 0);
#pragma unroll
            for (int g = 0; g < GPT; ++g) ci[g] = *reinterpret_cast<const v4f*>(xg + g * XGS);
        }
    };
    const int8_t* sc_lane = sc_lds + l16 * (GPT * 2);
    auto read_scales = [&](int i, uint32_t (&sc)[2]) {       // tile i of the run
        if constexpr (G == 128) {
            sc[0] = *reinterpret_cast<const uint32_t*>(sc_lane + i * SPT);
            sc[1] = 0;
        } else {
            const uint2 t = *reinterpret_cast<const uint2*>(sc_lane + i * SPT);
            sc[0] = t.x; sc[1] = t.y;
        }
    };
    auto compute = [&](int kt, const u32x4& cur, const uint32_t (&sc)[2], const v4i (&aop)[RT][NA], const v4f (&ci)[GPT]) {
        const uint32_t wd[4] = {cur[0], cur[1], cur[2], cur[3]};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int gi = G == 64 ? t : t >> 1;             // group inside the tile
            const int b = gi & 1;                            // its accumulator (groups per tile are even)
            const bool first = G == 64 || !(t & 1);
            if constexpr (A16) {
                v4i b0, b1;
                upconvert_bf16(wd[t], kc, b0, b1);
                accf[b] = mfma_bf16(aop[0][2 * t], b0, first ? ci[gi] : accf[b]);
                accf[b] = mfma_bf16(aop[0][2 * t + 1], b1, accf[b]);
            } else {
                int u[4];
                upconvert(wd[t], u);
                const v4i bop = {u[0], u[1], u[2], u[3]};
                const v4i zero = {0, 0, 0, 0};
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[b][rt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[rt][t], bop, first ? zero : acc[b][rt], 0, 0, 0);
            }
            if (first) dequant(b ^ 1);                       // the group before this one
            if (G == 64 || (t & 1)) {
                const uint32_t pair = (G == 128 || gi < 2) ? sc[0] : sc[1];
                pend_sw = (gi & 1) ? __uint_as_float(pair & 0xffff0000u) : __uint_as_float(pair << 16);
                pend_g = kt * GPT + gi;
            }
        }
    };
    v4i aop[2][RT][NA];
    uint32_t scl[2][2];
    v4f cin[2][GPT];
    read_aop(kt_b, aop[0]);
    read_scales(0, scl[0]);
    read_cinit(kt_b, cin[0]);
    for (int base = 0; base < T; base += W) {
#pragma unroll
        for (int u = 0; u < W; ++u) {
            const int i = base + u;
            // the slot is refilled before its tile is multiplied (the tile moves to other registers): a wave's
            // requests stay W deep while it computes, instead of W - 1 and a gap
            const u32x4 cur = tr[u];
            issue(i + W, tr[u]);                             // unconditional: keeps the count of loads in flight static
            if (i < T) {                                     // uniform
                read_aop(kt_b + min(i + 1, T - 1), aop[(u + 1) & 1]);     // a tile ahead; clamped: stays inside the rows
                read_scales(min(i + 1, T - 1), scl[(u + 1) & 1]);
                read_cinit(kt_b + min(i + 1, T - 1), cin[(u + 1) & 1]);
                compute(kt_b + i, cur, scl[u & 1], aop[u & 1], cin[u & 1]);
                if (i == 0) { W2_GEMV_MARK(3); }
            }
        }
    }
    dequant(1);                                              // the last group (it sits in acc[1])
    W2_GEMV_MARK(4);
    if constexpr (DBG) return;

    // ---- 5. reduce the k-ranges through LDS (fixed order), dequantise, store
    float* red = reinterpret_cast<float*>(smem + a.red_off);   // [waves][RL][16]; its own region: no barrier before the writes
    if (WIDE ? 4 * q < RL : q == 0) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int r = 0; r < RA; ++r) red[(wave * RL + rt * 16 + (WIDE ? 4 * q : 0) + r) * 16 + l16] = y[rt][r];
    }
    __syncthreads();
    W2_GEMV_MARK(5);
    const bool gated = a.epi.act == ACT_SILU_MUL;
    const int outs = gated ? (a.cbw >> 1) * 16 : a.cbw * 16;
    if constexpr (SX_IN_REGS) {
        // one or two rows: a thread per output column, the rows in turn
        if (tid < outs) {
            if constexpr (XT == 1 || XT == 2) {
#pragma unroll
                for (int r = 0; r < RL; ++r) sxv[r] = sxv[r] > 0.f ? __fdiv_rn(sxv[r], 127.0f) : 0.f;   // amax until here
            }
            const int nl = tid & 15, ci = tid >> 4;
            const int kstride = RL * 16 * a.cbw;             // floats between two k-ranges' partial sums
            auto z = [&](int c, int r) {                     // finished fp32 result of column block c, row r
                const float* p0 = red + (c * RL + r) * 16 + nl;
                float s = 0.f;
                for (int k0 = 0; k0 < a.ks; k0 += 4) {       // four reads in flight, added in order
                    float part[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) part[j] = p0[min(k0 + j, a.ks - 1) * kstride];
#pragma unroll
                    for (int j = 0; j < 4; ++j) s = k0 + j < a.ks ? s + part[j] : s;
                }
                return s * (sxv[r] * 0.015625f);
            };
            if (!gated) {
                const int64_t nn = ((int64_t)blockIdx.x * a.cbw + ci) * TILE_N + nl;
                if (nn < a.N) {
                    const float bias = a.epi.bias ? bf16_to_f32(a.epi.bias[nn]) : 0.f;
#pragma unroll
                    for (int r = 0; r < RL; ++r) {
                        if (r < a.M) {
                            float v = z(ci, r) + bias;
                            if (a.epi.act == ACT_SILU) v = silu_f32(v);
                            a.Y[(int64_t)r * a.ldy + nn] = f32_to_bf16_rne(v);
                        }
                    }
                }
            } else {
                const int64_t first_cb = (int64_t)blockIdx.x * a.cbw;       // even
                const int64_t ng = (first_cb + 2 * ci) * TILE_N + nl, nu = ng + TILE_N;
                if (nu < a.N) {                              // N % 32 == 0: both or neither
                    const float bg = a.epi.bias ? bf16_to_f32(a.epi.bias[ng]) : 0.f;
                    const float bu = a.epi.bias ? bf16_to_f32(a.epi.bias[nu]) : 0.f;
#pragma unroll
                    for (int r = 0; r < RL; ++r) {
                        if (r < a.M) {
                            const float g = z(2 * ci, r) + bg, u = z(2 * ci + 1, r) + bu;
                            a.Y[(int64_t)r * a.ldy + ((first_cb >> 1) + ci) * TILE_N + nl] = f32_to_bf16_rne(silu_f32(g) * u);
                        }
                    }
                }
            }
        }
        W2_GEMV_MARK(6);
        return;
    }
    // one output per thread and step: column `item % outs` (a power of two), row `item / outs`; the k-ranges'
    // partial sums are fetched four at a time, then added in a fixed order
    const int kstride = RL * 16 * a.cbw;                     // floats between two k-ranges' partial sums
    for (int item = tid; item < a.M * outs; item += threads) {
        int r;
        // item / outs: by the magic multiplier below 4096 items; the wide form (up to 32 x 256 items) in fp32, exact
        // for these sizes (item + 0.5 keeps the quotient clear of an integer by more than the rounding error)
        if constexpr (WIDE) r = (int)(((float)item + 0.5f) * __frcp_rn((float)outs));
        else r = (int)(((uint32_t)item * (uint32_t)a.outs_magic) >> 20);
        const int col = item - r * outs;
        const int nl = col & 15, ci = col >> 4;
        const float sxr = s_red[SX_SLOT + r] * 0.015625f;
        auto z = [&](int c) {                                // finished fp32 result of column block c, row r
            const float* p0 = red + (c * RL + r) * 16 + nl;
            float s = 0.f;
            for (int k0 = 0; k0 < a.ks; k0 += 4) {           // four reads in flight, added in order
                float part[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) part[j] = p0[min(k0 + j, a.ks - 1) * kstride];
#pragma unroll
                for (int j = 0; j < 4; ++j) s = k0 + j < a.ks ? s + part[j] : s;
            }
            return s * sxr;
        };
        if (!gated) {
            const int64_t nn = ((int64_t)blockIdx.x * a.cbw + ci) * TILE_N + nl;
            if (nn < a.N) {
                float v = z(ci) + (a.epi.bias ? bf16_to_f32(a.epi.bias[nn]) : 0.f);
                if (a.epi.act == ACT_SILU) v = silu_f32(v);
                a.Y[(int64_t)r * a.ldy + nn] = f32_to_bf16_rne(v);
            }
        } else {
            const int64_t first_cb = (int64_t)blockIdx.x * a.cbw;           // even
            const int64_t ng = (first_cb + 2 * ci) * TILE_N + nl, nu = ng + TILE_N;
            if (nu < a.N) {                                  // N % 32 == 0: both or neither
                const float g = z(2 * ci) + (a.epi.bias ? bf16_to_f32(a.epi.bias[ng]) : 0.f);
                const float u = z(2 * ci + 1) + (a.epi.bias ? bf16_to_f32(a.epi.bias[nu]) : 0.f);
                a.Y[(int64_t)r * a.ldy + ((first_cb >> 1) + ci) * TILE_N + nl] = f32_to_bf16_rne(silu_f32(g) * u);
            }
        }
    }
    W2_GEMV_MARK(6);
}

// Workgroup shape: waves = cbw column blocks x ks k-ranges.  Rules from graph-timed sweeps over the 8B-
// and 27B-class projections at M = 1 (waves per workgroup 4 / 8 / 16, every split, windows 2 / 4 / 8):
//   - K is split (ks, a power of two) until the grid has at least 2048 waves, two per SIMD: 4096 x 4096 and
//     4096 x 6144 want ks = 8 (runs of two tiles), 4096 x 28672 ks = 2 (runs of eight), 14336 x 4096 ks = 8
//     (runs of seven); more waves than that only add per-wave fixed work, fewer leave the memory system short
//     of requests;
//   - eight waves per workgroup (sixteen when ks = 16, or when the rows need the threads);
//   - five rows and more (the wide form): the rows re-read by every workgroup weigh as much as the weights, so
//     the workgroups are as wide as still leaves about 192 of them (4096 x 28672 at M = 16: 10.1 us with 8 x 1
//     against 12.5 with 4 x 2; 4096 x 6144: 5.2 with 2 x 4 against 7.5 with 1 x 8);
//   - window 2 for runs of up to four tiles.  Longer runs: 4 in grids of more than 768 workgroups (8192 x
//     57344 gains 10 %) and of up to 256 (14336 x 4096: 5 %), 2 between (5120 x 34816 loses 11 to 15 % to the
//     deeper window, 4096 x 28672 3 % with int8 rows and gains 1 % with rows quantised in the kernel: more
//     bytes in flight than about 10 MB over the chip does not pay); 8 was never better.
struct Cfg { int cbw, ks, window; };

static Cfg pick(const w2_tuning_t& tune, int64_t n_cb, int64_t n_kt, bool even_cbw, int min_threads, int max_w, int rows, int xt)
{
    Cfg c;
    if (tune.gemv_cbw || tune.gemv_ks) {                     // forced shape, any numbers: the caller of pick checks it
        c.cbw = tune.gemv_cbw ? tune.gemv_cbw : 1;
        c.ks = tune.gemv_ks ? tune.gemv_ks : (8 / c.cbw > 0 ? 8 / c.cbw : 1);
        if (c.ks > n_kt) c.ks = (int)n_kt;
        const int64_t run = (n_kt + c.ks - 1) / c.ks;
        c.window = tune.gemv_window ? tune.gemv_window : run > 4 ? 4 : 2;
        return c;
    }
    if (tune.small_waves || tune.small_cbw) {                // forced shape (tests, sweeps)
        int waves = tune.small_waves ? tune.small_waves : 8;
        int p = 1;
        while (p * 2 <= waves) p <<= 1;                      // powers of two only
        waves = p;
        c.cbw = tune.small_cbw ? tune.small_cbw : waves;
        if (c.cbw > waves) c.cbw = waves;
        c.ks = waves / c.cbw;
    } else if (rows > 4) {
        // the wide form: every workgroup stages all rows, so as many column blocks per workgroup (up to 4;
        // 8 from 13 rows on) as leave about 192 workgroups; eight waves
        // (w2a16: 8 from 9 rows on: 4096 x 28672 at M = 9 13.1 us with 8 x 1 waves, 17.0 with 4 x 2)
        int cbw = rows > (xt == 3 ? 8 : 12) ? 8 : 4;
        while (cbw > 1 && n_cb / cbw < 192) cbw >>= 1;
        // ... unless another width unloads the busiest CU by a fifth or more (the rule of the narrow form below:
        // 5120 x 34816 at M = 8 in 726 workgroups of 3 x 2 waves 11.8 us, in 544 of 4 x 2 13.9)
        if (n_cb >= 1024) {
            auto busiest = [&](int cb) { const int64_t w = (n_cb + cb - 1) / cb; return ((w + 255) / 256) * cb; };
            int best = cbw;
            for (int cb = 8; cb >= 1; --cb) {
                const int ks = 8 / cb;
                if ((even_cbw && (cb & 1)) || cb * ks * 64 < min_threads || (n_kt + ks - 1) / ks > MAX_RUN || n_cb / cb < 192) continue;
                if (busiest(cb) * 5 <= busiest(cbw) * 4 && busiest(cb) < busiest(best)) best = cb;
            }
            cbw = best;
        }
        // w2a16 rows that leave room for one workgroup on a CU, narrow projection, more workgroups than CUs: twice
        // as wide, one round of workgroups that stage the rows once (5120 x 5120 at M = 8)
        if (xt == 3 && (int64_t)rows * (n_kt * 512 + XS_PAD) > 78 * 1024 && n_cb <= 512 && n_cb / cbw > 256 && cbw < 8 &&
            (n_kt + 8 / (cbw * 2) - 1) / (8 / (cbw * 2)) <= MAX_RUN)
            cbw <<= 1;
        c.cbw = cbw;
        c.ks = 8 / cbw;
    } else {
        int ks = 1;
        while (ks < max_w && n_cb * ks < 2048 && n_kt / (ks * 2) >= 1) ks <<= 1;
        while (ks < max_w && (n_kt + ks - 1) / ks > MAX_RUN) ks <<= 1;
        c.ks = ks;
        c.cbw = ks >= 8 ? 1 : 8 / ks;                        // eight waves; sixteen when ks = 16
        if ((xt == 1 || xt == 2) && ks == 8 && n_kt <= 32 && (n_cb >= 320 || rows <= 2) && 4 * (n_cb >= 320 ? 2 : 1) * 64 >= min_threads) {
            // rows quantised in the kernel, narrow projection: every workgroup re-reads and re-quantises the
            // row, so half as many k-ranges (runs of four or five tiles) and, from 320 column blocks on, two
            // column blocks per workgroup (4096 x 6144 4.5 against 4.9 us, 5120 x 5120 4.9 against 5.5;
            // 4096 x 4096 keeps one column block, in workgroups of four waves, for one or two rows: 3.5
            // against 3.9; at three and four rows it loses), where that many threads can hold the rows
            c.ks = 4;
            c.cbw = n_cb >= 320 ? 2 : 1;
        }
    }
    if (xt == 3 && rows == 1 && n_cb >= 1024 && n_kt >= 4 && n_kt <= 4 * MAX_RUN && !tune.small_waves && !tune.small_cbw && !even_cbw) {
        // w2a16 (twice the vector work per code word), one row, wide projection: small workgroups of four waves
        // spread evenly over the CUs (4096 x 28672: 9.4 us against 10.0 with 4 x 2 waves; 5120 x 34816: 13.7 against 14.7)
        c.cbw = 1;
        c.ks = 4;
    }
    if (even_cbw && (c.cbw & 1)) c.cbw = 2;                  // the gated epilogue pairs adjacent column blocks
    while (c.cbw * c.ks > max_w) {                           // at most 16 waves (8 in the wide form)
        if (c.ks > 1) c.ks >>= 1; else c.cbw >>= 1;
    }
    if (rows <= 4) {
        // Up to four rows the workgroup may hold any number of column blocks.
        // (a) The chip's time follows the CU that holds the most column blocks: with every workgroup resident,
        //     ceil(workgroups / 256) of them share the busiest CU.  Where another width cuts that by a fifth or
        //     more, take it (5120 x 34816: three column blocks, 726 workgroups, at most 9 blocks on a CU against 12
        //     with four: 9.9 against 10.9 us at M = 1; smaller differences do not show: 4096 x 28672 with 7 x 256).
        auto busiest = [&](int cb) { const int64_t w = (n_cb + cb - 1) / cb; return ((w + 255) / 256) * cb; };
        if (rows == 1 && !tune.small_waves && !tune.small_cbw && n_cb >= 1024) {
            int best = c.cbw;
            for (int cb = 8; cb >= 1; --cb) {
                if ((even_cbw && (cb & 1)) || cb * c.ks > max_w || cb * c.ks * 64 < min_threads) continue;
                if (busiest(cb) * 5 <= busiest(c.cbw) * 4 && busiest(cb) < busiest(best)) best = cb;
            }
            // (4096 x 28672 in 896 workgroups of 2 x 2 waves: 1 % faster than 4 x 2 back to back in a replayed graph,
            // 4 % slower per launch as the profiler times it, dispatch included: not taken)
            c.cbw = best;
        }
    }
    if (c.ks > n_kt) {
        c.ks = 1;
        while (c.ks * 2 <= n_kt) c.ks <<= 1;
    }
    // a run is at most MAX_RUN tiles: split K further (fewer column blocks per workgroup, then more waves)
    while ((n_kt + c.ks - 1) / c.ks > MAX_RUN && c.cbw > 1 && !(c.cbw & 1) && !(even_cbw && c.cbw == 2)) { c.cbw >>= 1; c.ks <<= 1; }
    while ((n_kt + c.ks - 1) / c.ks > MAX_RUN && c.cbw * c.ks * 2 <= max_w) c.ks <<= 1;
    // The rows need the threads.  Up to four rows: one column block more at a time, not the next power of two
    // (5120 x 34816 with four fp32 rows quantised in the kernel: ten waves 14.8 us, sixteen 20.5).
    if (rows <= 4) {
        const int step = even_cbw ? 2 : 1;
        while (c.cbw * c.ks * 64 < min_threads && (c.cbw + step) * c.ks <= max_w) c.cbw += step;
    }
    while (c.cbw * c.ks * 64 < min_threads && c.cbw * c.ks * 2 <= max_w) c.cbw <<= 1;
    const int64_t run = (n_kt + c.ks - 1) / c.ks;
    const int64_t wgs = (n_cb + c.cbw - 1) / c.cbw;
    // (w2a16: a window of two everywhere; deeper ones lost on every shape of the sweep)
    c.window = tune.gemv_window ? tune.gemv_window : xt == 3 ? 2 : (run > 4 && (wgs > 768 || wgs <= 256)) || c.cbw * c.ks == 4 ? 4 : 2;
    return c;
}

template <int G, int RL, int XT, int NP, bool DBG>
static int launch_w(const Args& a, const Cfg& c, size_t lds, hipStream_t stream)
{
    const dim3 grid((unsigned)((a.n_cb + c.cbw - 1) / c.cbw)), block(64 * c.cbw * c.ks);
    auto go = [&](auto kern) {
        if (int rc = ensure_dynamic_lds((const void*)kern, lds, "w2_matmul_a8[gemv]")) return rc;
        ArgsRest r;
        r.outs_magic = a.outs_magic; r.red_off = a.red_off; r.sc_off = a.sc_off; r.xg_off = a.xg_off;
        r.sx = a.sx; r.Y = a.Y; r.acc_out = a.acc_out; r.ldy = a.ldy; r.N = a.N; r.epi = a.epi;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, a.X, a.ldx, a.codes, a.scales, a.K, a.M, a.n_cb, a.n_kt,
                           a.cbw_rcp, a.cbw | (a.ks << 8) | (a.t_lo << 16) | (a.t_rem << 24), r);
        return check_launch("w2_matmul_a8[gemv]");
    };
    if (c.window >= 8) return go(a8_gemv_kernel<G, RL, XT, 8, NP, DBG>);
    if (c.window >= 4) return go(a8_gemv_kernel<G, RL, XT, 4, NP, DBG>);
    return go(a8_gemv_kernel<G, RL, XT, 2, NP, DBG>);
}

template <int G, int RL, int XT, bool DBG>
static int launch_np(const Args& a, const Cfg& c, size_t lds, int np, hipStream_t stream)
{
    constexpr int MAXNP = xslots(RL, XT) / RL;
    if (np <= 1) return launch_w<G, RL, XT, 1, DBG>(a, c, lds, stream);
    if constexpr (MAXNP >= 2) { if (np <= 2) return launch_w<G, RL, XT, 2, DBG>(a, c, lds, stream); }
    if constexpr (MAXNP >= 4) { if (np <= 4) return launch_w<G, RL, XT, 4, DBG>(a, c, lds, stream); }
    if constexpr (MAXNP >= 8) { if (np <= 8) return launch_w<G, RL, XT, 8, DBG>(a, c, lds, stream); }
    return launch_w<G, RL, XT, MAXNP, DBG>(a, c, lds, stream);
}

}  // namespace gemv

// int8 rows: up to 32 (the wide form from five rows on); rows quantised in the kernel: up to eight
bool a8_gemv_supports(int64_t M) { return M >= 1 && M <= 32; }

// xt: 0 = int8 rows (X = xq, sx given), 1 = fp32 rows, 2 = bf16 rows.  Returns W2_ERR_UNSUPPORTED_SHAPE
// (with a message, nothing launched) when the rows do not fit a workgroup.
int launch_a8_gemv(const A8Args& a8, const void* X, int xt, int64_t ldx, hipStream_t stream)
{
    using namespace gemv;
    const int64_t M = a8.M, K = a8.K;
    if (!a8_gemv_supports(M) || (xt != 0 && M > 8)) {
        set_error("w2_matmul_a8[gemv]: M must be 1..32 (1..8 for rows quantised in the kernel)");
        return W2_ERR_UNSUPPORTED_SHAPE;
    }
    const int rl = M <= 1 ? 1 : M <= 2 ? 2 : M <= 4 ? 4 : M <= 8 ? 8 : M <= 16 ? 16 : 32;
    const int max_w = rl > 4 ? 8 : 16;                       // max_waves(rl)
    const int es = xt == 1 ? 4 : xt == 2 ? 2 : 1;
    const int64_t ppr = K * es / 16;                         // 16-byte pieces per row
    const int pr = xslots(rl, xt) / rl;                      // register slots per row and thread
    const int min_threads = (int)((ppr + pr - 1) / pr);
    const size_t xs_bytes = ((size_t)(M < rl ? M : rl) * (K + XS_PAD) + 15) & ~(size_t)15;
    const char* too_large = "w2_matmul_a8[gemv]: M*K too large for one workgroup (use w2_quantize_rows + w2_matmul_a8)";
    if (min_threads > 64 * max_w || xs_bytes > 160 * 1024) {
        set_error(too_large);
        return W2_ERR_UNSUPPORTED_SHAPE;
    }
    const Cfg c = pick(a8.tune, a8.n_cb, a8.n_kt, a8.epi.act == ACT_SILU_MUL, min_threads, max_w, (int)M, xt);
    const int waves = c.cbw * c.ks;
    if (waves > max_w || (a8.epi.act == ACT_SILU_MUL && (c.cbw & 1))) {
        set_error("w2_matmul_a8[gemv]: workgroup shape %d x %d: at most %d waves, an even number of column blocks for the gated epilogue", c.cbw, c.ks, max_w);
        return W2_ERR_INVALID_ARG;
    }
    // local memory: header, rows, reduction scratch, the waves' scale slices; a CU has 160 KiB
    const size_t lds_need = HDR + xs_bytes + (size_t)waves * rl * 16 * sizeof(float) +
                            (size_t)waves * MAX_RUN * (TILE_N * (TILE_K / a8.G) * 2);
    if (lds_need > 160 * 1024) {
        set_error(too_large);
        return W2_ERR_UNSUPPORTED_SHAPE;
    }
    if (waves * 64 < min_threads) {
        set_error("w2_matmul_a8[gemv]: the forced workgroup shape cannot hold the activation rows");
        return W2_ERR_UNSUPPORTED_SHAPE;
    }
    if ((a8.n_kt + c.ks - 1) / c.ks > MAX_RUN) {
        set_error("w2_matmul_a8[gemv]: K too deep for this workgroup shape (a wave's run is limited to %d tiles)", MAX_RUN);
        return W2_ERR_UNSUPPORTED_SHAPE;
    }
    Args a = {};
    a.codes = a8.codes; a.scales = a8.scales; a.X = X; a.sx = a8.sx; a.Y = a8.Y; a.acc_out = a8.acc_out;
    a.ldx = ldx; a.ldy = a8.ldy; a.N = a8.N; a.K = (int)K; a.M = (int)M;
    a.n_cb = (int)a8.n_cb; a.n_kt = (int)a8.n_kt;
    a.cbw = c.cbw; a.ks = c.ks;
    a.cbw_rcp = (256 + c.cbw - 1) / c.cbw;
    {
        const int outs = (a8.epi.act == ACT_SILU_MUL ? c.cbw / 2 : c.cbw) * 16;
        a.outs_magic = ((1 << 20) + outs - 1) / outs;
    }
    a.t_lo = (int)(a8.n_kt / c.ks); a.t_rem = (int)(a8.n_kt % c.ks);
    a.red_off = (int)(HDR + xs_bytes);
    a.sc_off = a.red_off + waves * rl * 16 * (int)sizeof(float);
    a.epi = a8.epi;
    const size_t lds = lds_need;
    const bool dbg = a8.acc_out != nullptr;
    const int np = (int)((ppr + waves * 64 - 1) / (waves * 64));       // pieces per row and thread (<= XSLOTS / rl: checked above)
#define W2_GEMV(GG, RLL)                                                                               \
    do {                                                                                               \
        if (dbg) return launch_np<GG, RLL, 0, true>(a, c, lds, np, stream);                            \
        if (xt == 0) return launch_np<GG, RLL, 0, false>(a, c, lds, np, stream);                       \
        if (xt == 1) return launch_np<GG, RLL, 1, false>(a, c, lds, np, stream);                       \
        return launch_np<GG, RLL, 2, false>(a, c, lds, np, stream);                                    \
    } while (0)
#define W2_GEMV_WIDE(GG, RLL)                                                                          \
    do {                                                                                               \
        if (dbg) return launch_np<GG, RLL, 0, true>(a, c, lds, np, stream);                            \
        if constexpr (RLL == 8) {                                                                      \
            if (xt == 1) return launch_np<GG, RLL, 1, false>(a, c, lds, np, stream);                   \
            if (xt == 2) return launch_np<GG, RLL, 2, false>(a, c, lds, np, stream);                   \
        }                                                                                              \
        return launch_np<GG, RLL, 0, false>(a, c, lds, np, stream);                                    \
    } while (0)
    if (a8.G == 128) {
        if (rl == 1) W2_GEMV(128, 1);
        if (rl == 2) W2_GEMV(128, 2);
        if (rl == 4) W2_GEMV(128, 4);
        if (rl == 8) W2_GEMV_WIDE(128, 8);
        if (rl == 16) W2_GEMV_WIDE(128, 16);
        W2_GEMV_WIDE(128, 32);
    }
    if (rl == 1) W2_GEMV(64, 1);
    if (rl == 2) W2_GEMV(64, 2);
    if (rl == 4) W2_GEMV(64, 4);
    if (rl == 8) W2_GEMV_WIDE(64, 8);
    if (rl == 16) W2_GEMV_WIDE(64, 16);
    W2_GEMV_WIDE(64, 32);
#undef W2_GEMV_WIDE
#undef W2_GEMV
}

// w2a16 through the same kernel: bf16 rows as they are, up to sixteen of them (the wide form from five on),
// where a workgroup of eight waves can hold them (local memory and registers); false: the caller takes
// another kernel.
static int a16_rl(int64_t M) { return M <= 1 ? 1 : M <= 2 ? 2 : M <= 4 ? 4 : M <= 8 ? 8 : 16; }

bool a16_gemv_supports(const A16Args& a)
{
    using namespace gemv;
    if (a.M < 1 || a.M > 16) return false;
    const int rl = a16_rl(a.M);
    const int64_t ppr = a.K * 2 / 16;
    const int pr = xslots(rl, 3) / rl;
    const size_t lds = HDR + (size_t)a.M * (a.K * 2 + XS_PAD) + 16 + 8 * (size_t)rl * 16 * sizeof(float) +
                       8 * (size_t)MAX_RUN * (TILE_N * (TILE_K / a.G) * 2) + (size_t)(a.K / a.G) * (rl > 4 ? 64 : 16);
    return (ppr + pr - 1) / pr <= 64 * 8 && lds <= 160 * 1024 && (a.n_kt + 7) / 8 <= MAX_RUN;
}

int launch_a16_gemv(const A16Args& a16, hipStream_t stream)
{
    using namespace gemv;
    if (!a16_gemv_supports(a16)) {
        set_error("w2_matmul_a16[gemv]: M must be 1..16 and the rows must fit one workgroup");
        return W2_ERR_UNSUPPORTED_SHAPE;
    }
    const int64_t M = a16.M, K = a16.K;
    const int rl = a16_rl(M);
    const int max_w = max_waves(rl, 3);
    const int64_t ppr = K * 2 / 16;
    const int pr = xslots(rl, 3) / rl;
    const int min_threads = (int)((ppr + pr - 1) / pr);
    const size_t xs_bytes = ((size_t)M * (K * 2 + XS_PAD) + 15) & ~(size_t)15;
    const Cfg c = pick(a16.tune, a16.n_cb, a16.n_kt, a16.epi.act == ACT_SILU_MUL, min_threads, max_w, (int)M, 3);
    const int waves = c.cbw * c.ks;
    if (waves > max_w || waves * 64 < min_threads || (a16.epi.act == ACT_SILU_MUL && (c.cbw & 1)) ||
        (a16.n_kt + c.ks - 1) / c.ks > MAX_RUN) {
        set_error("w2_matmul_a16[gemv]: workgroup shape %d x %d cannot run this problem (at most %d waves, %d threads for the rows, runs of %d tiles)",
                  c.cbw, c.ks, max_w, min_threads, MAX_RUN);
        return a16.tune.gemv_cbw || a16.tune.gemv_ks ? W2_ERR_INVALID_ARG : W2_ERR_UNSUPPORTED_SHAPE;
    }
    Args a;
    a.codes = a16.codes; a.scales = a16.scales; a.X = a16.X; a.sx = nullptr; a.Y = a16.Y; a.acc_out = nullptr;
    a.ldx = a16.ldx; a.ldy = a16.ldy; a.N = a16.N; a.K = (int)K; a.M = (int)M;
    a.n_cb = (int)a16.n_cb; a.n_kt = (int)a16.n_kt;
    a.cbw = c.cbw; a.ks = c.ks;
    a.cbw_rcp = (256 + c.cbw - 1) / c.cbw;
    {
        const int outs = (a16.epi.act == ACT_SILU_MUL ? c.cbw / 2 : c.cbw) * 16;
        a.outs_magic = ((1 << 20) + outs - 1) / outs;
    }
    a.t_lo = (int)(a16.n_kt / c.ks); a.t_rem = (int)(a16.n_kt % c.ks);
    a.red_off = (int)(HDR + xs_bytes);
    a.sc_off = a.red_off + waves * rl * 16 * (int)sizeof(float);
    a.xg_off = a.sc_off + waves * MAX_RUN * (TILE_N * (TILE_K / a16.G) * 2);
    a.epi = a16.epi;
    const size_t lds = (size_t)a.xg_off + (size_t)(K / a16.G) * (rl > 4 ? 64 : 16);
    if (lds > 160 * 1024) {
        set_error("w2_matmul_a16[gemv]: the rows do not fit a workgroup's local memory");
        return W2_ERR_UNSUPPORTED_SHAPE;
    }
    const int np = (int)((ppr + waves * 64 - 1) / (waves * 64));
    if (a16.G == 128) {
        if (rl == 1) return launch_np<128, 1, 3, false>(a, c, lds, np, stream);
        if (rl == 2) return launch_np<128, 2, 3, false>(a, c, lds, np, stream);
        if (rl == 4) return launch_np<128, 4, 3, false>(a, c, lds, np, stream);
        if (rl == 8) return launch_np<128, 8, 3, false>(a, c, lds, np, stream);
        return launch_np<128, 16, 3, false>(a, c, lds, np, stream);
    }
    if (rl == 1) return launch_np<64, 1, 3, false>(a, c, lds, np, stream);
    if (rl == 2) return launch_np<64, 2, 3, false>(a, c, lds, np, stream);
    if (rl == 4) return launch_np<64, 4, 3, false>(a, c, lds, np, stream);
    if (rl == 8) return launch_np<64, 8, 3, false>(a, c, lds, np, stream);
    return launch_np<64, 16, 3, false>(a, c, lds, np, stream);
}

}  // namespace w2
