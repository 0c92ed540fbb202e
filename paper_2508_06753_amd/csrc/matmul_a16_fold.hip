// w2a16 for large M with the scale folded into the weights (Sec. II-D,
// "Alternative implementation": the 2-bit code and the 16-bit group scale are
// mixed into one 16-bit weight, which goes to a 16-bit matrix instruction with
// fp32 accumulation; nothing is dequantised afterwards).  With bf16 the four
// possible weights of a group and column, 0, +sw, -2 sw and -sw, are exact
// (sign flip, exponent + 1), so the matrix instruction sums exact products
// and ONE accumulator per output runs over the whole K: no zero-point term, no
// group sums of the activations, no per-group fma on the accumulators.
//
// Per lane and (group, column) the four weights sit in two registers, low
// bytes in one and high bytes in the other.  A dword of the packed tile holds
// 16 codes, four per byte; (w >> 2j) & 0x03030303 is four codes as four byte
// selectors, two v_perm_b32 look the low and the high bytes up, two more
// interleave them into [k even pair] and [k odd pair] registers: 23 vector
// instructions per 16 weights.  They are amortised over a 128-row wave tile
// (RI = 8 row tiles x CJ = 2 column blocks of v_mfma_f32_16x16x32_bf16: 32
// matrix instructions per 64-k stage and wave), which is what makes this
// construction the faster one for prefill: measured, it issues 2.3 vector
// instructions per matrix instruction where the zero-point kernel issues 5.9.
//
// Workgroup: 128 rows x (32 columns per wave) x 64 k per stage; activations go
// through LDS (three or five buffers, rows de-interleaved [even k | odd k] per
// 16-k block to match the order the codes come out of a dword, row stride
// 160 B: conflict-free operand reads); weights go from global memory to
// registers, one 16-byte load per lane, column block and 256-k tile, a whole
// tile ahead.  Each wave is software-pipelined on its own (next stage's weights
// are up-converted and its first operands read under this stage's matrix
// instructions).  Tried and slower: 256-row wave tiles at one wave per SIMD.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "w2_small_common.h"

namespace w2 {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

namespace fold16 {

constexpr int CJ = 2;                              // 16-column blocks per wave
constexpr int BK = 64;
constexpr int WN = 16 * CJ;
constexpr int A_STRIDE = BK * 2 + 32;              // 32 mod 64 bytes: conflict-free A-operand reads
// LDS buffers: 3 with a barrier after every stage; 5 with a barrier after every other stage (eight-wave
// workgroups, one per CU, where the LDS is there for it)
constexpr int nbuf_of(int bn) { return bn >= 256 ? 5 : 3; }
constexpr int E_STRIDE = WN * 2 + 16;              // epilogue: bytes per LDS row of a wave's result
constexpr int waves_of(int bn) { return bn / WN; }
constexpr int lds_bytes(int bn, int bm)
{
    return nbuf_of(bn) * bm * A_STRIDE > waves_of(bn) * bm * E_STRIDE ? nbuf_of(bn) * bm * A_STRIDE
                                                                      : waves_of(bn) * bm * E_STRIDE;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// The four weights of one (group, column): low bytes and high bytes, indexed by the raw code
// (00 -> 0, 01 -> +sw, 10 -> -2 sw, 11 -> -sw).
struct Lut { uint32_t lo4, hi4; };

__device__ __forceinline__ Lut make_lut(uint32_t s)          // s: bf16 bit pattern of the group scale
{
    const uint32_t neg = s ^ 0x8000u;
    // -2 sw: exponent + 1; a zero (or denormal) scale keeps its exponent field: -0 stays -0
    const uint32_t neg2 = (s & 0x7f80u) ? ((s + 0x0080u) ^ 0x8000u) : neg;
    const uint32_t a = s << 16;                              // [0, +sw]
    const uint32_t b = neg2 | (neg << 16);                   // [-2 sw, -sw]
    Lut l;
    l.lo4 = __builtin_amdgcn_perm(b, a, 0x06040200u);
    l.hi4 = __builtin_amdgcn_perm(b, a, 0x07050301u);
    return l;
}

// 16 codes of one dword -> b0 (even k of the lane's 16-k block), b1 (odd k)
__device__ __forceinline__ void upconvert(uint32_t w, const Lut& l, v4i& b0, v4i& b1)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t t = (w >> (2 * j)) & 0x03030303u;     // the codes of k = 4j .. 4j+3 as byte selectors
        const uint32_t lo = __builtin_amdgcn_perm(0u, l.lo4, t);
        const uint32_t hi = __builtin_amdgcn_perm(0u, l.hi4, t);
        b0[j] = (int)__builtin_amdgcn_perm(hi, lo, 0x06020400u);   // k = 4j, 4j+2
        b1[j] = (int)__builtin_amdgcn_perm(hi, lo, 0x07030501u);   // k = 4j+1, 4j+3
    }
}

__device__ __forceinline__ v4f mfma_bf16(const v4i& a, const v4i& b, const v4f& c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a),
                                                   __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

template <int G>
struct WTile {
    uint4 w[CJ];                                   // 16 bytes of codes per column block: dword t = k 64t .. 64t+63
    uint32_t s[CJ][G == 128 ? 1 : 2];              // the lane's column: 2 (G=128) or 4 (G=64) bf16 group scales
};

// RI: 16-row tiles per wave (the workgroup's rows: BM = 16 RI)
template <int G, int BN, int RI>
__global__ void __launch_bounds__(64 * waves_of(BN), (waves_of(BN) > 4 || RI > 8) ? 1 : 2)
a16_fold_tiled_kernel(A16Args a, int tiles_m, int tiles_n, int group_m, int splits)
{
    constexpr int BM = 16 * RI, A_BUF = BM * A_STRIDE;
    constexpr int WAVES = waves_of(BN), THREADS = 64 * WAVES;
    constexpr int GPT = TILE_K / G;
    constexpr int NBUF = nbuf_of(BN);
    constexpr int NP = BM * 8 / THREADS;           // 16-byte activation pieces per thread and stage: 2 or 4
    extern __shared__ __align__(16) int8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wn = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4, l16 = lane & 15;

    // workgroup -> tile: one contiguous chunk of ids per XCD, bands of group_m row tiles inside
    const int64_t total = (int64_t)tiles_m * tiles_n;
    int64_t id = blockIdx.x;
    if (total % 8 == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int64_t band = id / ((int64_t)group_m * tiles_n);
    const int64_t first_m = band * group_m;
    const int gm = (int)min((int64_t)group_m, tiles_m - first_m);
    const int64_t in_band = id - band * group_m * tiles_n;
    const int64_t tile_m = first_m + in_band % gm;
    const int64_t tile_n = in_band / gm;
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

    const char* wb[CJ];
    const char* sb[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
        int64_t c = tile_n * (BN / TILE_N) + wn * CJ + j;
        c = c < a.n_cb ? c : a.n_cb - 1;                     // clamp: loads stay in bounds
        wb[j] = reinterpret_cast<const char*>(a.codes + c * a.n_kt * 256);
        sb[j] = reinterpret_cast<const char*>(a.scales + c * a.n_kt * TILE_N * GPT);
    }
    uint32_t w_lane = (uint32_t)lane * 16u;
    uint32_t s_lane = (uint32_t)l16 * (GPT * 2u);

    // copy: eight threads per row, 16 B (eight k) each, NP rows per thread; rows past M repeat the
    // last row.  Lane offsets stay below 128 * 2 * ldx <= 2^32 (ldx <= 2^24).
    const int cp_seg = tid & 7;
    const char* cp_base = reinterpret_cast<const char*>(a.X + m0 * a.ldx);               // uniform
    uint32_t cp_lane[NP];
    int cp_dst[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int row = (tid >> 3) + p * (THREADS / 8);
        int64_t m = m0 + row;
        if (m >= a.M) m = a.M - 1;
        cp_lane[p] = (uint32_t)((m - m0) * a.ldx * 2) + (uint32_t)cp_seg * 16u;
        cp_dst[p] = row * A_STRIDE + (cp_seg >> 1) * 16 + (cp_seg & 1) * 8;
    }

    v4f acc[RI][CJ];
#pragma unroll
    for (int i = 0; i < RI; ++i)
#pragma unroll
        for (int j = 0; j < CJ; ++j) acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};

    // this workgroup's K range (split-K: blockIdx.y of `splits` near-equal ranges of whole tiles)
    const int64_t kt_b = a.n_kt * blockIdx.y / splits, kt_e = a.n_kt * (blockIdx.y + 1) / splits;
    const int64_t st_b = kt_b * 4, n_st = kt_e * 4;          // stages of 64 k: [st_b, n_st)
    // two register sets: a load has two stages to land before its data goes to LDS
    // (four-wave workgroups copy twice as much per thread and keep one set: the registers do not allow two)
    constexpr bool TWO_SETS = NP <= 2;
    uint4 ar0[NP], ar1[TWO_SETS ? NP : 1];
    auto load_a = [&](int64_t st, uint4 (&ar)[NP]) {
        st = min(st, n_st - 1);
        const char* p = cp_base + st * (BK * 2);             // uniform
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            asm volatile("" : "+v"(cp_lane[i]));             // keeps "scalar base + 32-bit offset" addressing
            ar[i] = *reinterpret_cast<const uint4*>(p + cp_lane[i]);
        }
    };
    // eight k of a row: the even ones to the [even] half of the 16-k block's image, the odd ones 64 B on
    auto store_a = [&](int buf, const uint4 (&ar)[NP]) {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const uint32_t d[4] = {ar[i].x, ar[i].y, ar[i].z, ar[i].w};
            uint2 ev, od;
            ev.x = __builtin_amdgcn_perm(d[1], d[0], 0x05040100u);
            ev.y = __builtin_amdgcn_perm(d[3], d[2], 0x05040100u);
            od.x = __builtin_amdgcn_perm(d[1], d[0], 0x07060302u);
            od.y = __builtin_amdgcn_perm(d[3], d[2], 0x07060302u);
            int8_t* dst = smem + buf * A_BUF + cp_dst[i];
            *reinterpret_cast<uint2*>(dst) = ev;
            *reinterpret_cast<uint2*>(dst + 64) = od;
        }
    };
    auto load_w = [&](int64_t kt, WTile<G>& r) {
        kt = min(kt, kt_e - 1);
        const int64_t w_off = kt * 1024;
        const int64_t s_off = kt * (TILE_N * GPT * 2);
        asm volatile("" : "+v"(w_lane), "+v"(s_lane));
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            r.w[j] = *reinterpret_cast<const uint4*>(wb[j] + w_off + w_lane);
            if constexpr (G == 128) {
                r.s[j][0] = *reinterpret_cast<const uint32_t*>(sb[j] + s_off + s_lane);
            } else {
                const uint2 v = *reinterpret_cast<const uint2*>(sb[j] + s_off + s_lane);
                r.s[j][0] = v.x;
                r.s[j][1] = v.y;
            }
        }
    };

    WTile<G> w0, w1;
    load_w(kt_b, w0);
    // stages 0 .. WR-1 go to LDS up front; the registers then hold stages WR and WR+1
    constexpr int WR = NBUF == 3 ? 2 : 3;          // stage it writes the activations of stage it+WR
#pragma unroll
    for (int p = 0; p < WR; ++p) {
        load_a(st_b + p, ar0);
        store_a(p, ar0);
    }
    load_a(st_b + WR, ar0);
    if constexpr (TWO_SETS) load_a(st_b + WR + 1, ar1);
    __syncthreads();

    const int8_t* a_base = smem + l16 * A_STRIDE + q * 16;
    Lut lut[CJ];
    struct BSet { v4i b0[CJ], b1[CJ]; };

    // the weights of stage t of tile w, column block j (a group's look-up table is rebuilt where it begins)
    auto prep_b = [&](auto tc, const WTile<G>& w, int j, BSet& out) {
        constexpr int t = decltype(tc)::value;
        if constexpr (G == 64 || (t & 1) == 0) {
            const uint32_t pair = w.s[j][G == 128 ? 0 : t >> 1];
            const int g_in_pair = G == 128 ? t >> 1 : t & 1;
            lut[j] = make_lut(g_in_pair ? pair >> 16 : pair & 0xffffu);
        }
        const uint32_t wd = t == 0 ? w.w[j].x : t == 1 ? w.w[j].y : t == 2 ? w.w[j].z : w.w[j].w;
        upconvert(wd, lut[j], out.b0[j], out.b1[j]);
    };

    // Software pipeline.  A wave enters stage `it` with the stage's weights up-converted (bc) and its
    // even-k activation operands (a0) in registers.  Under the stage's 32 matrix instructions it
    // reads the odd-k operands, up-converts the weights of stage it+1 (bn) and reads that stage's
    // even-k operands, so every wave keeps the matrix pipe and the vector pipe busy at the same
    // time whatever the other waves of the workgroup, which the barriers keep in step, are doing.
    // LDS, three buffers: stage it reads buffers it and it+1 and writes the activations of stage it+2
    // (loaded from global memory two stages earlier) into the third; the barrier at the end of a stage
    // orders both.  Five buffers: a barrier after every other stage only; the pair of stages (2S, 2S+1)
    // reads stages 2S .. 2S+2 and writes stages 2S+3 and 2S+4, five different buffers, so waves of a
    // workgroup may be a stage apart inside a pair.
    v4i a0[RI];
#pragma unroll
    for (int i = 0; i < RI; ++i) a0[i] = *reinterpret_cast<const v4i*>(a_base + i * 16 * A_STRIDE);
    BSet bA, bB;
    prep_b(std::integral_constant<int, 0>{}, w0, 0, bA);
    prep_b(std::integral_constant<int, 0>{}, w0, 1, bA);
    int buf = 0;

    auto stage = [&](int64_t it, auto tc, const WTile<G>& wc, WTile<G>& wnx, const BSet& bc, BSet& bn) {
        constexpr int t = decltype(tc)::value;
        constexpr std::integral_constant<int, (t + 1) & 3> tn{};
        const WTile<G>& wn_tile = t == 3 ? wnx : wc;         // where stage it+1 finds its weights
        const int buf1 = buf == NBUF - 1 ? 0 : buf + 1;
        const int bufw = buf + WR >= NBUF ? buf + WR - NBUF : buf + WR;
        if constexpr (TWO_SETS) store_a(bufw, (t & 1) ? ar1 : ar0);      // activations of stage it+WR
        else store_a(bufw, ar0);
        if constexpr (t == 0) load_w((it >> 2) + 1, wnx);
        if constexpr (TWO_SETS) load_a(it + WR + 2, (t & 1) ? ar1 : ar0);
        else load_a(it + WR + 1, ar0);
        __builtin_amdgcn_sched_barrier(0);                   // all loads are issued up here, unconditionally
        const int8_t* ab = a_base + buf * A_BUF;
        const int8_t* abn = a_base + buf1 * A_BUF;
        v4i a1[RI];
#pragma unroll
        for (int i = 0; i < RI; ++i) a1[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE + 64);
        prep_b(tn, wn_tile, 0, bn);
#pragma unroll
        for (int j = 0; j < CJ; ++j)
#pragma unroll
            for (int i = 0; i < RI; ++i) acc[i][j] = mfma_bf16(a0[i], bc.b0[j], acc[i][j]);
        prep_b(tn, wn_tile, 1, bn);
#pragma unroll
        for (int i = 0; i < RI; ++i) a0[i] = *reinterpret_cast<const v4i*>(abn + i * 16 * A_STRIDE);
#pragma unroll
        for (int j = 0; j < CJ; ++j)
#pragma unroll
            for (int i = 0; i < RI; ++i) acc[i][j] = mfma_bf16(a1[i], bc.b1[j], acc[i][j]);
        // issue order: one matrix instruction, then the LDS read and the two vector instructions it hides
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int k = 0; k < RI; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
            }
#pragma unroll
            for (int k = RI; k < RI * CJ; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
            }
        }
        buf = buf1;
        if constexpr (NBUF == 3 || (t & 1)) __syncthreads();
    };
    auto tile = [&](int64_t kt, const WTile<G>& wc, WTile<G>& wnx) {
        stage(kt * 4, std::integral_constant<int, 0>{}, wc, wnx, bA, bB);
        stage(kt * 4 + 1, std::integral_constant<int, 1>{}, wc, wnx, bB, bA);
        stage(kt * 4 + 2, std::integral_constant<int, 2>{}, wc, wnx, bA, bB);
        stage(kt * 4 + 3, std::integral_constant<int, 3>{}, wc, wnx, bB, bA);
    };
    for (int64_t kt = kt_b; kt < kt_e; kt += 2) {
        tile(kt, w0, w1);
        if (kt + 1 < kt_e) tile(kt + 1, w1, w0);             // uniform
    }

    if (a.part) {
        // split-K: this range's fp32 partial results go to the workspace.  A lane holds single columns of
        // four rows per tile (4-byte stores in 64-byte runs: measured on the w2a8 kernel, 5 us of a 29 us
        // launch); the wave's tile goes through LDS, 64 rows at a time (a region of its own: the barrier at
        // the end of the last stage freed the activation buffers; rows padded by 16 bytes, conflict-free both
        // ways), and leaves as 16-byte stores in 128-byte runs.
        constexpr int P_STRIDE = WN * 4 + 16;
        static_assert(WAVES * 64 * P_STRIDE <= lds_bytes(BN, BM), "partial-result staging fits the activation buffers");
        float* dst = a.part + (int64_t)blockIdx.y * a.M * a.N;
        int8_t* pbase = smem + wn * (64 * P_STRIDE);
        const int prow = lane >> 3, pcol = (lane & 7) * 4;   // eight lanes per row piece
        const int64_t n = n0 + wn * WN + pcol;
#pragma unroll
        for (int h = 0; h < RI / 4; ++h) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int j = 0; j < CJ; ++j)
                        *reinterpret_cast<float*>(pbase + (i * 16 + 4 * q + r) * P_STRIDE + (j * 16 + l16) * 4) = acc[h * 4 + i][j][r];
            // the wave reads back only what it wrote itself: LDS operations of one wave complete in order
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int row = p * 8 + prow;
                const int64_t m = m0 + h * 64 + row;
                const float4 v = *reinterpret_cast<const float4*>(pbase + row * P_STRIDE + pcol * 4);
                if (m < a.M && n < a.N) *reinterpret_cast<float4*>(dst + m * a.N + n) = v;   // N % 8 == 0: all 4 or none
            }
        }
        return;
    }

    // The wave's 128 x 32 result goes through LDS (its own region; the barrier at the end of the last
    // stage freed the activation buffers) and leaves as 16-byte stores, four lanes per 64-byte row piece.
    int8_t* ebase = smem + wn * (BM * E_STRIDE);
    uint16_t* eb = reinterpret_cast<uint16_t*>(ebase);
    // Fused epilogue (Sec. II-D: bias and activation applied while the outputs are in registers).  The
    // gated form combines the wave's two column blocks, an even (gate) and an odd (up) one, into one.
    const bool gated = a.epi.act == ACT_SILU_MUL;
    float bias[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
        const int64_t n = n0 + wn * WN + j * 16 + l16;
        bias[j] = (a.epi.bias && n < a.N) ? bf16_to_f32(a.epi.bias[n]) : 0.f;
    }
    // (one copy of the loop per epilogue, picked here: a choice per element would have the compiler
    // evaluate the SiLU for every output and select afterwards)
    auto emit = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;        // ACT_NONE, ACT_SILU, ACT_SILU_MUL
        static_assert(CJ == 2, "the epilogue pairs the wave's two column blocks");
#pragma unroll
        for (int i = 0; i < RI; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = i * 16 + 4 * q + r;
                const float z0 = acc[i][0][r] + bias[0], z1 = acc[i][1][r] + bias[1];
                if constexpr (MODE == ACT_SILU_MUL) {
                    eb[row * (E_STRIDE / 2) + l16] = f32_to_bf16_rne(silu_f32(z0) * z1);
                } else {
                    const uint32_t pk = MODE == ACT_SILU ? pack_bf16x2(silu_f32(z0), silu_f32(z1)) : pack_bf16x2(z0, z1);
                    eb[row * (E_STRIDE / 2) + l16] = (uint16_t)pk;
                    eb[row * (E_STRIDE / 2) + 16 + l16] = (uint16_t)(pk >> 16);
                }
            }
    };
    if (gated) emit(std::integral_constant<int, ACT_SILU_MUL>{});
    else if (a.epi.act == ACT_SILU) emit(std::integral_constant<int, ACT_SILU>{});
    else emit(std::integral_constant<int, ACT_NONE>{});
    // the wave reads back only what it wrote itself: LDS operations of one wave complete in order
    const int wcols = gated ? WN / 2 : WN;                   // output columns of this wave
    const int lpr = wcols * 2 / 16;                          // lanes per row piece (16 bytes each): 4 or 2
    const int rpp = 64 / lpr;                                // rows per pass
    const int64_t ncol = (gated ? (n0 + wn * WN) / 2 : n0 + wn * WN) + (lane % lpr) * 8;   // first of this lane's 8 columns
    const int64_t n_out = gated ? a.N / 2 : a.N;
    for (int p = 0; p < BM / rpp; ++p) {
        const int row = p * rpp + lane / lpr;
        const int64_t m = m0 + row;
        const uint4 v = *reinterpret_cast<const uint4*>(ebase + row * E_STRIDE + (lane % lpr) * 16);
        if (m < a.M && ncol < n_out) *reinterpret_cast<uint4*>(a.Y + m * a.ldy + ncol) = v;   // N % 8 == 0: all 8 or none
    }
}

}  // namespace fold16

template <int G, int BN, int RI>
static int launch_fold_bn(const A16Args& a_in, int splits, hipStream_t stream)
{
    using namespace fold16;
    constexpr int BM = 16 * RI;
    A16Args a = a_in;
    if (splits < 2) a.part = nullptr;
    const int tiles_m = (int)((a.M + BM - 1) / BM);
    const int tiles_n = (int)((a.N + BN - 1) / BN);
    const int group_m = a.tune.tiled_group_m ? a.tune.tiled_group_m : 8;
    const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n), (unsigned)(splits < 2 ? 1 : splits)), block(64 * waves_of(BN));
    constexpr int lds = lds_bytes(BN, BM);
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(a16_fold_tiled_kernel<G, BN, RI>), lds,
                                    "w2_matmul_a16[scaled16 tiled]"))
        return rc;
    hipLaunchKernelGGL((a16_fold_tiled_kernel<G, BN, RI>), grid, block, lds, stream, a, tiles_m, tiles_n, group_m,
                       (int)grid.y);
    int rc = check_launch("w2_matmul_a16[scaled16 tiled]");
    if (rc || !a.part) return rc;
    return launch_splitk_reduce(a.part, splits, a.M, a.N, a.Y, a.ldy, a.epi, stream);
}

// Columns per workgroup and K ranges across workgroups.  With room for partial results: 256-column workgroups
// (eight waves, one per CU) and as many K ranges (up to 8, at least two 256-k tiles each, at most 64 MiB of
// partial results) as bring the grid up to one workgroup per CU -- floor(256 / tiles), never more than one
// round.  From sweeps over 4096 x 4096, 4096 x 6144, 5120 x 7168, 8192 x 8192, 14336 x 4096, 4096 x 28672 and
// 28672 x 8192 at M = 65..512 that rule is within 5 % of the best (columns, ranges) everywhere and up to 17 %
// ahead of the older one (128 columns when 256 leave half the chip idle, about 1.5 workgroups per CU): 4096 x
// 6144 at M = 256 32.1 -> 26.8 us, 8192 x 8192 at M = 512 76.7 -> 67.7, 14336 x 4096 at M = 512 70.2 -> 62.1,
// 4096 x 28672 at M = 65 40.6 -> 34.7.  Without room: 128 columns when 256 would leave half the chip idle.
struct FoldPlan { int bn, splits; };

static FoldPlan fold_plan(int64_t M, int64_t N, int64_t n_kt, int64_t cap, const w2_tuning_t& tune)
{
    FoldPlan p;
    const int64_t tiles_m = (M + 127) / 128;
    const int64_t t256 = tiles_m * ((N + 255) / 256);
    const int forced = tune.splitk;                          // tuning and tests: 1 = never, n = n parts if they fit
    p.bn = tune.tiled_bn == 128 || tune.tiled_bn == 256 ? tune.tiled_bn : 0;
    if (forced > 0) {
        p.splits = (int)max((int64_t)1, min((int64_t)forced, min(cap, n_kt)));
        if (!p.bn) p.bn = t256 <= 128 && p.splits < 2 ? 128 : 256;
        return p;
    }
    int64_t s = 256 / max(t256, (int64_t)1);
    s = min(s, (int64_t)8);
    s = min(s, n_kt / 2);
    s = min(s, ((int64_t)64 << 20) / (M * N * (int64_t)sizeof(float)));
    s = min(s, cap);
    if (p.bn == 128) {                                       // forced narrow workgroups: two fit a CU
        const int64_t t128 = tiles_m * ((N + 127) / 128);
        s = min(s, max((int64_t)1, 512 / max(t128, (int64_t)1)));
    }
    if (s < 2) {
        p.splits = 1;
        if (!p.bn) p.bn = t256 <= 128 ? 128 : 256;
        return p;
    }
    p.splits = (int)s;
    if (!p.bn) p.bn = 256;
    return p;
}

size_t a16_fold_splitk_bytes(int64_t M, int64_t N, int64_t n_kt, const w2_tuning_t& tune)
{
    const int s = fold_plan(M, N, n_kt, 16, tune).splits;
    return s < 2 ? 0 : (size_t)s * M * N * sizeof(float);
}

int launch_a16_fold_tiled(const A16Args& a, hipStream_t stream)
{
    const int64_t cap = a.part ? (int64_t)(a.part_bytes / ((size_t)a.M * a.N * sizeof(float))) : 0;
    const FoldPlan p = fold_plan(a.M, a.N, a.n_kt, cap, a.tune);
    if (p.bn == 256)
        return a.G == 128 ? launch_fold_bn<128, 256, 8>(a, p.splits, stream) : launch_fold_bn<64, 256, 8>(a, p.splits, stream);
    return a.G == 128 ? launch_fold_bn<128, 128, 8>(a, p.splits, stream) : launch_fold_bn<64, 128, 8>(a, p.splits, stream);
}

}  // namespace w2
