// w2a16: bf16 activations left unquantised (Sec. II-D, "Alternative
// implementation": the 2-bit weights are turned into 16-bit values in
// registers and fed to a 16-bit matrix instruction with fp32 accumulation; no
// activation quantisation, no output dequantisation of an integer result).
//
// Up-convert for CDNA4.  The packed dword holds 2-bit two's-complement values q.
// One XOR with 0xAAAAAAAA turns all 16 fields into s = q + 2 (0..3).  OR-ing a
// field into the low mantissa bits of the bf16 constant 128.0 (0x4300) gives
// exactly the bf16 number 128 + s = 130 + q, so
//     pair_j = ((w ^ 0xAAAAAAAA) >> 2j) & 0x00030003 | 0x43004300,   j = 0..7
// is a dword of two ready bf16 weights: one shift and one and-or per two
// weights.  The matrix instruction therefore computes S = sum x * (130 + q) per
// group; the constant is removed with the group sums X_g = sum_{k in g} x[m,k]
// that the activation staging pass produces once per workgroup:
//     y += sw[g,n] * (S - 130 * X_g[m]).
// |130 X_g| exceeds the wanted sum by ~2^7, which fp32 (24 bits) absorbs with
// room to spare for a bf16 (8 bit) result.  The paper's own construction (sign
// bit XOR-ed into the fp16 scale, predicated zero) needs the scale per weight
// and handles ternary only; this one serves both codecs with the same blob.
//
// Pairs 0..3 take their two weights from bytes 0 and 2 of the dword and pairs
// 4..7 from bytes 1 and 3, i.e. the first MFMA operand of a lane holds the even
// k of its 16-k block and the second the odd k.  The staging pass stores the
// activations de-interleaved the same way ([8 even k | 8 odd k] per 16-k
// block), so both MFMA operands are single ds_read_b128.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "w2_small_common.h"

namespace w2 {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr float ZP = 130.0f;     // 128 (the bf16 constant) + 2 (s = q + 2)

// mask (0x00030003) and base (0x43004300) arrive in vector registers: (x & mask) | base is then
// ONE instruction (v_and_or_b32 can take neither two literals nor two scalar registers), so a pair
// of weights costs a shift and an and-or.
struct Bf16Consts { uint32_t mask, base; };

__device__ __forceinline__ Bf16Consts bf16_consts()
{
    Bf16Consts c = {0x00030003u, 0x43004300u};
    asm volatile("" : "+v"(c.mask), "+v"(c.base));           // opaque: stays in VGPRs
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

// The other construction of Sec. II-D ("Alternative implementation", the listing that mixes the
// 2-bit code with the 16-bit group scale): the weight handed to the matrix instruction IS
// sw * q, so nothing is dequantised afterwards and one accumulator runs over the whole K.  Here
// the mixing is a byte permute: per group and column a lane keeps the four possible weights as a
// table of four bf16 values (code 00 -> 0, 01 -> +sw, 10 -> -2 sw: sign flipped and exponent + 1,
// 11 -> -sw: sign flipped), eight bytes in two registers, and v_perm_b32 picks the two bytes of
// each weight: for a pair of codes f = c_a | c_b << 16 the selector is f * 0x0202 + 0x01000100
// (bytes 2c, 2c+1 per weight).  Four instructions per two weights instead of two, no zero-point
// term, no group sums, both codecs.
struct FoldLut { uint32_t lo, hi; };

__device__ __forceinline__ FoldLut fold_lut(uint32_t s)      // s: bf16 bit pattern of the group scale
{
    FoldLut l;
    const uint32_t neg = s ^ 0x8000u;
    // -2 sw: exponent + 1; a zero (or denormal) scale keeps its exponent field: -0 stays -0
    const uint32_t neg2 = (s & 0x7f80u) ? ((s + 0x0080u) ^ 0x8000u) : neg;
    l.lo = s << 16;                                          // [0, +sw]
    l.hi = neg2 | (neg << 16);                               // [-2 sw, -sw]
    return l;
}

__device__ __forceinline__ void upconvert_fold(uint32_t w, const FoldLut& l, v4i& b0, v4i& b1)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t f0 = (w >> (2 * j)) & 0x00030003u;        // bytes 0 and 2: even k
        const uint32_t f1 = (w >> (8 + 2 * j)) & 0x00030003u;    // bytes 1 and 3: odd k
        b0[j] = (int)__builtin_amdgcn_perm(l.hi, l.lo, f0 * 0x0202u + 0x01000100u);
        b1[j] = (int)__builtin_amdgcn_perm(l.hi, l.lo, f1 * 0x0202u + 0x01000100u);
    }
}

__device__ __forceinline__ v4f mfma_bf16(const v4i& a, const v4i& b, const v4f& c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a),
                                                   __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

// ---- activation staging: 16 bf16 (32 B) per piece -----------------------
struct Piece { uint4 lo, hi; };

__device__ __forceinline__ Piece piece_load(const uint16_t* __restrict__ X, int64_t ldx, int64_t k0,
                                            int ppr, int total, int i)
{
    i = i < total ? i : (int)((unsigned)i % (unsigned)total);   // surplus threads re-read pieces spread over the rows
    const int r = i / ppr, v = i - r * ppr;
    const uint4* p = reinterpret_cast<const uint4*>(X + (int64_t)r * ldx + k0 + v * 16);
    Piece pc;
    pc.lo = p[0];
    pc.hi = p[1];
    return pc;
}

__device__ __forceinline__ float pair_sum(uint32_t d)
{
    return __uint_as_float(d << 16) + __uint_as_float(d & 0xffff0000u);
}

// Writes one piece de-interleaved ([8 even k | 8 odd k]) and accumulates the
// group sums: G/16 consecutive pieces (consecutive lanes) form one group.
template <int G>
__device__ __forceinline__ void piece_store(const Piece& pc, int ppr, int total, int i, int row_stride,
                                            int8_t* xs, float* xsum)
{
    constexpr int PPG = G / 16;                  // pieces per group: 4 or 8
    const uint32_t d[8] = {pc.lo.x, pc.lo.y, pc.lo.z, pc.lo.w, pc.hi.x, pc.hi.y, pc.hi.z, pc.hi.w};
    float s = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += pair_sum(d[e]);
#pragma unroll
    for (int off = 1; off < PPG; off <<= 1) s += __shfl_xor(s, off);
    if (i < total) {
        const int r = i / ppr, v = i - r * ppr;
        uint4 ev, od;
        ev.x = __builtin_amdgcn_perm(d[1], d[0], 0x05040100u);
        ev.y = __builtin_amdgcn_perm(d[3], d[2], 0x05040100u);
        ev.z = __builtin_amdgcn_perm(d[5], d[4], 0x05040100u);
        ev.w = __builtin_amdgcn_perm(d[7], d[6], 0x05040100u);
        od.x = __builtin_amdgcn_perm(d[1], d[0], 0x07060302u);
        od.y = __builtin_amdgcn_perm(d[3], d[2], 0x07060302u);
        od.z = __builtin_amdgcn_perm(d[5], d[4], 0x07060302u);
        od.w = __builtin_amdgcn_perm(d[7], d[6], 0x07060302u);
        uint4* dst = reinterpret_cast<uint4*>(xs + r * row_stride + v * 32);
        dst[0] = ev;
        dst[1] = od;
        if ((v & (PPG - 1)) == 0) xsum[(v / PPG) * 16 + r] = s;
    }
}

constexpr int SVP = 2;    // pieces per thread that go through registers

// ---------------------------------------------------------------- SMALLM (bf16 MFMA)
template <int G, int TMAX, bool FOLD>
__global__ void __launch_bounds__(1024)
a16_smallm_kernel(A16Args a, SmallCfg cfg)
{
    W2_SMALL_PROLOGUE();
    const bool DBG = false;
    (void)DBG; (void)cb_ok;
    const int rows = (int)a.M;                              // 1..16
    const int arow = (lane & 15) < rows ? (lane & 15) : rows - 1;
    const Bf16Consts kc = bf16_consts();
    (void)kc;

    float y[4] = {0.f, 0.f, 0.f, 0.f};
    v4f acc = {0.f, 0.f, 0.f, 0.f};

    for (int c = 0; c < n_chunks; ++c) {
        const int64_t kt_begin = (int64_t)c * tiles_per_chunk;
        const int64_t kt_end = min(kt_begin + tiles_per_chunk, a.n_kt);
        int64_t kt0 = kt_begin + ((ks - kt_begin % cfg.ks) + cfg.ks) % cfg.ks;
        const int len = (int)(kt_end - kt_begin) * TILE_K;            // k in this chunk
        const int row_stride = len * 2 + XS_PAD;                      // bytes
        float* xsum = reinterpret_cast<float*>(smem + (size_t)rows * row_stride);   // [len/G][16]
        const int ppr = len >> 4, total = rows * ppr;

        auto load_batch = [&](int64_t kb, TileRegs (&tr)[TMAX]) {
#pragma unroll
            for (int i = 0; i < TMAX; ++i) {
                const int64_t kt = kb + (int64_t)i * cfg.ks;
                tr[i] = load_tile<G>(a.codes, a.scales, cbc * a.n_kt + (kt < kt_end ? kt : kt_end - 1), lane);
            }
        };
        auto compute_batch = [&](int64_t kb, const TileRegs (&tr)[TMAX]) {
#pragma unroll
            for (int i = 0; i < TMAX; ++i) {
                const int64_t kt = kb + (int64_t)i * cfg.ks;
                if (kt >= kt_end) break;
                const TileRegs cur = tr[i];
                const int8_t* xrow = smem + arow * row_stride + (int)(kt - kt_begin) * (TILE_K * 2) + q * 32;
                const uint32_t wd[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    v4i b0, b1;
                    if constexpr (FOLD) {
                        // the scale is folded into the weights: y is not used, acc runs over all of K
                        const int gi = G == 64 ? t : t >> 1;
                        const uint32_t pair = (G == 128 || gi < 2) ? cur.s0 : cur.s1;
                        const FoldLut lut = fold_lut((gi & 1) ? pair >> 16 : pair & 0xffffu);
                        upconvert_fold(wd[t], lut, b0, b1);
                    } else {
                        upconvert_bf16(wd[t], kc, b0, b1);
                    }
                    const v4i a0 = *reinterpret_cast<const v4i*>(xrow + t * 128);
                    const v4i a1 = *reinterpret_cast<const v4i*>(xrow + t * 128 + 16);
                    acc = mfma_bf16(a0, b0, acc);
                    acc = mfma_bf16(a1, b1, acc);
                    if (!FOLD && (G == 64 || (t & 1))) {
                        const int gi = G == 64 ? t : t >> 1;
                        const float sw = tile_scale<G>(cur, gi);
                        const int gl = (int)(kt - kt_begin) * GPT + gi;      // group inside the chunk
                        const v4f xg = *reinterpret_cast<const v4f*>(xsum + gl * 16 + 4 * q);
#pragma unroll
                        for (int r = 0; r < 4; ++r) y[r] = fmaf(sw, fmaf(-ZP, xg[r], acc[r]), y[r]);
                        acc = (v4f){0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        };
        {
            Piece p0 = piece_load(a.X, a.ldx, kt_begin * TILE_K, ppr, total, threadIdx.x);
            Piece p1 = piece_load(a.X, a.ldx, kt_begin * TILE_K, ppr, total, threadIdx.x + blockDim.x);
            TileRegs tr[TMAX];
            load_batch(kt0, tr);
            if (c > 0) __syncthreads();
            piece_store<G>(p0, ppr, total, threadIdx.x, row_stride, smem, xsum);
            piece_store<G>(p1, ppr, total, threadIdx.x + blockDim.x, row_stride, smem, xsum);
            for (int i = threadIdx.x + SVP * blockDim.x; i - (int)threadIdx.x < total; i += blockDim.x) {
                // whole waves stay in the loop together (the group sums use cross-lane shuffles)
                const Piece p = piece_load(a.X, a.ldx, kt_begin * TILE_K, ppr, total, i);
                piece_store<G>(p, ppr, total, i, row_stride, smem, xsum);
            }
            __syncthreads();
            compute_batch(kt0, tr);
        }
        for (kt0 += (int64_t)TMAX * cfg.ks; kt0 < kt_end; kt0 += (int64_t)TMAX * cfg.ks) {
            TileRegs tr[TMAX];
            load_batch(kt0, tr);
            compute_batch(kt0, tr);
        }
    }

    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);            // [waves][16 m][16 n]
#pragma unroll
    for (int r = 0; r < 4; ++r) red[(wave * 16 + 4 * q + r) * 16 + (lane & 15)] = FOLD ? acc[r] : y[r];
    __syncthreads();
    store_outputs(a.epi, a.Y, a.ldy, a.N, (int64_t)blockIdx.x * cfg.cbw, cfg.cbw, rows,
                  [&](int ci, int m, int nl, int) {
                      float s = 0.0f;
                      for (int k = 0; k < cfg.ks; ++k) s += red[((k * cfg.cbw + ci) * 16 + m) * 16 + nl];
                      return s;
                  });
}

bool a16_smallm_supports(const A16Args& a) { return a.M >= 1 && a.M <= 16; }

template <int G, bool FOLD>
static int launch_a16_smallm_t(const A16Args& a, hipStream_t stream)
{
    const int rows = (int)a.M;
    const SmallCfg c = pick_cfg(a.tune, a.n_cb, a.n_kt, rows, 2, 16, a.epi.act == ACT_SILU_MUL);
    const size_t extra = (size_t)(c.kc / G) * 16 * sizeof(float);
    const size_t lds = small_lds_bytes(c, rows, 16, 2, extra);
    const int tpw = tiles_per_wave(a.n_kt, c);
    if (tpw <= 2) return launch_small(a16_smallm_kernel<G, 2, FOLD>, "w2_matmul_a16[smallm]", a, c, lds, stream);
    if (tpw <= 4) return launch_small(a16_smallm_kernel<G, 4, FOLD>, "w2_matmul_a16[smallm]", a, c, lds, stream);
    return launch_small(a16_smallm_kernel<G, TMAX, FOLD>, "w2_matmul_a16[smallm]", a, c, lds, stream);
}

int launch_a16_smallm(const A16Args& a, hipStream_t stream)
{
    if (a.fold) return a.G == 128 ? launch_a16_smallm_t<128, true>(a, stream) : launch_a16_smallm_t<64, true>(a, stream);
    return a.G == 128 ? launch_a16_smallm_t<128, false>(a, stream) : launch_a16_smallm_t<64, false>(a, stream);
}

// ---------------------------------------------------------------- TILED (bf16 MFMA, any M)
// 64(M) x 256(N) per workgroup, eight waves of 64 x 32: 4 x 2 tiles of
// v_mfma_f32_16x16x32_bf16 each (32 accumulators + 32 running sums per lane,
// which leaves the registers for deep prefetch).  A stage is 64 k: one packed dword per column block
// and lane (two matrix instructions per tile: even k, odd k), and 64 rows x
// 128 B of activations in LDS, stored de-interleaved by the copy threads, which
// also leave the per-row sums of the stage in a ring of four slots.
//
// The zero-point term costs no instruction per accumulator: a group's
// accumulators START from -130 * X_g[m] (the third MFMA operand, one value per
// row, shared by the wave's four column tiles), so that at the group's end
// acc = sum x*q and the dequant is one fma, y += sw * acc.  For that the row
// sums of a stage must be in LDS before the group begins: activations are
// written to LDS two stages ahead (four buffers) and loaded from global memory
// four stages ahead (two register sets); weights are
// loaded three stages ahead (four register sets; the loop is unrolled by four,
// sets and buffers are indexed by the stage number mod 4).  All loads are issued
// unconditionally (clamped past the end) and pinned at the top of the stage, so
// the compiler's wait counts never wait for a load just issued.
namespace tiled16 {

constexpr int BM = 64, BN = 256, BK = 64;
constexpr int CJ = 2;                             // column blocks per wave
constexpr int THREADS = 512;
constexpr int CPT = THREADS / BM;                  // copy threads per row: 8, eight k (16 B) each
constexpr int A_STRIDE = BK * 2 + 16;             // bytes per LDS row
constexpr int A_BUF = BM * A_STRIDE;
constexpr int NBUF = 4;
constexpr int XS_OFF = NBUF * A_BUF;              // float xpart[4][BM]
constexpr int LDS_BYTES = XS_OFF + 4 * BM * 4;
constexpr int WN = 16 * CJ;

struct WSet { uint32_t w[CJ], sc[CJ]; };
struct ASet { uint4 v; };

template <int G>
__global__ void __launch_bounds__(THREADS)
a16_tiled_kernel(A16Args a, int tiles_m, int tiles_n, int group_m)
{
    extern __shared__ __align__(16) int8_t smem[];
    float* xpart = reinterpret_cast<float*>(smem + XS_OFF);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wn = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4, l16 = lane & 15;
    constexpr int GPT = TILE_K / G;

    const int64_t total = (int64_t)tiles_m * tiles_n;
    int64_t id = blockIdx.x;
    if (total % 8 == 0) id = (id & 7) * (total >> 3) + (id >> 3);       // one contiguous chunk per XCD
    const int64_t band = id / ((int64_t)group_m * tiles_n);
    const int64_t first_m = band * group_m;
    const int gm = (int)min((int64_t)group_m, tiles_m - first_m);
    const int64_t in_band = id - band * group_m * tiles_n;
    const int64_t tile_m = first_m + in_band % gm;
    const int64_t tile_n = in_band / gm;
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

    // wave-uniform base pointers of the four column blocks + 32-bit lane offsets
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

    // copy: 8 threads per row, eight k (16 B) each: the even k of a half block go to one 8-byte
    // slot of the block's [8 even | 8 odd] LDS image, the odd k to another; rows past M repeat the
    // last row
    const int cp_row = tid / CPT, cp_seg = tid % CPT;
    int64_t cp_m = m0 + cp_row;
    if (cp_m >= a.M) cp_m = a.M - 1;
    const char* cp_base = reinterpret_cast<const char*>(a.X + m0 * a.ldx);               // uniform
    uint32_t cp_lane = (uint32_t)((cp_m - m0) * a.ldx * 2) + (uint32_t)cp_seg * 16u;     // < 128 ldx: fits 32 bits
    const int cp_dst = cp_row * A_STRIDE + (cp_seg >> 1) * 32 + (cp_seg & 1) * 8;

    v4f acc[4][CJ];
    float y[4][CJ][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < 4; ++r) y[i][j][r] = 0.0f;
        }

    const int64_t n_st = a.n_kt * 4;                         // stages of 64 k; a multiple of 4
    auto load_a = [&](int64_t st, ASet& r) {
        st = min(st, n_st - 1);
        const char* p = cp_base + st * (BK * 2);             // uniform
        asm volatile("" : "+v"(cp_lane));                    // keeps "scalar base + 32-bit offset" addressing
        r.v = *reinterpret_cast<const uint4*>(p + cp_lane);
    };
    auto load_w = [&](int64_t st, WSet& r) {
        st = min(st, n_st - 1);
        const int64_t kt = st >> 2;
        const int t = (int)(st & 3);
        const int64_t w_off = kt * 1024 + t * 4;
        const int64_t s_off = kt * (TILE_N * GPT * 2) + (G == 128 ? (t >> 1) : t) * 2;
        asm volatile("" : "+v"(w_lane), "+v"(s_lane));
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            r.w[j] = *reinterpret_cast<const uint32_t*>(wb[j] + w_off + w_lane);
            r.sc[j] = *reinterpret_cast<const uint16_t*>(sb[j] + s_off + s_lane);
        }
    };
    // stores eight k de-interleaved into buffer `buf` and the row's partial sum into ring slot `buf`
    auto stage_store = [&](const ASet& r, int buf) {
        const uint32_t d[4] = {r.v.x, r.v.y, r.v.z, r.v.w};
        float s = (pair_sum(d[0]) + pair_sum(d[1])) + (pair_sum(d[2]) + pair_sum(d[3]));
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        s += __shfl_xor(s, 4);
        uint2 ev, od;
        ev.x = __builtin_amdgcn_perm(d[1], d[0], 0x05040100u);
        ev.y = __builtin_amdgcn_perm(d[3], d[2], 0x05040100u);
        od.x = __builtin_amdgcn_perm(d[1], d[0], 0x07060302u);
        od.y = __builtin_amdgcn_perm(d[3], d[2], 0x07060302u);
        int8_t* dst = smem + buf * A_BUF + cp_dst;
        *reinterpret_cast<uint2*>(dst) = ev;
        *reinterpret_cast<uint2*>(dst + 16) = od;
        if (cp_seg == 0) xpart[buf * BM + cp_row] = s;
    };

    ASet as0, as1;
    WSet ws0, ws1, ws2, ws3;
    load_a(0, as0);
    load_a(1, as1);
    load_w(0, ws0);
    load_w(1, ws1);
    load_w(2, ws2);
    stage_store(as0, 0);
    stage_store(as1, 1);
    load_a(2, as0);
    load_a(3, as1);
    __syncthreads();

    const int8_t* a_base = smem + l16 * A_STRIDE + q * 32;
    const Bf16Consts kc = bf16_consts();
    v4f cinit[4];                                            // -130 * X_g for the rows of each row tile

    // One stage.  T = stage index mod 4 (LDS buffer, ring slot, weight set); `as` holds the
    // activations of stage st+2 and then receives those of st+4; wfar receives the weights of st+3.
    auto stage = [&](int64_t st, auto Tc, ASet& as, const WSet& wc, WSet& wfar) {
        constexpr int T = decltype(Tc)::value;
        stage_store(as, (T + 2) & 3);                        // activations of stage st+2
        load_a(st + 4, as);
        load_w(st + 3, wfar);
        __builtin_amdgcn_sched_barrier(0);                   // the loads stay up here
        const int8_t* ab = a_base + T * A_BUF;
        v4i a0[4], a1[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a0[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE);
            a1[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE + 16);
        }
        constexpr bool group_begin = (G == 64) || !(T & 1);
        constexpr bool group_end = (G == 64) || (T & 1);
        if constexpr (group_begin) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v4f xg = *reinterpret_cast<const v4f*>(xpart + T * BM + i * 16 + 4 * q);
                if constexpr (G == 128) xg += *reinterpret_cast<const v4f*>(xpart + ((T + 1) & 3) * BM + i * 16 + 4 * q);
                cinit[i] = xg * -ZP;
            }
        }
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            v4i b0, b1;
            upconvert_bf16(wc.w[j], kc, b0, b1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[i][j] = mfma_bf16(a0[i], b0, group_begin ? cinit[i] : acc[i][j]);
                acc[i][j] = mfma_bf16(a1[i], b1, acc[i][j]);
            }
            if constexpr (group_end) {
                if (j > 0) {                                 // the previous column's results, under these MFMAs
                    const float sw = __uint_as_float(wc.sc[j - 1] << 16);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int r = 0; r < 4; ++r) y[i][j - 1][r] = fmaf(sw, acc[i][j - 1][r], y[i][j - 1][r]);
                }
            }
        }
        if constexpr (group_end) {
            const float sw = __uint_as_float(wc.sc[CJ - 1] << 16);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) y[i][CJ - 1][r] = fmaf(sw, acc[i][CJ - 1][r], y[i][CJ - 1][r]);
        }
        __syncthreads();
    };

    for (int64_t st = 0; st < n_st; st += 4) {
        stage(st, std::integral_constant<int, 0>{}, as0, ws0, ws3);
        stage(st + 1, std::integral_constant<int, 1>{}, as1, ws1, ws0);
        stage(st + 2, std::integral_constant<int, 2>{}, as0, ws2, ws1);
        stage(st + 3, std::integral_constant<int, 3>{}, as1, ws3, ws2);
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t m = m0 + i * 16 + 4 * q + r;
            if (m >= a.M) continue;
            // fused epilogue: bias, SiLU, or silu(even block) * (odd block) for the wave's pair of column blocks
            float z[CJ];
#pragma unroll
            for (int j = 0; j < CJ; ++j) {
                const int64_t n = n0 + wn * WN + j * 16 + l16;
                z[j] = y[i][j][r] + ((a.epi.bias && n < a.N) ? bf16_to_f32(a.epi.bias[n]) : 0.f);
            }
            if (a.epi.act == ACT_SILU_MUL) {
                const int64_t no = (n0 + wn * WN) / 2 + l16;
                if (no < a.N / 2) a.Y[m * a.ldy + no] = f32_to_bf16_rne(silu_f32(z[0]) * z[1]);
            } else {
#pragma unroll
                for (int j = 0; j < CJ; ++j) {
                    const int64_t n = n0 + wn * WN + j * 16 + l16;
                    if (n < a.N) a.Y[m * a.ldy + n] = f32_to_bf16_rne(a.epi.act == ACT_SILU ? silu_f32(z[j]) : z[j]);
                }
            }
        }
    }
}

}  // namespace tiled16

template <int G>
static int launch_a16_tiled_t(const A16Args& a, hipStream_t stream)
{
    using namespace tiled16;
    const int tiles_m = (int)((a.M + BM - 1) / BM);
    const int tiles_n = (int)((a.N + BN - 1) / BN);
    const int group_m = a.tune.tiled_group_m ? a.tune.tiled_group_m : 8;
    const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n)), block(THREADS);
    hipLaunchKernelGGL(a16_tiled_kernel<G>, grid, block, LDS_BYTES, stream, a, tiles_m, tiles_n, group_m);
    return check_launch("w2_matmul_a16[tiled]");
}

int launch_a16_tiled(const A16Args& a, hipStream_t stream)
{
    return a.G == 128 ? launch_a16_tiled_t<128>(a, stream) : launch_a16_tiled_t<64>(a, stream);
}

}  // namespace w2
