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

#include "w2_small_common.h"

namespace w2 {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr float ZP = 130.0f;     // 128 (the bf16 constant) + 2 (s = q + 2)

__device__ __forceinline__ void upconvert_bf16(uint32_t w, v4i& b0, v4i& b1)
{
    const uint32_t x = w ^ 0xAAAAAAAAu;
    b0[0] = (int)((x & 0x00030003u) | 0x43004300u);
    b0[1] = (int)(((x >> 2) & 0x00030003u) | 0x43004300u);
    b0[2] = (int)(((x >> 4) & 0x00030003u) | 0x43004300u);
    b0[3] = (int)(((x >> 6) & 0x00030003u) | 0x43004300u);
    b1[0] = (int)(((x >> 8) & 0x00030003u) | 0x43004300u);
    b1[1] = (int)(((x >> 10) & 0x00030003u) | 0x43004300u);
    b1[2] = (int)(((x >> 12) & 0x00030003u) | 0x43004300u);
    b1[3] = (int)(((x >> 14) & 0x00030003u) | 0x43004300u);
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
template <int G, int TMAX>
__global__ void __launch_bounds__(1024)
a16_smallm_kernel(A16Args a, SmallCfg cfg)
{
    W2_SMALL_PROLOGUE();
    const bool DBG = false;
    (void)DBG; (void)cb_ok;
    const int rows = (int)a.M;                              // 1..16
    const int arow = (lane & 15) < rows ? (lane & 15) : rows - 1;

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
                    upconvert_bf16(wd[t], b0, b1);
                    const v4i a0 = *reinterpret_cast<const v4i*>(xrow + t * 128);
                    const v4i a1 = *reinterpret_cast<const v4i*>(xrow + t * 128 + 16);
                    acc = mfma_bf16(a0, b0, acc);
                    acc = mfma_bf16(a1, b1, acc);
                    if (G == 64 || (t & 1)) {
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
    for (int r = 0; r < 4; ++r) red[(wave * 16 + 4 * q + r) * 16 + (lane & 15)] = y[r];
    __syncthreads();
    const int outs = cfg.cbw * rows * 16;
    for (int i = threadIdx.x; i < outs; i += blockDim.x) {
        const int nl = i & 15, m = (i >> 4) % rows, ci = i / (16 * rows);
        float s = 0.0f;
        for (int k = 0; k < cfg.ks; ++k) s += red[((k * cfg.cbw + ci) * 16 + m) * 16 + nl];
        const int64_t nn = ((int64_t)blockIdx.x * cfg.cbw + ci) * TILE_N + nl;
        if (nn < a.N) a.Y[(int64_t)m * a.ldy + nn] = f32_to_bf16_rne(s);
    }
}

bool a16_smallm_supports(const A16Args& a) { return a.M >= 1 && a.M <= 16; }

template <int G>
static int launch_a16_smallm_t(const A16Args& a, hipStream_t stream)
{
    const int rows = (int)a.M;
    const SmallCfg c = pick_cfg(a.n_cb, a.n_kt, rows, 2);
    const size_t extra = (size_t)(c.kc / G) * 16 * sizeof(float);
    const size_t lds = small_lds_bytes(c, rows, 16, 2, extra);
    const int tpw = tiles_per_wave(a.n_kt, c);
    if (tpw <= 2) return launch_small(a16_smallm_kernel<G, 2>, "w2_matmul_a16[smallm]", a, c, lds, stream);
    if (tpw <= 4) return launch_small(a16_smallm_kernel<G, 4>, "w2_matmul_a16[smallm]", a, c, lds, stream);
    return launch_small(a16_smallm_kernel<G, TMAX>, "w2_matmul_a16[smallm]", a, c, lds, stream);
}

int launch_a16_smallm(const A16Args& a, hipStream_t stream)
{
    return a.G == 128 ? launch_a16_smallm_t<128>(a, stream) : launch_a16_smallm_t<64>(a, stream);
}

// ---------------------------------------------------------------- TILED (bf16 MFMA, any M)
// Same workgroup / wave geometry as the w2a8 tiled kernel: 128(M) x 256(N) per
// workgroup, eight waves of 64 x 64, 4 x 4 tiles of v_mfma_f32_16x16x32_bf16.
// A stage is 64 k: one packed dword per column block and lane (two matrix
// instructions per tile: even k, odd k), and 128 rows x 128 B of activations in
// LDS, stored de-interleaved by the copy threads, which also leave the
// per-row sums of the stage in a ring of four slots for the zero-point term.
namespace tiled16 {

constexpr int BM = 128, BN = 256, BK = 64;
constexpr int THREADS = 512;
constexpr int A_STRIDE = BK * 2 + 16;             // bytes per LDS row
constexpr int A_BUF = BM * A_STRIDE;
constexpr int XS_OFF = 2 * A_BUF;                 // float xpart[4][BM]
constexpr int LDS_BYTES = XS_OFF + 4 * BM * 4;
constexpr int WM = 64, WN = 64;

template <int G>
__global__ void __launch_bounds__(THREADS)
a16_tiled_kernel(A16Args a, int tiles_m, int tiles_n, int group_m)
{
    extern __shared__ __align__(16) int8_t smem[];
    float* xpart = reinterpret_cast<float*>(smem + XS_OFF);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int q = lane >> 4, l16 = lane & 15;

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

    const uint32_t* wp[4];
    const uint16_t* sp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int64_t c = tile_n * (BN / TILE_N) + wn * 4 + j;
        c = c < a.n_cb ? c : a.n_cb - 1;                     // clamp: loads stay in bounds
        wp[j] = a.codes + (c * a.n_kt * 64 + lane) * 4;
        sp[j] = a.scales + (c * a.n_kt * TILE_N + l16) * (TILE_K / G);
    }

    // copy: 4 threads per row, one 16-k block (32 B) each
    const int cp_row = tid >> 2, cp_seg = tid & 3;
    int64_t cp_m = m0 + cp_row;
    if (cp_m >= a.M) cp_m = a.M - 1;                         // padded rows repeat the last row
    const uint16_t* cp_src = a.X + cp_m * a.ldx + cp_seg * 16;
    const int cp_dst = cp_row * A_STRIDE + cp_seg * 32;

    v4f acc[4][4];
    float y[4][4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < 4; ++r) y[i][j][r] = 0.0f;
        }

    // stores one 16-k block de-interleaved and the row's partial sum of this stage
    auto stage_store = [&](const uint4& lo, const uint4& hi, int buf, int slot) __attribute__((always_inline)) {
        const uint32_t d[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        float s = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += pair_sum(d[e]);
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        uint4 ev, od;
        ev.x = __builtin_amdgcn_perm(d[1], d[0], 0x05040100u);
        ev.y = __builtin_amdgcn_perm(d[3], d[2], 0x05040100u);
        ev.z = __builtin_amdgcn_perm(d[5], d[4], 0x05040100u);
        ev.w = __builtin_amdgcn_perm(d[7], d[6], 0x05040100u);
        od.x = __builtin_amdgcn_perm(d[1], d[0], 0x07060302u);
        od.y = __builtin_amdgcn_perm(d[3], d[2], 0x07060302u);
        od.z = __builtin_amdgcn_perm(d[5], d[4], 0x07060302u);
        od.w = __builtin_amdgcn_perm(d[7], d[6], 0x07060302u);
        uint4* dst = reinterpret_cast<uint4*>(smem + buf * A_BUF + cp_dst);
        dst[0] = ev;
        dst[1] = od;
        if (cp_seg == 0) xpart[slot * BM + cp_row] = s;
    };
    auto load_w = [&](int64_t st, uint32_t (&w)[4], uint32_t (&sc)[4]) __attribute__((always_inline)) {
        const int64_t kt = st >> 2;
        const int t = (int)(st & 3);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            w[j] = wp[j][kt * 256 + t];
            if constexpr (G == 128)
                sc[j] = sp[j][kt * (TILE_N * 2) + (t >> 1)];
            else
                sc[j] = sp[j][kt * (TILE_N * 4) + t];
        }
    };

    const int64_t n_st = a.n_kt * 4;                         // stages of 64 k
    uint4 ar0 = *reinterpret_cast<const uint4*>(cp_src);
    uint4 ar1 = *reinterpret_cast<const uint4*>(cp_src + 8);
    uint32_t wc[4], sc[4], wnx[4], snx[4];
    load_w(0, wc, sc);
    stage_store(ar0, ar1, 0, 0);
    __syncthreads();

    const int8_t* a_base = smem + (wm * WM + l16) * A_STRIDE + q * 32;

    for (int64_t st = 0; st < n_st; ++st) {
        const int buf = (int)(st & 1);
        const bool more = st + 1 < n_st;
        if (more) {
            ar0 = *reinterpret_cast<const uint4*>(cp_src + (st + 1) * BK);
            ar1 = *reinterpret_cast<const uint4*>(cp_src + (st + 1) * BK + 8);
            load_w(st + 1, wnx, snx);
        }
        const int8_t* ab = a_base + buf * A_BUF;
        v4i a0[4], a1[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a0[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE);
            a1[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE + 16);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v4i b0, b1;
            upconvert_bf16(wc[j], b0, b1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[i][j] = mfma_bf16(a0[i], b0, acc[i][j]);
                acc[i][j] = mfma_bf16(a1[i], b1, acc[i][j]);
            }
        }
        const bool group_end = (G == 64) || (st & 1);
        if (group_end) {
            // X_g[m] for this lane's rows: the stage partials of the group (ring slots)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = wm * WM + i * 16 + 4 * q;
                v4f xg = *reinterpret_cast<const v4f*>(xpart + (int)(st & 3) * BM + row);
                if constexpr (G == 128) {
                    const v4f xp = *reinterpret_cast<const v4f*>(xpart + (int)((st - 1) & 3) * BM + row);
                    xg += xp;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float sw = __uint_as_float(sc[j] << 16);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        y[i][j][r] = fmaf(sw, fmaf(-ZP, xg[r], acc[i][j][r]), y[i][j][r]);
                    acc[i][j] = (v4f){0.f, 0.f, 0.f, 0.f};
                }
            }
        }
        if (more) {
            stage_store(ar0, ar1, buf ^ 1, (int)((st + 1) & 3));
#pragma unroll
            for (int j = 0; j < 4; ++j) { wc[j] = wnx[j]; sc[j] = snx[j]; }
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t m = m0 + wm * WM + i * 16 + 4 * q + r;
            if (m >= a.M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = n0 + wn * WN + j * 16 + l16;
                if (n < a.N) a.Y[m * a.ldy + n] = f32_to_bf16_rne(y[i][j][r]);
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
    int group_m = env_int("W2_TILED_GROUP_M", 4);
    if (group_m < 1) group_m = 1;
    const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n)), block(THREADS);
    hipLaunchKernelGGL(a16_tiled_kernel<G>, grid, block, LDS_BYTES, stream, a, tiles_m, tiles_n, group_m);
    return check_launch("w2_matmul_a16[tiled]");
}

int launch_a16_tiled(const A16Args& a, hipStream_t stream)
{
    return a.G == 128 ? launch_a16_tiled_t<128>(a, stream) : launch_a16_tiled_t<64>(a, stream);
}

}  // namespace w2
