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

typedef int v4i __attribute__((ext_vector_type(4)));
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
    i = i < total ? i : total - 1;               // branch-free: surplus threads re-read the last piece
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

int launch_a16_tiled(const A16Args&, hipStream_t)
{
    set_error("w2_matmul_a16: the tiled kernel is not built yet (M > 16)");
    return -2;
}

}  // namespace w2
