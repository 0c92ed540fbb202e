// Packed device layout of the 2-bit weights (this library's own design for
// CDNA4; the analog of the paper's off-line pre-formatting, Sec. II-B/II-D).
//
// Values, not caller codes, are stored: each weight is the 2-bit two's
// complement of q in {-2,-1,0,1}.  Moving a field to the top two bits of its
// byte, (w << (6-2j)) & 0xC0C0C0C0, therefore yields the signed int8 value
// 64*q in every byte lane: one shift and one mask per four weights give a
// ready operand for v_dot4_i32_i8 and for the int8 MFMA, with no zero-point
// term.  The factor 64 is removed exactly (a power of two) in the epilogue.
//
// Tile = 16 columns x 256 k = 1 KiB = 64 lanes x 16 B, so that one
// global_load_dwordx4 per lane reads a tile and a wave reads 1 KiB contiguous.
// Tiles of one column block are contiguous along k.
//
//   blob  = codes region | scales region
//   codes : [Np/16 cb][Kp/256 kt][64 lane][4 dword t]            uint32
//     dword (lane, t) holds column n = 16*cb + (lane & 15) and the 16 weights
//     k = 256*kt + 64*t + 16*(lane >> 4) + 4*j + b,  j = field, b = byte:
//     bits [8b+2j+1 : 8b+2j].  (lane & 15, lane >> 4) is exactly the
//     (column, k-block) a lane supplies to the B operand of
//     v_mfma_i32_16x16x64_i8, and field j is operand dword j.
//   scales: [Np/16 cb][Kp/256 kt][16 n][256/G]                    bf16
//     so a lane fetches all group scales of its column for a tile in one load.
//   Np = N rounded up to 16, Kp = K rounded up to 256; padding weights are 0,
//   padding scales are 0.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace w2 {

constexpr int TILE_N = 16;
constexpr int TILE_K = 256;
constexpr int TILE_BYTES = 1024;

struct Layout {
    int64_t K, N, Kp, Np;
    int G;
    int64_t n_cb;         // column blocks
    int64_t n_kt;         // k tiles per column block
    int gpt;              // groups per tile = 256 / G
    size_t codes_bytes;   // offset of the scales region
    size_t scales_bytes;
    size_t total_bytes;
};

inline Layout make_layout(int64_t K, int64_t N, int G)
{
    Layout L;
    L.K = K; L.N = N; L.G = G;
    L.Kp = (K + TILE_K - 1) / TILE_K * TILE_K;
    L.Np = (N + TILE_N - 1) / TILE_N * TILE_N;
    L.n_cb = L.Np / TILE_N;
    L.n_kt = L.Kp / TILE_K;
    L.gpt = TILE_K / G;
    L.codes_bytes = (size_t)L.n_cb * L.n_kt * TILE_BYTES;
    L.scales_bytes = (size_t)L.n_cb * L.n_kt * TILE_N * L.gpt * sizeof(uint16_t);
    L.total_bytes = L.codes_bytes + ((L.scales_bytes + 255) / 256) * 256;
    return L;
}

}  // namespace w2
