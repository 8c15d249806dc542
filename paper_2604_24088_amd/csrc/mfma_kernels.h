// Matrix-core kernels for block sizes B = 32 .. 512 on gfx950.
//
// The Hadamard rotation of Algorithm 1 runs as a dense product on MFMA.  A TILE is 2048
// consecutive elements, seen as 16 UNITS (rows) of 128 elements:  V[16, 128] = X[16, 128] H_128.
// Both operands are exact in the input format (bf16 data or FP8 / INT8 codes, +-1 entries), products
// are exact and accumulation is fp32.  A block of B = 128 kRB elements is kRB consecutive units;
// because H_B = H_kRB (x) H_128, its rotation is the 128-point product of each unit followed by
// log2(kRB) butterfly stages ACROSS the units of the block, which live in registers of one lane.
// A block of B = 128 / kSub elements (kSub = 2, 4) is an aligned part of a unit; the product
// then uses I_kSub (x) H_B instead of H_128: the same +-1 tiles with the entries that pair
// different blocks set to zero (a whole lane of the B operand at a time).
// Everything else (sum of squares, max|W|, the two block scalars, conversion) rides along in
// the same pass, so each byte of the tensor crosses HBM once.
//
// The last tile of a tensor may be partial (n not a multiple of 2048): the wave that owns it reads
// zeros past the end (the zero padding of the last block, which sigma still divides by B) and
// stores only the blocks and elements that exist, so every call is ONE kernel whatever n is.
//
// A 64-lane wavefront handles a few consecutive tiles (one to eight: the host picks the number from the call and the
// payload count) and exits: no persistent loop.  The
// dispatcher hands out workgroups in index order, so the tiles in flight form one dense,
// advancing window of memory, which measured ~15 % faster on HBM than a grid-stride loop over the
// same tiles.  Every wave works in an LDS region of its own (one or two waves per workgroup), so
// there is no workgroup barrier anywhere: wave_lds_sync() orders a wave's own LDS accesses.
//
//   global -> registers   coalesced 16-byte non-temporal loads, 1 KiB per wave instruction
//   registers -> LDS      the tile, unit row by unit row, swizzled
//   LDS -> A operand      lane (i = lane%16, g = lane/16) reads 16-byte pieces of unit row i
//   MFMA                  D[i][n] += sum_k A[i][k] B[k][n],  B = tiles of H_128 in registers
//   D -> HBM              lane (n = lane%16, g), register r holds row 4g+r, column n
//
// Index maps (all bijections; correctness only needs the A and B operands to agree on them):
//   unit of MFMA row i           u(i) = 4 (i % 4) + i / 4 for B = 128 (each store instruction of the
//                                wave then covers one contiguous span); u(i) = i for B > 128 (the
//                                units of a block must sit in one lane: rows 4g .. 4g+3)
//   output position of column n  p(nt, n) = 8 n + nt   (nt = which of 8 MFMA column tiles): every lane
//                                owns 8 consecutive outputs of each of its rows
//   element of A slot            compress: e(c, g, m, y) = 8 (4 g + m) + 2 c + y,  c = MFMA step 0..3
//                                decode:   e(m, g, b) = 64 m + 16 g + b,  m = 0..1, b = 0..15
//   B entry                      H[e][p] = (-1)^popcount(e & p)
#pragma once

#include "device_util.h"
#include "tables.h"

namespace taco {

constexpr int kTileElems = 2048;

template <int kBlock>
__device__ __forceinline__ constexpr float inv_sqrt_block() {
    return kBlock == 32 ? 0.17677669529663687f : kBlock == 64 ? 0.125f : kBlock == 128 ? 0.08838834764831845f
         : kBlock == 256 ? 0.0625f : 0.04419417382415922f;
}

template <int kRB>
__device__ __forceinline__ int unit_of_row(int i) {
    return kRB == 1 ? 4 * (i & 3) + (i >> 2) : i;
}

// Where codes and {alpha, s} records live.  Split layout: `payload` holds the codes in element
// order and `scales` the records.  Interleaved layout (the paper's placement, Section 4.4.2:
// the two scalars directly behind their block's codes): `payload` holds records of B + 8 bytes,
// B codes then {float alpha; float s;}, and `scales` is unused.  B + 8 is a multiple of 8 but not
// of 16, so the interleaved form is addressed in 8-byte words; a tile of 2048 elements still
// starts on a 16-byte boundary for every block size.
template <int kBlock, bool kInterleaved>
struct PayloadLayout {
    static constexpr int kBlocksPerTile = 2048 / kBlock;
    static constexpr int kRecordWords = kBlock / 8 + (kInterleaved ? 1 : 0);   // 8-byte words per block
    static constexpr int kTileWords = kBlocksPerTile * kRecordWords;           // 8-byte words per tile
    static constexpr int kTileChunks = kTileWords / 2;                         // 16-byte chunks per tile
    static constexpr int kRecordBytes = 8 * kRecordWords;
    static_assert(kTileWords % 2 == 0, "a tile must be a whole number of 16-byte chunks");

    // 8-byte word index, in the payload buffer, of codes 8 w .. 8 w + 7 of tile-local block blk.
    static __device__ __forceinline__ int64_t code_word(int64_t tile, int blk, int w) {
        return tile * kTileWords + blk * kRecordWords + w;
    }
    // Interleaved only: word index of the {alpha, s} record of tile-local block blk.
    static __device__ __forceinline__ int64_t scale_word(int64_t tile, int blk) {
        return tile * kTileWords + blk * kRecordWords + kBlock / 8;
    }
};

// In-register butterfly across the kRB units of a block: v[r] -> sum_h (-1)^popcount(h & r) v[h]
// within each aligned group of kRB registers (natural order, H_kRB).
template <int kRB>
__device__ __forceinline__ void units_butterfly(f32x4& v) {
    if (kRB >= 2) {
        const float a0 = v[0] + v[1], a1 = v[0] - v[1], a2 = v[2] + v[3], a3 = v[2] - v[3];
        v[0] = a0; v[1] = a1; v[2] = a2; v[3] = a3;
    }
    if (kRB == 4) {
        const float b0 = v[0] + v[2], b2 = v[0] - v[2], b1 = v[1] + v[3], b3 = v[1] - v[3];
        v[0] = b0; v[1] = b1; v[2] = b2; v[3] = b3;
    }
}

// ------------------------------------------------------------------------------------------
// compress
// ------------------------------------------------------------------------------------------
//
// Element map of the compress kernel.  A 16-byte chunk j (0..15) of a unit holds 8 elements,
// i.e. 4 dwords c = 0..3 of two bf16 (y = 0, 1):  e = 8 j + 2 c + y.  MFMA step c takes, from
// the four chunks j = 4g + m (m = 0..3) of the lane's unit row, dword c: A slot t = 2m + y.
// Against output position p = 8 n + nt the sign of H[e][p] splits into
//     parity((4g+m) & n) ^ (y & nt)           a pattern that depends on nt only through nt & 1
//   ^ parity(c & (nt >> 1))                   one sign for the whole MFMA
// so four register tiles (two patterns, two signs) serve all 32 MFMAs of a tile.
//
// To hand step c its operand with one 16-byte LDS read, the tile is written to LDS
// transposed at dword granularity: unit row b (padded to 512 bytes), 16-byte slot
// (4 (j/4) + c + b) holds dword c of chunks 4 (j/4) .. 4 (j/4) + 3.  The "+ b" rotation
// spreads the 16 rows a read instruction touches over all banks, and because rows are
// padded the rotation never wraps: every LDS address is one per-lane base plus an
// immediate.  Writes (4-byte) and reads (16-byte) are both bank-conflict free.

constexpr int kCompressLdsDwords = 16 * 128;   // 16 unit rows of 128 dwords (64 used + rotation room)

// Maximum, over the 16 lanes of a DPP row, of per-block values, for non-negative floats
// (compared as unsigned integers).  m[r] is this lane's maximum over row r.
//   kRB = 1: four blocks (rows); the maximum of row q ends up in the lanes with lane % 4 == q.
//   kRB = 2: two blocks (rows 0-1, 2-3); block j ends up in the lanes with lane % 2 == j.
//   kRB = 4: one block; every lane gets it.
template <int kRB>
__device__ __forceinline__ float row16_block_max(const float (&m)[4], int n16) {
    const bool b0 = (n16 & 1) != 0, b1 = (n16 & 2) != 0;
    uint32_t v;
    if (kRB == 1) {
        const uint32_t u0 = __builtin_bit_cast(uint32_t, m[0]), u1 = __builtin_bit_cast(uint32_t, m[1]);
        const uint32_t u2 = __builtin_bit_cast(uint32_t, m[2]), u3 = __builtin_bit_cast(uint32_t, m[3]);
        const uint32_t keep01 = b0 ? u1 : u0, send01 = b0 ? u0 : u1;
        const uint32_t keep23 = b0 ? u3 : u2, send23 = b0 ? u2 : u3;
        const uint32_t a0 = max(keep01, dpp_u32<0xB1>(send01));   // quad_perm [1,0,3,2]: lane ^ 1
        const uint32_t a1 = max(keep23, dpp_u32<0xB1>(send23));
        const uint32_t keep = b1 ? a1 : a0, send = b1 ? a0 : a1;
        v = max(keep, dpp_u32<0x4E>(send));                       // quad_perm [2,3,0,1]: lane ^ 2
    } else if (kRB == 2) {
        const uint32_t u0 = __builtin_bit_cast(uint32_t, __builtin_fmaxf(m[0], m[1]));
        const uint32_t u1 = __builtin_bit_cast(uint32_t, __builtin_fmaxf(m[2], m[3]));
        const uint32_t keep = b0 ? u1 : u0, send = b0 ? u0 : u1;
        v = max(keep, dpp_u32<0xB1>(send));
        v = max(v, dpp_u32<0x4E>(v));
    } else {
        v = __builtin_bit_cast(uint32_t, __builtin_fmaxf(__builtin_fmaxf(m[0], m[1]), __builtin_fmaxf(m[2], m[3])));
        v = max(v, dpp_u32<0xB1>(v));
        v = max(v, dpp_u32<0x4E>(v));
    }
    v = max(v, dpp_u32<kDppRowRor(4)>(v));
    v = max(v, dpp_u32<kDppRowRor(8)>(v));
    return __builtin_bit_cast(float, v);
}

// Blocks smaller than a unit (kSub = 2 or 4 blocks per row): the outputs of block (row, sub) sit
// in the 16 / kSub lanes with lane / (16 / kSub) == sub.  The maximum of row q's block ends up in
// the lanes with lane % 4 == q of that lane group.
template <int kSub>
__device__ __forceinline__ float sub_block_max(const float (&m)[4], int n16) {
    const bool b0 = (n16 & 1) != 0, b1 = (n16 & 2) != 0;
    uint32_t u[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        u[r] = __builtin_bit_cast(uint32_t, m[r]);
        if (kSub == 2) u[r] = max(u[r], dpp_u32<0x141>(u[r]));    // row_half_mirror: joins the two quads of an 8-lane half
    }
    const uint32_t keep01 = b0 ? u[1] : u[0], send01 = b0 ? u[0] : u[1];
    const uint32_t keep23 = b0 ? u[3] : u[2], send23 = b0 ? u[2] : u[3];
    const uint32_t a0 = max(keep01, dpp_u32<0xB1>(send01));
    const uint32_t a1 = max(keep23, dpp_u32<0xB1>(send23));
    const uint32_t keep = b1 ? a1 : a0, send = b1 ? a0 : a1;
    return __builtin_bit_cast(float, max(keep, dpp_u32<0x4E>(send)));
}

// Per-lane constants of the compress stage and the stage itself (everything after the tile
// has been written to LDS).  Shared by the compress kernel and by the fused
// decompress_sum -> compress kernel.
template <int kRB, int kSub>
struct CompressLane {
    static_assert((kRB == 1 || kRB == 2 || kRB == 4) && (kSub == 1 || kSub == 2 || kSub == 4) && (kRB == 1 || kSub == 1),
                  "block size must be 32, 64, 128, 256 or 512");
    static constexpr int kBlock = 128 * kRB / kSub;
    static constexpr int kBlocksPerTile = 2048 / kBlock;

    u32x4 hb[2][2];     // B operand: patterns P0 / P1 (nt even / odd) [first index] and their negatives [second]
    int g, n16, q;
    int rd_base;        // LDS dword address of this lane's A operand for step 0
    bool owns_scales;   // this lane computes and stores {alpha, s} of one block
    int my_block;       // ... that block (tile-local index)
    int energy_src;     // kSub > 1: lane that holds the block's sum of squares

    __device__ __forceinline__ explicit CompressLane(int lane) {
        g = lane >> 4;
        n16 = lane & 15;
        q = n16 & 3;
        // For kSub > 1 the element's block within the unit is eh (top bits of 4g+m, i.e. of g) and
        // the output's is ph (top bits of n16): the entry is H_B's where eh == ph (the eh & ph term
        // of the 128-point sign drops out) and zero elsewhere.
        const int eh = kSub == 2 ? (g >> 1) : g;
        const int ph = kSub == 2 ? (n16 >> 3) : (n16 >> 2);
        const bool same_block = kSub == 1 || eh == ph;
        const uint32_t block_flip = (kSub > 1 && parity32(eh & ph)) ? 0x80008000u : 0u;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t s0 = (parity32((4 * g + m) & n16) ? 0x80008000u : 0u) ^ block_flip;
            const uint32_t base = 0x3F803F80u ^ s0;
            hb[0][0][m] = same_block ? base : 0u;
            hb[1][0][m] = same_block ? base ^ 0x80000000u : 0u;      // y = 1 half flips when nt is odd
            hb[0][1][m] = same_block ? base ^ 0x80008000u : 0u;
            hb[1][1][m] = same_block ? base ^ 0x00008000u : 0u;
        }
        // Reader: MFMA row i = n16 is unit u(i); step c reads slot 4g + c + u.
        const int rd_unit = unit_of_row<kRB>(n16);
        rd_base = rd_unit * 128 + (4 * g + rd_unit) * 4;
        // Which block this lane finishes.  The Gram diagonal of row i sits in lane (i, i/4),
        // register i%4, so only the quad n16/4 == g of each DPP row holds energies; within it the
        // lane must also hold the block's max|W|.  For kSub > 1 the energy comes from VALU partial
        // sums instead: lane (n16, g) finishes block (row 4g + n16 % 4, part ph) and fetches its
        // energy from the A-layout lane that summed that part of the row.
        owns_scales = (n16 >> 2) == g;
        energy_src = 0;
        if (kSub == 4) { owns_scales = true; my_block = unit_of_row<1>(4 * g + q) * 4 + ph; energy_src = 16 * ph + 4 * g + q; }
        else if (kSub == 2) { owns_scales = ((n16 >> 2) & 1) == 0; my_block = unit_of_row<1>(4 * g + q) * 2 + ph; energy_src = 32 * ph + 4 * g + q; }
        else if (kRB == 1) { my_block = 4 * q + g; }
        else if (kRB == 2) { owns_scales = owns_scales && ((q >> 1) == (q & 1)); my_block = 2 * g + (q & 1); }
        else { owns_scales = owns_scales && q == 0; my_block = g; }
    }

    // LDS dword address at which the lane that holds elements 8j .. 8j+7 of unit `unit` (as four
    // dwords c = 0..3) stores dword c:  lds_slot(unit, j) + 4 c.
    static __device__ __forceinline__ int lds_slot(int unit, int j) {
        return unit * 128 + (4 * (j >> 2) + unit) * 4 + (j & 3);
    }

    // Sender side of Algorithm 1 for the tile that sits in LDS.  Ends with the wave past its last
    // LDS read (wave_lds_sync follows the reads), so the caller may overwrite the buffer afterwards.
    // In the interleaved layout the records (B + 8 bytes) do not line up with cache lines, and
    // storing codes and scalars straight from the lanes leaves every line written in pieces
    // (measured: 142 us instead of 99 us per compress of the bench tensor).  The tile's records are
    // therefore assembled in LDS (the input buffer is free once the A operands are read) and
    // leave as contiguous 16-byte chunks.
    // kFormat: 0 = E4M3, 1 = E5M2, 2 = INT8 (format ablation).  mode: the component ablations as a bit mask
    // (1 adaptive rescaling, 2 rotation, 4 post-rotation scale; 7 is the method).  Without the rescaling
    // alpha = 1.  Without the rotation the matrix cores multiply by the IDENTITY instead of H (8 of the 32
    // products, the rest would be zero): the tile takes the same way from the load layout to the store layout,
    // and everything after it is shared.  Without the post-rotation scale s = 1 and Z = alpha W / sqrt(B)
    // itself is converted, clamped to +-Q_max.
    // blocks_left: blocks of the tensor from this tile's first block on; only the first
    // min(blocks_left, kBlocksPerTile) blocks of the tile exist and are stored.
    // kGeneric = false is the method itself and its no-rescaling variant (rotation and post-rotation scale on:
    // the other two bits of `mode` are not looked at and their code is compiled out); kGeneric = true handles
    // any mode at run time, at the price of some twenty more registers.
    template <bool kInterleaved, int kFormat, bool kGeneric>
    __device__ __forceinline__ void tile_from_lds(uint32_t* lds, int64_t tile, int64_t blocks_left, float tau, float eps,
                                                  int mode, u32x2* __restrict__ payload, f32x2* __restrict__ scales) const {
        constexpr float kQ = format_qmax<kFormat>();
        const bool rescale = (mode & 1) != 0;
        const bool rotate = kGeneric ? (mode & 2) != 0 : true, postscale = kGeneric ? (mode & 4) != 0 : true;
        using Layout = PayloadLayout<kBlock, kInterleaved>;
        u32x2* records = reinterpret_cast<u32x2*>(lds);     // interleaved: the tile's records, 8-byte words
        u32x4 a[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) a[c] = *reinterpret_cast<const u32x4*>(&lds[rd_base + 4 * c]);
        wave_lds_sync();

        // V = X H_128 (unnormalised rotation of Eq. ash_rotation, per unit) and the Gram diagonal
        // sum_j x_j^2 of every unit (Eq. ash_sigma), all on the matrix cores.
        f32x4 acc[8];
        f32x4 gram = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[nt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (rotate) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bf16x8 av = __builtin_bit_cast(bf16x8, a[c]);
                if (kSub == 1) gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, av, gram, 0, 0, 0);
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    const int sign = __builtin_popcount(c & (nt >> 1)) & 1;
                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        av, __builtin_bit_cast(bf16x8, hb[nt & 1][sign]), acc[nt], 0, 0, 0);
                }
            }
            // W = H_B G for blocks of more than one unit: butterfly across the block's units.
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) units_butterfly<kRB>(acc[nt]);
        } else {
            // W = G.  Identity entries: element e = 8 (4g + m) + 2c + y meets position p = 8 n + nt where
            // 4g + m = n and 2c + y = nt, so output tile nt needs step c = nt / 2 only, with a 1.0 in half
            // y = nt % 2 of register m of the lanes whose chunk 4g + m is the column n.
            u32x4 id[2];
#pragma unroll
            for (int mm = 0; mm < 4; ++mm) {
                const bool hit = 4 * g + mm == n16;
                id[0][mm] = hit ? 0x00003F80u : 0u;
                id[1][mm] = hit ? 0x3F800000u : 0u;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bf16x8 av = __builtin_bit_cast(bf16x8, a[c]);
                if (kSub == 1) gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, av, gram, 0, 0, 0);
                acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, id[0]), acc[2 * c], 0, 0, 0);
                acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, id[1]), acc[2 * c + 1], 0, 0, 0);
            }
        }

        // max|W| of each block.
        float m[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float v = 0.0f;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) v = __builtin_fmaxf(v, __builtin_fabsf(acc[nt][r]));
            m[r] = v;
        }
        const float wmax = kSub == 1 ? row16_block_max<kRB>(m, n16) : sub_block_max<kSub>(m, n16);
        // Energy of the block whose factor this lane supplies (row 4g + q; kRB = 2: block q % 2 of the lane
        // group; kRB = 4: the group's one block).  The Gram diagonal of row i sits in lane (i, i / 4), register
        // i % 4, i.e. in quad n16 / 4 == g of each DPP row: summed over the block's units there, then handed
        // to the other three quads (they add zeros).
        // Only the lane that stores the block's scalars needs it, unless the codes themselves depend on alpha
        // (no post-rotation scale: kGeneric).
        float energy;
        if (kSub == 1) {
            energy = q == 0 ? gram[0] : q == 1 ? gram[1] : q == 2 ? gram[2] : gram[3];
            if (kGeneric && (n16 >> 2) != g) energy = 0.0f;
            if (kRB >= 2) energy += dpp_f32<0xB1>(energy);
            if (kRB == 4) energy += dpp_f32<0x4E>(energy);
            if (kGeneric) {
                if (kRB == 2) energy = dpp_f32<0x88>(energy);          // quad_perm [0,2,0,2]: block q % 2 sits in lanes 2 (q % 2)
                energy += dpp_f32<kDppRowRor(4)>(energy);
                energy += dpp_f32<kDppRowRor(8)>(energy);
            }
        } else {
            // A-layout lane (i, g) holds elements 32g .. 32g+31 of unit row i: one block for
            // B = 32, half a block for B = 64 (the other half is 16 lanes away).
            float e0 = 0.0f, e1 = 0.0f;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t w0 = a[c][0], w1 = a[c][1], w2 = a[c][2], w3 = a[c][3];
                e0 = dot2_self_bf16(w0, e0);
                e1 = dot2_self_bf16(w1, e1);
                e0 = dot2_self_bf16(w2, e0);
                e1 = dot2_self_bf16(w3, e1);
            }
            energy = e0 + e1;
            if (kSub == 2) energy += __shfl_xor(energy, 16, 64);
            energy = __shfl(energy, energy_src, 64);
        }
        // Eq. ash_sigma, ash_alpha.  A sum of squares that overflows fp32 (elements beyond about 2^58) is taken as the largest
        // finite number: alpha then differs from tau / sigma, but the codes do not depend on alpha and the reconstruction
        // only on s / alpha = max|W| / (Q_max sqrt(B)), so both stay right; without the clamp alpha would be 0 and decode NaN.
        const float alpha = rescale ? tau * __builtin_amdgcn_rsqf(__builtin_fminf(energy * (1.0f / kBlock), 0x1.fffffep+127f) + eps) : 1.0f;
        const float norm = rotate ? inv_sqrt_block<kBlock>() : 1.0f;
        // With the post-rotation scale: Z / s = W * Q_max / max|W| in exact arithmetic (Eq. post_scale,
        // Eq. quantization), s = max|Z| / Q_max; an all-zero block stores s = 0 whatever alpha is (with
        // eps = 0 it is infinite).  Without it: s = 1 and the codes are those of Z = alpha W / sqrt(B).
        float to_code, s;
        if (postscale) {
            to_code = wmax > 0.0f ? kQ * __builtin_amdgcn_rcpf(wmax) : 0.0f;
            s = wmax > 0.0f ? (wmax * alpha) * (norm / kQ) : 0.0f;
        } else {
            to_code = alpha * norm;
            s = 1.0f;
        }
        // Q_max / max|W| leaves fp32 when max|W| < 2^-118 (blocks of bf16 subnormals get there): such a block takes a
        // power of two out of its rotated values first.  One wave-uniform test per tile, next to never true.
        if (postscale) {
            const bool tiny = wmax > 0.0f && wmax < 0x1p-100f;
            if (__builtin_amdgcn_ballot_w64(tiny) != 0) {
                const int lift = tiny ? 64 : 0;
                to_code = wmax > 0.0f ? kQ * __builtin_amdgcn_rcpf(__builtin_ldexpf(wmax, lift)) : 0.0f;
                const float lift_bits = __builtin_bit_cast(float, lift);
                const int l0 = __builtin_bit_cast(int, dpp_f32<kDppQuadBcast(0)>(lift_bits));
                const int l1 = __builtin_bit_cast(int, dpp_f32<kDppQuadBcast(kRB == 1 ? 1 : 0)>(lift_bits));
                const int l2 = __builtin_bit_cast(int, dpp_f32<kDppQuadBcast(kRB == 1 ? 2 : kRB == 2 ? 1 : 0)>(lift_bits));
                const int l3 = __builtin_bit_cast(int, dpp_f32<kDppQuadBcast(kRB == 1 ? 3 : kRB == 2 ? 1 : 0)>(lift_bits));
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    acc[nt][0] = __builtin_ldexpf(acc[nt][0], l0);
                    acc[nt][1] = __builtin_ldexpf(acc[nt][1], l1);
                    acc[nt][2] = __builtin_ldexpf(acc[nt][2], l2);
                    acc[nt][3] = __builtin_ldexpf(acc[nt][3], l3);
                }
            }
        }
        if (owns_scales && my_block < blocks_left) {
            if (kInterleaved)
                records[Layout::scale_word(0, my_block)] = __builtin_bit_cast(u32x2, f32x2{alpha, s});
            else
                store_stream<true>(&scales[tile * kBlocksPerTile + my_block], f32x2{alpha, s});
        }

        // 8 consecutive codes per lane and row.  The factor of row R's block comes from the quad
        // lane that holds it (kRB = 1: lane R; kRB = 2: lane R / 2; kRB = 4: any).
        // Codes 8 n16 .. 8 n16 + 7 of unit u belong to block u / kRB (word 16 (u % kRB) + n16 of it) when
        // a block is one or more units, and to block u kSub + n16 / (16 / kSub) when it is part of a unit.
#define TACO_STORE_ROW(R)                                                                      \
        {                                                                                      \
            const float f = dpp_f32<kDppQuadBcast(kRB == 1 ? R : kRB == 2 ? R / 2 : 0)>(to_code); \
            u32x2 w;                                                                           \
            if (postscale) {                                                                   \
                w.x = pack_codes4<kFormat>(acc[0][R], acc[1][R], acc[2][R], acc[3][R], f);      \
                w.y = pack_codes4<kFormat>(acc[4][R], acc[5][R], acc[6][R], acc[7][R], f);      \
            } else {                                                                           \
                w.x = pack_codes4_clamped<kFormat>(acc[0][R], acc[1][R], acc[2][R], acc[3][R], f); \
                w.y = pack_codes4_clamped<kFormat>(acc[4][R], acc[5][R], acc[6][R], acc[7][R], f); \
            }                                                                                  \
            const int unit = unit_of_row<kRB>(4 * g + R);                                      \
            const int blk = kSub == 1 ? unit / kRB : unit * kSub + n16 / (16 / kSub);          \
            const int word = kSub == 1 ? 16 * (unit % kRB) + n16 : n16 % (16 / kSub);          \
            if (kInterleaved) records[Layout::code_word(0, blk, word)] = w;                    \
            else if (blk < blocks_left) store_stream<true>(&payload[Layout::code_word(tile, blk, word)], w); \
        }
        TACO_STORE_ROW(0)
        TACO_STORE_ROW(1)
        TACO_STORE_ROW(2)
        TACO_STORE_ROW(3)
#undef TACO_STORE_ROW
        if (kInterleaved) {
            wave_lds_sync();
            const u32x4* chunks = reinterpret_cast<const u32x4*>(lds);
            u32x4* dst = reinterpret_cast<u32x4*>(payload) + tile * Layout::kTileChunks;
            const int lane = 16 * g + n16;
            if (blocks_left >= kBlocksPerTile) {
#pragma unroll
                for (int c = 0; c < (Layout::kTileChunks + 63) / 64; ++c) {
                    const int chunk = 64 * c + lane;
                    if (chunk < Layout::kTileChunks) store_stream<true>(&dst[chunk], chunks[chunk]);
                }
            } else {
                // partial last tile: only the 8-byte words of the records that exist (a whole number of words, not of chunks)
                const int words = static_cast<int>(blocks_left) * Layout::kRecordWords;
#pragma unroll
                for (int c = 0; c < (Layout::kTileChunks + 63) / 64; ++c) {
                    const int chunk = 64 * c + lane;
                    if (2 * chunk + 2 <= words) store_stream<true>(&dst[chunk], chunks[chunk]);
                    else if (2 * chunk + 1 <= words)
                        store_stream<true>(reinterpret_cast<u32x2*>(&dst[chunk]), u32x2{chunks[chunk].x, chunks[chunk].y});
                }
            }
            wave_lds_sync();
        }
    }
};

// tab: the tensors of the launch (tables.h): x = n bf16 values (16-byte aligned); payload, scales: see
// PayloadLayout.  Block size B = 128 kRB / kSub (at most one of kRB, kSub differs from 1).
// One wave per workgroup, one tile per wave: workgroup w of a tensor handles its tile w.
template <int kRB, int kSub, bool kInterleaved, int kFormat, bool kGeneric>
__global__ __launch_bounds__(64) void compress_mfma_kernel(CompressTable tab, int count, float tau, float eps, int mode) {
    __shared__ uint32_t lds[kCompressLdsDwords];
    constexpr int kBlock = 128 * kRB / kSub;
    const int lane = threadIdx.x;
    int idx;
    int64_t tile;
    tab.locate(blockIdx.x, count, idx, tile);
    const u32x4* __restrict__ x = static_cast<const u32x4*>(tab.x(idx));
    const int64_t n = tab.n(idx);
    const int64_t first_elem = tile * kTileElems;

    u32x4 stage[4];
    if (first_elem + kTileElems <= n) {
#pragma unroll
        for (int c = 0; c < 4; ++c) stage[c] = load16<true>(&x[tile * 256 + 64 * c + lane]);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) stage[c] = load_chunk_guarded(x, first_elem + 8 * (64 * c + lane), n);
    }
    const int64_t blocks_left = (n - first_elem + kBlock - 1) / kBlock;

    const CompressLane<kRB, kSub> cl(lane);
    // Writer: load cp covers tile units 4cp .. 4cp+3; this lane holds chunk j = lane % 16 of unit
    // 4cp + lane / 16.  One base address, the rest are immediates (unit + 4 -> + 528 dwords).
    const int wr_base = CompressLane<kRB, kSub>::lds_slot(lane >> 4, lane & 15);
#pragma unroll
    for (int cp = 0; cp < 4; ++cp) {
#pragma unroll
        for (int c = 0; c < 4; ++c) lds[wr_base + cp * 528 + 4 * c] = stage[cp][c];
    }
    wave_lds_sync();
    cl.template tile_from_lds<kInterleaved, kFormat, kGeneric>(lds, tile, blocks_left, tau, eps, mode,
                                                     static_cast<u32x2*>(tab.payload(idx)), static_cast<f32x2*>(tab.scales(idx)));
}

// ------------------------------------------------------------------------------------------
// decompress / decompress_sum
// ------------------------------------------------------------------------------------------

// out = bf16( sum_i  H_B (codes_i) * s_i / (alpha_i sqrt(B)) ), fp32 accumulation, i ascending.
// tab: the tensors of the launch (tables.h): k payloads (+ scales) each, see PayloadLayout; out: n bf16.
// Wave v of a tensor (v = workgroup-in-tensor * kWaves + wave-in-workgroup) handles its output tiles
// [v * tiles_per_wave, (v+1) * tiles_per_wave) and exits; the waves of a workgroup share nothing
// (each has its own LDS region, there is no workgroup barrier).  A wave's work is the flattened
// list of (tile, payload) items, payload fastest; a ring of kRing items is kept in flight in
// registers.  For blocks of several units the per-payload work is the 128-point product of every
// unit times the block factor; the butterfly across units is linear, so it runs once on the
// accumulated sums.
//
// kFormat: 0 = E4M3 and 1 = E5M2 codes go straight into the FP8 matrix instruction (K = 128, one
// block row per instruction); 2 = INT8 codes into the 8-bit integer one (K = 64, two per row,
// exact int32 sums).
//
// mode: the component ablations (bit 2 = rotation: without it the product is with the identity and the
// butterfly across units is skipped; the other two bits only matter to the recompress form).
//
// kRecompress = true turns the kernel into decompress_sum followed by compress of the
// bf16-rounded sum (the receive side of the reduce-scatter feeding the send side of the
// all-gather, Section 4.4.2): the finished tile goes to LDS in the compress stage's layout
// instead of HBM.  The payload tile and the bf16 tile use the SAME LDS region: a wave's LDS
// accesses execute in order, and the payload tile is dead once its A operand has been read.
// The work of one wave: output tiles [tile_begin, tile_end) of tensor idx.  kGuarded = true is the copy that the
// one wave owning a partial last tile runs (bounds-checked loads and stores for that tile); every other wave runs
// the kGuarded = false copy, in which all of those checks are compiled out.
template <int kRB, int kSub, int kRing, bool kInterleaved, bool kRecompress, int kFormat, bool kGeneric, bool kGray, bool kGuarded,
          bool kAligned = false>
__device__ __forceinline__ void decode_wave(const DecodeTable& tab, int idx, int k, int64_t n, int64_t tile_begin, int64_t tile_end,
                                            u32x4* lds, float tau, float eps, int mode) {
    constexpr int kBlock = 128 * kRB / kSub;
    constexpr int kBlocksPerTile = 2048 / kBlock;
    using Layout = PayloadLayout<kBlock, kInterleaved>;
    constexpr int kLoads = 2;                                    // 16-byte loads per lane and item
    // Interleaved: a tile is 2048 + 8 * blocks bytes; what lies past the first 2048 (at most 512 bytes) is a third,
    // 8-byte load of the first kExtraWords lanes.
    constexpr int kExtraWords = kInterleaved ? 2 * (Layout::kTileChunks - 128) : 0;
    static_assert(kExtraWords <= 64, "the third load covers at most one 8-byte word per lane");
    uint32_t* lds_c = reinterpret_cast<uint32_t*>(lds);
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4;
    const int n16 = lane & 15;
    // Block whose factor this lane computes: the one that contains this lane's outputs of row
    // 4g + n16 % 4 (for kSub > 1 the part ph of that row; a quad never straddles two parts).
    const int ph = kSub == 1 ? 0 : kSub == 2 ? (n16 >> 3) : (n16 >> 2);
    const int my_block = kSub == 1 ? unit_of_row<kRB>(4 * g + (n16 & 3)) / kRB
                                   : unit_of_row<kRB>(4 * g + (n16 & 3)) * kSub + ph;

    const int64_t n_blocks = (n + kBlock - 1) / kBlock;
    // The one tile that may be partial, and how many of its blocks exist (-1: every tile of this wave is whole).
    const int64_t partial_tile = kGuarded ? tile_end - 1 : -1;
    const int partial_blocks = kGuarded ? static_cast<int>(n_blocks - (tile_end - 1) * kBlocksPerTile) : kBlocksPerTile;
    u32x4* __restrict__ out = static_cast<u32x4*>(tab.output(idx));
    const int n_items = static_cast<int>(tile_end - tile_begin) * k;

    // Ring fill.  (pf_tile, pf_i) walks the item list ahead of the consumer.
    u32x4 stage[kRing][kLoads];
    u32x2 stage_x[kRing];       // interleaved: the third load
    f32x2 stage_sc[kRing];      // split: this lane's block scalars
    int64_t pf_tile = tile_begin;
    int pf_i = 0;
    auto fetch = [&](int p) {
        const u32x4* src = static_cast<const u32x4*>(tab.payload(idx, k, pf_i)) + pf_tile * Layout::kTileChunks;
        if (!kGuarded || pf_tile != partial_tile) {
            stage[p][0] = load16<true>(&src[lane]);
            stage[p][1] = load16<true>(&src[64 + lane]);
            if (kInterleaved) {
                if (lane < kExtraWords) stage_x[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src + 128) + lane);
            } else {
                stage_sc[p] = static_cast<const f32x2*>(tab.scales(idx, k, pf_i))[pf_tile * kBlocksPerTile + my_block];
            }
        } else {
            // Partial last tile: only the records / codes of the blocks that exist are read, zeros elsewhere.
            const int words = partial_blocks * Layout::kRecordWords;       // 8-byte words of the tile that exist
#pragma unroll
            for (int c = 0; c < kLoads; ++c) {
                const int chunk = 64 * c + lane;
                u32x4 v = u32x4{0u, 0u, 0u, 0u};
                if (2 * chunk + 2 <= words) v = load16<true>(&src[chunk]);
                else if (2 * chunk + 1 <= words) {
                    const u32x2 h = *reinterpret_cast<const u32x2*>(&src[chunk]);
                    v = u32x4{h.x, h.y, 0u, 0u};
                }
                stage[p][c] = v;
            }
            if (kInterleaved) {
                stage_x[p] = u32x2{0u, 0u};
                if (256 + lane < words) stage_x[p] = *(reinterpret_cast<const u32x2*>(src + 128) + lane);
            } else {
                stage_sc[p] = f32x2{1.0f, 0.0f};
                if (my_block < partial_blocks)
                    stage_sc[p] = static_cast<const f32x2*>(tab.scales(idx, k, pf_i))[pf_tile * kBlocksPerTile + my_block];
            }
        }
        if (++pf_i == k) { pf_i = 0; ++pf_tile; }
    };
#pragma unroll
    for (int p = 0; p < kRing; ++p) {
        if (p < n_items) fetch(p);
    }

    // B operand: 8 column tiles of H_128 as +-1 in the code format's companion (E4M3 +1 = 0x38, -1 = 0xB8
    // for the two FP8 code books; int8 +1 = 0x01, -1 = 0xFF for INT8), 32 bytes per lane each.
    // Slot (m, b) of lane (n16, g) is element e = 64 m + 16 g + b against position p = 8 n16 + nt:
    // sign = parity(b%8 & nt) ^ (b/8 & n16) ^ parity(g & (n16 >> 1)) ^ (m & n16 >> 3).
    // For kSub > 1 the element's block within the unit is eh (top bits of e: m, then g / 2) and the
    // output's is ph: entries with eh != ph are zero and the eh & ph term of the sign drops out.
    // Variants without the rotation (mode bit 2 clear) multiply by the identity instead: entry 1 where
    // e = p, i.e. 64 m + 16 g + b = 8 n16 + nt, zero elsewhere.
    //
    // All 8 tiles in registers take 64 of them.  The lean plain decode (kGray) keeps ONE: the sign splits into parity(b%8 & nt), the same for every lane, and a part that does not depend
    // on nt, so tile nt is tile 0 with fixed bytes negated, and walking nt through a Gray code
    // (0 1 3 2 6 7 5 4) takes one XOR mask per step: bit 0 of nt negates bytes 1 and 3 of every dword, bit 1
    // bytes 2 and 3, bit 2 every byte of the odd dwords.  The 52 XORs per (tile, payload) item run in the
    // shadow of the matrix instructions; the 56 registers saved let a third wave share the SIMD.  Measured on
    // MI355X this pays for one payload (decompress: 2-3 % faster) and costs 3 % from two payloads on, where more
    // waves in flight mean more open DRAM pages per stream; the host side picks the flavour accordingly.
    constexpr uint32_t kPlusOne = kFormat == 2 ? 0x01010101u : 0x38383838u;
    constexpr uint32_t kNegate = kFormat == 2 ? 0xFEu : 0x80u;              // +1 ^ -1, per byte
    constexpr uint32_t kFlipMask[3] = {kNegate << 8 | kNegate << 24, kNegate << 16 | kNegate << 24, kNegate * 0x01010101u};
    static_assert(!(kGray && (kGeneric || kRecompress)), "the running sign tile serves the lean plain decode only");
    const bool rotate = kGeneric ? (mode & 2) != 0 : true;
    uint32_t hb[kGray ? 1 : 8][8];
    uint32_t live_half[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};     // lean flavour, kSub > 1: all ones where half m of the operand is not zero
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        const int m = d >> 2;
        const int b_hi = (d & 3) >> 1;    // bit 3 of b for the 4 bytes of dword d
        const int eh = kSub == 2 ? m : 2 * m + (g >> 1);
        const bool same_block = kSub == 1 || eh == ph;
        int sgn = (b_hi & n16) ^ parity32(g & (n16 >> 1) & 3) ^ (m & (n16 >> 3));
        if (kSub > 1) sgn ^= parity32(eh & ph);
        const uint32_t lane_sign = (sgn & 1) ? kNegate * 0x01010101u : 0u;
        const int e0 = 64 * m + 16 * g + 4 * (d & 3);      // element of byte 0 of this dword
        if (!same_block) live_half[m] = 0u;
#pragma unroll
        for (int nt = 0; nt < (kGray ? 1 : 8); ++nt) {
            uint32_t w = kPlusOne;
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                const int b_lo = (4 * (d & 3) + bb) & 7;
                if (__builtin_popcount(b_lo & nt) & 1) w ^= kNegate << (8 * bb);
            }
            const uint32_t hadamard = same_block ? (w ^ lane_sign) : 0u;
            const int hit = 8 * n16 + nt - e0;              // byte of this dword that is on the diagonal, if 0..3
            const uint32_t identity = (hit >= 0 && hit < 4) ? (kPlusOne & 0xFFu) << (8 * hit) : 0u;
            hb[nt][d] = rotate ? hadamard : identity;
        }
    }

    // LDS addressing.
    // Split layout (16-byte slots, 8 per unit row): writer load m covers tile units 8m .. 8m+7, this
    // lane holds chunk lane%8 of unit 8m + lane/8; reader row i = n16 is unit u(i), half m wants chunk
    // 4m + g.  The XOR swizzle keeps both sides bank-conflict free.
    // Interleaved layout: the tile is copied as it is; the reader computes the byte offset of its
    // 16 codes inside the records (8-byte aligned), and the block's {alpha, s} is read from LDS too.
    int wr_slot[2], rd_slot[2];     // split: 16-byte slot indices; interleaved: rd_slot = byte offsets
    int sc_byte = 0;
    const int rd_unit = unit_of_row<kRB>(n16);
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        if (kInterleaved) {
            wr_slot[m] = 64 * m + lane;
            const int c = 4 * m + g;                         // 16-byte chunk of the unit
            constexpr int kChunksPerBlock = kBlock >= 128 ? 8 : kBlock / 16;
            const int blk = kSub == 1 ? rd_unit / kRB : rd_unit * kSub + c / kChunksPerBlock;
            const int in_block = kSub == 1 ? 128 * (rd_unit % kRB) + 16 * c : 16 * (c % kChunksPerBlock);
            rd_slot[m] = blk * Layout::kRecordBytes + in_block;
        } else {
            const int wb = 8 * m + (lane >> 3);
            wr_slot[m] = wb * 8 + ((lane & 7) ^ ((wb >> 1) & 7));
            rd_slot[m] = rd_unit * 8 + ((4 * m + g) ^ ((rd_unit >> 1) & 7));
        }
    }
    if (kInterleaved) sc_byte = my_block * Layout::kRecordBytes + kBlock;
    const float inv_root_b = rotate ? inv_sqrt_block<kBlock>() : 1.0f;

    f32x4 sum[8];
    int64_t tile = tile_begin;
    int i = 0;
    // One (tile, payload) item from ring slot p.  refill: fetch the item kRing places ahead into the slot;
    // tile_may_end: whether this item can be the last payload of its tile (the epilogue is compiled in).
    auto item = [&](int p, bool refill, bool tile_may_end) {
            // items stay in program order: without the fence the scheduler overlaps the straight-line items of a round and
            // the kernel no longer fits the register budget of two waves per SIMD
            __builtin_amdgcn_sched_barrier(0);
            lds[wr_slot[0]] = stage[p][0];
            lds[wr_slot[1]] = stage[p][1];
            if (kInterleaved && lane < kExtraWords) reinterpret_cast<u32x2*>(lds + 128)[lane] = stage_x[p];
            f32x2 sc = stage_sc[p];
            wave_lds_sync();
            u32x4 a0, a1;
            if (kInterleaved) {
                const unsigned char* bytes = reinterpret_cast<const unsigned char*>(lds);
                const u32x2* p0 = reinterpret_cast<const u32x2*>(bytes + rd_slot[0]);
                const u32x2* p1 = reinterpret_cast<const u32x2*>(bytes + rd_slot[1]);
                const u32x2 lo0 = p0[0], hi0 = p0[1], lo1 = p1[0], hi1 = p1[1];
                a0 = u32x4{lo0.x, lo0.y, hi0.x, hi0.y};
                a1 = u32x4{lo1.x, lo1.y, hi1.x, hi1.y};
                sc = *reinterpret_cast<const f32x2*>(bytes + sc_byte);
            } else {
                a0 = lds[rd_slot[0]];
                a1 = lds[rd_slot[1]];
            }
            wave_lds_sync();
            // Eq. recon_dequant .. recon_rescale: factor s / (alpha sqrt(B)) for this lane's block; zero for a
            // block past the end of the tensor (its codes read as zeros, its scalars are not read at all).
            // Taken before the refill below, so that the slot's old scalars are dead when it is issued.
            float factor = sc.y * __builtin_amdgcn_rcpf(sc.x) * inv_root_b;
            if (kGuarded && tile == partial_tile && my_block >= partial_blocks) factor = 0.0f;
            if (refill) fetch(p);
            f32x4 d[8];
            // The B operand of column tile nt: from the table, or (lean flavour) the running tile, which starts
            // every item as tile 0 and is stepped along the Gray code.  The empty asm keeps the optimiser from
            // recognising the stepped tiles as loop invariants and holding all eight in registers again.
            uint32_t cur[8];
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                cur[w] = hb[0][w];
                if (kGray) asm volatile("" : "+v"(cur[w]));
            }
#pragma unroll
            for (int step = 0; step < 8; ++step) {
                const int nt = kGray ? (step ^ (step >> 1)) : step;           // Gray code: 0 1 3 2 6 7 5 4
                if (!kGray) {
#pragma unroll
                    for (int w = 0; w < 8; ++w) cur[w] = hb[nt][w];
                }
                if (kFormat == 2) {
                    const i32x4 av0 = __builtin_bit_cast(i32x4, a0), av1 = __builtin_bit_cast(i32x4, a1);
                    const i32x4 b0 = {static_cast<int>(cur[0]), static_cast<int>(cur[1]), static_cast<int>(cur[2]), static_cast<int>(cur[3])};
                    const i32x4 b1 = {static_cast<int>(cur[4]), static_cast<int>(cur[5]), static_cast<int>(cur[6]), static_cast<int>(cur[7])};
                    i32x4 di = __builtin_amdgcn_mfma_i32_16x16x64_i8(av0, b0, i32x4{0, 0, 0, 0}, 0, 0, 0);
                    di = __builtin_amdgcn_mfma_i32_16x16x64_i8(av1, b1, di, 0, 0, 0);
                    d[nt] = f32x4{static_cast<float>(di[0]), static_cast<float>(di[1]), static_cast<float>(di[2]), static_cast<float>(di[3])};
                } else {
                    i32x8 av, bv;
                    av[0] = a0.x; av[1] = a0.y; av[2] = a0.z; av[3] = a0.w;
                    av[4] = a1.x; av[5] = a1.y; av[6] = a1.z; av[7] = a1.w;
#pragma unroll
                    for (int w = 0; w < 8; ++w) bv[w] = cur[w];
                    // A operand format: 0 = E4M3 codes, 1 = E5M2 codes; the +-1 entries of B stay E4M3.
                    d[nt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                        av, bv, f32x4{0.0f, 0.0f, 0.0f, 0.0f}, kFormat, 0, 0, 0, 0, 0);
                }
                if (kGray && step < 7) {
                    const int next = (step + 1) ^ ((step + 1) >> 1);
                    const int bit = (nt ^ next) == 1 ? 0 : (nt ^ next) == 2 ? 1 : 2;
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        if (bit == 2 && (w & 1) == 0) continue;
                        cur[w] ^= kSub == 1 ? kFlipMask[bit] : (kFlipMask[bit] & live_half[w >> 2]);
                    }
                }
            }
            // Row r of this lane belongs to the block whose factor quad lane r computed.
            const float f0 = dpp_f32<kDppQuadBcast(0)>(factor), f1 = dpp_f32<kDppQuadBcast(1)>(factor);
            const float f2 = dpp_f32<kDppQuadBcast(2)>(factor), f3 = dpp_f32<kDppQuadBcast(3)>(factor);
            if (i == 0) {
#pragma unroll
                for (int nt = 0; nt < 8; ++nt)
                    sum[nt] = f32x4{d[nt][0] * f0, d[nt][1] * f1, d[nt][2] * f2, d[nt][3] * f3};
            } else {
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    sum[nt][0] = __builtin_fmaf(d[nt][0], f0, sum[nt][0]);
                    sum[nt][1] = __builtin_fmaf(d[nt][1], f1, sum[nt][1]);
                    sum[nt][2] = __builtin_fmaf(d[nt][2], f2, sum[nt][2]);
                    sum[nt][3] = __builtin_fmaf(d[nt][3], f3, sum[nt][3]);
                }
            }
            if (tile_may_end && ++i == k) {
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    if (rotate) units_butterfly<kRB>(sum[nt]);
                }
                const bool whole = !kGuarded || tile != partial_tile;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    u32x4 w;
                    w.x = pack_bf16x2(sum[0][r], sum[1][r]);
                    w.y = pack_bf16x2(sum[2][r], sum[3][r]);
                    w.z = pack_bf16x2(sum[4][r], sum[5][r]);
                    w.w = pack_bf16x2(sum[6][r], sum[7][r]);
                    const int unit = unit_of_row<kRB>(4 * g + r);
                    // this lane holds elements e0 .. e0 + 7 of the tensor: chunk j = n16 of the unit
                    const int64_t e0 = tile * kTileElems + unit * 128 + 8 * n16;
                    if (kRecompress) {
                        if (!whole) {
                            // what lies past the end of the tensor is the zero padding of the compress stage
                            uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                            for (int h = 0; h < 4; ++h) {
                                if (e0 + 2 * h >= n) ww[h] = 0u;
                                else if (e0 + 2 * h + 1 >= n) ww[h] &= 0xFFFFu;
                            }
                            w = u32x4{ww[0], ww[1], ww[2], ww[3]};
                        }
                        const int slot = CompressLane<kRB, kSub>::lds_slot(unit, n16);
                        lds_c[slot] = w.x;
                        lds_c[slot + 4] = w.y;
                        lds_c[slot + 8] = w.z;
                        lds_c[slot + 12] = w.w;
                    } else if (whole || e0 + 8 <= n) {
                        store_stream<true>(&out[e0 >> 3], w);
                    } else {
                        uint16_t* oe = reinterpret_cast<uint16_t*>(out);
                        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                        for (int h = 0; h < 8; ++h)
                            if (e0 + h < n) oe[e0 + h] = static_cast<uint16_t>(ww[h >> 1] >> (16 * (h & 1)));
                    }
                }
                if (kRecompress) {
                    wave_lds_sync();
                    // The compress stage's per-lane constants (16 registers of sign tiles among them) are rebuilt for
                    // every output tile, a few dozen ALU operations, instead of living through the decode loop: with
                    // them resident the kernel needs more than 256 registers and only one wave fits a SIMD.  The
                    // empty asm hides the lane number from the optimiser, which would otherwise hoist the constants
                    // out of the loop again.
                    const CompressLane<kRB, kSub> cl(lane);
                    // (every tile of the unguarded copy is whole: a constant lets its bounds checks fold away)
                    cl.template tile_from_lds<kInterleaved, kFormat, kGeneric>(lds_c, tile, kGuarded ? n_blocks - tile * kBlocksPerTile : INT64_MAX, tau, eps, mode,
                                                                     static_cast<u32x2*>(tab.payload_output(idx)),
                                                                     static_cast<f32x2*>(tab.scales_output(idx)));
                }
                i = 0;
                ++tile;
            }
    };

    // kAligned: k is a multiple of the ring size (k = 4, 8, 12, 16 with a ring of 4).  Every round of kRing items then
    // lies inside one tile, a tile ends only with the last slot of a round, and every round but the last refills all
    // its slots: no condition stands between a load and its use, so the compiler can wait for exactly the slot it
    // needs (vmcnt counts the loads issued since) instead of draining all loads in flight.
    if (kAligned) {
        static_assert(!kAligned || (!kGuarded && kRing > 1), "the aligned loop has no bounds checks");
        const int rounds = n_items / kRing;
        for (int r = 0; r + 1 < rounds; ++r) {
#pragma unroll
            for (int p = 0; p < kRing; ++p) {
                if (p < kRing - 1) { item(p, true, false); ++i; }
                else item(p, true, true);
            }
        }
#pragma unroll
        for (int p = 0; p < kRing; ++p) {
            if (p < kRing - 1) { item(p, false, false); ++i; }
            else item(p, false, true);
        }
        return;
    }
    for (int q0 = 0; q0 < n_items; q0 += kRing) {
#pragma unroll
        for (int p = 0; p < kRing; ++p) {
            const int q = q0 + p;
            if (q >= n_items) break;
            item(p, q + kRing < n_items, true);
        }
    }
}

// kGray: the lean plain decode with one running sign tile; it is held to the register budget of three waves per
// SIMD (168), which it needs a few registers less than it would otherwise take for.
template <int kRB, int kSub, int kRing, bool kInterleaved, bool kRecompress, int kWaves, int kFormat, bool kGeneric, bool kGray = false>
__global__ __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu((kGray && kSub == 1) ? 3 : 2)))
void decompress_sum_mfma_kernel(
    DecodeTable tab, int count, int k, int tiles_per_wave, float tau, float eps, int mode) {
    static_assert((kRB == 1 || kRB == 2 || kRB == 4) && (kSub == 1 || kSub == 2 || kSub == 4) && (kRB == 1 || kSub == 1),
                  "block size must be 32, 64, 128, 256 or 512");
    using Layout = PayloadLayout<128 * kRB / kSub, kInterleaved>;
    // Per wave: one tile of the payload (split layout swizzled, interleaved as it is); the recompress
    // form puts the bf16 tile for the compress stage into the same region afterwards.
    constexpr int kLdsChunks = kRecompress && kCompressLdsDwords / 4 > Layout::kTileChunks ? kCompressLdsDwords / 4 : Layout::kTileChunks;
    __shared__ u32x4 lds_all[kWaves][kLdsChunks];
    const int wave = kWaves == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int idx;
    int64_t group;
    tab.locate(blockIdx.x, count, idx, group);
    const int64_t n = tab.n(idx);
    const int64_t n_tiles = (n + kTileElems - 1) / kTileElems;
    const int64_t tile_begin = (group * kWaves + wave) * tiles_per_wave;
    int64_t tile_end = tile_begin + tiles_per_wave;
    if (tile_end > n_tiles) tile_end = n_tiles;
    if (tile_end <= tile_begin) return;      // a wave past the end (last workgroup of a tensor only)
    // The guarded copy runs in one wave per tensor; it keeps two items in flight instead of kRing so that its extra
    // bookkeeping does not raise the register count of the kernel (which every wave pays for in occupancy).
    // The loop with exact waits (decode_wave, kAligned) is compiled where it pays and fits the register budget of two
    // waves per SIMD: the fused form of the method (measured on MI355X, k = 8: 5-10 % faster at every block size in the
    // split layout, 1-8 % with interleaved records, where a few registers are spilled once per wave outside the loops).
    // The plain sum is faster back to back (2-3 %) but slower inside the benchmark step, where it follows other
    // kernels, so it keeps the generic loop.
    constexpr bool kHasAligned = kRecompress && !kGeneric && kRing > 1;
    if (tile_end == n_tiles && (n % kTileElems) != 0)
        decode_wave<kRB, kSub, 2, kInterleaved, kRecompress, kFormat, kGeneric, kGray, true>(tab, idx, k, n, tile_begin, tile_end, lds_all[wave], tau, eps, mode);
    else if (kHasAligned && k % kRing == 0)
        decode_wave<kRB, kSub, kRing, kInterleaved, kRecompress, kFormat, kGeneric, kGray, false, kHasAligned>(tab, idx, k, n, tile_begin, tile_end, lds_all[wave], tau, eps, mode);
    else
        decode_wave<kRB, kSub, kRing, kInterleaved, kRecompress, kFormat, kGeneric, kGray, false>(tab, idx, k, n, tile_begin, tile_end, lds_all[wave], tau, eps, mode);
}

}  // namespace taco
