// Matrix-core kernels for block size B = 128 on gfx950.
//
// The Hadamard rotation of Algorithm 1 is the dense product  W[16 blocks, 128] =
// X[16 blocks, 128] * H_128, run on MFMA: both operands are exact in the input format
// (bf16 data or E4M3 codes, +-1 entries), products are exact and accumulation is fp32.
// Everything else (sum of squares, max|W|, the two block scalars, conversion) rides along
// in the same pass, so each byte of the tensor crosses HBM once.
//
// Work unit: one TILE = 16 consecutive blocks = 2048 elements, handled by one 64-lane
// wavefront (one workgroup = one wave, so the workgroup barrier is free).
//
//   global -> registers   coalesced 16-byte loads, 1 KiB per wave instruction
//   registers -> LDS      the tile, stored block-row by block-row with an XOR swizzle
//   LDS -> A operand      lane (i = lane%16, g = lane/16) reads 16-byte chunks of block
//                         row i; the swizzle makes 16 lanes hit 16 different bank groups
//   MFMA                  D[i][n] += sum_k A[i][k] B[k][n],  B = tiles of H_128 in registers
//   D -> HBM              lane (n = lane%16, g), register r holds row 4g+r, column n; the
//                         row -> block and column -> position maps below are chosen so that
//                         each lane owns 8 consecutive outputs and each store instruction
//                         of the wave covers one contiguous span.
//
// Index maps (all bijections; correctness only needs A and B to agree on them):
//   block of MFMA row i          beta(i) = 4 (i % 4) + i / 4      (tile-local block index)
//   output position of column n  p(nt, n) = 8 n + nt              (nt = which of 8 MFMA column tiles)
//   element of A slot            compress: e(c, g, t) = 8 (4 c + g) + t,  c = MFMA step 0..3, t = 0..7
//                                decode:   e(m, g, b) = 64 m + 16 g + b,  m = 0..1, b = 0..15
//   B entry                      H[e][p] = (-1)^popcount(e & p)
#pragma once

#include "butterfly_kernels.h"  // PayloadTable
#include "device_util.h"

namespace taco {

constexpr int kTileBlocks = 16;
constexpr int kTileElems = kTileBlocks * 128;

__device__ __forceinline__ int tile_block_of_row(int i) { return 4 * (i & 3) + (i >> 2); }

// ------------------------------------------------------------------------------------------
// compress
// ------------------------------------------------------------------------------------------

// x: n_tiles * 2048 bf16 (as 16-byte words); payload: n_tiles * 2048 codes (as 8-byte
// words); scales: n_tiles * 16 records {alpha, s}.
__global__ __launch_bounds__(64) void compress_b128_mfma_kernel(
    const u32x4* __restrict__ x, int64_t n_tiles, float tau, float eps,
    u32x2* __restrict__ payload, float2* __restrict__ scales) {
    __shared__ u32x4 lds[256];   // one tile: 16 block rows x 16 chunks of 16 bytes
    const int lane = threadIdx.x;
    const int g = lane >> 4;
    const int n16 = lane & 15;

    // B operand: the 32 tiles (c, nt) of H_128, 8 bf16 (+-1) per lane each.
    // Sign of entry (c, g, t) x (nt, n16): parity((4c+g) & n16) ^ parity(t & nt).
    uint32_t hb[4][8][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t lane_sign = parity32((4 * c + g) & n16) ? 0x80008000u : 0u;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t lo = __builtin_popcount((2 * u) & nt) & 1;
                const uint32_t hi = __builtin_popcount((2 * u + 1) & nt) & 1;
                hb[c][nt][u] = (0x3F803F80u ^ (lo << 15) ^ (hi << 31)) ^ lane_sign;
            }
        }
    }

    // LDS slots.  Writer: load c covers tile blocks 4c .. 4c+3, this lane holds chunk n16 of
    // block 4c+g.  Reader: MFMA row i = n16 is block beta(i); step c wants chunk 4c+g.
    int wr_slot[4], rd_slot[4];
    const int rd_block = tile_block_of_row(n16);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int wb = 4 * c + g;
        wr_slot[c] = wb * 16 + (n16 ^ wb);
        rd_slot[c] = rd_block * 16 + ((4 * c + g) ^ rd_block);
    }
    // Lane that ends up holding the sum of squares of the block this lane finishes:
    // row 4g + (n16 % 4) of the A layout, i.e. any lane whose lane%16 equals that row.
    const int energy_src = 4 * g + (n16 & 3);

    int64_t tile = blockIdx.x;
    if (tile >= n_tiles) return;
    u32x4 stage[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) stage[c] = x[tile * 256 + 64 * c + lane];
    for (; tile < n_tiles; tile += gridDim.x) {
#pragma unroll
        for (int c = 0; c < 4; ++c) lds[wr_slot[c]] = stage[c];
        __syncthreads();
        u32x4 a[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) a[c] = lds[rd_slot[c]];
        __syncthreads();
        // Prefetch the next tile of this wave (the last iteration re-reads a valid tile).
        const int64_t next = (tile + gridDim.x < n_tiles) ? tile + gridDim.x : n_tiles - 1;
#pragma unroll
        for (int c = 0; c < 4; ++c) stage[c] = x[next * 256 + 64 * c + lane];

        // Sum of squares of this lane's 32 values (Eq. ash_sigma), two chains.
        float e0 = 0.0f, e1 = 0.0f;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t w0 = a[c][0], w1 = a[c][1], w2 = a[c][2], w3 = a[c][3];
            e0 = dot2_self_bf16(w0, e0);
            e1 = dot2_self_bf16(w1, e1);
            e0 = dot2_self_bf16(w2, e0);
            e1 = dot2_self_bf16(w3, e1);
        }
        float energy = e0 + e1;
        energy += __shfl_xor(energy, 16, 64);
        energy += __shfl_xor(energy, 32, 64);     // every lane (i, *) now has the sum for row i
        energy = __shfl(energy, energy_src, 64);  // ... and this lane the sum for its own block

        // W = X H_128 (unnormalised rotation, Eq. ash_rotation without alpha / sqrt(B)).
        f32x4 acc[8];
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[nt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bf16x8 av = __builtin_bit_cast(bf16x8, a[c]);
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) {
                const u32x4 hw = {hb[c][nt][0], hb[c][nt][1], hb[c][nt][2], hb[c][nt][3]};
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, hw), acc[nt], 0, 0, 0);
            }
        }

        // max|W| per block row (16 lanes of a row share rows 4g .. 4g+3).
        float wmax[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float m = 0.0f;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) m = fmaxf(m, __builtin_fabsf(acc[nt][r]));
            wmax[r] = row16_allreduce_max(m);
        }
        // Block scalars, computed by the lane for row r = n16 % 4 only.
        const int my_r = n16 & 3;
        const float my_wmax = my_r == 0 ? wmax[0] : my_r == 1 ? wmax[1] : my_r == 2 ? wmax[2] : wmax[3];
        const float alpha = tau * __builtin_amdgcn_rsqf(energy * (1.0f / 128.0f) + eps);   // Eq. ash_sigma, ash_alpha
        const float s = (my_wmax * alpha) * (0.08838834764831845f / kQmax);               // Eq. post_scale, 1/sqrt(128)
        const float to_code = my_wmax > 0.0f ? kQmax * __builtin_amdgcn_rcpf(my_wmax) : 0.0f;
        if (n16 < 4) scales[tile * 16 + 4 * n16 + g] = make_float2(alpha, s);

        // Eq. quantization: codes of Z / s = W * (Q_max / max|W|); 8 consecutive codes per lane and row.
#define TACO_STORE_ROW(R)                                                                      \
        {                                                                                      \
            const float f = dpp_f32<kDppQuadBcast(R)>(to_code);                                \
            u32x2 w;                                                                           \
            w.x = pack_e4m3x4(acc[0][R] * f, acc[1][R] * f, acc[2][R] * f, acc[3][R] * f);     \
            w.y = pack_e4m3x4(acc[4][R] * f, acc[5][R] * f, acc[6][R] * f, acc[7][R] * f);     \
            payload[tile * 256 + 64 * R + lane] = w;                                           \
        }
        TACO_STORE_ROW(0)
        TACO_STORE_ROW(1)
        TACO_STORE_ROW(2)
        TACO_STORE_ROW(3)
#undef TACO_STORE_ROW
    }
}

// ------------------------------------------------------------------------------------------
// decompress / decompress_sum
// ------------------------------------------------------------------------------------------

// out = bf16( sum_i  H (codes_i) * s_i / (alpha_i sqrt(128)) ), fp32 accumulation, i ascending.
// payloads: n_tiles * 2048 codes each; scales: n_tiles * 16 records; out: n_tiles * 2048 bf16.
__global__ __launch_bounds__(64) void decompress_sum_b128_mfma_kernel(
    PayloadTable tab, int k, int64_t n_tiles, u32x4* __restrict__ out) {
    __shared__ u32x4 lds[128];   // one tile of codes: 16 block rows x 8 chunks of 16 bytes
    const int lane = threadIdx.x;
    const int g = lane >> 4;
    const int n16 = lane & 15;

    // B operand: 8 column tiles of H_128 in E4M3 (+1 = 0x38, -1 = 0xB8), 32 bytes per lane each.
    // Slot (m, b) of lane (n16, g) is element e = 64 m + 16 g + b against position p = 8 n16 + nt:
    // sign = parity(b%8 & nt) ^ (b/8 & n16) ^ parity(g & (n16 >> 1)) ^ (m & n16 >> 3).
    uint32_t hb[8][8];
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        const int m = d >> 2;
        const int b_hi = (d & 3) >> 1;    // bit 3 of b for the 4 bytes of dword d
        const int sgn = (b_hi & n16) ^ parity32(g & (n16 >> 1) & 3) ^ (m & (n16 >> 3));
        const uint32_t lane_sign = (sgn & 1) ? 0x80808080u : 0u;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            uint32_t w = 0x38383838u;
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                const int b_lo = (4 * (d & 3) + bb) & 7;
                w ^= static_cast<uint32_t>(__builtin_popcount(b_lo & nt) & 1) << (8 * bb + 7);
            }
            hb[nt][d] = w ^ lane_sign;
        }
    }

    // LDS slots (16-byte units, 8 per block row).  Writer: load m covers tile blocks 8m .. 8m+7,
    // this lane holds chunk lane%8 of block 8m + lane/8.  Reader: row i = n16 is block beta(i),
    // half m wants chunk 4m + g.
    int wr_slot[2], rd_slot[2];
    const int rd_block = tile_block_of_row(n16);
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int wb = 8 * m + (lane >> 3);
        wr_slot[m] = wb * 8 + ((lane & 7) ^ ((wb >> 1) & 7));
        rd_slot[m] = rd_block * 8 + ((4 * m + g) ^ ((rd_block >> 1) & 7));
    }
    const int my_block = 4 * (n16 & 3) + g;   // block whose factor this lane computes

    const int64_t total = n_tiles * k;
    int64_t item = static_cast<int64_t>(blockIdx.x) * k;   // (tile, payload) pairs, payload fastest
    const int64_t item_stride = static_cast<int64_t>(gridDim.x) * k;
    if (item >= total) return;
    u32x4 stage[2];
    float2 stage_sc;
    {
        const u32x4* src = static_cast<const u32x4*>(tab.payload[0]);
        stage[0] = src[(item / k) * 128 + lane];
        stage[1] = src[(item / k) * 128 + 64 + lane];
        stage_sc = static_cast<const float2*>(tab.scales[0])[(item / k) * 16 + my_block];
    }
    for (; item < total; item += item_stride) {
        const int64_t tile = item / k;
        f32x4 sum[8];
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) sum[nt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        for (int i = 0; i < k; ++i) {
            lds[wr_slot[0]] = stage[0];
            lds[wr_slot[1]] = stage[1];
            const float2 sc = stage_sc;
            __syncthreads();
            const u32x4 a0 = lds[rd_slot[0]];
            const u32x4 a1 = lds[rd_slot[1]];
            __syncthreads();
            // Prefetch the next (tile, payload) pair (the very last one re-reads a valid tile).
            {
                int ni = i + 1;
                int64_t nt_tile = tile;
                if (ni == k) { ni = 0; nt_tile = tile + gridDim.x; }
                if (nt_tile >= n_tiles) nt_tile = n_tiles - 1;
                const u32x4* src = static_cast<const u32x4*>(tab.payload[ni]);
                stage[0] = src[nt_tile * 128 + lane];
                stage[1] = src[nt_tile * 128 + 64 + lane];
                stage_sc = static_cast<const float2*>(tab.scales[ni])[nt_tile * 16 + my_block];
            }
            i32x8 av;
            av[0] = a0.x; av[1] = a0.y; av[2] = a0.z; av[3] = a0.w;
            av[4] = a1.x; av[5] = a1.y; av[6] = a1.z; av[7] = a1.w;
            // Eq. recon_dequant .. recon_rescale: factor s / (alpha sqrt(B)) for this lane's block.
            const float factor = sc.y * __builtin_amdgcn_rcpf(sc.x) * 0.08838834764831845f;
            f32x4 d[8];
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) {
                i32x8 bv;
#pragma unroll
                for (int q = 0; q < 8; ++q) bv[q] = hb[nt][q];
                d[nt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                    av, bv, f32x4{0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0, 0, 0, 0);
            }
#define TACO_ACC_ROW(R)                                                                        \
            {                                                                                  \
                const float f = dpp_f32<kDppQuadBcast(R)>(factor);                             \
                _Pragma("unroll") for (int nt = 0; nt < 8; ++nt)                               \
                    sum[nt][R] = __builtin_fmaf(d[nt][R], f, sum[nt][R]);                      \
            }
            TACO_ACC_ROW(0)
            TACO_ACC_ROW(1)
            TACO_ACC_ROW(2)
            TACO_ACC_ROW(3)
#undef TACO_ACC_ROW
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            u32x4 w;
            w.x = pack_bf16x2(sum[0][r], sum[1][r]);
            w.y = pack_bf16x2(sum[2][r], sum[3][r]);
            w.z = pack_bf16x2(sum[4][r], sum[5][r]);
            w.w = pack_bf16x2(sum[6][r], sum[7][r]);
            out[tile * 256 + 64 * r + lane] = w;
        }
    }
}

}  // namespace taco
