// Stage 1 of Alg. 1 for any batch size: a workgroup of 4 waves computes one
// (128 vocabulary ids) x (16*NB batch rows) tile of logits with an LDS-tiled K loop, then runs
// the sampling epilogue on the accumulators.
//
// Orientation: MFMA A operand = W rows (M = vocabulary), B operand = hidden rows (N = batch).
// With v_mfma_f32_16x16x32_bf16 a lane then holds, per 16x16 output block, 4 consecutive
// vocabulary ids of ONE batch row -- exactly the 4 ids one Philox block covers.
//
// K loop: 64 contraction elements per step; W tile [128][64] and hidden tile [16*NB][64] are
// fetched with 128-bit loads (8 lanes cover one 128-byte row segment), parked in registers while
// the previous step computes, then written to the other LDS buffer: one barrier per step.
// LDS rows are 128 bytes; chunk c of row r sits in slot c ^ ((r & 7) ^ ((r >> 3) & 1)), which is
// conflict free for the row-major writes and for the 16-rows-per-pass operand reads.
//
// Wave w owns vocabulary rows [32 w, 32 w + 32) of the tile (two 16-row blocks) and all NB batch
// blocks: 2*NB accumulators of 4 VGPRs.
#pragma once

#include "fs_common.hpp"

namespace fs {

template <int NB>
struct TiledCfg {
    static constexpr int kNB = NB;
    static constexpr int kBatchTile = 16 * NB;
    static constexpr int kKS = 64;                       // contraction elements per step
    static constexpr int kRowBytes = kKS * 2;            // 128
    static constexpr int kWBytes = kVocabTile * kRowBytes;
    static constexpr int kHBytes = kBatchTile * kRowBytes;
    static constexpr int kWLoads = kVocabTile * 8 / 256;            // 16-byte loads per thread
    static constexpr int kHLoads = (kBatchTile * 8 + 255) / 256;
    static constexpr size_t lds_bytes() { return 2 * (size_t)(kWBytes + kHBytes) + 4 * kBatchTile * 8; }
};

// Byte offset of 16-byte chunk c (0..7) of row r inside an LDS tile of 128-byte rows.
// Rows are laid out in blocks of 16 (2 KB): rows r and r + 8 of a block share a 256-byte line
// (row r & 7 picks the line, (r >> 3) & 1 the 128-byte half) and the chunk index is XORed with
// r & 7.  An MFMA operand read (16 lanes = the 16 rows of a block, one chunk) then touches the 16
// distinct 16-byte bank groups as  lane -> group 8 (r >> 3) + (c ^ (r & 7)).  Measured on gfx950
// (ds_read_b128 at two waves per SIMD): this form runs at the rate of a linear read, while the
// layout r * 128 + ((c ^ (r & 7) ^ (r >> 3 & 1)) << 4) -- also 16 distinct groups per 16 lanes --
// takes 25 % longer per instruction and counts four bank-conflict cycles per read in
// SQ_LDS_BANK_CONFLICT.  Row-contiguous ds_write_b128 parking showed no sensitivity to either.
__device__ __forceinline__ int tile_off(int r, int c)
{
    return ((r >> 4) << 11) + ((r & 7) << 8) + (((r >> 3) & 1) << 7) + ((c ^ (r & 7)) << 4);
}

template <int NB>
__global__ void __launch_bounds__(256)
stage1_tiled_kernel(const Stage1Params p)
{
    using Cfg = TiledCfg<NB>;
    constexpr int BT = Cfg::kBatchTile;
    constexpr int KS = Cfg::kKS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int kBufBytes = Cfg::kWBytes + Cfg::kHBytes;   // one K-step buffer: W tile then H tile
    auto w_lds = [&](int buf) { return smem + buf * kBufBytes; };
    auto h_lds = [&](int buf) { return smem + buf * kBufBytes + Cfg::kWBytes; };
    float2* wave_cand = reinterpret_cast<float2*>(smem + 2 * (Cfg::kWBytes + Cfg::kHBytes));

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;
    const int B = p.B, D = p.D, V = p.V, T = p.T;

    // blockIdx.x enumerates (vocabulary tile, batch tile) with the batch tile fastest, so the
    // workgroups that share a W tile are dispatched back to back.
    const int nbt = (B + BT - 1) / BT;
    const int tile = (int)blockIdx.x / nbt;
    const int b0 = ((int)blockIdx.x % nbt) * BT;
    const int tile_row0 = tile * kVocabTile;

    // global -> register staging geometry
    const int ld_chunk = tid & 7;
    const int ld_row = tid >> 3;   // 0..31
    uint4 wst[Cfg::kWLoads];
    uint4 hst[Cfg::kHLoads];

    auto fetch = [&](int k0) {
        const int k = k0 + ld_chunk * 8;
#pragma unroll
        for (int i = 0; i < Cfg::kWLoads; ++i) {
            const int row = tile_row0 + ld_row + 32 * i;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (row < V && k < D) v = ld_global_16B_stream(p.W + (size_t)row * D + k);
            wst[i] = v;
        }
#pragma unroll
        for (int i = 0; i < Cfg::kHLoads; ++i) {
            const int r = ld_row + 32 * i;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (r < BT && b0 + r < B && k < D) v = ld_global_16B(p.H + (size_t)(b0 + r) * D + k);
            hst[i] = v;
        }
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int i = 0; i < Cfg::kWLoads; ++i) {
            const int r = ld_row + 32 * i;
            *reinterpret_cast<uint4*>(w_lds(buf) + tile_off(r, ld_chunk)) = wst[i];
        }
#pragma unroll
        for (int i = 0; i < Cfg::kHLoads; ++i) {
            const int r = ld_row + 32 * i;
            if (r < BT)
                *reinterpret_cast<uint4*>(h_lds(buf) + tile_off(r, ld_chunk)) = hst[i];
        }
    };

    f32x4 acc[2][NB];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[i][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nk = (D + KS - 1) / KS;
    fetch(0);
    park(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) fetch((kt + 1) * KS);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int c = 4 * s + g;
            bf16x8 a[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = wave * 32 + i * 16 + n;
                a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                                                      w_lds(buf) + tile_off(r, c)));
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int r = nb * 16 + n;
                const bf16x8 b = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                                                                h_lds(buf) + tile_off(r, c)));
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b, acc[i][nb], 0, 0, 0);
            }
        }
        if (kt + 1 < nk) park(buf ^ 1);
        __syncthreads();
    }

    // epilogue: acc[i][nb][j] is the logit of vocabulary row tile_row0 + 32 wave + 16 i + 4 g + j
    // and batch row b0 + 16 nb + n
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int b = b0 + nb * 16 + n;
        float best = -__builtin_inff();
        int best_id = -1;
        if (b < B) {
            RowEpi repi = {1.0f, p.seed, (uint32_t)(uint64_t)(p.row_offset + b), nullptr};
            if (p.cand_val) repi = make_row_epi<false>(p, b);
            float unused_m = 0.0f, unused_s = 0.0f;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const f32x4 y = acc[i][nb];
                const int v0 = tile_row0 + wave * 32 + i * 16 + 4 * g;
                if (v0 < V) {
                    if (p.logits) {
                        float* dst = p.logits + (size_t)b * V + v0;
                        if (v0 + 3 < V && (V & 3) == 0) {
                            *reinterpret_cast<f32x4*>(dst) = y;
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (v0 + j < V) dst[j] = y[j];
                        }
                    }
                    if (p.cand_val) epilogue_quad<false>(p, repi, y, v0, V, best, best_id, unused_m, unused_s);
                }
            }
        }
        cand_reduce_lane_groups(best, best_id);
        if (g == 0) wave_cand[wave * BT + nb * 16 + n] = make_float2(best, __int_as_float(best_id));
    }
    __syncthreads();
    if (p.cand_val && tid < BT && b0 + tid < B) {
        float bv = -__builtin_inff();
        int bi = -1;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float2 c = wave_cand[w * BT + tid];
            cand_merge(bv, bi, c.x, __float_as_int(c.y));
        }
        p.cand_val[(size_t)(b0 + tid) * T + tile] = bv;
        p.cand_idx[(size_t)(b0 + tid) * T + tile] = bi;
    }
}

}  // namespace fs
