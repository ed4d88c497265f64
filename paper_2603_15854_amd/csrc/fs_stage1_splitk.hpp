// Stage 1 of Alg. 1 for the bandwidth-bound decode regime (B <= 16): the whole batch is one
// 16-wide MFMA operand, so the kernel is a stream over W and nothing else matters.
//
// Work split.  A workgroup owns vocabulary tiles t = blockIdx.x, blockIdx.x + gridDim.x, ...
// (128 ids each = 8 row-tiles of 16 ids).  Its NW waves split the contraction dimension:
// wave w owns k-steps [w*kpw, (w+1)*kpw) (one k-step = 32 elements).  The wave's slice of the
// hidden states, in MFMA operand layout, is loaded ONCE into registers (<= KPW*4 VGPRs) and
// reused for every vocabulary row the workgroup ever touches, so the steady-state global traffic
// is W alone, read exactly once, in runs of up to KPW*64 contiguous bytes per row.
//
// Data path of W:  global --128-bit coalesced loads--> registers (the in-flight window, PF
// stages deep) --ds_write_b128--> wave-private LDS stage (XOR-swizzled) --ds_read_b128 in MFMA
// operand layout--> v_mfma_f32_16x16x32_bf16 with A = W rows (M = vocabulary), B = hidden
// (N = batch, zero-padded to 16).  The LDS hop only transposes lanes: a coalesced load gives
// a lane 16 consecutive bytes of ONE row per 64-lane instruction, the MFMA wants lane l to hold
// row l%16.  Stages are wave-private, so the main loop has no barrier.
//
// After the 8 row-tiles of a vocabulary tile each wave parks its fp32 partial tiles in LDS;
// one barrier; then wave w reduces the partials of row-tiles w, w+NW, ... in fixed wave order
// (deterministic), scales by 1/tau, adds Gumbel noise (one Philox block per lane per row-tile:
// a lane holds 4 consecutive vocabulary ids of one batch row), and keeps a running
// (max, id).  A second barrier, a 16-lane merge over waves, and the candidate is written.
#pragma once

#include "fs_common.hpp"
#include "fs_topk_common.hpp"   // wave_top_m

namespace fs {

// KPW: k-steps per wave (register-resident hidden slice); SK: k-steps per LDS stage;
// PF: stage register sets in flight; MAXW: upper bound on waves per workgroup (launch bounds).
// WB: bytes per W element (2 = bf16; 1 = FP8 E4M3 codes, converted to bf16 after the LDS hop).
template <int KPW, int SK, int PF, int MAXW, int WB = 2>
struct SplitKCfg {
    static constexpr int kWB = WB;
    static constexpr int kElemsPerChunk = 16 / WB;            // W elements in one 16-byte load
    static constexpr int kKPW = KPW;
    static constexpr int kSK = SK;
    static constexpr int kPF = PF;
    static constexpr int kMaxWaves = MAXW;
    static constexpr int kStagesPerRowTile = KPW / SK;
    static constexpr int kRowBytes = SK * 32 * WB;            // bytes of one row inside a stage
    static constexpr int kStageBytes = 16 * kRowBytes;        // 16 rows
    static constexpr int kLanesPerRow = kRowBytes / 16;       // lanes that cover one row
    static constexpr int kRowsPerInstr = kWave / kLanesPerRow;
    static constexpr int kInstrPerStage = 16 / kRowsPerInstr;
    static_assert(KPW % SK == 0, "stage must divide the wave's k-range");
    static_assert(kStagesPerRowTile % PF == 0 && PF <= kStagesPerRowTile, "static register sets");
    static_assert(kLanesPerRow >= 16 && kLanesPerRow <= 64, "swizzle needs >= 16 chunks per row");

    // LDS bytes for nw waves: stages + partial tiles [8][nw][64] float4 + wave candidates.
    static constexpr size_t lds_bytes(int nw)
    {
        return (size_t)nw * kStageBytes + (size_t)8 * nw * 1024 + (size_t)nw * 16 * 8 * 2;
    }
    // per-tile candidate epilogue (TOPK): the keys of the tile, [16 batch columns][128 + 4] floats, behind the rest
    static constexpr int kKeyStride = kVocabTile + 4;
    static constexpr size_t lds_bytes_topk(int nw) { return lds_bytes(nw) + (size_t)16 * kKeyStride * 4; }
};

// End of one vocabulary tile in the split-K kernels.  Every wave has stored its eight partial
// 16 x 16 tiles (rows 16 r8 .. 16 r8 + 15 of the tile, this wave's slice of K) in `partial`
// ([8][nw][64] f32x4).  Two barriers: after the first the partials are summed in a fixed wave
// order (deterministic), scaled if the weights carry per-row scales, optionally stored as logits,
// and run through the sampling epilogue; after the second one lane per batch column merges the
// waves' candidates (and log-sum-exp states) and writes the tile's entry of the candidate buffer.
// TOPK (Section "Top-k, Nucleus Sampling, and Masking", per-tile candidates): the summed keys go to
// `keys` ([16][128 + 4] floats) instead, and after the second barrier the waves find the p.topk_k <= 8
// best of each batch column's 128 keys, four columns at a time (wave_top_m), and write them packed.
template <bool FULL, bool ROW_SCALE, bool TOPK = false>
__device__ __forceinline__ void splitk_finish_tile(const Stage1Params& p, const RowEpi& repi, const f32x4* partial,
                                                   float2* wave_cand, float2* wave_lse, int nw, int wave,
                                                   int lane, int tile, float* keys = nullptr)
{
    static_assert(!TOPK || (!FULL && !ROW_SCALE), "per-tile candidates: bf16 weights, plain transform");
    constexpr int KSTRIDE = kVocabTile + 4;
    const int n = lane & 15, g = lane >> 4;
    const int B = p.B, V = p.V, T = p.T;
    const int tile_row0 = tile * kVocabTile;
    __syncthreads();   // all partial tiles of this vocabulary tile are in LDS
    float best = -__builtin_inff();
    int best_id = -1;
    float lmax = -__builtin_inff(), lsum = 0.0f;
    for (int r8 = wave; r8 < 8; r8 += nw) {
        f32x4 y = partial[(r8 * nw) * 64 + lane];
        for (int w = 1; w < nw; ++w) y += partial[(r8 * nw + w) * 64 + lane];
        const int v0 = tile_row0 + r8 * 16 + 4 * g;   // local vocabulary row of y[0]
        if constexpr (ROW_SCALE) {   // per-row scale of the FP8 weights
            if (p.w_scale && v0 < V) {
#pragma unroll
                for (int j = 0; j < 4; ++j) y[j] *= p.w_scale[v0 + j < V ? v0 + j : V - 1];
            }
        }
        if (v0 < V && n < B) {
            if (p.logits) {
                float* dst = p.logits + (size_t)n * V + v0;
                if (v0 + 3 < V && (V & 3) == 0) {
                    *reinterpret_cast<f32x4*>(dst) = y;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (v0 + j < V) dst[j] = y[j];
                }
            }
            if (p.cand_val) epilogue_quad<FULL>(p, repi, y, v0, V, best, best_id, lmax, lsum);
        }
        if constexpr (TOPK) {
            float gn[4] = {0.f, 0.f, 0.f, 0.f};
            if (p.topk_mode == kTopkGumbel)
                gumbel4(repi.seed, repi.row_word, (uint32_t)(p.vocab_offset + v0), gn, (p.epi_flags & kEpiExactLog) != 0u);
            f32x4 kq;
#pragma unroll
            for (int j = 0; j < 4; ++j) kq[j] = key_sanitize(fmaf(y[j], repi.inv_tau, gn[j]));
            *reinterpret_cast<f32x4*>(keys + n * KSTRIDE + r8 * 16 + 4 * g) = kq;
        }
    }
    if constexpr (TOPK) {
        __syncthreads();   // keys of the tile complete; partial buffer free again
        constexpr int U = 4;
        const int kt = p.topk_k;
        for (int ub = wave * U; ub < 16; ub += nw * U) {      // unit = batch column
            // every address is inside the key array: read first, all eight in flight, then mask
            float f0[U], f1[U];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                f0[q] = keys[(ub + q) * KSTRIDE + lane];
                f1[q] = keys[(ub + q) * KSTRIDE + 64 + lane];
            }
            uint32_t k0[U], k1[U];
            int32_t id0[U];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const int e0 = tile_row0 + lane, e1 = e0 + 64;
                const uint32_t o0 = topk_ordered(f0[q]), o1 = topk_ordered(f1[q]);
                k0[q] = e0 < V ? o0 : 0u;
                k1[q] = e1 < V ? o1 : 0u;
                id0[q] = p.vocab_offset + tile_row0;
            }
            uint64_t res[U];
            wave_top_m<U>(k0, k1, id0, kt, lane, res);
#pragma unroll
            for (int q = 0; q < U; ++q)
                if (ub + q < B && lane < kt) p.topk_out[((size_t)(ub + q) * T + tile) * (size_t)kt + lane] = res[q];
        }
        return;
    }
    cand_reduce_lane_groups(best, best_id);
    if (g == 0) wave_cand[wave * 16 + n] = make_float2(best, __int_as_float(best_id));
    if constexpr (FULL) {
        lse_reduce_lane_groups(lmax, lsum);
        if (g == 0) wave_lse[wave * 16 + n] = make_float2(lmax, lsum);
    }
    __syncthreads();   // wave candidates visible; partial buffer free again
    if (wave == 0 && lane < 16 && n < B && p.cand_val) {
        float bv = -__builtin_inff();
        int bi = -1;
        for (int w = 0; w < nw; ++w) {
            const float2 c = wave_cand[w * 16 + n];
            cand_merge(bv, bi, c.x, __float_as_int(c.y));
        }
        p.cand_val[(size_t)n * T + tile] = bv;
        p.cand_idx[(size_t)n * T + tile] = bi;
        if constexpr (FULL) {
            if (p.lse_max) {
                float m = -__builtin_inff(), sacc = 0.0f;
                for (int w = 0; w < nw; ++w) {
                    const float2 c = wave_lse[w * 16 + n];
                    lse_merge(m, sacc, c.x, c.y);
                }
                p.lse_max[(size_t)n * T + tile] = m;
                p.lse_sum[(size_t)n * T + tile] = sacc;
            }
        }
    }
}

template <class Cfg, bool FULL = false, bool TOPK = false>
__global__ void __launch_bounds__(Cfg::kMaxWaves * kWave)
stage1_splitk_kernel(const Stage1Params p, const int nw, const int kpw)
{
    constexpr int KPW = Cfg::kKPW, SK = Cfg::kSK, PF = Cfg::kPF;
    constexpr int NSTG = Cfg::kStagesPerRowTile;
    constexpr int NI = Cfg::kInstrPerStage;
    constexpr int LPR = Cfg::kLanesPerRow;
    constexpr int RPI = Cfg::kRowsPerInstr;
    constexpr int ROWB = Cfg::kRowBytes;
    constexpr int WB = Cfg::kWB, EPC = Cfg::kElemsPerChunk;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15;   // batch column of the MFMA B operand / of the output tile
    const int g = lane >> 4;   // k-group of the operands, row-group of the output tile
    const int B = p.B, D = p.D, V = p.V;

    // this wave's slice of the contraction dimension
    const int ksteps_total = (D + 31) >> 5;
    const int ks0 = wave * kpw;
    int nks = ksteps_total - ks0;
    nks = nks < 0 ? 0 : (nks > kpw ? kpw : nks);
    const int kbeg = ks0 * 32;
    int kend = kbeg + nks * 32;
    kend = kend > D ? D : kend;

    unsigned char* stage = smem + (size_t)wave * Cfg::kStageBytes;
    f32x4* partial = reinterpret_cast<f32x4*>(smem + (size_t)nw * Cfg::kStageBytes);
    float2* wave_cand = reinterpret_cast<float2*>(smem + (size_t)nw * Cfg::kStageBytes +
                                                  (size_t)8 * nw * 1024);
    float2* wave_lse = wave_cand + nw * 16;
    float* keys = reinterpret_cast<float*>(smem + Cfg::lds_bytes(nw));      // TOPK only

    // per-row epilogue constants (logits-only launches pass no temperatures)
    RowEpi repi = {1.0f, p.seed, (uint32_t)(uint64_t)(p.row_offset + n), nullptr};
    if (n < B && (p.cand_val || TOPK)) repi = make_row_epi<FULL>(p, n);

    // row-tiles of this workgroup, in processing order
    const int T = p.T;
    const int ntiles = ((int)blockIdx.x < T) ? (T - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    const int nrt = ntiles * 8;

    // stage load geometry of this lane
    const int ld_row = lane / LPR;           // row within one load instruction
    const int ld_chunk = lane % LPR;         // 16-byte chunk within the row
    const int ld_k = kbeg + ld_chunk * EPC;  // + h * SK * 32

    uint4 wreg[PF][NI];

    // The loads of the main loop are unconditional (addresses clamped into the matrix) so that
    // the compiler can count them and wait for exactly the stage it needs (s_waitcnt vmcnt(N))
    // instead of draining everything in flight.  Rows past V re-read row V-1 and only feed
    // logits the epilogue masks; the prefetch that runs past the workgroup's last row-tile
    // re-reads rows 0..15 (cache hits); chunks past the wave's k-range are zeroed when the
    // stage is written to LDS.
    auto row_base = [&](int rtl) -> int {
        if (rtl >= nrt) return 0;
        return ((int)blockIdx.x + (rtl >> 3) * (int)gridDim.x) * kVocabTile + (rtl & 7) * 16;
    };
    auto issue_loads = [&](uint4 (&dst)[NI], int rtl, int h) {
        const int rb = row_base(rtl);
        int k = ld_k + h * (SK * 32);
        k = k < kend - EPC ? k : kend - EPC;
        const unsigned char* src = reinterpret_cast<const unsigned char*>(p.W) + (size_t)k * WB;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            int row = rb + j * RPI + ld_row;
            row = row < V - 1 ? row : V - 1;
            dst[j] = ld_global_16B_stream(reinterpret_cast<const uint16_t*>(src + (size_t)row * D * WB));
        }
    };

    // LDS addresses: a stage is [16 rows][ROWB bytes]; 16-byte chunk c of row r sits in slot
    // c ^ (r & 15), which makes both the row-contiguous writes and the 16-rows-per-pass MFMA
    // operand reads bank-conflict free.  Row r = j*RPI + ld_row of load j; the two terms occupy
    // disjoint bits, so the offset is (st_base ^ const_j) + const_j'.
    const int st_base = ld_row * ROWB + ((ld_chunk ^ ld_row) << 4);
    auto st_off = [&](int j) -> int { return (st_base ^ (((j * RPI) & 15) << 4)) + j * RPI * ROWB; };
    const int rd_row_off = n * ROWB;   // A-operand row of this lane is lane & 15

    // start the W stream first: it does not depend on the hidden states
#pragma unroll
    for (int h = 0; h < PF; ++h) issue_loads(wreg[h], 0, h);

    // hidden slice in B-operand layout: lane (n, g) holds H[n, k .. k+8), k = kbeg + 32 s + 8 g
    bf16x8 hreg[KPW];
#pragma unroll
    for (int s = 0; s < KPW; ++s) {
        const int k = kbeg + s * 32 + g * 8;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (n < B && s < nks && k < D) v = ld_global_16B(p.H + (size_t)n * D + k);
        hreg[s] = __builtin_bit_cast(bf16x8, v);
    }


    for (int rtl = 0; rtl < nrt; ++rtl) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int h = 0; h < NSTG; ++h) {
            const int set = h % PF;
            const bool active = h * SK < nks;   // wave-uniform
            if (active) {
                const bool in_range = ld_k + h * (SK * 32) < kend;   // false only in a ragged K tail
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    uint4 v = wreg[set][j];
                    if (!in_range) v = make_uint4(0u, 0u, 0u, 0u);
                    *reinterpret_cast<uint4*>(stage + st_off(j)) = v;
                }
            }
            // refill the register set with the stage PF ahead in the stream
            if (h + PF < NSTG) issue_loads(wreg[set], rtl, h + PF);
            else               issue_loads(wreg[set], rtl + 1, h + PF - NSTG);
            if (active) {
#pragma unroll
                for (int s = 0; s < SK; ++s) {
                    bf16x8 a;
                    if constexpr (WB == 2) {
                        const int c = 4 * s + g;
                        a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(stage + rd_row_off + ((c ^ n) << 4)));
                    } else {   // 8 one-byte elements: half of chunk 2 s + g / 2
                        // slot (c ^ n) with c = 2 s + g / 2: the lane's part of the XOR is one register and the
                        // XOR is redone at every read; kept as SK loop-invariant offsets it cost scratch spills
                        uint32_t gn = (uint32_t)((g >> 1) ^ n) << 4;
                        asm volatile("" : "+v"(gn));
                        const uint2 q = *reinterpret_cast<const uint2*>(stage + rd_row_off + (((uint32_t)s << 5) ^ gn) + ((g & 1) << 3));
                        a = e4m3x8_to_bf16x8(q.x, q.y);
                    }
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, hreg[h * SK + s], acc, 0, 0, 0);
                }
            }
        }
        const int rt = rtl & 7;
        partial[(rt * nw + wave) * 64 + lane] = acc;

        if (rt == 7) {
            const int tile = (int)blockIdx.x + (rtl >> 3) * (int)gridDim.x;
            splitk_finish_tile<FULL, WB == 1, TOPK>(p, repi, partial, wave_cand, wave_lse, nw, wave, lane, tile, keys);
        }
    }
}

}  // namespace fs
