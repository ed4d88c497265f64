// Stage 1 of Alg. 1 for large batches (B > 128): 256 vocabulary ids x BT batch rows per workgroup,
// four waves of 128 x BT/2 each, global memory -> LDS by direct loads (no staging registers),
// three W stages and two hidden stages in flight.
//
// Why this shape.  At B >= 128 the tiled kernel of fs_stage1_tiled2.hpp is bound by LDS bandwidth
// and by how many bytes it keeps in flight, not by HBM or the MFMA pipe: with eight waves of
// 64 x 128 every K step moves 256 KB through the 128 B/clk LDS port (2048 clk) for 2048 clk of
// MFMA work, and its prefetch window is what fits in staging registers.  Here
//  * a wave tile of 128 x 128 needs (128 + 128) operand rows per K step instead of 2 x (64 + 128)
//    for the same flops: LDS reads per step fall from 192 KB to 128 KB;
//  * tiles go from global memory straight into LDS (global_load_lds_dwordx4: each lane names a
//    global address, the 64 x 16 bytes of a wave land contiguously at the LDS address in M0), so
//    there are no ds_write instructions and no staging registers, and the 256 accumulator
//    registers of a wave fit beside everything else at one wave per SIMD;
//  * the W stream (HBM latency) runs two K steps ahead in a three-stage ring, the hidden tile
//    (L2 hits) one step ahead in a two-stage ring: 3 x 32 KB + 2 x 32 KB = all 160 KB of LDS.
//
// The compiler does not model these loads when written as inline assembly, so the kernel counts
// them itself: every K step issues the same number of loads per wave (hidden first, then W), and
// the wait at the top of a step allows exactly the newest W stage to be outstanding.  Loads past
// the end of K wrap around to valid K steps (their stage is never read) so the count never
// changes; everything is drained before the epilogue.
//
// LDS tiles have the layout of tile_off() (16-row blocks of 2 KB, chunk index XORed with r & 7).
// A wave-level load fills 1 KB = rows {r7, r7 + 8 : r7 in 4 j .. 4 j + 3} of one block, so lane l
// fetches row 8 ((l >> 3) & 1) + 4 j + ((l >> 4) & 3), chunk (l & 7) ^ (r7): eight lanes cover
// the 128 contiguous bytes of a row's K step.
//
// MFMA orientation and epilogue are those of the tiled kernel: A = W rows, B = hidden rows,
// v_mfma_f32_16x16x32_bf16, a lane owns four consecutive vocabulary ids of one batch row per
// 16 x 16 block.  A wave's 128 vocabulary rows are exactly one candidate tile, so candidates go
// from the lane-group merge straight to the candidate buffer, without a cross-wave merge.
// TOPK (Section "Top-k, Nucleus Sampling, and Masking": per-tile candidates): the epilogue writes the
// p.topk_k <= 8 best keys of every (batch row, 128-id tile), sorted and packed, instead of one
// candidate.
#pragma once

#include "fs_common.hpp"
#include "fs_stage1_tiled2.hpp"   // tile_off

namespace fs {

template <int BT_>
struct DmaCfg {
    static_assert(BT_ == 128 || BT_ == 256, "128 or 256 batch rows per workgroup (the launcher uses 256)");
    static constexpr int VT = 256, BT = BT_, kThreads = 256;
    static constexpr int kKS = 64;                         // contraction elements per K step
    static constexpr int kWStage = VT * 128;               // bytes of one W stage
    static constexpr int kHStage = BT * 128;
    static constexpr int kWStages = 3, kHStages = 2;
    static constexpr int RB = 8;                           // 16-row blocks per wave (128 vocabulary rows)
    static constexpr int CB = BT / 32;                     // 16-column blocks per wave (BT / 2 batch rows)
    static constexpr int kWLoads = VT / 32;                // 1 KB loads per wave and W stage
    static constexpr int kHLoads = BT / 32;
    static constexpr int kParkPerWave = RB * (CB < 4 ? CB : 4) * 1024;   // accumulator tiles parked for the epilogue
    static constexpr int kRowConstPerWave = CB * 1024;                   // per-row epilogue constants
    static constexpr size_t stage_bytes() { return (size_t)kWStages * kWStage + (size_t)kHStages * kHStage; }
    static constexpr size_t epilogue_bytes() { return (size_t)4 * (kParkPerWave + kRowConstPerWave); }
    static constexpr size_t lds_bytes() { return stage_bytes() > epilogue_bytes() ? stage_bytes() : epilogue_bytes(); }
};

// One wave-level direct load: lane l reads 16 bytes at sbase + voff + OFF and they land at LDS byte
// address m0 + OFF + 16 l (the immediate offset applies to both addresses).  SET_M0: write m0 = lds
// first; loads that follow with the same base reuse it and differ only in OFF (a multiple of 1024
// below 4096, which the caller has subtracted from voff).  NT: non-temporal (data read once).
// Increments vmcnt like any load.
template <bool NT, bool SET_M0, int OFF>
__device__ __forceinline__ void load_to_lds_16B(const void* sbase, uint32_t voff, uint32_t lds)
{
    static_assert(OFF >= 0 && OFF < 4096, "13-bit signed immediate offset");
    if constexpr (SET_M0) {
        if constexpr (NT)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3 nt"
                         :: "s"(lds), "v"(voff), "s"(sbase), "n"(OFF) : "memory", "m0");
        else
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
                         :: "s"(lds), "v"(voff), "s"(sbase), "n"(OFF) : "memory", "m0");
    } else {
        if constexpr (NT)
            asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2 nt" :: "v"(voff), "s"(sbase), "n"(OFF) : "memory");
        else
            asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" :: "v"(voff), "s"(sbase), "n"(OFF) : "memory");
    }
}

// LDS byte address of a pointer into shared memory (what M0 takes)
__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) unsigned char*)p;
}

template <int N>
__device__ __forceinline__ void wait_loads_outstanding()   // s_waitcnt vmcnt(N)
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// acc += a x b with the accumulator pinned to accumulation registers, in place.  Written as
// assembly because with 256 accumulator registers per lane the register allocator otherwise
// gives an MFMA a destination different from its addend and copies tiles around in every K step
// (352 copies for 128 MFMAs).  Every accumulator tile is touched once per 64 MFMAs, so no
// dependent MFMAs are ever close enough to need wait states.
__device__ __forceinline__ void mfma_acc(f32x4& acc, const bf16x8 a, const bf16x8 b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

template <class Cfg, bool STREAM_W, bool FULL = false, bool TOPK = false>
__global__ void __launch_bounds__(Cfg::kThreads, 1)
stage1_dma_kernel(const Stage1Params p, const int nbt)
{
    constexpr int BT = Cfg::BT, VT = Cfg::VT, RB = Cfg::RB, CB = Cfg::CB, KS = Cfg::kKS;
    constexpr int NWL = Cfg::kWLoads, NHL = Cfg::kHLoads;

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const uint32_t lds0 = lds_address(smem);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int n = lane & 15, g = lane >> 4;
    const int B = p.B, D = p.D, V = p.V, T = p.T;

    // dispatch id -> (vocabulary macro tile, batch tile): ids of one W tile are 8 apart (same XCD)
    const int id = (int)blockIdx.x;
    const int group = id / (8 * nbt);
    const int rem = id - group * (8 * nbt);
    const int tile = group * 8 + (rem & 7);
    const int bt = rem >> 3;
    if (tile * VT >= V) return;                  // whole workgroup leaves: no barrier is skipped
    const int b0 = bt * BT;
    const int tile_row0 = tile * VT;

    // K steps in rotated order (eight phases), as in the tiled kernel: workgroups that run at the
    // same time read different column ranges of their rows
    const int nk = D / KS;
    const int kfirst = (int)(((unsigned)tile + ((unsigned)tile >> 3)) & 7u) * (nk >> 3);   // K step of logical step 0
    auto knext = [&](int k) { return k + 1 == nk ? 0 : k + 1; };

    // per-lane source offsets of this wave's loads (rows clamped into the matrix: rows past V or
    // B re-read the last valid row and only feed outputs nobody reads)
    const int rlow = (lane >> 4) & 3, half = (lane >> 3) & 1, slot = lane & 7;
    // Load q of a stage carries the immediate offset 1024 (q % 4), which the per-lane offset gives
    // back; kBias keeps that offset non-negative (it is unsigned) and comes off the scalar base.
    constexpr uint32_t kBias = 4096u;
    uint32_t voffW[NWL], voffH[NHL];
#pragma unroll
    for (int q = 0; q < NWL; ++q) {
        const int r7 = 4 * (q & 1) + rlow;
        const int rt = 16 * ((NWL / 2) * wave + (q >> 1)) + 8 * half + r7;      // row inside the tile
        int row = tile_row0 + rt;
        row = row < V - 1 ? row : V - 1;
        voffW[q] = (uint32_t)(((row - tile_row0) * D + 8 * (slot ^ r7)) * 2) - (uint32_t)((q & 3) * 1024) + kBias;
    }
#pragma unroll
    for (int q = 0; q < NHL; ++q) {
        const int r7 = 4 * (q & 1) + rlow;
        const int rt = 16 * ((NHL / 2) * wave + (q >> 1)) + 8 * half + r7;
        int row = b0 + rt;
        row = row < B - 1 ? row : B - 1;
        voffH[q] = (uint32_t)(((row - b0) * D + 8 * (slot ^ r7)) * 2) - (uint32_t)((q & 3) * 1024) + kBias;
    }
    const unsigned char* wsrc = reinterpret_cast<const unsigned char*>(p.W) + (size_t)tile_row0 * D * 2 - kBias;
    const unsigned char* hsrc = reinterpret_cast<const unsigned char*>(p.H) + (size_t)b0 * D * 2 - kBias;
    const uint32_t ldsW = lds0 + (uint32_t)((NWL / 2) * wave) * 2048u;
    const uint32_t ldsH = lds0 + (uint32_t)(Cfg::kWStages * Cfg::kWStage) + (uint32_t)((NHL / 2) * wave) * 2048u;

    // One wave-level load (index q, a compile-time constant at every call) of a stage.  Four
    // consecutive loads share one M0 value and differ in the immediate offset: M0 is written by
    // the first of each group of four.  Nothing else in the K loop writes M0 (its body holds
    // MFMAs, LDS reads and waits only), and the loads of a stage are issued in order q = 0, 1, ...
    auto issue_w1 = [&](const unsigned char* src, uint32_t dst, auto qc) {
        constexpr int q = decltype(qc)::value;
        load_to_lds_16B<STREAM_W, (q & 3) == 0, (q & 3) * 1024>(src, voffW[q], dst + (uint32_t)(q & ~3) * 1024u);
    };
    auto issue_h1 = [&](const unsigned char* src, uint32_t dst, auto qc) {
        constexpr int q = decltype(qc)::value;
        load_to_lds_16B<false, (q & 3) == 0, (q & 3) * 1024>(src, voffH[q], dst + (uint32_t)(q & ~3) * 1024u);
    };
    auto w_src = [&](int k) { return wsrc + (size_t)k * (KS * 2); };
    auto h_src = [&](int k) { return hsrc + (size_t)k * (KS * 2); };
    auto w_dst = [&](int stage) { return ldsW + (uint32_t)stage * Cfg::kWStage; };
    auto h_dst = [&](int stage) { return ldsH + (uint32_t)stage * Cfg::kHStage; };
    auto issue_w = [&](int k, int stage) {
        static_for<NWL>([&](auto q) { issue_w1(w_src(k), w_dst(stage), q); });
    };
    auto issue_h = [&](int k, int stage) {
        static_for<NHL>([&](auto q) { issue_h1(h_src(k), h_dst(stage), q); });
    };

    f32x4 acc[RB][CB];
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < CB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // MFMA operand reads: lane (n, g) takes row 16 I + n, chunk 4 s + g of block I
    const int rd_lane = ((n & 7) << 8) + ((n >> 3) << 7);
    // One K step: 2 x CB groups of 8 MFMAs.  The NHL + NWL loads of the step are issued one (or
    // two) per group instead of in a burst at the top: a wave whose loads wait for room in the
    // memory pipeline cannot issue its MFMAs either, and it is the only wave on its SIMD.
    constexpr int NGRP = (KS / 32) * CB;
    constexpr int NLD = NHL + NWL;
    static_assert(NLD <= 2 * NGRP, "at most two loads per MFMA group");
    auto compute = [&](int wstage, int hstage, const unsigned char* hs_src, uint32_t hs_dst,
                       const unsigned char* ws_src, uint32_t ws_dst) {
        const unsigned char* wb = smem + wstage * Cfg::kWStage + (wm * RB) * 2048 + rd_lane;
        const unsigned char* hb = smem + Cfg::kWStages * Cfg::kWStage + hstage * Cfg::kHStage + (wn * CB) * 2048 + rd_lane;
        auto issue = [&](auto lc) {           // l-th load of the step: hidden loads first, then W
            constexpr int l = decltype(lc)::value;
            if constexpr (l < NHL) issue_h1(hs_src, hs_dst, std::integral_constant<int, l>{});
            else if constexpr (l < NLD) issue_w1(ws_src, ws_dst, std::integral_constant<int, l - NHL>{});
        };
        // Operand fragments are read ahead of their use so that the LDS latency (which grows while
        // the direct loads write into LDS) stays behind the MFMAs: the hidden fragment of column
        // block j + AHEAD and one W fragment of the NEXT half step are requested in group j.
        constexpr int AHEAD = 3;
        constexpr int NS = KS / 32;
        auto coff = [&](int s) { return ((4 * s + g) ^ (n & 7)) << 4; };
        auto rd_a = [&](int s, int i) {
            return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(wb + i * 2048 + coff(s)));
        };
        auto rd_b = [&](int s, int j) {
            return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(hb + j * 2048 + coff(s)));
        };
        bf16x8 a[2][RB], b[NS * CB];
#pragma unroll
        for (int i = 0; i < RB; ++i) a[0][i] = rd_a(0, i);
#pragma unroll
        for (int j = 0; j < AHEAD; ++j) b[j] = rd_b(j / CB, j % CB);
        static_for<NS * CB>([&](auto gc) {
            constexpr int grp = decltype(gc)::value, s = grp / CB, j = grp % CB;
            asm volatile("" ::: "memory");
            if constexpr (grp + AHEAD < NS * CB) b[grp + AHEAD] = rd_b((grp + AHEAD) / CB, (grp + AHEAD) % CB);
            if constexpr (s + 1 < NS) {       // W fragments of the next half step, spread over this one
#pragma unroll
                for (int i = j * RB / CB; i < (j + 1) * RB / CB; ++i) a[(s + 1) & 1][i] = rd_a(s + 1, i);
            }
            if constexpr (NLD <= NGRP) {
                issue(std::integral_constant<int, grp>{});
            } else {
                issue(std::integral_constant<int, 2 * grp>{});
                issue(std::integral_constant<int, 2 * grp + 1>{});
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) mfma_acc(acc[i][j], a[s & 1][i], b[grp]);
        });
    };

    // per-row epilogue constants of this lane's CB batch rows, requested now so that their latency
    // is long gone when the epilogue needs them
    f32x4 rowc[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) {
        int b = b0 + wn * (BT / 2) + j * 16 + n;
        b = b < B - 1 ? b : B - 1;
        const float tau = p.tau ? p.tau[b] : 1.0f;
        const uint64_t sd = p.row_seeds ? p.row_seeds[b] : p.seed;
        rowc[j] = f32x4{1.0f / tau, __uint_as_float((uint32_t)sd), __uint_as_float((uint32_t)(sd >> 32)), 0.0f};
    }

    // prologue: W steps 0 and 1 and hidden step 0 in flight (issue order W0, H0, W1)
    int k1 = knext(kfirst), k2 = knext(k1);            // K steps of logical steps t + 1, t + 2
    issue_w(kfirst, 0);
    issue_h(kfirst, 0);
    issue_w(k1, 1);
    int ws = 0, hs = 0;                                // stages of logical step t
    for (int t = 0; t < nk; ++t) {
        // own loads of step t have landed (the newest W stage may still be in flight) ...
        wait_loads_outstanding<NWL>();
        // ... and so have everybody's; every wave is done reading the stages overwritten next
        __syncthreads();
        const int ws2 = ws == 0 ? 2 : ws - 1;          // (t + 2) % 3
        compute(ws, hs, h_src(k1), h_dst(hs ^ 1), w_src(k2), w_dst(ws2));
        ws = ws == 2 ? 0 : ws + 1;
        hs ^= 1;
        k1 = k2;
        k2 = knext(k2);
    }
    wait_loads_outstanding<0>();                       // nothing may still be writing LDS when the wave ends
    // The MFMAs above are opaque to the compiler's hazard handling: it would read the accumulator of
    // the very last one in the next instruction.  An MFMA issues every 16 cycles and needs at most
    // 18 wait states before its result may be read, so only the last two are in question; the
    // last column's accumulators are operands of the wait so that no read can move above it.
    asm volatile("s_nop 15\n\ts_nop 15"
                 : "+a"(acc[0][CB - 1]), "+a"(acc[1][CB - 1]), "+a"(acc[2][CB - 1]), "+a"(acc[3][CB - 1]),
                   "+a"(acc[4][CB - 1]), "+a"(acc[5][CB - 1]), "+a"(acc[6][CB - 1]), "+a"(acc[7][CB - 1]));

    // Epilogue.  acc[i][j][q] = logit of vocabulary row tile_row0 + 128 wm + 16 i + 4 g + q, batch row
    // b0 + (BT/2) wn + 16 j + n.  Registers cannot be indexed by a loop variable, and the epilogue
    // unrolled over all 8 x CB accumulator tiles is several hundred KB of code that each wave walks
    // through once per tile (instruction fetch and spills then cost more than its arithmetic).  So
    // each wave parks its accumulators in LDS, which is free now, CJ column blocks at a time, and
    // reads them back in a rolled loop: four independent tiles per iteration, which is what lets
    // a lone wave on its SIMD overlap the dependent chains of the Philox rounds.
    constexpr int CJ = CB < 4 ? CB : 4;                   // 8 x CJ tiles x 1 KB = 32 KB per wave
    constexpr int U = 4;
    static_assert(RB % U == 0 && CB % CJ == 0, "epilogue blocking");
    __syncthreads();                                       // every wave is done with the stages
    f32x4* park = reinterpret_cast<f32x4*>(smem) + (size_t)wave * (Cfg::kParkPerWave / 16) + lane;
    f32x4* rowc_lds = reinterpret_cast<f32x4*>(smem + 4 * Cfg::kParkPerWave) + (size_t)wave * (Cfg::kRowConstPerWave / 16) + lane;
#pragma unroll
    for (int j = 0; j < CB; ++j) rowc_lds[j * 64] = rowc[j];
    const int ctile = tile * (VT / kVocabTile) + wm;
    if constexpr (TOPK) {
        // Truncated supports: the m best keys of every (batch row, 128-id tile) instead of one
        // candidate.  A wave's 128 ids are one candidate tile and a lane holds 32 of them for each of
        // its batch rows, so a lane keeps a sorted list of the best m of those 32 in registers (one
        // insertion per key), the four lanes that share a row merge their lists, and each writes its
        // share of the m words.  No scalar work, no cross-lane traffic before the merge.
        const int vl0 = tile_row0 + wm * kVocabTile;            // first vocabulary row of this wave
        const int kt = p.topk_k;
        const int nvalid = vl0 + kVocabTile <= V ? 1 << 20 : V - vl0 - 4 * g;   // local ids 16 i + q below this exist
        auto rows = [&](auto mc, auto noisyc) {
            constexpr int M = decltype(mc)::value;
            constexpr bool NOISY = decltype(noisyc)::value;
#pragma unroll
            for (int jc = 0; jc < CB; jc += CJ) {
#pragma unroll
                for (int jj = 0; jj < CJ; ++jj)
#pragma unroll
                    for (int i = 0; i < RB; ++i) park[(jj * RB + i) * 64] = acc[i][jc + jj];
#pragma unroll 1
                for (int jj = 0; jj < CJ; ++jj) {
                    const int b = b0 + wn * (BT / 2) + (jc + jj) * 16 + n;
                    const f32x4 rc = rowc_lds[(jc + jj) * 64];
                    const float inv_tau = rc[0];
                    const uint64_t sd = (uint64_t)__float_as_uint(rc[1]) | ((uint64_t)__float_as_uint(rc[2]) << 32);
                    uint32_t ka[M];
                    int32_t ke[M];
#pragma unroll
                    for (int s = 0; s < M; ++s) { ka[s] = 0u; ke[s] = 0; }
#pragma unroll 1
                    for (int i0 = 0; i0 < RB; i0 += U) {
                        f32x4 y[U];
                        float gn[U][4];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            y[u] = park[(jj * RB + i0 + u) * 64];
#pragma unroll
                            for (int q = 0; q < 4; ++q) gn[u][q] = 0.0f;
                        }
                        if constexpr (NOISY) {
                            uint32_t vid0[U];
#pragma unroll
                            for (int u = 0; u < U; ++u) vid0[u] = (uint32_t)(p.vocab_offset + vl0 + (i0 + u) * 16 + 4 * g);
                            gumbel4_multi<U>(sd, (uint32_t)(uint64_t)(p.row_offset + (b < B ? b : B - 1)), vid0, gn,
                                             (p.epi_flags & kEpiExactLog) != 0u);
                        }
#pragma unroll
                        for (int u = 0; u < U; ++u)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const int e = (i0 + u) * 16 + q;
                                const uint32_t o = topk_ordered(fmaf(y[u][q], inv_tau, gn[u][q]));
                                top_insert<M>(ka, ke, e < nvalid ? o : 0u, e);
                            }
                    }
                    // the row's best m: merge with the lanes 16 and 32 away (same row, other ids)
                    uint64_t w[M];
                    const int32_t id0 = p.vocab_offset + vl0 + 4 * g;
#pragma unroll
                    for (int s = 0; s < M; ++s)
                        w[s] = ka[s] ? ((uint64_t)ka[s] << 32) | (uint64_t)(~(uint32_t)(id0 + ke[s])) : kTopkPad;
                    top_merge<M>(w, 16);
                    top_merge<M>(w, 32);
                    if (b < B && ctile < T) {
                        uint64_t* dst = p.topk_out + ((size_t)b * T + ctile) * (size_t)kt;
#pragma unroll
                        for (int s0 = 0; s0 < M; s0 += 4) {
                            uint64_t mine = w[s0];
#pragma unroll
                            for (int t = 1; t < 4; ++t) mine = g == t ? w[s0 + t] : mine;
                            // non-temporal: 32 bytes per (row, tile), read once by the selection.  Stored
                            // normally these lines crowd the hidden tile out of L2 (it fills most of it at
                            // D >= 7168): the launch took 9 % longer at D = 7168, B = 256
                            if (s0 + g < kt) __builtin_nontemporal_store(mine, dst + s0 + g);
                        }
                    }
                }
            }
        };
        using M4 = std::integral_constant<int, 4>;
        using M8 = std::integral_constant<int, 8>;
        if (p.topk_mode == kTopkGumbel) {
            if (kt <= 4) rows(M4{}, std::true_type{});
            else rows(M8{}, std::true_type{});
        } else {
            if (kt <= 4) rows(M4{}, std::false_type{});
            else rows(M8{}, std::false_type{});
        }
        return;
    }
    // No check is needed inside a quad when the whole tile lies inside the vocabulary, ids are
    // aligned to the Philox blocks, and nothing but the default sampling epilogue is asked for.
    const bool fast = !FULL && p.cand_val && !p.logits && p.epi_flags == 0u && (p.vocab_offset & 3) == 0 &&
                      tile_row0 + VT <= V;
#pragma unroll
    for (int jc = 0; jc < CB; jc += CJ) {
#pragma unroll
        for (int jj = 0; jj < CJ; ++jj)
#pragma unroll
            for (int i = 0; i < RB; ++i) park[(jj * RB + i) * 64] = acc[i][jc + jj];
#pragma unroll 1
        for (int jj = 0; jj < CJ; ++jj) {
            const int b = b0 + wn * (BT / 2) + (jc + jj) * 16 + n;
            const f32x4 rc = rowc_lds[(jc + jj) * 64];
            RowEpi repi;
            repi.inv_tau = rc[0];
            repi.seed = (uint64_t)__float_as_uint(rc[1]) | ((uint64_t)__float_as_uint(rc[2]) << 32);
            repi.row_word = (uint32_t)(uint64_t)(p.row_offset + b);
            repi.allowed_row = nullptr;
            if constexpr (FULL) {
                if (p.allowed && b < B) repi.allowed_row = p.allowed + (size_t)b * (size_t)p.mask_stride;
            }
            float best = -__builtin_inff();
            int best_id = -1;
            float lmax = -__builtin_inff(), lsum = 0.0f;
            if (fast) {
                // U independent quads per iteration, each with its own running candidate
                float bs[U];
                int bi[U];
#pragma unroll
                for (int u = 0; u < U; ++u) { bs[u] = -__builtin_inff(); bi[u] = -1; }
#pragma unroll 1
                for (int i0 = 0; i0 < RB; i0 += U) {
                    f32x4 y[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) y[u] = park[(jj * RB + i0 + u) * 64];
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        epilogue_quad_fast(repi.seed, repi.row_word, repi.inv_tau, y[u],
                                           p.vocab_offset + tile_row0 + wm * 128 + (i0 + u) * 16 + 4 * g, bs[u], bi[u]);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) cand_merge(best, best_id, bs[u], bi[u]);
            } else if (b < B) {
#pragma unroll 1
                for (int i0 = 0; i0 < RB; ++i0) {
                    const f32x4 y = park[(jj * RB + i0) * 64];
                    const int v0 = tile_row0 + wm * 128 + i0 * 16 + 4 * g;
                    if (v0 < V) {
                        if (p.logits) {
                            float* dst = p.logits + (size_t)b * V + v0;
                            if (v0 + 3 < V && (V & 3) == 0) {
                                *reinterpret_cast<f32x4*>(dst) = y;
                            } else {
#pragma unroll
                                for (int q = 0; q < 4; ++q)
                                    if (v0 + q < V) dst[q] = y[q];
                            }
                        }
                        if (p.cand_val) epilogue_quad<FULL>(p, repi, y, v0, V, best, best_id, lmax, lsum);
                    }
                }
            }
            cand_reduce_lane_groups(best, best_id);
            if constexpr (FULL) lse_reduce_lane_groups(lmax, lsum);
            if (p.cand_val && g == 0 && b < B && ctile < T) {
                p.cand_val[(size_t)b * T + ctile] = best;
                p.cand_idx[(size_t)b * T + ctile] = best_id;
                if constexpr (FULL) {
                    if (p.lse_max) {
                        p.lse_max[(size_t)b * T + ctile] = lmax;
                        p.lse_sum[(size_t)b * T + ctile] = lsum;
                    }
                }
            }
        }
    }
}

}  // namespace fs
