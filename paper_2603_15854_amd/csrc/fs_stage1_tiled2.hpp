// Stage 1 of Alg. 1 for B > 16: LDS-tiled matmul with the sampling epilogue.
//
// Workgroup: 4 or 8 waves as WM x WN; tile = VT vocabulary ids (128, 256 or 512) x BT batch rows;
// wave tile = (VT/WM) x (BT/WN).  MFMA A operand = W rows (M = vocabulary), B operand = hidden rows
// (N = batch), v_mfma_f32_16x16x32_bf16, fp32 accumulators.  The four-wave shapes leave room for
// two workgroups per compute unit, so that one workgroup's VALU-heavy epilogue (Philox, logs,
// argmax) overlaps the other's main loop; the eight-wave shapes run one workgroup per compute
// unit and re-read the hidden tile less often per W byte.
//
// K loop, 64 elements per step, two LDS buffers (steps k and k+1), one barrier per step.
// Global loads run ahead of use in registers: the hidden tile two steps ahead, the W tile in
// groups of GS steps (GS*128 contiguous bytes of every row are requested back to back), two
// groups in flight.  LDS tiles have 128-byte rows placed by tile_off().
//
// When the batch needs several tiles (B > BT), the workgroups that share a W tile get dispatch
// ids 8 apart: workgroups are dealt round-robin to the 8 XCDs, so they land on the same XCD at
// the same time and the second read of the W tile is served by that XCD's L2.  W is then loaded
// with plain loads; with a single batch tile it is streamed with non-temporal loads.
#pragma once

#include <type_traits>

#include "fs_common.hpp"
#include "fs_topk_common.hpp"   // top_insert, top_merge

namespace fs {

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

// VT: vocabulary rows per workgroup (128, 256 or 512 = one, two or four candidate tiles); BT: batch rows;
// WM x WN waves (4 or 8); GS: K steps per W prefetch group; OCC: waves per SIMD asked for.
// NSET: register sets of prefetched loads (2: hidden two steps and W two groups ahead; 1: one
// step / one group ahead, for the tile shapes whose accumulators leave no room for more).
template <int BT_, int WM_, int WN_, int GS_, int OCC_ = 2, int VT_ = kVocabTile, int NSET_ = 2>
struct Tiled2Cfg {
    static constexpr int BT = BT_, WM = WM_, WN = WN_, GS = GS_, OCC = OCC_, VT = VT_, NSET = NSET_;
    static_assert(NSET_ == 1 || NSET_ == 2, "one or two prefetch register sets");
    static constexpr int kWaves = WM * WN;
    static constexpr int kThreads = kWaves * kWave;
    static_assert(kWaves == 4 || kWaves == 8, "four or eight waves per workgroup");
    static_assert(VT % kVocabTile == 0, "whole candidate tiles");
    static constexpr int RB = VT / (16 * WM);            // 16-row blocks per wave
    static constexpr int CB = BT / (16 * WN);            // 16-column blocks per wave
    static_assert(RB >= 1 && CB >= 1 && kVocabTile % (16 * RB) == 0, "wave tile inside one candidate tile");
    static constexpr int kWavesPerCandTile = kVocabTile / (16 * RB);
    static constexpr int kCandTiles = VT / kVocabTile;
    static constexpr int kKS = 64;
    static constexpr int kWBytes = VT * 128;
    static constexpr int kHBytes = BT * 128;
    static constexpr int kBufBytes = kWBytes + kHBytes;
    static constexpr int kRowsPerPass = kThreads / 8;    // rows one workgroup-wide load covers
    static constexpr int kWLoads = VT / kRowsPerPass;
    // a batch tile with fewer rows than one load pass: every thread still loads (rows repeat
    // modulo BT, so the loads stay unconditional) and only the first BT rows are parked
    static constexpr bool kHPartial = BT < kRowsPerPass;
    static constexpr int kHLoads = kHPartial ? 1 : BT / kRowsPerPass;
    static_assert(kWLoads >= 1 && (kHPartial ? kRowsPerPass % BT == 0 : BT % kRowsPerPass == 0),
                  "tile rows per load pass");
    // the per-wave candidate / log-sum-exp scratch of the epilogue reuses the tile buffers
    static_assert((size_t)WM * BT * 8 * 2 <= 2 * (size_t)kBufBytes, "epilogue scratch fits the tile buffers");
    static constexpr size_t lds_bytes() { return 2 * (size_t)kBufBytes; }
};

// WB: bytes per W element.  2 = bf16.  1 = FP8 E4M3 codes, in one of two forms:
//   WCODES = false: a K step stays 64 elements (four 16-byte loads per row), the codes are widened
//     to bf16 when the step is parked, and LDS and the MFMA loop are those of the bf16 path;
//   WCODES = true: a K step is 128 elements, i.e. the same 128 bytes (one cache line) of a W row
//     as on the bf16 path; LDS holds the codes (same W tile bytes, half the LDS writes per
//     element), the hidden tile of a step is two 64-element sub-tiles, and a lane widens the 8
//     codes of its MFMA operand after reading them (ds_read_b64).
// KRAG: D need not be a multiple of the K step (the chunks of the last step that lie past D are
// zeroed when parked).  The zeroing selects cost registers and time in the main loop (256 x 128:
// 202 -> 158 VGPRs and -5 % time without them), so whole-step hidden sizes get KRAG = false.
// TOPK (Section "Top-k, Nucleus Sampling, and Masking": per-tile candidates): instead of one
// candidate per (row, 128-id tile) the epilogue writes the p.topk_k <= 8 best, sorted and packed
// (per-lane sorted lists in registers, merged across the lanes and waves that share a tile).
// W4 (with WB = 1, WCODES): MXFP4 weights.  p.W holds E2M1 codes, two per byte, p.w4_scales one E8M0 byte
// per 32 elements of a row.  A K step is 256 elements = again the same 128 bytes of a W row; LDS holds
// the codes and, behind the tiles, the step's 8 scale bytes of every row; the hidden tile of a step is
// four 64-element sub-tiles; a lane reads the 8 codes of its MFMA operand as one dword and widens them
// with the block scale (mxfp4x8_to_bf16x8).  Whole K steps only (D % 256 == 0).
template <class Cfg, bool STREAM_W, bool FULL = false, int WB = 2, bool WCODES = false, bool KRAG = true, bool TOPK = false,
          bool W4 = false>
__global__ void __launch_bounds__(Cfg::kThreads, Cfg::OCC)
stage1_tiled2_kernel(const Stage1Params p, const int nbt)
{
    static_assert(!TOPK || (!FULL && WB == 2), "per-tile top-k: bf16 weights, plain transform");
    static_assert(!WCODES || WB == 1, "codes in LDS only for one-byte W elements");
    static_assert(!W4 || (WCODES && !KRAG && !FULL && Cfg::VT <= Cfg::kThreads), "MXFP4: codes in LDS, whole K steps, plain transform");
    constexpr int BT = Cfg::BT, WM = Cfg::WM, WN = Cfg::WN, RB = Cfg::RB, CB = Cfg::CB, GS = Cfg::GS;
    constexpr int KS = W4 ? 4 * Cfg::kKS : WCODES ? 2 * Cfg::kKS : Cfg::kKS, VT = Cfg::VT, RPP = Cfg::kRowsPerPass;
    constexpr int HH = KS / 64;                      // 64-element hidden sub-tiles per K step
    constexpr int NHL = Cfg::kHLoads * HH;           // hidden loads per thread and K step
    constexpr int WEPC = W4 ? 32 : 16 / WB;          // W elements per 16-byte load
    constexpr int WCH = KS / WEPC;                   // loads per W row and K step (8 or 4)
    constexpr int WRPP = Cfg::kThreads / WCH;        // W rows one workgroup-wide load covers
    constexpr int NWL = VT / WRPP;                   // W loads per thread and K step
    static_assert(VT % WRPP == 0 && NWL >= 1, "W tile rows per load pass");
    constexpr int HSUB = BT * 128;                   // bytes of one hidden sub-tile
    constexpr int SCB = W4 ? VT * 8 : 0;             // scale bytes of one K step (MXFP4)
    constexpr int BUFB = Cfg::kWBytes + HH * HSUB + SCB;   // bytes of one LDS buffer (one K step)

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    auto w_lds = [&](int buf) { return smem + buf * BUFB; };
    auto h_lds = [&](int buf) { return smem + buf * BUFB + Cfg::kWBytes; };
    auto s_lds = [&](int buf) { return smem + buf * BUFB + Cfg::kWBytes + HH * HSUB; };
    // epilogue scratch, aliased onto the tile buffers: first written after the barrier that ends
    // the last K step, when no wave reads or parks tiles any more
    float2* wave_cand = reinterpret_cast<float2*>(smem);                        // [WM][BT]
    float2* wave_lse = wave_cand + WM * BT;                                    // [WM][BT]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int n = lane & 15, g = lane >> 4;
    const int B = p.B, D = p.D, V = p.V, T = p.T;

    // dispatch id -> (vocabulary macro tile, batch tile): ids of one W tile are 8 apart (same XCD)
    const int id = (int)blockIdx.x;
    const int group = id / (8 * nbt);
    const int rem = id - group * (8 * nbt);
    const int tile = group * 8 + (rem & 7);      // macro tile of VT vocabulary rows
    const int bt = rem >> 3;
    if (tile * VT >= V) return;                  // whole workgroup leaves: no barrier is skipped
    const int b0 = bt * BT;
    const int tile_row0 = tile * VT;

    // K steps of this tile, visited in rotated order: workgroups that run at the same time start
    // at different offsets along K (eight phases), so that at any instant the rows being read are
    // spread over column ranges, hence over HBM channels, instead of all sitting at the same
    // offset of 8 KB-strided rows.  Logical step t is K step kmap(t); t >= nk stays out of range.
    const int nk = (D + KS - 1) / KS;
    const int kstart = (int)(((unsigned)tile + ((unsigned)tile >> 3)) & 7u) * (nk >> 3);
    auto kmap = [&](int t) -> int {
        const int a = t + kstart;
        return t >= nk ? t : (a >= nk ? a - nk : a);
    };

    const int ld_chunk = tid & 7;
    const int ld_row = tid >> 3;   // 0..RPP-1
    const int wld_chunk = tid % WCH;
    const int wld_row = tid / WCH;   // 0..WRPP-1
    constexpr int NSET = Cfg::NSET;
    uint4 wst[NSET][GS][NWL];        // NSET groups of GS steps
    uint4 hst[NSET][NHL];            // NSET steps
    uint2 sst[NSET][GS];             // MXFP4: the 8 scale bytes of row tid % VT, per step

    // Every load of the K loop is unconditional, so the compiler can count the loads in flight and
    // wait for exactly the step it parks (s_waitcnt vmcnt(N)) instead of draining the prefetch:
    // rows past V (or B) re-read the last valid row and only feed outputs nobody reads (each
    // output row/column depends on its own operand row only); a prefetch that runs past the end
    // of K reads one fixed cache line; a chunk past D inside the last step is zeroed when parked.
    const bool k_ragged = KRAG && (D & (KS - 1)) != 0;
    auto fetch_w = [&](uint4 (&wr)[NWL], int k0) {
        const bool over = k0 >= D;                          // uniform
        int k = over ? wld_chunk * WEPC : k0 + wld_chunk * WEPC;
        k = k < D - WEPC ? k : D - WEPC;     // also when the fixed line is wider than a short row
#pragma unroll
        for (int i = 0; i < NWL; ++i) {
            int row = tile_row0 + wld_row + WRPP * i;
            row = row < V - 1 ? row : V - 1;
            row = over ? tile_row0 : row;
            const size_t off = W4 ? ((size_t)row * D + k) >> 1 : ((size_t)row * D + k) * WB;
            const uint16_t* src = reinterpret_cast<const uint16_t*>(reinterpret_cast<const unsigned char*>(p.W) + off);
            wr[i] = STREAM_W ? ld_global_16B_stream(src) : ld_global_16B(src);
        }
    };
    // MXFP4: scale bytes k0/32 .. k0/32 + 7 of row tile_row0 + tid % VT (clamped like the W rows)
    auto fetch_s = [&](uint2& sr, int k0) {
        const bool over = k0 >= D;
        int row = tile_row0 + (tid % VT);
        row = row < V - 1 ? row : V - 1;
        row = over ? tile_row0 : row;
        const int kb = over ? 0 : k0 >> 5;
        sr = *reinterpret_cast<const uint2*>(p.w4_scales + (size_t)row * (D >> 5) + kb);
    };
    auto fetch_w_group = [&](uint4 (&grp)[GS][NWL], uint2 (&sgrp)[GS], int group) {
#pragma unroll
        for (int s = 0; s < GS; ++s) {
            fetch_w(grp[s], kmap(group * GS + s) * KS);
            if constexpr (W4) fetch_s(sgrp[s], kmap(group * GS + s) * KS);
        }
    };
    auto fetch_h = [&](uint4 (&hr)[NHL], int k0) {
        const bool over = k0 >= D;
#pragma unroll
        for (int hh = 0; hh < HH; ++hh) {
            int k = over ? ld_chunk * 8 : k0 + hh * 64 + ld_chunk * 8;
            k = k < D - 8 ? k : D - 8;
#pragma unroll
            for (int i = 0; i < Cfg::kHLoads; ++i) {
                int r = b0 + (Cfg::kHPartial ? (ld_row & (BT - 1)) : ld_row + RPP * i);
                r = r < B - 1 ? r : B - 1;
                hr[hh * Cfg::kHLoads + i] = ld_global_16B(p.H + (size_t)r * D + k);
            }
        }
    };
    // park K step `step` (registers -> LDS buffer buf)
    auto park = [&](const uint4 (&wr)[NWL], const uint2& sr, const uint4 (&hr)[NHL], int buf, int step) {
        const bool wzero = k_ragged && (step * KS + wld_chunk * WEPC >= D);   // only in the last step
        if constexpr (W4) {
            if (tid < VT) *reinterpret_cast<uint2*>(s_lds(buf) + tid * 8) = sr;
        }
#pragma unroll
        for (int i = 0; i < NWL; ++i) {
            const int r = wld_row + WRPP * i;
            uint4 v = wr[i];
            if (wzero) v = make_uint4(0u, 0u, 0u, 0u);
            if constexpr (WB == 2 || WCODES) {
                *reinterpret_cast<uint4*>(w_lds(buf) + tile_off(r, wld_chunk)) = v;
            } else {   // 16 codes -> two bf16 chunks
                *reinterpret_cast<bf16x8*>(w_lds(buf) + tile_off(r, 2 * wld_chunk)) = e4m3x8_to_bf16x8(v.x, v.y);
                *reinterpret_cast<bf16x8*>(w_lds(buf) + tile_off(r, 2 * wld_chunk + 1)) = e4m3x8_to_bf16x8(v.z, v.w);
            }
        }
#pragma unroll
        for (int hh = 0; hh < HH; ++hh) {
            const bool zero = k_ragged && (step * KS + hh * 64 + ld_chunk * 8 >= D);
#pragma unroll
            for (int i = 0; i < Cfg::kHLoads; ++i) {
                const int r = ld_row + RPP * i;
                uint4 v = hr[hh * Cfg::kHLoads + i];
                if (zero) v = make_uint4(0u, 0u, 0u, 0u);
                if (!Cfg::kHPartial || r < BT)
                    *reinterpret_cast<uint4*>(h_lds(buf) + hh * HSUB + tile_off(r, ld_chunk)) = v;
            }
        }
    };

    f32x4 acc[RB][CB];
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < CB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf) {
        uint2 sc[RB];                         // MXFP4: the step's 8 scale bytes of this lane's RB operand rows
        if constexpr (W4) {
#pragma unroll
            for (int i = 0; i < RB; ++i)
                sc[i] = *reinterpret_cast<const uint2*>(s_lds(buf) + (wm * (16 * RB) + i * 16 + n) * 8);
        }
#pragma unroll
        for (int s = 0; s < KS / 32; ++s) {   // 32 contraction elements per MFMA
            const int c = 4 * (s & 1) + g;    // hidden chunk inside its 64-element sub-tile
            bf16x8 a[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int r = wm * (16 * RB) + i * 16 + n;
                if constexpr (W4) {           // 8 codes: dword g of 16-byte chunk s (= K step of 32 elements)
                    const uint32_t codes = *reinterpret_cast<const uint32_t*>(w_lds(buf) + tile_off(r, s) + (g << 2));
                    const uint32_t e = ((s < 4 ? sc[i].x : sc[i].y) >> (8 * (s & 3))) & 0xFFu;
                    a[i] = mxfp4x8_to_bf16x8(codes, e);
                } else if constexpr (WCODES) {       // 8 codes: half of 16-byte chunk 2 s + g / 2
                    const uint2 q = *reinterpret_cast<const uint2*>(
                        w_lds(buf) + tile_off(r, 2 * s + (g >> 1)) + ((g & 1) << 3));
                    a[i] = e4m3x8_to_bf16x8(q.x, q.y);
                } else {
                    a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                                                          w_lds(buf) + tile_off(r, c)));
                }
            }
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                const int r = wn * (16 * CB) + j * 16 + n;
                const bf16x8 b = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                                                                h_lds(buf) + (s >> 1) * HSUB + tile_off(r, c)));
#pragma unroll
                for (int i = 0; i < RB; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b, acc[i][j], 0, 0, 0);
            }
        }
    };

    // prologue: W groups 0 and 1 and hidden steps 0 and 1 in flight; step 0 parked
    // (fetches past the end of K read one fixed cache line)
    fetch_w_group(wst[0], sst[0], 0);
    if constexpr (NSET == 2) fetch_w_group(wst[1], sst[1], 1);
    fetch_h(hst[0], kmap(0) * KS);
    if constexpr (NSET == 2) fetch_h(hst[1], kmap(1) * KS);
    park(wst[0][0], sst[0][0], hst[0], 0, kmap(0));
    fetch_h(hst[0], kmap(NSET) * KS);
    if (GS == 1) fetch_w_group(wst[0], sst[0], NSET);
    __syncthreads();
    // One body = 2*GS steps, after which the register sets are back in their starting roles.
    // Full bodies run without any condition (parking a step past the end only fills the LDS
    // buffer nobody reads next); the ragged remainder uses the guarded form.
    auto body = [&](int base, auto guarded) {
#pragma unroll
        for (int u = 0; u < 2 * GS; ++u) {
            const int t = base + u;                 // step computed now, from LDS buffer u & 1
            if (!decltype(guarded)::value || t < nk) {
                const int nset = NSET == 2 ? ((u + 1) / GS) & 1 : 0;   // register set and slot of step t + 1
                const int hset = NSET == 2 ? (u + 1) & 1 : 0;
                const int nslot = (u + 1) % GS;
                park(wst[nset][nslot], sst[nset][nslot], hst[hset], (u + 1) & 1, kmap(t + 1));
                fetch_h(hst[hset], kmap(t + 1 + NSET) * KS);
                if (nslot == GS - 1) fetch_w_group(wst[nset], sst[nset], (t + 1) / GS + NSET);   // set is free again
                compute(u & 1);
                __syncthreads();
            }
        }
    };
    int base = 0;
    for (; base + 2 * GS <= nk; base += 2 * GS) body(base, std::false_type{});
    if (base < nk) body(base, std::true_type{});

    if constexpr (TOPK) {
        // A lane holds 4 RB ids of each of its CB batch rows: it keeps a sorted list of the best m of
        // them in registers (one insertion per key, ascending ids), the four lanes that share a row
        // merge their lists, and -- where two or four waves share a 128-id candidate tile -- the
        // waves' lists meet in LDS (the last K step ended with a barrier: the tile buffers are free).
        constexpr int WPT = Cfg::kWavesPerCandTile;
        static_assert(WPT == 1 || WPT == 2 || WPT == 4, "one, two or four waves per candidate tile");
        static_assert((size_t)WM * BT * kTopkTileM * 8 <= 2 * (size_t)BUFB, "wave lists fit the tile buffers");
        const int kt = p.topk_k;
        const int vw0 = tile_row0 + wm * (16 * RB);          // first vocabulary row of this wave
        const int nvalid = vw0 + 16 * RB <= V ? 1 << 20 : V - vw0 - 4 * g;   // local ids 16 i + q below this exist
        uint64_t* wave_list = reinterpret_cast<uint64_t*>(smem);             // [WM][BT][M], WPT > 1 only
        // M: list length; NOISY: keys carry Gumbel noise (compile-time, so that the plain form holds no
        // generator code and every unrolled loop stays within what the compiler unrolls)
        auto rows = [&](auto mc, auto noisyc) {
            constexpr int M = decltype(mc)::value;
            constexpr bool NOISY = decltype(noisyc)::value;
            static_for<CB>([&](auto jc) {      // not a loop: unrolled, its body is beyond what the compiler unrolls
                constexpr int j = decltype(jc)::value;
                const int bl = wn * (16 * CB) + j * 16 + n;
                const int b = b0 + bl;
                const int bc = b < B ? b : B - 1;
                const float inv_tau = 1.0f / p.tau[bc];
                const uint64_t sd = p.row_seeds ? p.row_seeds[bc] : p.seed;
                uint32_t ka[M];
                int32_t ke[M];
#pragma unroll
                for (int s = 0; s < M; ++s) { ka[s] = 0u; ke[s] = 0; }
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    float gn[4] = {0.f, 0.f, 0.f, 0.f};
                    if constexpr (NOISY)
                        gumbel4(sd, (uint32_t)(uint64_t)(p.row_offset + bc), (uint32_t)(p.vocab_offset + vw0 + i * 16 + 4 * g), gn,
                                (p.epi_flags & kEpiExactLog) != 0u);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int e = i * 16 + q;
                        const uint32_t o = topk_ordered(fmaf(acc[i][j][q], inv_tau, gn[q]));
                        top_insert<M>(ka, ke, e < nvalid ? o : 0u, e);
                    }
                }
                uint64_t w[M];
                const int32_t id0 = p.vocab_offset + vw0 + 4 * g;
#pragma unroll
                for (int s = 0; s < M; ++s)
                    w[s] = ka[s] ? ((uint64_t)ka[s] << 32) | (uint64_t)(~(uint32_t)(id0 + ke[s])) : kTopkPad;
                top_merge<M>(w, 16);
                top_merge<M>(w, 32);
                // all four lanes of the row hold its list now: lane group g keeps words g, g + 4
                const int ctile = tile * Cfg::kCandTiles + wm / WPT;
                uint64_t* dst = WPT == 1 ? p.topk_out + ((size_t)b * T + ctile) * (size_t)kt
                                         : wave_list + ((size_t)wm * BT + bl) * M;
                const bool live = WPT == 1 ? b < B && ctile < T : true;
#pragma unroll
                for (int s0 = 0; s0 < M; s0 += 4) {
                    uint64_t mine = w[s0];
#pragma unroll
                    for (int t = 1; t < 4; ++t) mine = g == t ? w[s0 + t] : mine;
                    if (live && (WPT > 1 || s0 + g < kt)) dst[s0 + g] = mine;
                }
                // rows are worked through one after the other: interleaved, their compare masks
                // would not fit the scalar registers
                __builtin_amdgcn_sched_barrier(0);
            });
            if constexpr (WPT > 1) {
                __syncthreads();
                for (int u = tid; u < BT * Cfg::kCandTiles; u += Cfg::kThreads) {
                    const int bl = u % BT, ct = u / BT;
                    const int b = b0 + bl, ctile = tile * Cfg::kCandTiles + ct;
                    uint64_t w[M];
                    const uint64_t* la = wave_list + ((size_t)(WPT * ct) * BT + bl) * M;
#pragma unroll
                    for (int s = 0; s < M; ++s) w[s] = la[s];
#pragma unroll
                    for (int x = 1; x < WPT; ++x) {
                        const uint64_t* lb = wave_list + ((size_t)(WPT * ct + x) * BT + bl) * M;
                        uint64_t o[M];
#pragma unroll
                        for (int s = 0; s < M; ++s) o[s] = lb[M - 1 - s];
                        top_merge_lists<M>(w, o);
                    }
                    if (b < B && ctile < T) {
#pragma unroll
                        for (int s = 0; s < M; ++s)
                            if (s < kt) p.topk_out[((size_t)b * T + ctile) * (size_t)kt + s] = w[s];
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

    // epilogue: acc[i][j][q] = logit of vocabulary row tile_row0 + wm*16*RB + 16 i + 4 g + q,
    // batch row b0 + wn*16*CB + 16 j + n
#pragma unroll
    for (int j = 0; j < CB; ++j) {
        const int bl = wn * (16 * CB) + j * 16 + n;   // row inside the batch tile
        const int b = b0 + bl;
        float best = -__builtin_inff();
        int best_id = -1;
        float lmax = -__builtin_inff(), lsum = 0.0f;
        if (b < B) {
            RowEpi repi = {1.0f, p.seed, (uint32_t)(uint64_t)(p.row_offset + b), nullptr};
            if (p.cand_val) repi = make_row_epi<FULL>(p, b);
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                f32x4 y = acc[i][j];
                const int v0 = tile_row0 + wm * (16 * RB) + i * 16 + 4 * g;
                if constexpr (WB == 1) {   // per-row scale of the FP8 weights
                    if (p.w_scale && v0 < V) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) y[q] *= p.w_scale[v0 + q < V ? v0 + q : V - 1];
                    }
                }
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
        if (g == 0) wave_cand[wm * BT + bl] = make_float2(best, __int_as_float(best_id));
        if constexpr (FULL) {
            lse_reduce_lane_groups(lmax, lsum);
            if (g == 0) wave_lse[wm * BT + bl] = make_float2(lmax, lsum);
        }
    }
    __syncthreads();
    // one candidate per (batch row, candidate tile of 128 ids): merge the waves that share the tile
    constexpr int WPT = Cfg::kWavesPerCandTile;
    const int cq = tid / BT;                      // candidate tile inside the macro tile
    const int bcol = tid - cq * BT;
    const int ctile = tile * Cfg::kCandTiles + cq;
    if (p.cand_val && tid < BT * Cfg::kCandTiles && b0 + bcol < B && ctile < T) {
        float bv = -__builtin_inff();
        int bi = -1;
#pragma unroll
        for (int w = 0; w < WPT; ++w) {
            const float2 c = wave_cand[(cq * WPT + w) * BT + bcol];
            cand_merge(bv, bi, c.x, __float_as_int(c.y));
        }
        p.cand_val[(size_t)(b0 + bcol) * T + ctile] = bv;
        p.cand_idx[(size_t)(b0 + bcol) * T + ctile] = bi;
        if constexpr (FULL) {
            if (p.lse_max) {
                float m = -__builtin_inff(), sacc = 0.0f;
#pragma unroll
                for (int w = 0; w < WPT; ++w) {
                    const float2 c = wave_lse[(cq * WPT + w) * BT + bcol];
                    lse_merge(m, sacc, c.x, c.y);
                }
                p.lse_max[(size_t)(b0 + bcol) * T + ctile] = m;
                p.lse_sum[(size_t)(b0 + bcol) * T + ctile] = sacc;
            }
        }
    }
}

}  // namespace fs
