// Stage 1 of Alg. 1 on MXFP4 weights (OCP microscaling FP4: E2M1 codes, two per byte, one E8M0
// scale byte per block of 32 elements of a row), B <= 16.  Lower-precision weights are what the
// paper names as the next saving in the bandwidth-bound regime; here W shrinks to D/2 + D/32 bytes
// per vocabulary row.
//
// Same design as the split-K kernel of the bf16 path (persistent workgroups, waves split K, the
// wave's hidden slice in registers, W: coalesced non-temporal 16-byte loads -> registers ->
// wave-private swizzled LDS stage -> MFMA operand layout), with these differences:
//  * one 16-byte load is exactly one K step (32 codes) of one row, so a wave's 16 (or 32) K steps are 256 (512)
//    bytes of a row; a row-tile of 16 rows is one 4 (8) KB stage, and the prefetch runs PFD whole
//    row-tiles ahead (the loop over row-tiles is unrolled PFD times so that the register sets
//    rotate statically);
//  * a lane's MFMA operand (8 codes of row n) is one ds_read_b32; it is widened to bf16 by four
//    v_cvt_scalef32_pk_bf16_fp4, which also apply the block scale (a power of two: exact);
//  * the scale bytes of (row n, this wave's K steps) are one or two more 16-byte loads per lane
//    and row-tile, straight into registers.
// Each scaled element is a bf16 value, so the products and the fp32 accumulation are those of the
// bf16 path on the dequantised weights.
#pragma once

#include "fs_common.hpp"
#include "fs_stage1_splitk.hpp"   // splitk_finish_tile

namespace fs {

// KPW: K steps (of 32 elements) per wave, 16 or 32; a stage is 16 rows x KPW * 16 bytes.
constexpr size_t w4_lds_bytes(int kpw, int nw)
{
    return (size_t)nw * (16 * kpw * 16) + (size_t)8 * nw * 1024 + (size_t)nw * 16 * 8 * 2;
}

// KPW: K steps per wave (16: hidden slice in 64 VGPRs, 32: in 128); MAXW: waves per workgroup
// (= D / (32 KPW)); PFD: row-tiles of W in flight per wave.
// p.W points at the codes [V, D/2] bytes, w_scales at the E8M0 bytes [V, D/32].
template <int KPW, int MAXW, int PFD, bool FULL = false>
__global__ void __launch_bounds__(MAXW * kWave)
stage1_w4_kernel(const Stage1Params p, const uint8_t* __restrict__ w_scales, const int nw)
{
    static_assert(KPW == 16 || KPW == 32, "16 or 32 K steps per wave");
    constexpr int ROWB = KPW * 16;            // bytes of one row inside a stage
    constexpr int RPI = kWave / KPW;          // rows one load instruction covers (4 or 2)
    constexpr int NI = 16 / RPI;              // load instructions per stage (4 or 8)
    constexpr int NS = KPW / 16;              // 16-byte loads of scale bytes per lane and row-tile
    constexpr int kStageBytes = 16 * ROWB;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;
    const int B = p.B, D = p.D, V = p.V;
    const int rowbytes = D >> 1;              // code bytes per vocabulary row
    const int scalebytes = D >> 5;            // scale bytes per vocabulary row

    const int ks0 = wave * KPW;               // this wave's first K step; D % 512 == 0: all waves full
    const int kbeg = ks0 * 32;

    unsigned char* stage = smem + (size_t)wave * kStageBytes;
    f32x4* partial = reinterpret_cast<f32x4*>(smem + (size_t)nw * kStageBytes);
    float2* wave_cand = reinterpret_cast<float2*>(smem + (size_t)nw * kStageBytes + (size_t)8 * nw * 1024);
    float2* wave_lse = wave_cand + nw * 16;

    RowEpi repi = {1.0f, p.seed, (uint32_t)(uint64_t)(p.row_offset + n), nullptr};
    if (n < B && p.cand_val) repi = make_row_epi<FULL>(p, n);

    const int T = p.T;
    const int ntiles = ((int)blockIdx.x < T) ? (T - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    const int nrt = ntiles * 8;               // row-tiles of 16 rows; a multiple of 8, hence of PFD

    const int ld_row = lane / KPW;            // row within one load instruction
    const int ld_chunk = lane % KPW;          // K step (16-byte chunk) within the wave's range

    uint4 wreg[PFD][NI];
    uint4 sreg[PFD][NS];

    // first vocabulary row of row-tile rtl of this workgroup; past the end: rows 0..15 (cache hits)
    auto row_base = [&](int rtl) -> int {
        if (rtl >= nrt) return 0;
        return ((int)blockIdx.x + (rtl >> 3) * (int)gridDim.x) * kVocabTile + (rtl & 7) * 16;
    };
    // All loads are unconditional (rows past V re-read row V - 1 and only feed masked outputs).
    // 32 steps per wave: address = a base that is uniform over the wave (the row-tile's first row, in
    // scalar registers) + a 32-bit lane offset inside the row-tile, so that no 64-bit address lives in
    // vector registers (the kernel has none to spare); 16 steps per wave: plain per-lane addresses,
    // which the compiler keeps in registers across row-tiles (measured 3 % faster there).
    auto issue_loads = [&](uint4 (&dst)[NI], uint4 (&sdst)[NS], int rtl) {
        if constexpr (KPW == 32) {
            const int rb = __builtin_amdgcn_readfirstlane(row_base(rtl));
            const uint32_t last = (uint32_t)(V - 1 - rb);      // rows of this tile past `last` do not exist
            const unsigned char* src = reinterpret_cast<const unsigned char*>(p.W) + (size_t)rb * rowbytes;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                uint32_t r = (uint32_t)(j * RPI + ld_row);
                r = r < last ? r : last;
                const uint32_t off = r * (uint32_t)rowbytes + (uint32_t)(ks0 + ld_chunk) * 16u;
                dst[j] = ld_global_16B_stream(reinterpret_cast<const uint16_t*>(src + off));
            }
            const unsigned char* ssrc = w_scales + (size_t)rb * scalebytes;
            uint32_t sr = (uint32_t)n;
            sr = sr < last ? sr : last;
#pragma unroll
            for (int u = 0; u < NS; ++u)
                sdst[u] = ld_global_16B(reinterpret_cast<const uint16_t*>(ssrc + sr * (uint32_t)scalebytes + (uint32_t)(ks0 + 16 * u)));
        } else {
            const int rb = row_base(rtl);
            const unsigned char* src = reinterpret_cast<const unsigned char*>(p.W) + (size_t)(ks0 + ld_chunk) * 16;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                int row = rb + j * RPI + ld_row;
                row = row < V - 1 ? row : V - 1;
                dst[j] = ld_global_16B_stream(reinterpret_cast<const uint16_t*>(src + (size_t)row * rowbytes));
            }
            int srow = rb + n;
            srow = srow < V - 1 ? srow : V - 1;
#pragma unroll
            for (int u = 0; u < NS; ++u)
                sdst[u] = ld_global_16B(reinterpret_cast<const uint16_t*>(w_scales + (size_t)srow * scalebytes + ks0 + 16 * u));
        }
    };

    // LDS stage: [16 rows][ROWB bytes], 16-byte chunk c of row r in slot c ^ r
    const int st_base = ld_row * ROWB + ((ld_chunk ^ ld_row) << 4);
    auto st_off = [&](int j) -> int {      // 32 steps per wave: recomputed at every use (see the reads below)
        int sb = st_base;
        if constexpr (KPW == 32) asm volatile("" : "+v"(sb));
        return (sb ^ (((j * RPI) & 15) << 4)) + j * RPI * ROWB;
    };
    const int rd_off = n * ROWB + (g << 2);

#pragma unroll
    for (int q = 0; q < PFD; ++q) issue_loads(wreg[q], sreg[q], q);

    // hidden slice in B-operand layout: lane (n, g) holds H[n, k .. k+8), k = kbeg + 32 s + 8 g
    bf16x8 hreg[KPW];
#pragma unroll
    for (int s = 0; s < KPW; ++s) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (n < B) v = ld_global_16B(p.H + (size_t)n * D + kbeg + s * 32 + g * 8);
        hreg[s] = __builtin_bit_cast(bf16x8, v);
    }

    for (int rtl0 = 0; rtl0 < nrt; rtl0 += PFD) {
#pragma unroll
        for (int q = 0; q < PFD; ++q) {
            const int rtl = rtl0 + q;
#pragma unroll
            for (int j = 0; j < NI; ++j) *reinterpret_cast<uint4*>(stage + st_off(j)) = wreg[q][j];
            uint32_t scw[4 * NS];
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                scw[4 * u] = sreg[q][u].x; scw[4 * u + 1] = sreg[q][u].y;
                scw[4 * u + 2] = sreg[q][u].z; scw[4 * u + 3] = sreg[q][u].w;
            }
            issue_loads(wreg[q], sreg[q], rtl + PFD);   // refill this set with the row-tile PFD ahead
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KPW; ++s) {
                // slot (s ^ n) of row n: the XOR is redone here (one instruction) rather than kept as KPW
                // loop-invariant offsets in registers, which is what pushed the 32-step kernel into scratch
                // (the 16-step kernel has the registers and is 6 % faster with the offsets kept)
                uint32_t nx = (uint32_t)n << 4;
                if constexpr (KPW == 32) asm volatile("" : "+v"(nx));
                const uint32_t codes = *reinterpret_cast<const uint32_t*>(stage + rd_off + (((uint32_t)s << 4) ^ nx));
                const uint32_t e = (scw[s >> 2] >> (8 * (s & 3))) & 0xFFu;
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mxfp4x8_to_bf16x8(codes, e), hreg[s], acc, 0, 0, 0);
            }
            const int rt = rtl & 7;
            partial[(rt * nw + wave) * 64 + lane] = acc;
            if (rt == 7) {
                const int tile = (int)blockIdx.x + (rtl >> 3) * (int)gridDim.x;
                splitk_finish_tile<FULL, false>(p, repi, partial, wave_cand, wave_lse, nw, wave, lane, tile);
            }
        }
    }
}

// Decode tap: the on-chip MXFP4 -> bf16 conversion on caller-given data, eight codes per thread.
__global__ void __launch_bounds__(256)
mxfp4_decode_kernel(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales, int n8,
                    float* __restrict__ out)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= n8) return;
    const bf16x8 v = mxfp4x8_to_bf16x8(codes[k], scales[k]);
    const uint4 bits = __builtin_bit_cast(uint4, v);
    const uint32_t w[4] = {bits.x, bits.y, bits.z, bits.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        out[8 * k + 2 * j] = __uint_as_float(w[j] << 16);
        out[8 * k + 2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
    }
}

}  // namespace fs
