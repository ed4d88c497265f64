/*
 * flash_sample.h -- C ABI of the MI355X (gfx950) fused LM-head + exact Gumbel-max sampler.
 *
 * The library draws, for every row b of a batch,
 *
 *        i*_b  ~  Cat( softmax( H_b W^T / tau_b ) )                 (paper, Section
 *                                                                    "FlashSampling Algorithm")
 *
 * by the Gumbel-max identity  i* = argmax_i ( y_i / tau + g_i ),  g_i iid Gumbel(0,1)
 * (Theorem "Gumbel-Max"), evaluated in two stages (Alg. 1 "FlashSampling (two-stages)"):
 *
 *   stage 1  for every vocabulary tile of FS_VOCAB_TILE ids: logits by a tiled bf16 matmul with
 *            fp32 accumulation kept on chip, scaled by 1/tau, perturbed with Gumbel noise, and
 *            reduced to one (max value, global vocabulary id) candidate per (row, tile);
 *   stage 2  argmax over the [B, T] candidate buffer, T = ceil(V / FS_VOCAB_TILE).
 *
 * The [B, V] logits never reach device memory on the fused path.
 *
 * Noise (Section "Further details of FlashSampling", "RNG determinism"; appendix "Numerically
 * Stable and Fast Gumbel Generation"): the 32-bit word for logical position (row, vocab id) is
 * word (id & 3) of Philox4x32-10 with counter (id >> 2, row, 0, 0) and key
 * (lo32(seed), hi32(seed)); x = min(fma((float)r, 2^-32, 2^-33), 1 - 2^-24); u = 1 - x lies in
 * the open interval (0,1); g = -log(-log u) in fp32.  `row` is row_offset + b and `id` is
 * vocab_offset + i, so a batch shard or a vocabulary shard reproduces the unsharded sample.
 * Exact ties go to the lowest vocabulary id (strict > in the appendix Alg. "Gumbel-Max sampling
 * (standalone logits)").  NaN scores never win; a row without any score > -inf returns
 * idx = -1, val = -inf.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; the library neither frees nor
 *     retains them.  `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   - Calls are asynchronous on `stream`; there is no host synchronisation inside.
 *   - hidden is bf16 [B, D] row-major, W is bf16 [V, D] row-major (one row per vocabulary id),
 *     temperature is fp32 [B] with every entry finite and > 0 (not checked: device memory).
 *   - hidden, W and logits must be 16-byte aligned and D a multiple of 8 (128-bit bf16 loads);
 *     other pointers must be aligned to their element type.
 *   - Returns FS_OK or an error code; never throws, never aborts.  Outputs are written only
 *     when FS_OK is returned.  B == 0 is a successful no-op.
 *   - Results are deterministic: the same inputs give the same outputs on every call.
 *   - Entry points that take a workspace allocate nothing and touch only `stream`, so a call can
 *     be recorded into a HIP graph.  The first call that uses a kernel configuration on a device
 *     does one-time set-up (function attributes, an occupancy query): issue one eager call of the
 *     same shape before capturing.  Calls on different streams share no state as long as their
 *     workspaces and outputs differ.
 */
#ifndef FLASH_SAMPLE_H
#define FLASH_SAMPLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FS_VOCAB_TILE 128 /* vocabulary ids per stage-1 candidate */

typedef enum {
    FS_OK = 0,
    FS_ERR_NULL = 1,        /* a required pointer is NULL */
    FS_ERR_SHAPE = 2,       /* B < 0, D <= 0, V <= 0, D % 8 != 0, or an id/row range overflows */
    FS_ERR_ALIGN = 3,       /* a pointer is not aligned as required */
    FS_ERR_WORKSPACE = 4,   /* workspace missing or smaller than flash_sample_workspace_bytes */
    FS_ERR_HIP = 5,         /* a HIP runtime call failed (launch, allocation) */
    FS_ERR_UNSUPPORTED = 6, /* unknown flag or a kernel variant that cannot run this shape */
    FS_ERR_DEVICE = 7,      /* current device ordinal >= 64 (the size of the per-device tables) */
    FS_ERR_SCRATCH_LIMIT = 8 /* flash_sample_static: 8 B T bytes exceed FS_STATIC_SCRATCH_BYTES */
} fs_status;

/* flags for the *_ex entry points */
#define FS_FLAG_NONE 0u
/* Deterministic decoding: no noise is drawn and every row returns the arg max of its transformed
 * logits (lowest id on ties), out_val = that logit.  The tau -> 0 limit of the draw; also what
 * the epilogue costs can be measured against. */
#define FS_FLAG_GREEDY 0x1u
/* Evaluate the Gumbel transform g = -log(-log u) with the device library's log1pf / logf instead
 * of the hardware log2 (the exact-math mode of the appendix "Numerically Stable and Fast Gumbel
 * Generation"; the default is its fast-math mode: series / v_log_f32).  The two modes differ by
 * a few ulp of g, so a draw may differ between them on rows whose top two scores are that close. */
#define FS_FLAG_EXACT_LOG 0x2u
/* bits 8..15: kernel variant for stage 1 (0 = automatic choice).  Every variant computes the
 * same candidates up to fp32 summation order; the tests use them to show tiling invariance. */
#define FS_VARIANT(v) (((uint32_t)(v) & 0xFFu) << 8)
#define FS_VARIANT_AUTO 0   /* B <= 16 and D <= 4096: FS_VARIANT_SPLITK; otherwise FS_VARIANT_TILED2 */
/* B <= 16, D <= 4096: the contraction dimension is split over the waves of a workgroup and each
 * wave keeps its slice of the hidden states in registers (32 k-steps of 32 elements per wave). */
#define FS_VARIANT_SPLITK 2
/* any B, any D: LDS-tiled {128,256,512} x {32,64,128,256} tiles, one or two register sets of
 * prefetch, XCD-paired batch tiles */
#define FS_VARIANT_TILED2 7
/* bits 16..19: tuning aid.  FS_VARIANT_SPLITK: workgroups per compute unit (0 = automatic).
 * FS_VARIANT_TILED2: tile shape (vocabulary rows x batch rows, waves), 0 = automatic,
 * 1 = 128x32 (4 waves), 2 = 256x64 (8), 3 = 256x128 (8), 4 = 128x128 (4), 5 = 128x64 (4),
 * 6 = 512x32 (8), 7 = 512x64 (8), 8 = 256x32 (4), 10 = 512x128 (8), 12 = 256x256 and 13 = 256x128 (4 waves,
 * tiles loaded from global memory straight into LDS).  A hidden size that is not a multiple of 64 always runs on
 * shapes 8, 5 or 4 (by batch size). */
#define FS_TUNE_WGS_PER_CU(n) (((uint32_t)(n) & 0xFu) << 16)
#define FS_TUNE_TILE_SHAPE(n) FS_TUNE_WGS_PER_CU(n)

/* Number of stage-1 candidates per row, T = ceil(V / FS_VOCAB_TILE). */
int flash_sample_num_tiles(int V);

/* Bytes of device workspace the *_ex entry points need for (B, V): the candidate buffer of
 * Alg. 1 (one fp32 value and one int32 id per row and vocabulary tile), 256-byte aligned parts. */
size_t flash_sample_workspace_bytes(int B, int V);

/*
 * Draw one vocabulary id per row: i*_b ~ Cat(softmax(hidden_b W^T / temperature_b)).
 *   out_idx [B] int32   0-based vocabulary id
 *   out_val [B] fp32    the winning perturbed score y/tau + g
 * One seed for all rows (rows are separated by the row word of the counter).  Runs on the null
 * stream and uses a workspace cached inside the library (grown with hipMalloc when a call needs
 * more than any earlier one on this device; never shrunk).
 */
fs_status flash_sample(const void* hidden, const void* W, int B, int D, int V,
                       const float* temperature, uint64_t seed,
                       int32_t* out_idx, float* out_val);

/*
 * Same operation with everything explicit.
 *   row_seeds    NULL, or [B] uint64: row b draws with row_seeds[b] instead of `seed`
 *   row_offset   added to b to form the row word of the noise counter (batch sharding)
 *   vocab_offset added to i to form the vocabulary id used by the noise and returned in
 *                out_idx (vocabulary sharding); vocab_offset >= 0, vocab_offset + V <= 2^31 - 1
 *   workspace    device buffer of at least flash_sample_workspace_bytes(B, V) bytes, 256-byte
 *                aligned; contents are overwritten; must not be shared by overlapping calls
 *   flags        FS_FLAG_NONE or FS_VARIANT(...)
 */
fs_status flash_sample_ex(const void* hidden, const void* W, int B, int D, int V,
                          const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                          int64_t row_offset, int32_t vocab_offset,
                          int32_t* out_idx, float* out_val,
                          void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/*
 * flash_sample_ex for callers that cannot allocate and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The candidate buffer of
 * Alg. 1 lives in a device array built into the library (FS_STATIC_SCRATCH_BYTES per device, held
 * until the process ends); the call allocates nothing and calls no allocating routine.
 *   - needs flash_sample_workspace_bytes(B, V) <= FS_STATIC_SCRATCH_BYTES (e.g. B = 512 at
 *     V = 129280), else FS_ERR_SCRATCH_LIMIT and nothing is launched;
 *   - the first call on a device looks up the array's address (hipGetSymbolAddress) and does the
 *     kernels' one-time set-up: make it outside any capture;
 *   - every call on a device uses that device's one array: calls that overlap in time on one device
 *     (different streams, or threads) race on it -- keep them on one stream, or use
 *     flash_sample_ex with separate workspaces.  Nothing in the array has to be cleared between
 *     calls: stage 1 writes every entry stage 2 reads.
 * All other arguments, results and error codes as in flash_sample_ex.
 */
#define FS_STATIC_SCRATCH_BYTES (8u << 20)
fs_status flash_sample_static(const void* hidden, const void* W, int B, int D, int V,
                              const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                              int64_t row_offset, int32_t vocab_offset,
                              int32_t* out_idx, float* out_val, void* stream, uint32_t flags);

/*
 * The same draw with the whole deterministic transform of the paper's notation ("additive bias,
 * temperature scaling, or masking", Section "Background"; Alg. 1, "transform"; Section "Top-k,
 * Nucleus Sampling, and Masking": forbidden ids are set to -inf before perturbation) and,
 * optionally, the log-normaliser (appendix "Returning Log-Normalizers or Max Values"):
 *      z_{b,i} = (y_{b,i} + bias_i) / temperature_b     if id i is allowed for row b, else -inf
 *      i*_b ~ Cat(softmax(z_b)),   out_val[b] = max_i (z_{b,i} + g_{b,i}),
 *      out_lse[b] = log sum_i exp(z_{b,i})
 *   bias               NULL, or fp32 [V] (indexed by the local id i), 16-byte aligned
 *   allowed            NULL (all allowed), or bit rows: bit (i % 32) of 32-bit word (i / 32) set
 *                      means local id i may be sampled; padding bits past V are ignored
 *   mask_stride_words  32-bit words between the bit rows of consecutive batch rows
 *                      (>= ceil(V/32)), or 0: one bit row shared by every batch row
 *   out_lse            NULL, or fp32 [B]
 *   workspace          at least flash_sample_full_workspace_bytes(B, V) bytes, 256-byte aligned
 *   flags              FS_FLAG_NONE, FS_FLAG_GREEDY, FS_FLAG_EXACT_LOG (the automatic kernel choice only)
 * A row whose ids are all masked returns idx = -1, val = -inf, lse = -inf.  The order
 * bias -> temperature -> mask is this library's reading; the paper does not fix it.
 */
size_t flash_sample_full_workspace_bytes(int B, int V);
fs_status flash_sample_full(const void* hidden, const void* W, int B, int D, int V,
                            const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                            int64_t row_offset, int32_t vocab_offset,
                            const float* bias, const uint32_t* allowed, int64_t mask_stride_words,
                            int32_t* out_idx, float* out_val, float* out_lse,
                            void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/*
 * Truncated supports (Section "Top-k, Nucleus Sampling, and Masking": the scheme given there is
 * per-tile candidate lists merged by a second stage into the k best of the row, with the nucleus
 * rule run on those k; the implementation is left open).  With
 * z_{b,i} = y_{b,i} / temperature_b and the per-id noise g of the main path:
 *   FS_TOPK_TRUNCATE  S_b = the k ids with the largest z (ties: lower id first).  If top_p < 1 the
 *                     candidates, in that order, get q_j = softmax over S_b, and only the shortest
 *                     prefix whose mass reaches top_p is kept (at least one).  The draw is
 *                     i*_b = argmax over the kept ids of z + g: an exact sample of the softmax
 *                     restricted to them (it is the masked draw of flash_sample_full with every other
 *                     id forbidden).  out_val = the winning perturbed score.
 *   FS_TOPK_GUMBEL    the k ids with the largest perturbed scores z + g, in descending order: a draw of
 *                     k ids without replacement (the Gumbel-top-k trick); out_idx / out_val are its
 *                     first element, which is exactly flash_sample_ex's sample.  top_p must be 1.
 *   k          1 .. FS_TOPK_MAX_K;  top_p in (0, 1]
 *   topk_val   NULL, or fp32 [B, k]: the keys of the k candidates in order (z, or z + g)
 *   topk_idx   NULL, or int32 [B, k]: their global ids; slots past V are (-inf, -1)
 *   n_kept     NULL, or int32 [B]: candidates kept by the nucleus rule (those with a key > -inf)
 *   workspace  at least flash_sample_topk_workspace_bytes(B, V, k) bytes, 256-byte aligned
 *   flags      FS_FLAG_NONE or FS_FLAG_EXACT_LOG; flash_sample_topk also takes, as a tuning aid,
 *              FS_TUNE_TILE_SHAPE(n) for its stage 1 (n = 1..8, 10, 12, 13: the tile shapes listed at
 *              FS_VARIANT_TILED2 above); 0 = automatic: split-K for B <= 16 and D <= 4096, else the shape the
 *              plain path takes, with 13 in place of 3 and 4
 * NaN logits count as -inf.  flash_sample_topk is the fused form: the [B, V] logits never reach device
 * memory.  Stage 1 writes the min(k, m) best candidates of every row and 128-id tile (m = 8 for
 * B <= 32, 4 above) and a selection reduces them to k per row.  For k > m a tile whose m-th candidate
 * is among a row's k may hold more of them (no other tile can): the last selection level recomputes
 * the 128 keys of just those tiles (at most k / m per row; none for typical logits) from the row's
 * hidden state and W by plain fp32
 * dot products and selects again, so the result is the top k for any input.  It needs D % 64 == 0
 * (FS_ERR_UNSUPPORTED otherwise).  flash_sample_topk_unfused is the comparison form for any D: the
 * logits-store GEMM writes `logits` (fp32 [B, V], the raw logits y), and the same selection runs over
 * the stored rows, forming the keys as it reads.  Same results up to fp32 rounding.
 */
#define FS_TOPK_TRUNCATE 0
#define FS_TOPK_GUMBEL 1
#define FS_TOPK_MAX_K 64
size_t flash_sample_topk_workspace_bytes(int B, int V, int k);
fs_status flash_sample_topk(const void* hidden, const void* W, int B, int D, int V,
                            const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                            int64_t row_offset, int32_t vocab_offset, int k, float top_p, int mode,
                            int32_t* out_idx, float* out_val, float* topk_val, int32_t* topk_idx, int32_t* n_kept,
                            void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);
fs_status flash_sample_topk_unfused(const void* hidden, const void* W, int B, int D, int V,
                                    const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                                    int64_t row_offset, int32_t vocab_offset, int k, float top_p, int mode,
                                    float* logits, int32_t* out_idx, float* out_val, float* topk_val,
                                    int32_t* topk_idx, int32_t* n_kept,
                                    void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/*
 * Grouped variants (Section "Group-Gumbel-Max: Hierarchical Exact Sampling"; appendix algorithms
 * "FlashSampling (parallel)" and "FlashSampling (sequential/online)").  The vocabulary is cut
 * into groups of 128 * group_tiles consecutive ids (the last group may be shorter).  Stage 1 is
 * the fused kernel of flash_sample_full; per group k it yields the local sample z_k (Gumbel-max
 * inside the group, same per-id noise as the default path) and the group log-mass
 * L_k = log sum_{i in group} exp(z_i).  The group is then chosen with independent noise:
 *   FS_GROUPED_PARALLEL  k* = argmax_k (L_k - log(-log ubar_k)), lowest k on ties
 *   FS_GROUPED_ONLINE    groups taken in ascending order with a running log-mass ell; group k
 *                        replaces the running sample when u_k < exp(L_k - log(e^ell + e^L_k))
 * and out_idx[b] = z_{k*}, out_lse[b] = log sum_k exp(L_k).  Zero-mass groups are skipped.  Both
 * are exact samples of Cat(softmax(z_b)) but, unlike the default path, not the same draw as a
 * Gumbel-max over the whole row.  ubar_k / u_k are word (k & 3) of
 * Philox4x32-10(counter = (k >> 2, row word, 1 / 2, 0)) with the row's key, k the global group id
 * (vocab_offset / (128 * group_tiles) + local group), mapped to (0,1) like the per-id noise.
 *   group_tiles        >= 1; vocab_offset must be a multiple of 128 * group_tiles
 *   out_lse            NULL, or fp32 [B]
 *   group_log_mass     NULL, or fp32 [B, m], m = flash_sample_num_groups(V, group_tiles): L_k
 *   group_sample       NULL, or int32 [B, m]: z_k as a global id, -1 for a zero-mass group
 *                      (one (L_k, z_k) pair per group is what a vocabulary-sharded deployment
 *                      exchanges between ranks, see flash_group_choose)
 *   workspace          at least flash_sample_full_workspace_bytes(B, V) bytes, 256-byte aligned
 * Other arguments as in flash_sample_full.  A row with no mass returns idx = -1, lse = -inf.
 */
#define FS_GROUPED_PARALLEL 0
#define FS_GROUPED_ONLINE 1
int flash_sample_num_groups(int V, int group_tiles);
fs_status flash_sample_grouped(const void* hidden, const void* W, int B, int D, int V,
                               const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                               int64_t row_offset, int32_t vocab_offset,
                               const float* bias, const uint32_t* allowed, int64_t mask_stride_words,
                               int group_tiles, int mode,
                               int32_t* out_idx, float* out_lse,
                               float* group_log_mass, int32_t* group_sample,
                               void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/*
 * The group choice alone, from per-group summaries: the coordinator step of the distributed
 * variant (appendix algorithm "FlashSampling (distributed, tensor-parallel vocab)"), where group
 * k is rank k's vocabulary shard and each rank contributes its shard log-mass and local sample.
 *   group_log_mass [B, m] fp32   L_k (-inf for a zero-mass group)
 *   group_sample   [B, m] int32  z_k as a global id (-1 for a zero-mass group)
 *   group_offset   global id of the first group (the noise is indexed by global group ids)
 *   out_idx [B] int32, out_lse NULL or [B] fp32
 * Same choice rule and noise as flash_sample_grouped; no workspace.
 */
fs_status flash_group_choose(const float* group_log_mass, const int32_t* group_sample, int B, int m,
                             int mode, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                             int64_t group_offset, int32_t* out_idx, float* out_lse, void* stream);

/*
 * The same draw on FP8 weights (Section "Limitations and Future Work" names lower-precision
 * weights as the next saving: W is the dominant 2 V D byte term of the bandwidth-bound regime).
 * This library's reading: W8 [V, D] holds OCP FP8 E4M3 codes (one byte per element, row-major),
 * w_scale [V] one fp32 scale per vocabulary row (NULL = all ones), hidden stays bf16:
 *      y_{b,i} = w_scale_i * sum_d hidden[b,d] * e4m3(W8[i,d]),   i*_b ~ Cat(softmax(y_b / temperature_b))
 * The codes are widened to bf16 on chip (exactly: every E4M3 value is a bf16 value) and contracted
 * with the same bf16 MFMA as the bf16 path, so the arithmetic and its tolerance are those of
 * flash_sample_ex on the decoded weights; noise, tie-breaking and outputs are identical.
 *   W8, w_scale   device pointers, 16-byte aligned; D % 16 == 0
 *   logits        NULL, or fp32 [B, V]: also store y (for tests and the comparison path)
 *   workspace     at least flash_sample_workspace_bytes(B, V) bytes, 256-byte aligned
 *   flags         FS_FLAG_NONE, FS_FLAG_GREEDY, FS_FLAG_EXACT_LOG; or, as a tuning aid, FS_VARIANT_SPLITK
 *                 (B <= 16, D <= 8192) / FS_VARIANT_TILED2 with FS_TUNE_TILE_SHAPE (shapes 10 and 12
 *                 run as shape 3; D % 128 != 0 always runs on shapes 8, 5 or 4)
 * NaN codes (S.1111.111) propagate to NaN logits, which never win.
 */
fs_status flash_sample_w8(const void* hidden, const void* W8, const float* w_scale, int B, int D, int V,
                          const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                          int64_t row_offset, int32_t vocab_offset, float* logits,
                          int32_t* out_idx, float* out_val,
                          void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/*
 * The same draw on MXFP4 weights (OCP microscaling FP4, the other lower-precision format the paper
 * names): W4 [V, D/2] bytes holds FP4 E2M1 codes, two per byte (element 2j of a row in the low
 * nibble of byte j); w_scales [V, D/32] bytes holds one E8M0 scale per 32 consecutive elements of
 * a row, worth 2^(e - 127); hidden stays bf16:
 *      y_{b,i} = sum_d hidden[b,d] * e2m1(W4[i,d]) * 2^(w_scales[i, d/32] - 127)
 * Codes and scale are combined into bf16 values on chip (exactly), then contracted like the bf16
 * path.  D must be a multiple of 256 (FS_ERR_UNSUPPORTED otherwise).  Two kernels: the split-K form
 * of the bandwidth-bound decode regime (B <= 16 and D % 512 == 0, D <= 4096, or D % 1024 == 0,
 * D <= 8192), and a tiled form with the codes and scale bytes kept in LDS for everything else (any B;
 * it pays off up to B = 64, where the call is still bound by the W bytes, which is all MXFP4 saves).
 *   W4, w_scales   device pointers, 16-byte aligned; scale bytes above 252 must not occur (253 and
 *                  254 overflow the bf16 range of a scaled element, 255 is NaN)
 *   logits         NULL, or fp32 [B, V]: also store y
 *   workspace      at least flash_sample_workspace_bytes(B, V) bytes, 256-byte aligned
 *   flags          FS_FLAG_NONE, FS_FLAG_GREEDY, FS_FLAG_EXACT_LOG, FS_TUNE_WGS_PER_CU(n)
 */
fs_status flash_sample_w4(const void* hidden, const void* W4, const void* w_scales, int B, int D, int V,
                          const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                          int64_t row_offset, int32_t vocab_offset, float* logits,
                          int32_t* out_idx, float* out_val,
                          void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/* Debug tap: the on-chip MXFP4 -> bf16 conversion: out[8 k + j] = e2m1(nibble j of dword k of
 * codes) * 2^(scales[k] - 127) for k < n8 (codes 4-byte aligned), widened to fp32. */
fs_status flash_sample_mxfp4_decode(const void* codes, const uint8_t* scales, int n8, float* out, void* stream);

/* Debug tap: the on-chip E4M3 -> bf16 conversion applied to n codes (n % 8 == 0, codes 8-byte
 * aligned), widened to fp32 out[n]. */
fs_status flash_sample_e4m3_decode(const uint8_t* codes, int n, float* out, void* stream);

/*
 * Stage 1 of Alg. 1 alone: writes the candidate buffer
 *   cand_val [B, T] fp32, cand_idx [B, T] int32 (global vocabulary ids), T = flash_sample_num_tiles(V).
 * If `logits` is not NULL the kernel also stores the raw logits y = hidden W^T as fp32 [B, V]
 * (the paper's logits-store flag, Section "IO Cost Model and Predicted Speedup" and appendix
 * "Logits-Store Ablation"); nothing else in the kernel changes.
 */
fs_status flash_sample_stage1(const void* hidden, const void* W, int B, int D, int V,
                              const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                              int64_t row_offset, int32_t vocab_offset,
                              float* cand_val, int32_t* cand_idx, float* logits,
                              void* stream, uint32_t flags);

/* Stage 2 of Alg. 1 alone: out[b] = candidate with the largest value over t in [0, T), lowest
 * id on exact ties.  cand_val / cand_idx are [B, T]. */
fs_status flash_sample_stage2(const float* cand_val, const int32_t* cand_idx, int B, int T,
                              int32_t* out_idx, float* out_val, void* stream);

/*
 * Unfused comparison path (the materialised-logits pipeline the paper's IO model calls the
 * baseline, Section "IO Cost Model and Predicted Speedup"): a GEMM kernel writes fp32 logits
 * [B, V] to device memory, a separate kernel re-reads them and runs streaming Gumbel-max
 * (appendix Alg. "Gumbel-Max sampling (standalone logits)"), and the tile argmax finishes.
 * Same noise, same result as flash_sample_ex up to fp32 rounding of the score.
 *   logits  [B, V] fp32 device buffer, 16-byte aligned, overwritten
 */
fs_status flash_sample_unfused(const void* hidden, const void* W, int B, int D, int V,
                               const float* temperature, uint64_t seed, const uint64_t* row_seeds,
                               int64_t row_offset, int32_t vocab_offset, float* logits,
                               int32_t* out_idx, float* out_val,
                               void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/* First half of the unfused path alone: logits[b, i] = sum_d hidden[b, d] * W[i, d] (fp32). */
fs_status flash_lm_head_logits(const void* hidden, const void* W, int B, int D, int V,
                               float* logits, void* stream, uint32_t flags);

/* Second half of the unfused path alone: Gumbel-max over stored fp32 logits [B, V]. */
fs_status flash_gumbel_argmax_logits(const float* logits, int B, int V, const float* temperature,
                                     uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                                     int32_t vocab_offset, int32_t* out_idx, float* out_val,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Debug tap: g_out[k] = Gumbel noise the stage-1 epilogue uses for (seed, row, v0 + k), k < n
 * (Alg. 1, "Draw u in (0,1) and set g = -log(-log u)").  g_out is an fp32 [n] device buffer. */
fs_status flash_sample_noise(uint64_t seed, int64_t row, int32_t v0, int n, float* g_out,
                             void* stream);

/* Debug tap of the uniform -> Gumbel map alone: g_out[k] = g(words[k]) for 32-bit words given by
 * the caller (device arrays of n elements), so a test can sweep every exponent and the edge words. */
fs_status flash_sample_gumbel_transform(const uint32_t* words, int n, float* g_out, void* stream,
                                        uint32_t flags /* FS_FLAG_NONE or FS_FLAG_EXACT_LOG */);

/* Static description of an error code (never NULL). */
const char* fs_status_string(fs_status s);

#ifdef __cplusplus
}
#endif
#endif /* FLASH_SAMPLE_H */
