// Skinny-M projection kernels: Y[M, N] = X[M, K] * W^T with M = segment length (<= 64 rows per pass).
// At these row counts every weight byte is used by only M rows, so the kernels are built around one
// coalesced pass over a re-tiled copy of W (the HBM stream is the roofline, the MFMA work rides along).
#pragma once
#include "common.hpp"

enum GemmEpilogue {
    EPI_QKV = 0,    // RMSNorm scale, bias, rotary embedding, write q and the K/V cache rows   (layer step: norm + QKV + RoPE + append)
    EPI_RESID = 1,  // residual add, write the fp32 residual stream and its T-typed copy       (output / down projection)
    EPI_SWIGLU = 2, // RMSNorm scale, silu(gate) * up                                           (gate / up projection)
    EPI_LOGITS = 3  // RMSNorm scale, fp32 logits                                               (LM head)
};

enum PackKind { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATEUP = 2 };

struct GemmArgs {
    const void* X;   // activations, element type T: row-major [M][ldx], or fragment-major (x_frag) with K = ldx
    int x_frag;
    const void* Wp;  // re-tiled weights: [n_groups][nkt][NT][64 lanes][16 bytes]; 4-bit: [n_groups][K/128][NT][64 lanes][16 bytes]
    const void* Sp;  // 4-bit only: scales, bf16 [n_groups][K/128][NT][16 rows]
    // 4-bit only.  The RMSNorm gain cannot be folded into integer codes, so the kernel that produces a normed
    // projection's input multiplies it in (gain_next) and leaves per-tile sums of squares of the un-gained rows
    // (ssp_out); the consumer adds the partial sums up (ssp_in) instead of squaring its activations.
    const float* ssp_in;   // [ssp_n][ssp_stride]: partial sums of squares per row
    int ssp_n, ssp_stride;
    int ldx, M, K, nkt;
    int red_copies;  // set by the launcher: copies of the workgroup's tiles the cross-wave reduction keeps in LDS
    int N;           // valid output features (packed order)
    float eps;
    const float* bias;  // packed order, or null
    // EPI_QKV
    const float2* rope;  // [M][hd/2] (cos, sin)
    void* q_out;         // [M][Hq*hd]
    const unsigned long long* krow;  // [M] address of the row's K cache slot (layer 0, head 0) in its request's cache
    long long layer_off;             // elements from there to this layer's K cache; V at + stride_kv
    long long stride_kv, stride_head;
    int Hq, Hkv, hd;
    // EPI_RESID
    const void* resid;  // [M][N] fp32 residual stream, or T-typed stage input when resid_is_T
    int resid_is_T;
    float* h_out;  // [M][N] fp32
    void* hb_out;  // [M][N] T, fragment-major if hb_frag
    int hb_frag;
    const void* gain_next;  // [N] T or null: hb_out = h * gain_next (the next RMSNorm's gain)
    float* ssp_out;         // [N/16][ssp_stride] or null: sum over the tile's 16 features of h^2, per row
    // EPI_SWIGLU
    void* act_out;  // [M][F] fragment-major
    int F;
    // EPI_LOGITS
    float* logits;  // [M][vocab]
};

struct PackArgs {
    const void* src0;  // PLAIN: W; QKV: wq; GATEUP: w_gate
    const void* src1;  // QKV: wk; GATEUP: w_up
    const void* src2;  // QKV: wv
    const void* gain;  // [K] RMSNorm gain folded into the columns, or null
    void* dst;
    int kind, N, K, nkt, NT, n_groups;
    int Hq, Hkv, hd;
    // bias (QKV only): packed fp32 copy
    const void* b0;
    const void* b1;
    const void* b2;
    float* bias_dst;
};

struct PackW4Args {
    // sources: codes uint8 [N][K/2] (k even in the low nibble), scales bf16 [N][K/128]; slots as in PackArgs
    const void *c0, *c1, *c2, *s0, *s1, *s2;
    void* dst;      // [n_groups][K/128][NT][64][16 B]
    void* sdst;     // bf16 [n_groups][K/128][NT][16]
    int kind, N, K, NT, n_groups;
    int Hq, Hkv, hd;
    const void *b0, *b1, *b2;  // biases (bf16) for QKV
    float* bias_dst;
};

void launch_pack(int dtype, const PackArgs& a, hipStream_t s);
void launch_pack_w4(const PackW4Args& a, hipStream_t s);
// bf16 only.  xg = bf16(X * gain) (gain may be null) fragment-major, rows padded to 16, and partial sums of squares of X
// per 512-column slice, ssp[slice][ssp_stride]; returns the number of slices through n_slices.
hipError_t launch_prenorm(const void* X, int ldx, int M, int K, const void* gain, void* xg, float* ssp, int ssp_stride, int* n_slices,
                             hipStream_t s);
// 4-bit weights, bf16 activations: w[n][k] = scale[n][k/128] * (code - 8)
hipError_t launch_gemm_w4(int epi, int NT, int NW, int n_groups, const GemmArgs& a, hipStream_t s);
// bf16, fragment-major activations: the many-row kernel (128-row blocks; one 64-row block up to 64 rows).  layout_nt and n_tiles
// describe the re-tiled weights (tiles per group, 16-feature tiles in total); normed projections need ssp_in from 384 rows on
// (256-feature blocks; the 128-feature blocks add up the squares of the activations themselves).  `part` (may be null) is scratch for K-split partial results of the d_model-wide
// residual projections (wide_partial_bytes gives a sufficient size for segments of up to max_rows rows and n_tiles output
// tiles); a residual
// projection leaves wide_ssp_parts(M, n_tiles) partial sums of squares per row in ssp_out.
int wide_ssp_parts(int M, int n_tiles);
size_t wide_partial_bytes(int max_rows, int n_tiles);
// block_mode: 0 never / 1 whenever possible / anything else: by rule — use of the 256-row kernel (both operands through LDS) from 384 rows on
hipError_t launch_gemm_wide(int epi, int layout_nt, int n_tiles, const GemmArgs& a, float* part, size_t part_bytes, int block_mode, hipStream_t s);
// MT = ceil(M/16) in {1,2,4}, NT in {1,2,4} (even for QKV / SWIGLU), waves per workgroup NW
hipError_t launch_gemm(int dtype, int epi, int NT, int NW, int n_groups, const GemmArgs& a, hipStream_t s);
