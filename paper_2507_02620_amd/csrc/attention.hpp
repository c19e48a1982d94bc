// Tree attention launch interface (see attention.hip).
#pragma once
#include "common.hpp"

constexpr int ATTN_MAX_REQ = 32;

// One request of a batch: its rows [row0, row0 + M) of the stacked q / o / anc arrays, its cache and its lengths.
struct AttnReq {
    const void* kbase;  // K cache of the request (layer 0); V at + stride_kv
    int row0, M;
    int l_glo, L;       // L = l_cache + l_s: slots [0, L) take part
};

struct AttnArgs {
    const void* q;        // [rows][Hq*hd], rows of all requests stacked
    long long layer_off;  // elements from a request's kbase to the layer's K cache
    long long stride_kv, stride_head, stride_tok;
    void* o;              // [rows][Hq*hd] in fragment-major layout (operand of the output projection)
    int Hq, Hkv, hd, G;
    int n_req, rows;      // requests, stacked rows in total
    int max_M, max_L;     // largest M and L of the batch (grid and split plan)
    const uint64_t* anc;  // [rows][FS_ANC_WORDS] ancestor-or-self masks of the segment rows (bit j = S index j of the row's own tree)
    float scale_log2;     // log2(e) / sqrt(hd)
    int n_splits, tiles_per_split, Rpad;
    float* part_o;        // [n_splits][Hkv][Rpad][hd], Rpad >= G * rows; row G * row0 + rho of a request
    float* part_ml;       // [n_splits][Hkv][Rpad][2]
    int nwc;              // compute waves per workgroup (workgroups have at least 4 waves for staging)
    int nset;             // tiles in flight per workgroup for long splits with one row tile per wave (2 .. 4; set by attn_plan)
    int dma;              // >= 2: the direct-to-LDS kernel with that many tile buffers (bf16, head dim 128, one row tile per wave, <= 4 waves)
    AttnReq req[ATTN_MAX_REQ];  // last: the fields above stay within the first cache lines of the kernel-argument segment
};

// slots per LDS tile for a given element size and head dim
static inline int attn_tile_slots(int elem_bytes, int hd) { return elem_bytes * hd >= 512 ? 32 : 64; }

// wgs_override / mtw_override / nset_override > 0 replace the plan's own choice of the workgroup target, of the row tiles per wave and of
// the K/V tiles in flight per workgroup (tuning knobs); dma_override: 0 = plan's choice, 1 = never the direct-to-LDS kernel, 2 .. 4 = that
// kernel with so many tile buffers wherever its shape allows
void attn_plan(int elem_bytes, int hd, int M, int G, int Hkv, int L, int max_splits, int wgs_override, int mtw_override, int nset_override,
               int nwc_override, int dma_override, int* NWC, int* MTW, int* row_blocks, int* n_splits, int* tiles_per_split, int* nset, int* dma);
hipError_t launch_attention(int dtype, const AttnArgs& a, int MTW, int row_blocks, hipStream_t s);
