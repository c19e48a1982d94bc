// Tree attention launch interface (see attention.hip).
#pragma once
#include "common.hpp"

struct AttnArgs {
    const void* q;        // [M][Hq*hd]
    const void* k_layer;  // K cache of this layer; V at + stride_kv
    long long stride_kv, stride_head, stride_tok;
    void* o;              // [M][Hq*hd] in fragment-major layout (operand of the output projection)
    int M, Hq, Hkv, hd, G;
    int l_glo, L;         // L = l_cache + l_s: slots [0, L) take part
    const uint64_t* anc;  // [M][FS_ANC_WORDS] ancestor-or-self masks of the segment rows (bit j = S index j)
    float scale_log2;     // log2(e) / sqrt(hd)
    int n_splits, tiles_per_split, Rpad;
    float* part_o;        // [n_splits][Hkv][Rpad][hd]
    float* part_ml;       // [n_splits][Hkv][Rpad][2]
    int nwc;              // compute waves per workgroup (workgroups have at least 4 waves for staging)
};

// slots per LDS tile for a given element size and head dim
static inline int attn_tile_slots(int elem_bytes, int hd) { return elem_bytes * hd >= 512 ? 32 : 64; }

void attn_plan(int elem_bytes, int hd, int M, int G, int Hkv, int L, int max_splits, int* NWC, int* MTW, int* row_blocks, int* n_splits,
               int* tiles_per_split);
hipError_t launch_attention(int dtype, const AttnArgs& a, int MTW, int row_blocks, hipStream_t s);
