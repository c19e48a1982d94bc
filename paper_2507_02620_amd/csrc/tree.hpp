// Tree bookkeeping, acceptance, KV-cache and segment pruning: launch interface (see tree.hip).
#pragma once
#include "common.hpp"

struct AcceptResultDev {
    int32_t n_acc, x_new, n_new, continuous, n_retain, n_pr_verified;
};

struct CompactArgs {
    void* base;
    long long stride_layer, stride_kv, stride_head, stride_tok;  // elements
    int elem_bytes, n_layers, n_kv_heads, hd;
    int l_glo, l_cache, colblocks;
    const int32_t* retain_dev;         // device list, or null -> use `host` below
    const AcceptResultDev* res_dev;    // counts on the device (with retain_dev)
    int n_retain, n_acc;               // counts for the host list
    int32_t* new_len;                  // optional [2]
};

hipError_t launch_rope_freq(double* inv_freq, int hd, float theta, hipStream_t s);
// Where the segment's K/V rows go: krow[r] = base + (slot0 + r) * tok_bytes, the address of row r's K slot (layer 0, head 0).
struct KRowArgs {
    unsigned long long* krow;  // [l_s]
    unsigned long long base;   // the request's cache
    unsigned long long tok_bytes;
    int slot0;                 // l_cache
};

// anc [l_s][FS_ANC_WORDS], rope [l_s][hd/2], kr.krow [l_s]; max_depth (of the tree, from the host's validation pass) picks the walking kernel
// or, for deep trees, the pointer-doubling one, which needs anc_all [2][seg_off + l_s][FS_ANC_WORDS] as scratch (two copies: each
// round reads one and writes the other).
hipError_t launch_tree_prepare(const IdxList& parent, int max_depth, int l_glo, int seg_off, int l_s, int hd, const double* inv_freq,
                               uint64_t* anc_all, uint64_t* anc, float2* rope, const KRowArgs& kr, hipStream_t s);
hipError_t launch_argmax(const float* logits, int rows, int vocab, int chunks, int32_t* work, int32_t* amax, hipStream_t s);
hipError_t launch_accept(const int32_t* amax, const int32_t* token, const int32_t* parent, int T, int n_ver, AcceptResultDev* res,
                         int32_t* retain, hipStream_t s);
hipError_t launch_accept_sample(const float* logits, int vocab, float inv_temp, const int32_t* token, const int32_t* parent, int T, int n_ver,
                                uint64_t seed, uint64_t step, AcceptResultDev* res, int32_t* retain, void* work, hipStream_t s);
hipError_t launch_kv_compact(const CompactArgs& a, const IdxList& host, hipStream_t s);
hipError_t launch_seg_prune(const void* seg_in, int l_s, size_t row_bytes, int off, const int32_t* retain_dev, const AcceptResultDev* res_dev,
                            const IdxList& host, void* seg_out, int32_t* l_s_out, hipStream_t s);
