/*
 * flowspec.h — C ABI of the MI355X (gfx950) tree-verification stage library.
 *
 * One FlowSpec verification stage V_n (paper, Sec. III-A): a block of decoder layers of the base
 * model run over one segment of the draft sequence S (draft-tree nodes in descending
 * cumulative-score order, Sec. III-B) with tree attention against the stage's KV cache, followed
 * — at the last stage — by next-token scores, acceptance with the continuous condition (Sec.
 * III-C, Eq. 2) and — at every stage — pruning of the KV cache and of in-flight segments by the
 * retain set I_retain (Sec. III-C).
 *
 * Conventions
 *   - Every function returns 0 (FS_OK) or a negative error code; nothing is thrown.
 *   - "device" pointers are HIP device memory owned by the caller (e.g. obtained from PyTorch);
 *     "host" pointers are ordinary host memory.  The library allocates no device memory: all it
 *     needs beyond the caller's tensors lives in the workspace passed to fs_stage_create, whose
 *     size fs_stage_workspace_bytes reports.  The workspace holds a private, re-tiled copy of the
 *     weights, so the caller's weight tensors may be released once fs_stage_create's stream work
 *     has finished.
 *   - All GPU work is enqueued on the caller's stream (hipStream_t passed as void*; NULL is the
 *     default stream) and is asynchronous to the host.  Only fs_accept_result_to_host waits.
 *   - A stage object is used by one stream at a time; calls on one stage that overlap in time race
 *     on its workspace.
 *   - Element type of weights, activations and KV cache is given by fs_stage_desc.dtype:
 *     FS_F32 (float) or FS_BF16 (bfloat16).  Accumulation and the residual stream are fp32.
 *   - S indices: node j of the current draft sequence lives at KV slot l_glo + j, where l_glo is
 *     the global context offset (prompt + accepted tokens, Sec. III-C).
 */
#ifndef FLOWSPEC_H
#define FLOWSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FS_OK 0
#define FS_EINVAL (-1) /* null pointer, bad shape or size, unmet precondition */
#define FS_ETOPO (-2)  /* parent array is not a topological order: needs parent[0] == -1 (verify) and -1 <= parent[i] < i */
#define FS_ECAP (-3)   /* l_cache + l_s exceeds kv_capacity, tree larger than max_tree, segment longer than max_seg */
#define FS_EDTYPE (-4) /* dtype is neither FS_F32 nor FS_BF16 */
#define FS_EHIP (-5)   /* a HIP call failed; fs_last_hip_error() returns its hipError_t */
#define FS_EWS (-6)    /* workspace missing, misaligned (256 B) or smaller than fs_stage_workspace_bytes */

#define FS_F32 0
#define FS_BF16 1

/* weight formats (fs_stage_desc.weight_format) */
#define FS_WFMT_DENSE 0     /* weights of element type dtype */
#define FS_WFMT_INT4_G128 1 /* W4A16 (the paper's 13B setting, Sec. IV-A / Appendix): 4-bit codes + bf16 scales per 128 input columns,
                               w[n][k] = scale[n][k/128] * (code[n][k] - 8); activations, KV cache and arithmetic stay bf16 / fp32.
                               Each weight pointer is a uint8 [out, in/2] array (column k even in the low nibble) and each scale pointer
                               a bf16 [out, in/128] array; d_model, d_ffn and n_q_heads*head_dim must be multiples of 128. */

#define FS_MAX_TREE 1024 /* largest draft tree (nodes of S) any entry point accepts */

/* Shape of a stage (decoder form per Appendix A and the LLaMA2 / Qwen2 models of Sec. IV-A). */
typedef struct {
    int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn;
    int vocab;       /* > 0: last stage with an LM head of that many rows; 0: no head */
    int dtype;       /* FS_F32 | FS_BF16 */
    float rms_eps;   /* RMSNorm epsilon */
    float rope_theta;/* rotary base; element t pairs with t + head_dim/2, angle = pos * theta^(-2t/head_dim) */
    int kv_capacity; /* slots per head of the KV cache the stage will be used with */
    int max_tree;    /* largest T (<= FS_MAX_TREE) */
    int max_seg;     /* largest segment length l_s (the paper's L_max) */
    int weight_format; /* FS_WFMT_DENSE | FS_WFMT_INT4_G128 (requires dtype == FS_BF16) */
} fs_stage_desc;

/* One layer's tensors, device, row-major [out, in], element type desc.dtype.  Biases may be NULL. */
typedef struct {
    const void *rms_attn, *wq, *wk, *wv, *wo, *rms_ffn, *w_gate, *w_up, *w_down;
    const void *bq, *bk, *bv;
    const void *sq, *sk, *sv, *so, *s_gate, *s_up, *s_down; /* FS_WFMT_INT4_G128 only: scales of the seven matrices */
} fs_layer_weights;

/* KV cache, device, element type desc.dtype.  Element (layer, kv, head, slot, t) is at
 * base + layer*stride_layer + kv*stride_kv + head*stride_head + slot*stride_tok + t   (strides in elements,
 * kv = 0 for K — stored after rotation — and 1 for V).  stride_tok must be a multiple of 8 (bf16) / 4 (f32)
 * elements and base 16-byte aligned; one head's slots must span less than 4 GiB (kv_capacity * stride_tok * element size),
 * else FS_EINVAL.  Slots [0, l_cache) are valid. */
typedef struct {
    void *base;
    long long stride_layer, stride_kv, stride_head, stride_tok;
} fs_kv_cache;

typedef struct fs_stage fs_stage;

/* Bytes of device workspace a stage of this shape needs (0 on a bad descriptor). */
size_t fs_stage_workspace_bytes(const fs_stage_desc *desc);

/*
 * Create a stage: validates the shape, re-tiles the weights into the workspace (kernels on `stream`).
 *   layers      host array [n_layers] of device pointers
 *   final_norm  device [d_model], lm_head device [vocab, d_model] (codes for 4-bit weights); both required iff desc->vocab > 0
 *   workspace   device, 256-byte aligned, >= fs_stage_workspace_bytes(desc); owned by the caller and must
 *               outlive the stage
 * Errors: FS_EINVAL, FS_EDTYPE, FS_ECAP (max_tree > FS_MAX_TREE), FS_EWS, FS_EHIP.
 */
int fs_stage_create(const fs_stage_desc *desc, const fs_layer_weights *layers, const void *final_norm, const void *lm_head,
                    const void *lm_head_scale /* FS_WFMT_INT4_G128 with a head, else NULL */, void *workspace, size_t workspace_bytes,
                    void *stream, fs_stage **out);
int fs_stage_destroy(fs_stage *stage);

/*
 * Measurement aid (not part of the method): per-kernel GPU time of the stage's launches.  After
 * fs_stage_profile_begin every kernel the stage enqueues (verify, logits, compact) is bracketed by a pair of
 * HIP events on the caller's stream, up to max_records launches (later ones run untimed).
 * fs_stage_profile_end waits for `stream`, adds up the elapsed milliseconds and launch counts per kernel kind
 * into total_ms[FS_K_COUNT] / counts[FS_K_COUNT] (host arrays) and disarms the profiler.
 * The event records perturb back-to-back timing slightly; throughput is measured with the profiler off.
 */
enum {
    FS_K_PREPARE = 0, /* tree mask, positions, rotary table */
    FS_K_QKV = 1,     /* RMSNorm + Q/K/V projection + RoPE + cache append */
    FS_K_ATTN = 2,    /* tree attention (+ split merge) */
    FS_K_OPROJ = 3,   /* output projection + residual */
    FS_K_GATEUP = 4,  /* RMSNorm + gate/up projection + SiLU*up */
    FS_K_DOWN = 5,    /* down projection + residual */
    FS_K_HEAD = 6,    /* final RMSNorm + LM head */
    FS_K_ARGMAX = 7,  /* row argmax of the logits */
    FS_K_COMPACT = 8, /* KV-cache compaction */
    FS_K_COUNT = 9
};
int fs_stage_profile_begin(fs_stage *stage, int max_records);
int fs_stage_profile_end(fs_stage *stage, void *stream, double *total_ms, long long *counts);

/*
 * Measurement aids (not part of the method): what one launch reaches on this machine, for pricing the kernels against
 * an achievable peak beside the datasheet one.  Both wait for their own launches (HIP events) and are not capturable.
 *   fs_probe_stream_read  one-pass read of bytes_per_launch bytes (a multiple of 256 KiB, >= 1 MiB) with the access
 *                         pattern of the projection kernels' weight stream; consecutive launches rotate through
 *                         buf[0, buf_bytes) (device, 16-byte aligned, >= bytes_per_launch + 64; give several times the
 *                         last-level cache so that no launch finds its data cached).  Result: GB/s of one launch.
 *   fs_probe_mfma_bf16    register-resident loop of independent 16x16x32 bf16 MFMAs on every SIMD; scratch: >= 4 device
 *                         bytes.  Result: TFLOP/s.
 * Errors: FS_EINVAL, FS_EHIP.
 */
int fs_probe_stream_read(const void *buf, size_t buf_bytes, size_t bytes_per_launch, int launches, void *stream, double *gb_per_s);
int fs_probe_mfma_bf16(void *scratch, int launches, void *stream, double *tflop_per_s);
/*
 *   fs_probe_fill         rate at which compute units pull data in: `grid` workgroups of `waves` waves each stream iters x waves x 4 KiB
 *                         from a region of region_kib KiB (a multiple of waves x 4) that they re-read cyclically, with 16-byte-per-lane
 *                         loads, three rounds in flight; to_lds != 0: direct-to-LDS loads (the path of the 256-row projection
 *                         kernel), else loads into registers.  Workgroups `share` consecutive slots of one XCD read the same
 *                         region; buf (device, 16-byte aligned) must hold (grid / 8 / share + 2) * 8 regions + 64 bytes.
 *                         Result: GB/s summed over the workgroups.
 */
int fs_probe_fill(const void *buf, size_t buf_bytes, int grid, int waves, int region_kib, int iters, int share, int to_lds, int launches,
                  void *stream, double *gb_per_s);

/* hipError_t (as int) behind the most recent FS_EHIP on the calling thread, 0 if none. */
int fs_last_hip_error(void);

/*
 * Verification-stage forward (Sec. III-A: the forward pass of this stage's layers over one draft segment; a
 * segment carries its tree position IDs and attention mask, both derived here from the parent array).  Runs the stage's layers over segment S[seg_off, seg_off + l_s):
 *   per layer: RMSNorm -> Q/K/V projections (+bias) -> rotary embedding at position l_glo + depth(node) ->
 *   K/V of row r stored at slot l_cache + r -> tree attention (row r sees every slot < l_glo and the draft
 *   slots l_glo + j with j an ancestor-or-self of node seg_off + r) -> output projection + residual ->
 *   RMSNorm -> SwiGLU feed-forward + residual.
 *   hidden_in / hidden_out  device [l_s, d_model], may alias
 *   parent                  HOST [seg_off + l_s], S order, parent[0] == -1 (further roots allowed: such a node
 *                           sees the context and itself only); read before the call returns
 * Precondition: l_cache == l_glo + seg_off.  l_s == 0 is a valid no-op.
 * Errors: FS_EINVAL, FS_ETOPO, FS_ECAP, FS_EHIP.
 */
int fs_tree_verify_stage(fs_stage *stage, fs_kv_cache kv, int l_glo, int l_cache, const void *hidden_in, int seg_off, int l_s,
                         const int32_t *parent, void *hidden_out, void *stream);

/*
 * The same forward for a batch of requests that share the stage's weights (data-parallel serving: each request has its own
 * KV cache, tree and context length): the segments' rows are stacked, the projections run once over all of them — the
 * weights are streamed once per batch instead of once per request, and from a few dozen stacked rows on the projections are
 * bound by the matrix units and the on-chip caches instead of by the weight stream — and tree attention runs per request
 * inside the same launches.
 *   items       HOST array [n_items]; each item is one fs_tree_verify_stage call's worth of arguments (kv, l_glo, l_cache,
 *               seg_off, l_s, host parent array); l_s = 0 items are skipped.  All caches must share one set of strides.
 *   hidden_in / hidden_out  device [sum of l_s, d_model], the items' rows in item order; may alias
 * Every item is validated before anything is enqueued.  Errors: as fs_tree_verify_stage; FS_ECAP also when n_items >
 * FS_MAX_BATCH or the stacked rows exceed max_seg; FS_EINVAL when the caches' strides differ.
 */
#define FS_MAX_BATCH 32
typedef struct {
    fs_kv_cache kv;
    int l_glo, l_cache, seg_off, l_s;
    const int32_t *parent; /* HOST [seg_off + l_s] */
} fs_batch_item;
int fs_tree_verify_batch(fs_stage *stage, const fs_batch_item *items, int n_items, const void *hidden_in, void *hidden_out, void *stream);

/*
 * The tree position IDs and the attention mask of a segment (Sec. III-A names both as part of a draft segment; Sec. III-B:
 * S is a topological order) exactly as fs_tree_verify_stage derives them from the parent array, for inspection and tests:
 *   anc   device uint64 [l_s][16]: bit j of row r is set iff S index j is node seg_off + r itself or one of its ancestors
 *   rope  device float  [l_s][head_dim/2][2]: (cos, sin) of (l_glo + depth(seg_off + r)) * rope_theta^(-2t/head_dim)
 *   parent HOST [seg_off + l_s]
 * Same kernels and the same routing (short walk / pointer doubling beyond 32 levels / closed form for a chain) as the
 * forward; uses the stage's scratch, so it must not overlap other calls on the stage.
 * Errors: FS_EINVAL, FS_ETOPO, FS_ECAP (tree larger than max_tree, segment longer than max_seg), FS_EHIP.
 */
int fs_tree_mask(fs_stage *stage, int l_glo, int seg_off, int l_s, const int32_t *parent, uint64_t *anc, float *rope, void *stream);

/*
 * Last stage's verification output (Sec. III-A, continuous SD step: the next-token distribution sent to the
 * draft stage): logits = RMSNorm_final(hidden) * E^T in fp32 and their per-row argmax (lowest index on ties).
 *   hidden device [l_s, d_model]; logits device fp32 [l_s, vocab]; amax device int32 [l_s].
 * Errors: FS_EINVAL (stage has no head, l_s > max_seg), FS_EHIP.
 */
int fs_tree_logits(fs_stage *stage, const void *hidden, int l_s, float *logits, int32_t *amax, void *stream);

/* Acceptance result (Sec. III-C), device or host. */
typedef struct {
    int32_t n_acc;         /* |S_acc| = |I_acc|, counts the root x_new of the tree; 0 only if n_ver == 0 */
    int32_t x_new;         /* newly sampled token (greedy: argmax at the last accepted node); -1 if n_ver == 0 */
    int32_t n_new;         /* S index of the node with path(n_new) = S_acc || x_new, or -1 */
    int32_t continuous;    /* continuous condition, Eq. 2 */
    int32_t n_retain;      /* |I_retain| */
    int32_t n_pr_verified; /* retained draft nodes that already have a verification output */
} fs_accept_result;

/*
 * Greedy acceptance over the verified prefix [0, n_ver) of S (Sec. III-C: accepted tokens S_acc, x_new,
 * continuous condition Eq. 2, retain set I_retain = I_acc U I_pr with n_new's subtree in original order).
 *   logits  device fp32 [n_ver, vocab] or NULL; when given, amax[0, n_ver) is first recomputed from it
 *   amax    device int32 [n_ver] (output when logits != NULL, input otherwise)
 *   token, parent  device int32 [T], S order
 *   res     device; retain device int32 [T]: I_acc ascending, then I_pr ascending
 *   work    device int32 scratch, at least 2 * n_ver * FS_ARGMAX_CHUNKS entries when logits != NULL, else unused
 * A node whose parent array entry breaks the topological order makes res->n_acc = -1 (nothing else is written).
 * n_ver == 0: nothing accepted, everything retained.
 * Errors: FS_EINVAL, FS_ECAP (T > FS_MAX_TREE), FS_EHIP.
 */
#define FS_ARGMAX_CHUNKS 64
int fs_tree_accept(const float *logits, int32_t *amax, int vocab, const int32_t *token, const int32_t *parent, int T, int n_ver,
                   fs_accept_result *res, int32_t *retain, int32_t *work, void *stream);

/*
 * fs_tree_accept for callers that cannot allocate device memory or carry a scratch buffer around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as fs_tree_accept without
 * `work`: the partial maxima of the row argmax live in a static device array inside the library (512 KiB per GPU, held
 * until the process ends; sized for n_ver <= FS_MAX_TREE rows and any vocab).  Calls no hipMalloc / hipFree or other
 * allocating routine.  All calls on one GPU share that array: calls that overlap in time on one GPU (different streams
 * or threads) race on it; calls on one stream do not.  Nothing in it needs clearing between calls.
 * Errors: FS_EINVAL, FS_ECAP (T > FS_MAX_TREE: beyond what the static array is sized for), FS_EHIP.
 */
int fs_tree_accept_noalloc(const float *logits, int32_t *amax, int vocab, const int32_t *token, const int32_t *parent, int T, int n_ver,
                           fs_accept_result *res, int32_t *retain, void *stream);

/*
 * Stochastic acceptance at a temperature > 0 (the paper's temperature-1 runs, Table I; Sec. III-C gives no formula).
 * Reading taken: sequential candidate test.  At an accepted node u with p = softmax(logits_u / temperature) the children of
 * u are tried in S order; a child is accepted with probability p(token) / (mass not yet rejected at u); a rejected token's
 * mass is struck.  An accepted verified child continues the walk; an accepted unverified child is n_new (continuous);
 * if every child is rejected x_new is drawn from what is left.  The token leaving the step is distributed exactly as p.
 * Probabilities are 64-bit integer weights E_v = (uint64)(exp2_spec((z_v - max z) * log2 e) * 2^32), z_v = logits_v *
 * (1/temperature) in fp32, with exp2_spec a fixed sequence of IEEE fp32 operations, and uniform numbers come from a
 * counter-based generator keyed by (seed, step, draw index): every decision is an integer comparison, reproducible bit for
 * bit.  Outputs as fs_tree_accept.
 *   logits device fp32 [n_ver, vocab];  work device, 16-byte aligned, >= 16 + 12 * n_ver bytes
 * Errors: FS_EINVAL, FS_ECAP, FS_EHIP.
 */
int fs_tree_accept_sample(const float *logits, int vocab, float temperature, const int32_t *token, const int32_t *parent, int T,
                          int n_ver, uint64_t seed, uint64_t step, fs_accept_result *res, int32_t *retain, void *work, void *stream);

/* Copies the result and the first n_retain entries of retain to the host and waits for the stream: the one
 * synchronisation point of the path.  retain_host must hold T entries. */
int fs_accept_result_to_host(const fs_accept_result *res_dev, const int32_t *retain_dev, int T, fs_accept_result *res_host,
                             int32_t *retain_host, void *stream);

/*
 * KV-cache pruning (Sec. III-C, the paragraph on pruning the KV cache): with I_incache = { i in I_retain : l_glo + i < l_cache },
 * slot l_glo + j <- slot l_glo + I_incache[j] for every layer, K and V, every head; slots below l_glo are not
 * touched.  Bit-exact copy, in place.
 *   retain / res   either both device (straight from fs_tree_accept; counts are read on the device), or
 *                  res == NULL and retain a HOST array with n_retain_host entries of which the first n_acc_host
 *                  are accepted (the paper's case: the retain set arrives from the draft stage)
 *   new_len        device int32 [2], optional: { l_glo + n_acc, l_glo + |I_incache| }
 * Errors: FS_EINVAL, FS_ECAP, FS_EHIP.
 */
int fs_kv_compact(fs_stage *stage, fs_kv_cache kv, int l_glo, int l_cache, const int32_t *retain, const fs_accept_result *res,
                  int n_retain_host, int n_acc_host, int32_t *new_len, void *stream);

/*
 * Draft-segment pruning (Sec. III-C, the paragraph on pruning draft segments): the in-flight segment holds S indices
 * [off, off + l_s) with off = l_cache - l_glo; rows with off + r in I_retain are gathered, in order, into
 * seg_out (must not overlap seg_in); *l_s_out = number kept.
 *   seg_in / seg_out device [l_s, row_bytes]; row_bytes a multiple of 4
 *   retain / res as in fs_kv_compact;  l_s_out device int32 [1]
 */
int fs_seg_prune(const void *seg_in, int l_s, size_t row_bytes, int off, const int32_t *retain, const fs_accept_result *res,
                 int n_retain_host, void *seg_out, int32_t *l_s_out, void *stream);

/* ---- draft-stage tree bookkeeping on the host (Sec. III-B, III-C, III-D); plain CPU code, no GPU work ---------------
 * The paper keeps the tree structure on the draft stage only and runs these steps on the CPU (Sec. III-A: they offer
 * little parallelism);
 * all arrays below are HOST arrays owned by the caller. */

/*
 * Score-based draft segmentation (Sec. III-B): T_base has n_base nodes in any topological order (parent_base[0] == -1,
 * 0 <= parent_base[i] < i) with per-node confidences conf (the root's is taken as 1).  Cumulative scores follow Eq. 1
 * (product along the path, in double); the L0 nodes of highest cumulative score are kept (ties: lower base index first,
 * which keeps the selection connected) and ordered by descending score -> the draft sequence S, a topological order.
 * Outputs, each with room for min(L0, n_base) entries: parent (S indices, parent[0] = -1), token, score, base_index.
 * Consecutive slices of at most L_max entries of S are the draft segments.
 * Returns the number of nodes kept, or FS_EINVAL / FS_ETOPO.
 */
int fs_tree_segment(const int32_t *parent_base, const int32_t *token_base, const float *conf, int n_base, int L0, int32_t *parent,
                    int32_t *token, double *score, int32_t *base_index);

/*
 * Tree pruning on the draft stage (Sec. III-C): T_pr / S_pr from a retain list as produced by fs_tree_accept (I_acc first,
 * then I_pr ascending): retained draft nodes keep their order, parents are renumbered by rank, the new root (n_new) gets -1.
 * Outputs hold n_retain - n_acc entries.  Returns |S_pr| (0 when the round ended), or FS_EINVAL.
 */
int fs_tree_prune(const int32_t *parent, const int32_t *token, int T, const int32_t *retain, int n_acc, int n_retain,
                  int32_t *new_parent, int32_t *new_token);

/*
 * Tree expansion by merging (Sec. III-D): T_pr (n_pr nodes, S order) and a newly drafted tree T_new (n_new nodes in descending
 * score order, same root token).  A node of T_new whose root-to-node token path already exists in T_pr is identified with that
 * node (the paths of T_pr are kept in a hash table keyed by (node of the parent path, token)); the other nodes, at most
 * `limit` of them (limit < 0: all), are appended behind S_pr in T_new's order: S = S_pr || S_app.  With limit = L_se this is
 * also the score-aware expansion (top unseen nodes of a deeper base tree).
 * Outputs: parent / token [max_out] of the merged tree, app_src [n_app] = T_new index of each appended node,
 * map_new [n_new] = merged index of every T_new node (-1 if it fell beyond the limit).
 * Returns the merged size n_pr + n_app, or FS_EINVAL (root tokens differ), FS_ETOPO, FS_ECAP (max_out too small).
 */
int fs_tree_merge(const int32_t *parent_pr, const int32_t *token_pr, int n_pr, const int32_t *parent_new, const int32_t *token_new,
                  int n_new, int limit, int max_out, int32_t *parent, int32_t *token, int32_t *app_src, int32_t *map_new);

#ifdef __cplusplus
}
#endif
#endif /* FLOWSPEC_H */
