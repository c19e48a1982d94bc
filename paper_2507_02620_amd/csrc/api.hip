// Host side of the C ABI declared in include/flowspec.h: validation, workspace layout, launch sequencing.
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <algorithm>
#include <vector>

#include "../../include/flowspec.h"
#include "attention.hpp"
#include "gemm.hpp"
#include "tree.hpp"

thread_local int g_last_hip = 0;  // shared with probe.hip

#define HIP_TRY(expr)                 \
    do {                              \
        hipError_t e__ = (expr);      \
        if (e__ != hipSuccess) {      \
            g_last_hip = (int)e__;    \
            return FS_EHIP;           \
        }                             \
    } while (0)

// a launch that is timed when the stage's profiler is armed
#define HIP_TRY_K(st, kind, s, expr)               \
    do {                                           \
        const bool t__ = (st)->prof.begin(kind, s); \
        hipError_t e__ = (expr);                   \
        if (t__) (st)->prof.end(s);                \
        if (e__ != hipSuccess) {                   \
            g_last_hip = (int)e__;                 \
            return FS_EHIP;                        \
        }                                          \
    } while (0)

namespace {

struct GemmPlan {
    void* wp = nullptr;
    void* sp = nullptr;  // 4-bit: scales
    float* bias = nullptr;
    int N = 0, K = 0, nkt = 0, NT = 1, NW = 8, n_groups = 0, w4 = 0;
    size_t bytes() const { return w4 ? (size_t)n_groups * (nkt / 4) * NT * 1024 : (size_t)n_groups * nkt * NT * 1024; }
    size_t scale_bytes() const { return w4 ? (size_t)n_groups * (nkt / 4) * NT * 16 * 2 : 0; }
};

struct LayerPlan {
    GemmPlan qkv, o, gu, down;
};

constexpr int kMaxSplits = 64;

int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    return v ? atoi(v) : dflt;
}

// Tiles per group: the largest allowed NT that still leaves about two workgroups per compute unit;
// segments longer than 16 rows prefer NT >= 2 so that activation re-reads through L2 stay below the weight stream.
int choose_nt(int tiles, bool pair, int max_seg, const char* env, bool wide_n = false) {
    int nt = pair ? 2 : 1;
    if (tiles / 4 >= 512) nt = 4;
    else if (tiles / 2 >= 512) nt = 2;
    if (max_seg > 16 && nt < 2 && tiles / 2 >= 160) nt = 2;
    // segments of more than 32 rows: QKV and the LM head do better with 4 tiles per group (measured at 64 rows: QKV 42 -> 34 us,
    // head 92 -> 67 us; gate/up and the d_model-wide projections do not)
    if (max_seg > 32 && wide_n && tiles / 4 >= 160) nt = 4;
    // two row tiles (17 to 32 rows): the same from 192 groups on (24 rows, 960 tiles: QKV 33.6 -> 30.3 us, 2000 tiles: head 55.9 -> 54.0 us)
    if (max_seg > 16 && wide_n && tiles / 4 >= 192) nt = 4;
    int o = env_int(env, 0);
    if (o == 1 || o == 2 || o == 4) nt = (pair && o == 1) ? 2 : o;
    return nt;
}

void plan_gemm(GemmPlan& g, int tiles, int K, int elem, bool pair, int max_seg, const char* env_nt, int w4 = 0, bool wide_n = false) {
    const int KT = 64 / elem;  // 32 for bf16, 16 for f32
    g.K = K;
    g.w4 = w4;
    g.nkt = (K + KT - 1) / KT;
    g.NT = choose_nt(tiles, pair, max_seg, env_nt, wide_n);
    if (w4) {
        // a 4-bit tile is a quarter of the bytes: larger groups keep the per-workgroup stream long enough;
        // 64-row segments stay at NT <= 2 (registers)
        int nt = pair ? 2 : 1;
        // (QKV and the LM head already from 192 groups on: 24 rows, 960 tiles: QKV 27.4 -> 22.2 us; 16 rows, 768 tiles: 14.5 -> 13.8 us)
        if ((tiles / 4 >= 256 || (wide_n && tiles / 4 >= 192)) && max_seg <= 32) nt = 4;
        else if (tiles / 2 >= 128) nt = 2;
        const int o = env_int(env_nt, 0);
        if (o == 1 || o == 2 || o == 4) nt = (pair && o == 1) ? 2 : o;
        if (max_seg > 32 && nt > 2) nt = 2;
        g.NT = nt;
    }
    g.n_groups = (tiles + g.NT - 1) / g.NT;
    g.NW = env_int("FLOWSPEC_NW", 8);
    if (g.NW < 1 || g.NW > 16) g.NW = 8;
    const int ksteps = w4 ? g.nkt / 4 : g.nkt;
    if (g.NW > ksteps) g.NW = ksteps;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
    std::vector<LayerPlan> layers;
    GemmPlan head;
    size_t off_q, off_o, off_h, off_hb, off_act, off_anc, off_rope, off_po, off_pml, off_amw, off_invf, off_gain, off_sspa, off_sspb, off_part, part_bytes, off_ancall, off_krow, total;
    int ssp_stride;
};

bool valid_desc(const fs_stage_desc* d, int* err) {
    *err = FS_EINVAL;
    if (!d) return false;
    if (d->dtype != FS_F32 && d->dtype != FS_BF16) {
        *err = FS_EDTYPE;
        return false;
    }
    if (d->max_tree > FS_MAX_TREE) {
        *err = FS_ECAP;
        return false;
    }
    if (d->n_layers < 1 || d->d_model < 16 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->d_ffn < 8 || d->vocab < 0) return false;
    if (d->n_q_heads % d->n_kv_heads) return false;
    if (d->head_dim != 64 && d->head_dim != 128) return false;
    int kt = d->dtype == FS_F32 ? 16 : 32;  // k-tile of the projection kernels
    if (d->weight_format != FS_WFMT_DENSE && d->weight_format != FS_WFMT_INT4_G128) return false;
    if (d->weight_format == FS_WFMT_INT4_G128) {
        if (d->dtype != FS_BF16) {
            *err = FS_EDTYPE;
            return false;
        }
        kt = 128;  // one scale per 128 input columns
        if ((d->n_q_heads * d->head_dim) % kt) return false;
    }
    if (d->d_model % kt || d->d_ffn % kt) return false;
    if (d->kv_capacity < 1 || d->max_tree < 1 || d->max_seg < 1 || d->max_seg > FS_MAX_TREE) return false;
    if (!(d->rms_eps >= 0.f) || !(d->rope_theta > 0.f)) return false;
    return true;
}

void make_layout(const fs_stage_desc* d, Layout& L) {
    const int elem = d->dtype == FS_F32 ? 4 : 2;
    const int hd = d->head_dim, nq = d->n_q_heads * hd;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    const int w4 = d->weight_format == FS_WFMT_INT4_G128;
    L.layers.resize(d->n_layers);
    for (int l = 0; l < d->n_layers; ++l) {
        LayerPlan& p = L.layers[l];
        const int qkv_tiles = (d->n_q_heads + 2 * d->n_kv_heads) * hd / 16;
        plan_gemm(p.qkv, qkv_tiles, d->d_model, elem, true, d->max_seg, "FLOWSPEC_NT_QKV", w4, true);
        p.qkv.N = qkv_tiles * 16;
        plan_gemm(p.o, d->d_model / 16, nq, elem, false, d->max_seg, "FLOWSPEC_NT_O", w4);
        p.o.N = d->d_model;
        plan_gemm(p.gu, 2 * ((d->d_ffn + 15) / 16), d->d_model, elem, true, d->max_seg, "FLOWSPEC_NT_GU", w4);
        p.gu.N = d->d_ffn;
        plan_gemm(p.down, d->d_model / 16, d->d_ffn, elem, false, d->max_seg, "FLOWSPEC_NT_DOWN", w4);
        p.down.N = d->d_model;
        for (GemmPlan* g : {&p.qkv, &p.o, &p.gu, &p.down}) {
            g->wp = (void*)take(g->bytes());
            g->sp = (void*)take(g->scale_bytes());
        }
        p.qkv.bias = (float*)take((size_t)p.qkv.n_groups * p.qkv.NT * 16 * sizeof(float));
    }
    if (d->vocab > 0) {
        plan_gemm(L.head, (d->vocab + 15) / 16, d->d_model, elem, false, d->max_seg, "FLOWSPEC_NT_HEAD", w4, true);
        L.head.N = d->vocab;
        L.head.wp = (void*)take(L.head.bytes());
        L.head.sp = (void*)take(L.head.scale_bytes());
    }
    const size_t M = align_up((size_t)d->max_seg, 16);  // fragment-major buffers hold whole 16-row tiles
    const int G = d->n_q_heads / d->n_kv_heads;
    const size_t Rpad = align_up((size_t)G * M, 16);
    L.off_q = take(M * nq * elem);
    L.off_o = take(M * nq * elem);
    L.off_h = take(M * d->d_model * sizeof(float));
    L.off_hb = take(M * d->d_model * elem);
    L.off_act = take(M * d->d_ffn * elem);
    L.off_anc = take(M * FS_ANC_WORDS * sizeof(uint64_t));
    L.off_rope = take(M * (hd / 2) * sizeof(float2));
    L.off_po = take((size_t)kMaxSplits * d->n_kv_heads * Rpad * hd * sizeof(float));
    L.off_pml = take((size_t)kMaxSplits * d->n_kv_heads * Rpad * 2 * sizeof(float));
    L.off_amw = take(M * FS_ARGMAX_CHUNKS * 2 * sizeof(int32_t));
    L.off_invf = take((size_t)(hd / 2) * sizeof(double));
    L.off_gain = take(w4 ? (size_t)(2 * d->n_layers + 1) * d->d_model * 2 : 0);  // 4-bit: bf16 copies of the RMSNorm gains
    // 4-bit weights and many-row segments: two buffers of per-row partial sums of squares of the residual stream, at
    // most one entry per 16-feature tile (+ padding entries of the last feature block)
    L.ssp_stride = (int)M;
    const size_t ssp_bytes = d->dtype == FS_BF16 ? (size_t)(d->d_model / 16 + 4) * M * sizeof(float) : 0;
    L.off_sspa = take(ssp_bytes);
    L.off_sspb = take(ssp_bytes);
    // many-row segments: scratch for the K-split partial results of the two residual projections
    L.part_bytes = 0;
    if (d->dtype == FS_BF16 && !w4 && d->max_seg > 16) L.part_bytes = wide_partial_bytes(d->max_seg, d->d_model / 16);
    L.off_part = take(L.part_bytes);
    L.off_krow = take(M * sizeof(unsigned long long));  // cache slot address of every stacked row
    L.off_ancall = take((size_t)2 * d->max_tree * FS_ANC_WORDS * sizeof(uint64_t));  // two copies of every node's mask while a deep tree's are built
    L.total = off;
}

int valid_kv(const fs_stage_desc& d, const fs_kv_cache& kv) {
    const int elem = d.dtype == FS_F32 ? 4 : 2, epf = 16 / elem;
    if (!kv.base || ((uintptr_t)kv.base & 15)) return FS_EINVAL;
    if (kv.stride_tok < d.head_dim || kv.stride_tok % epf || kv.stride_head % epf || kv.stride_kv % epf || kv.stride_layer % epf) return FS_EINVAL;
    if (kv.stride_head < 0 || kv.stride_kv < 0 || kv.stride_layer < 0) return FS_EINVAL;
    // tree attention addresses the slots of one head with 32-bit byte offsets
    if ((long long)d.kv_capacity * kv.stride_tok * elem >= (1LL << 32)) return FS_EINVAL;
    return FS_OK;
}

int fill_idx(IdxList& L, const int32_t* v, int n) {
    if (n < 0 || n > 1024) return FS_ECAP;
    L.n = n;
    for (int i = 0; i < n; ++i) {
        if (v[i] < -1 || v[i] > 1023) return FS_EINVAL;
        L.v[i] = (short)v[i];
    }
    return FS_OK;
}

}  // namespace

// Optional per-kernel timing: when armed, every launch of the stage is bracketed by a pair of events on the
// caller's stream; fs_stage_profile_end waits for the stream and sums the elapsed times per kernel kind.
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;  // 2 per record
    std::vector<int> kind;
    size_t cap = 0;
    bool begin(int k, hipStream_t s) {
        if (!on || kind.size() >= cap) return false;
        kind.push_back(k);
        return hipEventRecord(ev[2 * (kind.size() - 1)], s) == hipSuccess;
    }
    void end(hipStream_t s) { (void)hipEventRecord(ev[2 * (kind.size() - 1) + 1], s); }
    void release() {
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
        ev.clear();
        kind.clear();
        cap = 0;
        on = false;
    }
};

// Tuning knobs from the environment, read once when the stage is created (a launch never calls getenv).
struct Tunables {
    int attn_wgs, attn_mtw, attn_nset, attn_nwc, attn_dma, wide_rows, mid_rows, block_gemm, compact_cb;
    void read() {
        attn_wgs = env_int("FLOWSPEC_ATTN_WGS", 0);    // > 0: workgroups the attention split plan aims for
        attn_mtw = env_int("FLOWSPEC_ATTN_MTW", 0);    // > 0: row tiles per wave of the attention kernel
        attn_nwc = env_int("FLOWSPEC_ATTN_NWC", 0);    // > 0: at most this many row-tile waves per workgroup (more row blocks)
        attn_dma = env_int("FLOWSPEC_ATTN_DMA", 0);    // 1: never the direct-to-LDS attention kernel; 2 .. 4: always, with so many tile buffers
        attn_nset = env_int("FLOWSPEC_ATTN_NSET", 0);  // > 0: K/V tiles in flight per workgroup on long splits
        wide_rows = env_int("FLOWSPEC_WIDE_ROWS", 65); // stacked rows from which every projection takes the many-row kernel
        mid_rows = env_int("FLOWSPEC_MID_ROWS", 17);   // ... from which the wide projections do
        compact_cb = env_int("FLOWSPEC_COMPACT_CB", 0);  // KV compaction: column blocks per row (0: by the grid size)
        block_gemm = env_int("FLOWSPEC_BLOCK_GEMM", -1);  // 256-row projection kernel: 0 never, 1 / 2 always (256- / 192-feature blocks), else by rule
    }
};

struct fs_stage {
    fs_stage_desc d;
    Layout L;
    Tunables tun;
    unsigned char* ws;
    int elem;
    Profiler prof;
    template <typename P>
    P* at(size_t off) const { return (P*)(ws + off); }
};

// ---- scratch of the entry point that allocates nothing ------------------------------------------------------------
// fs_tree_accept_noalloc keeps the per-chunk partial maxima of the row argmax (what fs_tree_accept takes as `work`) in a
// file-scope device array: 2 int32 (value bits, index) per row and chunk, FS_MAX_TREE rows at most, 512 KiB on every GPU
// the library runs on, held until the process ends.  The array's name is only a handle on the host: the device address
// is looked up once per device, with that device current, and kept.
static __device__ __align__(256) int32_t noalloc_scratch_mem[2 * FS_MAX_TREE * FS_ARGMAX_CHUNKS];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices] = {};

int noalloc_scratch(int32_t** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return FS_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(noalloc_scratch_mem)));
        if (!p) return FS_EHIP;
        g_scratch_ptr[dev] = (int32_t*)p;
    }
    *out = g_scratch_ptr[dev];
    return FS_OK;
}
}  // namespace

extern "C" {

int fs_last_hip_error(void) { return g_last_hip; }

size_t fs_stage_workspace_bytes(const fs_stage_desc* desc) {
    int err;
    if (!valid_desc(desc, &err)) return 0;
    Layout L;
    make_layout(desc, L);
    return L.total;
}

int fs_stage_create(const fs_stage_desc* desc, const fs_layer_weights* layers, const void* final_norm, const void* lm_head,
                    const void* lm_head_scale, void* workspace, size_t workspace_bytes, void* stream, fs_stage** out) {
    int err;
    if (!out) return FS_EINVAL;
    *out = nullptr;
    if (!valid_desc(desc, &err)) return err;
    if (!layers) return FS_EINVAL;
    const int w4 = desc->weight_format == FS_WFMT_INT4_G128;
    if (desc->vocab > 0 && (!final_norm || !lm_head || (w4 && !lm_head_scale))) return FS_EINVAL;
    for (int l = 0; l < desc->n_layers; ++l) {
        const fs_layer_weights& w = layers[l];
        if (!w.rms_attn || !w.wq || !w.wk || !w.wv || !w.wo || !w.rms_ffn || !w.w_gate || !w.w_up || !w.w_down) return FS_EINVAL;
        if (w4 && (!w.sq || !w.sk || !w.sv || !w.so || !w.s_gate || !w.s_up || !w.s_down)) return FS_EINVAL;
    }
    fs_stage* st = new (std::nothrow) fs_stage;
    if (!st) return FS_EINVAL;
    st->d = *desc;
    st->tun.read();
    st->elem = desc->dtype == FS_F32 ? 4 : 2;
    make_layout(desc, st->L);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < st->L.total) {
        delete st;
        return FS_EWS;
    }
    st->ws = (unsigned char*)workspace;
    hipStream_t s = (hipStream_t)stream;
    const int hd = desc->head_dim;
    bf16_t* gains = st->at<bf16_t>(st->L.off_gain);  // 4-bit: [2 * layer + {0: attn, 1: ffn}][d_model], final norm last
    const size_t gain_bytes = (size_t)desc->d_model * 2;
    for (int l = 0; l < desc->n_layers; ++l) {
        LayerPlan& p = st->L.layers[l];
        const fs_layer_weights& w = layers[l];
        for (GemmPlan* g : {&p.qkv, &p.o, &p.gu, &p.down}) {
            g->wp = st->ws + (size_t)g->wp;
            g->sp = st->ws + (size_t)g->sp;
        }
        p.qkv.bias = (float*)(st->ws + (size_t)p.qkv.bias);
        if (w4) {
            PackW4Args a{};
            a.Hq = desc->n_q_heads; a.Hkv = desc->n_kv_heads; a.hd = hd;
            a.kind = PACK_QKV; a.c0 = w.wq; a.c1 = w.wk; a.c2 = w.wv; a.s0 = w.sq; a.s1 = w.sk; a.s2 = w.sv; a.dst = p.qkv.wp; a.sdst = p.qkv.sp;
            a.N = p.qkv.N; a.K = p.qkv.K; a.NT = p.qkv.NT; a.n_groups = p.qkv.n_groups;
            a.b0 = w.bq; a.b1 = w.bk; a.b2 = w.bv; a.bias_dst = p.qkv.bias;
            launch_pack_w4(a, s);
            if (!w.bq && !w.bk && !w.bv) p.qkv.bias = nullptr;
            a = PackW4Args{};
            a.kind = PACK_PLAIN; a.c0 = w.wo; a.s0 = w.so; a.dst = p.o.wp; a.sdst = p.o.sp; a.N = p.o.N; a.K = p.o.K; a.NT = p.o.NT;
            a.n_groups = p.o.n_groups;
            launch_pack_w4(a, s);
            a = PackW4Args{};
            a.kind = PACK_GATEUP; a.c0 = w.w_gate; a.c1 = w.w_up; a.s0 = w.s_gate; a.s1 = w.s_up; a.dst = p.gu.wp; a.sdst = p.gu.sp;
            a.N = p.gu.N; a.K = p.gu.K; a.NT = p.gu.NT; a.n_groups = p.gu.n_groups;
            launch_pack_w4(a, s);
            a = PackW4Args{};
            a.kind = PACK_PLAIN; a.c0 = w.w_down; a.s0 = w.s_down; a.dst = p.down.wp; a.sdst = p.down.sp; a.N = p.down.N; a.K = p.down.K;
            a.NT = p.down.NT; a.n_groups = p.down.n_groups;
            launch_pack_w4(a, s);
            // the gains stay separate (they cannot be folded into integer codes): private bf16 copies
            if (hipMemcpyAsync(gains + (size_t)(2 * l) * desc->d_model, w.rms_attn, gain_bytes, hipMemcpyDeviceToDevice, s) != hipSuccess ||
                hipMemcpyAsync(gains + (size_t)(2 * l + 1) * desc->d_model, w.rms_ffn, gain_bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) {
                g_last_hip = (int)hipGetLastError();
                delete st;
                return FS_EHIP;
            }
            continue;
        }
        PackArgs a{};
        a.Hq = desc->n_q_heads; a.Hkv = desc->n_kv_heads; a.hd = hd;
        // QKV (attention RMSNorm gain folded in)
        a.kind = PACK_QKV; a.src0 = w.wq; a.src1 = w.wk; a.src2 = w.wv; a.gain = w.rms_attn; a.dst = p.qkv.wp;
        a.N = p.qkv.N; a.K = p.qkv.K; a.nkt = p.qkv.nkt; a.NT = p.qkv.NT; a.n_groups = p.qkv.n_groups;
        a.b0 = w.bq; a.b1 = w.bk; a.b2 = w.bv; a.bias_dst = p.qkv.bias;
        launch_pack(desc->dtype, a, s);
        if (!w.bq && !w.bk && !w.bv) p.qkv.bias = nullptr;  // packed zeros stay unused
        // O
        a = PackArgs{};
        a.kind = PACK_PLAIN; a.src0 = w.wo; a.dst = p.o.wp; a.N = p.o.N; a.K = p.o.K; a.nkt = p.o.nkt; a.NT = p.o.NT; a.n_groups = p.o.n_groups;
        launch_pack(desc->dtype, a, s);
        // gate / up (FFN RMSNorm gain folded in)
        a = PackArgs{};
        a.kind = PACK_GATEUP; a.src0 = w.w_gate; a.src1 = w.w_up; a.gain = w.rms_ffn; a.dst = p.gu.wp;
        a.N = p.gu.N; a.K = p.gu.K; a.nkt = p.gu.nkt; a.NT = p.gu.NT; a.n_groups = p.gu.n_groups;
        launch_pack(desc->dtype, a, s);
        // down
        a = PackArgs{};
        a.kind = PACK_PLAIN; a.src0 = w.w_down; a.dst = p.down.wp; a.N = p.down.N; a.K = p.down.K; a.nkt = p.down.nkt; a.NT = p.down.NT;
        a.n_groups = p.down.n_groups;
        launch_pack(desc->dtype, a, s);
    }
    if (desc->vocab > 0) {
        GemmPlan& g = st->L.head;
        g.wp = st->ws + (size_t)g.wp;
        g.sp = st->ws + (size_t)g.sp;
        if (w4) {
            PackW4Args a{};
            a.kind = PACK_PLAIN; a.c0 = lm_head; a.s0 = lm_head_scale; a.dst = g.wp; a.sdst = g.sp; a.N = g.N; a.K = g.K; a.NT = g.NT;
            a.n_groups = g.n_groups;
            launch_pack_w4(a, s);
            if (hipMemcpyAsync(gains + (size_t)(2 * desc->n_layers) * desc->d_model, final_norm, gain_bytes, hipMemcpyDeviceToDevice, s) !=
                hipSuccess) {
                g_last_hip = (int)hipGetLastError();
                delete st;
                return FS_EHIP;
            }
        } else {
            PackArgs a{};
            a.kind = PACK_PLAIN; a.src0 = lm_head; a.gain = final_norm; a.dst = g.wp; a.N = g.N; a.K = g.K; a.nkt = g.nkt; a.NT = g.NT;
            a.n_groups = g.n_groups;
            launch_pack(desc->dtype, a, s);
        }
    }
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = launch_rope_freq(st->at<double>(st->L.off_invf), hd, desc->rope_theta, s);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        delete st;
        return FS_EHIP;
    }
    *out = st;
    return FS_OK;
}

int fs_stage_destroy(fs_stage* stage) {
    if (stage) stage->prof.release();
    delete stage;
    return FS_OK;
}

int fs_stage_profile_begin(fs_stage* st, int max_records) {
    if (!st || max_records < 1 || max_records > (1 << 20)) return FS_EINVAL;
    st->prof.release();
    st->prof.ev.resize(2 * (size_t)max_records);
    for (size_t i = 0; i < st->prof.ev.size(); ++i) {
        hipError_t e = hipEventCreate(&st->prof.ev[i]);
        if (e != hipSuccess) {
            st->prof.ev.resize(i);
            st->prof.release();
            g_last_hip = (int)e;
            return FS_EHIP;
        }
    }
    st->prof.cap = (size_t)max_records;
    st->prof.kind.reserve(st->prof.cap);
    st->prof.on = true;
    return FS_OK;
}

int fs_stage_profile_end(fs_stage* st, void* stream, double* total_ms, long long* counts) {
    if (!st || !total_ms || !counts) return FS_EINVAL;
    for (int k = 0; k < FS_K_COUNT; ++k) {
        total_ms[k] = 0.0;
        counts[k] = 0;
    }
    if (!st->prof.on) return FS_EINVAL;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    for (size_t i = 0; i < st->prof.kind.size() && e == hipSuccess; ++i) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, st->prof.ev[2 * i], st->prof.ev[2 * i + 1]);
        total_ms[st->prof.kind[i]] += ms;
        counts[st->prof.kind[i]] += 1;
    }
    st->prof.release();
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return FS_EHIP;
    }
    return FS_OK;
}

// One row block of the many-row kernel has a workgroup per 128 features: that is a good launch if they all run at once
// (at most one per compute unit) or if there are many rounds of them, not if a few compute units get a second one
// (measured: 296 workgroups, 60 us against 52 us with the few-row kernel; 216 workgroups, 49 against 57 us).
static bool mid_cols_ok(int n_tiles) {
    const int n_cols = (n_tiles + 7) / 8;
    return n_cols <= 256 || n_cols >= 512;
}

// dense or 4-bit projection launch, by the stage's weight format; `wide`: through the many-row kernel
static hipError_t launch_proj(const fs_stage* st, int epi, const GemmPlan& p, GemmArgs& g, hipStream_t s, bool wide = false) {
    if (wide) return launch_gemm_wide(epi, p.NT, p.n_groups * p.NT, g, st->at<float>(st->L.off_part), st->L.part_bytes, st->tun.block_gemm, s);
    if (p.w4) {
        g.Sp = p.sp;
        return launch_gemm_w4(epi, p.NT, p.NW, p.n_groups, g, s);
    }
    return launch_gemm(st->d.dtype, epi, p.NT, p.NW, p.n_groups, g, s);
}

// The forward of one batch: every request's segment is prepared on its own (tree mask, positions, cache slots), then the
// layers run over the stacked rows — projections once for all rows, attention per request inside one launch.
static int verify_batch(fs_stage* st, const fs_batch_item* items, int n, const void* hidden_in, void* hidden_out, void* stream) {
    if (!st || !items || n < 1) return FS_EINVAL;
    if (n > FS_MAX_BATCH) return FS_ECAP;
    const fs_stage_desc& d = st->d;
    const Layout& L = st->L;
    // ---- validation of every item before anything is enqueued ----
    int rows = 0, max_M = 0, max_L = 0, n_live = 0;
    const fs_kv_cache* kv0 = nullptr;
    for (int i = 0; i < n; ++i) {
        const fs_batch_item& it = items[i];
        if (it.l_s < 0 || it.seg_off < 0 || it.l_glo < 0) return FS_EINVAL;
        if (it.l_cache != it.l_glo + it.seg_off) return FS_EINVAL;
        if (it.l_s == 0) continue;
        if (!it.parent) return FS_EINVAL;
        const int T = it.seg_off + it.l_s;
        if (T > d.max_tree) return FS_ECAP;
        if ((long long)it.l_cache + it.l_s > d.kv_capacity) return FS_ECAP;
        int rc = valid_kv(d, it.kv);
        if (rc) return rc;
        if (!kv0) kv0 = &it.kv;
        // one launch addresses every request's cache with the same strides
        if (it.kv.stride_layer != kv0->stride_layer || it.kv.stride_kv != kv0->stride_kv || it.kv.stride_head != kv0->stride_head ||
            it.kv.stride_tok != kv0->stride_tok)
            return FS_EINVAL;
        if (it.parent[0] != -1) return FS_ETOPO;
        for (int j = 1; j < T; ++j)
            if (it.parent[j] < -1 || it.parent[j] >= j) return FS_ETOPO;
        rows += it.l_s;
        max_M = std::max(max_M, it.l_s);
        max_L = std::max(max_L, it.l_cache + it.l_s);
        ++n_live;
    }
    if (rows == 0) return FS_OK;
    if (rows > d.max_seg) return FS_ECAP;
    if (!hidden_in || !hidden_out) return FS_EINVAL;

    hipStream_t s = (hipStream_t)stream;
    const int hd = d.head_dim, nq = d.n_q_heads * hd, G = d.n_q_heads / d.n_kv_heads;
    void* q = st->at<void>(L.off_q);
    void* o = st->at<void>(L.off_o);
    float* h = st->at<float>(L.off_h);
    void* hb = st->at<void>(L.off_hb);
    void* act = st->at<void>(L.off_act);
    uint64_t* anc = st->at<uint64_t>(L.off_anc);
    float2* rope = st->at<float2>(L.off_rope);
    unsigned long long* krow = st->at<unsigned long long>(L.off_krow);
    const bf16_t* gains = st->at<bf16_t>(L.off_gain);

    AttnArgs at{};
    at.q = q; at.o = o; at.Hq = d.n_q_heads; at.Hkv = d.n_kv_heads; at.hd = hd; at.G = G;
    at.anc = anc;
    at.scale_log2 = 1.4426950408889634f / sqrtf((float)hd);
    at.stride_kv = kv0->stride_kv; at.stride_head = kv0->stride_head; at.stride_tok = kv0->stride_tok;
    at.part_o = st->at<float>(L.off_po); at.part_ml = st->at<float>(L.off_pml);
    at.n_req = n_live; at.rows = rows; at.max_M = max_M; at.max_L = max_L;
    at.Rpad = (int)align_up((size_t)G * rows, 16);

    // ---- per request: ancestor masks, positions (rotary table) and cache slots of its rows, into the stacked arrays ----
    int row0 = 0, rq = 0;
    for (int i = 0; i < n; ++i) {
        const fs_batch_item& it = items[i];
        if (it.l_s == 0) continue;
        const int T = it.seg_off + it.l_s;
        short depth[FS_MAX_TREE];
        int max_depth = 0;
        depth[0] = 0;
        for (int j = 1; j < T; ++j) {
            depth[j] = it.parent[j] < 0 ? 0 : (short)(depth[it.parent[j]] + 1);
            if (depth[j] > max_depth) max_depth = depth[j];
        }
        IdxList pl;
        int rc = fill_idx(pl, it.parent, T);
        if (rc) return rc;
        KRowArgs kr{krow + row0, (unsigned long long)(uintptr_t)it.kv.base, (unsigned long long)it.kv.stride_tok * st->elem, it.l_cache};
        HIP_TRY_K(st, FS_K_PREPARE, s,
                  launch_tree_prepare(pl, max_depth, it.l_glo, it.seg_off, it.l_s, hd, st->at<double>(L.off_invf), st->at<uint64_t>(L.off_ancall),
                                      anc + (size_t)row0 * FS_ANC_WORDS, rope + (size_t)row0 * (hd / 2), kr, s));
        at.req[rq] = AttnReq{it.kv.base, row0, it.l_s, it.l_glo, it.l_cache + it.l_s};
        row0 += it.l_s;
        ++rq;
    }
    int aMTW, aRB;
    attn_plan(st->elem, hd, max_M, G, d.n_kv_heads * n_live, max_L, kMaxSplits, st->tun.attn_wgs, st->tun.attn_mtw, st->tun.attn_nset, st->tun.attn_nwc,
              st->tun.attn_dma, &at.nwc, &aMTW, &aRB, &at.n_splits, &at.tiles_per_split, &at.nset, &at.dma);

    // 4-bit stages: activations entering a normed projection carry the norm's gain, and the rows' sums of squares
    // travel beside them as partial sums (see GemmArgs::gain_next)
    // 65 rows and more (chunked prefill, batches of segments) take the many-row projection kernel; it uses the same
    // hand-over of fragment-major activations + partial sums of squares, without gains (they are folded into the bf16 weights).
    const int l_s = rows;
    const bool w4 = d.weight_format == FS_WFMT_INT4_G128;
    const bool wide = !w4 && d.dtype == FS_BF16 && l_s >= st->tun.wide_rows;
    // In between (17 .. 64 stacked rows: more than one row tile, less than a row block and a half) the few-row kernel re-reads
    // the activations once per workgroup and is bound by the L2; gate/up, the down projection (and the LM head) then go
    // through the many-row kernel with one 64-row block of 128-feature column blocks, which works out its own RMSNorm scale
    // (gate/up) or splits K (down); QKV and the attention output have too few column blocks for that and stay with the
    // few-row kernel.
    const bool mid = !w4 && !wide && d.dtype == FS_BF16 && l_s >= st->tun.mid_rows;
    const bool mid_gu = mid && mid_cols_ok(L.layers[0].gu.n_groups * L.layers[0].gu.NT);
    const bool mid_down = mid;
    const bool handover = w4 || wide;
    float* sspa = st->at<float>(L.off_sspa);
    float* sspb = st->at<float>(L.off_sspb);
    const int res_parts = wide ? wide_ssp_parts(l_s, d.d_model / 16) : d.d_model / 16;  // partial sums per row a residual epilogue leaves
    int ssp_n_first = 0;
    if (handover)
        HIP_TRY_K(st, FS_K_PREPARE, s,
                  launch_prenorm(hidden_in, d.d_model, l_s, d.d_model, w4 ? gains : nullptr, hb, sspa, L.ssp_stride, &ssp_n_first, s));

    for (int l = 0; l < d.n_layers; ++l) {
        const LayerPlan& p = L.layers[l];
        const long long layer_off = (long long)l * kv0->stride_layer;
        const bool first = (l == 0), last = (l == d.n_layers - 1);
        // RMSNorm + QKV + RoPE + cache append
        GemmArgs g{};
        g.X = (first && !handover) ? hidden_in : hb; g.x_frag = (first && !handover) ? 0 : 1; g.ldx = d.d_model; g.M = l_s; g.K = p.qkv.K; g.nkt = p.qkv.nkt; g.N = p.qkv.N; g.Wp = p.qkv.wp;
        g.eps = d.rms_eps; g.bias = p.qkv.bias; g.rope = rope; g.q_out = q; g.krow = krow; g.layer_off = layer_off;
        g.stride_kv = kv0->stride_kv; g.stride_head = kv0->stride_head;
        g.Hq = d.n_q_heads; g.Hkv = d.n_kv_heads; g.hd = hd;
        g.ssp_in = sspa; g.ssp_n = first ? ssp_n_first : res_parts; g.ssp_stride = L.ssp_stride;
        HIP_TRY_K(st, FS_K_QKV, s, launch_proj(st, EPI_QKV, p.qkv, g, s, wide));
        // tree attention
        at.layer_off = layer_off;
        HIP_TRY_K(st, FS_K_ATTN, s, launch_attention(d.dtype, at, aMTW, aRB, s));
        // output projection + residual
        g = GemmArgs{};
        g.X = o; g.x_frag = 1; g.ldx = nq; g.M = l_s; g.K = p.o.K; g.nkt = p.o.nkt; g.N = p.o.N; g.Wp = p.o.wp;
        g.resid = first ? hidden_in : (const void*)h; g.resid_is_T = first ? 1 : 0; g.h_out = h; g.hb_out = hb; g.hb_frag = 1;
        if (handover) {
            g.gain_next = w4 ? gains + (size_t)(2 * l + 1) * d.d_model : nullptr; g.ssp_out = sspb; g.ssp_stride = L.ssp_stride;
        }
        HIP_TRY_K(st, FS_K_OPROJ, s, launch_proj(st, EPI_RESID, p.o, g, s, wide));
        // RMSNorm + gate/up + SiLU * up
        g = GemmArgs{};
        g.X = hb; g.x_frag = 1; g.ldx = d.d_model; g.M = l_s; g.K = p.gu.K; g.nkt = p.gu.nkt; g.N = 2 * p.gu.N; g.Wp = p.gu.wp; g.eps = d.rms_eps;
        g.act_out = act; g.F = d.d_ffn;
        g.ssp_in = sspb; g.ssp_n = res_parts; g.ssp_stride = L.ssp_stride;
        HIP_TRY_K(st, FS_K_GATEUP, s, launch_proj(st, EPI_SWIGLU, p.gu, g, s, wide || mid_gu));
        // down projection + residual
        g = GemmArgs{};
        g.X = act; g.x_frag = 1; g.ldx = d.d_ffn; g.M = l_s; g.K = p.down.K; g.nkt = p.down.nkt; g.N = p.down.N; g.Wp = p.down.wp;
        g.resid = h; g.resid_is_T = 0; g.h_out = h; g.hb_out = last ? hidden_out : hb; g.hb_frag = last ? 0 : 1;
        if (handover && !last) {
            g.gain_next = w4 ? gains + (size_t)(2 * l + 2) * d.d_model : nullptr; g.ssp_out = sspa; g.ssp_stride = L.ssp_stride;
        }
        HIP_TRY_K(st, FS_K_DOWN, s, launch_proj(st, EPI_RESID, p.down, g, s, wide || mid_down));
    }
    return FS_OK;
}

int fs_tree_verify_batch(fs_stage* st, const fs_batch_item* items, int n_items, const void* hidden_in, void* hidden_out, void* stream) {
    return verify_batch(st, items, n_items, hidden_in, hidden_out, stream);
}

int fs_tree_verify_stage(fs_stage* st, fs_kv_cache kv, int l_glo, int l_cache, const void* hidden_in, int seg_off, int l_s, const int32_t* parent,
                         void* hidden_out, void* stream) {
    if (!st || l_s < 0 || seg_off < 0 || l_glo < 0) return FS_EINVAL;
    if (l_cache != l_glo + seg_off) return FS_EINVAL;
    if (l_s == 0) return FS_OK;
    if (!hidden_in || !hidden_out || !parent) return FS_EINVAL;
    fs_batch_item it{kv, l_glo, l_cache, seg_off, l_s, parent};
    return verify_batch(st, &it, 1, hidden_in, hidden_out, stream);
}

int fs_tree_mask(fs_stage* st, int l_glo, int seg_off, int l_s, const int32_t* parent, uint64_t* anc, float* rope, void* stream) {
    if (!st || l_s < 0 || seg_off < 0 || l_glo < 0) return FS_EINVAL;
    if (l_s == 0) return FS_OK;
    if (!parent || !anc || !rope) return FS_EINVAL;
    const int T = seg_off + l_s;
    if (T > st->d.max_tree || l_s > st->d.max_seg) return FS_ECAP;
    if (parent[0] != -1) return FS_ETOPO;
    short depth[FS_MAX_TREE];
    int max_depth = 0;
    depth[0] = 0;
    for (int j = 1; j < T; ++j) {
        if (parent[j] < -1 || parent[j] >= j) return FS_ETOPO;
        depth[j] = parent[j] < 0 ? 0 : (short)(depth[parent[j]] + 1);
        if (depth[j] > max_depth) max_depth = depth[j];
    }
    IdxList pl;
    int rc = fill_idx(pl, parent, T);
    if (rc) return rc;
    const Layout& L = st->L;
    // the rows' cache-slot table is a by-product of the same kernels: it goes to the stage's own scratch
    KRowArgs kr{st->at<unsigned long long>(L.off_krow), 0ull, 0ull, 0};
    HIP_TRY(launch_tree_prepare(pl, max_depth, l_glo, seg_off, l_s, st->d.head_dim, st->at<double>(L.off_invf), st->at<uint64_t>(L.off_ancall), anc,
                                (float2*)rope, kr, (hipStream_t)stream));
    return FS_OK;
}

int fs_tree_logits(fs_stage* st, const void* hidden, int l_s, float* logits, int32_t* amax, void* stream) {
    if (!st || l_s < 0) return FS_EINVAL;
    if (st->d.vocab <= 0) return FS_EINVAL;
    if (l_s == 0) return FS_OK;
    if (!hidden || !logits || !amax) return FS_EINVAL;
    if (l_s > st->d.max_seg) return FS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const GemmPlan& p = st->L.head;
    GemmArgs g{};
    g.X = hidden; g.ldx = st->d.d_model; g.M = l_s; g.K = p.K; g.nkt = p.nkt; g.N = p.N; g.Wp = p.wp; g.eps = st->d.rms_eps; g.logits = logits;
    const bool wide = !p.w4 && st->d.dtype == FS_BF16 &&  // many-row kernel (see verify_batch)
                      (l_s >= st->tun.wide_rows || (l_s >= st->tun.mid_rows && mid_cols_ok(p.n_groups * p.NT)));
    if (p.w4 || wide) {  // (gained) fragment-major copy of the rows + their sums of squares, as at the entry of such a stage
        void* hb = st->at<void>(st->L.off_hb);
        float* ssp = st->at<float>(st->L.off_sspa);
        const bf16_t* gain = p.w4 ? st->at<bf16_t>(st->L.off_gain) + (size_t)(2 * st->d.n_layers) * st->d.d_model : nullptr;
        HIP_TRY_K(st, FS_K_PREPARE, s, launch_prenorm(hidden, st->d.d_model, l_s, st->d.d_model, gain, hb, ssp, st->L.ssp_stride, &g.ssp_n, s));
        g.X = hb; g.x_frag = 1; g.ssp_in = ssp; g.ssp_stride = st->L.ssp_stride;
    }
    HIP_TRY_K(st, FS_K_HEAD, s, launch_proj(st, EPI_LOGITS, p, g, s, wide));
    HIP_TRY_K(st, FS_K_ARGMAX, s, launch_argmax(logits, l_s, st->d.vocab, FS_ARGMAX_CHUNKS, st->at<int32_t>(st->L.off_amw), amax, s));
    return FS_OK;
}

int fs_tree_accept(const float* logits, int32_t* amax, int vocab, const int32_t* token, const int32_t* parent, int T, int n_ver,
                   fs_accept_result* res, int32_t* retain, int32_t* work, void* stream) {
    if (!token || !parent || !res || !retain || T < 1 || n_ver < 0 || n_ver > T) return FS_EINVAL;
    if (T > FS_MAX_TREE) return FS_ECAP;
    if (n_ver > 0 && !amax) return FS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    if (logits && n_ver > 0) {
        if (vocab < 1 || !work) return FS_EINVAL;
        HIP_TRY(launch_argmax(logits, n_ver, vocab, FS_ARGMAX_CHUNKS, work, amax, s));
    }
    static_assert(sizeof(fs_accept_result) == sizeof(AcceptResultDev), "result layouts must agree");
    HIP_TRY(launch_accept(amax, token, parent, T, n_ver, (AcceptResultDev*)res, retain, s));
    return FS_OK;
}

int fs_tree_accept_noalloc(const float* logits, int32_t* amax, int vocab, const int32_t* token, const int32_t* parent, int T, int n_ver,
                           fs_accept_result* res, int32_t* retain, void* stream) {
    if (!token || !parent || !res || !retain || T < 1 || n_ver < 0 || n_ver > T) return FS_EINVAL;
    if (T > FS_MAX_TREE) return FS_ECAP;  // the static scratch holds the partial maxima of at most FS_MAX_TREE rows
    if (n_ver > 0 && !amax) return FS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    if (logits && n_ver > 0) {
        if (vocab < 1) return FS_EINVAL;
        int32_t* work = nullptr;
        const int rc = noalloc_scratch(&work);
        if (rc) return rc;
        // every (row, chunk) entry the second argmax pass reads is written by the first: nothing has to start at zero
        HIP_TRY(launch_argmax(logits, n_ver, vocab, FS_ARGMAX_CHUNKS, work, amax, s));
    }
    HIP_TRY(launch_accept(amax, token, parent, T, n_ver, (AcceptResultDev*)res, retain, s));
    return FS_OK;
}

int fs_tree_accept_sample(const float* logits, int vocab, float temperature, const int32_t* token, const int32_t* parent, int T, int n_ver,
                          uint64_t seed, uint64_t step, fs_accept_result* res, int32_t* retain, void* work, void* stream) {
    if (!token || !parent || !res || !retain || T < 1 || n_ver < 0 || n_ver > T) return FS_EINVAL;
    if (T > FS_MAX_TREE) return FS_ECAP;
    if (!(temperature > 0.f) || vocab < 1) return FS_EINVAL;
    if (n_ver > 0 && (!logits || !work || ((uintptr_t)work & 15))) return FS_EINVAL;
    const float inv_temp = 1.0f / temperature;
    if (!(inv_temp > 0.f)) return FS_EINVAL;
    HIP_TRY(launch_accept_sample(logits, vocab, inv_temp, token, parent, T, n_ver, seed, step, (AcceptResultDev*)res, retain, work,
                                 (hipStream_t)stream));
    return FS_OK;
}

int fs_accept_result_to_host(const fs_accept_result* res_dev, const int32_t* retain_dev, int T, fs_accept_result* res_host, int32_t* retain_host,
                             void* stream) {
    if (!res_dev || !res_host || T < 0) return FS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(res_host, res_dev, sizeof(fs_accept_result), hipMemcpyDeviceToHost, s));
    if (retain_dev && retain_host && T > 0) HIP_TRY(hipMemcpyAsync(retain_host, retain_dev, sizeof(int32_t) * (size_t)T, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    return FS_OK;
}

int fs_kv_compact(fs_stage* st, fs_kv_cache kv, int l_glo, int l_cache, const int32_t* retain, const fs_accept_result* res, int n_retain_host,
                  int n_acc_host, int32_t* new_len, void* stream) {
    if (!st || !retain || l_glo < 0 || l_cache < l_glo) return FS_EINVAL;
    const fs_stage_desc& d = st->d;
    if (l_cache > d.kv_capacity) return FS_ECAP;
    int rc = valid_kv(d, kv);
    if (rc) return rc;
    CompactArgs a{};
    IdxList host;
    host.n = 0;
    if (res) {
        a.retain_dev = retain;
        a.res_dev = (const AcceptResultDev*)res;
    } else {
        if (n_retain_host < 0 || n_acc_host < 0 || n_acc_host > n_retain_host) return FS_EINVAL;
        if (n_retain_host > FS_MAX_TREE) return FS_ECAP;
        for (int j = 0; j < n_retain_host; ++j)
            if (retain[j] < 0 || (j > 0 && retain[j] <= retain[j - 1])) return FS_EINVAL;
        rc = fill_idx(host, retain, n_retain_host);
        if (rc) return rc;
        a.n_retain = n_retain_host;
        a.n_acc = n_acc_host;
    }
    a.base = kv.base; a.stride_layer = kv.stride_layer; a.stride_kv = kv.stride_kv; a.stride_head = kv.stride_head; a.stride_tok = kv.stride_tok;
    a.elem_bytes = st->elem; a.n_layers = d.n_layers; a.n_kv_heads = d.n_kv_heads; a.hd = d.head_dim;
    a.l_glo = l_glo; a.l_cache = l_cache; a.new_len = new_len;
    // split rows over column blocks until the grid has about four workgroups per compute unit (measured at 512 moved rows per
    // head, 32 heads x 8 layers: 512 workgroups 21.8 us, 1024 20.8 us, 2048 28 us)
    const int ppr = d.head_dim * st->elem / 16;
    int cb = 1;
    while ((long long)d.n_layers * 2 * d.n_kv_heads * cb < 1024 && cb * 2 <= ppr) cb *= 2;
    if (st->tun.compact_cb > 0 && st->tun.compact_cb <= ppr && ppr % st->tun.compact_cb == 0) cb = st->tun.compact_cb;
    a.colblocks = cb;
    HIP_TRY_K(st, FS_K_COMPACT, (hipStream_t)stream, launch_kv_compact(a, host, (hipStream_t)stream));
    return FS_OK;
}

int fs_seg_prune(const void* seg_in, int l_s, size_t row_bytes, int off, const int32_t* retain, const fs_accept_result* res, int n_retain_host,
                 void* seg_out, int32_t* l_s_out, void* stream) {
    if (l_s < 0 || off < 0 || !retain || (row_bytes & 3) || row_bytes == 0) return FS_EINVAL;
    if (l_s > 0 && (!seg_in || !seg_out || seg_in == seg_out)) return FS_EINVAL;
    IdxList host;
    host.n = 0;
    const int32_t* rdev = nullptr;
    if (res) {
        rdev = retain;
    } else {
        if (n_retain_host < 0) return FS_EINVAL;
        if (n_retain_host > FS_MAX_TREE) return FS_ECAP;
        for (int j = 0; j < n_retain_host; ++j)
            if (retain[j] < 0 || (j > 0 && retain[j] <= retain[j - 1])) return FS_EINVAL;
        int rc = fill_idx(host, retain, n_retain_host);
        if (rc) return rc;
    }
    HIP_TRY(launch_seg_prune(seg_in, l_s, row_bytes, off, rdev, (const AcceptResultDev*)res, host, seg_out, l_s_out, (hipStream_t)stream));
    return FS_OK;
}

}  // extern "C"
