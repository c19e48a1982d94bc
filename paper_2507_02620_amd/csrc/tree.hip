// Small latency-bound kernels around the stage forward: tree mask / positions, argmax, greedy acceptance
// with the continuous condition, KV-cache compaction and segment pruning.
#include "tree.hpp"

#include <limits.h>

// ---- tree mask + tree position ids -> rotary table ------------------------------------------------
// One thread per segment row walks its parent links to the root: every visited node sets one bit of the
// row's ancestor-or-self mask, the number of links is the node's depth.  Position id = l_glo + depth.
// The rotary table holds cos / sin of pos * theta^(-2t/hd): the angle is formed and reduced modulo 2*pi in fp64
// (inverse frequencies come from a table computed once per stage), then evaluated in fp32 on [0, 2*pi).
__global__ void rope_freq_kernel(double* __restrict__ inv_freq, int hd, float theta) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < hd / 2) inv_freq[t] = pow((double)theta, -2.0 * (double)t / (double)hd);
}
hipError_t launch_rope_freq(double* inv_freq, int hd, float theta, hipStream_t s) {
    hipLaunchKernelGGL(rope_freq_kernel, dim3(1), dim3(hd / 2), 0, s, inv_freq, hd, theta);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) tree_prepare_kernel(const IdxList parent, int l_glo, int seg_off, int l_s, int hd,
                                                           const double* __restrict__ inv_freq, uint64_t* __restrict__ anc,
                                                           float2* __restrict__ rope, KRowArgs kr) {
    for (int r = threadIdx.x; r < l_s; r += blockDim.x) kr.krow[r] = kr.base + (unsigned long long)(kr.slot0 + r) * kr.tok_bytes;
    __shared__ short par[1024];
    __shared__ int pos[1024];
    const int T = seg_off + l_s;
    for (int i = threadIdx.x; i < T; i += blockDim.x) par[i] = parent.v[i];
    __syncthreads();
    for (int r = threadIdx.x; r < l_s; r += blockDim.x) {
        uint64_t m[FS_ANC_WORDS];
#pragma unroll
        for (int w = 0; w < FS_ANC_WORDS; ++w) m[w] = 0;
        int depth = -1;
        // parent[i] < i was checked on the host, so the walk ends after at most T steps
        for (int j = seg_off + r; j >= 0; j = par[j]) {
#pragma unroll
            for (int w = 0; w < FS_ANC_WORDS; ++w)
                if (w == (j >> 6)) m[w] |= 1ull << (j & 63);
            ++depth;
        }
#pragma unroll
        for (int w = 0; w < FS_ANC_WORDS; ++w) anc[(size_t)r * FS_ANC_WORDS + w] = m[w];
        pos[r] = l_glo + depth;
    }
    __syncthreads();
    const int half = hd >> 1;
    for (int i = threadIdx.x; i < l_s * half; i += blockDim.x) {
        const int r = i / half, t = i % half;
        const double two_pi = 6.283185307179586476925286766559;
        double ang = (double)pos[r] * inv_freq[t];
        ang -= two_pi * floor(ang / two_pi);
        float sn, cs;
        sincosf((float)ang, &sn, &cs);
        rope[i] = make_float2(cs, sn);
    }
}

// Deep trees (more than 32 levels): walking to the root costs one dependent step per level, so the masks and depths are
// built by pointer doubling instead — thread i owns node i; A[i] is the set of nodes from i up to (excluding) J[i], D[i] the
// number of edges between them; each round forms A'[i] = A[i] | A[J[i]] and jumps J[i] <- J[J[i]], D[i] += D[J[i]].
// A lives in global scratch as two copies of T x 16 words: a round reads one copy and writes the other (every row is
// rewritten in full, rows that have reached the root are carried over), and J / D are read into registers before the
// barrier that precedes their update, so no location is read and written between the same two barriers.
__global__ void __launch_bounds__(1024) tree_prepare_deep_kernel(const IdxList parent, int l_glo, int seg_off, int l_s, int hd,
                                                                 const double* __restrict__ inv_freq, uint64_t* A0, uint64_t* A1,
                                                                 uint64_t* __restrict__ anc, float2* __restrict__ rope, KRowArgs kr) {
    for (int r = threadIdx.x; r < l_s; r += blockDim.x) kr.krow[r] = kr.base + (unsigned long long)(kr.slot0 + r) * kr.tok_bytes;
    __shared__ short J[1024];
    __shared__ int D[1024];
    const int T = seg_off + l_s, i = threadIdx.x;
    const int wi = i >> 6;  // ancestors of i are <= i: words above wi stay zero in both copies
    if (i < T) {
        const int p = parent.v[i];
        J[i] = (short)p;
        D[i] = p >= 0 ? 1 : 0;
        for (int w = 0; w < FS_ANC_WORDS; ++w) {
            A0[(size_t)i * FS_ANC_WORDS + w] = (w == wi) ? (1ull << (i & 63)) : 0ull;
            A1[(size_t)i * FS_ANC_WORDS + w] = 0ull;
        }
    }
    __syncthreads();
    uint64_t* cur = A0;
    uint64_t* nxt = A1;
    for (int span = 1; span < T; span <<= 1) {  // after the round every A[i] covers 2 * span levels (or reaches the root)
        const int j = (i < T) ? J[i] : -1;
        int jn = -1, dn = 0;
        if (i < T) {
            for (int w = 0; w <= wi; ++w) {
                uint64_t v = cur[(size_t)i * FS_ANC_WORDS + w];
                if (j >= 0 && w <= (j >> 6)) v |= cur[(size_t)j * FS_ANC_WORDS + w];
                nxt[(size_t)i * FS_ANC_WORDS + w] = v;
            }
            if (j >= 0) {
                jn = J[j];
                dn = D[i] + D[j];
            }
        }
        __syncthreads();  // every read of J, D and of the current copy is done
        if (j >= 0) {
            J[i] = (short)jn;
            D[i] = dn;
        }
        uint64_t* t = cur;
        cur = nxt;
        nxt = t;
        __syncthreads();  // the new copy, J and D are visible to the whole workgroup
    }
    for (int e = i; e < l_s * FS_ANC_WORDS; e += blockDim.x)
        anc[e] = cur[(size_t)(seg_off + e / FS_ANC_WORDS) * FS_ANC_WORDS + e % FS_ANC_WORDS];
    const int half = hd >> 1;
    for (int e = i; e < l_s * half; e += blockDim.x) {
        const int r = e / half, t = e % half;
        const double two_pi = 6.283185307179586476925286766559;
        double ang = (double)(l_glo + D[seg_off + r]) * inv_freq[t];
        ang -= two_pi * floor(ang / two_pi);
        float sn, cs;
        sincosf((float)ang, &sn, &cs);
        rope[e] = make_float2(cs, sn);
    }
}

// A chain (parent[i] = i - 1: a chunk of a prompt rather than a tree) needs no walk at all: node i sees nodes 0 .. i and
// sits at depth i.  One thread per mask word / rotary pair, as many workgroups as that takes.
__global__ void __launch_bounds__(256) tree_prepare_chain_kernel(int l_glo, int seg_off, int l_s, int hd, const double* __restrict__ inv_freq,
                                                                 uint64_t* __restrict__ anc, float2* __restrict__ rope, KRowArgs kr) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < l_s) kr.krow[e] = kr.base + (unsigned long long)(kr.slot0 + e) * kr.tok_bytes;
    if (e < l_s * FS_ANC_WORDS) {
        const int i = seg_off + e / FS_ANC_WORDS, w = e % FS_ANC_WORDS;
        anc[e] = w < (i >> 6) ? ~0ull : (w == (i >> 6) ? ((2ull << (i & 63)) - 1) : 0ull);
    }
    const int half = hd >> 1;
    if (e < l_s * half) {
        const int r = e / half, t = e % half;
        const double two_pi = 6.283185307179586476925286766559;
        double ang = (double)(l_glo + seg_off + r) * inv_freq[t];
        ang -= two_pi * floor(ang / two_pi);
        float sn, cs;
        sincosf((float)ang, &sn, &cs);
        rope[e] = make_float2(cs, sn);
    }
}

hipError_t launch_tree_prepare(const IdxList& parent, int max_depth, int l_glo, int seg_off, int l_s, int hd, const double* inv_freq,
                               uint64_t* anc_all, uint64_t* anc, float2* rope, const KRowArgs& kr, hipStream_t s) {
    bool chain = max_depth > 32;  // only worth looking for where the pointer-doubling kernel would run
    for (int i = 0; chain && i < seg_off + l_s; ++i) chain = parent.v[i] == i - 1;
    if (chain) {
        const int n = l_s * (FS_ANC_WORDS > hd / 2 ? FS_ANC_WORDS : hd / 2);
        hipLaunchKernelGGL(tree_prepare_chain_kernel, dim3((n + 255) / 256), dim3(256), 0, s, l_glo, seg_off, l_s, hd, inv_freq, anc, rope, kr);
        return hipGetLastError();
    }
    if (max_depth > 32)
        hipLaunchKernelGGL(tree_prepare_deep_kernel, dim3(1), dim3(1024), 0, s, parent, l_glo, seg_off, l_s, hd, inv_freq, anc_all,
                           anc_all + (size_t)(seg_off + l_s) * FS_ANC_WORDS, anc, rope, kr);
    else
        hipLaunchKernelGGL(tree_prepare_kernel, dim3(1), dim3(256), 0, s, parent, l_glo, seg_off, l_s, hd, inv_freq, anc, rope, kr);
    return hipGetLastError();
}

// ---- row argmax (lowest index of the maximum; '>' comparisons, so NaN never wins) -----------------
struct Best {
    float v;
    int i;
};
static __device__ __forceinline__ Best better(Best a, Best b) { return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a; }

static __device__ Best block_best(Best b) {
    __shared__ float sv[16];
    __shared__ int si[16];
    for (int o = 32; o > 0; o >>= 1) {
        Best t{__shfl_xor(b.v, o, FS_WAVE), __shfl_xor(b.i, o, FS_WAVE)};
        b = better(b, t);
    }
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        sv[w] = b.v;
        si[w] = b.i;
    }
    __syncthreads();
    Best r{sv[0], si[0]};
    for (int k = 1; k < nw; ++k) r = better(r, Best{sv[k], si[k]});
    return r;
}

__global__ void __launch_bounds__(256) argmax_partial_kernel(const float* __restrict__ logits, int vocab, int chunk_len, int32_t* __restrict__ work) {
    const int row = blockIdx.y, c = blockIdx.x;
    const int lo = c * chunk_len, hi = min(vocab, lo + chunk_len);
    const float* p = logits + (size_t)row * vocab;
    Best b{-INFINITY, lo < vocab ? lo : 0};
    for (int i = lo + threadIdx.x; i < hi; i += blockDim.x) {
        const float v = p[i];
        if (v > b.v) b = Best{v, i};
    }
    b = block_best(b);
    if (threadIdx.x == 0) {
        work[((size_t)row * gridDim.x + c) * 2] = __float_as_int(b.v);
        work[((size_t)row * gridDim.x + c) * 2 + 1] = b.i;
    }
}

__global__ void __launch_bounds__(64) argmax_final_kernel(const int32_t* __restrict__ work, int chunks, int32_t* __restrict__ amax) {
    const int row = blockIdx.x;
    Best b{-INFINITY, 0};
    for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
        Best t{__int_as_float(work[((size_t)row * chunks + c) * 2]), work[((size_t)row * chunks + c) * 2 + 1]};
        b = better(b, t);
    }
    for (int o = 32; o > 0; o >>= 1) {
        Best t{__shfl_xor(b.v, o, FS_WAVE), __shfl_xor(b.i, o, FS_WAVE)};
        b = better(b, t);
    }
    if (threadIdx.x == 0) amax[row] = b.i;
}

// From 64 rows on there are enough workgroups with one per row: a single launch, every thread with several independent
// 16-byte loads in flight (512 rows x 32000: 35 -> 16 us; at 16 - 32 rows the two-launch form with 64 chunks per row is as
// fast or faster).
__global__ void __launch_bounds__(1024) argmax_row_kernel(const float* __restrict__ logits, int vocab, int32_t* __restrict__ amax) {
    const int row = blockIdx.x;
    const float* p = logits + (size_t)row * vocab;
    Best b{-INFINITY, 0};
    if ((vocab & 3) == 0 && ((uintptr_t)logits & 15) == 0) {
        const f32x4* p4 = (const f32x4*)p;
        const int n4 = vocab >> 2;
#pragma unroll 4
        for (int i = threadIdx.x; i < n4; i += blockDim.x) {
            const f32x4 v = p4[i];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (v[e] > b.v) b = Best{v[e], 4 * i + e};
        }
    } else {
        for (int i = threadIdx.x; i < vocab; i += blockDim.x) {
            const float v = p[i];
            if (v > b.v) b = Best{v, i};
        }
    }
    b = block_best(b);
    if (threadIdx.x == 0) amax[row] = b.i;
}

hipError_t launch_argmax(const float* logits, int rows, int vocab, int chunks, int32_t* work, int32_t* amax, hipStream_t s) {
    if (rows >= 64) {
        hipLaunchKernelGGL(argmax_row_kernel, dim3(rows), dim3(1024), 0, s, logits, vocab, amax);
        return hipGetLastError();
    }
    const int chunk_len = (vocab + chunks - 1) / chunks;
    hipLaunchKernelGGL(argmax_partial_kernel, dim3(chunks, rows), dim3(256), 0, s, logits, vocab, chunk_len, work);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(argmax_final_kernel, dim3(rows), dim3(64), 0, s, work, chunks, amax);
    return hipGetLastError();
}

// ---- greedy acceptance, continuous condition, retain set ------------------------------------------
// One workgroup of 256 threads, thread t owns nodes 4t .. 4t+3 (T <= 1024).  Everything that follows a
// parent chain (depth, "all edges on the path match", k-th ancestor) is done by pointer doubling in
// ceil(log2 T) rounds, keeping the 2^k-th ancestor table up[k][] in LDS for the ancestor queries.
#define ACC_THREADS 256
#define ACC_NPT 4
#define ACC_LOG 10

static __device__ int block_reduce_max(int v, int* sh) {
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, FS_WAVE));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = sh[0];
    for (int k = 1; k < (int)(blockDim.x >> 6); ++k) r = max(r, sh[k]);
    return r;
}
static __device__ int block_reduce_add(int v, int* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, FS_WAVE);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = 0;
    for (int k = 0; k < (int)(blockDim.x >> 6); ++k) r += sh[k];
    return r;
}

__global__ void __launch_bounds__(ACC_THREADS) accept_kernel(const int32_t* __restrict__ amax, const int32_t* __restrict__ token,
                                                             const int32_t* __restrict__ parent, int T, int n_ver,
                                                             AcceptResultDev* __restrict__ res, int32_t* __restrict__ retain) {
    __shared__ short up[ACC_LOG + 1][1024];  // up[k][i] = 2^k-th ancestor of i, -1 beyond the root
    __shared__ int cnt[2][1024];             // low 16 bits: nodes on the path so far; high bits: non-matching nodes
    __shared__ int red[8];
    __shared__ int scan[ACC_THREADS];
    const int tid = threadIdx.x;

    // topology check: -1 <= parent[i] < i, parent[0] == -1
    int bad_topo = 0;
    for (int i = tid; i < T; i += ACC_THREADS) {
        const int p = parent[i];
        bad_topo |= (p < -1 || p >= i || (i == 0 && p != -1));
        up[0][i] = (short)((p < -1 || p >= i) ? -1 : p);
    }
    if (__syncthreads_or(bad_topo)) {
        if (tid == 0) res->n_acc = -1;
        return;
    }
    if (n_ver == 0) {  // nothing verified: keep everything, the context is not updated
        for (int i = tid; i < T; i += ACC_THREADS) retain[i] = i;
        if (tid == 0) *res = AcceptResultDev{0, -1, 0, 1, T, 0};
        return;
    }
    // match flags
    for (int i = tid; i < T; i += ACC_THREADS) {
        const int p = up[0][i];
        const bool match = (i > 0) && (p >= 0) && (p < n_ver) && (token[i] == amax[p]);
        cnt[0][i] = 1 | ((i > 0 && !match) ? (1 << 16) : 0);
    }
    __syncthreads();
    int cur = 0;
    for (int k = 0; k < ACC_LOG; ++k) {
        for (int i = tid; i < T; i += ACC_THREADS) {
            const int j = up[k][i];
            cnt[cur ^ 1][i] = cnt[cur][i] + (j >= 0 ? cnt[cur][j] : 0);
            up[k + 1][i] = (j >= 0) ? up[k][j] : (short)-1;
        }
        cur ^= 1;
        __syncthreads();
    }
    const int* c = cnt[cur];  // depth[i] = (c[i] & 0xffff) - 1, ok[i] = (c[i] >> 16) == 0

    // e = verified ok node of maximum depth, lowest S index among equals
    int key = -1;
    for (int i = tid; i < n_ver; i += ACC_THREADS)
        if ((c[i] >> 16) == 0) key = max(key, (((c[i] & 0xffff) - 1) << 11) | (2047 - i));
    key = block_reduce_max(key, red);
    const int e = 2047 - (key & 2047), depth_e = key >> 11;
    const int x_new = amax[e];
    // n_new = lowest-index child of e carrying x_new
    int cand = -1;
    for (int i = tid; i < T; i += ACC_THREADS)
        if (up[0][i] == e && token[i] == x_new) cand = max(cand, 2047 - i);
    cand = block_reduce_max(cand, red);
    const int n_new = cand < 0 ? -1 : 2047 - cand;
    const int depth_n = depth_e + 1;

    // membership: I_acc = ancestors-or-self of e; I_pr = descendants-or-self of n_new
    int flags[ACC_NPT], local = 0, prv = 0;
#pragma unroll
    for (int q = 0; q < ACC_NPT; ++q) {
        const int i = tid * ACC_NPT + q;
        int f = 0;
        if (i < T) {
            const int di = (c[i] & 0xffff) - 1;
            if (di <= depth_e) {
                int x = e, d = depth_e - di;
                for (int k = 0; k < ACC_LOG; ++k)
                    if ((d >> k) & 1) x = up[k][x];
                f = (x == i);
            } else if (n_new >= 0) {
                int x = i, d = di - depth_n;
                for (int k = 0; k < ACC_LOG; ++k)
                    if ((d >> k) & 1) x = up[k][x];
                f = (x == n_new);
                prv += (f && i < n_ver);
            }
        }
        flags[q] = f;
        local += f;
    }
    // exclusive scan of per-thread counts -> positions in the ascending retain list
    scan[tid] = local;
    __syncthreads();
    for (int o = 1; o < ACC_THREADS; o <<= 1) {
        const int v = (tid >= o) ? scan[tid - o] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    int posn = scan[tid] - local;
    const int total = scan[ACC_THREADS - 1];
#pragma unroll
    for (int q = 0; q < ACC_NPT; ++q)
        if (flags[q]) retain[posn++] = tid * ACC_NPT + q;
    prv = block_reduce_add(prv, red);
    if (tid == 0) *res = AcceptResultDev{depth_e + 1, x_new, n_new, n_new >= 0, total, prv};
}

hipError_t launch_accept(const int32_t* amax, const int32_t* token, const int32_t* parent, int T, int n_ver, AcceptResultDev* res,
                         int32_t* retain, hipStream_t s) {
    hipLaunchKernelGGL(accept_kernel, dim3(1), dim3(ACC_THREADS), 0, s, amax, token, parent, T, n_ver, res, retain);
    return hipGetLastError();
}

// ---- KV-cache compaction --------------------------------------------------------------------------
// Block (item, cb): item = (layer, K|V, head); cb = column block of the row's 16-byte pieces.  Rows move
// towards lower slots (I_incache[j] >= j), in place.  A block moves CH rows per step: all loads of the step,
// a barrier, then all stores.  Stores of a step only hit slots below every source of later steps, and
// different blocks touch disjoint bytes, so no other ordering is needed.
// 256 threads with 8 pieces of 16 bytes in flight each (measured at 512 moved rows per head, 134 MB read + written: 4 pieces
// 21.8 us, 8 pieces 20.8 us, 16 pieces or 512 / 1024 threads 36 - 60 us: a launch whose workgroups all read and then all
// write floods the L2 with dirty lines; streaming stores 21.5 us, streaming loads 28.5 us).  The pieces are native 4 x 32-bit
// vectors: with the runtime's uint4 struct type the same loop took 32 - 36 us.
template <int THREADS, int UNROLL>
__global__ void __launch_bounds__(THREADS) kv_compact_kernel(const CompactArgs a, const IdxList host) {
    __shared__ short src[1024];
    __shared__ int sh_n;
    const int tid = threadIdx.x;
    const int n_retain = a.retain_dev ? a.res_dev->n_retain : a.n_retain;
    const int n_acc = a.retain_dev ? a.res_dev->n_acc : a.n_acc;
    if (n_acc < 0) return;  // acceptance reported a broken tree: leave the cache alone
    const int n_draft = a.l_cache - a.l_glo;
    if (tid == 0) sh_n = 0;
    __syncthreads();
    // I_incache is a prefix of the ascending retain list
    int cntl = 0;
    for (int j = tid; j < n_retain && j < 1024; j += THREADS) {
        const int i = a.retain_dev ? a.retain_dev[j] : (int)host.v[j];
        src[j] = (short)i;
        cntl += (i < n_draft);
    }
    if (cntl) atomicAdd(&sh_n, cntl);
    __syncthreads();
    const int n_in = sh_n;
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0 && a.new_len) {
        a.new_len[0] = a.l_glo + n_acc;
        a.new_len[1] = a.l_glo + n_in;
    }
    const int item = blockIdx.x, cb = blockIdx.y;
    const int head = item % a.n_kv_heads, kv = (item / a.n_kv_heads) & 1, layer = item / (2 * a.n_kv_heads);
    unsigned char* hp = (unsigned char*)a.base +
                        ((size_t)layer * a.stride_layer + (size_t)kv * a.stride_kv + (size_t)head * a.stride_head) * a.elem_bytes;
    const size_t tok_bytes = (size_t)a.stride_tok * a.elem_bytes;
    const int ppr = a.hd * a.elem_bytes / 16;      // 16-byte pieces per row
    const int ppb = ppr / a.colblocks;             // pieces per row handled by this block
    const int rows_per_pass = THREADS / ppb;       // ppb divides THREADS (checked on the host)
    const int piece = cb * ppb + tid % ppb, rloc = tid / ppb;
    const int CH = rows_per_pass * UNROLL;
    // leading rows that already sit in place need no move
    int j0 = 0;
    while (j0 < n_in && src[j0] == j0) ++j0;
    for (int jb = j0; jb < n_in; jb += CH) {
        u32x4 buf[UNROLL];
        // no branch around a load: rows past the end re-read the last one (never stored), so the loads of a step go out
        // back to back and the compiler counts them exactly instead of waiting for each in turn
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int j = min(jb + u * rows_per_pass + rloc, n_in - 1);
            const u32x4* sp = (const u32x4*)(hp + (size_t)(a.l_glo + src[j]) * tok_bytes + (size_t)piece * 16);
            buf[u] = *sp;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int j = jb + u * rows_per_pass + rloc;
            u32x4* dp = (u32x4*)(hp + (size_t)(a.l_glo + j) * tok_bytes + (size_t)piece * 16);
            if (j < n_in) *dp = buf[u];
        }
        __syncthreads();  // (only matters with several steps) the step's stores are issued before the next step's loads
    }
}

hipError_t launch_kv_compact(const CompactArgs& a, const IdxList& host, hipStream_t s) {
    hipLaunchKernelGGL((kv_compact_kernel<256, 8>), dim3(a.n_layers * 2 * a.n_kv_heads, a.colblocks), dim3(256), 0, s, a, host);
    return hipGetLastError();
}

// ---- segment pruning ------------------------------------------------------------------------------
// One block per input row r (S index off + r): binary search in the ascending retain list gives membership
// and the row's rank among the kept rows of this segment.
static __device__ __forceinline__ int idx_at(const int32_t* dev, const IdxList& host, int j) { return dev ? dev[j] : (int)host.v[j]; }
static __device__ int lower_bound(const int32_t* dev, const IdxList& host, int n, int key) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (idx_at(dev, host, mid) < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ void __launch_bounds__(256) seg_prune_kernel(const unsigned char* __restrict__ seg_in, int l_s, size_t row_bytes, int off,
                                                        const int32_t* retain_dev, const AcceptResultDev* res_dev, const IdxList host,
                                                        unsigned char* __restrict__ seg_out, int32_t* l_s_out) {
    const int n_retain = retain_dev ? res_dev->n_retain : host.n;
    if (retain_dev && res_dev->n_acc < 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0 && l_s_out) *l_s_out = -1;
        return;
    }
    const int first = lower_bound(retain_dev, host, n_retain, off);
    if (blockIdx.x == 0 && threadIdx.x == 0 && l_s_out) *l_s_out = lower_bound(retain_dev, host, n_retain, off + l_s) - first;
    const int r = blockIdx.x;
    if (r >= l_s) return;
    const int p = lower_bound(retain_dev, host, n_retain, off + r);
    if (p >= n_retain || idx_at(retain_dev, host, p) != off + r) return;
    const uint32_t* s = (const uint32_t*)(seg_in + (size_t)r * row_bytes);
    uint32_t* d = (uint32_t*)(seg_out + (size_t)(p - first) * row_bytes);
    for (size_t i = threadIdx.x; i < row_bytes / 4; i += blockDim.x) d[i] = s[i];
}

hipError_t launch_seg_prune(const void* seg_in, int l_s, size_t row_bytes, int off, const int32_t* retain_dev, const AcceptResultDev* res_dev,
                            const IdxList& host, void* seg_out, int32_t* l_s_out, hipStream_t s) {
    hipLaunchKernelGGL(seg_prune_kernel, dim3(l_s > 0 ? l_s : 1), dim3(256), 0, s, (const unsigned char*)seg_in, l_s, row_bytes, off, retain_dev,
                       res_dev, host, (unsigned char*)seg_out, l_s_out);
    return hipGetLastError();
}
