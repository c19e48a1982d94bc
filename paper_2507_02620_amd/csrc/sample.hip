// Stochastic acceptance (temperature > 0): sequential candidate test along the tree with integer probability
// weights, so that every decision is an integer comparison and reproducible bit for bit.
//
//   z_v = logits_v * inv_temp;  m = max_v z_v;  e_v = exp2_spec((z_v - m) * log2 e);  E_v = (uint64)(e_v * 2^32);  Z = sum E_v
//   at accepted node u (remaining mass R = Z_u): children in S order; child c accepted iff r24 * R < E_c * 2^24, else
//   R -= E_c and the token is struck; no child accepted -> x_new = first v with running sum of unstruck E > u48*R/2^48.
//   Uniform numbers: counter-based generator keyed by (seed, step, draw index).
//
// exp2_spec is a fixed sequence of IEEE fp32 operations (no contraction), so any implementation produces the same bits.
#include "tree.hpp"

#pragma clang fp contract(off)

static __device__ __forceinline__ uint64_t rng64(uint64_t seed, uint64_t step, uint64_t k) {
    uint64_t z = seed ^ (step * 0x9E3779B97F4A7C15ull) ^ (k * 0xBF58476D1CE4E5B9ull);
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

static __device__ __forceinline__ uint64_t exp_weight(float z, float m) {
    const float t = __fmul_rn(__fsub_rn(z, m), 1.44269504088896341f);
    if (!(t >= -64.0f)) return 0;
    const float n = floorf(t), f = __fsub_rn(t, n);
    float p = 1.52527338e-5f;
    p = fmaf(p, f, 1.54035304e-4f);
    p = fmaf(p, f, 1.33335581e-3f);
    p = fmaf(p, f, 9.61812911e-3f);
    p = fmaf(p, f, 5.55041087e-2f);
    p = fmaf(p, f, 2.40226507e-1f);
    p = fmaf(p, f, 6.93147181e-1f);
    p = fmaf(p, f, 1.0f);
    return (uint64_t)__fmul_rn(ldexpf(p, (int)n), 4294967296.0f);
}

static __device__ uint64_t block_sum_u64(uint64_t v, uint64_t* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, FS_WAVE);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    uint64_t r = 0;
    for (int k = 0; k < (int)(blockDim.x >> 6); ++k) r += sh[k];
    return r;
}

// per verified row: m = max z, Z = sum of integer weights
__global__ void __launch_bounds__(256) sample_rowstats_kernel(const float* __restrict__ logits, int vocab, float inv_temp, float* __restrict__ rowm,
                                                              unsigned long long* __restrict__ rowZ) {
    __shared__ float shm[4];
    __shared__ uint64_t shz[4];
    const float* p = logits + (size_t)blockIdx.x * vocab;
    float m = -INFINITY;
    for (int v = threadIdx.x; v < vocab; v += blockDim.x) m = fmaxf(m, __fmul_rn(p[v], inv_temp));
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, FS_WAVE));
    if ((threadIdx.x & 63) == 0) shm[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(shm[0], shm[1]), fmaxf(shm[2], shm[3]));
    uint64_t z = 0;
    for (int v = threadIdx.x; v < vocab; v += blockDim.x) z += exp_weight(__fmul_rn(p[v], inv_temp), m);
    z = block_sum_u64(z, shz);
    if (threadIdx.x == 0) {
        rowm[blockIdx.x] = m;
        rowZ[blockIdx.x] = z;
    }
}

#define SMP_THREADS 256
#define SMP_NPT 4

__global__ void __launch_bounds__(SMP_THREADS) accept_sample_kernel(const float* __restrict__ logits, int vocab, float inv_temp,
                                                                    const float* __restrict__ rowm, const unsigned long long* __restrict__ rowZ,
                                                                    const int32_t* __restrict__ token, const int32_t* __restrict__ parent, int T,
                                                                    int n_ver, uint64_t seed, uint64_t step, AcceptResultDev* __restrict__ res,
                                                                    int32_t* __restrict__ retain) {
    __shared__ short par[1024];
    __shared__ int tok[1024];
    __shared__ unsigned char keep[1024];
    __shared__ short child[1024];
    __shared__ int rej[1024];
    __shared__ int scan[SMP_THREADS];
    __shared__ uint64_t scan64[SMP_THREADS];
    __shared__ uint64_t sh64[4];
    __shared__ int s_u, s_next, s_nrej, s_xnew, s_nnew, s_nacc;
    __shared__ uint64_t s_draw, s_target;
    const int tid = threadIdx.x;

    int bad_topo = 0;
    for (int i = tid; i < T; i += SMP_THREADS) {
        const int p = parent[i];
        bad_topo |= (p < -1 || p >= i || (i == 0 && p != -1));
        par[i] = (short)((p < -1 || p >= i) ? -1 : p);
        tok[i] = token[i];
        keep[i] = 0;
    }
    if (__syncthreads_or(bad_topo)) {
        if (tid == 0) res->n_acc = -1;
        return;
    }
    if (n_ver == 0) {
        for (int i = tid; i < T; i += SMP_THREADS) retain[i] = i;
        if (tid == 0) *res = AcceptResultDev{0, -1, 0, 1, T, 0};
        return;
    }
    if (tid == 0) {
        s_u = 0; s_draw = 0; s_nacc = 0; s_xnew = -1; s_nnew = -1;
    }
    __syncthreads();

    for (;;) {  // one iteration per accepted node: at most T of them
        const int u = s_u;
        // children of u in ascending order (parallel compaction)
        int flags[SMP_NPT], local = 0;
#pragma unroll
        for (int q = 0; q < SMP_NPT; ++q) {
            const int i = tid * SMP_NPT + q;
            flags[q] = (i < T && i > u && par[i] == u);
            local += flags[q];
        }
        scan[tid] = local;
        __syncthreads();
        for (int o = 1; o < SMP_THREADS; o <<= 1) {
            const int v = (tid >= o) ? scan[tid - o] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        int pos = scan[tid] - local;
        const int n_child = scan[SMP_THREADS - 1];
#pragma unroll
        for (int q = 0; q < SMP_NPT; ++q)
            if (flags[q]) child[pos++] = (short)(tid * SMP_NPT + q);
        __syncthreads();
        if (tid == 0) {
            keep[u] = 1;
            ++s_nacc;
            const float* row = logits + (size_t)u * vocab;
            const float m = rowm[u];
            uint64_t R = rowZ[u], draw = s_draw;
            int n_rej = 0, next = -1;
            for (int k = 0; k < n_child && next < 0; ++k) {
                const int c = child[k], t = tok[c];
                bool dup = (t < 0 || t >= vocab);
                for (int j = 0; j < n_rej && !dup; ++j) dup = (rej[j] == t);
                if (dup) continue;
                const uint64_t Ec = exp_weight(__fmul_rn(row[t], inv_temp), m);
                const uint64_t r24 = rng64(seed, step, draw++) >> 40;
                const uint64_t hi = __umul64hi(r24, R), lo = r24 * R;
                if (hi == 0 && lo < (Ec << 24)) {
                    next = c;
                } else {
                    R -= Ec;
                    rej[n_rej++] = t;
                }
            }
            s_next = next; s_nrej = n_rej;
            if (next < 0) {
                const uint64_t u48 = ((rng64(seed, step, draw) >> 40) << 24) | (rng64(seed, step, draw + 1) >> 40);
                draw += 2;
                s_target = (__umul64hi(u48, R) << 16) | ((u48 * R) >> 48);
            }
            s_draw = draw;
        }
        __syncthreads();
        const int next = s_next;
        if (next >= 0 && next < n_ver) {  // accepted and verified: descend
            if (tid == 0) s_u = next;
            __syncthreads();
            continue;
        }
        if (next >= 0) {  // accepted, not verified yet: the node n_new of the continuous condition
            if (tid == 0) {
                s_xnew = tok[next];
                s_nnew = next;
            }
        } else {  // residual draw over the vocabulary: thread t owns a contiguous chunk, integer prefix sums locate the token
            const float* row = logits + (size_t)u * vocab;
            const float m = rowm[u];
            const int n_rej = s_nrej;
            const int chunk = (vocab + SMP_THREADS - 1) / SMP_THREADS;
            const int lo = min(vocab, tid * chunk), hi = min(vocab, lo + chunk);
            auto weight = [&](int v) -> uint64_t {
                for (int j = 0; j < n_rej; ++j)
                    if (rej[j] == v) return 0;
                return exp_weight(__fmul_rn(row[v], inv_temp), m);
            };
            uint64_t mine = 0;
            for (int v = lo; v < hi; ++v) mine += weight(v);
            scan64[tid] = mine;
            __syncthreads();
            for (int o = 1; o < SMP_THREADS; o <<= 1) {
                const uint64_t v = (tid >= o) ? scan64[tid - o] : 0;
                __syncthreads();
                scan64[tid] += v;
                __syncthreads();
            }
            const uint64_t before = scan64[tid] - mine, target = s_target;
            if (tid == 0) s_xnew = vocab - 1;  // only reached if the weights changed under us; mirrors the definition's default
            __syncthreads();
            if (target >= before && target < before + mine) {
                uint64_t run = before;
                for (int v = lo; v < hi; ++v) {
                    run += weight(v);
                    if (run > target) {
                        s_xnew = v;
                        break;
                    }
                }
            }
        }
        __syncthreads();
        break;
    }

    // retain list: path nodes (keep = 1), then n_new and its descendants (keep = 2); parents precede children
    const int n_new = s_nnew;
    if (tid == 0 && n_new >= 0) {
        keep[n_new] = 2;
        for (int i = n_new + 1; i < T; ++i)
            if (par[i] >= 0 && keep[par[i]] == 2) keep[i] = 2;
    }
    __syncthreads();
    int flags[SMP_NPT], local = 0, prv = 0;
#pragma unroll
    for (int q = 0; q < SMP_NPT; ++q) {
        const int i = tid * SMP_NPT + q;
        flags[q] = (i < T && keep[i] != 0);
        local += flags[q];
        prv += (i < T && keep[i] == 2 && i < n_ver);
    }
    scan[tid] = local;
    __syncthreads();
    for (int o = 1; o < SMP_THREADS; o <<= 1) {
        const int v = (tid >= o) ? scan[tid - o] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    int pos = scan[tid] - local;
    const int total = scan[SMP_THREADS - 1];
#pragma unroll
    for (int q = 0; q < SMP_NPT; ++q)
        if (flags[q]) retain[pos++] = tid * SMP_NPT + q;
    const uint64_t prv_total = block_sum_u64((uint64_t)prv, sh64);
    if (tid == 0) *res = AcceptResultDev{s_nacc, s_xnew, n_new, n_new >= 0, total, (int)prv_total};
}

hipError_t launch_accept_sample(const float* logits, int vocab, float inv_temp, const int32_t* token, const int32_t* parent, int T, int n_ver,
                                uint64_t seed, uint64_t step, AcceptResultDev* res, int32_t* retain, void* work, hipStream_t s) {
    float* rowm = (float*)work;
    unsigned long long* rowZ = (unsigned long long*)((char*)work + (((size_t)n_ver * sizeof(float) + 15) / 16) * 16);
    if (n_ver > 0) {
        hipLaunchKernelGGL(sample_rowstats_kernel, dim3(n_ver), dim3(256), 0, s, logits, vocab, inv_temp, rowm, rowZ);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(accept_sample_kernel, dim3(1), dim3(SMP_THREADS), 0, s, logits, vocab, inv_temp, rowm, rowZ, token, parent, T, n_ver, seed,
                       step, res, retain);
    return hipGetLastError();
}
