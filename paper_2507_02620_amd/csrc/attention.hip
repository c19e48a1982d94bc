// Tree attention of one draft segment against the stage's KV cache (split-KV, LDS-staged, MFMA).
//
// Rows: the segment's M rows of the G = Hq/Hkv query heads that share one KV head are stacked into
// R = G*M rows (rho = qh_local*M + r) so that each K/V element fetched from HBM serves all of them.
// Grid: (KV split, KV head, row block).  A workgroup walks its slots in tiles of BS = 64: the tile's K rows
// are copied to LDS as they are, its V rows transposed (Vt[t][slot]) so that both MFMA operands are
// 16-byte LDS reads.  Each wave owns MTW 16-row tiles of R:
//     S^T = K . Q^T      (A = K fragment, rows = slots; B = Q fragment, rows = query rows)
//     O^T += V^T . P^T   (A = V^T fragment, rows = head-dim index; B = P fragment, rows = query rows)
// Both products leave lane l with values of query row l % 16, so the online-softmax state (running max,
// running sum, rescale factor) is per lane and P never leaves registers: lane (r, g) holds
// S^T[slot = 16*j + 4*g + v][r], which is exactly the B-fragment element order of a contraction index
// permuted as slot = 16*(e/4) + 4*g + e%4 — the V^T fragment is read with the same permutation.
//
// Visibility (tree mask): slot s is seen by row r iff s < l_glo, or bit (s - l_glo) of the row's
// ancestor-or-self mask is set.  Tiles that lie entirely below l_glo skip the mask test.
// With more than one split the kernel writes un-normalised partial outputs plus (max, sum) per row and
// attn_merge_kernel combines them in split order (deterministic).
#include "attention.hpp"

#define PADK 8   /* elements; keeps K rows 16-byte aligned and spreads LDS banks */
#define PADV 16
#define NEG_BIG (-1.0e30f)

template <typename T, int HD, int MTW>
__global__ void __launch_bounds__(512) tree_attn_kernel(const AttnArgs a) {
    using E = Elem<T>;
    using frag_t = typename E::frag_t;
    constexpr int EPF = E::EPF, KT = E::KT;
    constexpr int BS = (sizeof(T) * HD >= 512) ? 32 : 64;  // slots per LDS tile (keeps K + V^T within 64 KiB)
    constexpr int NKT = HD / KT;      // k-tiles of the head dim (QK^T contraction)
    constexpr int NHT = HD / 16;      // 16-wide tiles of the head dim (rows of O^T)
    constexpr int NSUB = EPF / 4;     // 16-slot sub-tiles per P fragment
    constexpr int NPF = BS / (16 * NSUB);
    constexpr int KROW = HD + PADK, VROW = BS + PADV;
    __shared__ __align__(16) T Ks[BS * KROW];
    __shared__ __align__(16) T Vt[HD * VROW];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, NW = blockDim.x >> 6, nthr = blockDim.x;
    const int r16 = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, rb = blockIdx.z;
    const int R = a.G * a.M;
    const int ntiles = (a.L + BS - 1) / BS;
    const int t0 = split * a.tiles_per_split, t1 = min(ntiles, t0 + a.tiles_per_split);

    // rows of this wave
    int rho[MTW], seg_r[MTW];
    bool rok[MTW];
    frag_t qf[MTW][NKT];
#pragma unroll
    for (int i = 0; i < MTW; ++i) {
        rho[i] = ((rb * NW + w) * MTW + i) * 16 + r16;
        rok[i] = rho[i] < R;
        const int rr = rok[i] ? rho[i] : 0;
        seg_r[i] = rr % a.M;
        const int qh = kvh * a.G + rr / a.M;
        const T* qp = (const T*)a.q + (size_t)seg_r[i] * (a.Hq * HD) + (size_t)qh * HD + g * EPF;
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) qf[i][kt] = rok[i] ? *(const frag_t*)(qp + kt * KT) : E::zero();
    }

    f32x4 acc[MTW][NHT];
    float mrun[MTW], lrun[MTW];
#pragma unroll
    for (int i = 0; i < MTW; ++i) {
        mrun[i] = NEG_BIG;
        lrun[i] = 0.f;
#pragma unroll
        for (int nt = 0; nt < NHT; ++nt) acc[i][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const T* kbase = (const T*)a.k_layer + (size_t)kvh * a.stride_head;
    const T* vbase = kbase + a.stride_kv;
    constexpr int NCC = HD / EPF;  // 16-byte chunks per row

    for (int tile = t0; tile < t1; ++tile) {
        const int s0 = tile * BS;
        __syncthreads();  // previous tile fully consumed
        // ---- stage K (as is) and V (transposed) ----
        for (int c = tid; c < BS * NCC; c += nthr) {
            const int slot = c / NCC, col = (c % NCC) * EPF;
            frag_t f = (s0 + slot < a.L) ? *(const frag_t*)(kbase + (size_t)(s0 + slot) * a.stride_tok + col) : E::zero();
            *(frag_t*)(&Ks[slot * KROW + col]) = f;
        }
        for (int c = tid; c < BS * NCC; c += nthr) {
            // lane -> (slot_lo, chunk part) so that one store instruction spreads over the LDS banks
            const int it = c >> 6, ln = c & 63;
            const int ncb = NCC / 4;
            const int slot = (it / ncb) * 16 + (ln & 15), col = ((it % ncb) * 4 + (ln >> 4)) * EPF;
            frag_t f = (s0 + slot < a.L) ? *(const frag_t*)(vbase + (size_t)(s0 + slot) * a.stride_tok + col) : E::zero();
#pragma unroll
            for (int e = 0; e < EPF; ++e) Vt[(col + e) * VROW + slot] = f[e];
        }
        __syncthreads();

        // ---- S^T = K . Q^T ----
        f32x4 st[MTW][BS / 16];
#pragma unroll
        for (int j = 0; j < BS / 16; ++j) {
#pragma unroll
            for (int i = 0; i < MTW; ++i) st[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kt = 0; kt < NKT; ++kt) {
                frag_t kf = *(const frag_t*)(&Ks[(j * 16 + r16) * KROW + kt * KT + g * EPF]);
#pragma unroll
                for (int i = 0; i < MTW; ++i) st[i][j] = E::mma(kf, qf[i][kt], st[i][j]);
            }
        }

        // ---- mask, online softmax ----
        const bool need_mask = (s0 + BS > a.l_glo);  // tile touches draft slots or the tail beyond L
        frag_t pf[MTW][NPF];
#pragma unroll
        for (int i = 0; i < MTW; ++i) {
            float mx = NEG_BIG;
#pragma unroll
            for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float s = st[i][j][v] * a.scale_log2;
                    if (need_mask) {
                        const int slot = s0 + j * 16 + g * 4 + v;
                        bool vis = slot < a.l_glo;
                        if (!vis && slot < a.L) {
                            const int dj = slot - a.l_glo;
                            vis = (a.anc[(size_t)seg_r[i] * FS_ANC_WORDS + (dj >> 6)] >> (dj & 63)) & 1ull;
                        }
                        if (!vis) s = NEG_BIG;
                    }
                    st[i][j][v] = s;
                    mx = fmaxf(mx, s);
                }
            mx = wave_xor_max(wave_xor_max(mx, 16), 32);
            const float mnew = fmaxf(mrun[i], mx);
            const float alpha = exp2f(mrun[i] - mnew);
            mrun[i] = mnew;
            float psum = 0.f;
            float p[BS / 16][4];
#pragma unroll
            for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float s = st[i][j][v];
                    const float e = (s <= NEG_BIG) ? 0.f : exp2f(s - mnew);
                    p[j][v] = e;
                    psum += e;
                }
            lrun[i] = lrun[i] * alpha + psum;
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][nt][v] *= alpha;
#pragma unroll
            for (int jj = 0; jj < NPF; ++jj)
#pragma unroll
                for (int e = 0; e < EPF; ++e) pf[i][jj][e] = E::from_f(p[jj * NSUB + e / 4][e % 4]);
        }

        // ---- O^T += V^T . P^T ----
#pragma unroll
        for (int jj = 0; jj < NPF; ++jj)
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt) {
                frag_t vf;
                const T* vr = &Vt[(nt * 16 + r16) * VROW + jj * NSUB * 16 + g * 4];
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
                    for (int v = 0; v < 4; ++v) vf[sub * 4 + v] = vr[sub * 16 + v];
#pragma unroll
                for (int i = 0; i < MTW; ++i) acc[i][nt] = E::mma(vf, pf[i][jj], acc[i][nt]);
            }
    }

    // ---- write out ----
#pragma unroll
    for (int i = 0; i < MTW; ++i) {
        const float l = wave_xor_add(wave_xor_add(lrun[i], 16), 32);
        if (!rok[i]) continue;
        if (a.n_splits == 1) {
            const float inv = 1.0f / l;
            const int qh = kvh * a.G + rho[i] / a.M;
            T* op = (T*)a.o + (size_t)seg_r[i] * (a.Hq * HD) + (size_t)qh * HD + g * 4;
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt)
                *(typename E::out4_t*)(op + nt * 16) = E::pack4(acc[i][nt][0] * inv, acc[i][nt][1] * inv, acc[i][nt][2] * inv, acc[i][nt][3] * inv);
        } else {
            const size_t prow = ((size_t)split * a.Hkv + kvh) * a.Rpad + rho[i];
            float* po = a.part_o + prow * HD + g * 4;
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt) *(f32x4*)(po + nt * 16) = acc[i][nt];
            if (g == 0) *(float2*)(a.part_ml + prow * 2) = make_float2(mrun[i], l);
        }
    }
}

// Combine the splits of one (KV head, row): out = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s, in split order.
template <typename T>
__global__ void attn_merge_kernel(const AttnArgs a) {
    using E = Elem<T>;
    const int R = a.G * a.M, hd4 = a.hd / 4;
    const size_t total = (size_t)a.Hkv * R * hd4;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % hd4);
        const int rho = (int)((idx / hd4) % R);
        const int kvh = (int)(idx / ((size_t)hd4 * R));
        float m = NEG_BIG;
        for (int s = 0; s < a.n_splits; ++s) m = fmaxf(m, a.part_ml[(((size_t)s * a.Hkv + kvh) * a.Rpad + rho) * 2]);
        float den = 0.f;
        f32x4 o{0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < a.n_splits; ++s) {
            const size_t prow = ((size_t)s * a.Hkv + kvh) * a.Rpad + rho;
            const float2 ml = *(const float2*)(a.part_ml + prow * 2);
            const float wgt = exp2f(ml.x - m);
            den += wgt * ml.y;
            const f32x4 po = *(const f32x4*)(a.part_o + prow * a.hd + c * 4);
            o += po * wgt;
        }
        const float inv = 1.0f / den;
        const int qh = kvh * a.G + rho / a.M, r = rho % a.M;
        *(typename E::out4_t*)((T*)a.o + (size_t)r * (a.Hq * a.hd) + (size_t)qh * a.hd + c * 4) =
            E::pack4(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv);
    }
}

template <typename T, int HD>
static hipError_t launch_hd(const AttnArgs& a, int NW, int MTW, int row_blocks, hipStream_t s) {
    dim3 grid(a.n_splits, a.Hkv, row_blocks), block(NW * 64);
    if (MTW == 1)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 2>), grid, block, 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.n_splits > 1) {
        const size_t total = (size_t)a.Hkv * a.G * a.M * (a.hd / 4);
        int blocks = (int)((total + 255) / 256);
        hipLaunchKernelGGL(attn_merge_kernel<T>, dim3(blocks), dim3(256), 0, s, a);
        e = hipGetLastError();
    }
    return e;
}

void attn_plan(int elem_bytes, int hd, int M, int G, int Hkv, int L, int max_splits, int* NW, int* MTW, int* row_blocks, int* n_splits, int* tiles_per_split) {
    const int R = G * M, mtiles = (R + 15) / 16;
    // up to 8 waves per workgroup, each with 1 or 2 row tiles
    int nw = mtiles < 8 ? mtiles : 8;
    int mtw = (mtiles + nw - 1) / nw > 1 ? 2 : 1;
    nw = (mtiles + mtw - 1) / mtw;
    if (nw > 8) nw = 8;
    *NW = nw;
    *MTW = mtw;
    *row_blocks = (mtiles + nw * mtw - 1) / (nw * mtw);
    const int BS = attn_tile_slots(elem_bytes, hd);
    const int ntiles = (L + BS - 1) / BS;
    int want = (1024 + Hkv * *row_blocks - 1) / (Hkv * *row_blocks);  // about 4 workgroups per CU
    if (want > max_splits) want = max_splits;
    if (want > ntiles) want = ntiles;
    if (want < 1) want = 1;
    *tiles_per_split = (ntiles + want - 1) / want;
    *n_splits = (ntiles + *tiles_per_split - 1) / *tiles_per_split;
}

hipError_t launch_attention(int dtype, const AttnArgs& a, int NW, int MTW, int row_blocks, hipStream_t s) {
    if (a.hd == 64) return dtype == 0 ? launch_hd<float, 64>(a, NW, MTW, row_blocks, s) : launch_hd<bf16_t, 64>(a, NW, MTW, row_blocks, s);
    if (a.hd == 128) return dtype == 0 ? launch_hd<float, 128>(a, NW, MTW, row_blocks, s) : launch_hd<bf16_t, 128>(a, NW, MTW, row_blocks, s);
    return hipErrorInvalidValue;
}
