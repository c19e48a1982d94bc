// Skinny-M projection kernels and the one-time weight re-tiling.
//
// Work decomposition: workgroup (grp, mb) owns NT consecutive 16-feature tiles ("group" grp) for the
// MT*16 rows of row block mb.  Its NW waves split the K range round-robin; wave w streams the weight
// fragments of k-tiles w, w + NW, ... — NT contiguous KiB per k-tile in the re-tiled layout — and
// multiplies them with the activation fragments of the same k-tiles (read through L2).
// Partial 16x16 tiles are summed across waves through LDS, then the epilogue runs on the reduced tile.
//
// Operand roles: A = weights (rows = output features), B = activations (rows = segment rows), so the
// result tile is Y^T: lane l holds features n = (l/16)*4 + v, v = 0..3, of row m = l % 16 — four
// consecutive features of one row per lane: vector stores, and per-row scalars (RMSNorm scale) are
// per-lane.
//
// RMSNorm is split algebraically: norm(x) . w = rs(x) * sum_k x_k g_k w_k.  The gain g is folded into the
// re-tiled weights once; rs(x) = rsqrt(mean(x^2) + eps) is computed from the activation fragments the
// workgroup reads anyway (it covers the whole K range) and applied in the epilogue.
#include "gemm.hpp"


typedef __attribute__((ext_vector_type(2))) bf16_t bf16x2;
struct bf16x2x4 {
    bf16x2 v[4];
};

template <typename T>
static __device__ __forceinline__ typename Elem<T>::frag_t load_w(const void* p) {
    using frag_t = typename Elem<T>::frag_t;
    return __builtin_nontemporal_load((const frag_t*)p);
}

// Residual-stream values [m][n .. n+3] (fp32 stream, or the T-typed stage input at the first layer).
template <typename T>
static __device__ __forceinline__ f32x4 load_resid(const GemmArgs& a, int m, int n) {
    using E = Elem<T>;
    if (a.resid_is_T) {
        const T* p = (const T*)a.resid + (size_t)m * a.N + n;
        return f32x4{E::to_f(p[0]), E::to_f(p[1]), E::to_f(p[2]), E::to_f(p[3])};
    }
    return *(const f32x4*)((const float*)a.resid + (size_t)m * a.N + n);
}

// The residual values of the item a wave will finish first (item w), fetched before the K loop so that the epilogue does
// not start with a dependent global load.  Only this workgroup ever writes those elements, so reading them early is safe
// even when the projection updates the residual stream in place.
template <typename T, int MT, int NT, int EPI>
static __device__ __forceinline__ f32x4 prefetch_resid(const GemmArgs& a, int w, int grp, int row0, int r16, int g) {
    f32x4 v{0.f, 0.f, 0.f, 0.f};
    if constexpr (EPI == EPI_RESID) {
        if (w < MT * NT) {
            const int m = row0 + (w / NT) * 16 + r16, n = (grp * NT + w % NT) * 16 + g * 4;
            if (m < a.M && n < a.N) v = load_resid<T>(a, m, n);
        }
    }
    return v;
}

// Fused epilogue for one "item": one 16x16 result tile (RESID, LOGITS) or a pair of tiles (QKV, SWIGLU) in the
// MFMA result layout — this lane holds features g*4 + v of row m; rs is the row's RMSNorm scale.
// Returns this lane's share of the sum of squares of the new residual-stream values (RESID), else 0.
template <typename T, int EPI>
static __device__ __forceinline__ float epilogue_item(const GemmArgs& a, const float (&y)[(EPI == EPI_QKV || EPI == EPI_SWIGLU) ? 2 : 1][4],
                                                      float rs, int m, int ptile, int g, const f32x4* resid_pre = nullptr) {
    using E = Elem<T>;
    float hsq = 0.f;
    if constexpr (EPI != EPI_RESID) {
        if (m >= a.M) return 0.f;
    }
    if constexpr (EPI == EPI_RESID) {
        const int n = ptile * 16 + g * 4;
        if (m < a.M && n < a.N) {
            const f32x4 rv = resid_pre ? *resid_pre : load_resid<T>(a, m, n);
            const float r[4] = {rv[0], rv[1], rv[2], rv[3]};
            f32x4 h{r[0] + y[0][0], r[1] + y[0][1], r[2] + y[0][2], r[3] + y[0][3]};
            *(f32x4*)(a.h_out + (size_t)m * a.N + n) = h;
            hsq = h[0] * h[0] + h[1] * h[1] + h[2] * h[2] + h[3] * h[3];
            if (a.gain_next) {
#pragma unroll
                for (int v = 0; v < 4; ++v) h[v] *= E::to_f(((const T*)a.gain_next)[n + v]);
            }
            const size_t hi = a.hb_frag ? frag_major_index<T>(m, n, a.N / E::KT) : (size_t)m * a.N + n;
            *(typename E::out4_t*)((T*)a.hb_out + hi) = E::pack4(h[0], h[1], h[2], h[3]);
        }
    } else if constexpr (EPI == EPI_LOGITS) {
        const int n = ptile * 16 + g * 4;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (n + v < a.N) a.logits[(size_t)m * a.N + n + v] = rs * y[0][v];
    } else if constexpr (EPI == EPI_SWIGLU) {
        const int f = (ptile >> 1) * 16 + g * 4;
        if (f < a.F) {
            float o[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float gt = rs * y[0][v], up = rs * y[1][v];
                o[v] = gt / (1.0f + expf(-gt)) * up;
            }
            *(typename E::out4_t*)((T*)a.act_out + frag_major_index<T>(m, f, a.F / E::KT)) = E::pack4(o[0], o[1], o[2], o[3]);
        }
    } else {  // EPI_QKV
        const int tph = a.hd >> 4;  // tiles per head
        const int head = ptile / tph, tih = ptile % tph;
        if (head >= a.Hq + 2 * a.Hkv) return 0.f;  // padding tiles of the last group
        float lo[4], hi[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            lo[v] = rs * y[0][v];
            hi[v] = rs * y[1][v];
            if (a.bias) {
                lo[v] += a.bias[ptile * 16 + g * 4 + v];
                hi[v] += a.bias[(ptile + 1) * 16 + g * 4 + v];
            }
        }
        if (head < a.Hq + a.Hkv) {
            // q / k head: the pair holds features t and t + hd/2, t = (tih/2)*16 + g*4 + v
            const int t = (tih >> 1) * 16 + g * 4, half = a.hd >> 1;
            const float2* cs = a.rope + (size_t)m * half + t;
            float olo[4], ohi[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float2 c = cs[v];
                olo[v] = lo[v] * c.x - hi[v] * c.y;
                ohi[v] = hi[v] * c.x + lo[v] * c.y;
            }
            T* dst;
            if (head < a.Hq)
                dst = (T*)a.q_out + (size_t)m * (a.Hq * a.hd) + (size_t)head * a.hd;
            else
                dst = (T*)a.krow[m] + a.layer_off + (size_t)(head - a.Hq) * a.stride_head;
            *(typename E::out4_t*)(dst + t) = E::pack4(olo[0], olo[1], olo[2], olo[3]);
            *(typename E::out4_t*)(dst + t + half) = E::pack4(ohi[0], ohi[1], ohi[2], ohi[3]);
        } else if (head < a.Hq + 2 * a.Hkv) {
            // v head: natural tile order, no rotation
            T* dst = (T*)a.krow[m] + a.layer_off + a.stride_kv + (size_t)(head - a.Hq - a.Hkv) * a.stride_head;
            const int t = tih * 16 + g * 4;
            *(typename E::out4_t*)(dst + t) = E::pack4(lo[0], lo[1], lo[2], lo[3]);
            *(typename E::out4_t*)(dst + t + 16) = E::pack4(hi[0], hi[1], hi[2], hi[3]);
        }
    }
    return hsq;
}

// Cross-wave reduction through LDS and the fused epilogue, shared by the dense and the 4-bit kernels.
template <typename T, int MT, int NT, int EPI>
static __device__ __forceinline__ void reduce_and_store(const GemmArgs& a, f32x4 (&acc)[MT][NT], float (&ss)[MT], unsigned char* smem,
                                                        int lane, int w, int NW, int grp, int row0, const f32x4& resid_first) {
    constexpr bool NORM = (EPI != EPI_RESID);
    const int r16 = lane & 15, g = lane >> 4;
    // ---- cross-wave reduction through LDS ---------------------------------------------------------
    // LDS holds NC = a.red_copies copies of the workgroup's tiles.  With more waves than copies, the last (up to NC) active
    // waves hand their tiles to the first ones, round by round, until NC waves are left; those write their copies and the
    // epilogue items add them up.  (Many-row tile shapes would otherwise have to run with fewer waves.)
    constexpr bool ROUNDS = (MT * NT > 6);  // only then can the launcher pick fewer copies than waves (48 KiB / (MT*NT) KiB < 8)
    const int NC = ROUNDS ? a.red_copies : NW;
    float* red = (float*)smem;                       // [NC][MT*NT][4][64]
    float* ssr = red + (size_t)NC * MT * NT * 256;   // [NW][MT][16]
    auto put = [&](int slot) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[(((size_t)slot * MT * NT + mt * NT + nt) * 4 + v) * 64 + lane] = acc[mt][nt][v];
    };
    for (int active = NW; ROUNDS && active > NC;) {  // uniform
        const int k = min(NC, active - NC);  // the top k active waves hand over to waves 0 .. k-1
        if (w >= active - k && w < active) put(w - (active - k));
        __syncthreads();
        if (w < k) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[mt][nt][v] += red[(((size_t)w * MT * NT + mt * NT + nt) * 4 + v) * 64 + lane];
        }
        __syncthreads();
        active -= k;
    }
    const int copies = ROUNDS ? (NW < NC ? NW : NC) : NW;
    if (!ROUNDS || w < copies) put(w);
    if (NORM) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float t = wave_xor_add(wave_xor_add(ss[mt], 16), 32);
            if (lane < 16) ssr[(w * MT + mt) * 16 + lane] = t;
        }
    }
    __syncthreads();

    // ---- epilogue: an "item" is one 16x16 tile (RESID, LOGITS) or a pair of tiles (QKV, SWIGLU) ---
    constexpr bool PAIR = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
    constexpr int TPI = PAIR ? 2 : 1;  // tiles per item
    constexpr int ITEMS = MT * NT / TPI;
    static_assert(!PAIR || NT % 2 == 0, "paired epilogues need an even NT");
    for (int item = w; item < ITEMS; item += NW) {
        const int mt = item / (NT / TPI), ntp = item % (NT / TPI);
        const int m = row0 + mt * 16 + r16;
        float y[TPI][4];
#pragma unroll
        for (int t = 0; t < TPI; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float s = 0.f;
                for (int ww = 0; ww < copies; ++ww) s += red[(((size_t)ww * MT * NT + mt * NT + ntp * TPI + t) * 4 + v) * 64 + lane];
                y[t][v] = s;
            }
        float rs = 1.f;
        if (NORM) {
            float s = 0.f;
            for (int ww = 0; ww < NW; ++ww) s += ssr[(ww * MT + mt) * 16 + r16];
            rs = 1.0f / sqrtf(s / (float)a.K + a.eps);
        }
        const int ptile = grp * NT + ntp * TPI;  // first packed tile of the item
        float hsq = epilogue_item<T, EPI>(a, y, rs, m, ptile, g, item == w ? &resid_first : nullptr);
        if constexpr (EPI == EPI_RESID) {
            if (a.ssp_out) {  // uniform over the workgroup; every lane of the wave is here
                hsq = wave_xor_add(wave_xor_add(hsq, 16), 32);
                if (g == 0 && ptile * 16 < a.N && m < a.ssp_stride) a.ssp_out[(size_t)ptile * a.ssp_stride + m] = hsq;
            }
        }
    }
}

// The values the first loads depend on travel as leading scalar kernel arguments: those can be preloaded into SGPRs with
// the wave (compiler option -amdgpu-kernarg-preload-count), whereas the fields of the by-value struct are fetched from
// the kernarg segment by a scalar load the whole prologue would have to wait for.
template <typename T, int MT, int NT, int EPI>
__global__ void __launch_bounds__(512) skinny_gemm_kernel(const void* Wp, const void* X, int nkt_, int ldx_, int M_, int x_frag_, const GemmArgs a) {
    using E = Elem<T>;
    using frag_t = typename E::frag_t;
    constexpr bool NORM = (EPI != EPI_RESID);
    constexpr int PF = (MT + NT <= 3) ? 8 : 4;  // k-steps of loads kept in flight per wave
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, NW = blockDim.x >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int grp = blockIdx.x, mb = blockIdx.y;
    const int row0 = mb * MT * 16;

    // k-tiles are dealt to the waves round-robin (wave w takes w, w + NW, ...): at any moment the workgroup's
    // waves read neighbouring KiBs, so the group's weight block is swept front to back as one stream.
    const int nsteps = (nkt_ - w + NW - 1) / NW;  // >= 1: the host never launches more waves than k-tiles
    const unsigned char* wbase = (const unsigned char*)Wp + ((size_t)grp * nkt_) * (size_t)(NT * 1024) + (size_t)lane * 16;
    // Rows beyond M read row M-1 instead: their results are never stored, and the loop stays free of branches.
    // Fragment-major activations (padded to whole 16-row tiles) are addressed like the weights.
    const T* xrow[MT];
    const size_t xstep = x_frag_ ? (size_t)64 * E::EPF : (size_t)E::KT;  // elements between consecutive k-tiles
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (x_frag_) {
            xrow[mt] = (const T*)X + (((size_t)(mb * MT + mt) * nkt_) * 64 + lane) * E::EPF;
        } else {
            const int m = min(row0 + mt * 16 + r16, M_ - 1);
            xrow[mt] = (const T*)X + (size_t)m * ldx_ + g * E::EPF;
        }
    }

    const f32x4 resid_first = prefetch_resid<T, MT, NT, EPI>(a, w, grp, row0, r16, g);
    f32x4 acc[MT][NT];
    float ss[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        ss[mt] = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Software pipeline of PF k-steps.  Everything inside is unconditional (step indices are clamped to the
    // wave's last k-tile, surplus steps multiply by zero) so that the loads of later steps stay in flight
    // while earlier ones are consumed.
    frag_t bq[PF][NT], aq[PF][MT];
    auto issue = [&](int s, int step) {
        const int kt = w + min(step, nsteps - 1) * NW;
        const unsigned char* wp = wbase + (size_t)kt * (NT * 1024);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bq[s][nt] = load_w<T>(wp + nt * 1024);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) aq[s][mt] = *(const frag_t*)(xrow[mt] + (size_t)kt * xstep);
    };
    auto consume = [&](int s, int step) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            frag_t av = aq[s][mt];
            if (step >= nsteps) av = E::zero();
            if (NORM) ss[mt] += E::sumsq(av);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = E::mma(bq[s][nt], av, acc[mt][nt]);
        }
    };
#pragma unroll
    for (int s = 0; s < PF; ++s) issue(s, s);
    const int nrounds = (nsteps + PF - 1) / PF;
    for (int rd = 0; rd + 1 < nrounds; ++rd) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            consume(s, rd * PF + s);
            issue(s, (rd + 1) * PF + s);
            __builtin_amdgcn_sched_barrier(0);  // keep the refill right behind its consumer: PF-1 stages stay in flight
        }
    }
#pragma unroll
    for (int s = 0; s < PF; ++s) consume(s, (nrounds - 1) * PF + s);

    reduce_and_store<T, MT, NT, EPI>(a, acc, ss, smem, lane, w, NW, grp, row0, resid_first);
}

// copies of the workgroup's tiles the cross-wave reduction keeps in LDS: as many as there are waves, within about 48 KiB
static int reduction_copies(int nw, int mt, int nt) {
    const int fit = 48 / (mt * nt);  // 1 KiB per tile and copy
    return nw < fit ? nw : (fit < 1 ? 1 : fit);
}

template <typename T, int MT, int NT, int EPI>
static hipError_t launch_one(int NW, int n_groups, const GemmArgs& a0, hipStream_t s) {
    GemmArgs a = a0;
    const int mblocks = (a.M + MT * 16 - 1) / (MT * 16);
    if (NW > 8) NW = 8;
    a.red_copies = reduction_copies(NW, MT, NT);
    const size_t lds = (size_t)a.red_copies * MT * NT * 1024 + (size_t)NW * MT * 16 * sizeof(float);
    hipLaunchKernelGGL((skinny_gemm_kernel<T, MT, NT, EPI>), dim3(n_groups, mblocks), dim3(NW * 64), lds, s, a.Wp, a.X, a.nkt, a.ldx, a.M, a.x_frag, a);
    return hipGetLastError();
}

template <typename T, int EPI>
static hipError_t launch_mt_nt(int MT, int NT, int NW, int n_groups, const GemmArgs& a, hipStream_t s) {
    constexpr bool PAIR = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
#define FS_CASE(mt, nt) \
    if (MT == mt && NT == nt) return launch_one<T, mt, nt, EPI>(NW, n_groups, a, s);
    if constexpr (!PAIR) {
        FS_CASE(1, 1) FS_CASE(2, 1) FS_CASE(4, 1)
    }
    FS_CASE(1, 2) FS_CASE(2, 2) FS_CASE(4, 2) FS_CASE(1, 4) FS_CASE(2, 4) FS_CASE(4, 4)
#undef FS_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(int dtype, int epi, int NT, int NW, int n_groups, const GemmArgs& a, hipStream_t s) {
    // 33 to 64 rows per block: 4 row tiles and at most 4 waves (several smaller workgroups per compute unit overlap each
    // other's start-up and epilogue; 8 waves: QKV 42 -> 44 us, gate/up 50 -> 53 us at 64 rows).  Two 32-row blocks per
    // group instead were slower as well (gate/up 54 -> 61 us).
    const int MT = a.M <= 16 ? 1 : (a.M <= 32 ? 2 : 4);
    if (MT == 4 && NW > 4) NW = 4;
    if (MT * NT >= 8 && NW > 4) NW = 4;  // 8 tiles per workgroup: 4 waves keep a copy each in LDS without reduction rounds
#define FS_EPI(e)                                                                      \
    if (epi == e) {                                                                    \
        if (dtype == 0) return launch_mt_nt<float, e>(MT, NT, NW, n_groups, a, s);     \
        return launch_mt_nt<bf16_t, e>(MT, NT, NW, n_groups, a, s);                    \
    }
    FS_EPI(EPI_QKV) FS_EPI(EPI_RESID) FS_EPI(EPI_SWIGLU) FS_EPI(EPI_LOGITS)
#undef FS_EPI
    return hipErrorInvalidValue;
}

// ---- many-row segments (chunked prefill, stacked requests): projection as a matrix product -------------------
// With more than a row tile or two the projections stop being a pure weight stream: the few-row kernel re-reads the
// activations once per workgroup and ends up bound by the path from L2 into the compute units.  This kernel shares the
// activations between the waves instead.  Workgroup = 4 waves; block = 128 rows x 256 features (from 384 rows), 128 rows
// x 128 features (65 .. 383 rows) or 64 rows x 128 features (up to 64 rows); wave w owns a quarter of the features for
// all rows of the block (8 x 4, 8 x 2 or 4 x 2 accumulator tiles).
//   * Weights are private to a wave, so they skip LDS: each wave streams its tiles per k-tile straight from the re-tiled
//     copy into registers, a ring of PFW k-tiles deep (the same coalesced 1 KiB fragment loads as the few-row kernel).
//   * Activations are shared by the four waves: the block's fragments per k-tile (fragment-major in memory, so a plain
//     copy of 8 or 4 KiB) go through a double-buffered LDS stage, one barrier per k-tile.
//   Per k-tile and wave of the largest block: 8 LDS fragment reads + 4 global fragment loads feed 32 MFMAs — half of the
//   LDS and of the vector-memory bandwidth at full MFMA rate.  What binds it there is the L2: every k-tile of a block
//   asks it for 24 KiB (16 KiB of weights, 8 KiB of activations) per 2.1 MFLOP.
//   * RMSNorm: the 256-feature blocks take the row scale from partial sums of squares left by the producer of the
//     activations (GemmArgs::ssp_in), so their loop contains no per-element arithmetic; the 128-feature blocks have
//     registers to spare and add the squares up while they stage the activations.
//   * Workgroups that share weights (the row blocks of one feature block) get consecutive slots on one XCD, so the
//     weights are fetched from HBM once and hit in that XCD's L2 afterwards.
//   * Projections too narrow to fill the chip (d_model outputs, a few row blocks) split K over `k_splits` workgroups;
//     each writes its raw accumulator tiles (MFMA lane order, so 16 bytes per lane, contiguous per wave) to a scratch
//     array and wide_fixup_kernel adds them up and runs the residual epilogue.
//   * Which projections come here at which row count is the caller's choice (with one 64-row block: gate/up, the down
//     projection and the LM head; QKV and the attention output have too few 128-feature blocks to fill the chip and a
//     wave has only 8 MFMAs per k-tile to hide a barrier and an LDS round trip behind: 64 rows, QKV 31 -> 38 us).
template <int EPI, bool PARTIAL, int BMT, int WNT, int WAVES, bool STREAMW>
__global__ void __launch_bounds__(WAVES * 64, BMT == 8 ? 2 : 3) wide_gemm_kernel(const GemmArgs a, int layout_nt, int n_tiles, int n_cols, int m_blocks, int k_splits,
                                                           float* part) {
    using T = bf16_t;
    using E = Elem<T>;
    using frag_t = E::frag_t;
    constexpr bool NORM = (EPI != EPI_RESID);
    constexpr bool PAIR = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
    constexpr int TPI = PAIR ? 2 : 1;
    // Weight fragments are fetched PFW k-tiles ahead and activation pieces XD k-tiles ahead.  Loads retire in order, so
    // waiting for an activation piece also waits for every weight fetch issued before it: XD, not PFW, is the latency
    // budget of a weight fetch, and PFW > XD + 1 only adds loads in flight.  (With XD = 2 a k-tile took 0.7 us whenever
    // the weights came from HBM — one row block — i.e. about a third of the memory latency.)
    constexpr int PFW = (BMT == 8 && WNT == 4) ? 4 : 8;
    constexpr int XD = (BMT == 8 && WNT == 4) ? 4 : 8;
    constexpr int XL = BMT / WAVES;        // 16-byte pieces of the activation stage per thread
    static_assert(BMT % WAVES == 0 && BMT % 4 == 0, "row tiles must split over the waves and over groups of 4");
    __shared__ __align__(16) unsigned char xs[2][BMT * 1024];
    __shared__ float rs_s[BMT * 16];

    // XCD-aware placement: slot s of XCD x (workgroup id = s * 8 + x) takes feature block (s / m_blocks) * 8 + x, row block s % m_blocks
    // (with split K the slot also runs over the K slices of a block, innermost)
    const int id = blockIdx.x, xcd = id & 7, slot = id >> 3;
    const int per_col = m_blocks * k_splits;
    const int col = (slot / per_col) * 8 + xcd, mb = (slot % per_col) / k_splits, ks = slot % k_splits;
    if (col >= n_cols) return;
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int kt_lo = (int)((long long)a.nkt * ks / k_splits), nkt = (int)((long long)a.nkt * (ks + 1) / k_splits) - kt_lo;  // >= 1 (host)
    const int mt0 = mb * BMT, m_tiles = (a.M + 15) >> 4;

    // RMSNorm scale of the rows.  The 256-feature blocks have no registers to spare and take it from the partial sums of
    // squares their producer left (one per workgroup column of that producer: a few dozen independent loads per row); the
    // 128-feature blocks add the squares up themselves while they stage the activations (see store_x), so that they can
    // also follow a producer that leaves no such sums.
    constexpr bool SELF_NORM = NORM && WNT == 2;
    if (NORM && !SELF_NORM && t < BMT * 16) {
        const int m = min(mt0 * 16 + t, a.M - 1);
        float s0 = 0.f, s1 = 0.f;
        int j = 0;
#pragma unroll 4
        for (; j + 1 < a.ssp_n; j += 2) {
            s0 += a.ssp_in[(size_t)j * a.ssp_stride + m];
            s1 += a.ssp_in[(size_t)(j + 1) * a.ssp_stride + m];
        }
        if (j < a.ssp_n) s0 += a.ssp_in[(size_t)j * a.ssp_stride + m];
        rs_s[t] = 1.0f / sqrtf((s0 + s1) / (float)a.K + a.eps);
    }

    // this wave's weight tiles; tiles beyond the matrix re-read the last one (their results are never stored).
    // Addresses are a uniform base plus a 32-bit byte offset per lane (one matrix is far below 4 GiB), advanced by one
    // k-tile per fetch until the last k-tile of the slice is reached.
    const int pt0 = (col * WAVES + w) * WNT;
    const unsigned char* wbase = (const unsigned char*)a.Wp;
    const unsigned char* xbase = (const unsigned char*)a.X;
    unsigned woff[WNT], xoff[XL];
#pragma unroll
    for (int nt = 0; nt < WNT; ++nt) {
        const int pc = min(pt0 + nt, n_tiles - 1);
        woff[nt] = (unsigned)((((size_t)(pc / layout_nt) * a.nkt + kt_lo) * layout_nt + pc % layout_nt) * 1024 + (size_t)lane * 16);
    }
    const unsigned wstep = (unsigned)layout_nt * 1024;
    // this thread's 16-byte pieces of the activation stage: fragments w, w + WAVES, ... of the block's BMT
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        const int mt = min(mt0 + w + WAVES * i, m_tiles - 1);
        xoff[i] = (unsigned)((((size_t)mt * a.nkt + kt_lo) * 64 + lane) * 16);
    }
    const unsigned xstep = 1024;
    int wk = 0, xk = 0;  // k-tiles already fetched (weights / activations)

    f32x4 acc[BMT][WNT];
#pragma unroll
    for (int mt = 0; mt < BMT; ++mt)
#pragma unroll
        for (int nt = 0; nt < WNT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    frag_t wq[PFW][WNT], xr[XD][XL];
    auto fetch_w = [&](int j, int) {
#pragma unroll
        for (int nt = 0; nt < WNT; ++nt)  // weights that other row blocks read again stay in L2; with one row block they stream past it
            wq[j][nt] = STREAMW ? load_w<T>(wbase + woff[nt]) : *(const frag_t*)(wbase + woff[nt]);
        const unsigned adv = (++wk < nkt) ? wstep : 0u;  // past the slice's end the last k-tile is re-read (and never used)
#pragma unroll
        for (int nt = 0; nt < WNT; ++nt) woff[nt] += adv;
    };
    auto load_x = [&](int j, int) {
#pragma unroll
        for (int i = 0; i < XL; ++i) xr[j][i] = *(const frag_t*)(xbase + xoff[i]);
        const unsigned adv = (++xk < nkt) ? xstep : 0u;
#pragma unroll
        for (int i = 0; i < XL; ++i) xoff[i] += adv;
    };
    // Self-computed RMSNorm scale: every 16-byte piece of the activations passes through exactly one thread on its way to
    // LDS (lane (r16, g) carries 8 consecutive k of row r16), which adds its squares up; pieces fetched past the end of the
    // K range (the ring runs ahead of the loop) are not counted.
    float ssq[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) ssq[i] = 0.f;
    int xstored = 0;  // k-tiles handed to LDS so far
    auto store_x = [&](int j, int buf) {
#pragma unroll
        for (int i = 0; i < XL; ++i) *(frag_t*)(xs[buf] + (size_t)(w + WAVES * i) * 1024 + (size_t)lane * 16) = xr[j][i];
        if constexpr (SELF_NORM) {
            const bool counts = xstored < nkt;  // uniform
#pragma unroll
            for (int i = 0; i < XL; ++i) {
                const bf16x2x4 pr = __builtin_bit_cast(bf16x2x4, xr[j][i]);
                float sq = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) sq = __builtin_amdgcn_fdot2_f32_bf16(pr.v[e], pr.v[e], sq, false);
                ssq[i] += counts ? sq : 0.f;
            }
            ++xstored;
        }
    };
    // Pipeline, k-tile kt: weights in wq[kt % PFW], activations in LDS buffer kt & 1; xr[n % XD] carries k-tile n from
    // memory to LDS (n = kt + 1 .. kt + XD are in registers or in flight when the iteration starts).  One barrier per
    // k-tile: it publishes buffer kt & 1 (filled during k-tile kt - 1) and tells that nobody still reads the other buffer,
    // which the refill at the end of the iteration overwrites.
#pragma unroll
    for (int j = 0; j < PFW; ++j) fetch_w(j, j);
#pragma unroll
    for (int j = 0; j < XD; ++j) load_x(j, j);
    store_x(0, 0);
    load_x(0, XD);
    constexpr int U = (PFW % XD == 0) ? PFW : ((XD % PFW == 0) ? XD : PFW * XD);  // kt % PFW, kt % XD and kt & 1 compile-time
    static_assert(U % 2 == 0 && U % PFW == 0 && U % XD == 0, "unroll factor must cover both rings and the buffer parity");
    auto ktile = [&](int ju) {  // k-tile kt0 + ju of a group of U: ring slots and buffer parity are compile-time
        const int j = ju % PFW;
        __syncthreads();
        const unsigned char* xb = xs[ju & 1] + (size_t)lane * 16;
#pragma unroll
        for (int h = 0; h < BMT / 4; ++h) {
            frag_t bf[4];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) bf[mt] = *(const frag_t*)(xb + (size_t)(h * 4 + mt) * 1024);
#pragma unroll
            for (int nt = 0; nt < WNT; ++nt)
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) acc[h * 4 + mt][nt] = E::mma(wq[j][nt], bf[mt], acc[h * 4 + mt][nt]);
        }
        store_x((ju + 1) % XD, (ju + 1) & 1);
        load_x((ju + 1) % XD, 0);
        fetch_w(j, 0);
    };
    // Whole groups of U k-tiles run as straight-line code: a k-tile that could be skipped inside the loop would make the
    // compiler assume that the fetch it is about to wait for might be the newest one in flight, and wait for all of them
    // (the weight ring would then drain once per group).  The last, partial group takes the guarded form.
    int kt0 = 0;
    for (; kt0 + U <= nkt; kt0 += U) {
#pragma unroll
        for (int ju = 0; ju < U; ++ju) ktile(ju);
    }
#pragma unroll
    for (int ju = 0; ju < U; ++ju)
        if (kt0 + ju < nkt) ktile(ju);  // uniform over the workgroup

    if constexpr (PARTIAL) {
        // raw tiles: part[ks][m tile][n tile][lane] (f32x4); tiles beyond the matrix are dropped
        const int nt_all = n_cols * WAVES * WNT;
#pragma unroll
        for (int mt = 0; mt < BMT; ++mt) {
            if (mt0 + mt >= m_tiles) break;
#pragma unroll
            for (int nt = 0; nt < WNT; ++nt)
                ((f32x4*)part)[(((size_t)ks * m_tiles + mt0 + mt) * nt_all + pt0 + nt) * 64 + lane] = acc[mt][nt];
        }
        return;
    }
    if constexpr (SELF_NORM) {
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const float tot = wave_xor_add(wave_xor_add(ssq[i], 16), 32);
            if (g == 0) rs_s[(w + WAVES * i) * 16 + r16] = 1.0f / sqrtf(tot / (float)a.K + a.eps);
        }
        __syncthreads();
    }
    // ---- epilogue straight from the accumulators -------------------------------------------------------------
    // (residual projections also leave one partial sum of squares per row and workgroup: the waves' shares meet in LDS,
    //  where the activation stage is free once every wave has left the loop)
    float* hs = (float*)xs[0];  // [WAVES][BMT * 16]
    if constexpr (EPI == EPI_RESID) {
        if (a.ssp_out) __syncthreads();
    }
#pragma unroll
    for (int mt = 0; mt < BMT; ++mt) {
        const int m = (mt0 + mt) * 16 + r16;
        const float rs = NORM ? rs_s[mt * 16 + r16] : 1.f;
        float hsq = 0.f;
#pragma unroll
        for (int ntp = 0; ntp < WNT / TPI; ++ntp) {
            float y[TPI][4];
#pragma unroll
            for (int tt = 0; tt < TPI; ++tt)
#pragma unroll
                for (int v = 0; v < 4; ++v) y[tt][v] = acc[mt][ntp * TPI + tt][v];
            hsq += epilogue_item<T, EPI>(a, y, rs, m, pt0 + ntp * TPI, g);
        }
        if constexpr (EPI == EPI_RESID) {
            if (a.ssp_out) {
                hsq = wave_xor_add(wave_xor_add(hsq, 16), 32);
                if (g == 0) hs[w * (BMT * 16) + mt * 16 + r16] = hsq;
            }
        }
    }
    if constexpr (EPI == EPI_RESID) {
        if (a.ssp_out) {
            __syncthreads();
            if (t < BMT * 16) {
                float sum = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) sum += hs[ww * (BMT * 16) + t];
                const int m = mt0 * 16 + t;
                if (m < a.ssp_stride) a.ssp_out[(size_t)col * a.ssp_stride + m] = sum;
            }
        }
    }
}

// Sum of the K slices' raw tiles + residual epilogue.  One wave per (row tile, group of wnt feature tiles = what one
// wave of the projection kernel owns): the same lane layout as the accumulators, the same partial sums of squares as the
// direct epilogue.
__global__ void __launch_bounds__(256) wide_fixup_kernel(const GemmArgs a, int nt_all, int wnt, int k_splits, const float* part) {
    const int lane = threadIdx.x & 63, r16 = lane & 15, g = lane >> 4;
    const int m_tiles = (a.M + 15) >> 4, groups = nt_all / wnt;
    __shared__ float hs[4][16];
    const int wv = threadIdx.x >> 6;
    const int unit = blockIdx.x * 4 + wv;  // groups is a multiple of 4: the workgroup's 4 units are the 4 waves' shares of one block
    if (unit >= m_tiles * groups) return;  // whole workgroup
    const int mt = unit / groups, grp = unit % groups;
    const int m = mt * 16 + r16;
    float hsq = 0.f;
    for (int nt = 0; nt < wnt; ++nt) {
        const int ptile = grp * wnt + nt;
        f32x4 sum{0.f, 0.f, 0.f, 0.f};
        for (int ks = 0; ks < k_splits; ++ks) sum += ((const f32x4*)part)[(((size_t)ks * m_tiles + mt) * nt_all + ptile) * 64 + lane];
        const float y[1][4] = {{sum[0], sum[1], sum[2], sum[3]}};
        hsq += epilogue_item<bf16_t, EPI_RESID>(a, y, 1.f, m, ptile, g);
    }
    if (a.ssp_out) {
        hsq = wave_xor_add(wave_xor_add(hsq, 16), 32);
        if (g == 0) hs[wv][r16] = hsq;
        __syncthreads();
        if (threadIdx.x < 16 && mt * 16 + (int)threadIdx.x < a.ssp_stride)
            a.ssp_out[(size_t)(grp >> 2) * a.ssp_stride + mt * 16 + threadIdx.x] = hs[0][threadIdx.x] + hs[1][threadIdx.x] + hs[2][threadIdx.x] + hs[3][threadIdx.x];
    }
}

// ---- many-row segments: 256-row blocks, both operands through LDS ------------------------------------------------------
// The 128-row kernel above moves 24 KiB from L2 per k-tile and block for 2.1 MFLOP and is bound by the path from L2 into a
// compute unit (about 50 GB/s per unit, whatever the kernel does).  This kernel gives a compute unit one block of 256 rows x
// 16 * BNT features at a time and brings both operands in through LDS, so that every byte that arrives serves the whole block:
// 256 x 256 features take 32 KiB per k-tile for 4.2 MFLOP.  WM x WN waves, each with MT x NT accumulator tiles (WM * MT = 16
// row tiles, WN * NT = BNT feature tiles); the shape in use is 2 x 4 waves of 8 x 4 tiles (two waves per SIMD, 128 accumulator
// registers each).
//   * Both operands are fragment-major in memory (one fragment = one contiguous KiB in MFMA operand order), so a fragment goes
//     from global memory straight into LDS with one 16-byte-per-lane direct-to-LDS load per wave: no staging registers.
//     A stage is the block's 16 activation fragments and BNT weight fragments of one k-tile; the waves share its loads.
//   * STAGES stage buffers; the loads of a stage are issued STAGES - 1 k-tiles before its MFMAs, into the buffer whose
//     fragments were read two k-tiles ago.
//   * Fragments travel LDS -> registers one k-tile ahead, without a second register set: an activation fragment is replaced
//     by the next k-tile's as soon as the MFMAs of its row tile are issued, a weight fragment during the last row tile.
//   * One barrier per k-tile.  It is the bare s_barrier with explicit wait counts: the workgroup fence of __syncthreads would
//     wait for every direct-to-LDS load in flight, i.e. drain the prefetch, and for the fragment reads of the k-tile about to
//     start.  Before the barrier of k-tile kt a wave waits for its own loads of stage kt + 1 (those of stage kt + 2 stay in
//     flight) and for all its LDS reads but the newest ones (reads return in order: everything read two k-tiles ago is then
//     done).  Behind the barrier stage kt + 1 is complete for every wave and the buffer of stage kt - 1 is free.
//   * Epilogues, RMSNorm hand-over (partial sums of squares from the producer) and XCD-aware placement are those of the
//     128-row kernel; K slices (PARTIAL) write the same raw tiles for the same fix-up kernel.

template <int EPI, bool PARTIAL, int WM, int WN, int MT, int NT, int STAGES>
__global__ void __launch_bounds__(WM * WN * 64) block_gemm_kernel(const GemmArgs a, int layout_nt, int n_tiles, int n_cols, int m_blocks, int k_splits,
                                                                  float* part) {
    using T = bf16_t;
    using E = Elem<T>;
    using frag_t = E::frag_t;
    constexpr bool NORM = (EPI != EPI_RESID);
    constexpr bool PAIR = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
    constexpr int TPI = PAIR ? 2 : 1;
    constexpr int NWAVES = WM * WN;
    constexpr int BMT = WM * MT, BNT = WN * NT, FR = BMT + BNT;  // row tiles, feature tiles, fragments (KiB) per stage
    constexpr int DIST = STAGES - 1;                             // k-tiles between a stage's loads and its MFMAs
    constexpr int LPW = (FR + NWAVES - 1) / NWAVES;              // direct-to-LDS loads per wave and stage
    constexpr int RPT = MT + NT;                                 // LDS fragment reads per wave and k-tile
    static_assert(BMT == 16, "blocks are 256 rows");
    static_assert(!PAIR || NT % 2 == 0, "paired epilogues need both tiles of a pair in one wave");
    static_assert(STAGES == 3 || STAGES == 4, "3 or 4 stage buffers");
    static_assert((STAGES * FR + 1) * 1024 <= 160 * 1024, "stage buffers must fit the 160 KiB of LDS");
    static_assert((DIST - 1) * LPW < 64, "vmcnt is a 6-bit counter");
    // one array per stage: distinct objects, so that the compiler's own wait-count tracking of the direct-to-LDS loads never
    // ties a read of one stage to a load into another
    __shared__ __align__(1024) unsigned char sb0[FR * 1024];
    __shared__ __align__(1024) unsigned char sb1[FR * 1024];
    __shared__ __align__(1024) unsigned char sb2[FR * 1024];
    __shared__ __align__(1024) unsigned char sb3[STAGES == 4 ? FR * 1024 : 16];
    __shared__ float rs_s[BMT * 16];
    auto stage_buf = [&](int j) -> unsigned char* { return j == 0 ? sb0 : (j == 1 ? sb1 : (j == 2 ? sb2 : sb3)); };

    const int id = blockIdx.x, xcd = id & 7, slot = id >> 3;
    const int per_col = m_blocks * k_splits;
    const int col = (slot / per_col) * 8 + xcd, mb = (slot % per_col) / k_splits, ks = slot % k_splits;
    if (col >= n_cols) return;
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w / WN, wn = w % WN;  // wave-uniform: scalar address arithmetic below
    const int r16 = lane & 15, g = lane >> 4;
    const int kt_lo = (int)((long long)a.nkt * ks / k_splits), nkt = (int)((long long)a.nkt * (ks + 1) / k_splits) - kt_lo;  // >= 1 (host)
    const int mt0 = mb * BMT, m_tiles = (a.M + 15) >> 4;

    if (NORM) {  // RMSNorm scale of the block's rows from the producer's partial sums of squares
        for (int r = t; r < BMT * 16; r += NWAVES * 64) {
            const int m = min(mt0 * 16 + r, a.M - 1);
            float s0 = 0.f, s1 = 0.f;
            int j = 0;
#pragma unroll 4
            for (; j + 1 < a.ssp_n; j += 2) {
                s0 += a.ssp_in[(size_t)j * a.ssp_stride + m];
                s1 += a.ssp_in[(size_t)(j + 1) * a.ssp_stride + m];
            }
            if (j < a.ssp_n) s0 += a.ssp_in[(size_t)j * a.ssp_stride + m];
            rs_s[r] = 1.0f / sqrtf((s0 + s1) / (float)a.K + a.eps);
        }
    }

    // this wave's share of a stage: fragments w * LPW .. + LPW - 1 (activation row tiles first, then weight tiles; a share that
    // runs past the stage's end loads its last fragment again); tiles beyond the matrix re-read the last one (their results
    // are never stored).  Wave-uniform 64-bit base + this lane's 16 bytes.
    const unsigned char* src[LPW];
    unsigned step[LPW], dst_off[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int f = min(w * LPW + i, FR - 1);
        const int mt = min(mt0 + f, m_tiles - 1);
        const int pc = min(col * BNT + max(f - BMT, 0), n_tiles - 1);
        const size_t xo = ((size_t)mt * a.nkt + kt_lo) * 1024;
        const size_t wo = (((size_t)(pc / layout_nt) * a.nkt + kt_lo) * layout_nt + pc % layout_nt) * 1024;
        src[i] = (f < BMT) ? (const unsigned char*)a.X + xo : (const unsigned char*)a.Wp + wo;
        step[i] = (f < BMT) ? 1024u : (unsigned)layout_nt * 1024u;
        dst_off[i] = (unsigned)f * 1024u;
    }
    const unsigned lane_off = (unsigned)lane * 16u;
    int issued = 0;
    auto issue = [&](int j) {  // next k-tile of this wave's fragments -> stage buffer j (past the slice's end: the last k-tile again)
        unsigned char* dst = stage_buf(j);
#pragma unroll
        for (int i = 0; i < LPW; ++i) __builtin_amdgcn_global_load_lds(FS_GLB_PTR(src[i] + lane_off), FS_LDS_PTR(dst + dst_off[i]), 16, 0, 0);
        const bool more = ++issued < nkt;
#pragma unroll
        for (int i = 0; i < LPW; ++i) src[i] += more ? step[i] : 0u;
    };
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    frag_t xf[MT], wf[NT];
    auto frag_at = [&](int j, int f) { return *(const frag_t*)(stage_buf(j) + (size_t)f * 1024 + lane_off); };

#pragma unroll
    for (int j = 0; j < DIST; ++j) issue(j);
    FS_WAIT_VM_LGKM((DIST - 1) * LPW, 0);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wf[nt] = frag_at(0, BMT + wn * NT + nt);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xf[mt] = frag_at(0, wm * MT + mt);
    auto ktile = [&](int ju) {  // k-tile kt0 + ju of a group of STAGES: the buffers are compile-time
        const int jn = (ju + 1) % STAGES;
        FS_WAIT_VM_LGKM((DIST - 2) * LPW, RPT < 15 ? RPT : 15);
        __builtin_amdgcn_s_barrier();
        issue((ju + DIST) % STAGES);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                acc[mt][nt] = E::mma(wf[nt], xf[mt], acc[mt][nt]);
                if (mt == MT - 1) wf[nt] = frag_at(jn, BMT + wn * NT + nt);
            }
            xf[mt] = frag_at(jn, wm * MT + mt);
        }
    };
    int kt0 = 0;
    for (; kt0 + STAGES <= nkt; kt0 += STAGES) {
#pragma unroll
        for (int ju = 0; ju < STAGES; ++ju) ktile(ju);
    }
#pragma unroll
    for (int ju = 0; ju < STAGES; ++ju)
        if (kt0 + ju < nkt) ktile(ju);  // uniform over the workgroup
    // every direct-to-LDS load has landed and every wave has left the loop before LDS is reused below
    FS_WAIT_VM_LGKM(0, 0);
    __builtin_amdgcn_s_barrier();

    if constexpr (PARTIAL) {
        const int nt_all = n_cols * BNT;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int mtile = mt0 + wm * MT + mt;
            if (mtile >= m_tiles) break;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                ((f32x4*)part)[(((size_t)ks * m_tiles + mtile) * nt_all + col * BNT + wn * NT + nt) * 64 + lane] = acc[mt][nt];
        }
        return;
    }
    const int pt0 = col * BNT + wn * NT;
    float* hs = (float*)sb0;  // [WN feature waves][256 rows]
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int lr = (wm * MT + mt) * 16 + r16;  // row within the block
        const int m = mt0 * 16 + lr;
        const float rs = NORM ? rs_s[lr] : 1.f;
        float hsq = 0.f;
#pragma unroll
        for (int ntp = 0; ntp < NT / TPI; ++ntp) {
            float y[TPI][4];
#pragma unroll
            for (int tt = 0; tt < TPI; ++tt)
#pragma unroll
                for (int v = 0; v < 4; ++v) y[tt][v] = acc[mt][ntp * TPI + tt][v];
            hsq += epilogue_item<T, EPI>(a, y, rs, m, pt0 + ntp * TPI, g);
        }
        if constexpr (EPI == EPI_RESID) {
            if (a.ssp_out) {
                hsq = wave_xor_add(wave_xor_add(hsq, 16), 32);
                if (g == 0) hs[wn * (BMT * 16) + lr] = hsq;
            }
        }
    }
    if constexpr (EPI == EPI_RESID) {
        if (a.ssp_out) {
            __syncthreads();
            for (int r = t; r < BMT * 16; r += NWAVES * 64) {
                float sum = 0.f;
#pragma unroll
                for (int x = 0; x < WN; ++x) sum += hs[x * (BMT * 16) + r];
                const int m = mt0 * 16 + r;
                if (m < a.ssp_stride) a.ssp_out[(size_t)col * a.ssp_stride + m] = sum;
            }
        }
    }
}

// Block geometry by projection kind and row count (see the kernel's header comment).
struct WideShape {
    int bmt, wnt, waves;
};
// Up to a few row blocks there are too few 256-feature blocks to fill the chip: 128-feature blocks (2 tiles per wave) then.
static int wide_narrow_rows() {
    static const int v = [] { const char* e = getenv("FLOWSPEC_WIDE_NARROW_ROWS"); return e ? atoi(e) : 384; }();
    return v;
}
static int env_int(const char* name, int dflt) { const char* e = getenv(name); return e ? atoi(e) : dflt; }
static WideShape wide_shape(int, int M) {
    if (M <= 64) return WideShape{4, 2, 4};  // one 64-row block (gate/up and LM head of segments of 33 to 64 rows)
    return M < wide_narrow_rows() ? WideShape{8, 2, 4} : WideShape{8, 4, 4};
}

struct WideGrid {
    int n_cols, m_blocks, k_splits;
};
// K slices for the d_model-wide residual projections: until there is about one workgroup per compute unit (measured: at 512
// rows 4 slices -> 256 workgroups take 36 / 60 us for the attention-output / down projection, 8 slices 52 / 80 us; every
// further slice adds a full set of partial tiles to write and to sum), at least 8 k-tiles per slice, and no more than the
// scratch array holds.
static WideGrid wide_grid(const WideShape& sh, int epi, int M, int n_tiles, int nkt, size_t part_bytes) {
    WideGrid g;
    const int col_tiles = sh.waves * sh.wnt;
    g.n_cols = (n_tiles + col_tiles - 1) / col_tiles;
    g.m_blocks = (M + sh.bmt * 16 - 1) / (sh.bmt * 16);
    g.k_splits = 1;
    if (epi == EPI_RESID) {
        const size_t per_split = (size_t)((M + 15) / 16) * g.n_cols * col_tiles * 1024;
        static const int target = env_int("FLOWSPEC_WIDE_SPLIT_WGS", 256);
        while (g.k_splits < 8 && g.n_cols * g.m_blocks * g.k_splits * 2 <= target && nkt / (g.k_splits * 2) >= 8 &&
               per_split * g.k_splits * 2 <= part_bytes)
            g.k_splits *= 2;
    }
    return g;
}

int wide_ssp_parts(int M, int n_tiles) {  // one per workgroup column of the residual projection
    const WideShape sh = wide_shape(EPI_RESID, M);
    const int col_tiles = sh.waves * sh.wnt;
    return (n_tiles + col_tiles - 1) / col_tiles;
}

size_t wide_partial_bytes(int max_rows, int n_tiles) {
    // slices * row tiles * feature tiles KiB: at most 8 slices of the whole result, and, with slices * blocks bounded by the
    // split rule, at most 512 blocks' worth of tiles (largest block shape)
    const size_t whole = (size_t)8 * ((max_rows + 15) / 16) * (size_t)(n_tiles + 15) * 1024;
    const size_t cap = (size_t)512 * 8 * 4 * 4 * 1024;
    return whole < cap ? whole : cap;
}

template <int EPI, int BMT, int WNT, int WAVES>
static hipError_t launch_wide_shape(int layout_nt, int n_tiles, const GemmArgs& a, float* part, size_t part_bytes, hipStream_t s) {
    const WideShape sh{BMT, WNT, WAVES};
    const WideGrid g = wide_grid(sh, EPI, a.M, n_tiles, a.nkt, part ? part_bytes : 0);
    const int grid = (g.n_cols + 7) / 8 * 8 * g.m_blocks * g.k_splits;
    // one row block (only the narrow shape has that few rows): every weight byte is read once
    const bool stream = (WNT == 2) && g.m_blocks == 1;
    if constexpr (EPI == EPI_RESID) {
        if (g.k_splits > 1) {
            if (stream)
                hipLaunchKernelGGL((wide_gemm_kernel<EPI, true, BMT, WNT, WAVES, WNT == 2>), dim3(grid), dim3(WAVES * 64), 0, s, a, layout_nt, n_tiles,
                                   g.n_cols, g.m_blocks, g.k_splits, part);
            else
                hipLaunchKernelGGL((wide_gemm_kernel<EPI, true, BMT, WNT, WAVES, false>), dim3(grid), dim3(WAVES * 64), 0, s, a, layout_nt, n_tiles,
                                   g.n_cols, g.m_blocks, g.k_splits, part);
            const int units = ((a.M + 15) / 16) * g.n_cols * WAVES;
            hipLaunchKernelGGL(wide_fixup_kernel, dim3((units + 3) / 4), dim3(256), 0, s, a, g.n_cols * WAVES * WNT, WNT, g.k_splits, part);
            return hipGetLastError();
        }
    }
    if (stream)
        hipLaunchKernelGGL((wide_gemm_kernel<EPI, false, BMT, WNT, WAVES, WNT == 2>), dim3(grid), dim3(WAVES * 64), 0, s, a, layout_nt, n_tiles, g.n_cols,
                           g.m_blocks, 1, nullptr);
    else
        hipLaunchKernelGGL((wide_gemm_kernel<EPI, false, BMT, WNT, WAVES, false>), dim3(grid), dim3(WAVES * 64), 0, s, a, layout_nt, n_tiles, g.n_cols,
                           g.m_blocks, 1, nullptr);
    return hipGetLastError();
}

// 256-row blocks of 256 or 192 features, both operands through LDS (block_gemm_kernel): 2 x 4 waves of 8 x 4 accumulator tiles, or
// 4 x 2 waves of 4 x 6.
template <int EPI, int WM, int WN, int MT, int NT>
static hipError_t launch_block(int layout_nt, int n_tiles, const GemmArgs& a, hipStream_t s) {
    constexpr int BNT = WN * NT;
    const int n_cols = (n_tiles + BNT - 1) / BNT, m_blocks = (a.M + 255) / 256;
    const int grid = (n_cols + 7) / 8 * 8 * m_blocks;
    hipLaunchKernelGGL((block_gemm_kernel<EPI, false, WM, WN, MT, NT, 4>), dim3(grid), dim3(WM * WN * 64), 0, s, a, layout_nt, n_tiles, n_cols, m_blocks, 1,
                       nullptr);
    return hipGetLastError();
}

// Which many-row kernel takes a projection: 0 = the 128-row kernel, 16 / 12 = the 256-row kernel with blocks of 16 / 12 feature
// tiles.  The 256-row block needs two thirds of the 128-row blocks' operand bytes per flop (a compute unit draws about 50 GB/s in
// either kernel; a fifth of the requests go beyond the XCD's L2 and a request takes 400 cycles and more on average), but the
// compute units take its blocks one at a time, so a launch costs whole rounds of blocks and what counts is how many of the 256
// units its one round keeps busy: the width whose blocks number at most 256 and come closest to it (1024 rows x 12288 features:
// 192 blocks of 256 features or 256 blocks of 192).  It wins when that is most of the chip while the 128-row kernel would have to
// give some compute units a second pair of blocks (measured, 1024 rows: QKV 111 -> 97 us; 512 rows: gate/up 108 -> 92 us); with
// more than 256 blocks its second round costs more than it saves (1024 rows: gate/up 159 -> 187 us), with few blocks the 128-row
// kernel's finer grain fills more compute units (512 rows: QKV 66 -> 92 us), and the K slices of the d_model-wide residual
// projections do no better either (1024 rows: 51 -> 58 us, 95 -> 96 us).
static int block_gemm_width(int mode, int epi, int M, int n_tiles) {  // mode 0 / 1 / 2: never / always 16 tiles / always 12 tiles (tuning knob)
    if (epi == EPI_RESID || mode == 0) return 0;
    if (mode == 1) return 16;
    if (mode == 2) return 12;
    const int m_blocks = (M + 255) / 256;
    const int b16 = (n_tiles + 15) / 16 * m_blocks, b12 = (n_tiles + 11) / 12 * m_blocks, blocks128 = (n_tiles + 15) / 16 * ((M + 127) / 128);
    if (blocks128 <= 256) return 0;
    if (b12 <= 256 && b12 >= 144) return 12;  // the narrower block has more blocks: closer to one per compute unit
    if (b16 <= 256 && b16 >= 144) return 16;
    return 0;
}

hipError_t launch_gemm_wide(int epi, int layout_nt, int n_tiles, const GemmArgs& a, float* part, size_t part_bytes, int block_mode, hipStream_t s) {
    if (!a.x_frag) return hipErrorInvalidValue;
    // the kernel addresses weights and activations with 32-bit byte offsets from their bases
    if ((unsigned long long)(n_tiles + layout_nt) * a.nkt * 1024ull >= (1ull << 32) || (unsigned long long)(a.M + 16) * a.nkt * 64ull >= (1ull << 32))
        return hipErrorInvalidValue;
    const WideShape sh = wide_shape(epi, a.M);
    const bool narrow = sh.wnt == 2, half = sh.bmt == 4;
    const int bw = (!narrow && !half) ? block_gemm_width(block_mode, epi, a.M, n_tiles) : 0;
    if (bw == 16) {
        switch (epi) {
            case EPI_QKV: return launch_block<EPI_QKV, 2, 4, 8, 4>(layout_nt, n_tiles, a, s);
            case EPI_SWIGLU: return launch_block<EPI_SWIGLU, 2, 4, 8, 4>(layout_nt, n_tiles, a, s);
            case EPI_LOGITS: return launch_block<EPI_LOGITS, 2, 4, 8, 4>(layout_nt, n_tiles, a, s);
        }
    } else if (bw == 12) {
        switch (epi) {
            case EPI_QKV: return launch_block<EPI_QKV, 4, 2, 4, 6>(layout_nt, n_tiles, a, s);
            case EPI_SWIGLU: return launch_block<EPI_SWIGLU, 4, 2, 4, 6>(layout_nt, n_tiles, a, s);
            case EPI_LOGITS: return launch_block<EPI_LOGITS, 4, 2, 4, 6>(layout_nt, n_tiles, a, s);
        }
    }
    switch (epi) {
        case EPI_QKV:
            if (half) return launch_wide_shape<EPI_QKV, 4, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
            return narrow ? launch_wide_shape<EPI_QKV, 8, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s)
                          : launch_wide_shape<EPI_QKV, 8, 4, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
        case EPI_SWIGLU:
            if (half) return launch_wide_shape<EPI_SWIGLU, 4, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
            return narrow ? launch_wide_shape<EPI_SWIGLU, 8, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s)
                          : launch_wide_shape<EPI_SWIGLU, 8, 4, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
        case EPI_RESID:
            if (half) return launch_wide_shape<EPI_RESID, 4, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
            return narrow ? launch_wide_shape<EPI_RESID, 8, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s)
                          : launch_wide_shape<EPI_RESID, 8, 4, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
        case EPI_LOGITS:
            if (half) return launch_wide_shape<EPI_LOGITS, 4, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
            return narrow ? launch_wide_shape<EPI_LOGITS, 8, 2, 4>(layout_nt, n_tiles, a, part, part_bytes, s)
                          : launch_wide_shape<EPI_LOGITS, 8, 4, 4>(layout_nt, n_tiles, a, part, part_bytes, s);
    }
    return hipErrorInvalidValue;
}

// ---- 4-bit weights (W4A16) ------------------------------------------------------------------------
// w[n][k] = scale[n][k/128] * (code[n][k] - 8), codes 0..15, scales bf16 per 128-column group.  The stream from HBM
// is a quarter of the bf16 one, so the unpacking has to stay cheap:
//   * a lane's 16 bytes hold its 8 codes for each of the 4 k-tiles of one 128-column chunk; inside a dword the
//     nibbles are ordered so that ((d >> 4j) & 0x000F000F) | 0x43004300 is the bf16 pair (128 + code[2j], 128 +
//     code[2j+1]) — two integer instructions per pair, no conversion;
//   * the constant 128 + 8 is taken out by one extra MFMA per k-tile whose weight operand is the constant -136
//     (it adds -136 * sum_k x_k to every row, exactly what the offset contributes);
//   * the group's partial result is scaled once per chunk: acc += scale[n] * acc_chunk.
// RMSNorm: the gain cannot be folded into integer codes; a normed projection gets activations that already carry
// the gain, and the rows' sums of squares as partial sums left by the kernel that produced them.
template <int MT, int NT, int EPI>
__global__ void __launch_bounds__(512) skinny_gemm_w4_kernel(const GemmArgs a) {
    using T = bf16_t;
    using E = Elem<T>;
    using frag_t = E::frag_t;
    constexpr bool NORM = (EPI != EPI_RESID);
    constexpr int PF = 2;  // 128-column chunks of loads kept in flight per wave (4 was measured slower: qkv 14.5 -> 16.9 us at 16 rows)
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, NW = blockDim.x >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int grp = blockIdx.x, mb = blockIdx.y;
    const int row0 = mb * MT * 16;
    const int nkc = a.nkt >> 2;                       // chunks of 4 k-tiles
    const int nsteps = (nkc - w + NW - 1) / NW;       // >= 1: the host never launches more waves than chunks
    const unsigned char* wbase = (const unsigned char*)a.Wp + ((size_t)grp * nkc) * (size_t)(NT * 1024) + (size_t)lane * 16;
    const bf16_t* sbase = (const bf16_t*)a.Sp + ((size_t)grp * nkc) * (size_t)(NT * 16) + g * 4;
    const T* xrow[MT];
    const size_t xstep = a.x_frag ? (size_t)64 * E::EPF : (size_t)E::KT;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (a.x_frag) {
            xrow[mt] = (const T*)a.X + (((size_t)(mb * MT + mt) * a.nkt) * 64 + lane) * E::EPF;
        } else {
            const int m = min(row0 + mt * 16 + r16, a.M - 1);
            xrow[mt] = (const T*)a.X + (size_t)m * a.ldx + g * E::EPF;
        }
    }

    const f32x4 resid_first = prefetch_resid<T, MT, NT, EPI>(a, w, grp, row0, r16, g);
    f32x4 acc[MT][NT];
    float ss[MT];
    constexpr int SSP_LOADS = 12;  // 8 waves x 4 lane groups x 12 = 384 partial sums: d_model up to 6144 without the tail loop
    float sp[MT][SSP_LOADS];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        ss[mt] = 0.f;
        if (NORM) {
            // This lane's share of the row's partial sums of squares; the cross-wave reduction adds the shares up.  The
            // loads go out together here (a loop of load-wait-add would put several memory round trips in front of the
            // first weight fetch); they are added up after the K loop.
            const int m = min(row0 + mt * 16 + r16, a.M - 1);
#pragma unroll
            for (int i = 0; i < SSP_LOADS; ++i) {
                const int j = w * 4 + g + i * 4 * NW;
                sp[mt][i] = j < a.ssp_n ? a.ssp_in[(size_t)j * a.ssp_stride + m] : 0.f;
            }
            for (int j = w * 4 + g + SSP_LOADS * 4 * NW; j < a.ssp_n; j += 4 * NW) ss[mt] += a.ssp_in[(size_t)j * a.ssp_stride + m];  // very wide models
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    frag_t koff;
#pragma unroll
    for (int e = 0; e < 8; ++e) koff[e] = (bf16_t)(-136.0f);

    u32x4 cq[PF][NT];
    bf16x4 sq[PF][NT];
    frag_t xq[PF][4][MT];
    auto issue = [&](int s, int step) {
        const int c = w + min(step, nsteps - 1) * NW;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            cq[s][nt] = __builtin_nontemporal_load((const u32x4*)(wbase + ((size_t)c * NT + nt) * 1024));
            sq[s][nt] = *(const bf16x4*)(sbase + ((size_t)c * NT + nt) * 16);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xq[s][q][mt] = *(const frag_t*)(xrow[mt] + (size_t)(c * 4 + q) * xstep);
        }
    };
    auto consume = [&](int s, int step) {
        const bool live = step < nsteps;
        f32x4 accg[MT][NT], acco[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acco[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) accg[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            frag_t wf[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const unsigned d = cq[s][nt][q];
                unsigned pr[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) pr[j] = ((d >> (4 * j)) & 0x000F000Fu) | 0x43004300u;
                wf[nt] = __builtin_bit_cast(frag_t, u32x4{pr[0], pr[1], pr[2], pr[3]});
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const frag_t av = xq[s][q][mt];
                acco[mt] = E::mma(koff, av, acco[mt]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) accg[mt][nt] = E::mma(wf[nt], av, accg[mt][nt]);
            }
        }
        if (live) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float sc = (float)sq[s][nt][v];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt][nt][v] += sc * (accg[mt][nt][v] + acco[mt][v]);
                }
        }
    };
#pragma unroll
    for (int s = 0; s < PF; ++s) issue(s, s);
    const int nrounds = (nsteps + PF - 1) / PF;
    for (int rd = 0; rd + 1 < nrounds; ++rd) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            consume(s, rd * PF + s);
            issue(s, (rd + 1) * PF + s);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int s = 0; s < PF; ++s) consume(s, (nrounds - 1) * PF + s);

    if (NORM) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < SSP_LOADS; ++i) ss[mt] += sp[mt][i];
    }
    reduce_and_store<T, MT, NT, EPI>(a, acc, ss, smem, lane, w, NW, grp, row0, resid_first);
}

template <int MT, int NT, int EPI>
static hipError_t launch_one_w4(int NW, int n_groups, const GemmArgs& a0, hipStream_t s) {
    GemmArgs a = a0;
    const int mblocks = (a.M + MT * 16 - 1) / (MT * 16);
    a.red_copies = reduction_copies(NW, MT, NT);
    const size_t lds = (size_t)a.red_copies * MT * NT * 1024 + (size_t)NW * MT * 16 * sizeof(float);
    hipLaunchKernelGGL((skinny_gemm_w4_kernel<MT, NT, EPI>), dim3(n_groups, mblocks), dim3(NW * 64), lds, s, a);
    return hipGetLastError();
}

template <int EPI>
static hipError_t launch_mt_nt_w4(int MT, int NT, int NW, int n_groups, const GemmArgs& a, hipStream_t s) {
    constexpr bool PAIR = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
#define FS_CASE(mt, nt) \
    if (MT == mt && NT == nt) return launch_one_w4<mt, nt, EPI>(NW, n_groups, a, s);
    if constexpr (!PAIR) {
        FS_CASE(1, 1) FS_CASE(2, 1)
    }
    FS_CASE(1, 2) FS_CASE(2, 2) FS_CASE(1, 4) FS_CASE(2, 4)
#undef FS_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_w4(int epi, int NT, int NW, int n_groups, const GemmArgs& a, hipStream_t s) {
    // at most 32 rows per workgroup (register budget); longer segments take a second row block, whose pass over
    // the quarter-size weights mostly hits in L2
    const int MT = a.M <= 16 ? 1 : 2;
    if (NW > 8) NW = 8;
    if (MT * NT >= 8 && NW > 4) NW = 4;  // as in the dense launcher
    if (epi == EPI_QKV) return launch_mt_nt_w4<EPI_QKV>(MT, NT, NW, n_groups, a, s);
    if (epi == EPI_RESID) return launch_mt_nt_w4<EPI_RESID>(MT, NT, NW, n_groups, a, s);
    if (epi == EPI_SWIGLU) return launch_mt_nt_w4<EPI_SWIGLU>(MT, NT, NW, n_groups, a, s);
    if (epi == EPI_LOGITS) return launch_mt_nt_w4<EPI_LOGITS>(MT, NT, NW, n_groups, a, s);
    return hipErrorInvalidValue;
}

// Entry of a stage whose projections take fragment-major activations and the rows' sums of squares from their producer
// (4-bit weights, many-row segments; see GemmArgs::gain_next): row-major rows -> fragment-major copy (times the gain, if
// given) + partial sums of squares per 512-column slice.  Workgroup (row tile, slice); thread (r, g, j) converts the
// 8-element fragment pieces of k-tiles j, j + 4, ... of its slice.
__global__ void __launch_bounds__(256) prenorm_kernel(const bf16_t* X, int ldx, int M, int K, const bf16_t* gain, bf16_t* xg, float* ssp,
                                                         int ssp_stride) {
    __shared__ float red[16][17];
    const int t = threadIdx.x, r = t & 15, g = (t >> 4) & 3, j = t >> 6;
    const int mt = blockIdx.x, slice = blockIdx.y, nkt = K >> 5;
    const int m = mt * 16 + r, mc = min(m, M - 1);
    float ss = 0.f;
    const int kt_end = min(nkt, slice * 16 + 16);
    for (int kt = slice * 16 + j; kt < kt_end; kt += 4) {
        const int k = kt * 32 + g * 8;
        const bf16x8 x = *(const bf16x8*)(X + (size_t)mc * ldx + k);
        bf16x8 y = x;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float f = (float)x[e];
            ss += f * f;
        }
        if (gain) {
            const bf16x8 gn = *(const bf16x8*)(gain + k);
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = (bf16_t)((float)x[e] * (float)gn[e]);
        }
        *(bf16x8*)(xg + frag_major_index<bf16_t>(m, k, nkt)) = y;
    }
    red[t >> 4][r] = ss;
    __syncthreads();
    if (t < 16) {
        float s = 0.f;
        for (int i = 0; i < 16; ++i) s += red[i][t];
        if (mt * 16 + t < ssp_stride) ssp[(size_t)slice * ssp_stride + mt * 16 + t] = s;
    }
}

hipError_t launch_prenorm(const void* X, int ldx, int M, int K, const void* gain, void* xg, float* ssp, int ssp_stride, int* n_slices,
                             hipStream_t s) {
    const int slices = (K + 511) / 512;
    *n_slices = slices;
    hipLaunchKernelGGL(prenorm_kernel, dim3((M + 15) / 16, slices), dim3(256), 0, s, (const bf16_t*)X, ldx, M, K, (const bf16_t*)gain,
                       (bf16_t*)xg, ssp, ssp_stride);
    return hipGetLastError();
}

// Source row of packed row (ptile, r) for the three matrix kinds; -1 if beyond the matrix.  `which` selects the source slot.
static __device__ __forceinline__ long long packed_source_row(int kind, int ptile, int r, int N, int Hq, int Hkv, int hd, int* which) {
    *which = 0;
    if (kind == PACK_PLAIN) {
        const long long row = (long long)ptile * 16 + r;
        return row < N ? row : -1;
    }
    if (kind == PACK_GATEUP) {
        *which = ptile & 1;
        const long long row = (long long)(ptile >> 1) * 16 + r;
        return row < N ? row : -1;
    }
    const int tph = hd >> 4, head = ptile / tph, tih = ptile % tph;
    if (head < Hq + Hkv) {
        const int orig = (tih >> 1) + (tih & 1) * (tph >> 1);
        *which = head < Hq ? 0 : 1;
        return (long long)(head < Hq ? head : head - Hq) * hd + orig * 16 + r;
    }
    if (head < Hq + 2 * Hkv) {
        *which = 2;
        return (long long)(head - Hq - Hkv) * hd + tih * 16 + r;
    }
    return -1;
}

__global__ void pack_w4_kernel(const PackW4Args a) {
    const int nkc = a.K / 128;
    const size_t total = (size_t)a.n_groups * nkc * a.NT * 64;
    for (size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(c & 63);
        size_t t = c >> 6;
        const int nt = (int)(t % a.NT);
        t /= a.NT;
        const int chunk = (int)(t % nkc), grp = (int)(t / nkc);
        const int r = lane & 15, g = lane >> 4;
        const int ptile = grp * a.NT + nt;
        int which;
        const long long row = packed_source_row(a.kind, ptile, r, a.N, a.Hq, a.Hkv, a.hd, &which);
        const unsigned char* codes = (const unsigned char*)(which == 0 ? a.c0 : (which == 1 ? a.c1 : a.c2));
        unsigned d[4];
        for (int q = 0; q < 4; ++q) {
            unsigned v = 0;
            for (int e = 0; e < 8; ++e) {
                unsigned code = 8;  // rows beyond the matrix: zero weight
                if (row >= 0) {
                    const int k = chunk * 128 + q * 32 + g * 8 + e;
                    const unsigned char b = codes[(size_t)row * (a.K / 2) + (k >> 1)];
                    code = (k & 1) ? (b >> 4) : (b & 15);
                }
                v |= code << (4 * ((e & 1) * 4 + (e >> 1)));
            }
            d[q] = v;
        }
        ((u32x4*)a.dst)[c] = u32x4{d[0], d[1], d[2], d[3]};
        if (g == 0) {
            const bf16_t* sc = (const bf16_t*)(which == 0 ? a.s0 : (which == 1 ? a.s1 : a.s2));
            ((bf16_t*)a.sdst)[(((size_t)grp * nkc + chunk) * a.NT + nt) * 16 + r] = row >= 0 ? sc[(size_t)row * nkc + chunk] : (bf16_t)0.f;
        }
    }
    if (a.kind == PACK_QKV && a.bias_dst) {
        const int np = a.n_groups * a.NT * 16;
        for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < np; i += gridDim.x * blockDim.x) {
            int which;
            const long long row = packed_source_row(PACK_QKV, i >> 4, i & 15, a.N, a.Hq, a.Hkv, a.hd, &which);
            const bf16_t* b = (const bf16_t*)(which == 0 ? a.b0 : (which == 1 ? a.b1 : a.b2));
            a.bias_dst[i] = (row >= 0 && b) ? (float)b[row] : 0.f;
        }
    }
}

void launch_pack_w4(const PackW4Args& a, hipStream_t s) {
    const size_t total = (size_t)a.n_groups * (a.K / 128) * a.NT * 64;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(pack_w4_kernel, dim3(blocks), dim3(256), 0, s, a);
}

// ---- one-time weight re-tiling ------------------------------------------------------------------
// One thread per 16-byte fragment slot of the destination.  Rows of Q and K heads are re-ordered so that
// tiles (2i, 2i+1) of a head hold features [16i, 16i+16) and [hd/2 + 16i, hd/2 + 16i + 16): the two halves
// of the rotary pairs land in one workgroup.  Gate and up rows alternate tile by tile so that silu(gate)*up
// is formed in the epilogue.  Rows / columns beyond N / K are zero.
template <typename T>
__global__ void pack_kernel(const PackArgs a) {
    using E = Elem<T>;
    const size_t total = (size_t)a.n_groups * a.nkt * a.NT * 64;
    for (size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(c & 63);
        size_t t = c >> 6;
        const int nt = (int)(t % a.NT);
        t /= a.NT;
        const int kt = (int)(t % a.nkt);
        const int grp = (int)(t / a.nkt);
        const int r = lane & 15, g = lane >> 4;
        const int ptile = grp * a.NT + nt;
        const int k = kt * E::KT + g * E::EPF;
        const T* src = nullptr;
        long long row = -1;
        if (a.kind == PACK_PLAIN) {
            row = (long long)ptile * 16 + r;
            src = (const T*)a.src0;
            if (row >= a.N) row = -1;
        } else if (a.kind == PACK_GATEUP) {
            row = (long long)(ptile >> 1) * 16 + r;
            src = (const T*)((ptile & 1) ? a.src1 : a.src0);
            if (row >= a.N) row = -1;  // N = d_ffn here
        } else {
            const int tph = a.hd >> 4;
            const int head = ptile / tph, tih = ptile % tph;
            if (head < a.Hq + a.Hkv) {
                const int orig = (tih >> 1) + (tih & 1) * (tph >> 1);
                const int hh = head < a.Hq ? head : head - a.Hq;
                src = (const T*)(head < a.Hq ? a.src0 : a.src1);
                row = (long long)hh * a.hd + orig * 16 + r;
            } else if (head < a.Hq + 2 * a.Hkv) {
                src = (const T*)a.src2;
                row = (long long)(head - a.Hq - a.Hkv) * a.hd + tih * 16 + r;
            }
        }
        typename E::frag_t f = E::zero();
        if (row >= 0 && k < a.K) {
#pragma unroll
            for (int e = 0; e < E::EPF; ++e) {
                float v = E::to_f(src[(size_t)row * a.K + k + e]);
                if (a.gain) v *= E::to_f(((const T*)a.gain)[k + e]);
                f[e] = E::from_f(v);
            }
        }
        ((typename E::frag_t*)a.dst)[c] = f;
    }
    // packed-order bias (QKV only)
    if (a.kind == PACK_QKV && a.bias_dst) {
        const int np = a.n_groups * a.NT * 16;
        for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < np; i += gridDim.x * blockDim.x) {
            const int ptile = i >> 4, r = i & 15;
            const int tph = a.hd >> 4;
            const int head = ptile / tph, tih = ptile % tph;
            float v = 0.f;
            if (head < a.Hq + a.Hkv) {
                const int orig = (tih >> 1) + (tih & 1) * (tph >> 1);
                const int hh = head < a.Hq ? head : head - a.Hq;
                const T* b = (const T*)(head < a.Hq ? a.b0 : a.b1);
                if (b) v = E::to_f(b[hh * a.hd + orig * 16 + r]);
            } else if (head < a.Hq + 2 * a.Hkv) {
                const T* b = (const T*)a.b2;
                if (b) v = E::to_f(b[(head - a.Hq - a.Hkv) * a.hd + tih * 16 + r]);
            }
            a.bias_dst[i] = v;
        }
    }
}

void launch_pack(int dtype, const PackArgs& a, hipStream_t s) {
    const size_t total = (size_t)a.n_groups * a.nkt * a.NT * 64;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    if (dtype == 0)
        hipLaunchKernelGGL(pack_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(pack_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, a);
}
