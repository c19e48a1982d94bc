// Tree attention of one draft segment against the stage's KV cache (split-KV, LDS-staged, MFMA).
//
// Rows: the segment's M rows of the G = Hq/Hkv query heads that share one KV head are stacked into
// R = G*M rows (rho = qh_local*M + r) so that each K/V element fetched from HBM serves all of them.
// Grid: (KV split, KV head, row block).  A workgroup walks its slots in tiles of 64 (32 for 512-byte rows): the tile's K rows
// are copied to LDS as they are; V rows too for bf16 (the V^T operand is then fetched with the LDS transpose
// load ds_read_b64_tr_b16), while f32 V rows are transposed as they are stored (Vt[t][slot]).  Each wave owns MTW 16-row tiles of R:
//     S^T = K . Q^T      (A = K fragment, rows = slots; B = Q fragment, rows = query rows)
//     O^T += V^T . P^T   (A = V^T fragment, rows = head-dim index; B = P fragment, rows = query rows)
// Both products leave lane l with values of query row l % 16, so the online-softmax state (running max,
// running sum, rescale factor) is per lane and P never leaves registers: lane (r, g) holds
// S^T[slot = 16*j + 4*g + v][r], which is exactly the B-fragment element order of a contraction index
// permuted as slot = 16*(e/4) + 4*g + e%4 — the V^T fragment is read with the same permutation.
//
// Visibility (tree mask): slot s is seen by row r iff s < l_glo, or bit (s - l_glo) of the row's
// ancestor-or-self mask is set.  Tiles that lie entirely below l_glo skip the mask test.
// With more than one split each workgroup writes un-normalised partial outputs plus (max, sum) per row and
// attn_merge_kernel combines them in a fixed order (deterministic).  (Letting the last workgroup to arrive do
// the merge was measured and rejected: the device-scope fences it needs write back and invalidate the whole
// per-XCD L2 once per workgroup, several times the cost of a second launch.)
// (tree_attn_dma_kernel below is the variant for 16-bit K/V of head dim 128 with at most four row tiles: its tiles go from
// global memory straight into LDS.)
// All threads of the workgroup (256 or 512) stage a tile together; the next tile's global loads — the next two for long
// splits — are issued before the current tile is computed, so HBM latency overlaps the MFMA work.  The kernel is bound
// by that stream: with the arithmetic removed it is only about 7 % faster at a 16k context.
#include "attention.hpp"

#include <stdlib.h>

#include <type_traits>

#ifndef PADK
#define PADK 8   /* elements; keeps K rows 16-byte aligned and spreads LDS banks */
#endif
#ifndef PADVR
#define PADVR 8  /* the same for V rows staged row-major (16-bit types) */
#endif
#define PADV 16
#define NEG_BIG (-1.0e30f)

// Merge of the splits of one (KV head, row): out = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s.  MERGE_LANES adjacent
// lanes share one output chunk: lane q takes splits q, q + MERGE_LANES, ... (all its loads are independent of the arithmetic
// and go out together), then the lanes combine pairwise in a fixed order (deterministic).  4 lanes from 4 splits on (few
// rows, many splits: the kernel is latency-bound and wants its loads spread), 1 lane below (many rows, 2-3 splits).
template <typename T, int MERGE_LANES>
static __device__ __forceinline__ void merge_row_chunk(const AttnArgs& a, int kvh, int rho, int c, int q) {  // rho: stacked over the batch
    using E = Elem<T>;
    float m = NEG_BIG, den = 0.f;
    f32x4 o{0.f, 0.f, 0.f, 0.f};
    const size_t sstride = (size_t)a.Hkv * a.Rpad;  // rows between consecutive splits
    const float* pml = a.part_ml + ((size_t)kvh * a.Rpad + rho) * 2;
    const float* po = a.part_o + ((size_t)kvh * a.Rpad + rho) * a.hd + c * 4;
#pragma unroll 4
    for (int s = q; s < a.n_splits; s += MERGE_LANES) {
        const float2 ml = *(const float2*)(pml + (size_t)s * sstride * 2);
        const f32x4 v = *(const f32x4*)(po + (size_t)s * sstride * a.hd);
        const float mn = fmaxf(m, ml.x);
        const float w_old = exp2f(m - mn), w_new = exp2f(ml.x - mn);
        den = den * w_old + ml.y * w_new;
        o = o * w_old + v * w_new;
        m = mn;
    }
#pragma unroll
    for (int x = 1; x < MERGE_LANES; x <<= 1) {
        const float m2 = __shfl_xor(m, x, FS_WAVE), den2 = __shfl_xor(den, x, FS_WAVE);
        f32x4 o2;
#pragma unroll
        for (int e = 0; e < 4; ++e) o2[e] = __shfl_xor(o[e], x, FS_WAVE);
        const float mn = fmaxf(m, m2);
        const float w1 = exp2f(m - mn), w2 = exp2f(m2 - mn);
        // both lanes of a pair add in the same order (lower lane's term first), so they hold identical results
        const bool lo = (q & x) == 0;
        den = lo ? den * w1 + den2 * w2 : den2 * w2 + den * w1;
        o = lo ? o * w1 + o2 * w2 : o2 * w2 + o * w1;
        m = mn;
    }
    if (q != 0) return;
    const float inv = 1.0f / den;
    // the request that owns this row: stacked rows [G * row0, G * (row0 + M))
    int rq = 0;
    while (rq + 1 < a.n_req && rho >= a.G * a.req[rq + 1].row0) ++rq;
    const int M = a.req[rq].M, loc = rho - a.G * a.req[rq].row0;
    const int qh = kvh * a.G + loc / M, r = a.req[rq].row0 + loc % M;
    *(typename E::out4_t*)((T*)a.o + frag_major_index<T>(r, qh * a.hd + c * 4, a.Hq * a.hd / E::KT)) =
        E::pack4(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv);
}

template <typename T, int HD, int MTW, int NWAVES, int NSET, bool STREAM>
__global__ void __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2))) tree_attn_kernel(int row_blocks, const AttnArgs a) {
    using E = Elem<T>;
    using frag_t = typename E::frag_t;
    constexpr int EPF = E::EPF, KT = E::KT;
    constexpr int BS = (sizeof(T) * HD >= 512) ? 32 : 64;  // slots per LDS tile (keeps K + V^T within 64 KiB)
    constexpr int NKT = HD / KT;      // k-tiles of the head dim (QK^T contraction)
    constexpr int NHT = HD / 16;      // 16-wide tiles of the head dim (rows of O^T)
    constexpr int NSUB = EPF / 4;     // 16-slot sub-tiles per P fragment
    constexpr int NPF = BS / (16 * NSUB);
    // bf16: V is staged row-major like K and read back transposed with the LDS transpose load of gfx950;
    // f32 (no 32-bit transpose load exists): V is transposed while it is stored.
    constexpr bool VTR = (sizeof(T) == 2);
    constexpr int KROW = HD + PADK, VROW = VTR ? (HD + PADVR) : (BS + PADV);
    constexpr int NCC = HD / EPF;     // 16-byte chunks per K/V row
    constexpr int CH = BS * NCC;      // chunks per tile (K and V each)
    constexpr int NTHR = NWAVES * 64; // every thread stages; waves beyond the compute waves do nothing else
    constexpr int CPT = CH / NTHR;    // chunks per thread (K and V each)
    static_assert(CH % NTHR == 0, "tile must split evenly over the workgroup");
    __shared__ __align__(16) T Ks[BS * KROW];
    __shared__ __align__(16) T Vt[VTR ? BS * VROW : HD * VROW];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    // grid: (KV split, KV head, request x row block); row_blocks is a leading scalar argument so that the request's table
    // entry can be fetched together with the other kernel arguments
    const int split = blockIdx.x, kvh = blockIdx.y, rqi = blockIdx.z / row_blocks, rb = blockIdx.z % row_blocks;
    const AttnReq rq = a.req[rqi];
    const int M = rq.M, L = rq.L, l_glo = rq.l_glo, row0 = rq.row0;
    const int R = a.G * M;
    // a shorter request of the batch may have no such row block: the workgroup then walks no tiles and stores nothing
    // (no early exit here: a branch on a freshly loaded kernel argument would hold back every other argument load)
    const bool dead = rb * a.nwc * MTW * 16 >= R;
    const int ntiles = dead ? 0 : (L + BS - 1) / BS;
    const int t0 = split * a.tiles_per_split, t1 = min(ntiles, t0 + a.tiles_per_split);
    // waves beyond the compute waves (or whose rows all lie beyond R) only help staging
    const bool computes = (w < a.nwc) && ((rb * a.nwc + w) * MTW * 16 < R);

    int rho[MTW], seg_r[MTW];
    bool rok[MTW];
    frag_t qf[MTW][NKT];
#pragma unroll
    for (int i = 0; i < MTW; ++i) {
        rho[i] = ((rb * a.nwc + w) * MTW + i) * 16 + r16;
        rok[i] = computes && rho[i] < R;
        const int rr = rok[i] ? rho[i] : 0;
        seg_r[i] = row0 + rr % M;  // row of the stacked arrays
        const int qh = kvh * a.G + rr / M;
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

    const T* kbase = (const T*)rq.kbase + a.layer_off + (size_t)kvh * a.stride_head;
    const T* vbase = kbase + a.stride_kv;

    // chunk c of a tile -> K: row-major (slot = c / NCC); V: lane -> (slot_lo, chunk part) so that the transposing
    // LDS stores of one instruction spread over the banks
    // NSET tiles in flight per workgroup, each in a register set of its own: 2 for long splits where the budget allows (one
    // row tile per wave), so that a fetch has two tile periods to arrive; 1 otherwise (less code for the short kernels).
    static_assert(NSET == 1 || MTW == 1, "two register sets only with one row tile per wave");
    frag_t kregs[NSET][CPT], vregs[NSET][CPT];
    // Byte offsets of chunk i of this thread relative to the head's K (or V) base: row part and column part apart, so that the
    // slot of a fetch is clamped to L - 1 with one add and one min per chunk (slots beyond L re-read the last valid one;
    // they are masked below).  No branch inside a fetch: the compiler then counts the loads in flight exactly.
    const unsigned row_bytes = (unsigned)(a.stride_tok * sizeof(T));
    const unsigned last_row = (unsigned)(L - 1) * row_bytes;
    unsigned krow_off[CPT], kcol_off[CPT], vrow_off[CPT], vcol_off[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid + i * NTHR;
        krow_off[i] = (unsigned)(c / NCC) * row_bytes;
        kcol_off[i] = (unsigned)((c % NCC) * EPF * sizeof(T));
        if (VTR) {
            vrow_off[i] = krow_off[i];
            vcol_off[i] = kcol_off[i];
        } else {
            const int it = c >> 6, ln = c & 63;
            vrow_off[i] = (unsigned)((it / (NCC / 4)) * 16 + (ln & 15)) * row_bytes;
            vcol_off[i] = (unsigned)(((it % (NCC / 4)) * 4 + (ln >> 4)) * EPF * sizeof(T));
        }
    }
    auto fetch = [&](int tile, frag_t (&kreg)[CPT], frag_t (&vreg)[CPT]) {
        const unsigned t = (unsigned)(tile * BS) * row_bytes;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const frag_t* kp = (const frag_t*)((const char*)kbase + (min(krow_off[i] + t, last_row) + kcol_off[i]));
            const frag_t* vp = (const frag_t*)((const char*)vbase + (min(vrow_off[i] + t, last_row) + vcol_off[i]));
            // K/V that one workgroup per head and split reads once is streamed past the caches; with several row blocks
            // the later ones find it in L2
            kreg[i] = STREAM ? __builtin_nontemporal_load(kp) : *kp;
            vreg[i] = STREAM ? __builtin_nontemporal_load(vp) : *vp;
        }
    };
    auto stash = [&](const frag_t (&kreg)[CPT], const frag_t (&vreg)[CPT]) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * NTHR;
            *(frag_t*)(&Ks[(c / NCC) * KROW + (c % NCC) * EPF]) = kreg[i];
            if (VTR) {
                *(frag_t*)(&Vt[(c / NCC) * VROW + (c % NCC) * EPF]) = vreg[i];
            } else {
                const int it = c >> 6, ln = c & 63;
                const int slot = (it / (NCC / 4)) * 16 + (ln & 15), col = ((it % (NCC / 4)) * 4 + (ln >> 4)) * EPF;
#pragma unroll
                for (int e = 0; e < EPF; ++e) Vt[(col + e) * VROW + slot] = vreg[i][e];
            }
        }
    };

    // The two words of every row's ancestor mask that cover a tile's draft slots, fetched ahead of the tile's refill in the
    // masked part of the tile range (below): a wait for them then leaves the refill in flight.
    const uint64_t* am[MTW];
#pragma unroll
    for (int i = 0; i < MTW; ++i) am[i] = a.anc + (size_t)seg_r[i] * FS_ANC_WORDS;
    uint64_t mw0[MTW], mw1[MTW];
    auto load_mask = [&](int tile) {
        const int wd = min(max((tile * BS - l_glo) >> 6, 0), FS_ANC_WORDS - 1), wd1 = min(wd + 1, FS_ANC_WORDS - 1);
#pragma unroll
        for (int i = 0; i < MTW; ++i) {
            mw0[i] = am[i][wd];
            mw1[i] = am[i][wd1];
        }
    };

    // one tile from the staged copy in LDS; MASKED: the tile may touch draft slots (its mask words are in mw0 / mw1)
    auto process = [&](int tile, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int s0 = tile * BS;
        if (!computes) return;

        // ---- visibility of the tile's slots for this lane's rows: bit b <-> slot s0 + b --------------------------
        // (slots below l_glo are always visible; draft slot l_glo + j by bit j of the row's ancestor mask; slots
        // beyond L never).  Tiles below l_glo need no mask; a wave none of whose rows sees any slot of the tile
        // skips it (deep chains: the upper triangle).
        const bool need_mask = MASKED && (s0 + BS > l_glo);  // tile touches draft slots or the tail beyond L
        uint64_t vm[MTW];
        if (need_mask) {
            const int d0 = s0 - l_glo, valid = L - s0;  // valid >= 1
            bool any = false;
#pragma unroll
            for (int i = 0; i < MTW; ++i) {
                uint64_t m;
                if (d0 >= 0) {
                    const int wd = d0 >> 6, sh = d0 & 63;
                    m = mw0[i] >> sh;
                    if (sh && wd + 1 < FS_ANC_WORDS) m |= mw1[i] << (64 - sh);
                } else {
                    m = ((1ull << (-d0)) - 1) | (mw0[i] << (-d0));  // 0 < -d0 < BS <= 64
                }
                if (valid < 64) m &= (1ull << valid) - 1;
                if (!rok[i]) m = 0;
                vm[i] = m >> (g * 4);
                any |= (m != 0);
            }
            if (__ballot(any) == 0) return;  // wave-uniform; the staging is already done
        }

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
        // Tiles below l_glo (almost all of a long context) take the short form: no visibility test, scale folded into the
        // exponent's multiply-add.  The running sums are rescaled only when some row's maximum moved (wave-uniform test).
        frag_t pf[MTW][NPF];
#pragma unroll
        for (int i = 0; i < MTW; ++i) {
            float mx = NEG_BIG;
            if (need_mask) {
#pragma unroll
                for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float s = st[i][j][v] * a.scale_log2;
                        const unsigned half = (j * 16 + v) < 32 ? (unsigned)vm[i] : (unsigned)(vm[i] >> 32);
                        if (!(half & (1u << ((j * 16 + v) & 31)))) s = NEG_BIG;
                        st[i][j][v] = s;
                        mx = fmaxf(mx, s);
                    }
            } else {
#pragma unroll
                for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) mx = fmaxf(mx, st[i][j][v]);
                mx *= a.scale_log2;  // the scale is positive: the maximum commutes with it
            }
            mx = wave_xor_max(wave_xor_max(mx, 16), 32);
            const float mnew = fmaxf(mrun[i], mx);
            if (__ballot(mnew != mrun[i]) != 0) {
                const float alpha = __builtin_amdgcn_exp2f(mrun[i] - mnew);  // arguments <= 0: the raw instruction is exact enough, underflow -> 0
                lrun[i] *= alpha;
#pragma unroll
                for (int nt = 0; nt < NHT; ++nt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[i][nt][v] *= alpha;
                mrun[i] = mnew;
            }
            float psum = 0.f;
            float p[BS / 16][4];
            if (need_mask) {
#pragma unroll
                for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float s = st[i][j][v];
                        const float e = (s <= NEG_BIG) ? 0.f : __builtin_amdgcn_exp2f(s - mnew);
                        p[j][v] = e;
                        psum += e;
                    }
            } else {
#pragma unroll
                for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(st[i][j][v], a.scale_log2, -mnew));
                        p[j][v] = e;
                        psum += e;
                    }
            }
            lrun[i] += psum;
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
                if constexpr (VTR) {
                    // Transpose load: within each group of 16 lanes, lane i addresses 4 consecutive head-dim elements of
                    // slot row (i >> 2); lane j receives element j of the group's 16 columns for 4 consecutive slots.
                    const T* vp = &Vt[(jj * NSUB * 16 + g * 4 + (r16 >> 2)) * VROW + nt * 16 + (r16 & 3) * 4];
                    const s16x4 t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)vp);
                    const s16x4 t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vp + 16 * VROW));
                    vf = __builtin_bit_cast(frag_t, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
                } else {
                    const T* vr = &Vt[(nt * 16 + r16) * VROW + jj * NSUB * 16 + g * 4];
#pragma unroll
                    for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
                        for (int v = 0; v < 4; ++v) vf[sub * 4 + v] = vr[sub * 16 + v];
                }
#pragma unroll
                for (int i = 0; i < MTW; ++i) acc[i][nt] = E::mma(vf, pf[i][jj], acc[i][nt]);
            }
    };

#pragma unroll
    for (int k = 0; k < NSET; ++k)
        if (t0 + k < t1) fetch(t0 + k, kregs[k], vregs[k]);
    // Wait here for every load issued so far (Q fragments, first tiles): inside the loop the only vector-memory loads left to
    // wait for are then tile fetches.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
    // The tile range has an unmasked part (slots below l_glo: [t0, tA)) and a masked part ([tA, t1): draft slots and the
    // tail beyond L); tA sits on a register-set boundary, so the masked part may begin with a tile that needs no mask.
    using unmasked_t = std::integral_constant<bool, false>;
    using masked_t = std::integral_constant<bool, true>;
    const int t_mask = max(t0, min(t1, l_glo / BS));
    const int tA = t0 + (t_mask - t0) / NSET * NSET;
    // Unmasked, steady state: every tile of the group has a successor NSET tiles ahead, so store-and-refill is straight-line
    // code and the wait before a store counts exactly the loads of the other register set that may stay in flight (a
    // conditional refill would make the compiler wait for all of them, and the compute phase would never overlap a fetch).
    int tile = t0;
    for (; tile + 2 * NSET <= t1 && tile + NSET <= tA; tile += NSET) {
#pragma unroll
        for (int k = 0; k < NSET; ++k) {
            __syncthreads();  // previous tile fully consumed
            stash(kregs[k], vregs[k]);
            fetch(tile + k + NSET, kregs[k], vregs[k]);  // in flight across the barriers and the next NSET tiles
            __syncthreads();
            process(tile + k, unmasked_t{});
        }
    }
    // Unmasked, last tiles of a range without a masked part: refilled only while a successor exists.
    for (; tile < tA; tile += NSET) {
#pragma unroll
        for (int k = 0; k < NSET; ++k) {
            __syncthreads();
            stash(kregs[k], vregs[k]);
            if (tile + k + NSET < t1) fetch(tile + k + NSET, kregs[k], vregs[k]);
            __syncthreads();
            process(tile + k, unmasked_t{});
        }
    }
    // Masked part, straight-line as well: the mask words are fetched before the refill, the refill is never skipped (past
    // the end it re-reads the range's last tile, a handful of loads that hit in L2), and a tile beyond the end only skips
    // its arithmetic.
    for (; tile < t1; tile += NSET) {
#pragma unroll
        for (int k = 0; k < NSET; ++k) {
            const bool live = tile + k < t1;  // uniform over the workgroup
            __syncthreads();
            stash(kregs[k], vregs[k]);
            load_mask(min(tile + k, t1 - 1));
            fetch(min(tile + k + NSET, t1 - 1), kregs[k], vregs[k]);
            __syncthreads();
            if (live) process(tile + k, masked_t{});
        }
    }

    // ---- write out ----
#pragma unroll
    for (int i = 0; i < MTW; ++i) {
        const float l = wave_xor_add(wave_xor_add(lrun[i], 16), 32);
        if (!rok[i]) continue;
        if (a.n_splits == 1) {
            const float inv = 1.0f / l;
            const int qh = kvh * a.G + rho[i] / M;
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt)
                *(typename E::out4_t*)((T*)a.o + frag_major_index<T>(seg_r[i], qh * HD + nt * 16 + g * 4, a.Hq * HD / KT)) =
                    E::pack4(acc[i][nt][0] * inv, acc[i][nt][1] * inv, acc[i][nt][2] * inv, acc[i][nt][3] * inv);
        } else {
            const size_t prow = ((size_t)split * a.Hkv + kvh) * a.Rpad + a.G * row0 + rho[i];
            float* po = a.part_o + prow * HD + g * 4;
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt) *(f32x4*)(po + nt * 16) = acc[i][nt];
            if (g == 0) *(float2*)(a.part_ml + prow * 2) = make_float2(mrun[i], l);
        }
    }
}


// ---- variant whose K/V tiles go straight from global memory into LDS ------------------------------------------------
// bf16, head dim 128, one row tile per wave, 4 waves.  The tile fetch is the direct-to-LDS load: no registers hold a tile in
// flight, so NBUF - 1 whole tiles (32 KiB each) are in flight per workgroup, behind ONE barrier per tile:
//     wait (own loads of tile t landed, own LDS reads of tile t - 1 done) -> barrier -> issue tile t + NBUF - 1 into the
//     buffer tile t - 1 used -> compute tile t.
// Such a load writes 64 lanes x 16 bytes contiguously, so rows cannot be padded; instead the 16-byte chunk c of slot row r
// sits at chunk position c ^ (r & 15) (each lane chooses which global chunk it fetches), which spreads the fragment reads
// of 16 rows over all banks as the padding does.  The barrier is the bare instruction with explicit wait counts: the fence
// of __syncthreads would wait for every tile in flight.  One array per buffer: distinct objects, so that the compiler's
// own tracking of the direct-to-LDS loads never ties a read of one buffer to a load into another.

template <int NBUF, bool STREAM>
__global__ void __launch_bounds__(256) tree_attn_dma_kernel(int row_blocks, const AttnArgs a) {
    using T = bf16_t;
    using E = Elem<T>;
    using frag_t = E::frag_t;
    constexpr int HD = 128, BS = 64, KT = E::KT, EPF = E::EPF;
    constexpr int NKT = HD / KT, NHT = HD / 16, NSUB = EPF / 4, NPF = BS / (16 * NSUB);
    constexpr int ROWB = HD * (int)sizeof(T);   // 256 bytes per K or V row in LDS
    constexpr int KBYTES = BS * ROWB;           // K part of a buffer; V follows
    constexpr int LPT = 8;                      // direct-to-LDS loads per wave and tile (4 K + 4 V, 4 rows each)
    constexpr int AUX = STREAM ? 2 : 0;         // non-temporal when one row block reads the K/V once
    static_assert(NBUF >= 2 && NBUF <= 4 && LPT * (NBUF - 1) < 64, "vmcnt is a 6-bit counter");
    __shared__ __align__(1024) unsigned char tb0[2 * KBYTES];
    __shared__ __align__(1024) unsigned char tb1[2 * KBYTES];
    __shared__ __align__(1024) unsigned char tb2[NBUF >= 3 ? 2 * KBYTES : 16];
    __shared__ __align__(1024) unsigned char tb3[NBUF >= 4 ? 2 * KBYTES : 16];
    auto buf_at = [&](int j) -> unsigned char* { return j == 0 ? tb0 : (j == 1 ? tb1 : (j == 2 ? tb2 : tb3)); };

    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, rqi = blockIdx.z / row_blocks, rb = blockIdx.z % row_blocks;
    const AttnReq rq = a.req[rqi];
    const int M = rq.M, L = rq.L, l_glo = rq.l_glo, row0 = rq.row0;
    const int R = a.G * M;
    const bool dead = rb * a.nwc * 16 >= R;  // a shorter request of the batch may have no such row block
    const int ntiles = dead ? 0 : (L + BS - 1) / BS;
    const int t0 = split * a.tiles_per_split, t1 = min(ntiles, t0 + a.tiles_per_split);
    const bool computes = (w < a.nwc) && ((rb * a.nwc + w) * 16 < R);

    const int rho = (rb * a.nwc + w) * 16 + r16;
    const bool rok = computes && rho < R;
    const int rr = rok ? rho : 0;
    const int seg_r = row0 + rr % M;
    frag_t qf[NKT];
    {
        const int qh = kvh * a.G + rr / M;
        const T* qp = (const T*)a.q + (size_t)seg_r * (a.Hq * HD) + (size_t)qh * HD + g * EPF;
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) qf[kt] = rok ? *(const frag_t*)(qp + kt * KT) : E::zero();
    }
    f32x4 acc[NHT];
#pragma unroll
    for (int nt = 0; nt < NHT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun = NEG_BIG, lrun = 0.f;

    const unsigned char* kbase = (const unsigned char*)((const T*)rq.kbase + a.layer_off + (size_t)kvh * a.stride_head);
    const unsigned char* vbase = kbase + (size_t)a.stride_kv * sizeof(T);
    // Load i of this wave brings slot rows 16 w + 4 i .. + 3 of the tile: the lane's row and (swizzled) chunk of it.  Slots beyond
    // L - 1 re-read the last valid row (they are masked below).
    const unsigned row_bytes = (unsigned)(a.stride_tok * sizeof(T));
    const unsigned last_row = (unsigned)(L - 1) * row_bytes;
    unsigned row_off[4], col_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 4 * i + (lane >> 4);  // row & 15
        row_off[i] = (unsigned)(16 * w + r) * row_bytes;
        col_off[i] = (unsigned)(((lane & 15) ^ r) * 16);
    }
    // A tile beyond the range (tile >= t1, uniform) is still "loaded", so that every step issues the same number of loads and
    // the wait counts below are exact; its row offset is pushed to the clamp, so all its loads fetch the one last valid row
    // (two cache lines) into a buffer nobody reads.
    auto issue = [&](int tile, unsigned char* buf) {
        const unsigned t = tile < t1 ? (unsigned)(tile * BS) * row_bytes : last_row;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned off = min(row_off[i] + t, last_row) + col_off[i];
            unsigned char* dst = buf + (16 * w + 4 * i) * ROWB;  // wave-uniform; the load adds lane * 16
            __builtin_amdgcn_global_load_lds(FS_GLB_PTR(kbase + off), FS_LDS_PTR(dst), 16, 0, AUX);
            __builtin_amdgcn_global_load_lds(FS_GLB_PTR(vbase + off), FS_LDS_PTR(dst + KBYTES), 16, 0, AUX);
        }
    };

    const uint64_t* am = a.anc + (size_t)seg_r * FS_ANC_WORDS;
    uint64_t mw0 = 0, mw1 = 0;
    auto load_mask = [&](int tile) {
        const int wd = min(max((tile * BS - l_glo) >> 6, 0), FS_ANC_WORDS - 1), wd1 = min(wd + 1, FS_ANC_WORDS - 1);
        mw0 = am[wd];
        mw1 = am[wd1];
    };

    // byte offsets of this lane's fragment reads inside a buffer (without the per-sub-tile strides)
    unsigned kread[NKT], vread[NHT];
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) kread[kt] = (unsigned)(r16 * ROWB + (((kt * 4 + g) ^ r16) * 16));
    {
        const int vr = g * 4 + (r16 >> 2);  // slot row & 15 of the transposing read
#pragma unroll
        for (int nt = 0; nt < NHT; ++nt) vread[nt] = (unsigned)(KBYTES + vr * ROWB + (((nt * 2 + ((r16 & 3) >> 1)) ^ vr) * 16) + (r16 & 1) * 8);
    }

    auto process = [&](int tile, const unsigned char* buf, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int s0 = tile * BS;
        if (!computes) return;
        const bool need_mask = MASKED && (s0 + BS > l_glo);  // the tile touches draft slots or the tail beyond L
        uint64_t vm = 0;
        if (need_mask) {
            const int d0 = s0 - l_glo, valid = L - s0;  // valid >= 1
            uint64_t m;
            if (d0 >= 0) {
                const int wd = d0 >> 6, sh = d0 & 63;
                m = mw0 >> sh;
                if (sh && wd + 1 < FS_ANC_WORDS) m |= mw1 << (64 - sh);
            } else {
                m = ((1ull << (-d0)) - 1) | (mw0 << (-d0));  // 0 < -d0 < BS <= 64
            }
            if (valid < 64) m &= (1ull << valid) - 1;
            if (!rok) m = 0;
            vm = m >> (g * 4);
            if (__ballot(m != 0) == 0) return;  // wave-uniform: none of the wave's rows sees a slot of this tile
        }
        // ---- S^T = K . Q^T ----
        f32x4 st[BS / 16];
#pragma unroll
        for (int j = 0; j < BS / 16; ++j) {
            st[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kt = 0; kt < NKT; ++kt) {
                const frag_t kf = *(const frag_t*)(buf + kread[kt] + j * 16 * ROWB);
                st[j] = E::mma(kf, qf[kt], st[j]);
            }
        }
        // ---- mask, online softmax (as in tree_attn_kernel) ----
        float mx = NEG_BIG;
        if (need_mask) {
#pragma unroll
            for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float sv = st[j][v] * a.scale_log2;
                    const unsigned half = (j * 16 + v) < 32 ? (unsigned)vm : (unsigned)(vm >> 32);
                    if (!(half & (1u << ((j * 16 + v) & 31)))) sv = NEG_BIG;
                    st[j][v] = sv;
                    mx = fmaxf(mx, sv);
                }
        } else {
#pragma unroll
            for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) mx = fmaxf(mx, st[j][v]);
            mx *= a.scale_log2;
        }
        mx = wave_xor_max(wave_xor_max(mx, 16), 32);
        const float mnew = fmaxf(mrun, mx);
        if (__ballot(mnew != mrun) != 0) {
            const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);
            lrun *= alpha;
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[nt][v] *= alpha;
            mrun = mnew;
        }
        float psum = 0.f;
        float p[BS / 16][4];
        if (need_mask) {
#pragma unroll
            for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float sv = st[j][v];
                    const float e = (sv <= NEG_BIG) ? 0.f : __builtin_amdgcn_exp2f(sv - mnew);
                    p[j][v] = e;
                    psum += e;
                }
        } else {
#pragma unroll
            for (int j = 0; j < BS / 16; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(st[j][v], a.scale_log2, -mnew));
                    p[j][v] = e;
                    psum += e;
                }
        }
        lrun += psum;
        frag_t pf[NPF];
#pragma unroll
        for (int jj = 0; jj < NPF; ++jj)
#pragma unroll
            for (int e = 0; e < EPF; ++e) pf[jj][e] = E::from_f(p[jj * NSUB + e / 4][e % 4]);
        // ---- O^T += V^T . P^T (transposing LDS load, rows jj * 32 + g * 4 + (r16 >> 2) and + 16) ----
#pragma unroll
        for (int jj = 0; jj < NPF; ++jj)
#pragma unroll
            for (int nt = 0; nt < NHT; ++nt) {
                const unsigned char* vp = buf + vread[nt] + jj * 32 * ROWB;
                const s16x4 t0v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)vp);
                const s16x4 t1v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vp + 16 * ROWB));
                const frag_t vf = __builtin_bit_cast(frag_t, __builtin_shufflevector(t0v, t1v, 0, 1, 2, 3, 4, 5, 6, 7));
                acc[nt] = E::mma(vf, pf[jj], acc[nt]);
            }
    };

    using unmasked_t = std::integral_constant<bool, false>;
    using masked_t = std::integral_constant<bool, true>;
    if (t1 > t0) {  // uniform over the workgroup
#pragma unroll
        for (int k = 0; k + 1 < NBUF; ++k) issue(t0 + k, buf_at(k));
        FS_WAIT_VM_LGKM(LPT * (NBUF - 1), 15);  // the Q fragments (issued before the tiles) are there; the tiles stay in flight
        // tile `tile` sits in buffer k.  Loads return in order and every step issues one tile's worth, so at each wait all
        // but the newest NBUF - 2 tiles' worth have landed (mask loads issued in between only make a wait stricter).
        auto step = [&](int tile, auto kc, auto masked_tag) {
            constexpr int k = decltype(kc)::value;
            constexpr bool MASKED = decltype(masked_tag)::value;
            asm volatile("" ::: "memory");
            FS_WAIT_VM_LGKM(LPT * (NBUF - 2), 0);
            __builtin_amdgcn_s_barrier();  // tile `tile` complete for every wave; every wave is done with tile - 1
            asm volatile("" ::: "memory");
            if (MASKED) load_mask(tile);
            issue(tile + NBUF - 1, buf_at((k + NBUF - 1) % NBUF));
            process(tile, buf_at(k), masked_tag);
        };
        using b0 = std::integral_constant<int, 0>;
        using b1 = std::integral_constant<int, 1>;
        using b2 = std::integral_constant<int, 2>;
        using b3 = std::integral_constant<int, 3>;
        // The tile range has an unmasked part (slots below l_glo: [t0, tA)) and a masked part ([tA, t1): draft slots and the tail
        // beyond L); tA sits on a buffer-ring boundary, so the masked part may begin with tiles that need no mask.
        const int t_mask = max(t0, min(t1, l_glo / BS));
        const int tA = t0 + (t_mask - t0) / NBUF * NBUF;
        int tile = t0;
        for (; tile < tA; tile += NBUF) {
            step(tile, b0{}, unmasked_t{});
            step(tile + 1, b1{}, unmasked_t{});
            if constexpr (NBUF >= 3) step(tile + 2, b2{}, unmasked_t{});
            if constexpr (NBUF >= 4) step(tile + 3, b3{}, unmasked_t{});
        }
        for (; tile < t1; tile += NBUF) {  // the conditions are uniform over the workgroup
            step(tile, b0{}, masked_t{});
            if (tile + 1 < t1) step(tile + 1, b1{}, masked_t{});
            if constexpr (NBUF >= 3)
                if (tile + 2 < t1) step(tile + 2, b2{}, masked_t{});
            if constexpr (NBUF >= 4)
                if (tile + 3 < t1) step(tile + 3, b3{}, masked_t{});
        }
        // every direct-to-LDS load has landed before the workgroup's LDS is given back
        FS_WAIT_VM_LGKM(0, 0);
    }

    // ---- write out (as tree_attn_kernel) ----
    const float l = wave_xor_add(wave_xor_add(lrun, 16), 32);
    if (!rok) return;
    if (a.n_splits == 1) {
        const float inv = 1.0f / l;
        const int qh = kvh * a.G + rho / M;
#pragma unroll
        for (int nt = 0; nt < NHT; ++nt)
            *(typename E::out4_t*)((T*)a.o + frag_major_index<T>(seg_r, qh * HD + nt * 16 + g * 4, a.Hq * HD / KT)) =
                E::pack4(acc[nt][0] * inv, acc[nt][1] * inv, acc[nt][2] * inv, acc[nt][3] * inv);
    } else {
        const size_t prow = ((size_t)split * a.Hkv + kvh) * a.Rpad + a.G * row0 + rho;
        float* po = a.part_o + prow * HD + g * 4;
#pragma unroll
        for (int nt = 0; nt < NHT; ++nt) *(f32x4*)(po + nt * 16) = acc[nt];
        if (g == 0) *(float2*)(a.part_ml + prow * 2) = make_float2(mrun, l);
    }
}

// Combine the splits: MERGE_LANES threads per (KV head, row, 4 head-dim elements).
template <typename T, int MERGE_LANES>
__global__ void __launch_bounds__(256) attn_merge_kernel(const AttnArgs a) {
    const int R = a.G * a.rows, hd4 = a.hd / 4;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    const int idx = t / MERGE_LANES, q = t % MERGE_LANES;
    if (idx >= a.Hkv * R * hd4) return;  // whole groups of MERGE_LANES lanes leave together
    merge_row_chunk<T, MERGE_LANES>(a, idx / (hd4 * R), (idx / hd4) % R, idx % hd4, q);
}

template <typename T, int HD>
static hipError_t launch_hd(const AttnArgs& a, int MTW, int row_blocks, hipStream_t s) {
    const int nw = a.nwc <= 4 ? 4 : 8;  // every wave stages the tiles; the first a.nwc also compute
    dim3 grid(a.n_splits, a.Hkv, row_blocks * a.n_req), block(nw * 64);
    // K/V tiles in flight per workgroup (a.nset, chosen by attn_plan): rings of 3 and 4 exist for 16-bit types with 4 waves only
    // (the 32-bit kernels would spill), rings of 2 only with one row tile per wave
    int ring = MTW == 1 ? a.nset : 1;
    if (ring > 2 && (sizeof(T) != 2 || nw != 4)) ring = 2;
    const bool deep = ring >= 2;
    bool done = false;
    if constexpr (sizeof(T) == 2 && HD == 128) {
        if (a.dma >= 2 && MTW == 1 && nw == 4) {
            const bool stream = row_blocks == 1;
            if (a.dma >= 4) {
                if (stream) hipLaunchKernelGGL((tree_attn_dma_kernel<4, true>), grid, block, 0, s, row_blocks, a);
                else hipLaunchKernelGGL((tree_attn_dma_kernel<4, false>), grid, block, 0, s, row_blocks, a);
            } else if (a.dma == 3) {
                if (stream) hipLaunchKernelGGL((tree_attn_dma_kernel<3, true>), grid, block, 0, s, row_blocks, a);
                else hipLaunchKernelGGL((tree_attn_dma_kernel<3, false>), grid, block, 0, s, row_blocks, a);
            } else {
                if (stream) hipLaunchKernelGGL((tree_attn_dma_kernel<2, true>), grid, block, 0, s, row_blocks, a);
                else hipLaunchKernelGGL((tree_attn_dma_kernel<2, false>), grid, block, 0, s, row_blocks, a);
            }
            done = true;
        }
    }
    if constexpr (sizeof(T) == 2) {
        if (done) {
        } else if (MTW == 1 && nw == 4 && ring >= 4) {
            hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 4, 4, true>), grid, block, 0, s, row_blocks, a);
            done = true;
        } else if (MTW == 1 && nw == 4 && ring == 3) {
            hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 4, 3, true>), grid, block, 0, s, row_blocks, a);
            done = true;
        }
    }
    if (done) {
    } else if (MTW == 1 && nw == 4 && deep)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 4, 2, true>), grid, block, 0, s, row_blocks, a);
    else if (MTW == 1 && nw == 4)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 4, 1, true>), grid, block, 0, s, row_blocks, a);
    else if (MTW == 1 && deep && row_blocks == 1)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 8, 2, true>), grid, block, 0, s, row_blocks, a);
    else if (MTW == 1 && deep)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 8, 2, false>), grid, block, 0, s, row_blocks, a);
    else if (MTW == 1 && row_blocks == 1)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 8, 1, true>), grid, block, 0, s, row_blocks, a);
    else if (MTW == 1)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 1, 8, 1, false>), grid, block, 0, s, row_blocks, a);
    else if (nw == 4)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 2, 4, 1, true>), grid, block, 0, s, row_blocks, a);
    else if (row_blocks == 1)
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 2, 8, 1, true>), grid, block, 0, s, row_blocks, a);
    else
        hipLaunchKernelGGL((tree_attn_kernel<T, HD, 2, 8, 1, false>), grid, block, 0, s, row_blocks, a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.n_splits > 1) {
        const int chunks = a.Hkv * a.G * a.rows * (a.hd / 4);
        if (a.n_splits >= 4)
            hipLaunchKernelGGL((attn_merge_kernel<T, 4>), dim3((chunks * 4 + 255) / 256), dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL((attn_merge_kernel<T, 1>), dim3((chunks + 255) / 256), dim3(256), 0, s, a);
        e = hipGetLastError();
    }
    return e;
}

void attn_plan(int elem_bytes, int hd, int M, int G, int Hkv, int L, int max_splits, int wgs_override, int mtw_override, int nset_override,
               int nwc_override, int dma_override, int* NWC, int* MTW, int* row_blocks, int* n_splits, int* tiles_per_split, int* nset, int* dma) {
    const int R = G * M, mtiles = (R + 15) / 16;
    const int BS = attn_tile_slots(elem_bytes, hd);
    const int ntiles = (L + BS - 1) / BS;
    // up to 8 compute waves per workgroup; with 4 to 16 row tiles every wave takes 2 of them (each K/V fragment read from
    // LDS then serves 32 rows).  Beyond that there are row blocks enough to fill the chip with few or no KV splits, and one
    // tile per wave is faster (1024-row chunk: 74 -> 65 us, no merge pass).
    int mtw = (mtiles >= 4 && mtiles <= 16) ? 2 : 1;
    // about 2 workgroups per CU for long contexts, fewer and longer splits for short ones (latency-bound: C2 256)
    int target = ntiles <= 32 ? 256 : 512;
    int ring = 2;
    // Long context, at most 64 rows per KV head (4 row tiles, one per wave) and 16-bit K/V: one workgroup per compute unit with
    // three K/V tiles in flight does better than two workgroups with one or two tiles each, and halves the partial results
    // the merge has to read (16k context, 64 rows: 59.0 -> 54.0 us; four tiles in flight 69 us, 320 workgroups 72 us).
    const bool deep_ring = elem_bytes == 2 && mtiles <= 4 && ntiles >= 6 * ((256 + Hkv - 1) / Hkv);
    if (deep_ring) {
        mtw = 1;
        target = 256;
        ring = 3;
    }
    // Long context, 9 to 16 row tiles on few KV heads (grouped-query attention with a wide group): one 8-wave workgroup per
    // head and split leaves half the chip idle and needs many splits, each writing partial results for every row.  Four
    // one-tile waves per workgroup give row blocks instead, which re-read K/V from L2 (4k context, 4 KV heads x 224 rows:
    // 23.2 -> 18.8 us with the merge; 2, 5 or 7 waves, or two tiles per wave, are all slower).
    int nw_cap = 8;
    if (!deep_ring && mtiles > 8 && mtiles <= 16 && Hkv <= 8 && ntiles > 32) {
        mtw = 1;
        nw_cap = 4;
    }
    // the direct-to-LDS kernel: 16-bit K/V, head dim 128, at most 4 one-tile waves
    const bool dma_shape = elem_bytes == 2 && hd == 128 && mtiles <= 4;
    int dma_bufs = 0;
    if (dma_override >= 2 && dma_shape) {
        dma_bufs = dma_override > 4 ? 4 : dma_override;
        mtw = 1;
    }
    if (mtw_override > 0 && !dma_bufs) mtw = (mtw_override >= 2 && mtiles > 1) ? 2 : 1;
    if (wgs_override > 0) target = wgs_override;
    if (nwc_override > 0) nw_cap = nwc_override < 8 ? nwc_override : 8;
    int nw = (mtiles + mtw - 1) / mtw;
    if (nw > nw_cap) nw = nw_cap;
    *NWC = nw;
    *MTW = mtw;
    *row_blocks = (mtiles + nw * mtw - 1) / (nw * mtw);
    const int per_split = Hkv * *row_blocks;  // workgroups per KV split
    int want = (target + per_split - 1) / per_split;
    // one workgroup per compute unit: a handful of workgroups beyond 256 would make a second round of their own
    if (deep_ring && wgs_override <= 0 && want * per_split > 256 && want > 1) --want;
    if (want > max_splits) want = max_splits;
    if (want > ntiles) want = ntiles;
    if (want < 1) want = 1;
    *tiles_per_split = (ntiles + want - 1) / want;
    *n_splits = (ntiles + *tiles_per_split - 1) / *tiles_per_split;
    // tiles in flight: two pay from about 4 tiles per workgroup on, three need two rounds of the ring; never more than the split has
    if (nset_override > 0)
        ring = nset_override;
    else if (ring == 3 && *tiles_per_split < 6)
        ring = 2;
    if (nset_override <= 0 && *tiles_per_split < 4) ring = 1;
    if (ring > *tiles_per_split) ring = *tiles_per_split;
    *nset = ring < 1 ? 1 : ring;
    // The direct-to-LDS kernel where it measured faster: one workgroup per compute unit on a long context with three tile
    // buffers (16k context, 64 rows: 54.6 -> 53.0 us with the merge; two or four buffers 56.7 / 55.2), and grids of two and more
    // workgroups per compute unit with two buffers, two workgroups sharing a unit's LDS (16 / 24 / 32 stacked requests of a
    // 1k context: 55.5 -> 49.9, 81.1 -> 78.0, 107.9 -> 99.0 us; three buffers: slower than the register ring).
    if (dma_override == 0 && dma_shape && mtw == 1 && nw <= 4 && *tiles_per_split >= 6) {
        if ((long long)per_split * *n_splits >= 512)
            dma_bufs = 2;
        else if (deep_ring)
            dma_bufs = 3;
    }
    *dma = dma_bufs;
}

hipError_t launch_attention(int dtype, const AttnArgs& a, int MTW, int row_blocks, hipStream_t s) {
    if (a.hd == 64) return dtype == 0 ? launch_hd<float, 64>(a, MTW, row_blocks, s) : launch_hd<bf16_t, 64>(a, MTW, row_blocks, s);
    if (a.hd == 128) return dtype == 0 ? launch_hd<float, 128>(a, MTW, row_blocks, s) : launch_hd<bf16_t, 128>(a, MTW, row_blocks, s);
    return hipErrorInvalidValue;
}
