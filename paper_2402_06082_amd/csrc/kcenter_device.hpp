// One-shot greedy k-center compression of a prompt's KV cache (Section 3.2 of the paper: the greedy k-center
// algorithm of Dyer and Frieze is applied once; the r most recent tokens are kept, k centers are selected from
// the remaining ones).  Farthest-point traversal: the first center is the oldest token, every next center is
// the token farthest from the centers chosen so far (lowest index on ties); squared distances in double
// precision from the exactly converted elements.  One workgroup per stream; the running nearest-center
// distance and assignment of every old token live in a caller-supplied workspace, and a token is always
// handled by the same lanes, so the k passes need no synchronisation besides the argmax.
#pragma once
#include "subgen_dot2_device.hpp"

namespace sg {

struct KCenterCall {
    const char *K, *V;       // [S][n][d]
    char *outK, *outV;       // [S][k + r][d]: centers in selection order, then the r most recent tokens
    int32_t *out_idx;        // [S][k + r] token index of every output row (-1 = unused)
    int32_t *out_counts;     // [S][k] tokens (older than the window) nearest to each center, or null
    double *mind;            // [S][n_old] workspace
    int32_t *assign;         // [S][n_old] workspace
    float *xnorm;            // [S][n_old] workspace (batched kernel): ||x||^2 of every old token
    int64_t n;
    int32_t k, r;
};

template <bool BF16, int LPR>
__global__ __launch_bounds__(kWG) void kcenter_kernel(const KCenterCall c)
{
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)LPR * 16;
    constexpr int U = kUnroll;
    __shared__ double wbest[kWaves];
    __shared__ int widx[kWaves];
    __shared__ int hist[1024];
    const size_t sid = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR, grp = wave * RPW + sub;
    const int64_t n = c.n;
    const int rwin = (int)(c.r < n ? c.r : n);
    const int nold = (int)(n - rwin);                 // tokens eligible as centers
    const int kk = c.k < nold ? c.k : nold;           // centers actually selected
    const int rows_out = c.k + c.r;
    const char *K = c.K + sid * (size_t)n * ROWB, *V = c.V + sid * (size_t)n * ROWB;
    char *oK = c.outK + sid * (size_t)rows_out * ROWB, *oV = c.outV + sid * (size_t)rows_out * ROWB;
    int32_t *oidx = c.out_idx + sid * (size_t)rows_out;
    double *mind = c.mind + sid * (size_t)(nold > 0 ? nold : 1);
    int32_t *assign = c.assign + sid * (size_t)(nold > 0 ? nold : 1);

    int center = 0;
    for (int it = 0; it < kk; ++it) {
        // emit center `it` and measure every old token against it
        float cf[VEC];
        {
            const uint4 ck = ld16(K + (size_t)center * ROWB + col * 16);
            unpack<BF16>(ck, cf);
            if (tid < LPR) {
                st16(oK + (size_t)it * ROWB + tid * 16, ld16(K + (size_t)center * ROWB + tid * 16));
                st16(oV + (size_t)it * ROWB + tid * 16, ld16(V + (size_t)center * ROWB + tid * 16));
            }
            if (tid == 0) oidx[it] = center;
        }
        double best = -1.0;
        int bidx = -1;
        for (int r0 = grp; r0 < nold; r0 += RPB * U) {
            uint4 raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPB;
                raw[u] = ld16(K + (size_t)(r < nold ? r : nold - 1) * ROWB + col * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPB;
                float x[VEC];
                unpack<BF16>(raw[u], x);
                double dist = 0.0;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double df = (double)x[v] - (double)cf[v];
                    dist = fma(df, df, dist);
                }
                dist = group_sum<LPR>(dist);
                if (r < nold) {
                    double md = dist;
                    if (it == 0) {
                        if (col == 0) {
                            mind[r] = dist;
                            assign[r] = 0;
                        }
                    } else {
                        const double old = mind[r];
                        if (dist < old) {                 // a tie keeps the earlier center
                            if (col == 0) {
                                mind[r] = dist;
                                assign[r] = it;
                            }
                        } else {
                            md = old;
                        }
                    }
                    if (md > best) {                      // rows come in increasing order: first maximum wins
                        best = md;
                        bidx = r;
                    }
                }
            }
        }
        // farthest token over the workgroup (lowest index on ties)
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) {
            const double ob = __shfl_xor(best, o);
            const int oi = __shfl_xor(bidx, o);
            if (ob > best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
                best = ob;
                bidx = oi;
            }
        }
        if (lane == 0) {
            wbest[wave] = best;
            widx[wave] = bidx;
        }
        __syncthreads();
        best = wbest[0];
        bidx = widx[0];
#pragma unroll
        for (int wv = 1; wv < kWaves; ++wv) {
            const double ob = wbest[wv];
            const int oi = widx[wv];
            if (ob > best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
                best = ob;
                bidx = oi;
            }
        }
        center = bidx;
        __syncthreads();
    }
    // unused center rows, then the window (the r most recent tokens, oldest first)
    for (int j = kk + grp; j < c.k; j += RPB) {
        st16(oK + (size_t)j * ROWB + col * 16, make_uint4(0, 0, 0, 0));
        st16(oV + (size_t)j * ROWB + col * 16, make_uint4(0, 0, 0, 0));
        if (col == 0) oidx[j] = -1;
    }
    for (int j = grp; j < c.r; j += RPB) {
        const bool have = j < rwin;
        const size_t src = (size_t)(nold + (have ? j : 0));
        st16(oK + (size_t)(c.k + j) * ROWB + col * 16, have ? ld16(K + src * ROWB + col * 16) : make_uint4(0, 0, 0, 0));
        st16(oV + (size_t)(c.k + j) * ROWB + col * 16, have ? ld16(V + src * ROWB + col * 16) : make_uint4(0, 0, 0, 0));
        if (col == 0) oidx[c.k + j] = have ? (int32_t)src : -1;
    }
    // cluster sizes: how many old tokens ended up nearest to each center
    if (c.out_counts != nullptr) {
        int32_t *oc = c.out_counts + sid * (size_t)c.k;
        for (int base = 0; base < c.k; base += 1024) {
            for (int j = tid; j < 1024; j += kWG) hist[j] = 0;
            __syncthreads();
            for (int r = tid; r < nold; r += kWG) {
                const int a = assign[r] - base;
                if (a >= 0 && a < 1024) atomicAdd(&hist[a], 1);
            }
            __syncthreads();
            for (int j = tid; j < 1024 && base + j < c.k; j += kWG) oc[base + j] = hist[j];
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// The same traversal for bf16 rows, several centers per pass over the keys.
//
// The farthest-point rule picks, after every new center, the token with the largest distance to its nearest
// center (lowest index on ties).  Distances only shrink, so after a pass that leaves every token's exact distance
// in memory, the tokens of a short candidate list can be proved to be the next few centers without touching the
// rest: the tokens are spread over NG groups (by index), the pass keeps each group's largest distance (value,
// token) and second largest (value); every token that is not a group's leader lies at or below
// V = max over groups of the second largest.  The leaders are re-measured against every center picked in the
// round (exact double arithmetic on rows parked in LDS), and while the best leader stays strictly above V it is
// the global maximum, hence the next center.  The first pick of a round is the exact global maximum whatever V
// is.  With 64 groups about ten centers come out of one pass, so the keys are streamed k/10 times, not k times.
//
// In the pass, a (token, center) pair first gets the approximate squared distance
// D~ = ||x||^2 + ||c||^2 - 2<x,c> (packed-bf16 dot products, fp32), whose error is at most
// kDistEps (||x||^2 + ||c||^2); only when D~ minus that bound is below the token's current distance can the pair
// lower it, and only then is the exact double distance computed and compared as the plain definition does.
// Selected tokens, cluster sizes and rows are therefore those of the one-center-per-pass kernel above.
// ---------------------------------------------------------------------------------------------------------
#ifndef SG_KC_BATCH
#define SG_KC_BATCH 16
#endif
#ifndef SG_KC_U
#define SG_KC_U 4
#endif
constexpr int kKcBatch = SG_KC_BATCH;   // centers applied per pass at most

template <int LPR>
__global__ __launch_bounds__(kWG) void kcenter_batched_kernel(const KCenterCall c)
{
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;   // row groups per workgroup
    constexpr size_t ROWB = (size_t)LPR * 16;
    constexpr int U = SG_KC_U;                          // rows in flight per row group = groups per row group
    constexpr int NG = RPB * U;                         // candidate groups (token r belongs to group r mod NG)
    __shared__ uint4 crow[kKcBatch][LPR];               // the centers of the current pass
    __shared__ float cnorm[kKcBatch];
    __shared__ int cidx[kKcBatch];
    __shared__ uint4 candrow[NG][LPR];                  // rows of the group leaders
    __shared__ double candv[NG], cand2[NG];
    __shared__ int candi[NG];
    __shared__ double wbest[kWaves], wsec[kWaves];
    __shared__ int widx[kWaves], wgrp[kWaves];
    __shared__ int hist[1024];
    const size_t sid = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR, grp = wave * RPW + sub;
    const int64_t n = c.n;
    const int rwin = (int)(c.r < n ? c.r : n);
    const int nold = (int)(n - rwin);
    const int kk = c.k < nold ? c.k : nold;
    const int rows_out = c.k + c.r;
    const char *K = c.K + sid * (size_t)n * ROWB, *V = c.V + sid * (size_t)n * ROWB;
    char *oK = c.outK + sid * (size_t)rows_out * ROWB, *oV = c.outV + sid * (size_t)rows_out * ROWB;
    int32_t *oidx = c.out_idx + sid * (size_t)rows_out;
    double *mind = c.mind + sid * (size_t)(nold > 0 ? nold : 1);
    int32_t *assign = c.assign + sid * (size_t)(nold > 0 ? nold : 1);
    float *xnorm = c.xnorm + sid * (size_t)(nold > 0 ? nold : 1);

    // exact squared distance of two rows whose chunks this row group holds: the arithmetic of the kernel above
    auto exact_dist = [&](const uint4 &xa, const uint4 &xb) __attribute__((always_inline)) {
        float a[8], b[8];
        unpack<true>(xa, a);
        unpack<true>(xb, b);
        double dist = 0.0;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const double df = (double)a[v] - (double)b[v];
            dist = fma(df, df, dist);
        }
        return group_sum<LPR>(dist);
    };

    int it = 0, t = 0;
    if (kk > 0) {   // the first center is the oldest token
        if (tid < LPR) crow[0][tid] = ld16(K + tid * 16);
        if (tid == 0) cidx[0] = 0;
        t = 1;
    }
    bool first = true;
    while (it < kk) {
        __syncthreads();   // crow / cidx of this pass are in LDS
        // ---- emit the pass's centers
        for (int i = tid; i < t * LPR; i += kWG) {
            const int j = i / LPR, ch = i % LPR;
            st16(oK + (size_t)(it + j) * ROWB + ch * 16, crow[j][ch]);
            st16(oV + (size_t)(it + j) * ROWB + ch * 16, ld16(V + (size_t)cidx[j] * ROWB + ch * 16));
            if (ch == 0) oidx[it + j] = cidx[j];
        }
        if (tid < t) {   // ||c||^2 as the pass uses it: fp32 rounding of the exact sum (the token's own entry after pass 0)
            float cf[8];
            double a = 0.0;
            for (int ch = 0; ch < LPR; ++ch) {
                unpack<true>(crow[tid][ch], cf);
#pragma unroll
                for (int v = 0; v < 8; ++v) a = fma((double)cf[v], (double)cf[v], a);
            }
            cnorm[tid] = (float)a;
        }
        __syncthreads();

        // ---- one pass over the old tokens: apply the t centers in order, keep the groups' leaders
        double v1[U], v2[U];
        int i1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            v1[u] = -1.0;
            v2[u] = -1.0;
            i1[u] = -1;
        }
        for (int r0 = grp; r0 < nold; r0 += RPB * U) {
            uint4 raw[U];
            double md[U];
            float xn[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPB;
                const int rr = r < nold ? r : nold - 1;
                raw[u] = ld16(K + (size_t)rr * ROWB + col * 16);
                md[u] = first ? INFINITY : mind[rr];
                xn[u] = first ? 0.f : xnorm[rr];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPB;
                if (r < nold) {   // uniform over the row group
                    int as = -1;
                    double m0 = md[u];
                    if (first) {   // ||x||^2 for the later passes (double sum, fp32 rounding)
                        float xf[8];
                        unpack<true>(raw[u], xf);
                        double a = 0.0;
#pragma unroll
                        for (int v = 0; v < 8; ++v) a = fma((double)xf[v], (double)xf[v], a);
                        xn[u] = (float)group_sum<LPR>(a);
                        if (col == 0) xnorm[r] = xn[u];
                    }
                    // fp32 upper bound of the current distance for the filter (refreshed when the distance drops)
                    float m0f = first ? INFINITY : __double2float_ru(m0);
                    for (int j = 0; j < t; ++j) {
                        const uint4 cj = crow[j][col];
                        bool look = first;
                        if (!first) {
                            float dot = dot8_bf16(raw[u], cj);
                            if constexpr (LPR == 16) dot = row_sum16(dot);   // DPP row rotations, no LDS traffic
                            else dot = group_sum<LPR>(dot);
                            const float s2 = xn[u] + cnorm[j];
                            const float dt = fmaf(-2.f, dot, s2);
                            // D >= D~ - eps (||x||^2 + ||c||^2) >= m0f >= m0: the pair cannot lower the distance
                            // (the bound has a fourfold margin, which also covers the rounding of this line)
                            look = dt - kDistEps * s2 < m0f;
                        }
                        if (look) {
                            const double dist = exact_dist(raw[u], cj);
                            if (dist < m0) {   // a tie keeps the earlier center
                                m0 = dist;
                                m0f = __double2float_ru(m0);
                                as = it + j;
                            }
                        }
                    }
                    if (as >= 0 && col == 0) {
                        mind[r] = m0;
                        assign[r] = as;
                    }
                    // leader and runner-up of group (r mod NG); rows come in increasing order: first maximum stays
                    if (m0 > v1[u]) {
                        v2[u] = v1[u];
                        v1[u] = m0;
                        i1[u] = r;
                    } else if (m0 > v2[u]) {
                        v2[u] = m0;
                    }
                }
            }
        }
        first = false;
        it += t;
        if (it >= kk) break;
        if (col == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                candv[grp * U + u] = v1[u];
                candi[grp * U + u] = i1[u];
                cand2[grp * U + u] = v2[u];
            }
        }
        __syncthreads();
        // ---- rows of the leaders, and V = the largest runner-up
        for (int i = tid; i < NG * LPR; i += kWG) {
            const int g = i / LPR, ch = i % LPR;
            const int ri = candi[g];
            candrow[g][ch] = ri >= 0 ? ld16(K + (size_t)ri * ROWB + ch * 16) : make_uint4(0, 0, 0, 0);
        }
        double vloc = -1.0;
        for (int g = tid; g < NG; g += kWG) vloc = fmax(vloc, cand2[g]);
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) vloc = fmax(vloc, __shfl_xor(vloc, o));
        if (lane == 0) wsec[wave] = vloc;
        __syncthreads();
        double Vb = wsec[0];
#pragma unroll
        for (int wv = 1; wv < kWaves; ++wv) Vb = fmax(Vb, wsec[wv]);

        // ---- picks of this round
        t = 0;
        while (true) {
            // best leader: largest current distance, lowest token index on ties
            double bv = -2.0;
            int bi = -1, bg = -1;
            for (int g = tid; g < NG; g += kWG) {
                const double v = candv[g];
                const int i = candi[g];
                if (i >= 0 && (v > bv || (v == bv && (uint32_t)i < (uint32_t)bi))) {
                    bv = v;
                    bi = i;
                    bg = g;
                }
            }
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const double ov = __shfl_xor(bv, o);
                const int oi = __shfl_xor(bi, o), og = __shfl_xor(bg, o);
                if (oi >= 0 && (ov > bv || (ov == bv && (uint32_t)oi < (uint32_t)bi))) {
                    bv = ov;
                    bi = oi;
                    bg = og;
                }
            }
            if (lane == 0) {
                wbest[wave] = bv;
                widx[wave] = bi;
                wgrp[wave] = bg;
            }
            __syncthreads();
            bv = wbest[0];
            bi = widx[0];
            bg = wgrp[0];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) {
                const double ov = wbest[wv];
                const int oi = widx[wv];
                if (oi >= 0 && (ov > bv || (ov == bv && (uint32_t)oi < (uint32_t)bi))) {
                    bv = ov;
                    bi = oi;
                    bg = wgrp[wv];
                }
            }
            // the first pick is the global maximum; a later one only while it is provably above every other token
            if (t > 0 && !(bv > Vb)) break;
            if (tid < LPR) crow[t][tid] = candrow[bg][tid];
            if (tid == 0) cidx[t] = bi;
            t += 1;
            if (t == kKcBatch || it + t >= kk) break;
            // the leaders against the new center (the picked one drops to 0 by itself)
            {
                const uint4 pc = candrow[bg][col];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int g = grp * U + u;
                    const double dist = exact_dist(candrow[g][col], pc);
                    if (col == 0 && candi[g] >= 0 && dist < candv[g]) candv[g] = dist;
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();
    // unused center rows, then the window (the r most recent tokens, oldest first)
    for (int j = kk + grp; j < c.k; j += RPB) {
        st16(oK + (size_t)j * ROWB + col * 16, make_uint4(0, 0, 0, 0));
        st16(oV + (size_t)j * ROWB + col * 16, make_uint4(0, 0, 0, 0));
        if (col == 0) oidx[j] = -1;
    }
    for (int j = grp; j < c.r; j += RPB) {
        const bool have = j < rwin;
        const size_t src = (size_t)(nold + (have ? j : 0));
        st16(oK + (size_t)(c.k + j) * ROWB + col * 16, have ? ld16(K + src * ROWB + col * 16) : make_uint4(0, 0, 0, 0));
        st16(oV + (size_t)(c.k + j) * ROWB + col * 16, have ? ld16(V + src * ROWB + col * 16) : make_uint4(0, 0, 0, 0));
        if (col == 0) oidx[c.k + j] = have ? (int32_t)src : -1;
    }
    // cluster sizes: how many old tokens ended up nearest to each center
    if (c.out_counts != nullptr) {
        int32_t *oc = c.out_counts + sid * (size_t)c.k;
        for (int base = 0; base < c.k; base += 1024) {
            for (int j = tid; j < 1024; j += kWG) hist[j] = 0;
            __syncthreads();
            for (int r = tid; r < nold; r += kWG) {
                const int a = assign[r] - base;
                if (a >= 0 && a < 1024) atomicAdd(&hist[a], 1);
            }
            __syncthreads();
            for (int j = tid; j < 1024 && base + j < c.k; j += kWG) oc[base + j] = hist[j];
            __syncthreads();
        }
    }
}

}  // namespace sg
