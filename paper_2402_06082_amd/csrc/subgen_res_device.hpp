// Decode step with per-cluster reservoirs (t >= 1): Algorithm 1 of the paper as printed.
//
// Every cluster keeps, beside its representative x_i and count n_i, a reservoir S_i of t keys that are
// uniform samples of the cluster (UpdateSoftmaxNormalizer: on a join each slot is replaced by the new key
// with probability 1/n_i, a new cluster starts with t copies of its key; Lemma 2 (5)), and the softmax
// normaliser is tau = sum_i (n_i / t) sum_{k in S_i} exp(<q, k>) (QueryStreamAttn).  The nearest-center
// search still runs on the representatives only, so the step reads m rows for the update and m*t rows for
// the normaliser; because these are different arrays the update is simply done first and the query scans
// the updated state (no fused single pass as in representative mode).
//
// Generic over dtype and row size (same row mapping as the generic path: LPR lanes per row, 16-byte
// non-temporal loads, four in flight); distances in double precision.
#pragma once
#include "subgen_device.hpp"

namespace sg {

template <int LPR, int G, int VEC>
struct SmemRes {
    alignas(16) uint4 ekrow[LPR], evrow[LPR];
    double wbest[kWaves];
    int widx[kWaves];
    float wmx[kWaves][G], wden[kWaves][G];
    float wacc[kWaves][G][LPR * VEC];
};

template <bool BF16, int LPR, int G, bool UPD, bool ATT>
__device__ __forceinline__ void token_step_res(const State &st, const size_t sid, const char *krow, const char *vrow,
                                               const char *qrows, float *outrows, const int64_t n_seen, int &m,
                                               double &mu, SmemRes<LPR, G, (BF16 ? 8 : 4)> &sm)
{
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)LPR * 16;
    constexpr int U = kUnroll;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR;
    const int T = st.t;

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    char *const R = st.R + sid * (size_t)st.Mcap * T * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;

    if constexpr (UPD) {
        // ---- window push; the token that leaves the window is the one that is compressed
        bool evict = false;
        int64_t etoken = 0;
        uint4 ek = make_uint4(0, 0, 0, 0), ev = make_uint4(0, 0, 0, 0);
        const char *esk = krow, *esv = vrow;
        char *kw = nullptr, *vw = nullptr;
        const Eviction wp = window_push(n_seen, st.w);
        evict = wp.evict;
        etoken = wp.token;
        if (wp.slot >= 0) {
            kw = Kw + (size_t)wp.slot * ROWB;
            vw = Vw + (size_t)wp.slot * ROWB;
            esk = kw;
            esv = vw;
        }
        if (evict) {
            ek = ld16(esk + col * 16);
            ev = ld16(esv + col * 16);
            if (tid < LPR) {
                sm.ekrow[tid] = ek;
                sm.evrow[tid] = ev;
            }
        }
        __syncthreads();  // every lane holds the evicted row (registers, LDS) before the slot is overwritten
        if (st.w > 0 && tid < LPR) {
            st16(kw + tid * 16, ld16(krow + tid * 16));
            st16(vw + tid * 16, ld16(vrow + tid * 16));
        }
        float ekf[VEC];
        unpack<BF16>(ek, ekf);
        double kk2 = 0.0;   // ||k'||^2
        float vn = 0.f;     // ||v'||^2
        {
            float evf[VEC];
            unpack<BF16>(ev, evf);
            double vv2 = 0.0;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                kk2 = fma((double)ekf[v], (double)ekf[v], kk2);
                vv2 = fma((double)evf[v], (double)evf[v], vv2);
            }
            kk2 = group_sum<LPR>(kk2);
            vn = (float)group_sum<LPR>(vv2);
            if (evict && !token_is_finite((float)kk2, vn)) {   // NaN or Inf in the token: dropped and flagged
                evict = false;
                if (tid == 0) st.flags[sid] |= 2u;
            }
        }
        if (evict) {
            // ---- nearest representative in double precision (lowest index on ties)
            double best = INFINITY;
            int bidx = -1;
            for (int r0 = wave * RPW; r0 < m; r0 += RPB * U) {
                uint4 raw[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RPB + sub;
                    raw[u] = ldnt16(X + (size_t)(r < m ? r : m - 1) * ROWB + col * 16);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RPB + sub;
                    float x[VEC];
                    unpack<BF16>(raw[u], x);
                    double dist = 0.0;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const double df = (double)x[v] - (double)ekf[v];
                        dist = fma(df, df, dist);
                    }
                    dist = group_sum<LPR>(dist);
                    if (r < m && dist < best) {
                        best = dist;
                        bidx = r;
                    }
                }
            }
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) {
                const double ob = __shfl_xor(best, o);
                const int oi = __shfl_xor(bidx, o);
                if (ob < best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
                    best = ob;
                    bidx = oi;
                }
            }
            if (lane == 0) {
                sm.wbest[wave] = best;
                sm.widx[wave] = bidx;
            }
            __syncthreads();
            best = sm.wbest[0];
            bidx = sm.widx[0];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) {
                const double ob = sm.wbest[wv];
                const int oi = sm.widx[wv];
                if (ob < best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
                    best = ob;
                    bidx = oi;
                }
            }
            // ---- join (count bump + reservoir coins) or open a cluster (t copies of the key)
            const bool join = bidx >= 0 && best <= st.delta2;
            const Decision dec = decide_cluster(join, bidx, m, st.Mcap);
            const bool forced = dec.forced, created = dec.created;
            const int target = dec.target;
            const int nnew = created ? 1 : cnt[target] + 1;   // read by every lane before lane 0 writes it
            __syncthreads();
            if (tid == 0) {
                cnt[target] = nnew;
                if (created) st.xn[sid * (size_t)st.McapS + m] = (float)kk2;
                if (forced) st.flags[sid] |= 1u;
                if (st.assign != nullptr && etoken < st.assign_cap) st.assign[sid * (size_t)st.assign_cap + etoken] = target;
            }
            if (created && tid < LPR) st16(X + (size_t)m * ROWB + tid * 16, ek);
            {
                const float pr = 1.0f / (float)nnew;   // 1 for a new cluster: every slot takes the key
                for (int j0 = tid * 4; j0 < T; j0 += kWG * 4) {
                    uint32_t r[4];
                    coin_block(st, sid, etoken, (uint32_t)(j0 >> 2), true, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int j = j0 + i;
                        if (j < T && (created || coin_accepts(r[i], pr))) {
                            for (int ch = 0; ch < LPR; ++ch)
                                st16(R + ((size_t)target * T + j) * ROWB + ch * 16, sm.ekrow[ch]);
                        }
                    }
                }
            }
            if (created) m += 1;

            // ---- sampling update: p from the old mu, one coin per slot, then mu += ||v||^2
            const float p = coin_probability(mu, vn);
            if (p > 0.f) {
                for (int j0 = tid * 4; j0 < st.s; j0 += kWG * 4) {
                    uint32_t r[4];
                    coin_block(st, sid, etoken, (uint32_t)(j0 >> 2), false, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int j = j0 + i;
                        if (j < st.s && coin_accepts(r[i], p)) {
                            for (int ch = 0; ch < LPR; ++ch) {
                                st16(Ks + (size_t)j * ROWB + ch * 16, sm.ekrow[ch]);
                                st16(Vs + (size_t)j * ROWB + ch * 16, sm.evrow[ch]);
                            }
                            st.sidx[sid * (size_t)st.sS + j] = (int32_t)etoken;
                            st.svn[sid * (size_t)st.sS + j] = vn;
                        }
                    }
                }
            }
            mu += (double)vn;
        }
        __syncthreads();  // window slot, cluster rows, reservoirs and sample rows are visible to the workgroup
    }

    if constexpr (ATT) {
        const int64_t n_after = UPD ? n_seen + 1 : n_seen;
        const int64_t n_evicted_after = st.w == 0 ? n_after : (n_after > st.w ? n_after - st.w : 0);
        float q[G][VEC];
#pragma unroll
        for (int g = 0; g < G; ++g) unpack<BF16>(ld16(qrows + (size_t)g * ROWB + col * 16), q[g]);
        Partial<VEC> part[G];
#pragma unroll
        for (int g = 0; g < G; ++g) part[g].init();

        // ---- reservoirs: tau terms (n_i / t) e^{<q, k>} for the t sampled keys of every cluster
        {
            const int nrows = m * T;
            const float invt = 1.0f / (float)T;
            for (int r0 = wave * RPW; r0 < nrows; r0 += RPB * U) {
                uint4 raw[U];
                float cf[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RPB + sub;
                    const int rr = r < nrows ? r : nrows - 1;
                    raw[u] = ldnt16(R + (size_t)rr * ROWB + col * 16);
                    cf[u] = (float)cnt[rr / T] * invt;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool valid = r0 + u * RPB + sub < nrows;
                    float x[VEC];
                    unpack<BF16>(raw[u], x);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        float a = 0.f;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) a = fmaf(q[g][v], x[v], a);
                        const float b = group_sum<LPR>(a);
                        if (valid) {
                            part[g].raise(b);
                            part[g].den = fmaf(cf[u], __expf(b - part[g].mx), part[g].den);
                        }
                    }
                }
            }
        }
        // ---- rows with values: sampled pairs (importance weights, numerator only), then the window
        auto scan = [&](const char *Kb, const char *Vb, const float *vnorm, const float wmul, const int nrows,
                        const bool to_den) __attribute__((always_inline)) {
            for (int r0 = wave * RPW; r0 < nrows; r0 += RPB * U) {
                uint4 rk[U], rv[U];
                float vnj[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int r = r0 + u * RPB + sub;
                    const int rr = r < nrows ? r : nrows - 1;
                    rk[u] = ldnt16(Kb + (size_t)rr * ROWB + col * 16);
                    rv[u] = ldnt16(Vb + (size_t)rr * ROWB + col * 16);
                    vnj[u] = vnorm != nullptr ? vnorm[rr] : 1.f;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool valid = r0 + u * RPB + sub < nrows;
                    float kx[VEC], vx[VEC];
                    unpack<BF16>(rk[u], kx);
                    unpack<BF16>(rv[u], vx);
                    const float wgt = vnorm != nullptr ? (vnj[u] > 0.f ? wmul / vnj[u] : 0.f) : 1.f;
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        float a = 0.f;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) a = fmaf(q[g][v], kx[v], a);
                        const float b = group_sum<LPR>(a);
                        if (valid) {
                            part[g].raise(b);
                            const float e = wgt * __expf(b - part[g].mx);
                            if (to_den) part[g].den += e;
#pragma unroll
                            for (int v = 0; v < VEC; ++v) part[g].acc[v] = fmaf(e, vx[v], part[g].acc[v]);
                        }
                    }
                }
            }
        };
        if (n_evicted_after > 0)
            scan(Ks, Vs, st.svn + sid * (size_t)st.sS, (float)(mu / (double)st.s), st.s, false);
        scan(Kw, Vw, nullptr, 1.f, (int)(n_after < st.w ? n_after : st.w), true);

        // ---- merge row groups inside the wavefront, then the wavefronts through LDS
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) {
                const float omx = __shfl_xor(part[g].mx, o);
                const float oden = __shfl_xor(part[g].den, o);
                float oacc[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) oacc[v] = __shfl_xor(part[g].acc[v], o);
                part[g].merge(omx, oden, oacc);
            }
            if (sub == 0) {
                if (col == 0) {
                    sm.wmx[wave][g] = part[g].mx;
                    sm.wden[wave][g] = part[g].den;
                }
#pragma unroll
                for (int v = 0; v < VEC; ++v) sm.wacc[wave][g][col * VEC + v] = part[g].acc[v];
            }
        }
        __syncthreads();
        const int d = LPR * VEC;
        for (int i = tid; i < G * d; i += kWG) {
            const int g = i / d, c = i % d;
            float M = sm.wmx[0][g];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) M = fmaxf(M, sm.wmx[wv][g]);
            float den = 0.f, num = 0.f;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) {
                const float wm = sm.wmx[wv][g];
                const float sc = (wm == -INFINITY) ? 0.f : __expf(wm - M);
                den = fmaf(sm.wden[wv][g], sc, den);
                num = fmaf(sm.wacc[wv][g][c], sc, num);
            }
            put_out(st, outrows, (size_t)g * d + c, num / den);
        }
    }
    __syncthreads();  // LDS and state are reusable by the next token
}

// n_tokens == 1 with Q: update / attend / step; n_tokens >= 1 without Q: prefix ingest (token loop)
template <bool BF16, int LPR, int G, bool UPD, bool ATT>
__global__ __launch_bounds__(kWG) void decode_res_kernel(const State st, const Call call)
{
    constexpr int VEC = BF16 ? 8 : 4;
    __shared__ SmemRes<LPR, G, VEC> sm;
    const size_t sid = blockIdx.x;
    int m = st.m[sid];
    double mu = st.mu[sid];
    const char *kbase = UPD ? call.K + sid * call.stream_stride : nullptr;
    const char *vbase = UPD ? call.V + sid * call.stream_stride : nullptr;
    const char *qrows = ATT ? call.Q + sid * call.q_stride : nullptr;
    float *outrows = ATT ? out_rows(st, call.out, sid * call.out_stride) : nullptr;
    const int64_t nt = UPD ? call.n_tokens : 1;
    const int64_t n0 = tokens_seen(st, call.n_seen);
    for (int64_t t = 0; t < nt; ++t)
        token_step_res<BF16, LPR, G, UPD, ATT>(st, sid, UPD ? kbase + t * call.token_stride : nullptr,
                                               UPD ? vbase + t * call.token_stride : nullptr, qrows, outrows,
                                               n0 + t, m, mu, sm);
    if constexpr (UPD) {
        if (threadIdx.x == 0) {
            st.m[sid] = m;
            st.mu[sid] = mu;
        }
    }
}

}  // namespace sg
