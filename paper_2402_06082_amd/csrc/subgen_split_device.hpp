// Decode step for contexts with fewer streams than the chip has compute units (gfx950).
//
// With one workgroup per stream a context of a few streams leaves most of the chip idle and one stream's step
// is bound by what a single workgroup can keep in flight.  Here P workgroups share one stream: workgroup p scans
// every P-th block of rows of the three sections of the state (representatives, sampled pairs, window) and
// leaves a partial result in device memory: online-softmax partials (maximum, normaliser, numerator) of its rows
// and its nearest representative (squared distance in double, index, scores).  The workgroup that arrives last
// (one counter per stream) combines the P partials in the fixed order p = 0 .. P-1, so the result does not depend
// on which workgroup that is, takes the clustering decision of Algorithm 1 (UpdateSoftmaxNormalizer) and does
// every write that other workgroups must not see earlier: the new representative or the count bump, the ring
// slot of the new token, mu, the outputs.  No floating-point atomics anywhere.
//
// The sampling update (UpdateMatrixProduct) needs no combine: the coin of slot j depends only on (seed, stream,
// token, j) and on p = ||v||^2 / (mu + ||v||^2), which every workgroup computes for itself; the workgroup that
// scans slot j draws its coin, overwrites the slot if it wins and, in the same step, scores the slot with the
// rows it has just been given.  The ring slot of the new token is likewise read from the call's input rows.
//
// Distances are evaluated in double precision from the exactly converted elements (every workgroup has only
// m / P rows to look at), so decisions equal those of the other kernel families bit for bit.
#pragma once
#include "subgen_device.hpp"

namespace sg {

// floats per partial of one (stream, workgroup): per query (max, normaliser, numerator[d]), then the nearest
// representative: squared distance (double), index, per-query score; rounded up to 16 bytes
__host__ __device__ constexpr int split_partial_floats(int G, int D) { return (G * (D + 2) + 2 + 1 + G + 3) / 4 * 4; }

template <int LPR, int G, int VEC>
struct SmemSplit {
    double wbest[kWaves];
    int widx[kWaves];
    float wbsc[kWaves][G];
    float wmx[kWaves][G], wden[kWaves][G];
    float wacc[kWaves][G][LPR * VEC];
    int last;
};

template <bool BF16, int LPR, int G, bool UPD, bool ATT>
__global__ __launch_bounds__(kWG) void decode_split_kernel(const State st, const Call call)
{
    constexpr int VEC = BF16 ? 8 : 4, D = LPR * VEC;
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)LPR * 16;
    constexpr int U = 4;                                  // row blocks in flight per lane
    constexpr int PF = split_partial_floats(G, D);
    constexpr int OFF_BEST = G * (D + 2), OFF_IDX = OFF_BEST + 2, OFF_BSC = OFF_IDX + 1;
    __shared__ SmemSplit<LPR, G, VEC> sm;

    const int P = st.split_P;
    const size_t sid = blockIdx.x / (unsigned)P;
    const int p = (int)(blockIdx.x % (unsigned)P);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR, grp = wave * RPW + sub;

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;
    float *const mine = st.split_part + (sid * (size_t)P + p) * PF;

    const int64_t n_seen = tokens_seen(st, call.n_seen);
    const int m = st.m[sid];
    const double mu = st.mu[sid];

    // ---- window push: the new token's rows stay in registers (the last workgroup writes the ring slot), the
    //      token that leaves the window is the one that is compressed
    bool evict = false;
    int64_t etoken = 0;
    int wslot = -1;
    uint4 ek = make_uint4(0, 0, 0, 0), ev = make_uint4(0, 0, 0, 0), kn = ek, vnw = ek;
    if constexpr (UPD) {
        kn = ld16(call.K + sid * call.stream_stride + col * 16);
        vnw = ld16(call.V + sid * call.stream_stride + col * 16);
        const Eviction e = window_push(n_seen, st.w);
        evict = e.evict;
        etoken = e.token;
        wslot = e.slot;
        if (wslot < 0) {
            ek = kn;
            ev = vnw;
        } else if (evict) {
            ek = ld16(Kw + (size_t)wslot * ROWB + col * 16);
            ev = ld16(Vw + (size_t)wslot * ROWB + col * 16);
        }
    }
    const int64_t n_after = UPD ? n_seen + 1 : n_seen;
    const int64_t n_evicted_after = st.w == 0 ? n_after : (n_after > st.w ? n_after - st.w : 0);
    const int fill = (int)(n_after < st.w ? n_after : st.w);

    float q[G][VEC];
    if constexpr (ATT) {
#pragma unroll
        for (int g = 0; g < G; ++g) unpack<BF16>(ld16(call.Q + sid * call.q_stride + (size_t)g * ROWB + col * 16), q[g]);
    }

    // ---- one stream's step is a chain of memory round trips, so the first batch of every section is requested
    //      here, before anything is waited for: the representatives without knowing how many there are (rows past
    //      the table are allocated, they are masked once m has arrived), the sample slots, the window
    const float *const svn = st.svn + sid * (size_t)st.sS;
    const bool want_c = ATT || (UPD && evict);
    const bool scan_s = ATT && n_evicted_after > 0;
    const bool scan_w = ATT && fill > 0;
    uint4 craw[U], srk[U], srv[U], wrk[U], wrv[U];
    float ccf[U], svj[U];
    auto c_issue = [&](const int b0, const int bound) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = (b0 + u * P) * RPB + grp;
            const int rr = r < bound ? r : bound - 1;
            craw[u] = ldnt16(X + (size_t)rr * ROWB + col * 16);
            if constexpr (ATT) ccf[u] = (float)cnt[rr];
        }
    };
    auto s_issue = [&](const int b0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = (b0 + u * P) * RPB + grp;
            const int rr = r < st.s ? r : st.s - 1;
            srk[u] = ldnt16(Ks + (size_t)rr * ROWB + col * 16);
            srv[u] = ldnt16(Vs + (size_t)rr * ROWB + col * 16);
            svj[u] = svn[rr];
        }
    };
    auto w_issue = [&](const int b0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = (b0 + u * P) * RPB + grp;
            const int rr = r < fill ? r : fill - 1;
            wrk[u] = ldnt16(Kw + (size_t)rr * ROWB + col * 16);
            wrv[u] = ldnt16(Vw + (size_t)rr * ROWB + col * 16);
        }
    };
    if (want_c) c_issue(p, st.Mcap);
    if (scan_s) s_issue(p);
    if (scan_w) w_issue(p);

    double ekd[VEC];
    double kk2 = 0.0;   // ||k'||^2
    float vn = 0.f;     // ||v'||^2
    float bnew[G];      // <q, evicted key>: score of the cluster this token would open
    bool dropped = false;
    if constexpr (UPD) {
        float ekf[VEC], evf[VEC];
        unpack<BF16>(ek, ekf);
        unpack<BF16>(ev, evf);
        double vv2 = 0.0;
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            ekd[v] = (double)ekf[v];
            kk2 = fma(ekd[v], ekd[v], kk2);
            vv2 = fma((double)evf[v], (double)evf[v], vv2);
        }
        kk2 = group_sum<LPR>(kk2);
        vn = (float)group_sum<LPR>(vv2);
        if (evict && !token_is_finite((float)kk2, vn)) {   // NaN or Inf: the token is dropped
            evict = false;
            dropped = true;
        }
        if constexpr (ATT) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float a = 0.f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) a = fmaf(q[g][v], ekf[v], a);
                bnew[g] = group_sum<LPR>(a);
            }
        }
    }
    // coin probability from the mu before this token; mu after it (the weight of the sampled pairs uses that)
    const float pcoin = evict ? coin_probability(mu, vn) : 0.f;
    const double mu_after = evict ? mu + (double)vn : mu;

    Partial<VEC> part[G];
#pragma unroll
    for (int g = 0; g < G; ++g) part[g].init();

    // ---- this workgroup's blocks of the representatives: squared distance to the evicted key (double) and
    //      count-weighted exp(<q, x_i>) for the softmax normaliser
    double best = INFINITY;
    int bidx = -1;
    float bsc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) bsc[g] = 0.f;
    auto c_consume = [&](const int b0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = (b0 + u * P) * RPB + grp;
            const bool valid = r < m;
            float x[VEC];
            unpack<BF16>(craw[u], x);
            double dist = 0.0;
            if constexpr (UPD) {
                if (evict) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const double df = (double)x[v] - ekd[v];
                        dist = fma(df, df, dist);
                    }
                    dist = group_sum<LPR>(dist);
                }
            }
            float b[G];
            if constexpr (ATT) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float a = 0.f;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) a = fmaf(q[g][v], x[v], a);
                    b[g] = group_sum<LPR>(a);
                    if (valid) {
                        part[g].raise(b[g]);
                        part[g].den += ccf[u] * __expf(b[g] - part[g].mx);
                    }
                }
            }
            if constexpr (UPD) {
                if (evict && valid && dist < best) {   // rows come in ascending order: the lowest index stays on ties
                    best = dist;
                    bidx = r;
                    if constexpr (ATT) {
#pragma unroll
                        for (int g = 0; g < G; ++g) bsc[g] = b[g];
                    }
                }
            }
        }
    };
    if ((UPD && evict) || ATT) {
        c_consume(p);   // the batch requested above; rows at or past m are masked
        for (int b0 = p + P * U; b0 * RPB < m; b0 += P * U) {
            c_issue(b0, m);
            c_consume(b0);
        }
    }

    // ---- this workgroup's blocks of the sample slots: the coin of every slot (UpdateMatrixProduct) and, for a
    //      query, the numerator terms  mu / (s ||v_j||^2) e^{<q,k_j>} v_j  of the slot as it is after the update
    if ((UPD && pcoin > 0.f) || scan_s) {
        const float wmul = (float)(mu_after / (double)st.s);
        for (int b0 = p; b0 * RPB < st.s; b0 += P * U) {
            if (scan_s && b0 != p) s_issue(b0);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = (b0 + u * P) * RPB + grp;
                const bool valid = r < st.s;
                bool take = false;
                if constexpr (UPD) {
                    if (valid && pcoin > 0.f) {
                        uint32_t rnd[4];
                        coin_block(st, sid, etoken, (uint32_t)(r >> 2), false, rnd);
                        const uint32_t word = (r & 3) == 0 ? rnd[0] : (r & 3) == 1 ? rnd[1] : (r & 3) == 2 ? rnd[2] : rnd[3];
                        take = coin_accepts(word, pcoin);
                        if (take) {
                            st16(Ks + (size_t)r * ROWB + col * 16, ek);
                            st16(Vs + (size_t)r * ROWB + col * 16, ev);
                            if (col == 0) {
                                st.sidx[sid * (size_t)st.sS + r] = (int32_t)etoken;
                                st.svn[sid * (size_t)st.sS + r] = vn;
                            }
                        }
                    }
                }
                if (scan_s) {
                    float kx[VEC], vx[VEC];
                    unpack<BF16>(take ? ek : srk[u], kx);
                    unpack<BF16>(take ? ev : srv[u], vx);
                    const float vnr = take ? vn : svj[u];
                    const float wgt = vnr > 0.f ? wmul / vnr : 0.f;
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        float a = 0.f;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) a = fmaf(q[g][v], kx[v], a);
                        const float b = group_sum<LPR>(a);
                        if (valid) {
                            part[g].raise(b);
                            const float e = wgt * __expf(b - part[g].mx);
#pragma unroll
                            for (int v = 0; v < VEC; ++v) part[g].acc[v] = fmaf(e, vx[v], part[g].acc[v]);
                        }
                    }
                }
            }
        }
    }

    // ---- this workgroup's blocks of the window: exact terms in numerator and normaliser; the slot of the new
    //      token still holds the evicted one in memory, so its rows are the call's input rows
    if constexpr (ATT) {
        for (int b0 = p; b0 * RPB < fill; b0 += P * U) {
            if (b0 != p) w_issue(b0);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = (b0 + u * P) * RPB + grp;
                const bool valid = r < fill;
                const bool fresh = UPD && r == wslot;
                float kx[VEC], vx[VEC];
                unpack<BF16>(fresh ? kn : wrk[u], kx);
                unpack<BF16>(fresh ? vnw : wrv[u], vx);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float a = 0.f;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) a = fmaf(q[g][v], kx[v], a);
                    const float b = group_sum<LPR>(a);
                    if (valid) {
                        part[g].raise(b);
                        const float e = __expf(b - part[g].mx);
                        part[g].den += e;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) part[g].acc[v] = fmaf(e, vx[v], part[g].acc[v]);
                    }
                }
            }
        }
    }

    // ---- the workgroup's partial: row groups of a wavefront by shuffles, wavefronts through LDS, then one copy
    //      in device memory
    if constexpr (UPD) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) {
            const double ob = __shfl_xor(best, o);
            const int oi = __shfl_xor(bidx, o);
            float osc[G];
#pragma unroll
            for (int g = 0; g < G; ++g) osc[g] = __shfl_xor(bsc[g], o);
            if (ob < best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
                best = ob;
                bidx = oi;
#pragma unroll
                for (int g = 0; g < G; ++g) bsc[g] = osc[g];
            }
        }
        if (lane == 0) {
            sm.wbest[wave] = best;
            sm.widx[wave] = bidx;
#pragma unroll
            for (int g = 0; g < G; ++g) sm.wbsc[wave][g] = bsc[g];
        }
    }
    if constexpr (ATT) {
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
    }
    __syncthreads();
    if constexpr (UPD) {
        if (tid == 0) {
            double wb = sm.wbest[0];
            int wi = sm.widx[0], bw = 0;
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) {
                const double ob = sm.wbest[wv];
                const int oi = sm.widx[wv];
                if (ob < wb || (ob == wb && (uint32_t)oi < (uint32_t)wi)) {
                    wb = ob;
                    wi = oi;
                    bw = wv;
                }
            }
            __hip_atomic_store(reinterpret_cast<double *>(mine + OFF_BEST), wb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(reinterpret_cast<int *>(mine + OFF_IDX), wi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int g = 0; g < G; ++g)
                __hip_atomic_store(mine + OFF_BSC + g, sm.wbsc[bw][g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if constexpr (ATT) {
        for (int i = tid; i < G * (D + 2); i += kWG) {
            const int g = i / (D + 2), e = i % (D + 2);
            float M = sm.wmx[0][g];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) M = fmaxf(M, sm.wmx[wv][g]);
            float val = M;
            if (e >= 1) {
                val = 0.f;
#pragma unroll
                for (int wv = 0; wv < kWaves; ++wv) {
                    const float wm = sm.wmx[wv][g];
                    const float sc = (wm == -INFINITY) ? 0.f : __expf(wm - M);
                    val = fmaf(e == 1 ? sm.wden[wv][g] : sm.wacc[wv][g][e - 2], sc, val);
                }
            }
            __hip_atomic_store(mine + (size_t)g * (D + 2) + e, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- arrival.  The partial is written with device-scope atomic stores (they go through to the level of the
    //      memory system that all workgroups share) and read back with device-scope atomic loads, so no cache has
    //      to be written back or invalidated as a whole: it is enough that every lane's stores have been
    //      acknowledged before the stream's counter is bumped.  The workgroup that brings it to P goes on alone.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) sm.last = atomicAdd(&st.split_cnt[sid], 1u) == (unsigned)(P - 1);
    __syncthreads();
    if (!sm.last) return;
    const float *const all = st.split_part + sid * (size_t)P * PF;
    auto ldf = [&](size_t i) { return __hip_atomic_load(all + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };

    // ---- requests first: lane l of every wavefront fetches the nearest-representative candidate of workgroup
    //      l, every output lane the first eight softmax partials of its column
    constexpr int CH = 8;   // partials merged per batch of loads
    double cb = INFINITY;
    int ci = -1;
    float csc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) csc[g] = 0.f;
    if constexpr (UPD) {
        if (evict && lane < P) {
            cb = __hip_atomic_load(reinterpret_cast<const double *>(all + (size_t)lane * PF + OFF_BEST), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            ci = __hip_atomic_load(reinterpret_cast<const int *>(all + (size_t)lane * PF + OFF_IDX), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            if constexpr (ATT) {
#pragma unroll
                for (int g = 0; g < G; ++g) csc[g] = ldf((size_t)lane * PF + OFF_BSC + g);
            }
        }
    }
    constexpr int NI = (G * D + kWG - 1) / kWG;   // (query, column) pairs per output lane
    float pm[NI][CH], pd[NI][CH], pn[NI][CH];
    auto fetch = [&](const int k, const int i, const int pp0) __attribute__((always_inline)) {
        const int g = i / D, c = i % D;
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int pp = pp0 + j < P ? pp0 + j : P - 1;
            const size_t o = (size_t)pp * PF + (size_t)g * (D + 2);
            pm[k][j] = ldf(o);
            pd[k][j] = ldf(o + 1);
            pn[k][j] = ldf(o + 2 + c);
        }
    };
    if constexpr (ATT) {
#pragma unroll
        for (int k = 0; k < NI; ++k)
            if (tid + k * kWG < G * D) fetch(k, tid + k * kWG, 0);
    }

    // ---- clustering decision from the P candidates (smallest distance, lowest index on ties; a 64-lane
    //      reduction whose result does not depend on the order)
    bool extra = false, created = false;
    int gm = m;
    float bx[G];
#pragma unroll
    for (int g = 0; g < G; ++g) bx[g] = 0.f;
    if constexpr (UPD) {
        if (evict) {
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const double ob = __shfl_xor(cb, o);
                const int oi = __shfl_xor(ci, o);
                float osc[G];
#pragma unroll
                for (int g = 0; g < G; ++g) osc[g] = __shfl_xor(csc[g], o);
                if (ob < cb || (ob == cb && (uint32_t)oi < (uint32_t)ci)) {
                    cb = ob;
                    ci = oi;
#pragma unroll
                    for (int g = 0; g < G; ++g) csc[g] = osc[g];
                }
            }
            const double gb = cb;
            int gi = ci;
            // join iff ||k - x_i*||^2 <= delta^2, else open a cluster (or force-join when the table is full)
            const bool join = gi >= 0 && gb <= st.delta2;
            const Decision dec = decide_cluster(join, gi, m, st.Mcap);
            const bool forced = dec.forced;
            created = dec.created;
            const int target = dec.target;
            if (created) {
                if (tid < LPR) st16(X + (size_t)m * ROWB + tid * 16, ek);   // lane tid < LPR holds chunk tid of the row
                if (tid == 0) {
                    cnt[m] = 1;
                    st.xn[sid * (size_t)st.McapS + m] = (float)kk2;
                }
                gm = m + 1;
            } else if (tid == 0) {
                cnt[target] += 1;
                if (forced) st.flags[sid] |= 1u;
            }
            if (tid == 0 && st.assign != nullptr && etoken < st.assign_cap)
                st.assign[sid * (size_t)st.assign_cap + etoken] = target;
            if constexpr (ATT) {
                extra = true;   // the count bump (or the new cluster) adds one more term to the normaliser
#pragma unroll
                for (int g = 0; g < G; ++g) bx[g] = created ? bnew[g] : csc[g];
            }
        }
        if (tid == 0) {
            st.m[sid] = gm;
            st.mu[sid] = mu_after;
            if (dropped) st.flags[sid] |= 2u;
        }
        if (wslot >= 0 && tid < LPR) {   // the new token enters the ring
            st16(Kw + (size_t)wslot * ROWB + tid * 16, kn);
            st16(Vw + (size_t)wslot * ROWB + tid * 16, vnw);
        }
    }

    // ---- outputs: the extra normaliser term, then the P softmax partials in the order p = 0 .. P-1
    if constexpr (ATT) {
        float *const outrows = out_rows(st, call.out, sid * call.out_stride);
#pragma unroll
        for (int k = 0; k < NI; ++k) {
            const int i = tid + k * kWG;
            if (i < G * D) {
                const int g = i / D;
                float M = extra ? bx[g] : -INFINITY, den = extra ? 1.f : 0.f, num = 0.f;
                for (int pp0 = 0; pp0 < P; pp0 += CH) {
                    if (pp0 > 0) fetch(k, i, pp0);
#pragma unroll
                    for (int j = 0; j < CH; ++j) {
                        const float wm = pm[k][j];
                        if (pp0 + j < P && wm != -INFINITY) {
                            if (wm > M) {
                                const float sc = __expf(M - wm);   // M = -inf gives 0
                                den *= sc;
                                num *= sc;
                                M = wm;
                            }
                            const float f = __expf(wm - M);
                            den = fmaf(pd[k][j], f, den);
                            num = fmaf(pn[k][j], f, num);
                        }
                    }
                }
                put_out(st, outrows, (size_t)i, num / den);
            }
        }
    }
    if (tid == 0) st.split_cnt[sid] = 0u;   // ready for the next launch
}

}  // namespace sg
