// Single-query decode step for bf16 rows of 128 elements (gfx950).
//
// With one query per stream the step is a pure stream over the state, so what matters is the shape of the
// loads and the number of vector-ALU instructions per byte:
//   - a row is read by 16 consecutive lanes with one 16-byte non-temporal load each, so every wavefront load
//     is one contiguous 1 KB piece of memory (four whole rows), four loads in flight per lane;
//   - dot products run on packed bf16 pairs (v_dot2c_f32_bf16: two multiply-adds per instruction, no
//     unpacking of key rows) and are reduced over the 16 lanes of a row with DPP row rotations (no LDS);
//   - the softmax reference is raised lazily, so accumulators are almost never rescaled.
// Nearest-center decisions stay exact the same way as on the matrix-core path: approximate squared distances
// D~ = ||x||^2 + ||k||^2 - 2<x,k> decide only when the best/runner-up gap and |D~ - delta^2| exceed their error
// bound; otherwise the workgroup re-evaluates all distances in double precision.
#pragma once
#include "subgen_mfma_device.hpp"

namespace sg {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ float dot8_bf16(const uint4 &x, const uint4 &y)
{
    float s = dot2_bf16(x.x, y.x, 0.f);
    s = dot2_bf16(x.y, y.y, s);
    s = dot2_bf16(x.z, y.z, s);
    return dot2_bf16(x.w, y.w, s);
}

template <int NW>
struct SmemDot2 {
    alignas(16) uint4 ekrow[16], evrow[16];   // the evicted (key, value) rows, for the sampling copies
    alignas(16) uint4 nkrow[16], nvrow[16];   // the new token's rows (they enter the ring at the end of the step)
    uint32_t accm[NW == 8 ? 256 : 1];         // slots that took the evicted token in this step (hoisted variant)
    float wb1[NW], wb2[NW], wb3[NW], wnx[NW];
    int wi1[NW], wi2[NW];
    double wbest[NW];
    int widx[NW];
    float bx;
    float wmx[NW], wden[NW];
    float wacc[NW][128];
};

template <bool UPD, bool ATT, int NW>
__device__ __forceinline__ void token_step_dot2(const State &st, const size_t sid, const char *krow, const char *vrow,
                                                const char *qrow, float *outrow, const int64_t n_seen, int &m,
                                                double &mu, SmemDot2<NW> &sm)
{
    constexpr int LPR = 16, RPW = 4, RPB = RPW * NW, WG = NW * 64;
    constexpr size_t ROWB = 256;
    constexpr int U = 8;   // row loads in flight per lane (8 measured slightly better than 4; 2 is 8 % slower)
    // Few streams (NW = 8, 512 lanes): one stream's step is a chain of memory round trips, so the first batch of
    // every kind of row is requested before anything is consumed: 10 representative rows, 8 sampled pairs and 2
    // window pairs per lane (320 + 256 + 64 rows per workgroup) are in flight together.
    constexpr bool WIDE = NW == 8;
    constexpr int UC = WIDE ? 10 : U;   // representative rows in flight per lane
    constexpr int UW = WIDE ? 2 : U;    // window pairs of the hoisted first batch
    constexpr int kAccWords = 256;      // accepted-slot mask of the hoisted variant: sample budgets up to 8192
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, sub = lane >> 4;

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    float *const xn = st.xn + sid * (size_t)st.McapS;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;

    uint4 qp = make_uint4(0, 0, 0, 0);   // this lane's 8 packed query elements
    if constexpr (ATT) qp = ld16(qrow + col * 16);

    // ---- window push; the token that leaves the window is the one that is compressed.  The new token's rows
    //      are parked in LDS: the ring slot in HBM is rewritten at the very end of the step (nothing has to wait
    //      for that store) and the window scan takes the slot's rows out of LDS instead.
    bool evict = false;
    int64_t etoken = 0;
    int wslot = -1;
    uint4 ek = make_uint4(0, 0, 0, 0), ev = make_uint4(0, 0, 0, 0);
    float nk = 0.f, vn = 0.f;
    if constexpr (UPD) {
        const char *esk = krow, *esv = vrow;
        const Eviction wp = window_push(n_seen, st.w);
        evict = wp.evict;
        etoken = wp.token;
        wslot = wp.slot;
        if (wslot >= 0) {
            esk = Kw + (size_t)wslot * ROWB;
            esv = Vw + (size_t)wslot * ROWB;
        }
        if (evict) {
            ek = ld16(esk + col * 16);
            ev = ld16(esv + col * 16);
        }
        if (st.w > 0 && tid < LPR) {
            sm.nkrow[tid] = ld16(krow + tid * 16);
            sm.nvrow[tid] = ld16(vrow + tid * 16);
        }
    }
    // the evicted rows are consumed only after the first rows of the representatives have been requested
    auto take_evicted = [&]() __attribute__((always_inline)) {
        if constexpr (UPD) {
            if (!evict) return;
            if (tid < LPR) {
                sm.ekrow[tid] = ek;
                sm.evrow[tid] = ev;
            }
            // ||k'||^2 and ||v'||^2 in double from the exactly converted elements
            float ekf[8], evf[8];
            unpack<true>(ek, ekf);
            unpack<true>(ev, evf);
            double a = 0.0, b = 0.0;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                a = fma((double)ekf[v], (double)ekf[v], a);
                b = fma((double)evf[v], (double)evf[v], b);
            }
            nk = (float)group_sum<LPR>(a);
            vn = (float)group_sum<LPR>(b);
            if (!token_is_finite(nk, vn)) {   // NaN or Inf in the token: it is dropped and flagged
                evict = false;
                if (tid == 0) st.flags[sid] |= 2u;
            }
        }
    };
    const int64_t n_after = UPD ? n_seen + 1 : n_seen;
    const int64_t n_evicted_after = st.w == 0 ? n_after : (n_after > st.w ? n_after - st.w : 0);

    // online softmax of this lane's row group: lazily raised reference, denominator, 8 output columns
    float mx = -INFINITY, den = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;

    // ---- one pass over the representatives: approximate squared distance to the evicted key and
    //      count-weighted exp(<q, x_i>) for the softmax normaliser
    Cand3 cd;   // nearest representatives of the evicted key by approximate distance
    float nxmax = 0.f;
    // (key, value) row pairs: request a batch into registers / consume it (sampled pairs and window)
    const float *const svn_base = st.svn + sid * (size_t)st.sS;
    const int fill = (int)(n_after < st.w ? n_after : st.w);
    const bool hoist_s = WIDE && ATT && n_evicted_after > 0 && st.s <= 32 * kAccWords;
    auto pair_issue = [&](const char *Kb, const char *Vb, const float *vnorm, const int nrows, const int r0, auto &rk,
                          auto &rv, auto &vnj) __attribute__((always_inline)) {
        constexpr int N = (int)(sizeof(rk) / sizeof(rk[0]));
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const int r = r0 + u * RPB + sub;
            const int rr = r < nrows ? r : nrows - 1;
            rk[u] = ldnt16(Kb + (size_t)rr * ROWB + col * 16);
            rv[u] = ldnt16(Vb + (size_t)rr * ROWB + col * 16);
            vnj[u] = vnorm != nullptr ? vnorm[rr] : 1.f;
        }
    };
    uint4 hsk[WIDE ? U : 1], hsv[WIDE ? U : 1], hwk[WIDE ? UW : 1], hwv[WIDE ? UW : 1];
    float hsn[WIDE ? U : 1], hwn[WIDE ? UW : 1];
    if constexpr (WIDE && UPD) {
        for (int i = tid; i < kAccWords; i += WG) sm.accm[i] = 0u;   // (visible behind the barriers of the update)
    }
    {
        uint4 raw[UC];
        float nx[UC], cf[UC];
        auto issue = [&](const int r0) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                const int r = r0 + u * RPB + sub;
                const int rr = r < m ? r : m - 1;
                raw[u] = ldnt16(X + (size_t)rr * ROWB + col * 16);
                if constexpr (UPD) nx[u] = xn[rr];
                if constexpr (ATT) cf[u] = (float)cnt[rr];
            }
        };
        const bool need = ATT || evict;   // an update without an evicted token has nothing to look up
        int r0 = wave * RPW;
        if (need && r0 < m) issue(r0);
        if constexpr (WIDE && ATT) {
            if (hoist_s) pair_issue(Ks, Vs, svn_base, st.s, wave * RPW, hsk, hsv, hsn);
            if (fill > 0) pair_issue(Kw, Vw, (const float *)nullptr, fill, wave * RPW, hwk, hwv, hwn);
        }
        take_evicted();
        for (; need && r0 < m; r0 += RPB * UC) {
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                const int r = r0 + u * RPB + sub;
                const bool valid = r < m;
                if constexpr (ATT) {
                    const float b = row_sum16(dot8_bf16(raw[u], qp));
                    if (valid) {
                        if (b > mx + kLazy || mx == -INFINITY) {
                            den *= __expf(mx - b);   // no value rows yet: acc is still zero
                            mx = b;
                        }
                        den = fmaf(cf[u], __expf(b - mx), den);
                    }
                }
                if constexpr (UPD) {
                    if (evict) {
                        const float dk = row_sum16(dot8_bf16(raw[u], ek));
                        if (valid) {
                            cd.insert(fmaf(-2.f, dk, nx[u] + nk), r);
                            nxmax = fmaxf(nxmax, nx[u]);
                        }
                    }
                }
            }
            if (r0 + RPB * UC < m) issue(r0 + RPB * UC);
        }
    }

    bool extra = false, decided = false, d_created = false, d_forced = false;
    int d_target = 0;
    uint4 xr = make_uint4(0, 0, 0, 0);
    if constexpr (UPD) {
        if (evict) {
            // ---- the nearest candidates over the workgroup
#pragma unroll
            for (int o = 16; o < 64; o <<= 1) {
                const float ob1 = __shfl_xor(cd.b1, o), ob2 = __shfl_xor(cd.b2, o), ob3 = __shfl_xor(cd.b3, o);
                const int oi1 = __shfl_xor(cd.i1, o), oi2 = __shfl_xor(cd.i2, o);
                cd.merge(ob1, oi1, ob2, oi2, ob3);
                nxmax = fmaxf(nxmax, __shfl_xor(nxmax, o));
            }
            if (lane == 0) {
                sm.wb1[wave] = cd.b1;
                sm.wb2[wave] = cd.b2;
                sm.wb3[wave] = cd.b3;
                sm.wi1[wave] = cd.i1;
                sm.wi2[wave] = cd.i2;
                sm.wnx[wave] = nxmax;
            }
            lds_barrier();
            cd.b1 = sm.wb1[0]; cd.b2 = sm.wb2[0]; cd.b3 = sm.wb3[0]; cd.i1 = sm.wi1[0]; cd.i2 = sm.wi2[0];
            nxmax = sm.wnx[0];
#pragma unroll
            for (int wv = 1; wv < NW; ++wv) {
                cd.merge(sm.wb1[wv], sm.wi1[wv], sm.wb2[wv], sm.wi2[wv], sm.wb3[wv]);
                nxmax = fmaxf(nxmax, sm.wnx[wv]);
            }
            // ---- decide from D~ when the error bound allows it, else re-evaluate exactly
            const float thr = (float)st.delta2;
            const float emax = kDistEps * (nxmax + nk);
            bool join;
            int bidx = cd.i1;
            const bool ambiguous = distances_ambiguous(cd.b1, cd.b2, thr, emax, m);
            if (ambiguous) {
                double best;
                exact_decide<LPR, NW>(X, m, ek, cd, emax, sm.wbest, sm.widx, best, bidx);
                join = bidx >= 0 && best <= st.delta2;
            } else {
                join = m > 0 && cd.b1 <= thr;
            }
            const Decision dec = decide_cluster(join, bidx, m, st.Mcap);
            const bool forced = dec.forced, created = dec.created;
            const int target = dec.target;
            if constexpr (ATT) {
                // the cluster that gained this token adds one more term to the normaliser: its row is only
                // requested here, the product waits until the row has landed (before the final merge)
                if (wave == 0 && sub == 0) {
                    xr = ek;
                    if (!created) xr = ld16(X + (size_t)target * ROWB + col * 16);
                }
                extra = true;
            }
            // the cluster table is written at the very end of the step: nothing below reads it, and the barrier
            // in between would have to wait for those stores (and the count's read-modify-write)
            decided = true;
            d_created = created;
            d_forced = forced;
            d_target = target;
            if (created) m += 1;

            // ---- sampling update: p from the old mu, one coin per slot, then mu += ||v||^2.  Accepts are rare
            //      (about s/n per token), so the lane that draws one copies the two rows itself.
            const float p = coin_probability(mu, vn);
            if (p > 0.f) {
                for (int j0 = tid * 4; j0 < st.s; j0 += WG * 4) {
                    uint32_t r[4];
                    coin_block(st, sid, etoken, (uint32_t)(j0 >> 2), false, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int j = j0 + i;
                        if (j < st.s && coin_accepts(r[i], p)) {
                            for (int ch = 0; ch < 16; ++ch) {
                                st16(Ks + (size_t)j * ROWB + ch * 16, sm.ekrow[ch]);
                                st16(Vs + (size_t)j * ROWB + ch * 16, sm.evrow[ch]);
                            }
                            st.sidx[sid * (size_t)st.sS + j] = (int32_t)etoken;
                            st.svn[sid * (size_t)st.sS + j] = vn;
                            if constexpr (WIDE) {
                                if (j < 32 * kAccWords) atomicOr(&sm.accm[j >> 5], 1u << (j & 31));
                            }
                            // the other lanes read these rows after the barrier below: wait for the stores here,
                            // in the rare lane that made them, rather than in a full barrier for everybody
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                        }
                    }
                }
            }
            mu += (double)vn;
        }
        lds_barrier();  // the new token's rows (LDS) and freshly sampled rows (released above) are visible
    }

    if constexpr (ATT) {
        // rows with values: sampled pairs (importance weights, numerator only), then the window (weight 1, both)
        // kind 1 = sampled pairs: a slot that took the evicted token in this very step may have been requested
        // before that store (hoisted batch): its rows are then taken from LDS; kind 2 = window: the new token's
        // rows are not in the ring yet, they come from LDS as well
        auto pair_process = [&](const int kind, const float wmul, const int nrows, const int r0, const auto &rk,
                                const auto &rv, const auto &vnj) __attribute__((always_inline)) {
            constexpr int N = (int)(sizeof(rk) / sizeof(rk[0]));
#pragma unroll
            for (int u = 0; u < N; ++u) {
                const int r = r0 + u * RPB + sub;
                const bool valid = r < nrows;
                const int rr = valid ? r : nrows - 1;
                uint4 k8 = rk[u], v8 = rv[u];
                float vnr = vnj[u];
                if (kind == 2) {
                    if (rr == wslot) {
                        k8 = sm.nkrow[col];
                        v8 = sm.nvrow[col];
                    }
                } else if constexpr (WIDE && UPD) {
                    if (rr < 32 * kAccWords && ((sm.accm[rr >> 5] >> (rr & 31)) & 1u)) {
                        k8 = sm.ekrow[col];
                        v8 = sm.evrow[col];
                        vnr = vn;
                    }
                }
                const float b = row_sum16(dot8_bf16(k8, qp));
                float e = 0.f;
                if (valid) {
                    if (b > mx + kLazy || mx == -INFINITY) {
                        const float sc = __expf(mx - b);   // mx = -inf gives 0
                        den *= sc;
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[i] *= sc;
                        mx = b;
                    }
                    const float wgt = kind == 1 ? (vnr > 0.f ? wmul * __builtin_amdgcn_rcpf(vnr) : 0.f) : 1.f;
                    e = wgt * __expf(b - mx);
                    if (kind == 2) den += e;
                }
                float vf[8];
                unpack<true>(v8, vf);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = fmaf(e, vf[i], acc[i]);
            }
        };
        auto scan = [&](const int kind, const char *Kb, const char *Vb, const float *vnorm, const float wmul,
                        const int nrows, const int rstart) __attribute__((always_inline)) {
            for (int r0 = rstart; r0 < nrows; r0 += RPB * U) {
                uint4 rk[U], rv[U];
                float vnj[U];
                pair_issue(Kb, Vb, vnorm, nrows, r0, rk, rv, vnj);
                pair_process(kind, wmul, nrows, r0, rk, rv, vnj);
            }
        };
        const float mus = (float)(mu / (double)st.s);
        if (n_evicted_after > 0) {
            int rstart = wave * RPW;
            if constexpr (WIDE) {
                if (hoist_s) {
                    pair_process(1, mus, st.s, rstart, hsk, hsv, hsn);
                    rstart += RPB * U;
                }
            }
            scan(1, Ks, Vs, svn_base, mus, st.s, rstart);
        }
        {
            int rstart = wave * RPW;
            if constexpr (WIDE) {
                if (fill > 0) {
                    pair_process(2, 1.f, fill, rstart, hwk, hwv, hwn);
                    rstart += RPB * UW;
                }
            }
            scan(2, Kw, Vw, nullptr, 1.f, fill, rstart);
        }

        if (extra && wave == 0 && sub == 0) {
            const float a = row_sum16(dot8_bf16(xr, qp));
            if (col == 0) sm.bx = a;
        }
        // ---- merge the four row groups of the wavefront, then the wavefronts through LDS
        float M = fmaxf(mx, __shfl_xor(mx, 16));
        M = fmaxf(M, __shfl_xor(M, 32));
        const float f = (mx == -INFINITY) ? 0.f : __expf(mx - M);
        float dsum = den * f;
        dsum += __shfl_xor(dsum, 16);
        dsum += __shfl_xor(dsum, 32);
        if (lane == 0) {
            sm.wmx[wave] = M;
            sm.wden[wave] = dsum;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float t = acc[i] * f;
            t += __shfl_xor(t, 16);
            t += __shfl_xor(t, 32);
            if (sub == 0) sm.wacc[wave][col * 8 + i] = t;
        }
        __syncthreads();
        if (tid < 128) {
            const float bx = extra ? sm.bx : -INFINITY;
            float Mx = bx;
#pragma unroll
            for (int wv = 0; wv < NW; ++wv) Mx = fmaxf(Mx, sm.wmx[wv]);
            float dn = extra ? __expf(bx - Mx) : 0.f, num = 0.f;
#pragma unroll
            for (int wv = 0; wv < NW; ++wv) {
                const float wm = sm.wmx[wv];
                const float sc = (wm == -INFINITY) ? 0.f : __expf(wm - Mx);
                dn = fmaf(sm.wden[wv], sc, dn);
                num = fmaf(sm.wacc[wv][tid], sc, num);
            }
            put_out(st, outrow, tid, num / dn);
        }
    }
    // ---- the update's writes to the ring and to the cluster table (see above)
    if constexpr (UPD) {
        if (wslot >= 0 && tid < LPR) {
            st16(Kw + (size_t)wslot * ROWB + tid * 16, sm.nkrow[tid]);
            st16(Vw + (size_t)wslot * ROWB + tid * 16, sm.nvrow[tid]);
        }
        if (decided) {
            if (d_created) {
                if (tid < LPR) st16(X + (size_t)d_target * ROWB + tid * 16, sm.ekrow[tid]);
                if (tid == 0) {
                    cnt[d_target] = 1;
                    xn[d_target] = nk;
                }
            } else if (tid == 0) {
                atomicAdd(&cnt[d_target], 1);
                if (d_forced) st.flags[sid] |= 1u;
            }
            if (tid == 0 && st.assign != nullptr && etoken < st.assign_cap)
                st.assign[sid * (size_t)st.assign_cap + etoken] = d_target;
        }
    }
}

// NW wavefronts per workgroup: 4 when there are streams enough to fill the chip; 8 for a few streams, where the
// step of one stream is a chain of memory round trips and the first batch of every kind of row is requested at once
template <bool UPD, bool ATT, int NW>
__global__ __launch_bounds__(NW * 64) void decode_dot2_kernel(const State st, const Call call)
{
    __shared__ SmemDot2<NW> sm;
    const size_t sid = blockIdx.x;
    int m = st.m[sid];
    double mu = st.mu[sid];
    const char *krow = UPD ? call.K + sid * call.stream_stride : nullptr;
    const char *vrow = UPD ? call.V + sid * call.stream_stride : nullptr;
    const char *qrow = ATT ? call.Q + sid * call.q_stride : nullptr;
    float *outrow = ATT ? out_rows(st, call.out, sid * call.out_stride) : nullptr;
    token_step_dot2<UPD, ATT, NW>(st, sid, krow, vrow, qrow, outrow, tokens_seen(st, call.n_seen), m, mu, sm);
    if constexpr (UPD) {
        if (threadIdx.x == 0) {
            st.m[sid] = m;
            st.mu[sid] = mu;
        }
    }
}

}  // namespace sg
