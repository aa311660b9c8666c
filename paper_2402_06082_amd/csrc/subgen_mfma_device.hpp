// bf16 decode step for gfx950 with the score contractions on the matrix cores.
//
// Every score of the step is a dot product of a stored row (representative,
// sampled key, window key) with one of a few vectors (the queries and the
// evicted key).  A wavefront takes 16 rows at a time and runs
// v_mfma_f32_16x16x32_bf16 with the 16 stored rows as the A operand and the
// vectors as the B operand (column n carries the vector of role(n): a query or
// the evicted key).  Lane (n, L) = lane 16L+n loads the 16-byte chunks L, L+4,
// L+8, ... of row n, which is exactly the A layout (k = 8L..8L+7 of each
// 32-wide K slice), so rows go from HBM into the MFMA operand with no shuffle,
// no LDS and no conversion.  The result register r of lane (n, L) is the score
// of row 4L+r against vector role(n): each lane row L owns four rows.
//
// Value rows are loaded one full row per 16 lanes (lane n takes chunk n of row
// 4L+u), so the weight a lane needs sits in a lane of its own quad (DPP
// quad broadcast) and a lane owns only 8 output columns per query.
//
// Nearest-center decisions stay exact: the matrix cores give
// D~_i = ||x_i||^2 + ||k||^2 - 2<x_i,k> with a bounded error; the decision is
// taken from D~ only when the best/runner-up gap and the distance to delta^2
// exceed that bound, otherwise the workgroup re-evaluates all distances in
// double precision (the generic path's arithmetic).
#pragma once
#include "subgen_device.hpp"

namespace sg {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4_t mfma_bf16(const uint4 &a, const uint4 &b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

// Relative bound used for |D~ - D| <= kDistEps * (||x||^2 + ||k||^2): 128..256 exact bf16 products
// accumulated in fp32 by the matrix cores (<= 2^-16 of sum |x_c k_c| even with truncating adds) plus
// the fp32 roundings of the two norms and of the final fma, with a 4x margin.
constexpr float kDistEps = 1.0f / 16384.0f;
constexpr float kLazy = 8.0f;  // the running softmax reference is raised only when a score exceeds it by this much

typedef short shortx4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

// rows k0..k0+3 of columns 16 cb .. 16 cb + 15 of a row-major bf16 tile in LDS, transposed: lane i of each 16-lane
// group passes the address of row k0 + i/4, columns 4 (i%4) .. +3, and receives column i (element e = row k0 + e)
__device__ __forceinline__ u32x2_t lds_read_tr16(const char *p)
{
    const shortx4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (shortx4_t __attribute__((address_space(3))) *)(p));
    return __builtin_bit_cast(u32x2_t, v);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)   // round to nearest even
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf16_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }

template <int NK, int G>
struct SmemMfma {
    alignas(16) uint4 ekrow[NK * 4], evrow[NK * 4];   // the evicted (key, value) rows, for the sampling copies
    // approximate nearest-center candidates per wavefront
    float wb1[kWaves], wb2[kWaves], wb3[kWaves], wnx[kWaves];
    int wi1[kWaves], wi2[kWaves];
    // exact re-evaluation
    double wbest[kWaves];
    int widx[kWaves];
    float bx[G];
    float wmx[kWaves][G], wden[kWaves][G];
    float wacc[kWaves][G][NK * 32];
};

// min(a, b) as the one instruction it is (fminf first quiets its operands with one more instruction each); a NaN
// operand is ignored.  Inline assembly: never hand it a matrix-core result directly (the compiler covers the read
// hazard of v_mfma results only for instructions of its own); results of ordinary vector instructions are fine.
__device__ __forceinline__ float min_f32(const float a, const float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Candidate list of a token: nearest (b1, i1), runner-up (b2, i2) and the third-smallest value b3 of the approximate
// distances.  Insert candidate (d, idx).  Equal values keep the order of arrival: the decision never rests on
// that order, since equal approximations are within the error bound of each other and go to the exact comparison.
__device__ __forceinline__ void top3_insert(const float d, const int idx, float &b1, int &i1, float &b2, int &i2, float &b3)
{
    const bool lt1 = d < b1, lt2 = d < b2;
    b3 = __builtin_amdgcn_fmed3f(b2, b3, d);
    int t2 = lt2 ? idx : i2;
    asm("" : "+v"(t2));   // two plain selects (nested, the compiler turns them into branches)
    i2 = lt1 ? i1 : t2;
    b2 = __builtin_amdgcn_fmed3f(b1, b2, d);
    i1 = lt1 ? idx : i1;
    b1 = min_f32(b1, d);
}
struct Cand3 {
    float b1 = INFINITY, b2 = INFINITY, b3 = INFINITY;
    int i1 = -1, i2 = -1;
    __device__ __forceinline__ void insert(const float d, const int idx) { top3_insert(d, idx, b1, i1, b2, i2, b3); }
    // another list over other rows
    __device__ __forceinline__ void merge(const float ob1, const int oi1, const float ob2, const int oi2, const float ob3)
    {
        insert(ob1, oi1);
        insert(ob2, oi2);
        b3 = min_f32(b3, ob3);
    }
};

// Exact squared distance of two bf16 rows in double precision: each of the LPR lanes of a row holds one 16-byte
// chunk of both; all of them get the sum.
template <int LPR>
__device__ __forceinline__ double exact_distance(const uint4 &xrow, const uint4 &krow)
{
    float x[8], k[8];
    unpack<true>(xrow, x);
    unpack<true>(krow, k);
    double dist = 0.0;
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const double df = (double)x[v] - (double)k[v];
        dist = fma(df, df, dist);
    }
    return group_sum<LPR>(dist);
}

// Exact nearest representative in double precision (lowest index on ties); block-uniform result.
template <int LPR, int NW = kWaves>
__device__ __forceinline__ void exact_nearest(const char *X, int m, const uint4 &ek, double *wbest, int *widx,
                                              double &best, int &bidx)
{
    constexpr int RPW = 64 / LPR, RPB = RPW * NW;
    constexpr size_t ROWB = (size_t)LPR * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR;
    best = INFINITY;
    bidx = -1;
    for (int r0 = wave * RPW; r0 < m; r0 += RPB * kUnroll) {
        uint4 raw[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = r0 + u * RPB + sub;
            raw[u] = ld16(X + (size_t)(r < m ? r : m - 1) * ROWB + col * 16);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = r0 + u * RPB + sub;
            const double dist = exact_distance<LPR>(raw[u], ek);
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
        wbest[wave] = best;
        widx[wave] = bidx;
    }
    __syncthreads();
    best = wbest[0];
    bidx = widx[0];
#pragma unroll
    for (int wv = 1; wv < NW; ++wv) {
        const double ob = wbest[wv];
        const int oi = widx[wv];
        if (ob < best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
            best = ob;
            bidx = oi;
        }
    }
    __syncthreads();
}

// The exact decision for an ambiguous token: every exact distance is at most emax away from its approximation, so
// the nearest representative is among those within 2 emax of the smallest approximation.  When the third-smallest
// approximation is beyond that, these are the best and (perhaps) the runner-up, and their one or two exact
// distances decide (every wavefront evaluates them by itself: no barrier); otherwise the whole table is
// re-evaluated.  `cd` is the same in every lane of the workgroup.  Block-uniform result.
template <int LPR, int NW = kWaves>
__device__ __forceinline__ void exact_decide(const char *X, const int m, const uint4 &ek, const Cand3 &cd, const float emax,
                                             double *wbest, int *widx, double &best, int &bidx)
{
    constexpr size_t ROWB = (size_t)LPR * 16;
    const int lane = threadIdx.x & 63, col = lane % LPR, sub = lane / LPR;
    if (cd.i1 >= 0 && (cd.b3 == INFINITY || cd.b3 - cd.b1 > 2.f * emax)) {
        const int r2 = cd.b2 - cd.b1 > 2.f * emax ? -1 : cd.i2;
        const int rsel = sub == 0 ? cd.i1 : (sub == 1 ? r2 : -1);
        double dist = INFINITY;
        if (rsel >= 0) dist = exact_distance<LPR>(ld16(X + (size_t)rsel * ROWB + col * 16), ek);
        const double d1 = __shfl(dist, 0), d2 = __shfl(dist, LPR);
        const bool second = r2 >= 0 && (d2 < d1 || (d2 == d1 && r2 < cd.i1));
        best = second ? d2 : d1;
        bidx = second ? r2 : cd.i1;
    } else {
        exact_nearest<LPR, NW>(X, m, ek, wbest, widx, best, bidx);
    }
}

// broadcast lane g of every quad (DPP quad_perm [g,g,g,g])
template <int Gq>
__device__ __forceinline__ float quad_bcast(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v),
                                                                 Gq | (Gq << 2) | (Gq << 4) | (Gq << 6), 0xf, 0xf, false));
}
template <int G>
__device__ __forceinline__ void bcast_roles(float v, float (&out)[G])
{
    if constexpr (G == 1) {
        out[0] = v;
    } else if constexpr (G == 2) {
        out[0] = quad_bcast<0>(v);
        out[1] = quad_bcast<1>(v);
    } else {
        out[0] = quad_bcast<0>(v);
        out[1] = quad_bcast<1>(v);
        out[2] = quad_bcast<2>(v);
        out[3] = quad_bcast<3>(v);
    }
}

// Lane layout of one 16-row step (lane = 16 L + n):
//   A operand  : lane (n, L) loads row r0 + n, 16-byte chunks L, L+4, ...         (stored rows)
//   B operand  : lane (n, L) holds the vector of column role(n), same chunks       (queries / evicted key)
//   result c[r]: <row r0 + 4L + r, vector role(n)>, r = 0..3
//   value rows : lane (n, L) loads chunk n of row r0 + 4L + u for u = 0..3 (one full row per 16 lanes),
//                so the weight it needs is its own row-L register e[u] of the lane holding that query
//                (same quad), and it owns 8 output columns per query.
template <int NK, int G, bool UPD, bool ATT>
__device__ __forceinline__ void token_step_mfma(const State &st, const size_t sid, const char *krow, const char *vrow,
                                                const char *qrows, float *outrows, const int64_t n_seen, int &m,
                                                double &mu, SmemMfma<NK, G> &sm)
{
    constexpr int CPR = 4 * NK;                    // 16-byte chunks per row
    constexpr int LPR = CPR;                       // lanes per row in the plain row layout (copies, norms)
    constexpr int RPW = 64 / LPR;
    constexpr size_t ROWB = (size_t)NK * 64;
    constexpr int D = NK * 32;
    constexpr int VL = CPR > 16 ? CPR / 16 : 1;    // value loads per row per lane (d = 256: 2)
    constexpr int RPLD = CPR < 16 ? 16 / CPR : 1;  // value rows per 16-lane load (d = 64: 2)
    constexpr int NVL = 4 / RPLD;                  // value row-steps per 16-row group
    constexpr int ACC = 8 * VL;                    // output columns per query per lane
    constexpr int NC = G == 1 ? 2 : (G == 2 ? 4 : 8);  // column roles in the center pass: G queries + the key
    constexpr int KR = ATT ? G : 0;                // column role of the evicted key in the center pass
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR;  // plain row layout
    const int grp = wave * RPW + sub;
    const int n16 = lane & 15, L = lane >> 4;
    const int vchunk = RPLD == 2 ? (n16 & (CPR - 1)) : n16;   // value chunk (+16 per extra load)
    const int vrsub = RPLD == 2 ? (n16 / CPR) : 0;             // which of the RPLD rows of a value load

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    float *const xn = st.xn + sid * (size_t)st.McapS;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;

    // ---- B operand of the center pass: queries in column roles 0..G-1, evicted key in role KR
    const int rc = n16 % NC;
    const bool qrole_c = ATT && rc < G;
    const bool krole_c = UPD && rc == KR;
    uint4 Bc[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) Bc[kk] = make_uint4(0, 0, 0, 0);
    if constexpr (ATT) {
        if (qrole_c) {
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) Bc[kk] = ld16(qrows + (size_t)rc * ROWB + (L + 4 * kk) * 16);
        }
    }

    // ---- window push; the token that leaves the window is the one that is compressed
    bool evict = false;
    int64_t etoken = 0;
    uint4 ek = make_uint4(0, 0, 0, 0), ev = make_uint4(0, 0, 0, 0);
    if constexpr (UPD) {
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
            if (krole_c) {
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) Bc[kk] = ld16(esk + (L + 4 * kk) * 16);
            }
        }
        __syncthreads();  // every lane holds the evicted row (registers, LDS) before the slot is overwritten
        if (st.w > 0) {
            if (tid < LPR) {
                st16(kw + tid * 16, ld16(krow + tid * 16));
                st16(vw + tid * 16, ld16(vrow + tid * 16));
            }
        }
    }
    const int64_t n_after = UPD ? n_seen + 1 : n_seen;
    const int64_t n_evicted_after = st.w == 0 ? n_after : (n_after > st.w ? n_after - st.w : 0);

    // ||k'||^2 and ||v'||^2 in double from the exactly converted elements
    float nk = 0.f, vn = 0.f;
    if constexpr (UPD) {
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
        if (evict && !token_is_finite(nk, vn)) {   // NaN or Inf in the token: dropped and flagged
            evict = false;
            if (tid == 0) st.flags[sid] |= 2u;
        }
    }

    // online softmax state of this lane's query role: lazily raised reference, denominator
    float mx = -INFINITY, den = 0.f;

    // ---- one pass over the representatives, 16 rows per wavefront step; the loads of the next step are
    //      issued before the arithmetic of the current one (two register sets, ping-pong)
    Cand3 cd;   // nearest representatives of the evicted key by approximate distance (key-role lanes)
    float nxmax = 0.f;
    if ((UPD && evict) || ATT) {
        struct Group {
            uint4 a[NK];
            float4 nx;
            int4 cn;
        };
        auto load = [&](Group &gq, const int base) {
            const int rr = base + n16 < m ? base + n16 : m - 1;
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) gq.a[kk] = ldnt16(X + (size_t)rr * ROWB + (L + 4 * kk) * 16);
            if constexpr (UPD) gq.nx = *reinterpret_cast<const float4 *>(xn + base + 4 * L);
            if constexpr (ATT) gq.cn = *reinterpret_cast<const int4 *>(cnt + base + 4 * L);
        };
        auto compute = [&](const Group &gq, const int base) {
            floatx4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(gq.a[kk], Bc[kk], c);
            const int row0 = base + 4 * L;   // rows of this lane's four results
            if constexpr (ATT) {
                if (qrole_c && row0 < m) {
                    const float cf[4] = {(float)gq.cn.x, (float)gq.cn.y, (float)gq.cn.z, (float)gq.cn.w};
                    float mc = c[0];
#pragma unroll
                    for (int r = 1; r < 4; ++r) mc = (row0 + r < m) ? fmaxf(mc, c[r]) : mc;
                    if (mc > mx + kLazy || mx == -INFINITY) {
                        den *= __expf(mx - mc);
                        mx = mc;
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (row0 + r < m) den = fmaf(cf[r], __expf(c[r] - mx), den);
                }
            }
            if constexpr (UPD) {
                if (krole_c && evict) {
                    const float nxr[4] = {gq.nx.x, gq.nx.y, gq.nx.z, gq.nx.w};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (row0 + r < m) {
                            cd.insert(fmaf(-2.f, c[r], nxr[r] + nk), row0 + r);
                            nxmax = fmaxf(nxmax, nxr[r]);
                        }
                    }
                }
            }
        };
        constexpr int STEP = 16 * kWaves;
        Group ga, gb;
        int r0 = wave * 16;
        if (r0 < m) load(ga, r0);
        while (r0 < m) {
            if (r0 + STEP < m) load(gb, r0 + STEP);
            compute(ga, r0);
            r0 += STEP;
            if (r0 >= m) break;
            if (r0 + STEP < m) load(ga, r0 + STEP);
            compute(gb, r0);
            r0 += STEP;
        }
    }

    if constexpr (UPD) {
        if (evict) {
            // ---- the nearest candidates: over the four lane rows, then the wavefronts
#pragma unroll
            for (int o = 16; o < 64; o <<= 1) {
                const float ob1 = __shfl_xor(cd.b1, o), ob2 = __shfl_xor(cd.b2, o), ob3 = __shfl_xor(cd.b3, o);
                const int oi1 = __shfl_xor(cd.i1, o), oi2 = __shfl_xor(cd.i2, o);
                cd.merge(ob1, oi1, ob2, oi2, ob3);
                nxmax = fmaxf(nxmax, __shfl_xor(nxmax, o));
            }
            if (lane == KR) {   // a key-role lane of lane row 0
                sm.wb1[wave] = cd.b1;
                sm.wb2[wave] = cd.b2;
                sm.wb3[wave] = cd.b3;
                sm.wi1[wave] = cd.i1;
                sm.wi2[wave] = cd.i2;
                sm.wnx[wave] = nxmax;
            }
            __syncthreads();
            cd.b1 = sm.wb1[0]; cd.b2 = sm.wb2[0]; cd.b3 = sm.wb3[0]; cd.i1 = sm.wi1[0]; cd.i2 = sm.wi2[0];
            nxmax = sm.wnx[0];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) {
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
                exact_decide<LPR>(X, m, ek, cd, emax, sm.wbest, sm.widx, best, bidx);
                join = bidx >= 0 && best <= st.delta2;
            } else {
                join = m > 0 && cd.b1 <= thr;
            }
            const Decision dec = decide_cluster(join, bidx, m, st.Mcap);
            const bool forced = dec.forced, created = dec.created;
            const int target = dec.target;
            if (created) {
                if (tid < LPR) st16(X + (size_t)m * ROWB + tid * 16, ek);
                if (tid == 0) {
                    cnt[m] = 1;
                    xn[m] = nk;
                }
            } else if (tid == 0) {
                cnt[target] += 1;
                if (forced) st.flags[sid] |= 1u;
            }
            if (tid == 0 && st.assign != nullptr && etoken < st.assign_cap)
                st.assign[sid * (size_t)st.assign_cap + etoken] = target;
            if constexpr (ATT) {
                // score of the cluster that gained this token: one more term of the normaliser
                if (grp == 0) {
                    uint4 xr = ek;
                    if (!created) xr = ld16(X + (size_t)target * ROWB + col * 16);
                    float xf[8];
                    unpack<true>(xr, xf);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        float qf[8];
                        unpack<true>(ld16(qrows + (size_t)g * ROWB + col * 16), qf);
                        float a = 0.f;
#pragma unroll
                        for (int v = 0; v < 8; ++v) a = fmaf(qf[v], xf[v], a);
                        a = group_sum<LPR>(a);
                        if (col == 0) sm.bx[g] = a;
                    }
                }
            }
            if (created) m += 1;

            // ---- sampling update: p from the old mu, one coin per slot, then mu += ||v||^2
            const float p = coin_probability(mu, vn);
            // accepts are rare (about s/n per token), so the lane that draws one copies the two rows itself
            if (p > 0.f) {
                for (int j0 = tid * 4; j0 < st.s; j0 += kWG * 4) {
                    uint32_t r[4];
                    coin_block(st, sid, etoken, (uint32_t)(j0 >> 2), false, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int j = j0 + i;
                        if (j < st.s && coin_accepts(r[i], p)) {
                            for (int ch = 0; ch < CPR; ++ch) {
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
        __syncthreads();  // window slot, center row and sample rows are visible to the whole workgroup
    }

    if constexpr (ATT) {
        const bool extra = UPD && evict;
        // ---- hand the normaliser state from the center-pass column roles to the query roles n % G
        {
            const int src = (lane & 48) | (n16 % G);
            mx = __shfl(mx, src);
            den = __shfl(den, src);
        }
        uint4 Bq[NK];
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) Bq[kk] = ld16(qrows + (size_t)(n16 % G) * ROWB + (L + 4 * kk) * 16);
        float acc[G][ACC];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < ACC; ++i) acc[g][i] = 0.f;

        // one 16-row group of (key rows, value rows): scores on the matrix cores, weights per lane row,
        // value rows accumulated into the lane's output columns
        struct RowGroup {
            uint4 a[NK], bv[NVL][VL];
            float4 vn4;
        };
        auto scan = [&](const char *Kb, const char *Vb, const float *vnorm, const float wmul, const int nrows,
                        const bool to_den) {
            auto load = [&](RowGroup &gq, const int r0) {
                const int rr = r0 + n16 < nrows ? r0 + n16 : nrows - 1;
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) gq.a[kk] = ldnt16(Kb + (size_t)rr * ROWB + (L + 4 * kk) * 16);
#pragma unroll
                for (int u = 0; u < NVL; ++u) {
                    const int vr = r0 + 4 * L + u * RPLD + vrsub;
                    const int vrr = vr < nrows ? vr : nrows - 1;
#pragma unroll
                    for (int vl = 0; vl < VL; ++vl)
                        gq.bv[u][vl] = ldnt16(Vb + (size_t)vrr * ROWB + (vchunk + 16 * vl) * 16);
                }
                if (vnorm != nullptr) gq.vn4 = *reinterpret_cast<const float4 *>(vnorm + r0 + 4 * L);
            };
            auto compute = [&](const RowGroup &gq, const int r0) {
                float wg[4] = {1.f, 1.f, 1.f, 1.f};
                if (vnorm != nullptr) {
                    const float vv[4] = {gq.vn4.x, gq.vn4.y, gq.vn4.z, gq.vn4.w};
#pragma unroll
                    for (int r = 0; r < 4; ++r) wg[r] = vv[r] > 0.f ? wmul * __builtin_amdgcn_rcpf(vv[r]) : 0.f;
                }
                floatx4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(gq.a[kk], Bq[kk], c);
                const int row0 = r0 + 4 * L;
                float scale = 1.f;
                float e[4] = {0.f, 0.f, 0.f, 0.f};
                if (row0 < nrows) {
                    float mc = c[0];
#pragma unroll
                    for (int r = 1; r < 4; ++r) mc = (row0 + r < nrows) ? fmaxf(mc, c[r]) : mc;
                    if (mc > mx + kLazy || mx == -INFINITY) {
                        scale = __expf(mx - mc);   // mx = -inf gives 0
                        den *= scale;
                        mx = mc;
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (row0 + r < nrows) e[r] = wg[r] * __expf(c[r] - mx);
                    if (to_den) den += (e[0] + e[1]) + (e[2] + e[3]);
                }
                if (__any(scale != 1.f)) {
                    float sg[G];
                    bcast_roles<G>(scale, sg);
#pragma unroll
                    for (int g = 0; g < G; ++g)
#pragma unroll
                        for (int i = 0; i < ACC; ++i) acc[g][i] *= sg[g];
                }
#pragma unroll
                for (int u = 0; u < NVL; ++u) {
                    float esel = e[u * RPLD];
                    if constexpr (RPLD == 2) esel = vrsub ? e[u * RPLD + 1] : esel;
                    float eg[G];
                    bcast_roles<G>(esel, eg);
#pragma unroll
                    for (int vl = 0; vl < VL; ++vl) {
                        float vf[8];
                        unpack<true>(gq.bv[u][vl], vf);
#pragma unroll
                        for (int g = 0; g < G; ++g)
#pragma unroll
                            for (int i = 0; i < 8; ++i) acc[g][vl * 8 + i] = fmaf(eg[g], vf[i], acc[g][vl * 8 + i]);
                    }
                }
            };
            constexpr int STEP = 16 * kWaves;
            RowGroup ga, gb;
            int r0 = wave * 16;
            if (r0 < nrows) load(ga, r0);
            while (r0 < nrows) {
                if (r0 + STEP < nrows) load(gb, r0 + STEP);
                compute(ga, r0);
                r0 += STEP;
                if (r0 >= nrows) break;
                if (r0 + STEP < nrows) load(ga, r0 + STEP);
                compute(gb, r0);
                r0 += STEP;
            }
        };
        // sampled pairs: numerator terms  mu/(s ||v_j||^2) e^{<q,k_j>} v_j
        if (n_evicted_after > 0)
            scan(Ks, Vs, st.svn + sid * (size_t)st.sS, (float)(mu / (double)st.s), st.s, false);
        // window: exact terms in numerator and normaliser
        const int fill = (int)(n_after < st.w ? n_after : st.w);
        scan(Kw, Vw, nullptr, 1.f, fill, true);

        // ---- merge the four lane rows of the wavefront, then the wavefronts through LDS
        float M = fmaxf(mx, __shfl_xor(mx, 16));
        M = fmaxf(M, __shfl_xor(M, 32));
        const float f = (mx == -INFINITY) ? 0.f : __expf(mx - M);
        float dsum = den * f;
        dsum += __shfl_xor(dsum, 16);
        dsum += __shfl_xor(dsum, 32);
        if (lane < G) {   // lane g of lane row 0 has query role g
            sm.wmx[wave][lane] = M;
            sm.wden[wave][lane] = dsum;
        }
        float fg[G];
        bcast_roles<G>(f, fg);
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int i = 0; i < ACC; ++i) {
                float t = acc[g][i] * fg[g];
                t += __shfl_xor(t, 16);
                t += __shfl_xor(t, 32);
                if constexpr (RPLD == 2) t += __shfl_xor(t, 8);
                if (L == 0 && n16 < CPR) sm.wacc[wave][g][(vchunk + 16 * (i / 8)) * 8 + (i % 8)] = t;
            }
        }
        __syncthreads();
        for (int i = tid; i < G * D; i += kWG) {
            const int g = i / D, c = i % D;
            const float bx = extra ? sm.bx[g] : -INFINITY;
            float Mx = bx;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) Mx = fmaxf(Mx, sm.wmx[wv][g]);
            float dn = extra ? __expf(bx - Mx) : 0.f, num = 0.f;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) {
                const float wm = sm.wmx[wv][g];
                const float sc = (wm == -INFINITY) ? 0.f : __expf(wm - Mx);
                dn = fmaf(sm.wden[wv][g], sc, dn);
                num = fmaf(sm.wacc[wv][g][c], sc, num);
            }
            put_out(st, outrows, (size_t)g * D + c, num / dn);
        }
    }
    __syncthreads();  // LDS and state are reusable by the next token
}

// at least two workgroups per CU (two wavefronts per SIMD) even for the widest accumulator sets
template <int NK, int G, bool UPD, bool ATT>
__global__ __launch_bounds__(kWG, 3) void decode_mfma_kernel(const State st, const Call call)
{
    __shared__ SmemMfma<NK, G> sm;
    const size_t sid = blockIdx.x;
    int m = st.m[sid];
    double mu = st.mu[sid];
    const char *krow = UPD ? call.K + sid * call.stream_stride : nullptr;
    const char *vrow = UPD ? call.V + sid * call.stream_stride : nullptr;
    const char *qrows = ATT ? call.Q + sid * call.q_stride : nullptr;
    float *outrows = ATT ? out_rows(st, call.out, sid * call.out_stride) : nullptr;
    token_step_mfma<NK, G, UPD, ATT>(st, sid, krow, vrow, qrows, outrows, tokens_seen(st, call.n_seen), m, mu, sm);
    if constexpr (UPD) {
        if (threadIdx.x == 0) {
            st.m[sid] = m;
            st.mu[sid] = mu;
        }
    }
}

}  // namespace sg
