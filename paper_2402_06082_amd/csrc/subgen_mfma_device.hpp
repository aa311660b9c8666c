// bf16 decode step for gfx950 with the score contractions on the matrix cores.
//
// Every score of the step is a dot product of a stored row (representative,
// sampled key, window key) with one of a few vectors (the queries and the
// evicted key).  A wavefront takes 16 rows at a time and runs
// v_mfma_f32_16x16x32_bf16 with the vectors as the A operand (the queries are
// replicated in rows 4L+r, so every 16-lane row L of the result holds all G
// scores of row n = lane % 16) and the 16 stored rows as the B operand: lane
// (n, L) loads the 16-byte chunks L, L+4, L+8, ... of row n, which is exactly
// the B layout (k = 8L..8L+7 of each 32-wide K slice), so rows go from HBM
// into the MFMA operands with no shuffle, no LDS and no conversion.  Values
// rows are loaded in the same layout and accumulated on the vector ALUs
// (lane (n, L) owns columns of chunks L, L+4, ... of the output).
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

// all-reduce over the 16 lanes of a DPP row (row rotations 8, 4, 2, 1)
template <int N>
__device__ __forceinline__ float row_ror(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xf, 0xf,
                                                                 false));
}
__device__ __forceinline__ float row_sum16(float v)
{
    v += row_ror<8>(v);
    v += row_ror<4>(v);
    v += row_ror<2>(v);
    v += row_ror<1>(v);
    return v;
}
__device__ __forceinline__ float row_max16(float v)
{
    v = fmaxf(v, row_ror<8>(v));
    v = fmaxf(v, row_ror<4>(v));
    v = fmaxf(v, row_ror<2>(v));
    v = fmaxf(v, row_ror<1>(v));
    return v;
}

// Relative bound used for |D~ - D| <= kDistEps * (||x||^2 + ||k||^2): 128..256 exact bf16 products
// accumulated in fp32 by the matrix cores (<= 2^-16 of sum |x_c k_c| even with truncating adds) plus
// the fp32 roundings of the two norms and of the final fma, with a 4x margin.
constexpr float kDistEps = 1.0f / 16384.0f;
constexpr float kLazy = 8.0f;  // the running softmax reference is raised only when a score exceeds it by this much

template <int NK, int G>
struct SmemMfma {
    // approximate nearest-center candidates per wavefront
    float wb1[kWaves], wb2[kWaves], wnx[kWaves];
    int wi1[kWaves];
    // exact re-evaluation
    double wbest[kWaves];
    int widx[kWaves];
    float bx[G];
    float wmx[kWaves][G], wden[kWaves][G];
    float wacc[kWaves][G][NK * 32];
    int qn;
    int queue[kQueue];
};

// Exact nearest representative in double precision (lowest index on ties); block-uniform result.
template <int LPR>
__device__ __forceinline__ void exact_nearest(const char *X, int m, const uint4 &ek, double *wbest, int *widx,
                                              double &best, int &bidx)
{
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)LPR * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR;
    float ekf[8];
    unpack<true>(ek, ekf);
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
            float x[8];
            unpack<true>(raw[u], x);
            double dist = 0.0;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
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
        if (ob < best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
            best = ob;
            bidx = oi;
        }
    }
    __syncthreads();
}

// per-lane online softmax state of one query: reference maximum (lazy), denominator, NK*8 output columns
template <int NK>
struct PartialM {
    float mx, den;
    float acc[NK * 8];
    __device__ __forceinline__ void init()
    {
        mx = -INFINITY;
        den = 0.f;
#pragma unroll
        for (int i = 0; i < NK * 8; ++i) acc[i] = 0.f;
    }
    __device__ __forceinline__ void raise(float b)
    {
        if (b > mx + kLazy || mx == -INFINITY) {
            const float sc = __expf(mx - b);  // mx = -inf gives 0
            den *= sc;
#pragma unroll
            for (int i = 0; i < NK * 8; ++i) acc[i] *= sc;
            mx = b;
        }
    }
};

template <int NK, int G, bool UPD, bool ATT>
__device__ __forceinline__ void token_step_mfma(const State &st, const size_t sid, const char *krow, const char *vrow,
                                                const char *qrows, float *outrows, const int64_t n_seen, int &m,
                                                double &mu, SmemMfma<NK, G> &sm)
{
    constexpr int LPR = 4 * NK;          // lanes per row in the plain row layout (copies, norms)
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)NK * 64;
    constexpr int D = NK * 32;
    constexpr bool KSEP = UPD && ATT && G == 4;   // four queries fill the replicated rows: the key gets its own MFMA
    constexpr int KROW = ATT ? G : 0;             // A row (mod 4) that carries the evicted key otherwise
    constexpr int KIDX = KSEP ? 0 : (KROW & 3);   // result register of the key's dot product
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR;   // plain row layout
    const int grp = wave * RPW + sub;
    const int n16 = lane & 15, L = lane >> 4;        // MFMA layout: row n16 of a 16-row group, K slice L

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.Mcap;
    float *const xn = st.xn + sid * (size_t)st.Mcap;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;

    // ---- A operands: queries in rows 4L'+r (r < G), the evicted key in row KROW (or its own operand)
    const int arow = n16 & 3;
    uint4 Aq[NK], Ak[KSEP ? NK : 1];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) Aq[kk] = make_uint4(0, 0, 0, 0);
    if constexpr (KSEP) {
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) Ak[kk] = make_uint4(0, 0, 0, 0);
    }
    if constexpr (ATT) {
        if (arow < G) {
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) Aq[kk] = ld16(qrows + (size_t)arow * ROWB + (L + 4 * kk) * 16);
        }
    }

    // ---- window push; the token that leaves the window is the one that is compressed
    bool evict = false;
    int64_t etoken = 0;
    uint4 ek = make_uint4(0, 0, 0, 0), ev = make_uint4(0, 0, 0, 0);
    if constexpr (UPD) {
        const char *esk = krow, *esv = vrow;
        char *kw = nullptr, *vw = nullptr;
        if (st.w == 0) {
            evict = true;
            etoken = n_seen;
        } else {
            const int slot = (int)(n_seen % st.w);
            kw = Kw + (size_t)slot * ROWB;
            vw = Vw + (size_t)slot * ROWB;
            esk = kw;
            esv = vw;
            if (n_seen >= st.w) {
                evict = true;
                etoken = n_seen - st.w;
            }
        }
        if (evict) {
            ek = ld16(esk + col * 16);
            ev = ld16(esv + col * 16);
            if (KSEP ? arow == 0 : arow == KROW) {
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) {
                    const uint4 t = ld16(esk + (L + 4 * kk) * 16);
                    if constexpr (KSEP) Ak[kk] = t;
                    else Aq[kk] = t;
                }
            }
        }
        if (st.w > 0) {
            __syncthreads();  // every lane holds the evicted row before the slot is overwritten
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
    }

    PartialM<NK> part[G];
#pragma unroll
    for (int g = 0; g < G; ++g) part[g].init();

    // ---- one pass over the representatives, 16 rows per wavefront step, two steps in flight
    float b1 = INFINITY, b2 = INFINITY, nxmax = 0.f;
    int i1 = -1;
    if ((UPD && evict) || ATT) {
        constexpr int U = 2;
        for (int r0 = wave * 16; r0 < m; r0 += 16 * kWaves * U) {
            uint4 b[U][NK];
            float nx[U], cf[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * 16 * kWaves + n16;
                const int rr = r < m ? r : m - 1;
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) b[u][kk] = ld16(X + (size_t)rr * ROWB + (L + 4 * kk) * 16);
                nx[u] = UPD ? xn[rr] : 0.f;
                cf[u] = ATT ? (float)cnt[rr] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * 16 * kWaves + n16;
                const bool valid = r < m;
                floatx4_t c = {0.f, 0.f, 0.f, 0.f}, ck = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(Aq[kk], b[u][kk], c);
                if constexpr (KSEP) {
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) ck = mfma_bf16(Ak[kk], b[u][kk], ck);
                }
                if constexpr (UPD) {
                    if (evict && valid) {
                        const float dotk = KSEP ? ck[KIDX] : c[KIDX];
                        const float dt = fmaf(-2.f, dotk, nx[u] + nk);
                        if (dt < b1) {
                            b2 = b1;
                            b1 = dt;
                            i1 = r;
                        } else if (dt < b2) {
                            b2 = dt;
                        }
                        nxmax = fmaxf(nxmax, nx[u]);
                    }
                }
                if constexpr (ATT) {
                    if (valid) {
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            part[g].raise(c[g]);
                            part[g].den = fmaf(cf[u], __expf(c[g] - part[g].mx), part[g].den);
                        }
                    }
                }
            }
        }
    }

    if constexpr (UPD) {
        if (evict) {
            // ---- best / runner-up of the approximate distances over the workgroup
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) {
                const float ob1 = __shfl_xor(b1, o), ob2 = __shfl_xor(b2, o);
                const int oi1 = __shfl_xor(i1, o);
                if (ob1 < b1 || (ob1 == b1 && (uint32_t)oi1 < (uint32_t)i1)) {
                    b2 = fminf(b1, ob2);
                    b1 = ob1;
                    i1 = oi1;
                } else {
                    b2 = fminf(b2, ob1);
                }
                nxmax = fmaxf(nxmax, __shfl_xor(nxmax, o));
            }
            if (lane == 0) {
                sm.wb1[wave] = b1;
                sm.wb2[wave] = b2;
                sm.wi1[wave] = i1;
                sm.wnx[wave] = nxmax;
            }
            __syncthreads();
            b1 = sm.wb1[0]; b2 = sm.wb2[0]; i1 = sm.wi1[0]; nxmax = sm.wnx[0];
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) {
                const float ob1 = sm.wb1[wv], ob2 = sm.wb2[wv];
                const int oi1 = sm.wi1[wv];
                if (ob1 < b1 || (ob1 == b1 && (uint32_t)oi1 < (uint32_t)i1)) {
                    b2 = fminf(b1, ob2);
                    b1 = ob1;
                    i1 = oi1;
                } else {
                    b2 = fminf(b2, ob1);
                }
                nxmax = fmaxf(nxmax, sm.wnx[wv]);
            }
            // ---- decide from D~ when the error bound allows it, else re-evaluate exactly
            const float thr = (float)st.delta2;
            const float emax = kDistEps * (nxmax + nk);
            bool join;
            int bidx = i1;
            const bool ambiguous = m > 0 && (!(b2 - b1 > 2.f * emax) || !(fabsf(b1 - thr) > emax + 1e-6f * thr));
            if (ambiguous) {
                double best;
                exact_nearest<LPR>(X, m, ek, sm.wbest, sm.widx, best, bidx);
                join = bidx >= 0 && best <= st.delta2;
            } else {
                join = m > 0 && b1 <= thr;
            }
            const bool forced = !join && m > 0 && m >= st.Mcap;
            const bool created = !join && !forced;
            const int target = created ? m : bidx;
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
            float p;
            if (mu == 0.0) p = 1.f;
            else if (vn == 0.f) p = 0.f;
            else p = (float)((double)vn / (mu + (double)vn));
            for (int base = 0; base < st.s; base += kQueue) {
                if (tid == 0) sm.qn = 0;
                __syncthreads();
                const int j0 = base + tid * 4;
                if (j0 < st.s && p > 0.f) {
                    uint32_t r[4];
                    philox4x32_10((uint32_t)(j0 >> 2), (uint32_t)etoken, (uint32_t)((uint64_t)etoken >> 32),
                                  (uint32_t)sid, st.seed_lo, st.seed_hi, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float u = (float)(r[i] >> 8) * (1.0f / 16777216.0f);
                        if (j0 + i < st.s && u < p) sm.queue[atomicAdd(&sm.qn, 1)] = j0 + i;
                    }
                }
                __syncthreads();
                const int nq = sm.qn;
                for (int e = grp; e < nq; e += RPB) {
                    const int j = sm.queue[e];
                    st16(Ks + (size_t)j * ROWB + col * 16, ek);
                    st16(Vs + (size_t)j * ROWB + col * 16, ev);
                    if (col == 0) {
                        st.sidx[sid * (size_t)st.s + j] = (int32_t)etoken;
                        st.svn[sid * (size_t)st.s + j] = vn;
                    }
                }
                __syncthreads();
            }
            mu += (double)vn;
        }
        __syncthreads();  // window slot, center row and sample rows are visible to the whole workgroup
    }

    if constexpr (ATT) {
        const bool extra = UPD && evict;
        // ---- sampled pairs: numerator terms  mu/(s ||v_j||^2) e^{<q,k_j>} v_j
        if (n_evicted_after > 0) {
            const float wmul = (float)(mu / (double)st.s);
            const float *svn = st.svn + sid * (size_t)st.s;
            for (int r0 = wave * 16; r0 < st.s; r0 += 16 * kWaves) {
                const int r = r0 + n16;
                const bool valid = r < st.s;
                const int rr = valid ? r : st.s - 1;
                uint4 bk[NK], bv[NK];
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) bk[kk] = ld16(Ks + (size_t)rr * ROWB + (L + 4 * kk) * 16);
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) bv[kk] = ld16(Vs + (size_t)rr * ROWB + (L + 4 * kk) * 16);
                const float vnj = svn[rr];
                floatx4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(Aq[kk], bk[kk], c);
                const float wgt = (valid && vnj > 0.f) ? wmul / vnj : 0.f;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (valid) part[g].raise(c[g]);
                    const float e = valid ? wgt * __expf(c[g] - part[g].mx) : 0.f;
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) {
                        float vf[8];
                        unpack<true>(bv[kk], vf);
#pragma unroll
                        for (int i = 0; i < 8; ++i) part[g].acc[kk * 8 + i] = fmaf(e, vf[i], part[g].acc[kk * 8 + i]);
                    }
                }
            }
        }
        // ---- window: exact terms in numerator and normaliser
        const int fill = (int)(n_after < st.w ? n_after : st.w);
        for (int r0 = wave * 16; r0 < fill; r0 += 16 * kWaves) {
            const int r = r0 + n16;
            const bool valid = r < fill;
            const int rr = valid ? r : fill - 1;
            uint4 bk[NK], bv[NK];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) bk[kk] = ld16(Kw + (size_t)rr * ROWB + (L + 4 * kk) * 16);
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) bv[kk] = ld16(Vw + (size_t)rr * ROWB + (L + 4 * kk) * 16);
            floatx4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(Aq[kk], bk[kk], c);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (valid) part[g].raise(c[g]);
                const float e = valid ? __expf(c[g] - part[g].mx) : 0.f;
                part[g].den += e;
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) {
                    float vf[8];
                    unpack<true>(bv[kk], vf);
#pragma unroll
                    for (int i = 0; i < 8; ++i) part[g].acc[kk * 8 + i] = fmaf(e, vf[i], part[g].acc[kk * 8 + i]);
                }
            }
        }
        // ---- merge the 16 lanes of each DPP row, then the wavefronts through LDS
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float M = row_max16(part[g].mx);
            const float sc = (part[g].mx == -INFINITY) ? 0.f : __expf(part[g].mx - M);
            const float den = row_sum16(part[g].den * sc);
            if (lane == 0) {
                sm.wmx[wave][g] = M;
                sm.wden[wave][g] = den;
            }
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float a = row_sum16(part[g].acc[kk * 8 + i] * sc);
                    if (n16 == 0) sm.wacc[wave][g][(L + 4 * kk) * 8 + i] = a;
                }
            }
        }
        __syncthreads();
        for (int i = tid; i < G * D; i += kWG) {
            const int g = i / D, c = i % D;
            const float bx = extra ? sm.bx[g] : -INFINITY;
            float M = bx;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) M = fmaxf(M, sm.wmx[wv][g]);
            float den = extra ? __expf(bx - M) : 0.f, num = 0.f;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) {
                const float wm = sm.wmx[wv][g];
                const float sc = (wm == -INFINITY) ? 0.f : __expf(wm - M);
                den = fmaf(sm.wden[wv][g], sc, den);
                num = fmaf(sm.wacc[wv][g][c], sc, num);
            }
            outrows[(size_t)g * D + c] = num / den;
        }
    }
    __syncthreads();  // LDS and state are reusable by the next token
}

// at least two workgroups per CU (two wavefronts per SIMD) even for the widest accumulator sets
template <int NK, int G, bool UPD, bool ATT>
__global__ __launch_bounds__(kWG, 2) void decode_mfma_kernel(const State st, const Call call)
{
    __shared__ SmemMfma<NK, G> sm;
    const size_t sid = blockIdx.x;
    int m = st.m[sid];
    double mu = st.mu[sid];
    const size_t rowb = (size_t)NK * 64;
    const char *krow = UPD ? call.K + sid * call.stream_stride : nullptr;
    const char *vrow = UPD ? call.V + sid * call.stream_stride : nullptr;
    const char *qrows = ATT ? call.Q + sid * G * rowb : nullptr;
    float *outrows = ATT ? call.out + sid * (size_t)G * NK * 32 : nullptr;
    token_step_mfma<NK, G, UPD, ATT>(st, sid, krow, vrow, qrows, outrows, call.n_seen, m, mu, sm);
    if constexpr (UPD) {
        if (threadIdx.x == 0) {
            st.m[sid] = m;
            st.mu[sid] = mu;
        }
    }
}

}  // namespace sg
