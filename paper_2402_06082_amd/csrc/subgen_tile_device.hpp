// bf16 decode step (attend, or update + attend) for a few queries per stream with every contraction on the
// matrix cores and the stored rows staged through LDS tiles.
//
// One workgroup per stream.  All 256 lanes load 128 rows at a time with whole-row 16-byte accesses into four
// 32-row tiles in LDS (the next 128 rows are in flight while the current ones are consumed); wavefront w takes
// tile w:
//
//   scores   C[row][col] = <row, vector(col)>:  A = 16 stored rows out of the tile, B = the vectors in
//            registers: columns 0..G-1 the queries, columns G..G+7 the key that leaves the window (update).
//            Lane (n, L) = lane 16L + n gets rows 4L..4L+3 and 16+4L..16+4L+3 of the tile against column n.
//   representatives: query columns add n_i e^{score} to the normaliser; the key column turns its scores into
//            approximate squared distances ||x_i||^2 + ||k||^2 - 2<x_i,k> and keeps best / runner-up.
//            The decision is taken from them only when the gap and the distance to delta^2 exceed the
//            error bound, else the workgroup re-evaluates every distance in double precision.
//   sampled pairs, window: weights e = w_row e^{score - mx}; O[col][c] += sum_row e[row][col] V[row][c] is a
//            second contraction: A = the lane's eight weights as they are (slot 8L + j <-> row 4L + j, j < 4,
//            row 16 + 4L + j - 4 otherwise), B = the value rows in the same slot order, read transposed out of
//            the row-major value tile with ds_read_b64_tr_b16.  Weights enter as a bf16 pair hi + lo.
//
// The softmax reference mx of a query is shared by its four lanes and raised lazily.  At the end the four
// wavefronts (four row splits) are merged through LDS.
#pragma once
#include <type_traits>

#include "subgen_mfma_device.hpp"

namespace sg {

constexpr int kTileRows = 32;
constexpr int kTiles = 4;                       // tiles staged per iteration of a four-wavefront workgroup
constexpr int kSuper = kTileRows * kTiles;      // rows staged per iteration

// NWV wavefronts per workgroup = tiles staged per iteration
template <int NK, int G, int NWV>
struct SmemTile {
    static constexpr int kWaves = NWV, kTiles = NWV, kSuper = kTileRows * NWV;
    static constexpr int KS = NK * 64 + 16;   // key tile row stride (bytes): 16-byte operand reads hit distinct banks
    static constexpr int VS = NK * 64 + 32;   // value tile row stride: the transposing reads hit distinct banks
    alignas(16) char kt[kTiles][kTileRows * KS];
    alignas(16) char vt[kTiles][kTileRows * VS];
    alignas(16) float wrow[kSuper];           // weight of each staged row
    alignas(16) float xnrow[kSuper];          // ||x_i||^2 of each staged representative (update)
    alignas(16) uint4 ekrow[NK * 4], evrow[NK * 4];   // the evicted (key, value) rows, for the sampling copies
    alignas(16) uint4 qrow[G][NK * 4];                // the queries in plain row layout (extra normaliser term)
    float wb1[kWaves], wb2[kWaves], wb3[kWaves], wnx[kWaves];
    int wi1[kWaves], wi2[kWaves];
    double wbest[kWaves];
    int widx[kWaves];
    float bx[G];
    float wmx[kWaves][16], wden[kWaves][16];
};

template <int NK, int G, bool UPD, int NWV>
__global__ __launch_bounds__(64 * NWV, 2) void decode_tile_kernel(const State st, const Call call)
{
    // workgroup shape of this kernel (these names hide the library-wide ones): NWV wavefronts, one tile per
    // wavefront and iteration
    constexpr int kWG = 64 * NWV, kWaves = NWV, kSuper = kTileRows * NWV;
    static_assert(G + 8 <= 16, "the queries and the eight key copies share the 16 operand columns");
    constexpr int CPR = 4 * NK;              // 16-byte chunks per row
    constexpr int LPR = CPR;                 // lanes per row in the plain row layout (copies, norms)
    constexpr int RPW = 64 / LPR;
    constexpr size_t ROWB = (size_t)NK * 64;
    constexpr int D = NK * 32;
    constexpr int NCB = NK * 2;              // 16-column blocks of the output
    constexpr int KS = SmemTile<NK, G, NWV>::KS, VS = SmemTile<NK, G, NWV>::VS;
    constexpr int LD = kSuper * CPR / kWG;   // 16-byte loads per thread and operand per iteration
    __shared__ SmemTile<NK, G, NWV> sm;

    const size_t sid = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, L = lane >> 4;
    const int col = lane % LPR, sub = lane / LPR, grp = wave * RPW + sub;   // plain row layout
    // operand columns: 0..G-1 the queries; G..G+7 eight copies of the key that leaves the window, copy j looks
    // after row j of the eight rows a lane sees per tile (so the nearest-representative search costs every
    // lane one candidate per tile instead of eight for a few)
    const bool qcol = n16 < G, kcol = UPD && n16 >= G && n16 < G + 8;
    const int kj = n16 - G;

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    float *const xn = st.xn + sid * (size_t)st.McapS;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;
    const float *const svn = st.svn + sid * (size_t)st.sS;
    const char *const krow = UPD ? call.K + sid * call.stream_stride : nullptr;
    const char *const vrow = UPD ? call.V + sid * call.stream_stride : nullptr;
    const char *const qrows = call.Q + sid * call.q_stride;
    float *const outrows = out_rows(st, call.out, sid * call.out_stride);
    const int64_t n_seen = tokens_seen(st, call.n_seen);
    int m = st.m[sid];
    double mu = st.mu[sid];

    // ---- B operand: queries in columns 0..G-1, the evicted key in columns G..G+7, zeros elsewhere
    uint4 Bq[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) Bq[kk] = make_uint4(0, 0, 0, 0);
    if (qcol) {
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) Bq[kk] = ld16(qrows + (size_t)n16 * ROWB + (L + 4 * kk) * 16);
    }
    if constexpr (UPD) {
        if (tid < G * LPR) sm.qrow[tid / LPR][tid % LPR] = ld16(qrows + (size_t)tid * 16);   // read after many barriers
    }

    // The stored rows come in three sections: 0 = representatives (weight n_i, normaliser only; distances for
    // the key column), 2 = window (weight 1, numerator and normaliser), 1 = sampled pairs (weight
    // mu/(s ||v||^2), numerator only).  They run through one software pipeline of 128-row blocks:
    //   prefetch (global -> registers)  ->  stage (registers -> LDS tiles, row weights)  ->  compute (tiles).
    // The prefetch of a block is issued before the compute of the block in front of it, across the section
    // boundaries as well, so the only time without loads in flight is the decision of the update, and the
    // window rows are on their way during that.
    uint4 rk[LD], rv[LD];
    auto prefetch = [&](const bool hasv, const char *Kb, const char *Vb, const int nrows, const int r0) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int idx = tid + kWG * i, row = idx / CPR, ch = idx % CPR;
            const int rr = r0 + row < nrows ? r0 + row : nrows - 1;
            rk[i] = ldnt16(Kb + (size_t)rr * ROWB + ch * 16);
            if (hasv) rv[i] = ldnt16(Vb + (size_t)rr * ROWB + ch * 16);
        }
    };
    const int fill0 = (int)(n_seen < st.w ? n_seen : st.w);   // window rows before this call's token
    if (m > 0) prefetch(false, X, X, m, 0);   // on its way during the window push below
    else if (!UPD && fill0 > 0) prefetch(true, Kw, Vw, fill0, 0);

    // ---- window push; the token that leaves the window is the one that is compressed.  The lanes that copy the
    //      new token into the ring slot first move the slot's old rows into LDS (same lane, same addresses: the
    //      loads are served before the stores); everybody else picks them up there after the next barrier.
    bool evict = false;
    int64_t etoken = 0;
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
        if (tid < LPR) {
            if (evict) {
                sm.ekrow[tid] = ld16(esk + tid * 16);
                sm.evrow[tid] = ld16(esv + tid * 16);
            }
            if (st.w > 0) {
                st16(kw + tid * 16, ld16(krow + tid * 16));
                st16(vw + tid * 16, ld16(vrow + tid * 16));
            }
        }
    }
    const int64_t n_after = UPD ? n_seen + 1 : n_seen;
    const int64_t n_evicted_after = st.w == 0 ? n_after : (n_after > st.w ? n_after - st.w : 0);

    // after the first barrier: the evicted rows out of LDS; ||k'||^2 and ||v'||^2 in double from the exactly
    // converted elements; the key as operand column G
    uint4 ek = make_uint4(0, 0, 0, 0);
    float nk = 0.f, vn = 0.f;
    auto take_evicted = [&]() {
        if constexpr (UPD) {
            if (!evict) return;
            ek = sm.ekrow[col];
            const uint4 ev = sm.evrow[col];
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
            if (!token_is_finite(nk, vn)) {   // NaN or Inf in the token: dropped and flagged
                evict = false;
                if (tid == 0) st.flags[sid] |= 2u;
                return;
            }
            if (kcol) {
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) Bq[kk] = sm.ekrow[L + 4 * kk];
            }
        }
    };

    float mx = -INFINITY, den = 0.f;   // per query column; mx is the same in the four lanes of a column
    floatx4_t acc[NCB];                // O[column 4L + r][output column 16 cb + n16]
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[cb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    Cand3 cd;   // nearest representatives of the evicted key by approximate distance (key columns)
    float nxmax = 0.f;

    // full: global memory written by other lanes of the workgroup since the last full barrier is read after it
    auto stage = [&](auto kind_c, const int nrows, const int r0, const float mus, const bool full) {
        constexpr int KIND = decltype(kind_c)::value;
        constexpr bool HASV = KIND != 0, DIST = KIND == 0 && UPD;
        if (full) __syncthreads();
        else lds_barrier();   // the previous tiles have been consumed
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int idx = tid + kWG * i, row = idx / CPR, ch = idx % CPR;
            *reinterpret_cast<uint4 *>(&sm.kt[row / kTileRows][(row % kTileRows) * KS + ch * 16]) = rk[i];
            if constexpr (HASV)
                *reinterpret_cast<uint4 *>(&sm.vt[row / kTileRows][(row % kTileRows) * VS + ch * 16]) = rv[i];
        }
        if (tid < kSuper) {
            const int r = r0 + tid;
            float wv = 0.f, xv = 0.f;
            if (r < nrows) {
                if constexpr (KIND == 0) {
                    wv = (float)cnt[r];
                    if constexpr (DIST) xv = xn[r];
                } else if constexpr (KIND == 1) {
                    const float v2 = svn[r];
                    wv = v2 > 0.f ? mus / v2 : 0.f;
                } else {
                    wv = 1.f;
                }
            }
            sm.wrow[tid] = wv;
            if constexpr (DIST) sm.xnrow[tid] = xv;
        }
        lds_barrier();
    };
    auto compute = [&](auto kind_c, const int nrows, const int r0) {
        constexpr int KIND = decltype(kind_c)::value;
        constexpr bool HASV = KIND != 0, TODEN = KIND != 1, DIST = KIND == 0 && UPD;
        const int t = wave, trow = r0 + t * kTileRows;
        if (trow >= nrows) return;   // (whole wavefront; no barrier below)
        // ---- scores of the tile's 32 rows against the 16 columns
        floatx4_t c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
            const uint4 a0 = *reinterpret_cast<const uint4 *>(&sm.kt[t][n16 * KS + (L + 4 * kk) * 16]);
            const uint4 a1 = *reinterpret_cast<const uint4 *>(&sm.kt[t][(16 + n16) * KS + (L + 4 * kk) * 16]);
            c0 = mfma_bf16(a0, Bq[kk], c0);
            c1 = mfma_bf16(a1, Bq[kk], c1);
        }
        if constexpr (DIST) {
            if (kcol && evict) {
                const float4 x0 = *reinterpret_cast<const float4 *>(&sm.xnrow[t * kTileRows + 4 * L]);
                const float4 x1 = *reinterpret_cast<const float4 *>(&sm.xnrow[t * kTileRows + 16 + 4 * L]);
                const int jr = kj & 3;
                const floatx4_t cs = kj < 4 ? c0 : c1;
                const float4 xs = kj < 4 ? x0 : x1;
                const float sc = jr == 0 ? cs[0] : (jr == 1 ? cs[1] : (jr == 2 ? cs[2] : cs[3]));
                const float nx = jr == 0 ? xs.x : (jr == 1 ? xs.y : (jr == 2 ? xs.z : xs.w));
                const int row = trow + (kj < 4 ? 0 : 16) + 4 * L + jr;   // ascending from tile to tile
                if (row < nrows) {
                    cd.insert(fmaf(-2.f, sc, nx + nk), row);
                    nxmax = fmaxf(nxmax, nx);
                }
            }
        }
        if (!qcol) {   // the other columns take no part in the softmax
            c0 = floatx4_t{0.f, 0.f, 0.f, 0.f};
            c1 = floatx4_t{0.f, 0.f, 0.f, 0.f};
        }
        const float4 w0 = *reinterpret_cast<const float4 *>(&sm.wrow[t * kTileRows + 4 * L]);
        const float4 w1 = *reinterpret_cast<const float4 *>(&sm.wrow[t * kTileRows + 16 + 4 * L]);
        // ---- lazy softmax reference (rows beyond nrows repeat the last row, so every score is a real one)
        float lm = fmaxf(fmaxf(fmaxf(c0[0], c0[1]), fmaxf(c0[2], c0[3])),
                         fmaxf(fmaxf(c1[0], c1[1]), fmaxf(c1[2], c1[3])));
        if (__any(lm > mx + kLazy || mx == -INFINITY)) {
            lm = fmaxf(lm, __shfl_xor(lm, 16));
            lm = fmaxf(lm, __shfl_xor(lm, 32));
            float scale = 1.f;
            if (lm > mx + kLazy || mx == -INFINITY) {
                scale = __expf(mx - lm);   // mx = -inf gives 0
                den *= scale;
                mx = lm;
            }
            if constexpr (HASV) {
                // the accumulators hold columns 4L + r: fetch their factors from the lanes of those columns
                float sr[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) sr[r] = __shfl(scale, 4 * L + r);
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[cb][r] *= sr[r];
            }
        }
        float e[8];
        e[0] = w0.x * __expf(c0[0] - mx); e[1] = w0.y * __expf(c0[1] - mx);
        e[2] = w0.z * __expf(c0[2] - mx); e[3] = w0.w * __expf(c0[3] - mx);
        e[4] = w1.x * __expf(c1[0] - mx); e[5] = w1.y * __expf(c1[1] - mx);
        e[6] = w1.z * __expf(c1[2] - mx); e[7] = w1.w * __expf(c1[3] - mx);
        if constexpr (TODEN) den += ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
        if constexpr (HASV) {
            // ---- weights as bf16 hi + lo, in contraction-slot order (slot j <-> e[j])
            uint4 ah, al;
            ah.x = pack_bf16(e[0], e[1]); ah.y = pack_bf16(e[2], e[3]);
            ah.z = pack_bf16(e[4], e[5]); ah.w = pack_bf16(e[6], e[7]);
            al.x = pack_bf16(e[0] - bf16_lo(ah.x), e[1] - bf16_hi(ah.x));
            al.y = pack_bf16(e[2] - bf16_lo(ah.y), e[3] - bf16_hi(ah.y));
            al.z = pack_bf16(e[4] - bf16_lo(ah.z), e[5] - bf16_hi(ah.z));
            al.w = pack_bf16(e[6] - bf16_lo(ah.w), e[7] - bf16_hi(ah.w));
            const char *v0 = &sm.vt[t][(4 * L + (n16 >> 2)) * VS + (n16 & 3) * 8];
            const char *v1 = v0 + 16 * VS;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const u32x2_t t0 = lds_read_tr16(v0 + cb * 32), t1 = lds_read_tr16(v1 + cb * 32);
                const uint4 b = make_uint4(t0[0], t0[1], t1[0], t1[1]);
                acc[cb] = mfma_bf16(ah, b, acc[cb]);
                acc[cb] = mfma_bf16(al, b, acc[cb]);
            }
        }
    };
    auto blocks = [](const int nrows) { return (nrows + kSuper - 1) / kSuper; };

    using K0 = std::integral_constant<int, 0>;
    using K1 = std::integral_constant<int, 1>;
    using K2 = std::integral_constant<int, 2>;
    const int fill = (int)(n_after < st.w ? n_after : st.w);
    // the window rows are prefetched before the decision of the update; its own push into the ring (above) is
    // ordered before these loads by the barriers of the stages in between, or by this one
    if constexpr (UPD) {
        if (m == 0) {
            __syncthreads();
            take_evicted();
            if (fill > 0) prefetch(true, Kw, Vw, fill, 0);
        }
    }

    // ---- representatives: normaliser terms n_i e^{<q,x_i>} and, for the update, the nearest one
    {
        const int nb = blocks(m);
        for (int b = 0; b < nb; ++b) {
            stage(K0{}, m, b * kSuper, 0.f, UPD && b == 0);
            if (b + 1 < nb) prefetch(false, X, X, m, (b + 1) * kSuper);
            else if (fill > 0) prefetch(true, Kw, Vw, fill, 0);
            if (b == 0) take_evicted();
            compute(K0{}, m, b * kSuper);
        }
    }

    bool extra = false, decided = false, d_created = false, d_forced = false;
    int d_target = 0;
    uint4 xg = make_uint4(0, 0, 0, 0);
    auto finish_extra = [&]() {
        if (extra && grp == 0) {
            float xf[8];
            unpack<true>(xg, xf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float qf[8];
                unpack<true>(sm.qrow[g][col], qf);
                float a = 0.f;
#pragma unroll
                for (int v = 0; v < 8; ++v) a = fmaf(qf[v], xf[v], a);
                a = group_sum<LPR>(a);
                if (col == 0) sm.bx[g] = a;
            }
        }
    };
    if constexpr (UPD) {
        if (evict) {
            // ---- the nearest candidates: over the lanes (the other columns hold +inf): the 16 lanes of a DPP row
            //      by rotations, then the four rows; then the wavefronts
            auto merge = [&](const float ob1, const int oi1, const float ob2, const int oi2, const float ob3,
                             const float onx) __attribute__((always_inline)) {
                cd.merge(ob1, oi1, ob2, oi2, ob3);
                nxmax = fmaxf(nxmax, onx);
            };
            merge(row_ror<8>(cd.b1), row_ror<8>(cd.i1), row_ror<8>(cd.b2), row_ror<8>(cd.i2), row_ror<8>(cd.b3), row_ror<8>(nxmax));
            merge(row_ror<4>(cd.b1), row_ror<4>(cd.i1), row_ror<4>(cd.b2), row_ror<4>(cd.i2), row_ror<4>(cd.b3), row_ror<4>(nxmax));
            merge(row_ror<2>(cd.b1), row_ror<2>(cd.i1), row_ror<2>(cd.b2), row_ror<2>(cd.i2), row_ror<2>(cd.b3), row_ror<2>(nxmax));
            merge(row_ror<1>(cd.b1), row_ror<1>(cd.i1), row_ror<1>(cd.b2), row_ror<1>(cd.i2), row_ror<1>(cd.b3), row_ror<1>(nxmax));
#pragma unroll
            for (int o = 16; o < 64; o <<= 1)
                merge(__shfl_xor(cd.b1, o), __shfl_xor(cd.i1, o), __shfl_xor(cd.b2, o), __shfl_xor(cd.i2, o),
                      __shfl_xor(cd.b3, o), __shfl_xor(nxmax, o));
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
                exact_decide<LPR, NWV>(X, m, ek, cd, emax, sm.wbest, sm.widx, best, bidx);
                join = bidx >= 0 && best <= st.delta2;
            } else {
                join = m > 0 && cd.b1 <= thr;
            }
            const Decision dec = decide_cluster(join, bidx, m, st.Mcap);
            const bool forced = dec.forced, created = dec.created;
            const int target = dec.target;
            // the cluster table itself is written at the very end of the kernel: nothing below reads it, and a
            // barrier in between would have to wait for those stores to be acknowledged
            decided = true;
            d_created = created;
            d_forced = forced;
            d_target = target;
            // score of the cluster that gained this token, one more term of the normaliser: its row is only
            // requested here (the queries sit in LDS); the products wait until the load has landed (after the
            // next full barrier), so no wavefront sits out its latency
            if (grp == 0) {
                xg = ek;
                if (!created) xg = ld16(X + (size_t)target * ROWB + col * 16);
            }
            extra = true;
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
    }

    // ---- window: exact terms in numerator and normaliser (its first block was prefetched above); the sampled
    //      rows are final by now, so their first block goes in flight behind the window's last one
    const float mus = (float)(mu / (double)st.s);
    const bool have_samples = n_evicted_after > 0;
    {
        const int nb = blocks(fill);
        for (int b = 0; b < nb; ++b) {
            stage(K2{}, fill, b * kSuper, 0.f, UPD && b == 0);   // full: the sampled rows written by the update
            if (b + 1 < nb) prefetch(true, Kw, Vw, fill, (b + 1) * kSuper);
            else if (have_samples) prefetch(true, Ks, Vs, st.s, 0);
            if constexpr (UPD) {
                if (b == 0) finish_extra();
            }
            compute(K2{}, fill, b * kSuper);
        }
        if (nb == 0) {
            if constexpr (UPD) {
                __syncthreads();
                finish_extra();
            }
            if (have_samples) prefetch(true, Ks, Vs, st.s, 0);
        }
    }
    // ---- sampled pairs: numerator terms mu/(s ||v_j||^2) e^{<q,k_j>} v_j
    if (have_samples) {
        const int nb = blocks(st.s);
        for (int b = 0; b < nb; ++b) {
            stage(K1{}, st.s, b * kSuper, mus, false);
            if (b + 1 < nb) prefetch(true, Ks, Vs, st.s, (b + 1) * kSuper);
            compute(K1{}, st.s, b * kSuper);
        }
    }

    // ---- totals per wavefront, then the four row splits are merged through LDS
    den += __shfl_xor(den, 16);
    den += __shfl_xor(den, 32);
    __syncthreads();   // the tiles are dead: their memory carries the accumulators
    float *const accbuf = reinterpret_cast<float *>(&sm.kt[0][0]);   // [wave][16 columns][D]
    static_assert(sizeof(sm.kt) >= (size_t)kWaves * 16 * D * sizeof(float), "accumulators fit in the key tiles");
    if (L == 0) {
        sm.wmx[wave][n16] = mx;
        sm.wden[wave][n16] = den;
    }
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (4 * L + r < G) accbuf[((size_t)wave * 16 + 4 * L + r) * D + cb * 16 + n16] = acc[cb][r];
    __syncthreads();
    for (int i = tid; i < G * D; i += kWG) {
        const int g = i / D, c = i % D;
        const float bx = extra ? sm.bx[g] : -INFINITY;
        float M = bx;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) M = fmaxf(M, sm.wmx[wv][g]);
        float dn = extra ? __expf(bx - M) : 0.f, num = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) {
            const float wm = sm.wmx[wv][g];
            if (wm != -INFINITY) {
                const float sc = __expf(wm - M);
                dn = fmaf(sm.wden[wv][g], sc, dn);
                num = fmaf(accbuf[((size_t)wv * 16 + g) * D + c], sc, num);
            }
        }
        put_out(st, outrows, (size_t)g * D + c, num / dn);
    }

    // ---- the update's writes to the cluster table (see the decision above)
    if constexpr (UPD) {
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
        if (tid == 0) {
            st.m[sid] = m;
            st.mu[sid] = mu;
        }
    }
}

}  // namespace sg
