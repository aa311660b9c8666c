// Many queries per stream against the compressed state (QueryStreamAttn of Algorithm 1 with the window of
// Section 3.2, evaluated for a whole block of queries at once): bf16, matrix cores for both contractions.
//
// With 16 or more queries per stream the query-key scores and the weight-value products are real dense
// contractions, so the state of a stream is read from HBM once per workgroup into LDS tiles of 32 rows and
// every wavefront runs v_mfma_f32_16x16x32_bf16 on them for its own 16 queries:
//
//   scores   C[row][query] = sum_c K[row][c] Q[query][c]      A = 16 stored rows (k = 8L..8L+7 of each 32-wide
//                                                              slice, straight out of the row-major LDS tile),
//                                                              B = the wavefront's 16 queries (registers).
//            Lane (n, L) = lane 16L + n ends up with the scores of rows 4L..4L+3 (first 16 rows of the tile)
//            and 16+4L..16+4L+3 (second 16 rows) against query n.
//   weights  e = w_row exp(score - mx_query): w_row = n_i for representatives (normaliser only),
//            mu / (s ||v_j||^2) for sampled pairs (numerator only), 1 for window rows (both).
//   output   O[query][col] += sum_row e[row][query] V[row][col]   A = the eight weights of lane (n, L) as they
//            are (contraction slot 8L + j <-> row 4L + j for j < 4, row 16 + 4L + j - 4 otherwise),
//            B = V in the same slot order: lane (col, L) needs rows 4L..4L+3 and 16+4L..16+4L+3 of one
//            column, which ds_read_b64_tr_b16 delivers from the row-major tile (each 16-lane group reads a
//            4 rows x 16 columns patch and gets it back transposed: lane i receives column i).
//            The weights go in as a bf16 pair hi + lo (two MFMAs), so the product keeps ~16 mantissa bits.
//
// The softmax reference mx is per query and shared by the three kinds of rows; it is raised lazily (only when
// a score exceeds it by kLazy), and then the accumulators are rescaled.
//
// Workgroup = one stream x 16*QT*QW queries; the four wavefronts are QT query groups x 4/QT row splits, and a
// wavefront answers QW tiles of 16 queries with every operand it reads from LDS (QW = 2 for large blocks: the
// key and value tiles are then read once per 32 queries, which moves the bound from LDS reads to the matrix
// cores).  Every iteration stages 128 rows (four tiles); a wavefront takes the tiles of its row split.
#pragma once
#include <type_traits>

#include "subgen_tile_device.hpp"

namespace sg {

// max(a, b, c) as the one instruction it is (fmaxf first quiets each operand with an instruction of its own)
__device__ __forceinline__ float max3_f32(const float a, const float b, const float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

struct ManyCall {
    const char *Q;   // [S][Gm][d] bf16
    float *out;      // [S][Gm][d] fp32
    int32_t Gm;      // queries per stream
    int32_t tiles;   // workgroups per stream = ceil(Gm / (16 QT QW))
    int64_t n_seen;  // tokens seen by every stream
    int64_t streams;
};

template <int NK>
struct SmemMany {
    static constexpr int KS = NK * 64 + 16;   // key tile row stride (bytes): 16-byte operand reads hit distinct banks
    static constexpr int VS = NK * 64 + 32;   // value tile row stride: the transposing reads hit distinct banks
    alignas(16) char kt[kTiles][kTileRows * KS];
    alignas(16) char vt[kTiles][kTileRows * VS];
    alignas(16) float wrow[kSuper];
    float wmx[kWaves][16], wden[kWaves][16];
};

template <int NK, int QT, bool NT, int QW = 1>
__global__ __launch_bounds__(kWG, 2) void attend_many_kernel(const State st, const ManyCall call)
{
    static_assert(kWaves == 4, "four wavefronts: QT query tiles x 4/QT row splits");
    constexpr int RS = kWaves / QT;          // row splits
    constexpr int CPR = 4 * NK;              // 16-byte chunks per row
    constexpr size_t ROWB = (size_t)NK * 64;
    constexpr int D = NK * 32;
    constexpr int NCB = NK * 2;              // 16-column blocks of the output
    constexpr int KS = SmemMany<NK>::KS, VS = SmemMany<NK>::VS;
    constexpr int LD = kSuper * CPR / kWG;   // 16-byte loads per thread and operand per iteration
    __shared__ SmemMany<NK> sm;

    // workgroups of one stream sit next to each other on one XCD (block b runs on XCD b % 8), so that the
    // second and later query tiles of a stream find its rows in that XCD's L2
    const int xcd = blockIdx.x & 7;
    const size_t j = blockIdx.x >> 3;
    const size_t sid = (j / call.tiles) * 8 + xcd;
    const int tile = (int)(j % call.tiles);
    if (sid >= (size_t)call.streams) return;   // padding of the stream count to a multiple of 8 (whole workgroup leaves)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, L = lane >> 4;
    const int qt = wave % QT, rs = wave / QT;

    const char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    const char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    const char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    const char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    const char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;
    const int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    const float *const svn = st.svn + sid * (size_t)st.sS;
    const int m = st.m[sid];
    const float mus = (float)(st.mu[sid] / (double)st.s);
    const int64_t n_seen = tokens_seen(st, call.n_seen);
    const int64_t n_evicted = st.w == 0 ? n_seen : (n_seen > st.w ? n_seen - st.w : 0);
    const int fill = (int)(n_seen < st.w ? n_seen : st.w);

    // the wavefront's QW tiles of 16 queries as the B operands of the score contraction
    const int q0 = (tile * QT + qt) * QW * 16;
    uint4 Bq[QW][NK];
#pragma unroll
    for (int w2 = 0; w2 < QW; ++w2) {
        const int q = q0 + w2 * 16 + n16 < call.Gm ? q0 + w2 * 16 + n16 : call.Gm - 1;
        const char *qp = call.Q + (sid * (size_t)call.Gm + q) * ROWB;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) Bq[w2][kk] = ld16(qp + (L + 4 * kk) * 16);
    }

    float mx[QW], den[QW];             // per query n16 of tile w2; mx is the same in the four lanes of a query
    floatx4_t acc[QW][NCB];            // O[query 4L + r][column 16 cb + n16]
#pragma unroll
    for (int w2 = 0; w2 < QW; ++w2) {
        mx[w2] = -INFINITY;
        den[w2] = 0.f;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) acc[w2][cb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    }

    // kind: 0 = representatives (weight n_i, normaliser only), 1 = sampled pairs (weight mu/(s ||v||^2),
    // numerator only), 2 = window (weight 1, both)
    auto scan = [&](auto kind_c, const char *Kb, const char *Vb, const int nrows) {
        constexpr int KIND = decltype(kind_c)::value;
        constexpr bool HASV = KIND != 0, TODEN = KIND != 1;
        uint4 rk[LD], rv[LD];
        auto prefetch = [&](const int r0) {
#pragma unroll
            for (int i = 0; i < LD; ++i) {
                const int idx = tid + kWG * i, row = idx / CPR, ch = idx % CPR;
                const int rr = r0 + row < nrows ? r0 + row : nrows - 1;
                // streamed once (one workgroup per stream): non-temporal; shared by several workgroups: cached
                if constexpr (NT) {
                    rk[i] = ldnt16(Kb + (size_t)rr * ROWB + ch * 16);
                    if constexpr (HASV) rv[i] = ldnt16(Vb + (size_t)rr * ROWB + ch * 16);
                } else {
                    rk[i] = ld16(Kb + (size_t)rr * ROWB + ch * 16);
                    if constexpr (HASV) rv[i] = ld16(Vb + (size_t)rr * ROWB + ch * 16);
                }
            }
        };
        prefetch(0);
        for (int r0 = 0; r0 < nrows; r0 += kSuper) {
            lds_barrier();   // the previous tiles have been consumed (prefetched rows stay in flight)
#pragma unroll
            for (int i = 0; i < LD; ++i) {
                const int idx = tid + kWG * i, row = idx / CPR, ch = idx % CPR;
                *reinterpret_cast<uint4 *>(&sm.kt[row / kTileRows][(row % kTileRows) * KS + ch * 16]) = rk[i];
                if constexpr (HASV)
                    *reinterpret_cast<uint4 *>(&sm.vt[row / kTileRows][(row % kTileRows) * VS + ch * 16]) = rv[i];
            }
            if (tid < kSuper) {
                const int r = r0 + tid;
                float wv = 0.f;
                if (r < nrows) {
                    if constexpr (KIND == 0) wv = (float)cnt[r];
                    else if constexpr (KIND == 1) {
                        const float vn = svn[r];
                        wv = vn > 0.f ? mus / vn : 0.f;
                    } else wv = 1.f;
                }
                sm.wrow[tid] = wv;
            }
            lds_barrier();
            if (r0 + kSuper < nrows) prefetch(r0 + kSuper);   // in flight while the matrix cores work

#pragma unroll
            for (int tt = 0; tt < kTiles / RS; ++tt) {
                const int t = rs + RS * tt;
                if (r0 + t * kTileRows >= nrows) break;
                // ---- scores of the tile's 32 rows against the wavefront's queries (every A operand read from LDS
                //      serves all QW query tiles)
                floatx4_t c0[QW], c1[QW];
#pragma unroll
                for (int w2 = 0; w2 < QW; ++w2) c0[w2] = c1[w2] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) {
                    const uint4 a0 = *reinterpret_cast<const uint4 *>(&sm.kt[t][n16 * KS + (L + 4 * kk) * 16]);
                    const uint4 a1 = *reinterpret_cast<const uint4 *>(&sm.kt[t][(16 + n16) * KS + (L + 4 * kk) * 16]);
#pragma unroll
                    for (int w2 = 0; w2 < QW; ++w2) {
                        c0[w2] = mfma_bf16(a0, Bq[w2][kk], c0[w2]);
                        c1[w2] = mfma_bf16(a1, Bq[w2][kk], c1[w2]);
                    }
                }
                const float4 w0 = *reinterpret_cast<const float4 *>(&sm.wrow[t * kTileRows + 4 * L]);
                const float4 w1 = *reinterpret_cast<const float4 *>(&sm.wrow[t * kTileRows + 16 + 4 * L]);
                uint4 ah[QW], al[QW];
#pragma unroll
                for (int w2 = 0; w2 < QW; ++w2) {
                    // ---- exponents a = (c - mx) log2(e), one fused multiply-add per score, and the lazy softmax
                    //      reference: mx is only raised when a score exceeds it by kLazy (rows beyond nrows repeat
                    //      the last row, so every score is a real one).  (The three-operand maximum is inline
                    //      assembly: it reads the products of the multiply-adds, never a matrix-core result, whose
                    //      read hazard the compiler only covers for its own instructions.)
                    constexpr float kLog2e = 1.4426950408889634f;
                    const float cs[8] = {c0[w2][0], c0[w2][1], c0[w2][2], c0[w2][3], c1[w2][0], c1[w2][1], c1[w2][2], c1[w2][3]};
                    float ax[8];
                    {
                        const float mxl = -mx[w2] * kLog2e;   // +inf before the first row
#pragma unroll
                        for (int i = 0; i < 8; ++i) ax[i] = fmaf(cs[i], kLog2e, mxl);
                    }
                    const float am = max3_f32(max3_f32(ax[0], ax[1], ax[2]), max3_f32(ax[3], ax[4], ax[5]),
                                              max3_f32(ax[6], ax[7], ax[7]));
                    if (__any(am > kLazy * kLog2e || mx[w2] == -INFINITY)) {
                        float lm = fmaxf(fmaxf(fmaxf(cs[0], cs[1]), fmaxf(cs[2], cs[3])), fmaxf(fmaxf(cs[4], cs[5]), fmaxf(cs[6], cs[7])));
                        lm = fmaxf(lm, __shfl_xor(lm, 16));
                        lm = fmaxf(lm, __shfl_xor(lm, 32));
                        float scale = 1.f;
                        if (lm > mx[w2] + kLazy || mx[w2] == -INFINITY) {
                            scale = __expf(mx[w2] - lm);   // mx = -inf gives 0
                            den[w2] *= scale;
                            mx[w2] = lm;
                        }
                        // the accumulators hold queries 4L + r: fetch their factors from the lanes of those queries
                        float sr[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) sr[r] = __shfl(scale, 4 * L + r);
#pragma unroll
                        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                            for (int r = 0; r < 4; ++r) acc[w2][cb][r] *= sr[r];
                        const float mxl = -mx[w2] * kLog2e;
#pragma unroll
                        for (int i = 0; i < 8; ++i) ax[i] = fmaf(cs[i], kLog2e, mxl);
                    }
                    const float ws[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
                    float e[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) e[i] = ws[i] * __builtin_amdgcn_exp2f(ax[i]);
                    if constexpr (TODEN) den[w2] += ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
                    if constexpr (HASV) {
                        // ---- weights as bf16 hi + lo, in contraction-slot order (slot j <-> e[j])
                        ah[w2].x = pack_bf16(e[0], e[1]); ah[w2].y = pack_bf16(e[2], e[3]);
                        ah[w2].z = pack_bf16(e[4], e[5]); ah[w2].w = pack_bf16(e[6], e[7]);
                        al[w2].x = pack_bf16(e[0] - bf16_lo(ah[w2].x), e[1] - bf16_hi(ah[w2].x));
                        al[w2].y = pack_bf16(e[2] - bf16_lo(ah[w2].y), e[3] - bf16_hi(ah[w2].y));
                        al[w2].z = pack_bf16(e[4] - bf16_lo(ah[w2].z), e[5] - bf16_hi(ah[w2].z));
                        al[w2].w = pack_bf16(e[6] - bf16_lo(ah[w2].w), e[7] - bf16_hi(ah[w2].w));
                    }
                }
                if constexpr (HASV) {
                    // every transposed value operand read from LDS serves all QW query tiles
                    const char *v0 = &sm.vt[t][(4 * L + (n16 >> 2)) * VS + (n16 & 3) * 8];
                    const char *v1 = v0 + 16 * VS;
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb) {
                        const u32x2_t b0 = lds_read_tr16(v0 + cb * 32), b1 = lds_read_tr16(v1 + cb * 32);
                        const uint4 b = make_uint4(b0[0], b0[1], b1[0], b1[1]);
#pragma unroll
                        for (int w2 = 0; w2 < QW; ++w2) {
                            acc[w2][cb] = mfma_bf16(ah[w2], b, acc[w2][cb]);
                            acc[w2][cb] = mfma_bf16(al[w2], b, acc[w2][cb]);
                        }
                    }
                }
            }
        }
    };
    if (m > 0) scan(std::integral_constant<int, 0>{}, X, X, m);
    if (n_evicted > 0) scan(std::integral_constant<int, 1>{}, Ks, Vs, st.s);
    if (fill > 0) scan(std::integral_constant<int, 2>{}, Kw, Vw, fill);

    // ---- totals per wavefront, then the row splits of a query group are merged through LDS, one query tile of
    //      the wavefronts at a time (the key tiles' memory carries the accumulators)
    float *const accbuf = reinterpret_cast<float *>(&sm.kt[0][0]);   // [wave][16 queries][D]
    static_assert(sizeof(sm.kt) >= (size_t)kWaves * 16 * D * sizeof(float), "accumulators fit in the key tiles");
#pragma unroll
    for (int w2 = 0; w2 < QW; ++w2) {
        float dsum = den[w2];
        dsum += __shfl_xor(dsum, 16);
        dsum += __shfl_xor(dsum, 32);
        __syncthreads();   // the tiles (or the previous query tile's accumulators) are dead
        if (L == 0) {
            sm.wmx[wave][n16] = mx[w2];
            sm.wden[wave][n16] = dsum;
        }
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r = 0; r < 4; ++r) accbuf[((size_t)wave * 16 + 4 * L + r) * D + cb * 16 + n16] = acc[w2][cb][r];
        __syncthreads();
        for (int i = tid; i < QT * 16 * D; i += kWG) {
            const int ql = i / D, c = i % D;       // query of this workgroup, output column
            const int qgrp = ql / 16, qn = ql % 16;
            const int q = ((tile * QT + qgrp) * QW + w2) * 16 + qn;
            if (q >= call.Gm) continue;
            float M = -INFINITY;
#pragma unroll
            for (int r = 0; r < RS; ++r) M = fmaxf(M, sm.wmx[qgrp + QT * r][qn]);
            float dn = 0.f, num = 0.f;
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                const int wv = qgrp + QT * r;
                const float wm = sm.wmx[wv][qn];
                const float sc = (wm == -INFINITY) ? 0.f : __expf(wm - M);
                dn = fmaf(sm.wden[wv][qn], sc, dn);
                num = fmaf(accbuf[((size_t)wv * 16 + qn) * D + c], sc, num);
            }
            put_out(st, call.out, (sid * (size_t)call.Gm + q) * D + c, num / dn);
        }
    }
}

}  // namespace sg
