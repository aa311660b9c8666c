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

// v * f in the register of v.  The rescaling of the accumulators sits in a rarely taken branch; written as plain
// multiplications the compiler puts the products into a second set of registers and copies the whole first set on
// the common path.  (The operands are accumulators of matrix-core instructions issued before this tile's score
// contraction, whose results have been consumed by then: in-order completion covers the read hazard that the
// compiler does not insert for inline assembly.)
__device__ __forceinline__ float scaled_in_place(float v, const float f)
{
    asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v) : "v"(f));
    return v;
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

// ---- The same block of queries, 128-element bf16 rows, 33 or more queries (every wavefront owns its queries for
//      all rows): the rows go from HBM straight into LDS (global_load_lds_dwordx4: lane i's 16 bytes land at
//      M0 + 16 i), so no register holds a row in flight, nothing is stored to LDS by hand, and one barrier per
//      stage is enough.  A stage is two halves of 32 rows x 256 bytes in one of three buffers: the next two stages
//      are in flight while one is consumed, across the three kinds of rows (the pipeline never drains between
//      them).  Representatives fill both halves with keys (64 rows per stage); sampled pairs and window rows put
//      32 keys in the first half and their 32 values in the second.  Rows are unpadded; instead the 16-byte
//      pieces of a row are permuted on the way in (the loading lane picks the global piece for its LDS slot):
//      keys by piece ^ (row mod 16), values by piece ^ 2 (row mod 8), which keeps the operand reads of both
//      contractions free of bank conflicts.  The weights of all representatives and sampled pairs of the stream
//      are computed once, up front, into LDS (window rows weigh 1).
constexpr int kDmaHalf = 32 * 256;           // bytes of 32 rows
constexpr int kDmaStage = 2 * kDmaHalf;
// rows with weights in LDS (representatives padded to 64, sampled pairs to 32) that fit beside three stage buffers
// with two workgroups per CU: 3 x 16 KB + 28 KB = 76 KB of the CU's 160 KB each
constexpr int kDmaBufs = 3;
constexpr int kDmaRows = 7168;

// NB stage buffers; WCAP = rows of one stream (each kind padded to whole stages) whose weights fit
template <int NB, int WCAP>
struct SmemManyDma {
    alignas(16) char buf[NB][kDmaStage];
    alignas(16) float w[WCAP];
};

// one direct load: 16 bytes per lane from base + off to LDS byte address lds + 16 lane (lds is wave-uniform); counted by
// vmcnt like any load.  (The compiler does not know of these loads: the waits for them are written out below.)
template <bool NT>
__device__ __forceinline__ void dma16(const char *base, const uint32_t off, const uint32_t lds)
{
    // base (wave-uniform) + off (per lane, unsigned 32 bits); M0 carries the LDS address and is put back afterwards
    // (the compiler keeps no account of M0 across inline assembly)
    uint32_t m0_saved;
    if constexpr (NT)
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt\n\ts_mov_b32 m0, %0"
                     : "=&s"(m0_saved) : "v"(off), "s"(base), "s"(lds) : "memory");
    else
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
                     : "=&s"(m0_saved) : "v"(off), "s"(base), "s"(lds) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads()   // until at most N of this wavefront's loads are outstanding
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <bool NT, int QW, int NB, int WCAP, int OCC>
__global__ __launch_bounds__(kWG, OCC) void attend_many_dma_kernel(const State st, const ManyCall call)
{
    static_assert(NB == 2 || NB == 3, "two or three stage buffers");
    static_assert(kWaves == 4 && kWG == 256, "four wavefronts, each with its own QW tiles of 16 queries");
    constexpr int NK = 4, NCB = 8, D = 128;
    constexpr size_t ROWB = 256;
    constexpr int LPS = 4;   // direct loads per wavefront and stage
    __shared__ SmemManyDma<NB, WCAP> sm;

    const int xcd = blockIdx.x & 7;
    const size_t j = blockIdx.x >> 3;
    const size_t sid = (j / call.tiles) * 8 + xcd;
    const int tile = (int)(j % call.tiles);
    if (sid >= (size_t)call.streams) return;   // padding of the stream count to a multiple of 8 (whole workgroup leaves)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, L = lane >> 4;

    const char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    const char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    const char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    const char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    const char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;
    const int m = st.m[sid];
    const int64_t n_seen = tokens_seen(st, call.n_seen);
    const int64_t n_evicted = st.w == 0 ? n_seen : (n_seen > st.w ? n_seen - st.w : 0);
    const int fill = (int)(n_seen < st.w ? n_seen : st.w);

    // stages: n0 of 64 representatives, n1 of 32 sampled pairs, n2 of 32 window rows
    const int n0 = (m + 63) >> 6, n1 = n_evicted > 0 ? (st.s + 31) >> 5 : 0, n2 = (fill + 31) >> 5;
    const int NS = n0 + n1 + n2;
    const int W1 = n0 * 64, W2 = W1 + n1 * 32;   // where the weights of the sampled pairs start; rows with weights
    if (W2 > WCAP) return;   // (the host has checked the context's capacity against WCAP: never taken)

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)&sm.buf[0][0];
    // this lane's slots of the wavefront's two 1 KB pieces of a half: row of the half and 16-byte position in LDS;
    // the global piece that belongs there, as an offset from the half's first row (keys / values)
    const int prow = lane >> 4, ppc = lane & 15;
    uint32_t koff[2], voff_g[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = (wave * 2 + i) * 4 + prow;
        koff[i] = (uint32_t)(row * 256 + ((ppc ^ (row & 15)) << 4));
        voff_g[i] = (uint32_t)(row * 256 + ((ppc ^ ((row & 7) << 1)) << 4));
    }
    auto issue = [&](const int stg, const int b) __attribute__((always_inline)) {
        const char *ba, *bb;
        int ra0, rb0, nrows;
        bool bkeys = false;
        if (stg < n0) {
            ba = bb = X; ra0 = stg * 64; rb0 = ra0 + 32; nrows = m; bkeys = true;
        } else if (stg < n0 + n1) {
            ba = Ks; bb = Vs; ra0 = rb0 = (stg - n0) * 32; nrows = st.s;
        } else {
            ba = Kw; bb = Vw; ra0 = rb0 = (stg - n0 - n1) * 32; nrows = fill;
        }
        const uint32_t la = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)b * kDmaStage + (uint32_t)wave * 2048u);
        if (rb0 + 32 <= nrows) {
            // whole halves: the lane's offsets are the loop-invariant ones
            const char *pa = ba + (size_t)ra0 * ROWB, *pb = bb + (size_t)rb0 * ROWB;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                dma16<NT>(pa, koff[i], la + i * 1024);
                dma16<NT>(pb, bkeys ? koff[i] : voff_g[i], la + kDmaHalf + i * 1024);
            }
        } else {
            // the last rows of a kind: rows past the end repeat the last one
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = (wave * 2 + i) * 4 + prow;   // row of the half
                int ra = ra0 + row, rb = rb0 + row;
                ra = ra < nrows ? ra : nrows - 1;
                rb = rb < nrows ? rb : nrows - 1;
                const int ca = ppc ^ (row & 15);
                const int cb = bkeys ? ca : ppc ^ ((row & 7) << 1);
                dma16<NT>(ba, (uint32_t)(ra * 256 + ca * 16), la + i * 1024);
                dma16<NT>(bb, (uint32_t)(rb * 256 + cb * 16), la + kDmaHalf + i * 1024);
            }
        }
    };
    if (NS > 0) issue(0, 0);
    if (NB > 2 && NS > 1) issue(1, 1);

    // the wavefront's QW tiles of 16 queries as the B operands of the score contraction
    const int q0 = (tile * 4 + wave) * QW * 16;
    uint4 Bq[QW][NK];
#pragma unroll
    for (int w2 = 0; w2 < QW; ++w2) {
        const int q = q0 + w2 * 16 + n16 < call.Gm ? q0 + w2 * 16 + n16 : call.Gm - 1;
        const char *qp = call.Q + (sid * (size_t)call.Gm + q) * ROWB;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) Bq[w2][kk] = ld16(qp + (L + 4 * kk) * 16);
    }

    // ---- weights of the rows: n_i for representatives, mu / (s ||v_j||^2) for sampled pairs, 0 for the padding of
    //      each kind to whole stages (window rows weigh 1: no array)
    {
        const int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
        const float *const svn = st.svn + sid * (size_t)st.sS;
        const float mus = (float)(st.mu[sid] / (double)st.s);
        for (int i = tid; i < W2; i += kWG) {
            float wv = 0.f;
            if (i < W1) {
                if (i < m) wv = (float)cnt[i];
            } else if (i - W1 < st.s) {
                const float vn = svn[i - W1];
                wv = vn > 0.f ? mus / vn : 0.f;
            }
            sm.w[i] = wv;
        }
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

    // operand offsets inside a half (see the permutations above)
    const int aoff = n16 * 256 + ((L ^ (n16 & 3)) << 4) + ((n16 >> 2) << 6);      // key piece L of row n16; ^ (kk << 6)
    const int vrow = 4 * L + (n16 >> 2);
    const int voff = vrow * 256 + ((vrow & 7) << 5) + (n16 & 3) * 8;               // ^ (cb << 5)

    // One tile of 32 rows in two parts.  scores_weights: scores from the keys at `A`, weights e, the normaliser's
    // share, (HASV) the weights as bf16 operands ah + al; returns whether a reference was raised, with the factors of
    // the accumulators in rescale[].  products: the products of ah + al with the values at `B`.
    uint4 ah[QW], al[QW];
    float rescale[QW];     // factor of the accumulators of query n16 (1 unless its reference was raised)
    auto scores_weights = [&](auto hasv_c, auto toden_c, const char *A, const float4 w0, const float4 w1) __attribute__((always_inline)) -> bool {
        constexpr bool HASV = decltype(hasv_c)::value, TODEN = decltype(toden_c)::value;
        floatx4_t c0[QW], c1[QW];
#pragma unroll
        for (int w2 = 0; w2 < QW; ++w2) c0[w2] = c1[w2] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
            const uint4 a0 = *reinterpret_cast<const uint4 *>(A + (aoff ^ (kk << 6)));
            const uint4 a1 = *reinterpret_cast<const uint4 *>(A + 4096 + (aoff ^ (kk << 6)));
#pragma unroll
            for (int w2 = 0; w2 < QW; ++w2) {
                c0[w2] = mfma_bf16(a0, Bq[w2][kk], c0[w2]);
                c1[w2] = mfma_bf16(a1, Bq[w2][kk], c1[w2]);
            }
        }
        bool raised = false;
#pragma unroll
        for (int w2 = 0; w2 < QW; ++w2) {
            __builtin_amdgcn_sched_barrier(0);   // one query tile's weights at a time: bounds the live registers
            rescale[w2] = 1.f;
            // exponents a = (c - mx) log2(e), one fused multiply-add per score; the reference mx is only raised when
            // a score exceeds it by kLazy (rows beyond the end repeat the last row, so every score is a real one).
            // (The three-operand maximum is inline assembly: it reads the products of the multiply-adds, never a
            // matrix-core result, whose read hazard the compiler only covers for its own instructions.)
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
                if (lm > mx[w2] + kLazy || mx[w2] == -INFINITY) {
                    rescale[w2] = __expf(mx[w2] - lm);   // mx = -inf gives 0
                    den[w2] *= rescale[w2];
                    mx[w2] = lm;
                }
                raised = true;
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
                // weights as bf16 hi + lo, in contraction-slot order (slot j <-> e[j]): hi = the upper half of
                // the fp32 word (truncated; one AND gives it as a float, one byte permute packs a pair), lo = the
                // exact remainder rounded to bf16: together 16 mantissa bits
                uint32_t hp[4], lp[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t b0 = __float_as_uint(e[2 * i]), b1 = __float_as_uint(e[2 * i + 1]);
                    hp[i] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
                    lp[i] = pack_bf16(e[2 * i] - __uint_as_float(b0 & 0xffff0000u),
                                      e[2 * i + 1] - __uint_as_float(b1 & 0xffff0000u));
                }
                ah[w2] = make_uint4(hp[0], hp[1], hp[2], hp[3]);
                al[w2] = make_uint4(lp[0], lp[1], lp[2], lp[3]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        return raised;
    };
    auto products = [&](const char *B) __attribute__((always_inline)) {
        // two column blocks at a time, all hi products before the lo ones: the two products into one accumulator
        // are then four (QW = 2) or two matrix-core instructions apart instead of back to back
#pragma unroll
        for (int cb = 0; cb < NCB; cb += 2) {
            uint4 bv[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const char *v0 = B + (voff ^ ((cb + u) << 5));
                const u32x2_t b0 = lds_read_tr16(v0), b1 = lds_read_tr16(v0 + 4096);
                bv[u] = make_uint4(b0[0], b0[1], b1[0], b1[1]);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int w2 = 0; w2 < QW; ++w2) acc[w2][cb + u] = mfma_bf16(ah[w2], bv[u], acc[w2][cb + u]);
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int w2 = 0; w2 < QW; ++w2) acc[w2][cb + u] = mfma_bf16(al[w2], bv[u], acc[w2][cb + u]);
        }
    };
    // the accumulators of a tile that raised a reference: O[query 4L + r] takes the factor of that query's lanes
    auto rescale_accumulators = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int w2 = 0; w2 < QW; ++w2) {
            float sr[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) sr[r] = __shfl(rescale[w2], 4 * L + r);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[w2][cb][r] *= sr[r];
        }
    };

    // every load the compiler knows of (queries, weights) is complete from here on: it then places no wait of its
    // own inside the loop, where it would also wait for the direct loads of the stages ahead
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)

    using T = std::true_type;
    using F = std::false_type;
    // Start of a stage: its rows are in LDS for everybody, the buffer of the stage before it is free, the stage
    // NB - 1 ahead is requested into that buffer.  Returns the stage's first half.
    int b = 0;
    auto next_stage = [&](const int it) __attribute__((always_inline)) -> const char * {
        // this wavefront's loads of stage `it` have landed (those of the next stage may still be in flight) ...
        if (NB > 2 && it + 1 < NS) wait_loads<LPS>();
        else wait_loads<0>();
        lds_barrier();   // ... and so have everybody's; the buffer of stage it - 1 is free (also orders the weights)
        if (it + NB - 1 < NS) issue(it + NB - 1, b == 0 ? NB - 1 : b - 1);
        // (the buffer's offset is made opaque: otherwise the operand addresses of all buffers are kept in
        // registers across the loop)
        uint32_t boff = (uint32_t)b * kDmaStage;
        asm volatile("" : "+v"(boff));
        b = b == NB - 1 ? 0 : b + 1;
        return &sm.buf[0][0] + boff;
    };
    // the weights of this lane's rows 4L..4L+3 and 16+4L..16+4L+3 of a tile
    auto weights = [&](const int at, float4 &w0, float4 &w1) __attribute__((always_inline)) {
        w0 = *reinterpret_cast<const float4 *>(&sm.w[at + 4 * L]);
        w1 = *reinterpret_cast<const float4 *>(&sm.w[at + 16 + 4 * L]);
    };
    // One loop per kind of row, each around a single copy of the tile code, and the rare tile that raises a reference
    // is finished outside the loop of the common ones: with the kinds (or the rescaling) in branches of one loop the
    // accumulators end every iteration in other registers than they started in and are copied back, 64 to 130
    // moves per stage.
    int it = 0;
    for (; it < n0; ++it) {
        const char *A = next_stage(it);
#pragma unroll 1
        for (int h = 0; h < 2; ++h) {
            if (it * 64 + 32 * h >= m) break;
            float4 w0, w1;
            weights(it * 64 + 32 * h, w0, w1);
            scores_weights(F{}, T{}, A + h * kDmaHalf, w0, w1);   // (the accumulators are still zero: nothing to rescale)
        }
    }
    while (it < n0 + n1) {
        const char *A = nullptr;
        bool raised = false;
        for (; it < n0 + n1; ++it) {
            A = next_stage(it);
            float4 w0, w1;
            weights(W1 + (it - n0) * 32, w0, w1);
            raised = scores_weights(T{}, F{}, A, w0, w1);
            if (raised) break;
            products(A + kDmaHalf);
        }
        if (raised) {
            rescale_accumulators();
            products(A + kDmaHalf);
            ++it;
        }
    }
    while (it < NS) {
        const char *A = nullptr;
        bool raised = false;
        for (; it < NS; ++it) {
            A = next_stage(it);
            const int left = fill - (it - n0 - n1) * 32 - 4 * L;   // window rows from this lane's first one on
            const float4 w0 = make_float4(left > 0 ? 1.f : 0.f, left > 1 ? 1.f : 0.f, left > 2 ? 1.f : 0.f, left > 3 ? 1.f : 0.f);
            const float4 w1 = make_float4(left > 16 ? 1.f : 0.f, left > 17 ? 1.f : 0.f, left > 18 ? 1.f : 0.f, left > 19 ? 1.f : 0.f);
            raised = scores_weights(T{}, T{}, A, w0, w1);
            if (raised) break;
            products(A + kDmaHalf);
        }
        if (raised) {
            rescale_accumulators();
            products(A + kDmaHalf);
            ++it;
        }
    }

    // ---- every wavefront owns its queries: normalise and store straight from the accumulators (16 lanes write 64
    //      consecutive bytes of one query's row)
#pragma unroll
    for (int w2 = 0; w2 < QW; ++w2) {
        float dsum = den[w2];
        dsum += __shfl_xor(dsum, 16);
        dsum += __shfl_xor(dsum, 32);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float dn = __shfl(dsum, 4 * L + r);
            const int q = q0 + w2 * 16 + 4 * L + r;
            if (q < call.Gm) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    put_out(st, call.out, (sid * (size_t)call.Gm + q) * D + cb * 16 + n16, acc[w2][cb][r] / dn);
            }
        }
    }
}

}  // namespace sg
