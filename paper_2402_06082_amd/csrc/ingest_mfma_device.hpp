// Chunked prefix ingest for bf16 rows on gfx950.
//
// A stream's tokens must be clustered in order (the greedy rule is order
// dependent), but the arithmetic of T = 128 (or 64) consecutive tokens can be
// batched:
//   1. distances of the T tokens to all representatives that exist at the
//      start of the chunk are one dense (m x T x d) contraction on the matrix
//      cores (representatives as the A operand, the token keys as T / 16 B
//      operands read from an LDS tile), so the table is read once per T
//      tokens; every lane tracks the three smallest distances of its token,
//      each with its row in the low mantissa bits;
//   2. wavefront 0 replays the order, one lane per token (two tokens with
//      T = 128: first the lower 64, then the upper 64): a token only sees the
//      clusters that the chunk opened before it.  The loop advances from one
//      creation (or one ambiguous token) to the next, so it runs a few
//      iterations per chunk once the table has filled; the distances of a
//      new representative to the later tokens of the chunk are computed when
//      it appears (packed dot products over the LDS tile);
//   3. ambiguous decisions (gap or threshold distance within the error bound
//      of the approximate distances) are re-evaluated exactly in double: as a
//      rule only against the best and the runner-up (the third-smallest
//      distance shows that no other row can be the nearest), else against the
//      whole table;
//   4. the sampling coins do not depend on the clustering: the chunks only
//      leave each token's probability behind, and once per 1024 evicted tokens (or at the end of the call) one pass draws the
//      coins per 4-slot block; the last accepting token of a slot wins
//      (sequential overwrite semantics), so a slot is copied at most once
//      per pass.
// The window is handled by index arithmetic: the tokens that leave the window
// during the call come first from the ring, then from the call's own input;
// the ring is rewritten once at the end.
#pragma once
#include <cstddef>
#include <type_traits>

#include "subgen_dot2_device.hpp"
#include "subgen_mfma_device.hpp"

namespace sg {


// per-cluster reservoirs (t >= 1): cluster of every token of the chunk, its coin probability 1/n_i, and which
// reservoir slots it wins
template <int T, bool RES>
struct SmemReservoir {
    int tgt[T];
    float pr[T];
    uint8_t win[T][16];
};
template <int T>
struct SmemReservoir<T, false> {};

template <int NK, int T, bool RES>
struct SmemIngest {
    // evicted tokens per coin pass (a multiple of the chunk)
    static constexpr int kSpan = 1024;
    alignas(16) float nk[T];
    float vn[T];
    // coin bound (coin_limit: a word r is accepted iff r <= bound; 0 = never) of the evicted tokens whose coins are
    // still to be drawn (up to kSpan)
    uint32_t plim[kSpan];
    // candidate lists of the tokens, one per wavefront (each wavefront scans a quarter of the rows)
    float wb1[kWaves][T], wb2[kWaves][T], wb3[kWaves][T];
    int wi1[kWaves][T], wi2[kWaves][T];
    float wnx[kWaves];
    int mnew;
    SmemReservoir<T, RES> res;
    // the chunk's keys, one padded row per token (the pad spreads the 16 rows an operand read touches over
    // all banks): the B operands of every contraction of the chunk are read from here
    static constexpr int KS = NK * 64 + 16;
    alignas(16) char kt[T * KS];
};

// median of three signed integers (inline assembly: operands must not be matrix-core results, see min_f32)
__device__ __forceinline__ int med3_i32(const int a, const int b, const int c)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Lane exchanges of gfx950 that stay in the vector unit.  from_row_above: lanes of DPP row 0 get the value of the
// same lane of row 1, row 2 gets row 3 (rows 1 and 3 get something else); from_upper_half: lanes 0..31 get lanes
// 32..63.
__device__ __forceinline__ uint32_t from_row_above(const uint32_t v) { return __builtin_amdgcn_permlane16_swap(v, v, false, false)[1]; }
__device__ __forceinline__ uint32_t from_upper_half(const uint32_t v) { return __builtin_amdgcn_permlane32_swap(v, v, false, false)[1]; }
template <bool HALF>
__device__ __forceinline__ float lanes_above(const float v)
{
    const uint32_t b = __builtin_bit_cast(uint32_t, v);
    return __builtin_bit_cast(float, HALF ? from_upper_half(b) : from_row_above(b));
}
template <bool HALF>
__device__ __forceinline__ int lanes_above(const int v)
{
    return (int)(HALF ? from_upper_half((uint32_t)v) : from_row_above((uint32_t)v));
}
// lane l gets the value of lane l - 1, lane 0 gets `first` (a DPP wavefront shift)
__device__ __forceinline__ double from_lane_below(const double v, const double first)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v), f = __builtin_bit_cast(uint64_t, first);
    const uint32_t lo = __builtin_amdgcn_update_dpp((uint32_t)f, (uint32_t)b, 0x138, 0xf, 0xf, false);
    const uint32_t hi = __builtin_amdgcn_update_dpp((uint32_t)(f >> 32), (uint32_t)(b >> 32), 0x138, 0xf, 0xf, false);
    return __builtin_bit_cast(double, (uint64_t)lo | ((uint64_t)hi << 32));
}

template <int NK, int T, bool RES>
__global__ __launch_bounds__(kWG, 3) void ingest_mfma_kernel(const State st, const Call call)
{
    static_assert(kWaves == 4, "the chunk layout assumes four wavefronts per workgroup");
    static_assert(T == 64 || T == 128, "one or two tokens per lane of the resolving wavefront");
    constexpr int H = T / 64;      // 64-token halves of a chunk
    constexpr int NTS = T / 16;    // 16-token operand sets
    constexpr int CPR = 4 * NK, LPR = CPR;
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)NK * 64;
    constexpr int KS = SmemIngest<NK, T, RES>::KS;
    constexpr int kCoinSpan = SmemIngest<NK, T, RES>::kSpan;
    constexpr int PF = 2;   // groups of 16 representatives in flight per wavefront (a third one spills)
    __shared__ SmemIngest<NK, T, RES> sm;

    const size_t sid = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR, grp = wave * RPW + sub;
    const int n16 = lane & 15, L = lane >> 4;

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    float *const xn = st.xn + sid * (size_t)st.McapS;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;
    const char *const kin = call.K + sid * call.stream_stride;
    const char *const vin = call.V + sid * call.stream_stride;

    const int64_t n0 = tokens_seen(st, call.n_seen), n = call.n_tokens, w = st.w;
    // global indices [ge0, ge1) of the tokens that leave the window during this call
    const int64_t ge0 = w == 0 ? n0 : (n0 > w ? n0 - w : 0);
    int64_t ge1 = w == 0 ? n0 + n : n0 + n - w;
    if (ge1 < ge0) ge1 = ge0;
    // ring slot of token ge0 + i (i < w): one 64-bit remainder per kernel, 32-bit arithmetic per row afterwards
    const uint32_t slot0 = w > 0 ? (uint32_t)(ge0 % w) : 0u;
    auto ring_slot = [&](int64_t ge) -> uint32_t {
        const uint32_t sl = slot0 + (uint32_t)(ge - ge0);
        return sl >= (uint32_t)w ? sl - (uint32_t)w : sl;
    };
    auto krow_of = [&](int64_t ge) -> const char * {
        return ge < n0 ? Kw + (size_t)ring_slot(ge) * ROWB : kin + (ge - n0) * call.token_stride;
    };
    auto vrow_of = [&](int64_t ge) -> const char * {
        return ge < n0 ? Vw + (size_t)ring_slot(ge) * ROWB : vin + (ge - n0) * call.token_stride;
    };

    int m = st.m[sid];
    double mu = st.mu[sid];
    const float thr = (float)st.delta2;

    // ---- coin pass over the evicted tokens [g0, g0 + cnt) whose probabilities are in LDS.  A wavefront takes 64
    //      consecutive 4-slot blocks (one per lane) and one sub-range of the tokens, so the token is the same in
    //      all its lanes and everything of the Philox rounds that depends on the token alone runs on the scalar
    //      unit; every lane walks the tokens from the oldest to the newest and keeps the newest accept per slot.
    //      The sub-ranges meet in LDS (maximum per slot; the candidate lists of the scan are dead by now and lend
    //      their memory), then one lane per accepted slot copies the rows.
    auto coin_pass = [&](const int64_t g0, const int cnt) {
        using Sm = SmemIngest<NK, T, RES>;
        constexpr int kLastCap = 5 * kWaves * T;   // slots per segment
        static_assert(offsetof(Sm, wi2) + sizeof(sm.wi2) - offsetof(Sm, wb1) == kLastCap * sizeof(int),
                      "the candidate lists are one block of memory");
        int *const lastbuf = reinterpret_cast<int *>(&sm.wb1[0][0]);
        const int wave_s = __builtin_amdgcn_readfirstlane(wave);
        for (int seg0 = 0; seg0 < st.s; seg0 += kLastCap) {
            const int nslot = st.s - seg0 < kLastCap ? st.s - seg0 : kLastCap;
            const int nb = (nslot + 3) >> 2, ngrp = (nb + 63) >> 6;
            int nparts = 1;   // sub-ranges of the tokens, so that all wavefronts have coins to draw
            while (ngrp * nparts * 2 <= kWaves) nparts *= 2;
            const int per = (cnt + nparts - 1) / nparts;
            if (seg0 > 0) __syncthreads();   // the copies of the segment before this one have read the buffer
            for (int i = tid; i < nslot; i += kWG) lastbuf[i] = -1;
            __syncthreads();
            for (int u = wave_s; u < ngrp * nparts; u += kWaves) {
                const int blk = (u % ngrp) * 64 + lane, part = u / ngrp;
                const int lo = part * per, hi = lo + per < cnt ? lo + per : cnt;
                int last[4] = {-1, -1, -1, -1};
                for (int jj = lo; jj < hi; ++jj) {   // oldest first: a later accept overwrites an earlier one
                    const uint32_t lim = sm.plim[jj];
                    if (lim != 0u) {
                        uint32_t r[4];
                        coin_block(st, sid, g0 + jj, (uint32_t)((seg0 >> 2) + blk), false, r);
#pragma unroll
                        for (int i = 0; i < 4; ++i) last[i] = r[i] <= lim ? jj : last[i];
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (last[i] >= 0 && 4 * blk + i < nslot) atomicMax(&lastbuf[4 * blk + i], last[i]);
            }
            __syncthreads();
            for (int sl = tid; sl < nslot; sl += kWG) {
                const int l = lastbuf[sl];
                if (l >= 0) {
                    const int slot = seg0 + sl;
                    const char *ks = krow_of(g0 + l), *vs = vrow_of(g0 + l);
                    // ||v||^2 of the token once more, with the additions in the order of the chunk's norms (eight
                    // products per 16-byte piece, then the pieces pairwise): the same double, the same float
                    double piece[CPR];
#pragma unroll
                    for (int ch = 0; ch < CPR; ++ch) {
                        st16(Ks + (size_t)slot * ROWB + ch * 16, ld16(ks + ch * 16));
                        const uint4 v16 = ld16(vs + ch * 16);
                        st16(Vs + (size_t)slot * ROWB + ch * 16, v16);
                        float vf[8];
                        unpack<true>(v16, vf);
                        double b = 0.0;
#pragma unroll
                        for (int v = 0; v < 8; ++v) b = fma((double)vf[v], (double)vf[v], b);
                        piece[ch] = b;
                    }
#pragma unroll
                    for (int o = 1; o < CPR; o <<= 1)
#pragma unroll
                        for (int ch = 0; ch < CPR; ch += 2 * o) piece[ch] += piece[ch + o];
                    st.sidx[sid * (size_t)st.sS + slot] = (int32_t)(g0 + l);
                    st.svn[sid * (size_t)st.sS + slot] = (float)piece[0];
                }
            }
        }
    };
    int64_t span0 = ge0;   // first evicted token of the pending coin pass
    int span_fill = 0;     // tokens whose probabilities wait in LDS


    for (int64_t c0 = ge0; c0 < ge1; c0 += T) {
        const int nt = (int)(ge1 - c0 < T ? ge1 - c0 : T);
        const int m0 = m;

        // ---- the first groups of representatives are requested before anything else of the chunk
        uint4 q[PF][NK];
        float4 qn[PF];
        auto request = [&](uint4(&dst)[NK], float4 &dn, int r) __attribute__((always_inline)) {
            dn = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < m0) {
                const int rr = r + n16 < m0 ? r + n16 : m0 - 1;
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) dst[kk] = ld16(X + (size_t)rr * ROWB + (L + 4 * kk) * 16);
                dn = *reinterpret_cast<const float4 *>(xn + r + 4 * L);
            }
        };
#pragma unroll
        for (int pf = 0; pf < PF; ++pf) request(q[pf], qn[pf], (wave + kWaves * pf) * 16);

        // ---- squared norms of the chunk's keys and values (double, exact products), one token per lane group;
        //      64 tokens per batch (a batch's rows are all requested before the first is used)
#pragma unroll 1
        for (int t0 = 0; t0 < T; t0 += 64) {
            constexpr int NB = 64 / RPB;   // passes of the lane groups over a batch
            uint4 rk[NB], rv[NB];
#pragma unroll
            for (int it = 0; it < NB; ++it) {
                const int jr = t0 + grp + it * RPB;
                const int jj = jr < nt ? jr : nt - 1;
                rk[it] = ld16(krow_of(c0 + jj) + col * 16);
                rv[it] = ld16(vrow_of(c0 + jj) + col * 16);
            }
#pragma unroll
            for (int it = 0; it < NB; ++it) {
                const int jr = t0 + grp + it * RPB;
                float kf[8], vf[8];
                unpack<true>(rk[it], kf);
                unpack<true>(rv[it], vf);
                *reinterpret_cast<uint4 *>(&sm.kt[jr * KS + col * 16]) = rk[it];
                double a = 0.0, b = 0.0;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    a = fma((double)kf[v], (double)kf[v], a);
                    b = fma((double)vf[v], (double)vf[v], b);
                }
                a = group_sum<LPR>(a);
                b = group_sum<LPR>(b);
                // a token with NaN or Inf in it (or a norm beyond fp32) is dropped: it joins nothing, opens
                // nothing and is never sampled; it is marked by ||k||^2 = +inf, ||v||^2 = 0
                const bool bad = !token_is_finite((float)a, (float)b);
                if (col == 0) {
                    sm.nk[jr] = bad ? INFINITY : (float)a;
                    sm.vn[jr] = bad ? 0.f : (float)b;
                    if (bad && jr < nt) atomicOr(&st.flags[sid], 2u);
                }
            }
        }
        // ---- B operand (ts, kk): token 16 ts + n in column n, read from the LDS tile
        auto bop = [&](int ts, int kk) __attribute__((always_inline)) {
            return *reinterpret_cast<const uint4 *>(&sm.kt[(16 * ts + n16) * KS + (L + 4 * kk) * 16]);
        };
        __syncthreads();

        // ---- distances to the representatives that exist at the start of the chunk.  Per (token, row) the loop
        //      spends six vector instructions: e = ||x||^2 - 2 <x, k> + ||k||^2; the low bits of e are replaced by the
        //      position of the row in the lane's sequence of rows (4 g + r: group g of the wavefront, row r of the
        //      lane's four), and the three smallest of these keys are kept with integer minimum / median (as
        //      signed integers the keys order like the distances; the few negative ones, all within the error
        //      bound of zero, order among themselves in reverse, which the exact comparison sorts out).  The
        //      key of a distance d is within 2^(KB-23) |d| of d (KB index bits).
        const int KB = 32 - __builtin_clz((unsigned)(m0 > 64 ? (m0 + 63) >> 6 : 1) * 4u - 1u);   // positions < 4 groups
        const int kmask = (1 << KB) - 1;
        const float ek = ldexpf(1.0005f, KB - 23);
        constexpr int kEmpty = 0x7f800000;   // +inf
        int k1[NTS], k2[NTS], k3[NTS];
        float nkt[NTS], nxmax = 0.f;
#pragma unroll
        for (int ts = 0; ts < NTS; ++ts) {
            k1[ts] = kEmpty;
            k2[ts] = kEmpty;
            k3[ts] = kEmpty;
            nkt[ts] = sm.nk[16 * ts + n16];
        }
        const int wave_s = __builtin_amdgcn_readfirstlane(wave);
        // one group of 16 rows from a request slot
        auto scan_group = [&](uint4(&qs)[NK], float4 &qns, const int r0) __attribute__((always_inline)) {
            const float nxraw[4] = {qns.x, qns.y, qns.z, qns.w};
            // the B operands do not change from group to group: without this the compiler keeps all of them
            // in registers over the loop, which is what the LDS tile is there to avoid
            asm volatile("" ::: "memory");
            const int row0 = r0 + 4 * L;
            const int pos0 = (r0 - 16 * wave_s) >> 4;   // 4 g
            float nxr[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // rows past the table (the clamped loads of the last group) take part as +inf
                const bool in = row0 + r < m0;
                nxr[r] = in ? nxraw[r] : INFINITY;
                nxmax = fmaxf(nxmax, in ? nxraw[r] : 0.f);
            }
#pragma unroll
            for (int ts = 0; ts < NTS; ++ts) {
                floatx4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(qs[kk], bop(ts, kk), c);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float e = fmaf(-2.f, c[r], nxr[r]) + nkt[ts];
                    const int key = (__builtin_bit_cast(int, e) & ~kmask) | (pos0 + r);
                    k3[ts] = med3_i32(k2[ts], k3[ts], key);
                    k2[ts] = med3_i32(k1[ts], k2[ts], key);
                    k1[ts] = min(k1[ts], key);
                }
            }
            // the slot's rows are consumed: it takes the group PF groups ahead (in flight while the other slot's
            // group is on the matrix cores)
            request(qs, qns, r0 + 16 * kWaves * PF);
        };
        for (int r0 = wave * 16; r0 < m0; r0 += 16 * kWaves * PF) {
            static_assert(PF == 2, "the loop alternates between two request slots");
            scan_group(q[0], qn[0], r0);
            if (r0 + 16 * kWaves < m0) scan_group(q[1], qn[1], r0 + 16 * kWaves);
        }
        // distance and row out of a key; an empty entry (or a row past the table) is (+inf, -1)
        auto key_value = [&](const int key) { return __builtin_bit_cast(float, key & ~kmask); };
        auto key_row = [&](const int key) {
            const int pos = key & kmask;
            return (key & ~kmask) == kEmpty ? -1 : ((pos >> 2) << 6) + 16 * wave + 4 * L + (pos & 3);
        };
#pragma unroll
        for (int ts = 0; ts < NTS; ++ts) {
            float b1 = key_value(k1[ts]), b2 = key_value(k2[ts]), b3 = key_value(k3[ts]);
            int i1 = key_row(k1[ts]), i2 = key_row(k2[ts]);
            // the four lanes of a token hold disjoint rows; lane L = 0 collects them: first from L = 1 (and L = 2
            // from L = 3), then from L = 2
            auto collect = [&](auto half) __attribute__((always_inline)) {
                constexpr bool HALF = decltype(half)::value;
                const float x1 = lanes_above<HALF>(b1), x2 = lanes_above<HALF>(b2), x3 = lanes_above<HALF>(b3);
                const int xi1 = lanes_above<HALF>(i1), xi2 = lanes_above<HALF>(i2);
                top3_insert(x1, xi1, b1, i1, b2, i2, b3);
                top3_insert(x2, xi2, b1, i1, b2, i2, b3);
                b3 = min_f32(b3, x3);
            };
            collect(std::false_type{});
            collect(std::true_type{});
            if (L == 0) {
                sm.wb1[wave][16 * ts + n16] = b1;
                sm.wb2[wave][16 * ts + n16] = b2;
                sm.wb3[wave][16 * ts + n16] = b3;
                sm.wi1[wave][16 * ts + n16] = i1;
                sm.wi2[wave][16 * ts + n16] = i2;
            }
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) nxmax = fmaxf(nxmax, __shfl_xor(nxmax, o));
        if (lane == 0) sm.wnx[wave] = nxmax;
        if constexpr (RES) {
            if (tid < T) sm.res.tgt[tid] = -1;   // dropped tokens and the ragged tail keep -1
        }
        __syncthreads();

        // ---- resolve in token order (wavefront 0): lane j holds token j of every 64-token half of the chunk
        if (wave == 0) {
            const int j = lane;
            const uint64_t below = j == 0 ? 0ull : (~0ull >> (64 - j));
            // the token's candidate list over the representatives of the chunk's start; the clusters that the
            // chunk opens are inserted as they appear
            float c1[H], c2[H], c3[H], nxl[H], nkj[H];
            int ci[H], ci2[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const int tok = 64 * h + j;
                nkj[h] = sm.nk[tok];
                c1[h] = sm.wb1[0][tok];
                c2[h] = sm.wb2[0][tok];
                c3[h] = sm.wb3[0][tok];
                ci[h] = sm.wi1[0][tok];
                ci2[h] = sm.wi2[0][tok];
                nxl[h] = sm.wnx[0];
#pragma unroll
                for (int wv = 1; wv < kWaves; ++wv) {
                    top3_insert(sm.wb1[wv][tok], sm.wi1[wv][tok], c1[h], ci[h], c2[h], ci2[h], c3[h]);
                    top3_insert(sm.wb2[wv][tok], sm.wi2[wv][tok], c1[h], ci[h], c2[h], ci2[h], c3[h]);
                    c3[h] = min_f32(c3[h], sm.wb3[wv][tok]);
                    nxl[h] = fmaxf(nxl[h], sm.wnx[wv]);
                }
            }
            uint64_t cmask[H];   // tokens of each half that opened a cluster (uniform)
#pragma unroll
            for (int h = 0; h < H; ++h) cmask[h] = 0;
            // chunk position of the token that opened cluster idx >= m0
            auto opener = [&](const int idx) {
                int q = idx - m0, tok0 = 0;
                uint64_t mm = cmask[0];
                if constexpr (H > 1) {
                    const int n0h = __builtin_popcountll(cmask[0]);
                    if (q >= n0h) {
                        q -= n0h;
                        mm = cmask[H - 1];
                        tok0 = 64;
                    }
                }
                for (; q > 0; --q) mm &= mm - 1;
                return tok0 + (int)__builtin_ctzll(mm);
            };
            // approximate squared distance of two tokens of the chunk (lane-wise: jtok differs per lane)
            auto token_distance = [&](const int etok, const int jtok) {
                float acc = 0.f;
#pragma unroll 4   // (a full unroll makes the compiler spill the scan's registers)
                for (int ch = 0; ch < CPR; ++ch) {
                    const uint4 a = *reinterpret_cast<const uint4 *>(&sm.kt[etok * KS + ch * 16]);
                    const uint4 b = *reinterpret_cast<const uint4 *>(&sm.kt[jtok * KS + ch * 16]);
                    acc = dot2_bf16(a.x, b.x, acc);
                    acc = dot2_bf16(a.y, b.y, acc);
                    acc = dot2_bf16(a.z, b.z, acc);
                    acc = dot2_bf16(a.w, b.w, acc);
                }
                return fmaf(-2.f, acc, sm.nk[etok] + sm.nk[jtok]);
            };
            // row idx of the table as it stands inside the chunk: rows that the chunk opened come from the LDS tile
            auto table_chunk = [&](const int idx) {
                return idx < m0 ? ld16(X + (size_t)idx * ROWB + col * 16)
                                : *reinterpret_cast<const uint4 *>(&sm.kt[opener(idx) * KS + col * 16]);
            };
            int base = m0;   // clusters that exist at the start of the half
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const int nth = nt - 64 * h < 0 ? 0 : (nt - 64 * h > 64 ? 64 : nt - 64 * h);
                const bool valid = j < nth && nkj[h] < INFINITY;
                int done = 0;   // tokens below `done` are final (uniform)
                while (done < nth) {
                    const int mcur = base + __builtin_popcountll(cmask[h] & below);   // clusters when token j arrives
                    // error bound of the approximate distances, and the same plus the index bits of the keys
                    // (relative to the value; a candidate that the chunk itself opened has none, it is treated
                    // alike)
                    const float emax = kDistEps * (nxl[h] + nkj[h]);
                    const float emaxk = emax + ek * fmaxf(fabsf(c1[h]), c2[h] < INFINITY ? fabsf(c2[h]) : 0.f);
                    const bool live = valid && j >= done;
                    const bool amb = distances_ambiguous(c1[h], c2[h], thr, emaxk, mcur);
                    const bool join = mcur > 0 && c1[h] <= thr;
                    const bool forced = decide_cluster(join, ci[h], mcur, st.Mcap).forced;
                    const bool event = live && (amb || (!join && !forced));
                    const uint64_t evmask = __ballot(event);
                    const int e = evmask ? __builtin_ctzll(evmask) : nth;   // first creation / ambiguous token
                    // tokens before the event are final: they join (or are force-joined to) their nearest cluster
                    if (live && j < e) {
                        const int cj = ci[h] < 0 ? 0 : ci[h];   // < 0 only with non-finite representatives (imported state)
                        if constexpr (RES) sm.res.tgt[64 * h + j] = cj;
                        atomicAdd(&cnt[cj], 1);
                        if (forced) atomicOr(&st.flags[sid], 1u);
                        if (st.assign != nullptr && c0 + 64 * h + j < st.assign_cap)
                            st.assign[sid * (size_t)st.assign_cap + c0 + 64 * h + j] = cj;
                    }
                    if (e >= nth) break;
                    const int etok = 64 * h + e;
                    const bool e_amb = (__ballot(amb && live) >> e) & 1ull;
                    const int me = base + __builtin_popcountll(cmask[h]);   // clusters that exist when token e arrives
                    bool create = true;
                    int target = me;
                    if (e_amb) {
                        const uint4 ekey = *reinterpret_cast<const uint4 *>(&sm.kt[etok * KS + col * 16]);
                        double best;
                        int bidx;
                        // every exact distance is at most the bound away from its approximation, so the nearest
                        // representative is among those within twice the bound of the smallest approximation:
                        // when the third smallest is beyond that, these are the best and (perhaps) the
                        // runner-up, and their one or two exact distances decide
                        const bool few = ci[h] >= 0 && (c3[h] == INFINITY ||
                                                        c3[h] - c1[h] > 2.f * emax + ek * (fabsf(c1[h]) + fabsf(c3[h])));
                        if ((__ballot(few) >> e) & 1ull) {
                            const int r1 = __shfl(ci[h], e), r2x = __shfl(ci2[h], e);
                            const int r2 = (__ballot(c2[h] - c1[h] > 2.f * emaxk) >> e) & 1ull ? -1 : r2x;
                            const int rsel = sub == 0 ? r1 : (sub == 1 ? r2 : -1);
                            double dist = INFINITY;
                            if (rsel >= 0) dist = exact_distance<LPR>(table_chunk(rsel), ekey);
                            const double d1 = __shfl(dist, 0), d2 = __shfl(dist, LPR);
                            const bool second = r2 >= 0 && (d2 < d1 || (d2 == d1 && r2 < r1));
                            best = second ? d2 : d1;
                            bidx = second ? r2 : r1;
                        } else {
                            // every row, RPW at a time (rare)
                            best = INFINITY;
                            bidx = -1;
                            for (int r0 = 0; r0 < me; r0 += RPW) {
                                const int r = r0 + sub;
                                const double dist = exact_distance<LPR>(table_chunk(r < me ? r : me - 1), ekey);
                                if (r < me && dist < best) {
                                    best = dist;
                                    bidx = r;
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
                        }
                        const bool ejoin = bidx >= 0 && best <= st.delta2;
                        const Decision dec = decide_cluster(ejoin, bidx, me, st.Mcap);
                        create = dec.created;
                        if (!create) {
                            target = dec.target;
                            if (lane == 0) {
                                atomicAdd(&cnt[target], 1);
                                if (dec.forced) atomicOr(&st.flags[sid], 1u);
                            }
                        }
                    }
                    if (create) {
                        if (lane < LPR)   // the new representative's row comes out of the LDS tile
                            st16(X + (size_t)me * ROWB + lane * 16, *reinterpret_cast<const uint4 *>(&sm.kt[etok * KS + lane * 16]));
                        if (lane == 0) {
                            atomicAdd(&cnt[me], 1);
                            xn[me] = sm.nk[etok];
                        }
                        cmask[h] |= 1ull << e;
                        // the later tokens of the chunk see the new cluster
                        const float nke = sm.nk[etok];
#pragma unroll
                        for (int hh = 0; hh < H; ++hh) {
                            if (hh < h) continue;
                            const float d = token_distance(etok, 64 * hh + j);
                            if (hh > h || j > e) {
                                top3_insert(d, me, c1[hh], ci[hh], c2[hh], ci2[hh], c3[hh]);
                                nxl[hh] = fmaxf(nxl[hh], nke);
                            }
                        }
                    }
                    if (lane == 0 && st.assign != nullptr && c0 + etok < st.assign_cap)
                        st.assign[sid * (size_t)st.assign_cap + c0 + etok] = target;
                    if constexpr (RES) {
                        if (lane == 0) sm.res.tgt[etok] = target;
                    }
                    done = e + 1;
                }
                base += __builtin_popcountll(cmask[h]);
            }
            m = base;

            // ---- sampling: p_j from the running mu (sequential double adds, token order); the coins wait for the
            //      coin pass
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const int nth = nt - 64 * h < 0 ? 0 : (nt - 64 * h > 64 ? 64 : nt - 64 * h);
                if (nth > 0) {
                    const float vnj = sm.vn[64 * h + j];
                    // mu before token j = ((mu + ||v_0||^2) + ...) + ||v_{j-1}||^2, added in this order: every lane
                    // adds the value of the lane below to that lane's sum, so after step l the lanes up to l are
                    // final
                    const double vd = j < nth ? (double)vnj : 0.0;
                    const double vbelow = from_lane_below(vd, 0.0);
                    double muj = mu;
                    for (int l = 1; l < nth; ++l) muj = from_lane_below(muj, muj) + vbelow;   // lane 0 keeps mu
                    const float pj = coin_probability(muj, vnj);
                    const bool valid = j < nth && nkj[h] < INFINITY;
                    sm.plim[span_fill + 64 * h + j] = valid ? coin_limit(pj) : 0u;
                    const double mend = muj + vd;
                    mu = __shfl(mend, nth - 1);
                }
            }
            if (lane == 0) sm.mnew = m;
        }

        // ---- per-cluster reservoirs (UpdateSoftmaxNormalizer of Algorithm 1 as printed): a token that joins a
        //      cluster of (then) n members takes each of the t slots with probability 1/n; the opener of a
        //      cluster takes them all (n = 1).  Within the chunk the last winner of a (cluster, slot) stays.
        if constexpr (RES) {
            const int TT = st.t, TB = (TT + 3) >> 2;
            char *const R = st.R + sid * (size_t)st.Mcap * TT * ROWB;
            __syncthreads();   // every token's cluster is in LDS, the counts of the chunk are in memory
            if (tid < T) {
                const int c = tid < nt ? sm.res.tgt[tid] : -1;
                float prj = -1.f;
                if (c >= 0) {
                    int later = 0;
                    for (int l = tid + 1; l < nt; ++l) later += sm.res.tgt[l] == c;
                    const int nj = atomicAdd(&cnt[c], 0) - later;   // members when this token arrived (itself included)
                    prj = 1.0f / (float)nj;
                }
                sm.res.pr[tid] = prj;
            }
            __syncthreads();
            for (int it = tid; it < T * TB; it += kWG) {
                const int jj = it / TB, b = it % TB;
                const float prj = sm.res.pr[jj];
                uint32_t wbits = 0;
                if (prj > 0.f) {
                    const uint64_t ge = (uint64_t)(c0 + jj);
                    uint32_t r[4];
                    coin_block(st, sid, (int64_t)ge, (uint32_t)b, true, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (4 * b + i < TT && coin_accepts(r[i], prj)) wbits |= 1u << i;
                }
                sm.res.win[jj][b] = (uint8_t)wbits;
            }
            __syncthreads();
            for (int it = tid; it < T * TT; it += kWG) {
                const int jj = it / TT, sl = it % TT;
                if (!((sm.res.win[jj][sl >> 2] >> (sl & 3)) & 1)) continue;
                const int c = sm.res.tgt[jj];
                bool last = true;
                for (int l = jj + 1; l < nt; ++l)
                    if (sm.res.tgt[l] == c && ((sm.res.win[l][sl >> 2] >> (sl & 3)) & 1)) last = false;
                if (last) {
                    const char *ks = krow_of(c0 + jj);
                    char *dst = R + ((size_t)c * TT + sl) * ROWB;
#pragma unroll
                    for (int ch = 0; ch < CPR; ++ch) st16(dst + ch * 16, ld16(ks + ch * 16));
                }
            }
        }
        span_fill += nt;
        if (span_fill + T > kCoinSpan || c0 + T >= ge1) {
            __syncthreads();
            coin_pass(span0, span_fill);
            span0 += span_fill;
            span_fill = 0;
        }
        __syncthreads();   // LDS is reused by the next chunk; new rows are visible
        m = sm.mnew;
    }

    // ---- the ring ends up holding the last min(n, w) tokens of the call
    if (w > 0) {
        __syncthreads();
        const int64_t tfirst = n > w ? n - w : 0;
        const uint32_t sfirst = (uint32_t)((n0 + tfirst) % w);
        for (int64_t t = tfirst + grp; t < n; t += RPB) {
            uint32_t slot = sfirst + (uint32_t)(t - tfirst);
            if (slot >= (uint32_t)w) slot -= (uint32_t)w;
            st16(Kw + slot * ROWB + col * 16, ld16(kin + t * call.token_stride + col * 16));
            st16(Vw + slot * ROWB + col * 16, ld16(vin + t * call.token_stride + col * 16));
        }
    }
    if (tid == 0) {
        st.m[sid] = m;
        st.mu[sid] = mu;
    }
}

}  // namespace sg
