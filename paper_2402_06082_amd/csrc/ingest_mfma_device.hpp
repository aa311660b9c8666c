// Chunked prefix ingest for bf16 rows on gfx950.
//
// A stream's tokens must be clustered in order (the greedy rule is order
// dependent), but the arithmetic of 64 consecutive tokens can be batched:
//   1. distances of the 64 tokens to all representatives that exist at the
//      start of the chunk are one dense (m x 64 x d) contraction on the matrix
//      cores (representatives as the A operand, the 64 token keys as four B
//      operands); every lane tracks best / runner-up for its token;
//   2. distances between the 64 tokens themselves (one more 64 x 64 x d
//      contraction) cover the representatives created inside the chunk;
//   3. a resolve loop, one lane per token, replays the order: a token only
//      sees the chunk's creators that precede it; the loop advances from one
//      creation (or one ambiguous token) to the next, so it runs a few
//      iterations per chunk once the table has filled;
//   4. ambiguous decisions (gap or threshold distance within the error bound
//      of the matrix-core distances) are re-evaluated exactly in double;
//   5. the sampling coins do not depend on the clustering: the chunks only
//      leave each token's probability behind, and once per 1024 evicted
//      tokens (or at the end of the call) one pass draws the coins per 4-slot
//      block; the last accepting token of a slot wins (sequential overwrite
//      semantics), so a slot is copied at most once per pass.
// The window is handled by index arithmetic: the tokens that leave the window
// during the call come first from the ring, then from the call's own input;
// the ring is rewritten once at the end.
#pragma once
#include "subgen_mfma_device.hpp"

namespace sg {

constexpr int kChunkT = 64;  // tokens per chunk = one lane per token in the resolve loop
#ifndef SG_COINSPAN
#define SG_COINSPAN 1024
#endif
constexpr int kCoinSpan = SG_COINSPAN;  // evicted tokens per coin pass (a multiple of the chunk)

template <int NK>
struct SmemIngest {
    alignas(16) float nk[kChunkT];
    float vn[kChunkT];
    // coin bound (coin_limit: a word r is accepted iff r <= bound; 0 = never) and ||v||^2 of the evicted tokens
    // whose coins are still to be drawn (up to kCoinSpan)
    uint32_t plim[kCoinSpan];
    float vnall[kCoinSpan];
    float wb1[kWaves][kChunkT], wb2[kWaves][kChunkT];
    int wi1[kWaves][kChunkT];
    float wnx[kWaves];
    float tt[kChunkT][kChunkT + 1];
    double wbest[kWaves];
    int widx[kWaves];
    // per-cluster reservoirs (t >= 1): cluster of every token of the chunk, its coin probability 1/n_i, and
    // which reservoir slots it wins
    int tgt[kChunkT];
    float pr[kChunkT];
    uint8_t win[kChunkT][16];
    // the chunk's keys, one padded row per token (the pad spreads the 16 rows an operand read touches over
    // all banks): the B operands of every contraction of the chunk are read from here
    static constexpr int KS = NK * 64 + 16;
    alignas(16) char kt[kChunkT * KS];
};

// merge candidate (d, idx) into best / runner-up; lower index wins exact ties of the approximate value
__device__ __forceinline__ void cand_merge(float d, int idx, float &b1, int &i1, float &b2)
{
    if (d < b1 || (d == b1 && (uint32_t)idx < (uint32_t)i1)) {
        b2 = b1;
        b1 = d;
        i1 = idx;
    } else {
        b2 = fminf(b2, d);
    }
}

template <int NK, bool RES>
__global__ __launch_bounds__(kWG, 3) void ingest_mfma_kernel(const State st, const Call call)
{
    static_assert(kWaves == 4, "the chunk layout assumes four wavefronts per workgroup");
    constexpr int T = kChunkT;
    constexpr int CPR = 4 * NK, LPR = CPR;
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)NK * 64;
    constexpr int KS = SmemIngest<NK>::KS;
    constexpr int PF = 2;   // groups of 16 representatives in flight per wavefront (a third one spills)
    __shared__ SmemIngest<NK> sm;

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

    // ---- coin pass over the evicted tokens [g0, g0 + cnt) whose probabilities are in LDS: every lane takes one
    //      4-slot block (and one sub-range of the tokens, so that all lanes have coins to draw) and walks its
    //      tokens from the oldest to the newest; the last accept per slot is the one that stays
    auto coin_pass = [&](int64_t g0, int cnt) {
        const int nblk = (st.s + 3) >> 2;
        int nsplit = 1;
        while (nsplit < 16 && nblk * nsplit * 2 <= kWG) nsplit *= 2;
        const int per = kCoinSpan / nsplit;
        for (int item = tid; item < ((nblk * nsplit + kWG - 1) / kWG) * kWG; item += kWG) {
            const int blk = item / nsplit, part = item % nsplit;
            int last[4] = {-1, -1, -1, -1};
            if (blk < nblk) {
                const int lo = part * per, hi = (part + 1) * per < cnt ? (part + 1) * per : cnt;
                for (int jj = lo; jj < hi; ++jj) {   // oldest first: a later accept overwrites an earlier one
                    const uint32_t lim = sm.plim[jj];
                    if (lim != 0u) {
                        const uint64_t ge = (uint64_t)(g0 + jj);
                        uint32_t r[4];
                        coin_block(st, sid, (int64_t)ge, (uint32_t)blk, false, r);
#pragma unroll
                        for (int i = 0; i < 4; ++i) last[i] = r[i] <= lim ? jj : last[i];
                    }
                }
            }
            // the largest token index over the sub-ranges wins
            for (int o = 1; o < nsplit; o <<= 1) {
#pragma unroll
                for (int i = 0; i < 4; ++i) last[i] = max(last[i], __shfl_xor(last[i], o));
            }
            if (blk < nblk) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int slot = blk * 4 + i;
                    const int owner = nsplit >= 4 ? i : (i % nsplit);   // spread the row copies over the lanes
                    if (part == owner && last[i] >= 0 && slot < st.s) {
                        const char *ks = krow_of(g0 + last[i]), *vs = vrow_of(g0 + last[i]);
#pragma unroll
                        for (int ch = 0; ch < CPR; ++ch) {
                            st16(Ks + (size_t)slot * ROWB + ch * 16, ld16(ks + ch * 16));
                            st16(Vs + (size_t)slot * ROWB + ch * 16, ld16(vs + ch * 16));
                        }
                        st.sidx[sid * (size_t)st.sS + slot] = (int32_t)(g0 + last[i]);
                        st.svn[sid * (size_t)st.sS + slot] = sm.vnall[last[i]];
                    }
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

        // ---- squared norms of the chunk's keys and values (double, exact products), one token per lane group
        {
            constexpr int NP = T / RPB;   // passes of the lane groups over the 64 tokens
            uint4 rk[NP], rv[NP];
#pragma unroll
            for (int it = 0; it < NP; ++it) {   // all row loads first
                const int j = grp + it * RPB;
                const int jj = j < nt ? j : nt - 1;
                rk[it] = ld16(krow_of(c0 + jj) + col * 16);
                rv[it] = ld16(vrow_of(c0 + jj) + col * 16);
            }
#pragma unroll
            for (int it = 0; it < NP; ++it) {
                float kf[8], vf[8];
                unpack<true>(rk[it], kf);
                unpack<true>(rv[it], vf);
                *reinterpret_cast<uint4 *>(&sm.kt[(grp + it * RPB) * KS + col * 16]) = rk[it];
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
                    sm.nk[grp + it * RPB] = bad ? INFINITY : (float)a;
                    sm.vn[grp + it * RPB] = bad ? 0.f : (float)b;
                    if (bad && grp + it * RPB < nt) atomicOr(&st.flags[sid], 2u);
                }
            }
        }
        // ---- B operand (ts, kk): token 16 ts + n in column n, read from the LDS tile
        auto bop = [&](int ts, int kk) __attribute__((always_inline)) {
            return *reinterpret_cast<const uint4 *>(&sm.kt[(16 * ts + n16) * KS + (L + 4 * kk) * 16]);
        };
        __syncthreads();
        float nkt[4];
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) nkt[ts] = sm.nk[16 * ts + n16];

        // ---- token-token distances: wavefront `wave` takes rows 16 wave .. 16 wave + 15 (its A operand is
        //      B set `wave`)
        {
            const float4 nkr = *reinterpret_cast<const float4 *>(&sm.nk[16 * wave + 4 * L]);
            const float nkrow[4] = {nkr.x, nkr.y, nkr.z, nkr.w};
            uint4 arow[NK];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) arow[kk] = bop(wave, kk);
#pragma unroll
            for (int ts = 0; ts < 4; ++ts) {
                floatx4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(arow[kk], bop(ts, kk), c);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    sm.tt[16 * wave + 4 * L + r][16 * ts + n16] = fmaf(-2.f, c[r], nkrow[r] + nkt[ts]);
            }
        }

        // ---- distances to the representatives that exist at the start of the chunk
        float b1[4], b2[4], nxmax = 0.f;
        int i1[4];
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) {
            b1[ts] = INFINITY;
            b2[ts] = INFINITY;
            i1[ts] = -1;
        }
        for (int r0 = wave * 16; r0 < m0; r0 += 16 * kWaves) {
            // the oldest request is this group; the queue moves up and takes one more request at its end
            uint4 a[NK];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) a[kk] = q[0][kk];
            const float nxr[4] = {qn[0].x, qn[0].y, qn[0].z, qn[0].w};
#pragma unroll
            for (int pf = 0; pf + 1 < PF; ++pf) {
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) q[pf][kk] = q[pf + 1][kk];
                qn[pf] = qn[pf + 1];
            }
            request(q[PF - 1], qn[PF - 1], r0 + 16 * kWaves * PF);
            // the B operands do not change from group to group: without this the compiler keeps all of them
            // in registers over the loop, which is what the LDS tile is there to avoid
            asm volatile("" ::: "memory");
            const int row0 = r0 + 4 * L;
            uint4 bq[NK];   // operands of the next token set, read while the current one is on the matrix cores
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) bq[kk] = bop(0, kk);
#pragma unroll
            for (int ts = 0; ts < 4; ++ts) {
                floatx4_t c = {0.f, 0.f, 0.f, 0.f};
                uint4 b[NK];
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) b[kk] = bq[kk];
                if (ts + 1 < 4) {
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) bq[kk] = bop(ts + 1, kk);
                }
#pragma unroll
                for (int kk = 0; kk < NK; ++kk) c = mfma_bf16(a[kk], b[kk], c);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // rows past the table (the clamped loads of the last group) take part as +inf
                    const float dt = row0 + r < m0 ? fmaf(-2.f, c[r], nxr[r] + nkt[ts]) : INFINITY;
                    const bool first = dt < b1[ts];
                    b2[ts] = first ? b1[ts] : fminf(b2[ts], dt);
                    i1[ts] = first ? row0 + r : i1[ts];
                    b1[ts] = first ? dt : b1[ts];
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) nxmax = fmaxf(nxmax, row0 + r < m0 ? nxr[r] : 0.f);
        }
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) {
#pragma unroll
            for (int o = 16; o < 64; o <<= 1) {
                const float ob1 = __shfl_xor(b1[ts], o), ob2 = __shfl_xor(b2[ts], o);
                const int oi1 = __shfl_xor(i1[ts], o);
                if (ob1 < b1[ts] || (ob1 == b1[ts] && (uint32_t)oi1 < (uint32_t)i1[ts])) {
                    b2[ts] = fminf(b1[ts], ob2);
                    b1[ts] = ob1;
                    i1[ts] = oi1;
                } else {
                    b2[ts] = fminf(b2[ts], ob1);
                }
            }
            if (L == 0) {
                sm.wb1[wave][16 * ts + n16] = b1[ts];
                sm.wb2[wave][16 * ts + n16] = b2[ts];
                sm.wi1[wave][16 * ts + n16] = i1[ts];
            }
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) nxmax = fmaxf(nxmax, __shfl_xor(nxmax, o));
        if (lane == 0) sm.wnx[wave] = nxmax;
        if constexpr (RES) {
            if (wave == 0) sm.tgt[lane] = -1;   // dropped tokens and the ragged tail keep -1
        }
        __syncthreads();

        // ---- resolve in token order: lane j = token j of the chunk; every wavefront runs the same loop
        //      (same LDS inputs, same results), wavefront 0 applies the side effects
        const int j = lane;
        const float nkj = sm.nk[j];
        const bool valid = j < nt && nkj < INFINITY;
        float ob1 = sm.wb1[0][j], ob2 = sm.wb2[0][j];
        int oi1 = sm.wi1[0][j];
        float nxold = sm.wnx[0];
#pragma unroll
        for (int wv = 1; wv < kWaves; ++wv) {
            const float x1 = sm.wb1[wv][j], x2 = sm.wb2[wv][j];
            const int xi = sm.wi1[wv][j];
            if (x1 < ob1 || (x1 == ob1 && (uint32_t)xi < (uint32_t)oi1)) {
                ob2 = fminf(ob1, x2);
                ob1 = x1;
                oi1 = xi;
            } else {
                ob2 = fminf(ob2, x1);
            }
            nxold = fmaxf(nxold, sm.wnx[wv]);
        }
        uint64_t cmask = 0;   // tokens of this chunk that opened a cluster (uniform)
        int done = 0;         // tokens below `done` are final (uniform)
        const uint64_t below = j == 0 ? 0ull : (~0ull >> (64 - j));
        while (done < nt) {
            float c1 = ob1, c2 = ob2, nxl = nxold;
            int ci = oi1;
            uint64_t rest = cmask;
            while (rest) {   // uniform loop over the creators; a lane only sees those before it
                const int l = __builtin_ctzll(rest);
                rest &= rest - 1;
                if (l < j) {
                    cand_merge(sm.tt[l][j], m0 + __builtin_popcountll(cmask & (l == 0 ? 0ull : (~0ull >> (64 - l)))), c1,
                               ci, c2);
                    nxl = fmaxf(nxl, sm.nk[l]);
                }
            }
            const int mcur = m0 + __builtin_popcountll(cmask & below);   // clusters that exist when token j arrives
            const float emax = kDistEps * (nxl + nkj);
            const bool live = valid && j >= done;
            const bool amb = distances_ambiguous(c1, c2, thr, emax, mcur);
            const bool join = mcur > 0 && c1 <= thr;
            const bool forced = decide_cluster(join, ci, mcur, st.Mcap).forced;
            const bool event = live && (amb || (!join && !forced));
            const uint64_t evmask = __ballot(event);
            const int e = evmask ? __builtin_ctzll(evmask) : nt;   // first creation / ambiguous token
            // tokens before the event are final: they join (or are force-joined to) their nearest cluster
            if (wave == 0 && live && j < e) {
                if (ci < 0) ci = 0;   // only with non-finite representatives (imported state)
                if constexpr (RES) sm.tgt[j] = ci;
                atomicAdd(&cnt[ci], 1);
                if (forced) atomicOr(&st.flags[sid], 1u);
                if (st.assign != nullptr && c0 + j < st.assign_cap) st.assign[sid * (size_t)st.assign_cap + c0 + j] = ci;
            }
            if (e >= nt) break;
            const bool e_amb = (__ballot(amb && live) >> e) & 1ull;
            const int me = m0 + __builtin_popcountll(cmask);   // clusters that exist when token e arrives
            bool create = true;
            int target = me;
            if (e_amb) {
                __syncthreads();   // rows of this chunk's creators are visible to every wavefront
                double best;
                int bidx;
                exact_nearest<LPR>(X, me, *reinterpret_cast<const uint4 *>(&sm.kt[e * KS + col * 16]), sm.wbest, sm.widx, best,
                              bidx);
                const bool ejoin = bidx >= 0 && best <= st.delta2;
                const Decision dec = decide_cluster(ejoin, bidx, me, st.Mcap);
                const bool eforced = dec.forced;
                create = dec.created;
                if (!create) {
                    bidx = dec.target;
                    target = bidx;
                    if (tid == 0) {
                        atomicAdd(&cnt[bidx], 1);
                        if (eforced) atomicOr(&st.flags[sid], 1u);
                    }
                }
            }
            if (create) {
                if (tid < LPR)   // the new representative's row comes out of the LDS tile
                    st16(X + (size_t)me * ROWB + tid * 16, *reinterpret_cast<const uint4 *>(&sm.kt[e * KS + tid * 16]));
                if (tid == 0) {
                    atomicAdd(&cnt[me], 1);
                    xn[me] = sm.nk[e];
                }
                cmask |= 1ull << e;
            }
            if (tid == 0 && st.assign != nullptr && c0 + e < st.assign_cap)
                st.assign[sid * (size_t)st.assign_cap + c0 + e] = target;
            if constexpr (RES) {
                if (tid == 0) sm.tgt[e] = target;
            }
            done = e + 1;
        }
        m = m0 + __builtin_popcountll(cmask);

        // ---- per-cluster reservoirs (UpdateSoftmaxNormalizer of Algorithm 1 as printed): a token that joins a
        //      cluster of (then) n members takes each of the t slots with probability 1/n; the opener of a
        //      cluster takes them all (n = 1).  Within the chunk the last winner of a (cluster, slot) stays.
        if constexpr (RES) {
            const int TT = st.t, TB = (TT + 3) >> 2;
            char *const R = st.R + sid * (size_t)st.Mcap * TT * ROWB;
            __syncthreads();   // every token's cluster is in LDS, the counts of the chunk are in memory
            if (tid < T) {
                const int c = tid < nt ? sm.tgt[tid] : -1;
                float prj = -1.f;
                if (c >= 0) {
                    int later = 0;
                    for (int l = tid + 1; l < nt; ++l) later += sm.tgt[l] == c;
                    const int nj = atomicAdd(&cnt[c], 0) - later;   // members when this token arrived (itself included)
                    prj = 1.0f / (float)nj;
                }
                sm.pr[tid] = prj;
            }
            __syncthreads();
            for (int it = tid; it < T * TB; it += kWG) {
                const int jj = it / TB, b = it % TB;
                const float prj = sm.pr[jj];
                uint32_t wbits = 0;
                if (prj > 0.f) {
                    const uint64_t ge = (uint64_t)(c0 + jj);
                    uint32_t r[4];
                    coin_block(st, sid, (int64_t)ge, (uint32_t)b, true, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (4 * b + i < TT && coin_accepts(r[i], prj)) wbits |= 1u << i;
                }
                sm.win[jj][b] = (uint8_t)wbits;
            }
            __syncthreads();
            for (int it = tid; it < T * TT; it += kWG) {
                const int jj = it / TT, sl = it % TT;
                if (!((sm.win[jj][sl >> 2] >> (sl & 3)) & 1)) continue;
                const int c = sm.tgt[jj];
                bool last = true;
                for (int l = jj + 1; l < nt; ++l)
                    if (sm.tgt[l] == c && ((sm.win[l][sl >> 2] >> (sl & 3)) & 1)) last = false;
                if (last) {
                    const char *ks = krow_of(c0 + jj);
                    char *dst = R + ((size_t)c * TT + sl) * ROWB;
#pragma unroll
                    for (int ch = 0; ch < CPR; ++ch) st16(dst + ch * 16, ld16(ks + ch * 16));
                }
            }
        }

        // ---- sampling: p_j from the running mu (sequential double adds, token order); the coins wait for the
        //      coin pass
        if (wave == 0) {
            const float vnj = sm.vn[j];
            const double vd = (double)vnj;
            const int vlo = (int)(__builtin_bit_cast(uint64_t, vd) & 0xffffffffull);
            const int vhi = (int)(__builtin_bit_cast(uint64_t, vd) >> 32);
            double muj = mu;
            for (int l = 0; l < nt; ++l) {   // lane l's value through the scalar unit, no LDS round trip per step
                const uint64_t bits = (uint64_t)(uint32_t)__builtin_amdgcn_readlane(vlo, l) |
                                      ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(vhi, l) << 32);
                if (l < j) muj += __builtin_bit_cast(double, bits);
            }
            const float pj = coin_probability(muj, vnj);
            sm.plim[span_fill + j] = valid ? coin_limit(pj) : 0u;
            sm.vnall[span_fill + j] = vnj;
            const double mend = muj + (double)vnj;
            mu = __shfl(mend, nt - 1);
        }
        span_fill += nt;
        if (span_fill + T > kCoinSpan || c0 + T >= ge1) {
            __syncthreads();
            coin_pass(span0, span_fill);
            span0 += span_fill;
            span_fill = 0;
        }
        __syncthreads();   // LDS is reused by the next chunk; new rows are visible
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
