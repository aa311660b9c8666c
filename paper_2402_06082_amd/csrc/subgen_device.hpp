// Device code of the SubGen decode step for gfx950 (wave64).
//
// One workgroup of 64*kWaves lanes (4 wavefronts by default) owns one stream for the whole
// kernel, so no two workgroups ever touch the same state.  Rows (centers,
// sampled keys/values, window keys/values) are d contiguous elements; a row is
// read by LPR consecutive lanes with one 16-byte load each, so one wavefront
// load instruction fetches 64/LPR complete rows, fully coalesced.  Dot
// products and squared distances are reduced across the LPR lanes of a row
// group with cross-lane shuffles.  The softmax is kept online (running
// maximum, denominator, fp32 accumulator) per row group and merged at the end.
//
// Decisions that produce integers (nearest center, threshold test, sampling
// coin flips) are taken in double precision from the exactly converted
// inputs, so they do not depend on the summation order beyond the last bits
// of a double.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sg {

#ifndef SG_WAVES
#define SG_WAVES 4
#endif
constexpr int kWaves = SG_WAVES;  // wavefronts per workgroup
constexpr int kWG = 64 * kWaves;
constexpr int kQueue = 4 * kWG;  // sample slots handled per round of the sampling update (4 per lane)
#ifndef SG_UNROLL
#define SG_UNROLL 4
#endif
constexpr int kUnroll = SG_UNROLL;  // row loads in flight per lane in the scans

// Pointers into the context's structure-of-arrays state (all device memory).
struct State {
    char *X;            // [S][Mcap][d]   cluster representatives x_i
    int32_t *cnt;       // [S][McapS]     cluster sizes n_i
    char *R;            // [S][Mcap][t][d] per-cluster reservoirs S_i (t >= 1), else null
    float *xn;          // [S][McapS]     ||x_i||^2 (fp32 rounding of the exact sum), used by the MFMA path
    int32_t *m;         // [S]            number of clusters
    char *Ks, *Vs;      // [S][s][d]      sampled pairs M
    int32_t *sidx;      // [S][sS]        token index held by each slot (-1 = null)
    float *svn;         // [S][sS]        ||v||^2 of that token
    char *Kw, *Vw;      // [S][w][d]      window ring, slot = token index mod w
    double *mu;         // [S]            sum of ||v||^2 over evicted tokens
    uint32_t *flags;    // [S]            sticky flag word
    int32_t *assign;    // [S][assign_cap] or null
    int64_t assign_cap;
    int32_t Mcap, s, w, d;
    int32_t t;          // reservoir slots per cluster (0 = representative mode)
    int32_t McapS, sS;  // strides of the per-center / per-slot scalar arrays (Mcap, s rounded up to 16)
    double delta2;      // delta^2
    uint32_t seed_lo, seed_hi;
    int64_t *seen;      // [1] tokens seen by every stream, kept on the device (contexts made for graph capture), or null
    int32_t out_bf16;   // outputs are written as bf16 (round to nearest even) instead of fp32
    // contexts of a few streams: split_P workgroups share a stream (0 = one workgroup per stream)
    int32_t split_P;
    uint32_t *split_cnt;   // [S]        workgroups of the stream that have arrived in the current launch
    float *split_part;     // [S][P][.]  their partial results
};

// Tokens seen before this launch: the host's count (a kernel argument), or, in contexts that keep the count on the
// device so that a captured launch can be replayed, the device's.
__device__ __forceinline__ int64_t tokens_seen(const State &st, const int64_t host_count)
{
    return st.seen != nullptr ? *st.seen : host_count;
}

// runs after the kernels of an update in such contexts
__global__ void bump_seen_kernel(int64_t *seen, int64_t n) { *seen += n; }

struct Call {
    const char *K, *V;        // new tokens; token t of stream j at K + j*stream_stride + t*token_stride (bytes)
    int64_t stream_stride, token_stride;
    int64_t n_tokens;         // tokens per stream in this call (1 for update / step)
    const char *Q;            // [S][G][d] or null
    float *out;               // [S][G][d] fp32 or null
    int64_t n_seen;           // tokens seen by every stream before this call
    int64_t q_stride;         // bytes between the query blocks of two streams
    int64_t out_stride;       // floats between the output blocks of two streams
};

// ---------------------------------------------------------------------------
// Philox-4x32, 10 rounds (Salmon et al., SC'11), written from the published
// description.  Counter (slot block, token lo, token hi, stream), key = seed.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1, uint32_t (&r)[4])
{
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        // one 32x32->64 multiply per half round (a single v_mad_u64_u32) instead of separate high and low products
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        c0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        c1 = (uint32_t)p1;
        c2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c3 = (uint32_t)p0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    r[0] = c0; r[1] = c1; r[2] = c2; r[3] = c3;
}

// ---------------------------------------------------------------------------
// The readings of Algorithm 1 that every kernel family shares, each in one place.
// ---------------------------------------------------------------------------

// Sliding window (Section 3.2) by deferred insertion: token n goes into ring slot n mod w and the token that was
// there, n - w, is the one that is clustered and offered to the sampler; with w = 0 the new token itself is
// (plain Algorithm 1).  slot is -1 when there is no ring.
struct Eviction {
    bool evict;       // a token leaves the window in this step
    int64_t token;    // its index
    int slot;         // ring slot of the new token (which still holds the leaving token's rows)
};
__device__ __forceinline__ Eviction window_push(const int64_t n_seen, const int w)
{
    if (w == 0) return Eviction{true, n_seen, -1};
    return Eviction{n_seen >= w, n_seen - w, (int)(n_seen % w)};
}

// A token whose ||k||^2 or ||v||^2 (double sums rounded to fp32) is not finite is dropped when it leaves the
// window: not clustered, not sampled, flag bit 2.
__device__ __forceinline__ bool token_is_finite(const float kk, const float vn) { return kk < INFINITY && vn < INFINITY; }

// UpdateSoftmaxNormalizer, the decision once the nearest representative is known: `join` says that there is one
// within delta (||k - x|| <= delta, tested on squared values; lowest index on ties is the caller's argmin rule).
// Otherwise a new cluster is opened, unless the table is full: then the token joins its nearest cluster
// regardless of delta (flag bit 1).  bidx < 0 with a full table only happens with non-finite representatives
// (imported state): cluster 0 takes the token.
struct Decision {
    bool created, forced;
    int target;       // cluster that gains the token (m for a new one)
};
__device__ __forceinline__ Decision decide_cluster(const bool join, int bidx, const int m, const int Mcap)
{
    if (!join && bidx < 0 && m >= Mcap) bidx = 0;
    const bool forced = !join && m > 0 && m >= Mcap;
    const bool created = !join && !forced;
    return Decision{created, forced, created ? m : bidx};
}

// Approximate squared distances D~ (error at most emax each) decide only when both the best / runner-up gap and
// the distance to the threshold exceed their error; otherwise the caller re-evaluates exactly in double.
__device__ __forceinline__ bool distances_ambiguous(const float b1, const float b2, const float thr, const float emax,
                                                    const int m)
{
    return m > 0 && (!(b2 - b1 > 2.f * emax) || !(fabsf(b1 - thr) > emax + 1e-6f * thr));
}

// UpdateMatrixProduct: probability of the coin of every slot, p = ||v||^2 / (mu + ||v||^2) with the mu from
// before this token, rounded to fp32; mu = 0 gives 1 (the first token fills all slots), a zero-norm value 0.
__device__ __forceinline__ float coin_probability(const double mu, const float vn)
{
    if (mu == 0.0) return 1.f;
    if (vn == 0.f) return 0.f;
    return (float)((double)vn / (mu + (double)vn));
}

// The coins: slot j of token t of stream sid takes word j mod 4 of the Philox block with counter
// (j div 4, t lo, t hi, sid) and the seed as key; the reservoir coins of a cluster (t >= 1 slots per cluster) use
// the same generator with the top bit of the third counter word set.  u = (word >> 8) 2^-24; accepted iff u < p.
__device__ __forceinline__ void coin_block(const State &st, const size_t sid, const int64_t token, const uint32_t block,
                                           const bool reservoir, uint32_t (&r)[4])
{
    philox4x32_10(block, (uint32_t)token, (uint32_t)((uint64_t)token >> 32) | (reservoir ? 0x80000000u : 0u),
                  (uint32_t)sid, st.seed_lo, st.seed_hi, r);
}
__device__ __forceinline__ bool coin_accepts(const uint32_t word, const float p)
{
    return (float)(word >> 8) * (1.0f / 16777216.0f) < p;
}
// The same test in integer form, for loops that draw many coins against one p: p 2^24 is exact in fp32, so
// u < p  <=>  (word >> 8) < ceil(p 2^24)  <=>  word <= 256 ceil(p 2^24) - 1 in 32-bit arithmetic (p = 1 wraps to
// 0xffffffff: always).  0 stands for p = 0 (never; the bound of a positive p is at least 255).
__device__ __forceinline__ uint32_t coin_limit(const float p)
{
    return p > 0.f ? (uint32_t)ceilf(p * 16777216.0f) * 256u - 1u : 0u;
}

// ---------------------------------------------------------------------------
// 16-byte row chunks
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint4 ld16(const char *p) { return *reinterpret_cast<const uint4 *>(p); }
// streaming load: the row is read once per kernel, so it should not displace anything in the caches
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ldnt16(const char *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16(char *p, uint4 v) { *reinterpret_cast<uint4 *>(p) = v; }

template <bool BF16>
__device__ __forceinline__ void unpack(const uint4 &r, float *f)
{
    if constexpr (BF16) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
    } else {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
}

template <int LPR, typename T>
__device__ __forceinline__ T group_sum(T v)
{
#pragma unroll
    for (int o = 1; o < LPR; o <<= 1) v += __shfl_xor(v, o);
    return v;
}

// Workgroup barrier that orders LDS traffic only: global loads that are in flight (the prefetched rows) stay in
// flight across it.  Use __syncthreads() where global memory written by one lane is read by another.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// all-reduce over the 16 lanes of a DPP row (row rotations by 8, 4, 2, 1)
template <int N>
__device__ __forceinline__ float row_ror(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xf, 0xf,
                                                                 false));
}
template <int N>
__device__ __forceinline__ int row_ror(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x120 + N, 0xf, 0xf, false);
}
__device__ __forceinline__ float row_sum16(float v)
{
    v += row_ror<8>(v);
    v += row_ror<4>(v);
    v += row_ror<2>(v);
    v += row_ror<1>(v);
    return v;
}

// Attention outputs are fp32 or bf16 (a context option).  `rows` is the base of one stream's outputs, found by
// out_rows() below; element i is stored in the context's output type.
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN (quiet)
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float *out_rows(const State &st, float *out, size_t elems)
{
    return reinterpret_cast<float *>(reinterpret_cast<char *>(out) + elems * (st.out_bf16 ? 2 : 4));
}
__device__ __forceinline__ void put_out(const State &st, float *rows, size_t i, float v)
{
    if (st.out_bf16) reinterpret_cast<uint16_t *>(rows)[i] = (uint16_t)f32_to_bf16_rne(v);
    else rows[i] = v;
}

// online-softmax partial of one row group for one query
template <int VEC>
struct Partial {
    float mx, den;
    float acc[VEC];
    __device__ __forceinline__ void init()
    {
        mx = -INFINITY;
        den = 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    }
    // bring the running maximum up to at least b
    __device__ __forceinline__ void raise(float b)
    {
        if (b > mx) {
            const float sc = __expf(mx - b);  // mx = -inf gives 0
            den *= sc;
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] *= sc;
            mx = b;
        }
    }
    __device__ __forceinline__ void merge(float omx, float oden, const float *oacc)
    {
        const float M = fmaxf(mx, omx);
        const float a = (mx == -INFINITY) ? 0.f : __expf(mx - M);
        const float b = (omx == -INFINITY) ? 0.f : __expf(omx - M);
        den = den * a + oden * b;
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = acc[v] * a + oacc[v] * b;
        mx = M;
    }
};

template <int LPR, int G, int VEC>
struct Smem {
    double wbest[kWaves];
    int widx[kWaves];
    float wbsc[kWaves][G];
    float wmx[kWaves][G], wden[kWaves][G];
    float wacc[kWaves][G][LPR * VEC];
    int qn;
    int queue[kQueue];
};

// ---------------------------------------------------------------------------
// One token of one stream: window push/evict, cluster update, sampling update
// (UPD) and/or the attention estimate for G queries (ATT).  Called by every
// lane of the workgroup with block-uniform arguments; m and mu are carried by
// the caller (block-uniform) and written back by it.
// ---------------------------------------------------------------------------
template <bool BF16, int LPR, int G, bool UPD, bool ATT>
__device__ __forceinline__ void token_step(const State &st, const size_t sid, const char *krow, const char *vrow,
                                           const char *qrows, float *outrows, const int64_t n_seen, int &m,
                                           double &mu, Smem<LPR, G, (BF16 ? 8 : 4)> &sm)
{
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int RPW = 64 / LPR;        // rows per wavefront load
    constexpr int RPB = RPW * kWaves;    // rows per workgroup iteration
    constexpr size_t ROWB = (size_t)LPR * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR;
    const int grp = wave * RPW + sub;

    char *const X = st.X + sid * (size_t)st.Mcap * ROWB;
    int32_t *const cnt = st.cnt + sid * (size_t)st.McapS;
    char *const Ks = st.Ks + sid * (size_t)st.s * ROWB;
    char *const Vs = st.Vs + sid * (size_t)st.s * ROWB;
    char *const Kw = st.Kw + sid * (size_t)st.w * ROWB;
    char *const Vw = st.Vw + sid * (size_t)st.w * ROWB;

    // ---- window push; the token that leaves the window is the one that is compressed
    bool evict = false;
    int64_t etoken = 0;
    uint4 ek = make_uint4(0, 0, 0, 0), ev = make_uint4(0, 0, 0, 0);
    if constexpr (UPD) {
        const Eviction wp = window_push(n_seen, st.w);
        evict = wp.evict;
        etoken = wp.token;
        if (wp.slot < 0) {
            ek = ld16(krow + col * 16);
            ev = ld16(vrow + col * 16);
        } else {
            const int slot = wp.slot;
            char *kw = Kw + (size_t)slot * ROWB, *vw = Vw + (size_t)slot * ROWB;
            if (evict) {
                ek = ld16(kw + col * 16);
                ev = ld16(vw + col * 16);
            }
            __syncthreads();  // every lane holds the evicted row before the slot is overwritten
            if (tid < LPR) {
                st16(kw + tid * 16, ld16(krow + tid * 16));
                st16(vw + tid * 16, ld16(vrow + tid * 16));
            }
        }
    }
    const int64_t n_after = UPD ? n_seen + 1 : n_seen;
    const int64_t n_evicted_after = st.w == 0 ? n_after : (n_after > st.w ? n_after - st.w : 0);

    float q[G][VEC];
    if constexpr (ATT) {
#pragma unroll
        for (int g = 0; g < G; ++g) unpack<BF16>(ld16(qrows + (size_t)g * ROWB + col * 16), q[g]);
    }
    double ekd[VEC];
    double kk2 = 0.0;   // ||k'||^2
    float vn = 0.f;     // ||v'||^2
    float bnew[G];  // <q, evicted key>: score of the cluster this token would open
    if constexpr (UPD) {
        float ekf[VEC];
        unpack<BF16>(ek, ekf);
#pragma unroll
        for (int v = 0; v < VEC; ++v) ekd[v] = (double)ekf[v];
        // ||k'||^2 and ||v'||^2 in double; a token with NaN or Inf in it is dropped and flagged
        {
            float evf[VEC];
            unpack<BF16>(ev, evf);
            double vv2 = 0.0;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                kk2 = fma(ekd[v], ekd[v], kk2);
                vv2 = fma((double)evf[v], (double)evf[v], vv2);
            }
            kk2 = group_sum<LPR>(kk2);
            vn = (float)group_sum<LPR>(vv2);
            if (evict && !token_is_finite((float)kk2, vn)) {
                evict = false;
                if (tid == 0) st.flags[sid] |= 2u;
            }
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

    Partial<VEC> part[G];
#pragma unroll
    for (int g = 0; g < G; ++g) part[g].init();

    // ---- one pass over the representatives: squared distance to the evicted key (double)
    //      and count-weighted exp(<q, x_i>) for the softmax normaliser
    double best = INFINITY;
    int bidx = -1;
    float bsc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) bsc[g] = 0.f;

    if ((UPD && evict) || ATT) {
        for (int r0 = wave * RPW; r0 < m; r0 += RPB * kUnroll) {
            // issue all row loads of this iteration before any arithmetic (memory-level parallelism)
            uint4 raw[kUnroll];
            float cf[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int r = r0 + u * RPB + sub;
                const int rr = r < m ? r : m - 1;
                raw[u] = ldnt16(X + (size_t)rr * ROWB + col * 16);
                if constexpr (ATT) cf[u] = (float)cnt[rr];
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int r = r0 + u * RPB + sub;
                const bool valid = r < m;
                float x[VEC];
                unpack<BF16>(raw[u], x);
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
                            part[g].den += cf[u] * __expf(b[g] - part[g].mx);
                        }
                    }
                }
                if constexpr (UPD) {
                    if (evict && valid && dist < best) {
                        best = dist;
                        bidx = r;
                        if constexpr (ATT) {
#pragma unroll
                            for (int g = 0; g < G; ++g) bsc[g] = b[g];
                        }
                    }
                }
            }
        }
    }

    if constexpr (UPD) {
        if (evict) {
            // ---- nearest representative over the workgroup (lowest index on ties)
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
            __syncthreads();
            best = sm.wbest[0];
            bidx = sm.widx[0];
            int bw = 0;
#pragma unroll
            for (int wv = 1; wv < kWaves; ++wv) {
                const double ob = sm.wbest[wv];
                const int oi = sm.widx[wv];
                if (ob < best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
                    best = ob;
                    bidx = oi;
                    bw = wv;
                }
            }
            // ---- join iff ||k - x_i*||^2 <= delta^2, else open a cluster (or force-join when full)
            const bool join = bidx >= 0 && best <= st.delta2;
            const Decision dec = decide_cluster(join, bidx, m, st.Mcap);
            const bool forced = dec.forced, created = dec.created;
            const int target = dec.target;
            if (created) {
                if (tid < LPR) st16(X + (size_t)m * ROWB + tid * 16, ek);
                if (tid == 0) {
                    cnt[m] = 1;
                    st.xn[sid * (size_t)st.McapS + m] = (float)kk2;
                }
            } else if (tid == 0) {
                cnt[target] += 1;
                if (forced) st.flags[sid] |= 1u;
            }
            if (tid == 0 && st.assign != nullptr && etoken < st.assign_cap)
                st.assign[sid * (size_t)st.assign_cap + etoken] = target;
            if constexpr (ATT) {
                // the count bump (or the new cluster) adds one more term to the normaliser;
                // every lane of one row group takes it so the group's partial stays consistent
                if (grp == 0) {
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const float bx = created ? bnew[g] : sm.wbsc[bw][g];
                        part[g].raise(bx);
                        part[g].den += __expf(bx - part[g].mx);
                    }
                }
            }
            if (created) m += 1;

            // ---- sampling update: p from the old mu, one coin per slot, then mu += ||v||^2
            const float p = coin_probability(mu, vn);

            for (int base = 0; base < st.s; base += kQueue) {
                if (tid == 0) sm.qn = 0;
                __syncthreads();
                const int j0 = base + tid * 4;
                if (j0 < st.s && p > 0.f) {
                    uint32_t r[4];
                    coin_block(st, sid, etoken, (uint32_t)(j0 >> 2), false, r);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (j0 + i < st.s && coin_accepts(r[i], p)) sm.queue[atomicAdd(&sm.qn, 1)] = j0 + i;
                    }
                }
                __syncthreads();
                const int nq = sm.qn;
                for (int e = grp; e < nq; e += RPB) {
                    const int j = sm.queue[e];
                    st16(Ks + (size_t)j * ROWB + col * 16, ek);
                    st16(Vs + (size_t)j * ROWB + col * 16, ev);
                    if (col == 0) {
                        st.sidx[sid * (size_t)st.sS + j] = (int32_t)etoken;
                        st.svn[sid * (size_t)st.sS + j] = vn;
                    }
                }
                __syncthreads();
            }
            mu += (double)vn;
        }
        __syncthreads();  // window slot, center row and sample rows are visible to the whole workgroup
    }

    if constexpr (ATT) {
        // ---- sampled pairs: numerator terms  mu/(s ||v_j||^2) e^{<q,k_j>} v_j
        if (n_evicted_after > 0) {
            const float wmul = (float)(mu / (double)st.s);
            const float *svn = st.svn + sid * (size_t)st.sS;
            for (int r0 = wave * RPW; r0 < st.s; r0 += RPB * kUnroll) {
                uint4 rk[kUnroll], rv[kUnroll];
                float vnj[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int r = r0 + u * RPB + sub;
                    const int rr = r < st.s ? r : st.s - 1;
                    rk[u] = ldnt16(Ks + (size_t)rr * ROWB + col * 16);
                    rv[u] = ldnt16(Vs + (size_t)rr * ROWB + col * 16);
                    vnj[u] = svn[rr];
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const bool valid = r0 + u * RPB + sub < st.s;
                    float kx[VEC], vx[VEC];
                    unpack<BF16>(rk[u], kx);
                    unpack<BF16>(rv[u], vx);
                    const float wgt = vnj[u] > 0.f ? wmul / vnj[u] : 0.f;
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
        // ---- window: exact terms in numerator and normaliser
        const int fill = (int)(n_after < st.w ? n_after : st.w);
        for (int r0 = wave * RPW; r0 < fill; r0 += RPB * kUnroll) {
            uint4 rk[kUnroll], rv[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int r = r0 + u * RPB + sub;
                const int rr = r < fill ? r : fill - 1;
                rk[u] = ldnt16(Kw + (size_t)rr * ROWB + col * 16);
                rv[u] = ldnt16(Vw + (size_t)rr * ROWB + col * 16);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const bool valid = r0 + u * RPB + sub < fill;
                float kx[VEC], vx[VEC];
                unpack<BF16>(rk[u], kx);
                unpack<BF16>(rv[u], vx);
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

// ---------------------------------------------------------------------------
// Kernels: grid = streams, block = kWG lanes
// ---------------------------------------------------------------------------
template <bool BF16, int LPR, int G, bool UPD, bool ATT>
__global__ __launch_bounds__(kWG) void decode_kernel(const State st, const Call call)
{
    constexpr int VEC = BF16 ? 8 : 4;
    __shared__ Smem<LPR, G, VEC> sm;
    const size_t sid = blockIdx.x;
    int m = st.m[sid];
    double mu = st.mu[sid];
    const char *krow = UPD ? call.K + sid * call.stream_stride : nullptr;
    const char *vrow = UPD ? call.V + sid * call.stream_stride : nullptr;
    const char *qrows = ATT ? call.Q + sid * call.q_stride : nullptr;
    float *outrows = ATT ? out_rows(st, call.out, sid * call.out_stride) : nullptr;
    token_step<BF16, LPR, G, UPD, ATT>(st, sid, krow, vrow, qrows, outrows, tokens_seen(st, call.n_seen), m, mu, sm);
    if constexpr (UPD) {
        if (threadIdx.x == 0) {
            st.m[sid] = m;
            st.mu[sid] = mu;
        }
    }
}

// Prefix ingest: the same per-token update, tokens of a stream taken in order.
template <bool BF16, int LPR>
__global__ __launch_bounds__(kWG) void ingest_kernel(const State st, const Call call)
{
    constexpr int VEC = BF16 ? 8 : 4;
    __shared__ Smem<LPR, 1, VEC> sm;
    const size_t sid = blockIdx.x;
    int m = st.m[sid];
    double mu = st.mu[sid];
    const char *kbase = call.K + sid * call.stream_stride;
    const char *vbase = call.V + sid * call.stream_stride;
    const int64_t n0 = tokens_seen(st, call.n_seen);
    for (int64_t t = 0; t < call.n_tokens; ++t)
        token_step<BF16, LPR, 1, true, false>(st, sid, kbase + t * call.token_stride, vbase + t * call.token_stride,
                                              nullptr, nullptr, n0 + t, m, mu, sm);
    if (threadIdx.x == 0) {
        st.m[sid] = m;
        st.mu[sid] = mu;
    }
}


// ||x_i||^2 of one stream's representatives (double sum of the exactly converted elements, rounded to fp32):
// the derived array the bf16 fast paths read.  Used after a state import.
template <bool BF16, int LPR>
__global__ __launch_bounds__(kWG) void center_norms_kernel(const State st, const int64_t stream)
{
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)LPR * 16;
    const size_t sid = (size_t)stream;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane % LPR, sub = lane / LPR;
    const int m = st.m[sid];
    const char *X = st.X + sid * (size_t)st.Mcap * ROWB;
    for (int r0 = wave * RPW; r0 < m; r0 += RPB) {
        const int r = r0 + sub;
        float x[VEC];
        unpack<BF16>(ld16(X + (size_t)(r < m ? r : m - 1) * ROWB + col * 16), x);
        double a = 0.0;
#pragma unroll
        for (int v = 0; v < VEC; ++v) a = fma((double)x[v], (double)x[v], a);
        a = group_sum<LPR>(a);
        if (r < m && col == 0) st.xn[sid * (size_t)st.McapS + r] = (float)a;
    }
}

}  // namespace sg
