// One-shot greedy k-center compression of a prompt's KV cache (Section 3.2 of the paper: the greedy k-center
// algorithm of Dyer and Frieze is applied once; the r most recent tokens are kept, k centers are selected from
// the remaining ones).  Farthest-point traversal: the first center is the oldest token, every next center is
// the token farthest from the centers chosen so far (lowest index on ties); squared distances in double
// precision from the exactly converted elements.  One workgroup per stream; the running nearest-center
// distance and assignment of every old token live in a caller-supplied workspace, and a token is always
// handled by the same lanes, so the k passes need no synchronisation besides the argmax.
#pragma once
#include "subgen_device.hpp"

namespace sg {

struct KCenterCall {
    const char *K, *V;       // [S][n][d]
    char *outK, *outV;       // [S][k + r][d]: centers in selection order, then the r most recent tokens
    int32_t *out_idx;        // [S][k + r] token index of every output row (-1 = unused)
    int32_t *out_counts;     // [S][k] tokens (older than the window) nearest to each center, or null
    double *mind;            // [S][n_old] workspace
    int32_t *assign;         // [S][n_old] workspace
    int64_t n;
    int32_t k, r;
};

template <bool BF16, int LPR>
__global__ __launch_bounds__(kWG) void kcenter_kernel(const KCenterCall c)
{
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int RPW = 64 / LPR, RPB = RPW * kWaves;
    constexpr size_t ROWB = (size_t)LPR * 16;
    constexpr int U = kUnroll;
    __shared__ double wbest[kWaves];
    __shared__ int widx[kWaves];
    __shared__ int hist[1024];
    const size_t sid = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane % LPR, sub = lane / LPR, grp = wave * RPW + sub;
    const int64_t n = c.n;
    const int rwin = (int)(c.r < n ? c.r : n);
    const int nold = (int)(n - rwin);                 // tokens eligible as centers
    const int kk = c.k < nold ? c.k : nold;           // centers actually selected
    const int rows_out = c.k + c.r;
    const char *K = c.K + sid * (size_t)n * ROWB, *V = c.V + sid * (size_t)n * ROWB;
    char *oK = c.outK + sid * (size_t)rows_out * ROWB, *oV = c.outV + sid * (size_t)rows_out * ROWB;
    int32_t *oidx = c.out_idx + sid * (size_t)rows_out;
    double *mind = c.mind + sid * (size_t)(nold > 0 ? nold : 1);
    int32_t *assign = c.assign + sid * (size_t)(nold > 0 ? nold : 1);

    int center = 0;
    for (int it = 0; it < kk; ++it) {
        // emit center `it` and measure every old token against it
        float cf[VEC];
        {
            const uint4 ck = ld16(K + (size_t)center * ROWB + col * 16);
            unpack<BF16>(ck, cf);
            if (tid < LPR) {
                st16(oK + (size_t)it * ROWB + tid * 16, ld16(K + (size_t)center * ROWB + tid * 16));
                st16(oV + (size_t)it * ROWB + tid * 16, ld16(V + (size_t)center * ROWB + tid * 16));
            }
            if (tid == 0) oidx[it] = center;
        }
        double best = -1.0;
        int bidx = -1;
        for (int r0 = grp; r0 < nold; r0 += RPB * U) {
            uint4 raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPB;
                raw[u] = ld16(K + (size_t)(r < nold ? r : nold - 1) * ROWB + col * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + u * RPB;
                float x[VEC];
                unpack<BF16>(raw[u], x);
                double dist = 0.0;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double df = (double)x[v] - (double)cf[v];
                    dist = fma(df, df, dist);
                }
                dist = group_sum<LPR>(dist);
                if (r < nold) {
                    double md = dist;
                    if (it == 0) {
                        if (col == 0) {
                            mind[r] = dist;
                            assign[r] = 0;
                        }
                    } else {
                        const double old = mind[r];
                        if (dist < old) {                 // a tie keeps the earlier center
                            if (col == 0) {
                                mind[r] = dist;
                                assign[r] = it;
                            }
                        } else {
                            md = old;
                        }
                    }
                    if (md > best) {                      // rows come in increasing order: first maximum wins
                        best = md;
                        bidx = r;
                    }
                }
            }
        }
        // farthest token over the workgroup (lowest index on ties)
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) {
            const double ob = __shfl_xor(best, o);
            const int oi = __shfl_xor(bidx, o);
            if (ob > best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
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
            if (ob > best || (ob == best && (uint32_t)oi < (uint32_t)bidx)) {
                best = ob;
                bidx = oi;
            }
        }
        center = bidx;
        __syncthreads();
    }
    // unused center rows, then the window (the r most recent tokens, oldest first)
    for (int j = kk + grp; j < c.k; j += RPB) {
        st16(oK + (size_t)j * ROWB + col * 16, make_uint4(0, 0, 0, 0));
        st16(oV + (size_t)j * ROWB + col * 16, make_uint4(0, 0, 0, 0));
        if (col == 0) oidx[j] = -1;
    }
    for (int j = grp; j < c.r; j += RPB) {
        const bool have = j < rwin;
        const size_t src = (size_t)(nold + (have ? j : 0));
        st16(oK + (size_t)(c.k + j) * ROWB + col * 16, have ? ld16(K + src * ROWB + col * 16) : make_uint4(0, 0, 0, 0));
        st16(oV + (size_t)(c.k + j) * ROWB + col * 16, have ? ld16(V + src * ROWB + col * 16) : make_uint4(0, 0, 0, 0));
        if (col == 0) oidx[c.k + j] = have ? (int32_t)src : -1;
    }
    // cluster sizes: how many old tokens ended up nearest to each center
    if (c.out_counts != nullptr) {
        int32_t *oc = c.out_counts + sid * (size_t)c.k;
        for (int base = 0; base < c.k; base += 1024) {
            for (int j = tid; j < 1024; j += kWG) hist[j] = 0;
            __syncthreads();
            for (int r = tid; r < nold; r += kWG) {
                const int a = assign[r] - base;
                if (a >= 0 && a < 1024) atomicAdd(&hist[a], 1);
            }
            __syncthreads();
            for (int j = tid; j < 1024 && base + j < c.k; j += kWG) oc[base + j] = hist[j];
            __syncthreads();
        }
    }
}

}  // namespace sg
