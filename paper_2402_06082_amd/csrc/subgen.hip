// Host side of the SubGen C ABI (see include/subgen.h): argument checks, state
// allocation in HBM, kernel dispatch.  No arithmetic of the method runs here.
#include "../../include/subgen.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "exact_device.hpp"
#include "subgen_device.hpp"
#include "subgen_mfma_device.hpp"
#include "subgen_tile_device.hpp"
#include "ingest_mfma_device.hpp"
#include "subgen_dot2_device.hpp"
#include "subgen_res_device.hpp"
#include "kcenter_device.hpp"
#include "attend_many_device.hpp"
#include "subgen_split_device.hpp"

using sg::Call;
using sg::State;

struct subgen_ctx {
    State st{};
    int64_t S = 0;
    int32_t d = 0, s = 0, w = 0, Mcap = 0, G = 1;
    int32_t dtype = SUBGEN_F32;
    int32_t esz = 4;       // element bytes
    int32_t LPR = 0;       // lanes per row = row bytes / 16
    float delta = 0.f;
    int64_t n_seen = 0;
    hipStream_t stream = nullptr;
    int device = 0;
    int last_hip = 0;
    bool mfma = false;     // bf16 rows scored on the matrix cores
    bool ingest_mfma = false;   // bf16 rows of 64 / 128 elements: chunked prefix ingest (also with reservoirs)
    bool wide = false;          // few streams: 8 wavefronts per workgroup and hoisted loads on the row path
    bool dev_seen = false;      // the token count lives on the device (launches can be captured and replayed)
    bool imported = false; // a stream state has been imported (pins n_seen)
    std::vector<void *> allocs;
};

namespace {

struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) switched = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard()
    {
        if (switched) (void)hipSetDevice(prev);
    }
};

int fail_hip(subgen_ctx *c, hipError_t e)
{
    if (c) c->last_hip = (int)e;
    return e == hipErrorOutOfMemory ? SUBGEN_ENOMEM : SUBGEN_EHIP;
}

template <typename T>
int dev_alloc(subgen_ctx *c, T **p, size_t count, int fill_byte)
{
    void *q = nullptr;
    const size_t bytes = (count ? count : 1) * sizeof(T);
    hipError_t e = hipMalloc(&q, bytes);
    if (e != hipSuccess) return fail_hip(c, e);
    try {
        c->allocs.push_back(q);
    } catch (const std::bad_alloc &) {   // nothing may throw across the C ABI
        (void)hipFree(q);
        return SUBGEN_ENOMEM;
    }
    e = hipMemsetAsync(q, fill_byte, bytes, c->stream);
    if (e != hipSuccess) return fail_hip(c, e);
    *p = reinterpret_cast<T *>(q);
    return SUBGEN_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

enum Mode { MODE_UPDATE, MODE_ATTEND, MODE_STEP };

template <bool BF16, int LPR, int G>
void launch_mode(Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    switch (mode) {
        case MODE_UPDATE:
            hipLaunchKernelGGL((sg::decode_kernel<BF16, LPR, 1, true, false>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_ATTEND:
            hipLaunchKernelGGL((sg::decode_kernel<BF16, LPR, G, false, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_STEP:
            hipLaunchKernelGGL((sg::decode_kernel<BF16, LPR, G, true, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
    }
}

template <bool BF16, int LPR>
void launch_g(int G, Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    if (G == 1) launch_mode<BF16, LPR, 1>(mode, grid, s, st, call);
    else if (G == 2) launch_mode<BF16, LPR, 2>(mode, grid, s, st, call);
    else launch_mode<BF16, LPR, 4>(mode, grid, s, st, call);
}

template <bool BF16>
void launch_lpr(int LPR, int G, Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    if (LPR == 8) launch_g<BF16, 8>(G, mode, grid, s, st, call);
    else if (LPR == 16) launch_g<BF16, 16>(G, mode, grid, s, st, call);
    else launch_g<BF16, 32>(G, mode, grid, s, st, call);
}

template <int NK, int G>
void launch_mfma_mode(Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    switch (mode) {
        case MODE_UPDATE:
            hipLaunchKernelGGL((sg::decode_mfma_kernel<NK, 1, true, false>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_ATTEND:
            hipLaunchKernelGGL((sg::decode_mfma_kernel<NK, G, false, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_STEP:
            hipLaunchKernelGGL((sg::decode_mfma_kernel<NK, G, true, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
    }
}

// matrix-core path: bf16 rows of 64, 128 or 256 elements, as long as the fp32 accumulators fit in registers
bool mfma_supported(int dtype, int LPR, int G) { return dtype == SUBGEN_BF16 && (LPR / 4) * G <= 16; }

// rows of 64 or 128 elements: the update alone scans the representatives straight from HBM; attend and step
// stage the rows through LDS tiles and run the value products on the matrix cores as well
// wavefronts per workgroup of the LDS-tiled kernels: the fused step runs four workgroups of two wavefronts per CU
// (its serial update phases overlap with three other streams instead of one), attend alone two of four
#ifndef SG_TILE_WAVES_ATT
#define SG_TILE_WAVES_ATT 4
#endif
#ifndef SG_TILE_WAVES_UPD
#define SG_TILE_WAVES_UPD 2
#endif
template <int NK, int G>
void launch_tile_mode(Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    switch (mode) {
        case MODE_UPDATE:
            hipLaunchKernelGGL((sg::decode_mfma_kernel<NK, 1, true, false>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_ATTEND:
            hipLaunchKernelGGL((sg::decode_tile_kernel<NK, G, false, SG_TILE_WAVES_ATT>), grid, dim3(64 * SG_TILE_WAVES_ATT), 0, s, st, call);
            break;
        case MODE_STEP:
            hipLaunchKernelGGL((sg::decode_tile_kernel<NK, G, true, SG_TILE_WAVES_UPD>), grid, dim3(64 * SG_TILE_WAVES_UPD), 0, s, st, call);
            break;
    }
}

void launch_mfma(int NK, int G, Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    if (NK == 2) {
        if (G == 1) launch_tile_mode<2, 1>(mode, grid, s, st, call);
        else if (G == 2) launch_tile_mode<2, 2>(mode, grid, s, st, call);
        else launch_tile_mode<2, 4>(mode, grid, s, st, call);
    } else if (NK == 4) {
        if (G == 1) launch_tile_mode<4, 1>(mode, grid, s, st, call);
        else if (G == 2) launch_tile_mode<4, 2>(mode, grid, s, st, call);
        else launch_tile_mode<4, 4>(mode, grid, s, st, call);
    } else {
        if (G == 1) launch_mfma_mode<8, 1>(mode, grid, s, st, call);
        else launch_mfma_mode<8, 2>(mode, grid, s, st, call);
    }
}

template <bool BF16, int LPR, int G>
void launch_res_mode(Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    switch (mode) {
        case MODE_UPDATE:
            hipLaunchKernelGGL((sg::decode_res_kernel<BF16, LPR, 1, true, false>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_ATTEND:
            hipLaunchKernelGGL((sg::decode_res_kernel<BF16, LPR, G, false, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_STEP:
            hipLaunchKernelGGL((sg::decode_res_kernel<BF16, LPR, G, true, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
    }
}

template <bool BF16, int LPR>
void launch_res_g(int G, Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    if (G == 1) launch_res_mode<BF16, LPR, 1>(mode, grid, s, st, call);
    else if (G == 2) launch_res_mode<BF16, LPR, 2>(mode, grid, s, st, call);
    else launch_res_mode<BF16, LPR, 4>(mode, grid, s, st, call);
}

// contexts with per-cluster reservoirs (t >= 1); MODE_UPDATE with n_tokens > 1 is the prefix ingest
void launch_res(subgen_ctx *c, Mode mode, const Call &call, int G)
{
    const dim3 grid((unsigned)c->S);
    if (c->dtype == SUBGEN_BF16) {
        if (c->LPR == 8) launch_res_g<true, 8>(G, mode, grid, c->stream, c->st, call);
        else if (c->LPR == 16) launch_res_g<true, 16>(G, mode, grid, c->stream, c->st, call);
        else launch_res_g<true, 32>(G, mode, grid, c->stream, c->st, call);
    } else {
        if (c->LPR == 8) launch_res_g<false, 8>(G, mode, grid, c->stream, c->st, call);
        else if (c->LPR == 16) launch_res_g<false, 16>(G, mode, grid, c->stream, c->st, call);
        else launch_res_g<false, 32>(G, mode, grid, c->stream, c->st, call);
    }
}

template <int NW>
void launch_dot2(Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    const dim3 wg(NW * 64);
    switch (mode) {
        case MODE_UPDATE:
            hipLaunchKernelGGL((sg::decode_dot2_kernel<true, false, NW>), grid, wg, 0, s, st, call);
            break;
        case MODE_ATTEND:
            hipLaunchKernelGGL((sg::decode_dot2_kernel<false, true, NW>), grid, wg, 0, s, st, call);
            break;
        case MODE_STEP:
            hipLaunchKernelGGL((sg::decode_dot2_kernel<true, true, NW>), grid, wg, 0, s, st, call);
            break;
    }
}

template <bool BF16, int LPR, int G>
void launch_split_mode(Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    switch (mode) {
        case MODE_UPDATE:
            hipLaunchKernelGGL((sg::decode_split_kernel<BF16, LPR, 1, true, false>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_ATTEND:
            hipLaunchKernelGGL((sg::decode_split_kernel<BF16, LPR, G, false, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
        case MODE_STEP:
            hipLaunchKernelGGL((sg::decode_split_kernel<BF16, LPR, G, true, true>), grid, dim3(sg::kWG), 0, s, st, call);
            break;
    }
}

template <bool BF16, int LPR>
void launch_split_g(int G, Mode mode, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    if (G == 1) launch_split_mode<BF16, LPR, 1>(mode, grid, s, st, call);
    else if (G == 2) launch_split_mode<BF16, LPR, 2>(mode, grid, s, st, call);
    else launch_split_mode<BF16, LPR, 4>(mode, grid, s, st, call);
}

// contexts of a few streams: split_P workgroups per stream
void launch_split(subgen_ctx *c, Mode mode, const Call &call, int G)
{
    const dim3 grid((unsigned)(c->S * c->st.split_P));
    if (c->dtype == SUBGEN_BF16) {
        if (c->LPR == 8) launch_split_g<true, 8>(G, mode, grid, c->stream, c->st, call);
        else if (c->LPR == 16) launch_split_g<true, 16>(G, mode, grid, c->stream, c->st, call);
        else launch_split_g<true, 32>(G, mode, grid, c->stream, c->st, call);
    } else {
        if (c->LPR == 8) launch_split_g<false, 8>(G, mode, grid, c->stream, c->st, call);
        else if (c->LPR == 16) launch_split_g<false, 16>(G, mode, grid, c->stream, c->st, call);
        else launch_split_g<false, 32>(G, mode, grid, c->stream, c->st, call);
    }
}

// G = queries per stream of this launch (the context's own, or a group of a many-query call)
int launch_decode(subgen_ctx *c, Mode mode, const Call &call, int G)
{
    const dim3 grid((unsigned)c->S);
    if (c->st.split_P > 1) {
        launch_split(c, mode, call, G);
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
    }
    const bool mfma = c->mfma && mfma_supported(c->dtype, c->LPR, G);
    if (c->st.t > 0) {
        launch_res(c, mode, call, G);
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
    }
    // bf16 rows of 128 elements, one query per stream: whole-row loads (one contiguous 1 KB access per wavefront
    // load, which the memory system serves faster than the 64-byte pieces of the matrix-core operand layout)
    // with packed-bf16 dot products.  With several queries per stream the vector ALUs would be the bound, so
    // those go to the matrix cores.
    // (a query alone, with streams enough to fill the chip, is 3 % faster on the LDS-tiled kernel below: it has no
    // update whose serial part would need the row path's higher occupancy to hide)
    // (the update alone looks up one key, however many queries the context has: it takes the row path as well)
    if (mfma && c->LPR == 16 && (mode == MODE_UPDATE || (G == 1 && (mode != MODE_ATTEND || c->wide)))) {
        if (c->wide) launch_dot2<8>(mode, grid, c->stream, c->st, call);   // few streams: wide workgroups, hoisted loads
        else launch_dot2<4>(mode, grid, c->stream, c->st, call);
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
    }
    if (mfma) {
        launch_mfma(c->LPR / 4, G, mode, grid, c->stream, c->st, call);
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
    }
    if (c->dtype == SUBGEN_BF16) launch_lpr<true>(c->LPR, G, mode, grid, c->stream, c->st, call);
    else launch_lpr<false>(c->LPR, G, mode, grid, c->stream, c->st, call);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
}

template <bool BF16>
void launch_ingest_lpr(int LPR, dim3 grid, hipStream_t s, const State &st, const Call &call)
{
    if (LPR == 8) hipLaunchKernelGGL((sg::ingest_kernel<BF16, 8>), grid, dim3(sg::kWG), 0, s, st, call);
    else if (LPR == 16) hipLaunchKernelGGL((sg::ingest_kernel<BF16, 16>), grid, dim3(sg::kWG), 0, s, st, call);
    else hipLaunchKernelGGL((sg::ingest_kernel<BF16, 32>), grid, dim3(sg::kWG), 0, s, st, call);
}

bool row_bytes_ok(int64_t rb) { return rb == 128 || rb == 256 || rb == 512; }

// scratch of the entry point that allocates nothing (split partials of the exact attention); every device that
// loads the library holds its own copy of this array until the process ends
#ifndef SG_NOALLOC_BYTES
#define SG_NOALLOC_BYTES ((size_t)32 << 20)
#endif
constexpr size_t kNoAllocScratchBytes = SG_NOALLOC_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char g_noalloc_scratch[kNoAllocScratchBytes];
std::atomic<void *> g_noalloc_ptr[kMaxDevices];     // device address of the array, per device ordinal

int exact_splits(int64_t streams, int64_t n)
{
    int64_t want = (4096 + streams - 1) / streams;          // aim for >= 4096 workgroups
    int64_t most = (n + 255) / 256;                          // at least 256 rows per split
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 1024) want = 1024;
    return (int)want;
}

template <bool BF16, int LPR, int G>
void launch_exact(const sg::ExactCall &c, int64_t streams, hipStream_t s)
{
    constexpr int D = LPR * (BF16 ? 8 : 4);
    hipLaunchKernelGGL((sg::exact_partial_kernel<BF16, LPR, G>), dim3((unsigned)streams, c.splits), dim3(sg::kWG), 0,
                       s, c);
    hipLaunchKernelGGL((sg::exact_combine_kernel<D, G>), dim3((unsigned)streams), dim3(sg::kWG), 0, s, c);
}

template <bool BF16, int LPR>
void launch_exact_g(int g, const sg::ExactCall &c, int64_t streams, hipStream_t s)
{
    if (g == 1) launch_exact<BF16, LPR, 1>(c, streams, s);
    else if (g == 2) launch_exact<BF16, LPR, 2>(c, streams, s);
    else launch_exact<BF16, LPR, 4>(c, streams, s);
}

// contexts that keep the token count on the device: advance it behind the kernels of an update
int bump_seen(subgen_ctx *c, int64_t n)
{
    if (!c->dev_seen) return SUBGEN_OK;
    hipLaunchKernelGGL(sg::bump_seen_kernel, dim3(1), dim3(1), 0, c->stream, c->st.seen, n);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
}

// ... and bring the host's copy up to date (after replays of a captured graph the host has not counted)
int refresh_seen(subgen_ctx *c)
{
    if (!c->dev_seen) return SUBGEN_OK;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess) e = hipMemcpy(&c->n_seen, c->st.seen, sizeof(int64_t), hipMemcpyDeviceToHost);
    return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
}

}  // namespace

extern "C" {

int subgen_create(subgen_ctx **out, int64_t streams, int32_t d, float delta, int32_t sample_budget,
                  int32_t window, const subgen_opts *opts)
{
    if (!out) return SUBGEN_EINVAL;
    *out = nullptr;
    subgen_opts o;
    std::memset(&o, 0, sizeof(o));
    if (opts) {
        if (opts->struct_size < sizeof(uint32_t) || opts->struct_size > sizeof(subgen_opts)) return SUBGEN_EINVAL;
        std::memcpy(&o, opts, opts->struct_size);
    }
    const int32_t G = o.q_per_stream == 0 ? 1 : o.q_per_stream;
    const int32_t Mcap = o.max_centers == 0 ? 4096 : o.max_centers;
    if (o.dtype != SUBGEN_F32 && o.dtype != SUBGEN_BF16) return SUBGEN_EINVAL;
    const int32_t esz = o.dtype == SUBGEN_BF16 ? 2 : 4;
    if (streams < 1 || streams > 0x7fffffffLL || d < 1 || !row_bytes_ok((int64_t)d * esz)) return SUBGEN_EINVAL;
    if (!(delta >= 0.f) || !std::isfinite(delta)) return SUBGEN_EINVAL;
    if (sample_budget < 1 || sample_budget > (1 << 20) || window < 0 || window > (1 << 20)) return SUBGEN_EINVAL;
    if (G != 1 && G != 2 && G != 4) return SUBGEN_EINVAL;
    if (Mcap < 1 || Mcap > (1 << 24) || o.assign_log_tokens < 0) return SUBGEN_EINVAL;
    if (o.kernel_path < 0 || o.kernel_path > 2) return SUBGEN_EINVAL;
    if (o.t_per_cluster < 0 || o.t_per_cluster > 64) return SUBGEN_EINVAL;
    if (o.device_counter != 0 && o.device_counter != 1) return SUBGEN_EINVAL;
    if (o.out_dtype != SUBGEN_F32 && o.out_dtype != SUBGEN_BF16) return SUBGEN_EINVAL;
    if (o.split_workgroups < 0 || o.split_workgroups > 64) return SUBGEN_EINVAL;

    subgen_ctx *c = new (std::nothrow) subgen_ctx();
    if (!c) return SUBGEN_ENOMEM;
    hipError_t e;
    if (o.device_set) {
        c->device = o.device;
    } else if ((e = hipGetDevice(&c->device)) != hipSuccess) {
        delete c;
        return SUBGEN_EHIP;
    }
    DeviceGuard guard(c->device);
    c->S = streams; c->d = d; c->s = sample_budget; c->w = window; c->Mcap = Mcap; c->G = G;
    c->dtype = o.dtype; c->esz = esz; c->LPR = d * esz / 16; c->delta = delta;
    c->stream = reinterpret_cast<hipStream_t>(o.hip_stream);
    c->mfma = o.kernel_path != 1 && o.t_per_cluster == 0 && mfma_supported(o.dtype, c->LPR, G);
    c->ingest_mfma = o.kernel_path != 1 && o.dtype == SUBGEN_BF16 && (c->LPR == 8 || c->LPR == 16);
    c->wide = o.kernel_path == 0 && streams <= 256;   // measured crossover between 256 and 512 streams
    c->dev_seen = o.device_counter != 0;
    // a few streams (far fewer than the chip has compute units): several workgroups per stream.  Automatic
    // choice: up to 32 streams, the power of two that brings the launch to at most 256 workgroups, at most 32 per
    // stream (measured: 1 stream 38 -> 15 us with 32, 32 streams 17.1 -> 14.8 us with 8; at 4 per stream the
    // combine costs what the shorter scan saves, so larger contexts keep one workgroup per stream)
    int32_t split = o.split_workgroups;
    if (split == 0) {
        split = 1;
        if (o.kernel_path == 0 && o.t_per_cluster == 0 && streams <= 32)
            for (split = 32; split > 8 && split * streams > 256; split /= 2) {}
    }
    if (o.t_per_cluster > 0) split = 1;   // per-cluster reservoirs keep one workgroup per stream

    State &st = c->st;
    st.Mcap = Mcap; st.s = sample_budget; st.w = window; st.d = d;
    st.t = o.t_per_cluster;
    st.out_bf16 = o.out_dtype == SUBGEN_BF16 ? 1 : 0;
    st.split_P = split > 1 ? split : 0;
    st.McapS = (Mcap + 15) / 16 * 16; st.sS = (sample_budget + 15) / 16 * 16;
    st.delta2 = (double)delta * (double)delta;
    st.seed_lo = (uint32_t)o.seed; st.seed_hi = (uint32_t)(o.seed >> 32);
    st.assign_cap = o.assign_log_tokens;
    const size_t S = (size_t)streams, rowb = (size_t)d * esz;
    int rc = SUBGEN_OK;
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.X, S * Mcap * rowb, 0);
    if (rc == SUBGEN_OK && st.t > 0) rc = dev_alloc(c, &st.R, S * Mcap * st.t * rowb, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.cnt, S * st.McapS, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.xn, S * st.McapS, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.m, S, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.Ks, S * sample_budget * rowb, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.Vs, S * sample_budget * rowb, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.sidx, S * st.sS, 0xFF);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.svn, S * st.sS, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.Kw, S * window * rowb, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.Vw, S * window * rowb, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.mu, S, 0);
    if (rc == SUBGEN_OK) rc = dev_alloc(c, &st.flags, S, 0);
    if (rc == SUBGEN_OK && o.device_counter) rc = dev_alloc(c, &st.seen, 1, 0);
    if (rc == SUBGEN_OK && st.split_P > 1) rc = dev_alloc(c, &st.split_cnt, S, 0);
    if (rc == SUBGEN_OK && st.split_P > 1)
        rc = dev_alloc(c, &st.split_part, S * st.split_P * (size_t)sg::split_partial_floats(4, d), 0);
    if (rc == SUBGEN_OK && st.assign_cap > 0) rc = dev_alloc(c, &st.assign, S * (size_t)st.assign_cap, 0xFF);
    if (rc != SUBGEN_OK) {
        subgen_destroy(c);
        return rc;
    }
    *out = c;
    return SUBGEN_OK;
}

void subgen_destroy(subgen_ctx *c)
{
    if (!c) return;
    DeviceGuard guard(c->device);
    (void)hipStreamSynchronize(c->stream);
    for (void *p : c->allocs) (void)hipFree(p);
    delete c;
}

int subgen_update(subgen_ctx *c, const void *K_t, const void *V_t)
{
    if (!c || !K_t || !V_t || !aligned16(K_t) || !aligned16(V_t)) return SUBGEN_EINVAL;
    DeviceGuard guard(c->device);
    Call call{};
    call.K = (const char *)K_t; call.V = (const char *)V_t;
    call.stream_stride = (int64_t)c->d * c->esz; call.token_stride = call.stream_stride;
    call.n_tokens = 1; call.n_seen = c->n_seen;
    int rc = launch_decode(c, MODE_UPDATE, call, c->G);
    if (rc == SUBGEN_OK) rc = bump_seen(c, 1);
    if (rc == SUBGEN_OK) c->n_seen += 1;
    return rc;
}

int subgen_attend(subgen_ctx *c, const void *Q_t, void *out)
{
    if (!c || !Q_t || !out || !aligned16(Q_t) || !aligned16(out)) return SUBGEN_EINVAL;
    if (c->n_seen == 0) return SUBGEN_EEMPTY;
    DeviceGuard guard(c->device);
    Call call{};
    call.Q = (const char *)Q_t; call.out = (float *)out; call.n_seen = c->n_seen;
    call.q_stride = (int64_t)c->G * c->d * c->esz; call.out_stride = (int64_t)c->G * c->d;
    return launch_decode(c, MODE_ATTEND, call, c->G);
}

int subgen_attend_many(subgen_ctx *c, const void *Q, int32_t n_queries, void *out)
{
    if (!c || !Q || !out || !aligned16(Q) || !aligned16(out) || n_queries < 1 || n_queries > (1 << 20))
        return SUBGEN_EINVAL;
    if (c->n_seen == 0) return SUBGEN_EEMPTY;
    DeviceGuard guard(c->device);
    const int NK = c->LPR / 4;
    if (c->mfma && (NK == 2 || NK == 4)) {
        // bf16 rows of 64 or 128 elements, representative mode: both contractions on the matrix cores
        // up to 64 queries: one tile of 16 per wavefront (1, 2 or 4 query groups x row splits); more: two tiles
        // per wavefront, 128 queries per workgroup (measured: two tiles per wavefront with two row splits at 64
        // queries is slower, 0.95 against 0.89 ms on the n=16k state)
        const int QT = n_queries <= 16 ? 1 : (n_queries <= 32 ? 2 : 4);
        const int QW = n_queries <= 64 ? 1 : 2;
        sg::ManyCall mc{};
        mc.Q = (const char *)Q; mc.out = (float *)out; mc.Gm = n_queries;
        mc.tiles = (n_queries + 16 * QT * QW - 1) / (16 * QT * QW);
        mc.n_seen = c->n_seen; mc.streams = c->S;
        const int64_t blocks = (c->S + 7) / 8 * 8 * (int64_t)mc.tiles;
        if (blocks > 0x7fffffffLL) return SUBGEN_ECAPACITY;
        const dim3 grid((unsigned)blocks), wg(sg::kWG);
        // 128-element rows and more than 32 queries: the kernel that brings the rows into LDS without registers; it
        // keeps the weights of a stream's representatives and sampled pairs in LDS, which bounds their number
        const int64_t wrows = ((int64_t)c->st.Mcap + 63) / 64 * 64 + ((int64_t)c->st.s + 31) / 32 * 32;
        if (NK == 4 && QT == 4 && wrows <= sg::kDmaRows) {
            constexpr int NB = sg::kDmaBufs, WC = sg::kDmaRows;
            if (QW == 1) hipLaunchKernelGGL((sg::attend_many_dma_kernel<true, 1, NB, WC, 2>), grid, wg, 0, c->stream, c->st, mc);
            else if (mc.tiles == 1) hipLaunchKernelGGL((sg::attend_many_dma_kernel<true, 2, NB, WC, 2>), grid, wg, 0, c->stream, c->st, mc);
            else hipLaunchKernelGGL((sg::attend_many_dma_kernel<false, 2, NB, WC, 2>), grid, wg, 0, c->stream, c->st, mc);
        } else if (NK == 2) {
            if (QT == 1) hipLaunchKernelGGL((sg::attend_many_kernel<2, 1, true>), grid, wg, 0, c->stream, c->st, mc);
            else if (QT == 2) hipLaunchKernelGGL((sg::attend_many_kernel<2, 2, true>), grid, wg, 0, c->stream, c->st, mc);
            else if (QW == 1) hipLaunchKernelGGL((sg::attend_many_kernel<2, 4, true>), grid, wg, 0, c->stream, c->st, mc);
            else if (mc.tiles == 1) hipLaunchKernelGGL((sg::attend_many_kernel<2, 4, true, 2>), grid, wg, 0, c->stream, c->st, mc);
            else hipLaunchKernelGGL((sg::attend_many_kernel<2, 4, false, 2>), grid, wg, 0, c->stream, c->st, mc);
        } else {
            if (QT == 1) hipLaunchKernelGGL((sg::attend_many_kernel<4, 1, true>), grid, wg, 0, c->stream, c->st, mc);
            else if (QT == 2) hipLaunchKernelGGL((sg::attend_many_kernel<4, 2, true>), grid, wg, 0, c->stream, c->st, mc);
            else if (QW == 1) hipLaunchKernelGGL((sg::attend_many_kernel<4, 4, true>), grid, wg, 0, c->stream, c->st, mc);
            else if (mc.tiles == 1) hipLaunchKernelGGL((sg::attend_many_kernel<4, 4, true, 2>), grid, wg, 0, c->stream, c->st, mc);
            else hipLaunchKernelGGL((sg::attend_many_kernel<4, 4, false, 2>), grid, wg, 0, c->stream, c->st, mc);
        }
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SUBGEN_OK : fail_hip(c, e);
    }
    // every other context (fp32 rows, 256-element rows, reservoirs, the generic kernel path): the decode
    // kernels, four, two or one query at a time
    const int64_t rowb = (int64_t)c->d * c->esz;
    for (int32_t q0 = 0; q0 < n_queries;) {
        const int g = n_queries - q0 >= 4 ? 4 : (n_queries - q0 >= 2 ? 2 : 1);
        Call call{};
        call.Q = (const char *)Q + q0 * rowb; call.out = (float *)((char *)out + (int64_t)q0 * c->d * (c->st.out_bf16 ? 2 : 4)); call.n_seen = c->n_seen;
        call.q_stride = n_queries * rowb; call.out_stride = (int64_t)n_queries * c->d;
        const int rc = launch_decode(c, MODE_ATTEND, call, g);
        if (rc != SUBGEN_OK) return rc;
        q0 += g;
    }
    return SUBGEN_OK;
}

int subgen_step(subgen_ctx *c, const void *K_t, const void *V_t, const void *Q_t, void *out)
{
    if (!c || !K_t || !V_t || !Q_t || !out) return SUBGEN_EINVAL;
    if (!aligned16(K_t) || !aligned16(V_t) || !aligned16(Q_t) || !aligned16(out)) return SUBGEN_EINVAL;
    DeviceGuard guard(c->device);
    Call call{};
    call.K = (const char *)K_t; call.V = (const char *)V_t;
    call.stream_stride = (int64_t)c->d * c->esz; call.token_stride = call.stream_stride;
    call.n_tokens = 1; call.Q = (const char *)Q_t; call.out = (float *)out; call.n_seen = c->n_seen;
    call.q_stride = (int64_t)c->G * c->d * c->esz; call.out_stride = (int64_t)c->G * c->d;
    int rc = launch_decode(c, MODE_STEP, call, c->G);
    if (rc == SUBGEN_OK) rc = bump_seen(c, 1);
    if (rc == SUBGEN_OK) c->n_seen += 1;
    return rc;
}

#ifndef SG_INGEST_T
#define SG_INGEST_T 128   // tokens per chunk of the matrix-core ingest (64 with per-cluster reservoirs)
#endif

int subgen_ingest_prefix(subgen_ctx *c, const void *K, const void *V, int64_t n, int64_t stream_stride,
                         int64_t token_stride)
{
    if (!c || n < 0) return SUBGEN_EINVAL;
    if (n == 0) return SUBGEN_OK;
    if (!K || !V || !aligned16(K) || !aligned16(V)) return SUBGEN_EINVAL;
    if (token_stride < c->d || stream_stride < 0) return SUBGEN_EINVAL;
    if ((token_stride * c->esz) % 16 != 0 || (stream_stride * c->esz) % 16 != 0) return SUBGEN_EINVAL;
    if (c->S > 1 && stream_stride < c->d) return SUBGEN_EINVAL;
    DeviceGuard guard(c->device);
    // bounded launches: a kernel walks at most kChunk tokens of every stream
    constexpr int64_t kChunk = 2048;
    for (int64_t t0 = 0; t0 < n; t0 += kChunk) {
        Call call{};
        call.stream_stride = stream_stride * c->esz; call.token_stride = token_stride * c->esz;
        call.K = (const char *)K + t0 * call.token_stride; call.V = (const char *)V + t0 * call.token_stride;
        call.n_tokens = (n - t0 < kChunk) ? n - t0 : kChunk;
        call.n_seen = c->n_seen;
        const dim3 grid((unsigned)c->S);
        if (c->st.t > 0 && c->ingest_mfma && c->LPR == 8)
            hipLaunchKernelGGL((sg::ingest_mfma_kernel<2, 64, true>), grid, dim3(sg::kWG), 0, c->stream, c->st, call);
        else if (c->st.t > 0 && c->ingest_mfma && c->LPR == 16)
            hipLaunchKernelGGL((sg::ingest_mfma_kernel<4, 64, true>), grid, dim3(sg::kWG), 0, c->stream, c->st, call);
        else if (c->st.t > 0)
            launch_res(c, MODE_UPDATE, call, c->G);
        else if (c->mfma && c->LPR == 8)
            hipLaunchKernelGGL((sg::ingest_mfma_kernel<2, SG_INGEST_T, false>), grid, dim3(sg::kWG), 0, c->stream, c->st, call);
        else if (c->mfma && c->LPR == 16)
            hipLaunchKernelGGL((sg::ingest_mfma_kernel<4, SG_INGEST_T, false>), grid, dim3(sg::kWG), 0, c->stream, c->st, call);
        else if (c->dtype == SUBGEN_BF16) launch_ingest_lpr<true>(c->LPR, grid, c->stream, c->st, call);
        else launch_ingest_lpr<false>(c->LPR, grid, c->stream, c->st, call);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail_hip(c, e);
        const int rb = bump_seen(c, call.n_tokens);
        if (rb != SUBGEN_OK) return rb;
        c->n_seen += call.n_tokens;
    }
    return SUBGEN_OK;
}

/* ------------------------------------------------------------------ exact attention */

size_t subgen_exact_workspace_bytes(int64_t streams, int64_t n, int32_t d, int32_t g)
{
    if (streams < 1 || n < 1 || d < 1 || g < 1) return 0;
    return (size_t)streams * exact_splits(streams, n) * g * (d + 2) * sizeof(float);
}

static int exact_attend_impl(const void *K, const void *V, const void *Q, void *out, int64_t streams, int64_t n,
                             int32_t d, int32_t g, int32_t dtype, void *workspace, size_t workspace_bytes,
                             void *hip_stream)
{
    if (!K || !V || !Q || !out || !workspace) return SUBGEN_EINVAL;
    if (!aligned16(K) || !aligned16(V) || !aligned16(Q) || !aligned16(out) || !aligned16(workspace))
        return SUBGEN_EINVAL;
    if (dtype != SUBGEN_F32 && dtype != SUBGEN_BF16) return SUBGEN_EINVAL;
    const int esz = dtype == SUBGEN_BF16 ? 2 : 4;
    // one workgroup column per stream on grid.x (up to 2^31 - 1), the sequence splits on grid.y (at most 1024)
    if (streams < 1 || streams > 0x7fffffffLL || n < 1 || d < 1 || !row_bytes_ok((int64_t)d * esz))
        return SUBGEN_EINVAL;
    if (g != 1 && g != 2 && g != 4) return SUBGEN_EINVAL;
    if (workspace_bytes < subgen_exact_workspace_bytes(streams, n, d, g)) return SUBGEN_ECAPACITY;
    sg::ExactCall c{};
    c.K = (const char *)K; c.V = (const char *)V; c.Q = (const char *)Q; c.out = (float *)out;
    c.ws = (float *)workspace; c.n = n; c.splits = exact_splits(streams, n);
    hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
    const int LPR = d * esz / 16;
    if (dtype == SUBGEN_BF16) {
        if (LPR == 8) launch_exact_g<true, 8>(g, c, streams, s);
        else if (LPR == 16) launch_exact_g<true, 16>(g, c, streams, s);
        else launch_exact_g<true, 32>(g, c, streams, s);
    } else {
        if (LPR == 8) launch_exact_g<false, 8>(g, c, streams, s);
        else if (LPR == 16) launch_exact_g<false, 16>(g, c, streams, s);
        else launch_exact_g<false, 32>(g, c, streams, s);
    }
    return hipGetLastError() == hipSuccess ? SUBGEN_OK : SUBGEN_EHIP;
}

int subgen_exact_attend(const void *K, const void *V, const void *Q, void *out, int64_t streams, int64_t n,
                        int32_t d, int32_t g, int32_t dtype, void *workspace, size_t workspace_bytes,
                        void *hip_stream)
{
    return exact_attend_impl(K, V, Q, out, streams, n, d, g, dtype, workspace, workspace_bytes, hip_stream);
}

/* The same kernels with the split partials in a buffer that is part of the library's code object: no allocation
 * anywhere on the call path.  The array's name is only a host-side handle; its device address is looked up once
 * per device (with that device current) and that address is what the kernels are given. */
size_t subgen_exact_noalloc_max_bytes(void) { return kNoAllocScratchBytes; }

int subgen_exact_attend_noalloc(const void *K, const void *V, const void *Q, void *out, int64_t streams, int64_t n,
                                int32_t d, int32_t g, int32_t dtype, void *hip_stream)
{
    const size_t need = subgen_exact_workspace_bytes(streams, n, d, g);
    if (need == 0) return SUBGEN_EINVAL;
    if (need > kNoAllocScratchBytes) return SUBGEN_ECAPACITY;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SUBGEN_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return SUBGEN_EINVAL;
    void *ptr = g_noalloc_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_noalloc_scratch)) != hipSuccess || !ptr) return SUBGEN_EHIP;
        g_noalloc_ptr[dev].store(ptr, std::memory_order_release);     // every thread would find the same address
    }
    return exact_attend_impl(K, V, Q, out, streams, n, d, g, dtype, ptr, kNoAllocScratchBytes, hip_stream);
}

size_t subgen_kcenter_workspace_bytes(int64_t streams, int64_t n, int32_t r)
{
    if (streams < 1 || n < 1 || r < 0) return 0;
    const int64_t nold = n > r ? n - r : 1;
    return (size_t)streams * (size_t)nold * (sizeof(double) + sizeof(int32_t) + sizeof(float)) + 256;
}

int subgen_kcenter_compress(const void *K, const void *V, int64_t streams, int64_t n, int32_t d, int32_t dtype, int32_t k,
                            int32_t r, void *out_K, void *out_V, int32_t *out_idx, int32_t *out_counts,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!K || !V || !out_K || !out_V || !out_idx || !workspace) return SUBGEN_EINVAL;
    if (!aligned16(K) || !aligned16(V) || !aligned16(out_K) || !aligned16(out_V) || !aligned16(workspace))
        return SUBGEN_EINVAL;
    if (dtype != SUBGEN_F32 && dtype != SUBGEN_BF16) return SUBGEN_EINVAL;
    const int esz = dtype == SUBGEN_BF16 ? 2 : 4;
    if (streams < 1 || streams > 0x7fffffffLL || n < 1 || n > 0x7fffffffLL || d < 1 || !row_bytes_ok((int64_t)d * esz))
        return SUBGEN_EINVAL;
    if (k < 1 || r < 0 || k > (1 << 24) || r > (1 << 24)) return SUBGEN_EINVAL;
    if (workspace_bytes < subgen_kcenter_workspace_bytes(streams, n, r)) return SUBGEN_ECAPACITY;
    const int64_t nold = n > r ? n - r : 1;
    sg::KCenterCall c{};
    c.K = (const char *)K; c.V = (const char *)V; c.outK = (char *)out_K; c.outV = (char *)out_V;
    c.out_idx = out_idx; c.out_counts = out_counts; c.n = n; c.k = k; c.r = r;
    c.mind = (double *)workspace;
    c.assign = (int32_t *)((char *)workspace + (size_t)streams * (size_t)nold * sizeof(double));
    c.xnorm = (float *)((char *)c.assign + (size_t)streams * (size_t)nold * sizeof(int32_t));
    hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)streams), block(sg::kWG);
    const int LPR = d * esz / 16;
    if (dtype == SUBGEN_BF16) {   // several centers per pass over the keys, approximate distances as a filter
        if (LPR == 8) hipLaunchKernelGGL((sg::kcenter_batched_kernel<8>), grid, block, 0, s, c);
        else if (LPR == 16) hipLaunchKernelGGL((sg::kcenter_batched_kernel<16>), grid, block, 0, s, c);
        else hipLaunchKernelGGL((sg::kcenter_batched_kernel<32>), grid, block, 0, s, c);
    } else {
        if (LPR == 8) hipLaunchKernelGGL((sg::kcenter_kernel<false, 8>), grid, block, 0, s, c);
        else if (LPR == 16) hipLaunchKernelGGL((sg::kcenter_kernel<false, 16>), grid, block, 0, s, c);
        else hipLaunchKernelGGL((sg::kcenter_kernel<false, 32>), grid, block, 0, s, c);
    }
    return hipGetLastError() == hipSuccess ? SUBGEN_OK : SUBGEN_EHIP;
}

int subgen_hbm_read_probe(const void *buf, size_t bytes, int32_t workgroups, int32_t nontemporal,
                          size_t region_bytes, void *sink, void *hip_stream)
{
    if (!buf || !sink || !aligned16(buf) || bytes < 16 || workgroups < 1 || workgroups > (1 << 20)) return SUBGEN_EINVAL;
    hipLaunchKernelGGL(sg::hbm_read_probe_kernel, dim3((unsigned)workgroups), dim3(sg::kWG), 0,
                       reinterpret_cast<hipStream_t>(hip_stream), (const uint4 *)buf, bytes / 16, (uint32_t *)sink,
                       nontemporal != 0, region_bytes / 16);
    return hipGetLastError() == hipSuccess ? SUBGEN_OK : SUBGEN_EHIP;
}

/* ------------------------------------------------------------------ introspection */

int subgen_sync(subgen_ctx *c)
{
    if (!c) return SUBGEN_EINVAL;
    DeviceGuard guard(c->device);
    const hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail_hip(c, e);
    return refresh_seen(c);
}

static int64_t evicted(const subgen_ctx *c)
{
    if (c->w == 0) return c->n_seen;
    return c->n_seen > c->w ? c->n_seen - c->w : 0;
}

int subgen_center_counts(subgen_ctx *c, int32_t *host_m)
{
    if (!c || !host_m) return SUBGEN_EINVAL;
    DeviceGuard guard(c->device);
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess) e = hipMemcpy(host_m, c->st.m, (size_t)c->S * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(c, e);
    return refresh_seen(c);
}

int subgen_stats(subgen_ctx *c, subgen_stats_t *o)
{
    if (!c || !o) return SUBGEN_EINVAL;
    std::vector<int32_t> m;
    std::vector<uint32_t> fl;
    try {
        m.resize((size_t)c->S);
        fl.resize((size_t)c->S);
    } catch (const std::bad_alloc &) {   // nothing may throw across the C ABI
        return SUBGEN_ENOMEM;
    }
    int rc = subgen_center_counts(c, m.data());
    if (rc != SUBGEN_OK) return rc;
    DeviceGuard guard(c->device);
    const hipError_t e = hipMemcpy(fl.data(), c->st.flags, (size_t)c->S * sizeof(uint32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(c, e);
    std::memset(o, 0, sizeof(*o));
    o->struct_size = sizeof(*o);
    o->streams = c->S; o->n_seen = c->n_seen; o->n_evicted = evicted(c);
    o->min_centers = m[0]; o->max_centers = m[0];
    for (int64_t i = 0; i < c->S; ++i) {
        o->total_centers += m[i];
        if (m[i] < o->min_centers) o->min_centers = m[i];
        if (m[i] > o->max_centers) o->max_centers = m[i];
        o->flags_or |= fl[i];
        if (fl[i]) o->flagged_streams += 1;
    }
    return SUBGEN_OK;
}

int subgen_export_state(subgen_ctx *c, int64_t stream, subgen_state_view *v)
{
    if (!c || !v || stream < 0 || stream >= c->S) return SUBGEN_EINVAL;
    if (v->struct_size != sizeof(subgen_state_view)) return SUBGEN_EINVAL;
    DeviceGuard guard(c->device);
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail_hip(c, e);
    if (const int rs = refresh_seen(c); rs != SUBGEN_OK) return rs;
    const State &st = c->st;
    const size_t sid = (size_t)stream, rowb = (size_t)c->d * c->esz;
#define SG_D2H(dst, src, bytes)                                                       \
    do {                                                                              \
        if ((dst) != nullptr && (bytes) > 0) {                                        \
            e = hipMemcpy((dst), (src), (bytes), hipMemcpyDeviceToHost);              \
            if (e != hipSuccess) return fail_hip(c, e);                               \
        }                                                                             \
    } while (0)
    int32_t m = 0;
    SG_D2H(&m, st.m + sid, sizeof(int32_t));
    SG_D2H(&v->mu, st.mu + sid, sizeof(double));
    SG_D2H(&v->flags, st.flags + sid, sizeof(uint32_t));
    v->m = m;
    v->n_seen = c->n_seen;
    v->n_evicted = evicted(c);
    v->window_fill = (int32_t)(c->n_seen < c->w ? c->n_seen : c->w);
    if ((v->centers || v->counts) && v->centers_cap < m) return SUBGEN_EINVAL;
    SG_D2H(v->centers, st.X + sid * c->Mcap * rowb, (size_t)m * rowb);
    SG_D2H(v->counts, st.cnt + sid * st.McapS, (size_t)m * sizeof(int32_t));
    if (v->reservoirs != nullptr) {
        if (st.t == 0 || v->centers_cap < m) return SUBGEN_EINVAL;
        SG_D2H(v->reservoirs, st.R + sid * c->Mcap * st.t * rowb, (size_t)m * st.t * rowb);
    }
    SG_D2H(v->sample_K, st.Ks + sid * c->s * rowb, (size_t)c->s * rowb);
    SG_D2H(v->sample_V, st.Vs + sid * c->s * rowb, (size_t)c->s * rowb);
    SG_D2H(v->sample_idx, st.sidx + sid * st.sS, (size_t)c->s * sizeof(int32_t));
    SG_D2H(v->sample_vn, st.svn + sid * st.sS, (size_t)c->s * sizeof(float));
    SG_D2H(v->window_K, st.Kw + sid * c->w * rowb, (size_t)c->w * rowb);
    SG_D2H(v->window_V, st.Vw + sid * c->w * rowb, (size_t)c->w * rowb);
    v->assign_len = 0;
    if (v->assign != nullptr) {
        if (st.assign == nullptr) return SUBGEN_EINVAL;
        int64_t len = v->n_evicted < st.assign_cap ? v->n_evicted : st.assign_cap;
        if (len > v->assign_cap) len = v->assign_cap;
        SG_D2H(v->assign, st.assign + sid * (size_t)st.assign_cap, (size_t)len * sizeof(int32_t));
        v->assign_len = len;
    }
#undef SG_D2H
    return SUBGEN_OK;
}

int subgen_import_state(subgen_ctx *c, int64_t stream, const subgen_state_view *v)
{
    if (!c || !v || stream < 0 || stream >= c->S) return SUBGEN_EINVAL;
    if (v->struct_size != sizeof(subgen_state_view)) return SUBGEN_EINVAL;
    if (v->m < 0 || v->m > c->Mcap || v->n_seen < 0 || !std::isfinite(v->mu) || v->mu < 0.0) return SUBGEN_EINVAL;
    if (v->m > 0 && (!v->centers || !v->counts)) return SUBGEN_EINVAL;
    if (v->m > 0 && c->st.t > 0 && !v->reservoirs) return SUBGEN_EINVAL;
    if (!v->sample_K || !v->sample_V || !v->sample_idx || !v->sample_vn) return SUBGEN_EINVAL;
    if (c->w > 0 && (!v->window_K || !v->window_V)) return SUBGEN_EINVAL;
    // all streams of a context share one token counter: the first import into an untouched context sets it
    if (const int rs = refresh_seen(c); rs != SUBGEN_OK) return rs;
    if (c->n_seen != v->n_seen && (c->n_seen != 0 || c->imported)) return SUBGEN_EINVAL;
    DeviceGuard guard(c->device);
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail_hip(c, e);
    const State &st = c->st;
    const size_t sid = (size_t)stream, rowb = (size_t)c->d * c->esz;
#define SG_H2D(dst, src, bytes)                                                       \
    do {                                                                              \
        if ((bytes) > 0) {                                                            \
            e = hipMemcpy((dst), (src), (bytes), hipMemcpyHostToDevice);              \
            if (e != hipSuccess) return fail_hip(c, e);                               \
        }                                                                             \
    } while (0)
    const int32_t m = v->m;
    SG_H2D(st.m + sid, &m, sizeof(int32_t));
    SG_H2D(st.mu + sid, &v->mu, sizeof(double));
    SG_H2D(st.flags + sid, &v->flags, sizeof(uint32_t));
    SG_H2D(st.X + sid * c->Mcap * rowb, v->centers, (size_t)m * rowb);
    SG_H2D(st.cnt + sid * st.McapS, v->counts, (size_t)m * sizeof(int32_t));
    if (st.t > 0) SG_H2D(st.R + sid * c->Mcap * st.t * rowb, v->reservoirs, (size_t)m * st.t * rowb);
    SG_H2D(st.Ks + sid * c->s * rowb, v->sample_K, (size_t)c->s * rowb);
    SG_H2D(st.Vs + sid * c->s * rowb, v->sample_V, (size_t)c->s * rowb);
    SG_H2D(st.sidx + sid * st.sS, v->sample_idx, (size_t)c->s * sizeof(int32_t));
    SG_H2D(st.svn + sid * st.sS, v->sample_vn, (size_t)c->s * sizeof(float));
    SG_H2D(st.Kw + sid * c->w * rowb, v->window_K, (size_t)c->w * rowb);
    SG_H2D(st.Vw + sid * c->w * rowb, v->window_V, (size_t)c->w * rowb);
#undef SG_H2D
    // derived per-center norms
    const dim3 grid(1), block(sg::kWG);
    if (c->dtype == SUBGEN_BF16) {
        if (c->LPR == 8) hipLaunchKernelGGL((sg::center_norms_kernel<true, 8>), grid, block, 0, c->stream, st, stream);
        else if (c->LPR == 16) hipLaunchKernelGGL((sg::center_norms_kernel<true, 16>), grid, block, 0, c->stream, st, stream);
        else hipLaunchKernelGGL((sg::center_norms_kernel<true, 32>), grid, block, 0, c->stream, st, stream);
    } else {
        if (c->LPR == 8) hipLaunchKernelGGL((sg::center_norms_kernel<false, 8>), grid, block, 0, c->stream, st, stream);
        else if (c->LPR == 16) hipLaunchKernelGGL((sg::center_norms_kernel<false, 16>), grid, block, 0, c->stream, st, stream);
        else hipLaunchKernelGGL((sg::center_norms_kernel<false, 32>), grid, block, 0, c->stream, st, stream);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(c, e);
    c->n_seen = v->n_seen;
    c->imported = true;
    if (c->dev_seen) {
        e = hipMemcpy(c->st.seen, &c->n_seen, sizeof(int64_t), hipMemcpyHostToDevice);
        if (e != hipSuccess) return fail_hip(c, e);
    }
    return SUBGEN_OK;
}

const char *subgen_strerror(int code)
{
    switch (code) {
        case SUBGEN_OK: return "ok";
        case SUBGEN_EINVAL: return "invalid argument";
        case SUBGEN_ENOMEM: return "out of memory";
        case SUBGEN_EHIP: return "HIP runtime error";
        case SUBGEN_EEMPTY: return "attend before any token";
        case SUBGEN_ECAPACITY: return "capacity exceeded";
        default: return "unknown error";
    }
}

int subgen_last_hip_error(const subgen_ctx *c) { return c ? c->last_hip : 0; }

}  // extern "C"

