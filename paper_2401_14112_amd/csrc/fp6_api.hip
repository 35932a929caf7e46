// C ABI of the library (see include/fp6.h): argument checks on the host, kernel
// selection, launches on the caller's stream.  No allocation, no synchronization.
#include "../../include/fp6.h"

#include <atomic>

#include "fp6_device.hpp"
#include "linear_stream.hpp"
#include "linear_tiled.hpp"
#include "pack_unpack.hpp"

namespace {

using namespace fp6;

constexpr int kLayoutVersion = 1;
#ifndef FP6_STREAM_WAVES
#define FP6_STREAM_WAVES 8
#endif
#ifndef FP6_STREAM_DEPTH
#define FP6_STREAM_DEPTH 2
#endif
#ifndef FP6_TARGET_WAVES_PER_CU
#define FP6_TARGET_WAVES_PER_CU 8
#endif
constexpr int kStreamWaves = FP6_STREAM_WAVES;  // waves per block of the streaming kernel
constexpr int kStreamDepth = FP6_STREAM_DEPTH;  // weight tiles in flight per wave
constexpr int kTargetWaves = 256 * FP6_TARGET_WAVES_PER_CU;  // 256 CUs x resident waves aimed for

std::atomic<int> g_forced_split{0};

bool shape_ok(int64_t M, int64_t K) { return M > 0 && K > 0 && M % kTileRows == 0 && K % kTileK == 0 && M < (1ll << 31) && K < (1ll << 31); }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct StreamPlan {
    int nt;          // 16-token tiles handled per launch (1 or 2)
    int split;       // split-K factor
    int row_blocks;  // blocks along M
    size_t counter_bytes;
    size_t partial_bytes;
    size_t total_bytes() const { return split > 1 ? counter_bytes + partial_bytes : 0; }
};

StreamPlan plan_stream(int64_t M, int64_t N, int64_t K)
{
    StreamPlan p;
    const int64_t row_tiles = M / kTileRows;
    const int64_t KT = K / kTileK;
    p.nt = N <= 16 ? 1 : 2;
    int64_t s = g_forced_split.load(std::memory_order_relaxed);
    if (s <= 0)
        s = (kTargetWaves + row_tiles - 1) / row_tiles;
    const int64_t max_split = KT >= 4 ? KT / 2 : 1;  // at least two k-tiles per slice
    if (s > max_split)
        s = max_split;
    if (s > 64)
        s = 64;
    if (s < 1)
        s = 1;
    p.split = (int)s;
    p.row_blocks = (int)((row_tiles + kStreamWaves - 1) / kStreamWaves);
    p.counter_bytes = (((size_t)p.row_blocks * sizeof(int)) + 255) / 256 * 256;
    p.partial_bytes = (size_t)p.split * (size_t)row_tiles * (size_t)p.nt * 64 * sizeof(float4_t);
    return p;
}

// ---- tiled kernel (prefill-sized N) -----------------------------------------
constexpr int kTiledWaves = 4;
constexpr int kStreamMaxN = 32;  // token counts up to this use the streaming kernel

std::atomic<int> g_forced_tile{0};  // 0 = automatic, else RT*16 + NT (tuning hook)

struct TiledPlan {
    int rt, nt;      // 16-row tiles and 16-token tiles per wave
    int split;
    int row_blocks, n_blocks;
    size_t counter_bytes, partial_bytes;
    size_t lds_bytes;
    size_t total_bytes() const { return split > 1 ? counter_bytes + partial_bytes : 0; }
};

TiledPlan plan_tiled(int64_t M, int64_t N, int64_t K, bool wide_tile_ok)
{
    TiledPlan p;
    const int64_t row_tiles = M / kTileRows;
    const int64_t KT = K / kTileK;
    const int forced = g_forced_tile.load(std::memory_order_relaxed);
    if (forced > 0) {
        p.rt = forced / 16;
        p.nt = forced % 16;
    } else if (N <= 64) {
        p.rt = 2;
        p.nt = 4;
    } else {
        p.rt = 4;
        p.nt = 8;
    }
    if (p.rt == 4 && p.nt == 8 && !wide_tile_ok)
        p.rt = 2;
    p.row_blocks = (int)((row_tiles + kTiledWaves * p.rt - 1) / (kTiledWaves * p.rt));
    p.n_blocks = (int)((N + 16 * p.nt - 1) / (16 * p.nt));
    int64_t s = g_forced_split.load(std::memory_order_relaxed);
    if (s <= 0)
        s = 256 / ((int64_t)p.row_blocks * p.n_blocks);  // one block per CU
    const int64_t max_split = KT >= 8 ? KT / 4 : 1;  // at least four k-tiles per slice
    if (s > max_split)
        s = max_split;
    if (s > 16)
        s = 16;
    if (s < 1)
        s = 1;
    p.split = (int)s;
    p.counter_bytes = (((size_t)p.row_blocks * p.n_blocks * sizeof(int)) + 255) / 256 * 256;
    p.partial_bytes = (size_t)p.split * (size_t)row_tiles * (size_t)p.n_blocks * p.nt * 64 * sizeof(float4_t);
    p.lds_bytes = (size_t)2 * p.nt * 512 * 16;
    return p;
}

template <class Src, int RT, int NT>
fp6_status launch_tiled_cfg(const TiledPlan &p, const void *weights, const void *scales, const void *X, void *Y,
                            int64_t M, int64_t N, int64_t K, float4_t *partials, int *counters, hipStream_t stream)
{
    auto kernel = linear_tiled_kernel<Src, RT, NT, kTiledWaves>;
    static bool lds_ok = false;  // per instantiation: allow more than 64 KB of dynamic LDS
    if (!lds_ok) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)p.lds_bytes) != hipSuccess)
            return FP6_ERR_HIP;
        lds_ok = true;
    }
    const dim3 grid((unsigned)(p.row_blocks * p.n_blocks * p.split)), block(kTiledWaves * 64);
    hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, stream, weights, static_cast<const half_t *>(scales),
                       static_cast<const half_t *>(X), static_cast<half_t *>(Y), (int)M, (int)N, (int)K, p.split,
                       p.n_blocks, partials, counters);
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

template <class Src>
fp6_status launch_tiled(const void *weights, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                        int64_t K, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    const TiledPlan p = plan_tiled(M, N, K, Src::kWideTile);
    if ((uint64_t)N * (uint64_t)K * 2u >= (1ull << 31))
        return FP6_ERR_SHAPE;  // activations are addressed with 32-bit buffer offsets
    if (p.total_bytes() > 0) {
        if (!workspace || workspace_bytes < p.total_bytes())
            return FP6_ERR_WORKSPACE;
        if (!aligned16(workspace))
            return FP6_ERR_ALIGN;
    }
    int *counters = static_cast<int *>(workspace);
    float4_t *partials =
        p.total_bytes() ? reinterpret_cast<float4_t *>(static_cast<uint8_t *>(workspace) + p.counter_bytes) : nullptr;
#define FP6_TILED_CASE(RT_, NT_)                                                                                  \
    if (p.rt == RT_ && p.nt == NT_)                                                                               \
        return launch_tiled_cfg<Src, RT_, NT_>(p, weights, scales, X, Y, M, N, K, partials, counters, stream);
    FP6_TILED_CASE(2, 4)
    FP6_TILED_CASE(4, 4)
    FP6_TILED_CASE(2, 8)
    if constexpr (!Src::kWideTile)
        return FP6_ERR_SHAPE;  // plan_tiled never picks 4 x 8 for a source whose tiles do not fit in registers
    else
        FP6_TILED_CASE(4, 8)
#undef FP6_TILED_CASE
    return FP6_ERR_SHAPE;
}

template <class Src>
fp6_status launch_stream(const void *weights, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                         int64_t K, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    const StreamPlan p = plan_stream(M, N, K);
    if (p.total_bytes() > 0) {
        if (!workspace || workspace_bytes < p.total_bytes())
            return FP6_ERR_WORKSPACE;
        if (!aligned16(workspace))
            return FP6_ERR_ALIGN;
    }
    int *counters = static_cast<int *>(workspace);
    float4_t *partials =
        p.total_bytes() ? reinterpret_cast<float4_t *>(static_cast<uint8_t *>(workspace) + p.counter_bytes) : nullptr;
    const dim3 grid((unsigned)(p.row_blocks * p.split)), block(kStreamWaves * 64);
    // tokens are processed 32 (or 16) at a time; each pass re-streams the weights
    const int64_t step = 16 * p.nt;
    for (int64_t n0 = 0; n0 < N; n0 += step) {
        const int64_t n = (N - n0 < step) ? (N - n0) : step;
        const half_t *Xp = static_cast<const half_t *>(X) + n0 * K;
        half_t *Yp = static_cast<half_t *>(Y) + n0 * M;
        if (p.nt == 1)
            hipLaunchKernelGGL((linear_stream_kernel<Src, 1, kStreamWaves, kStreamDepth>), grid, block, 0, stream,
                               weights, static_cast<const half_t *>(scales), Xp, Yp, (int)M, (int)n, (int)K, p.split,
                               partials, counters);
        else
            hipLaunchKernelGGL((linear_stream_kernel<Src, 2, kStreamWaves, kStreamDepth>), grid, block, 0, stream,
                               weights, static_cast<const half_t *>(scales), Xp, Yp, (int)M, (int)n, (int)K, p.split,
                               partials, counters);
        if (hipGetLastError() != hipSuccess)
            return FP6_ERR_HIP;
    }
    return FP6_OK;
}

}  // namespace

extern "C" {

const char *fp6_status_str(int status)
{
    switch (status) {
    case FP6_OK: return "FP6_OK";
    case FP6_ERR_NULL: return "FP6_ERR_NULL: a required pointer is NULL";
    case FP6_ERR_SHAPE: return "FP6_ERR_SHAPE: need M % 16 == 0, K % 256 == 0, M, N, K > 0";
    case FP6_ERR_WORKSPACE: return "FP6_ERR_WORKSPACE: workspace missing or too small";
    case FP6_ERR_ALIGN: return "FP6_ERR_ALIGN: pointers must be 16-byte aligned";
    case FP6_ERR_HIP: return "FP6_ERR_HIP: kernel launch failed";
    default: return "unknown fp6 status";
    }
}

int fp6_layout_version(void) { return kLayoutVersion; }

size_t fp6_packed_bytes(int64_t M, int64_t K) { return shape_ok(M, K) ? (size_t)(M * K / 4 * 3) : 0; }

size_t fp6_linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (!shape_ok(M, K) || N <= 0)
        return 0;
    return N <= kStreamMaxN ? plan_stream(M, N, K).total_bytes()
                            : plan_tiled(M, N, K, PackedFp6Source::kWideTile).total_bytes();
}

size_t fp16_linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (!shape_ok(M, K) || N <= 0)
        return 0;
    return N <= kStreamMaxN ? plan_stream(M, N, K).total_bytes()
                            : plan_tiled(M, N, K, PlainFp16Source::kWideTile).total_bytes();
}

void fp6_tuning_set_split_k(int split_k) { g_forced_split.store(split_k < 0 ? 0 : split_k); }

void fp6_tuning_set_tile(int row_tiles_per_wave, int token_tiles_per_wave)
{
    const int rt = row_tiles_per_wave, nt = token_tiles_per_wave;
    const bool known = (rt == 2 || rt == 4) && (nt == 4 || nt == 8);
    g_forced_tile.store(known ? rt * 16 + nt : 0);
}

fp6_status fp6_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (workspace_bytes == 0)
        return FP6_OK;
    if (!workspace)
        return FP6_ERR_NULL;
    if (!aligned16(workspace) || workspace_bytes % 16)
        return FP6_ERR_ALIGN;
    const size_t n16 = workspace_bytes / 16;
    hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<u32x4 *>(workspace), n16);
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

fp6_status fp6_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16, void *stream)
{
    if (!W_f16 || !packed || !scales_f16)
        return FP6_ERR_NULL;
    if (!shape_ok(M, K))
        return FP6_ERR_SHAPE;
    if (!aligned16(W_f16) || !aligned16(packed) || !aligned16(scales_f16))
        return FP6_ERR_ALIGN;
    hipLaunchKernelGGL(quantize_pack_kernel, dim3((unsigned)(M / kTileRows)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const half_t *>(W_f16), (int)M, (int)K,
                       static_cast<uint8_t *>(packed), static_cast<half_t *>(scales_f16));
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

fp6_status fp6_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out, void *stream)
{
    if (!packed || !scales_f16 || !W_f16_out)
        return FP6_ERR_NULL;
    if (!shape_ok(M, K))
        return FP6_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(scales_f16) || !aligned16(W_f16_out))
        return FP6_ERR_ALIGN;
    const int64_t tiles = (M / kTileRows) * (K / kTileK);
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint8_t *>(packed),
                       static_cast<const half_t *>(scales_f16), (int)M, (int)K, static_cast<half_t *>(W_f16_out));
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

fp6_status fp6_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N,
                      int64_t K, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!packed || !scales_f16 || !X_f16 || !Y_f16)
        return FP6_ERR_NULL;
    if (!shape_ok(M, K) || N <= 0 || N >= (1ll << 31))
        return FP6_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(scales_f16) || !aligned16(X_f16) || !aligned16(Y_f16))
        return FP6_ERR_ALIGN;
    if (N > kStreamMaxN)
        return launch_tiled<PackedFp6Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                             static_cast<hipStream_t>(stream));
    return launch_stream<PackedFp6Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                          static_cast<hipStream_t>(stream));
}

fp6_status fp16_linear(const void *W_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N, int64_t K,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    if (!W_f16 || !X_f16 || !Y_f16)
        return FP6_ERR_NULL;
    if (!shape_ok(M, K) || N <= 0 || N >= (1ll << 31))
        return FP6_ERR_SHAPE;
    if (!aligned16(W_f16) || !aligned16(X_f16) || !aligned16(Y_f16))
        return FP6_ERR_ALIGN;
    if (N > kStreamMaxN)
        return launch_tiled<PlainFp16Source>(W_f16, nullptr, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                             static_cast<hipStream_t>(stream));
    return launch_stream<PlainFp16Source>(W_f16, nullptr, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                          static_cast<hipStream_t>(stream));
}

}  // extern "C"
