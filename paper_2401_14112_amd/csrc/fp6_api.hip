// C ABI of the library (see include/fp6.h): argument checks on the host, kernel
// selection, launches on the caller's stream.  No allocation, no synchronization.
#include "../../include/fp6.h"
#include "../../include/fp6_bench.h"

#include <atomic>

#include "fp6_device.hpp"
#include "linear_stream.hpp"
#include "linear_tiled.hpp"
#include "pack_unpack.hpp"

namespace {

using namespace fp6;

constexpr int kLayoutVersion = 4;  // 4: 3-bit tiles of 512 columns (6-, 5-, 4-bit streams as in 3)
// Configurations of the streaming kernel: {token tiles per wave, waves per block, weight tiles in flight per
// wave, k-tiles per activation stage, iterations over which the activation copies of a stage are spread,
// k-tiles dealt round-robin to the split-K slices}.
// For N <= 16 there are two block heights; the plan takes the one that fills the chip best for the shape.
struct StreamCfg {
    int nt, waves, depth, stage, spread;
    bool deal;
};
constexpr int kStreamCfgs = 4;
constexpr StreamCfg kStreamCfg[kStreamCfgs] = {{1, 4, 4, 4, 1, true}, {1, 8, 2, 1, 1, true}, {2, 8, 2, 1, 1, true},
                                               {4, 8, 2, 1, 1, true}};
// fp16 weights (staged through LDS, 8 KB per tile in flight): depths and block heights that fit the LDS of a
// CU beside the activation stages.  Measured on 8192x22016: all shapes of a token count within 2 us of each
// other, dealt slices 1-2 us ahead of contiguous ones.
constexpr StreamCfg kStreamCfgFp16[kStreamCfgs] = {{1, 4, 4, 1, 1, true}, {1, 8, 2, 2, 1, true}, {2, 8, 2, 1, 1, true},
                                                   {4, 4, 2, 1, 1, true}};
template <bool PACKED, int C>
struct StreamShapeOf {
    static constexpr StreamCfg c = PACKED ? kStreamCfg[C] : kStreamCfgFp16[C];
    typedef StreamShape<c.nt, c.waves, c.depth, c.stage, c.spread, c.deal> type;
};
constexpr int kStreamMaxN = 64;  // token counts up to this use the streaming kernel
constexpr int kCus = 256;

std::atomic<int> g_forced_split{0};

// The kernels address the activations of up to 64 tokens, and the 16 rows of an fp16 weight tile, with 32-bit
// byte offsets: 64 * K * 2 must stay below 2^31.
constexpr int64_t kMaxK = 1ll << 24;
bool shape_ok(int64_t M, int64_t K) { return M > 0 && K > 0 && M % kTileRows == 0 && K % kTileK == 0 && M < (1ll << 31) && K < kMaxK; }
// Packed weights: tiles are stored k-tile major and a wave addresses the tiles of its row tile with 32-bit
// offsets that step by one k-tile's worth of all row tiles; the pipelines request up to 64 tiles past the end
// of a slice (out of range: they read as zeros), and those offsets must not wrap either.  Priced at the 6-bit
// tile size for every width.
bool packed_shape_ok(int64_t M, int64_t K)
{
    return shape_ok(M, K) && (K / kTileK + 64) * (M / kTileRows) <= ((1ll << 31) - 1) / kTileBytes;
}
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Where a launch keeps its split-K state: arrival counters (zero before and after every launch) and the
// partial tiles.  A caller's workspace holds the counters first and the partial tiles right behind them, so
// the split depends on the plan; the library's own static buffer (fp6_linear_static) keeps the counters in a
// fixed region at its start, so that the partial tiles of one call can never be read as counters by the next.
constexpr size_t kStaticCounterBytes = 64 * 1024;

struct SplitBuffers {
    int *counters;
    uint8_t *partials;
};

struct WorkspaceRef {
    void *base;
    size_t bytes;
    bool fixed_regions;  // the library's static buffer
    // the buffers of a launch whose plan needs counter_bytes + partial_bytes; FP6_OK when they fit
    fp6_status view(size_t counter_bytes, size_t partial_bytes, SplitBuffers &out) const
    {
        out.counters = nullptr;
        out.partials = nullptr;
        if (partial_bytes == 0)
            return FP6_OK;  // no split-K: nothing is touched
        const size_t head = fixed_regions ? kStaticCounterBytes : counter_bytes;
        if (!base || counter_bytes > head || bytes < head || bytes - head < partial_bytes)
            return FP6_ERR_WORKSPACE;
        if (!aligned16(base))
            return FP6_ERR_ALIGN;
        out.counters = static_cast<int *>(base);
        out.partials = static_cast<uint8_t *>(base) + head;
        return FP6_OK;
    }
};

struct StreamPlan {
    int cfg;         // index into kStreamCfg / kStreamCfgFp16
    int nt;          // 16-token tiles handled per launch
    int split;       // split-K factor
    int row_blocks;  // blocks along M
    size_t counter_bytes;
    size_t partial_bytes;
    size_t total_bytes() const { return split > 1 ? counter_bytes + partial_bytes : 0; }
};

// The layer is bound by memory, every block streams the same number of bytes, and one block per CU is
// resident: the launch should be ONE round of at most 256 blocks, as many as possible.  Measured on the
// 70B-class shapes at N = 16: 240 blocks of 8 waves beat 320 or 480 blocks of 4 waves by 15-20 %, and 172
// blocks in one round beat 344 blocks in two.  So: for every available block height, the largest split-K
// factor that keeps row blocks x S <= 256 (at least two k-tiles per slice); take the candidate with the
// most blocks, on a tie the one with the taller blocks (more rows share each copy of the activations; with
// the k-tiles dealt to the slices a larger S no longer costs a sweeping front of its own).
StreamPlan plan_stream(int64_t M, int64_t N, int64_t K, bool packed, int tile_cols = kTileK)
{
    const StreamCfg *table = packed ? kStreamCfg : kStreamCfgFp16;
    const int64_t row_tiles = M / kTileRows;
    const int64_t KT = (K + tile_cols - 1) / tile_cols;  // steps of the streaming kernel for this source
    const int first = N <= 16 ? 0 : (N <= 32 ? 2 : 3);
    const int last = N <= 16 ? 1 : first;
    const int64_t forced = g_forced_split.load(std::memory_order_relaxed);
    const int64_t max_split = KT >= 4 ? KT / 2 : 1;  // at least two k-tiles per slice
    int best = first;
    int64_t best_s = 1, best_blocks = -1;
    bool best_single = false;
    for (int c = first; c <= last; ++c) {
        const int64_t rb = (row_tiles + table[c].waves - 1) / table[c].waves;
        int64_t s = forced > 0 ? forced : kCus / rb;
        if (s > max_split)
            s = max_split;
        if (s > 64)
            s = 64;
        if (s < 1)
            s = 1;
        // the kernel addresses the partial tiles with 32-bit byte offsets
        while (s > 1 && (uint64_t)s * (uint64_t)row_tiles * (uint64_t)table[c].nt * 1024u >= (1ull << 31))
            s /= 2;
        // ... and, with the k-tiles dealt to the slices, the weights with 32-bit offsets that step by s k-tiles
        // and run up to 20 steps past the end of a slice (look-ahead of the pipeline; those read as zeros)
        while (s > 1 && table[c].deal && (uint64_t)(KT + 20 * s) * (uint64_t)row_tiles * kTileBytes >= (1ull << 31))
            s /= 2;
        const int64_t blocks = rb * s;
        const bool single = blocks <= kCus;
        bool better;
        if (best_blocks < 0)
            better = true;
        else if (single != best_single)
            better = single;
        else if (single)
            better = blocks > best_blocks || (blocks == best_blocks && (table[c].deal ? s > best_s : s < best_s));
        else
            better = blocks < best_blocks;  // several rounds either way: the fewer, taller blocks
        if (better) {
            best = c;
            best_s = s;
            best_blocks = blocks;
            best_single = single;
        }
        if (forced > 0)
            break;  // the tuning hook pins the first candidate, so that tests reach every split factor
    }
    StreamPlan p;
    p.cfg = best;
    p.nt = table[best].nt;
    p.split = (int)best_s;
    p.row_blocks = (int)((row_tiles + table[best].waves - 1) / table[best].waves);
    p.counter_bytes = (((size_t)row_tiles * sizeof(int)) + 255) / 256 * 256;  // one arrival counter per row tile
    p.partial_bytes = (size_t)p.split * (size_t)row_tiles * (size_t)p.nt * 64 * sizeof(float4_t);
    return p;
}

// ---- tiled kernel (prefill-sized N) -----------------------------------------

// Block shapes offered by the tiled kernel: {RT, NT, WM, WN}; block = (16*RT*WM) rows x (16*NT*WN) tokens.
struct TileShape {
    int rt, nt, wm, wn;
    int rows() const { return 16 * rt * wm; }
    int tokens() const { return 16 * nt * wn; }
};
constexpr TileShape kTile256x128{2, 8, 8, 1};
constexpr TileShape kTile128x128{2, 4, 4, 2};
constexpr TileShape kTile256x64{2, 4, 8, 1};
constexpr TileShape kTile128x64{2, 4, 4, 1};

// A kernel that uses more than 64 KB of dynamic LDS has to be told so once per device.  `done` holds one
// bit per device ordinal (mod 64); safe to call from several host threads.
bool allow_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done)
{
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess)
        return false;
    const uint64_t bit = 1ull << (device & 63);
    if (done.load(std::memory_order_acquire) & bit)
        return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return false;
    done.fetch_or(bit, std::memory_order_release);
    return true;
}

std::atomic<int> g_forced_tile{0};  // 0 = automatic, else rows * 1024 + tokens (tuning hook)

struct TiledPlan {
    TileShape tile;
    int split;
    int row_blocks, n_blocks;
    size_t counter_bytes, partial_bytes;
    size_t lds_bytes;
    size_t total_bytes() const { return split > 1 ? counter_bytes + partial_bytes : 0; }
};

TiledPlan plan_tiled(int64_t M, int64_t N, int64_t K, bool tall_tile_ok)
{
    TiledPlan p;
    const int64_t row_tiles = M / kTileRows;
    const int64_t KT = K / kTileK;
    const int forced = g_forced_tile.load(std::memory_order_relaxed);
    const int rows = forced / 1024, tokens = forced % 1024;
    if (forced > 0)
        p.tile = rows == 256 ? (tokens == 128 ? kTile256x128 : kTile256x64) : (tokens == 128 ? kTile128x128 : kTile128x64);
    else if (N <= 128 && (M + 255) / 256 < 64)
        p.tile = kTile128x64;  // few row blocks: small blocks and little split-K (measured on 8192-row layers)
    else
        p.tile = kTile256x128;  // the shape that moves the fewest bytes per MFMA
    if (p.tile.rows() == 256 && p.tile.tokens() == 128 && !tall_tile_ok)  // this weight source does not fit 2 x 8 tiles per wave in registers
        p.tile = kTile128x128;
    p.row_blocks = (int)((M + p.tile.rows() - 1) / p.tile.rows());
    p.n_blocks = (int)((N + p.tile.tokens() - 1) / p.tile.tokens());
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
    const int bnt = p.tile.nt * p.tile.wn;
    p.counter_bytes = (((size_t)p.row_blocks * p.n_blocks * sizeof(int)) + 255) / 256 * 256;
    p.partial_bytes = (size_t)p.split * (size_t)row_tiles * (size_t)p.n_blocks * bnt * 64 * sizeof(float4_t);
    p.lds_bytes = (size_t)4 * bnt * 256 * 16;  // the kernel's ring of four half tiles of activations
    return p;
}

template <class Src, int RT, int NT, int WM, int WN>
fp6_status launch_tiled_cfg(const TiledPlan &p, const void *weights, const void *scales, const void *X, void *Y,
                            int64_t M, int64_t N, int64_t K, float4_t *partials, int *counters, const Epilogue &epi,
                            hipStream_t stream)
{
    auto kernel = linear_tiled_kernel<Src, RT, NT, WM, WN>;
    static std::atomic<uint64_t> lds_done{0};  // per instantiation
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(kernel), p.lds_bytes, lds_done))
        return FP6_ERR_HIP;
    // row blocks are dealt to the 8 XCDs round-robin: the grid is padded to a multiple of 8 row blocks
    const int padded_row_blocks = (p.row_blocks + 7) / 8 * 8;
    const dim3 grid((unsigned)(padded_row_blocks * p.n_blocks * p.split)), block(WM * WN * 64);
    hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, stream, weights, static_cast<const half_t *>(scales),
                       static_cast<const half_t *>(X), static_cast<half_t *>(Y), (int)M, (int)N, (int)K, p.split,
                       p.n_blocks, partials, counters, epi);
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

// The tiled kernel addresses the activations with 32-bit byte offsets, so one launch takes at most this many
// tokens (a multiple of the widest block); longer inputs are processed in chunks on the same stream.
int64_t tiled_chunk_tokens(int64_t K)
{
    const int64_t fit = ((1ll << 31) - 1) / (2 * K);
    return fit >= 128 ? fit / 128 * 128 : fit;  // shape_ok() admits K < 2^24 only: at least 64 tokens fit
}

// Workspace of the tiled path: the largest over the chunks a call is cut into (the last, shorter chunk may
// use more k slices than the full ones).
size_t tiled_workspace_bytes(int64_t M, int64_t N, int64_t K, bool tall_tile_ok)
{
    const int64_t chunk = tiled_chunk_tokens(K);
    if (chunk <= 0)
        return 0;
    if (N <= chunk)
        return plan_tiled(M, N, K, tall_tile_ok).total_bytes();
    size_t bytes = plan_tiled(M, chunk, K, tall_tile_ok).total_bytes();
    const int64_t last = N % chunk;
    if (last > 0) {
        const size_t b = plan_tiled(M, last, K, tall_tile_ok).total_bytes();
        bytes = b > bytes ? b : bytes;
    }
    return bytes;
}

template <class Src>
fp6_status launch_tiled_chunk(const void *weights, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                              int64_t K, const WorkspaceRef &workspace, const Epilogue &epi, hipStream_t stream)
{
    const TiledPlan p = plan_tiled(M, N, K, Src::kTallTile);
    SplitBuffers buf;
    const fp6_status fits = workspace.view(p.counter_bytes, p.split > 1 ? p.partial_bytes : 0, buf);
    if (fits != FP6_OK)
        return fits;
    int *counters = buf.counters;
    float4_t *partials = reinterpret_cast<float4_t *>(buf.partials);
    const TileShape &t = p.tile;
#define FP6_TILED_CASE(RT_, NT_, WM_, WN_)                                                                        \
    if (t.rt == RT_ && t.nt == NT_ && t.wm == WM_ && t.wn == WN_)                                                 \
        return launch_tiled_cfg<Src, RT_, NT_, WM_, WN_>(p, weights, scales, X, Y, M, N, K, partials, counters, epi, \
                                                         stream);
    FP6_TILED_CASE(2, 4, 4, 2)
    FP6_TILED_CASE(2, 4, 4, 1)
    FP6_TILED_CASE(2, 4, 8, 1)
    if constexpr (Src::kTallTile) {
        FP6_TILED_CASE(2, 8, 8, 1)
    }
#undef FP6_TILED_CASE
    return FP6_ERR_SHAPE;  // not reached: plan_tiled only picks the shapes above
}

template <class Src>
fp6_status launch_tiled(const void *weights, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                        int64_t K, const WorkspaceRef &workspace, const Epilogue &epi, hipStream_t stream)
{
    const int64_t chunk = tiled_chunk_tokens(K);
    if (chunk <= 0)
        return FP6_ERR_SHAPE;  // one token's activations exceed a 32-bit byte offset
    // every chunk's plan must fit before anything is launched (a full chunk and the shorter last one)
    for (int64_t n : {N < chunk ? N : chunk, N > chunk ? N % chunk : (int64_t)0}) {
        if (n <= 0)
            continue;
        const TiledPlan p = plan_tiled(M, n, K, Src::kTallTile);
        SplitBuffers unused;
        const fp6_status fits = workspace.view(p.counter_bytes, p.split > 1 ? p.partial_bytes : 0, unused);
        if (fits != FP6_OK)
            return fits;
    }
    const int64_t Mout = epi.gated ? M / 2 : M;
    for (int64_t n0 = 0; n0 < N; n0 += chunk) {
        // a short last chunk still goes through this kernel (it handles any token count)
        const int64_t n = N - n0 < chunk ? N - n0 : chunk;
        Epilogue e = epi;
        if (e.residual)
            e.residual += n0 * Mout;
        const fp6_status st = launch_tiled_chunk<Src>(weights, scales, static_cast<const half_t *>(X) + n0 * K,
                                                      static_cast<half_t *>(Y) + n0 * Mout, M, n, K, workspace, e,
                                                      stream);
        if (st != FP6_OK)
            return st;
    }
    return FP6_OK;
}

template <class Src, int C>
fp6_status launch_stream_cfg(const StreamPlan &p, const void *weights, const void *scales, const void *X, void *Y,
                             int64_t M, int64_t N, int64_t K, float4_t *partials, int *counters, const Epilogue &epi,
                             hipStream_t stream)
{
    typedef typename StreamShapeOf<Src::kPackedConfigs, C>::type Shape;
    constexpr StreamCfg c = StreamShapeOf<Src::kPackedConfigs, C>::c;
    auto kernel = linear_stream_kernel<Src, Shape>;
    constexpr size_t lds = Shape::template lds_bytes<Src>();
    static_assert(lds <= 160 * 1024, "activation stages and staged weight tiles exceed the LDS of a CU");
    static std::atomic<uint64_t> lds_done{0};  // per instantiation
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(kernel), lds, lds_done))
        return FP6_ERR_HIP;
    const dim3 grid((unsigned)p.row_blocks, (unsigned)p.split), block(c.waves * 64);  // x runs fastest: row blocks of one k slice
    // tokens are processed 16*nt at a time; each pass re-streams the weights
    const int64_t step = 16 * c.nt;
    const int64_t Mout = epi.gated ? M / 2 : M;
    for (int64_t n0 = 0; n0 < N; n0 += step) {
        const int64_t n = (N - n0 < step) ? (N - n0) : step;
        const half_t *Xp = static_cast<const half_t *>(X) + n0 * K;
        half_t *Yp = static_cast<half_t *>(Y) + n0 * Mout;
        Epilogue e = epi;
        if (e.residual)
            e.residual += n0 * Mout;
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, weights, static_cast<const half_t *>(scales), Xp, Yp,
                           (int)M, (int)n, (int)K, p.split, (int)((K + Src::kTileCols - 1) / Src::kTileCols / p.split),
                           partials, counters, e);
        if (hipGetLastError() != hipSuccess)
            return FP6_ERR_HIP;
    }
    return FP6_OK;
}

template <class Src>
fp6_status launch_stream(const void *weights, const void *scales, const void *X, void *Y, int64_t M, int64_t N,
                         int64_t K, const WorkspaceRef &workspace, const Epilogue &epi, hipStream_t stream)
{
    const StreamPlan p = plan_stream(M, N, K, Src::kPackedConfigs, Src::kTileCols);
    SplitBuffers buf;
    const fp6_status fits = workspace.view(p.counter_bytes, p.split > 1 ? p.partial_bytes : 0, buf);
    if (fits != FP6_OK)
        return fits;
    int *counters = buf.counters;
    float4_t *partials = reinterpret_cast<float4_t *>(buf.partials);
    switch (p.cfg) {
    case 0: return launch_stream_cfg<Src, 0>(p, weights, scales, X, Y, M, N, K, partials, counters, epi, stream);
    case 1: return launch_stream_cfg<Src, 1>(p, weights, scales, X, Y, M, N, K, partials, counters, epi, stream);
    case 2: return launch_stream_cfg<Src, 2>(p, weights, scales, X, Y, M, N, K, partials, counters, epi, stream);
    default: return launch_stream_cfg<Src, 3>(p, weights, scales, X, Y, M, N, K, partials, counters, epi, stream);
    }
}

template <class Fmt>
fp6_status quantize_pack_impl(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16, void *stream)
{
    if (!W_f16 || !packed || !scales_f16)
        return FP6_ERR_NULL;
    if (!packed_shape_ok(M, K))
        return FP6_ERR_SHAPE;
    if (!aligned16(W_f16) || !aligned16(packed) || !aligned16(scales_f16))
        return FP6_ERR_ALIGN;
    hipLaunchKernelGGL(row_scale_kernel<Fmt>, dim3((unsigned)((M + kScaleWavesPerBlock - 1) / kScaleWavesPerBlock)),
                       dim3(kScaleWavesPerBlock * 64), 0, static_cast<hipStream_t>(stream),
                       static_cast<const half_t *>(W_f16), (int)M, (int)K, static_cast<half_t *>(scales_f16));
    if (hipGetLastError() != hipSuccess)
        return FP6_ERR_HIP;
    const int64_t tiles = (M / kTileRows) * (K / kTileK);
    hipLaunchKernelGGL(quantize_tiles_kernel<Fmt>, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const half_t *>(W_f16), (int)M, (int)K,
                       static_cast<uint8_t *>(packed), static_cast<const half_t *>(scales_f16));
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

template <class Src>
fp6_status unpack_impl(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out, void *stream)
{
    if (!packed || !scales_f16 || !W_f16_out)
        return FP6_ERR_NULL;
    if (!packed_shape_ok(M, K))
        return FP6_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(scales_f16) || !aligned16(W_f16_out))
        return FP6_ERR_ALIGN;
    const int64_t tiles = (M / kTileRows) * (K / kTileK);
    hipLaunchKernelGGL(unpack_kernel<Src>, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint8_t *>(packed),
                       static_cast<const half_t *>(scales_f16), (int)M, (int)K, static_cast<half_t *>(W_f16_out));
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

// ---- the library's own split-K buffer (fp6_linear_static) ------------------------------------------
// A file-scope device array: every GPU the library runs on holds its own copy, at its own address, until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the device
// address that the kernels and the fill take is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[FP6_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

fp6_status static_scratch_address(void **out)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices)
        return FP6_ERR_HIP;
    void *ptr = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return FP6_ERR_HIP;
        g_scratch_ptr[device].store(ptr, std::memory_order_release);  // racing threads store the same address
    }
    *out = ptr;
    return FP6_OK;
}

// Counter bytes that a call of the packed 6-bit layer needs in the static buffer, or FP6_ERR_WORKSPACE when
// the call does not fit it.  Host arithmetic only.
fp6_status static_plan(int64_t M, int64_t N, int64_t K, size_t &counter_bytes)
{
    const WorkspaceRef probe{reinterpret_cast<void *>(uintptr_t(256)), FP6_STATIC_SCRATCH_BYTES, true};  // never dereferenced
    SplitBuffers unused;
    counter_bytes = 0;
    if (N <= kStreamMaxN) {
        const StreamPlan p = plan_stream(M, N, K, true);
        if (p.split > 1)
            counter_bytes = p.counter_bytes;
        return probe.view(p.counter_bytes, p.split > 1 ? p.partial_bytes : 0, unused);
    }
    const int64_t chunk = tiled_chunk_tokens(K);
    if (chunk <= 0)
        return FP6_ERR_SHAPE;
    for (int64_t n : {N < chunk ? N : chunk, N > chunk ? N % chunk : (int64_t)0}) {
        if (n <= 0)
            continue;
        const TiledPlan p = plan_tiled(M, n, K, PackedFp6Source::kTallTile);
        if (p.split > 1 && p.counter_bytes > counter_bytes)
            counter_bytes = p.counter_bytes;
        const fp6_status fits = probe.view(p.counter_bytes, p.split > 1 ? p.partial_bytes : 0, unused);
        if (fits != FP6_OK)
            return fits;
    }
    return FP6_OK;
}

template <class Src>
fp6_status packed_linear_impl(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                              int64_t N, int64_t K, void *workspace, size_t workspace_bytes, void *stream,
                              const Epilogue &epi = Epilogue{nullptr, nullptr, 0}, bool static_buffer = false)
{
    const WorkspaceRef ws{workspace, workspace_bytes, static_buffer};
    if (!packed || !scales_f16 || !X_f16 || !Y_f16)
        return FP6_ERR_NULL;
    if (!packed_shape_ok(M, K) || N <= 0 || N >= (1ll << 31))
        return FP6_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(scales_f16) || !aligned16(X_f16) || !aligned16(Y_f16) || !aligned16(epi.bias)
        || !aligned16(epi.residual))
        return FP6_ERR_ALIGN;
    if (N > kStreamMaxN)
        return launch_tiled<Src>(packed, scales_f16, X_f16, Y_f16, M, N, K, ws, epi, static_cast<hipStream_t>(stream));
    return launch_stream<typename Src::StreamSource>(packed, scales_f16, X_f16, Y_f16, M, N, K, ws, epi,
                                                     static_cast<hipStream_t>(stream));
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

size_t fp6_packed_bytes(int64_t M, int64_t K) { return packed_shape_ok(M, K) ? (size_t)(M * K / 4 * 3) : 0; }

size_t fp6_linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (!packed_shape_ok(M, K) || N <= 0)
        return 0;
    return N <= kStreamMaxN ? plan_stream(M, N, K, true).total_bytes()
                            : tiled_workspace_bytes(M, N, K, PackedFp6Source::kTallTile);
}

size_t fp16_linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (!shape_ok(M, K) || N <= 0)
        return 0;
    return N <= kStreamMaxN ? plan_stream(M, N, K, false).total_bytes()
                            : tiled_workspace_bytes(M, N, K, PlainFp16Source::kTallTile);
}

void fp6_tuning_set_split_k(int split_k) { g_forced_split.store(split_k < 0 ? 0 : split_k); }

void fp6_tuning_set_tile(int block_rows, int block_tokens)
{
    const bool known = (block_rows == 128 || block_rows == 256) && (block_tokens == 64 || block_tokens == 128);
    g_forced_tile.store(known ? block_rows * 1024 + block_tokens : 0);
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
    return quantize_pack_impl<E3M2Format>(W_f16, M, K, packed, scales_f16, stream);
}

fp6_status fp6_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out, void *stream)
{
    return unpack_impl<PackedFp6Source>(packed, scales_f16, M, K, W_f16_out, stream);
}

fp6_status fp6_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N,
                      int64_t K, void *workspace, size_t workspace_bytes, void *stream)
{
    return packed_linear_impl<PackedFp6Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                               stream);
}

fp6_status fp6_linear_static(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                             int64_t N, int64_t K, void *stream)
{
    if (!packed || !scales_f16 || !X_f16 || !Y_f16)
        return FP6_ERR_NULL;
    if (!packed_shape_ok(M, K) || N <= 0 || N >= (1ll << 31))
        return FP6_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(scales_f16) || !aligned16(X_f16) || !aligned16(Y_f16))
        return FP6_ERR_ALIGN;
    size_t counter_bytes = 0;
    const fp6_status fits = static_plan(M, N, K, counter_bytes);  // before the device is touched
    if (fits != FP6_OK)
        return fits;
    void *buffer = nullptr;
    if (counter_bytes > 0) {
        const fp6_status found = static_scratch_address(&buffer);
        if (found != FP6_OK)
            return found;
        // the array keeps what the last call left: the arrival counters must start at zero (a fill kernel,
        // not a memset node, so that the call can be captured into a graph)
        const size_t n16 = counter_bytes / 16;
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), static_cast<u32x4 *>(buffer), n16);
        if (hipGetLastError() != hipSuccess)
            return FP6_ERR_HIP;
    }
    return packed_linear_impl<PackedFp6Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, buffer,
                                               buffer ? (size_t)FP6_STATIC_SCRATCH_BYTES : 0, stream,
                                               Epilogue{nullptr, nullptr, 0}, true);
}

fp6_status fp6_linear_fused(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                            int64_t N, int64_t K, const void *bias_f16, const void *residual_f16, int gated,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    const Epilogue epi{static_cast<const half_t *>(bias_f16), static_cast<const half_t *>(residual_f16), gated ? 1 : 0};
    return packed_linear_impl<PackedFp6Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                               stream, epi);
}

fp6_status fp6g_quantize_pack(const void *W_f16, int64_t M, int64_t K, int64_t group, void *packed, void *scales_f16,
                              void *stream)
{
    if (!W_f16 || !packed || !scales_f16)
        return FP6_ERR_NULL;
    if (!packed_shape_ok(M, K) || group != kGroupColumns)
        return FP6_ERR_SHAPE;
    if (!aligned16(W_f16) || !aligned16(packed) || !aligned16(scales_f16))
        return FP6_ERR_ALIGN;
    const int64_t tiles = (M / kTileRows) * (K / kTileK);
    hipLaunchKernelGGL(quantize_pack_group_kernel, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const half_t *>(W_f16), (int)M, (int)K,
                       static_cast<uint8_t *>(packed), static_cast<half_t *>(scales_f16));
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

fp6_status fp6g_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, int64_t group, void *W_f16_out,
                       void *stream)
{
    if (group != kGroupColumns)
        return FP6_ERR_SHAPE;
    return unpack_impl<PackedFp6GroupSource>(packed, scales_f16, M, K, W_f16_out, stream);
}

fp6_status fp6g_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N,
                       int64_t K, int64_t group, void *workspace, size_t workspace_bytes, void *stream)
{
    if (group != kGroupColumns)
        return FP6_ERR_SHAPE;
    return packed_linear_impl<PackedFp6GroupSource>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace,
                                                    workspace_bytes, stream);
}

size_t fp5_packed_bytes(int64_t M, int64_t K) { return packed_shape_ok(M, K) ? (size_t)(M * K / 8 * 5) : 0; }

size_t fp5_linear_workspace_bytes(int64_t M, int64_t N, int64_t K) { return fp6_linear_workspace_bytes(M, N, K); }

fp6_status fp5_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16, void *stream)
{
    return quantize_pack_impl<E2M2Format>(W_f16, M, K, packed, scales_f16, stream);
}

fp6_status fp5_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out, void *stream)
{
    return unpack_impl<PackedFp5Source>(packed, scales_f16, M, K, W_f16_out, stream);
}

fp6_status fp5_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N,
                      int64_t K, void *workspace, size_t workspace_bytes, void *stream)
{
    return packed_linear_impl<PackedFp5Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                               stream);
}

size_t fp4_packed_bytes(int64_t M, int64_t K) { return packed_shape_ok(M, K) ? (size_t)(M * K / 2) : 0; }

size_t fp4_linear_workspace_bytes(int64_t M, int64_t N, int64_t K) { return fp6_linear_workspace_bytes(M, N, K); }

fp6_status fp4_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16, void *stream)
{
    return quantize_pack_impl<E2M1Format>(W_f16, M, K, packed, scales_f16, stream);
}

fp6_status fp4_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out, void *stream)
{
    return unpack_impl<PackedFp4Source>(packed, scales_f16, M, K, W_f16_out, stream);
}

fp6_status fp4_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N,
                      int64_t K, void *workspace, size_t workspace_bytes, void *stream)
{
    return packed_linear_impl<PackedFp4Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                               stream);
}

// tiles of 16 x 512 codes: a K that is an odd multiple of 256 pads its last tile
size_t fp3_packed_bytes(int64_t M, int64_t K)
{
    return packed_shape_ok(M, K) ? (size_t)((K + 511) / 512 * (M / kTileRows) * kTileBytes3) : 0;
}

size_t fp3_linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (!packed_shape_ok(M, K) || N <= 0)
        return 0;
    return N <= kStreamMaxN ? plan_stream(M, N, K, true, PackedFp3Source::StreamSource::kTileCols).total_bytes()
                            : tiled_workspace_bytes(M, N, K, PackedFp3Source::kTallTile);
}

fp6_status fp3_quantize_pack(const void *W_f16, int64_t M, int64_t K, void *packed, void *scales_f16, void *stream)
{
    return quantize_pack_impl<E2M0Format>(W_f16, M, K, packed, scales_f16, stream);
}

fp6_status fp3_unpack(const void *packed, const void *scales_f16, int64_t M, int64_t K, void *W_f16_out, void *stream)
{
    return unpack_impl<PackedFp3Source>(packed, scales_f16, M, K, W_f16_out, stream);
}

fp6_status fp3_linear(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N,
                      int64_t K, void *workspace, size_t workspace_bytes, void *stream)
{
    return packed_linear_impl<PackedFp3Source>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes,
                                               stream);
}

#define FP6_FUSED_ENTRY(NAME, SRC)                                                                                     \
    fp6_status NAME(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M, int64_t N, \
                    int64_t K, const void *bias_f16, const void *residual_f16, int gated, void *workspace,             \
                    size_t workspace_bytes, void *stream)                                                              \
    {                                                                                                                  \
        const Epilogue epi{static_cast<const half_t *>(bias_f16), static_cast<const half_t *>(residual_f16),         \
                           gated ? 1 : 0};                                                                             \
        return packed_linear_impl<SRC>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace, workspace_bytes, stream,  \
                                       epi);                                                                           \
    }
FP6_FUSED_ENTRY(fp5_linear_fused, PackedFp5Source)
FP6_FUSED_ENTRY(fp4_linear_fused, PackedFp4Source)
FP6_FUSED_ENTRY(fp3_linear_fused, PackedFp3Source)
#undef FP6_FUSED_ENTRY

fp6_status fp6g_linear_fused(const void *packed, const void *scales_f16, const void *X_f16, void *Y_f16, int64_t M,
                             int64_t N, int64_t K, int64_t group, const void *bias_f16, const void *residual_f16,
                             int gated, void *workspace, size_t workspace_bytes, void *stream)
{
    if (group != kGroupColumns)
        return FP6_ERR_SHAPE;
    const Epilogue epi{static_cast<const half_t *>(bias_f16), static_cast<const half_t *>(residual_f16), gated ? 1 : 0};
    return packed_linear_impl<PackedFp6GroupSource>(packed, scales_f16, X_f16, Y_f16, M, N, K, workspace,
                                                    workspace_bytes, stream, epi);
}

fp6_status fp6_probe_read(const void *buffer, size_t bytes, void *sink, void *stream)
{
    if (!buffer || !sink)
        return FP6_ERR_NULL;
    if (!aligned16(buffer))
        return FP6_ERR_ALIGN;
    // 1024 waves (four per CU), each at least one double step of 2 x 8 KB
    const unsigned blocks = kCus;
    if (bytes < (size_t)blocks * 4 * 16384)
        return FP6_ERR_SHAPE;
    hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint8_t *>(buffer), bytes, static_cast<uint32_t *>(sink));
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

size_t fp6_probe_read_bytes(size_t bytes) { return bytes / (kCus * 4) / 16384 * 16384 * (kCus * 4); }

size_t fp6_probe_mfma_sink_bytes(void) { return (size_t)kCus * 4 * 256 * sizeof(float); }

fp6_status fp6_probe_mfma(int64_t iters, void *sink, void *stream)
{
    if (!sink)
        return FP6_ERR_NULL;
    if (iters <= 0 || iters >= (1ll << 31))
        return FP6_ERR_SHAPE;
    // four blocks of four waves per CU: four waves per SIMD
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kCus * 4), dim3(256), 0, static_cast<hipStream_t>(stream), (int)iters,
                       static_cast<float *>(sink));
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
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
    const WorkspaceRef ws{workspace, workspace_bytes, false};
    if (N > kStreamMaxN)
        return launch_tiled<PlainFp16Source>(W_f16, nullptr, X_f16, Y_f16, M, N, K, ws, Epilogue{nullptr, nullptr, 0},
                                             static_cast<hipStream_t>(stream));
    return launch_stream<PlainFp16Source::StreamSource>(W_f16, nullptr, X_f16, Y_f16, M, N, K, ws, Epilogue{nullptr, nullptr, 0},
                                          static_cast<hipStream_t>(stream));
}

}  // extern "C"
