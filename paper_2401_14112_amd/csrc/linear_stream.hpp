// Weight-streaming linear-layer kernel for small token counts (N <= 64), where the
// layer is bound by reading the weights once from HBM (Section 3 and Section 7.1 of
// the paper: linear layers at batch < 128 are limited by weight traffic).
//
// Work split: one wave owns one 16-row tile and one split-K slice of its k-tiles (the
// weight source says how wide a tile is: 256 columns, 512 for the sources whose lane
// loads only come out as whole 128-bit pieces that way); weights go HBM -> VGPR with a
// few 128-bit loads per lane per tile (three for 6 bits), prefetched DEPTH tiles ahead,
// and are used by exactly one wave, so they never touch LDS (one source, row-major fp16
// weights, stages its tiles in a region of LDS private to the wave instead).  The
// activations (16*NT tokens) are the only shared operand: the block copies
// them global -> LDS without passing through registers, already in MFMA B-fragment
// order, a STAGE of G k-tiles at a time, double-buffered, with one barrier per stage.
// fp32 accumulation in v_mfma_f32_16x16x32_f16; the row scale is applied once in the
// epilogue.
//
// Split-K: every wave writes its fp32 partial tile, bumps the arrival counter of its
// row tile, and the wave that arrives last adds the S partials in split order (so the
// result does not depend on arrival order), scales, rounds and stores Y.  The counter
// is reset by that wave, so a zeroed workspace stays reusable.
#pragma once
#include "fp6_device.hpp"

namespace fp6 {

// Activation copies requested in the DEPTH-1 iterations before the iteration at stage position g, when
// each of the first XSPREAD iterations of a stage requests XPART of them.
constexpr int stream_copies_between(int g, int G, int DEPTH, int XSPREAD, int XPART)
{
    int c = 0;
    for (int d = 1; d < DEPTH; ++d)
        c += ((g - d + DEPTH * G) % G) < XSPREAD ? XPART : 0;
    return c;
}

// Shape of one instantiation: NT token tiles per wave, WAVES waves per block (one row tile each), DEPTH
// k-tiles of weights in flight per wave, G k-tiles per activation stage, the copies of a stage spread over the
// first XSPREAD iterations of the previous one.  DEAL: see the split-K comment in the kernel.
template <int NT_, int WAVES_, int DEPTH_, int G_, int XSPREAD_, bool DEAL_>
struct StreamShape {
    static constexpr int NT = NT_, WAVES = WAVES_, DEPTH = DEPTH_, G = G_, XSPREAD = XSPREAD_;
    static constexpr bool DEAL = DEAL_;
    // bytes of two stages of activations for weight tiles of tile_cols columns (1 KB per token tile and run of 32)
    static constexpr int x_bytes(int tile_cols) { return 2 * G_ * NT_ * (tile_cols / 32) * 1024; }
    static constexpr int kThreads = WAVES_ * 64;
    // dynamic LDS of a launch: the activation stages, then (sources that stage their weights in LDS) DEPTH
    // tiles per wave
    template <class Src>
    static constexpr int lds_bytes()
    {
        return x_bytes(Src::kTileCols) + WAVES_ * DEPTH_ * Src::kLdsTileBytes;
    }
};

template <class Src, class Shape>
__global__ __launch_bounds__(Shape::kThreads) void linear_stream_kernel(
    const void *__restrict__ weights, const half_t *__restrict__ scales, const half_t *__restrict__ X,
    half_t *Y, int M, int N, int K, int S, int kt_per_slice, float4_t *__restrict__ partials,
    int *__restrict__ counters, Epilogue epi)
{
    constexpr int NT = Shape::NT, WAVES = Shape::WAVES, DEPTH = Shape::DEPTH, G = Shape::G;
    constexpr int XSPREAD = Shape::XSPREAD;
    constexpr bool KDEAL = Shape::DEAL;
    constexpr int TILE_COLS = Src::kTileCols;  // columns of one weight tile: one step of the loop (a "k-tile" below)
    constexpr int RUNS = TILE_COLS / 32;        // MFMA steps per tile
    constexpr int COPIES = G * NT * RUNS;  // copy instructions (1 KB each: one token tile x one run) per stage
    static_assert(COPIES % WAVES == 0, "the copies of a stage must split evenly over the waves");
    constexpr int XPER = COPIES / WAVES;
    constexpr int STAGE_PIECES = COPIES * 64;  // 16-byte pieces of one stage
    // the copies of the next stage are requested in the first XSPREAD iterations of a stage
    static_assert(XSPREAD >= 1 && XSPREAD <= G && XPER % XSPREAD == 0, "bad spread of the activation copies");
    constexpr int XPART = XPER / XSPREAD;
    constexpr int U = G / stream_gcd(G, DEPTH) * DEPTH;  // unroll: both the stage position and the ring slot are static
    constexpr int WLOADS = Src::kLoads;  // weight loads of one wave per k-tile

    extern __shared__ u32x4 xs_dyn[];  // [2][STAGE_PIECES], then [WAVES][DEPTH] weight tiles for sources that stage them

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KT = (K + TILE_COLS - 1) / TILE_COLS;  // a K that is not a multiple of the tile: the last tile is padded
    const int n_row_tiles = M / kTileRows;
    // consecutive blocks take consecutive row blocks of the same k slice (measured a few per cent better at
    // N = 32, 64 than alternating the slices, no difference below)
    // The grid is (row blocks, k slices) and the host passes KT / S: nothing is divided here (a division by
    // a run-time value is a chain of ~30 dependent instructions, and the first request waits for it).
    const int row_block = blockIdx.x;
    const int split = blockIdx.y;
    const int row_tile = row_block * WAVES + wave;
    const bool active = row_tile < n_row_tiles;
    // Split-K, two ways of cutting the k-tiles of a row tile into S slices.  KDEAL: slice s takes k-tiles s,
    // s + S, s + 2S, ...: the waves of all slices then stand at the same depth of the k-tile-major weight
    // stream and the launch sweeps memory as one front, whatever S is.  Otherwise slice s is a contiguous
    // range (S fronts), the first `rem` slices one k-tile longer.
    const int rem = KT - S * kt_per_slice;
    const int kt_first = KDEAL ? split : split * kt_per_slice + (split < rem ? split : rem);
    const int kt_step = KDEAL ? S : 1;
    const int n_valid = kt_per_slice + (split < rem ? 1 : 0);  // k-tiles of this slice (>= 1)
    const int T = kt_per_slice + (rem > 0 ? 1 : 0);  // k-tiles computed: the same for every slice (>= n_valid)
    const int n_stages = (T + G - 1) / G;

    // Inactive waves (ragged last row block) stream the last valid row tile and drop the result,
    // so the main loop has no per-wave control flow.
    typename Src::Stream w_stream;
    w_stream.init(weights, scales, active ? row_tile : n_row_tiles - 1, kt_first, kt_step, n_valid, n_row_tiles, K, lane);
    const rsrc_t x_rsrc = make_rsrc(X, (uint32_t)N * (uint32_t)K * 2u);

    // ---- activation staging.  Copy j = wave + WAVES*i of a stage serves k-tile g = j / (RUNS*NT) of the
    // stage, token tile nt = (j/RUNS) % NT and run f = j % RUNS; lane p of the copy fetches
    // X[16*nt + n][k-tile*TILE_COLS + k_offset(f, q) ..+8] for the (n, q) that piece p of the 1 KB holds, and
    // its 16 bytes land at piece 64*j + p of the stage buffer.  Token columns >= N, k-tiles past the end of
    // the slice and columns >= K (the padding of a last tile) get an offset outside the buffer: nothing is
    // fetched and zeros land in LDS, which is what neutralises the k-tiles that the uniform trip count adds
    // to the shorter slices.
    int xn, xq;
    x_source_of_piece(lane, xn, xq);
    const uint32_t xs_lds = (uint32_t)reinterpret_cast<uintptr_t>(xs_dyn);  // LDS byte address
    auto x_issue = [&](int stage, int i0, int i1) {
        const int buf = stage & 1;
#pragma unroll
        for (int i = 0; i < XPER; ++i) {
            if (i < i0 || i >= i1)
                continue;
            const int j = wave + WAVES * i;
            const int f = j % RUNS, nt = (j / RUNS) % NT, g = j / (RUNS * NT);
            const int col = nt * 16 + xn;
            const int t = stage * G + g;
            const int k = (kt_first + t * kt_step) * TILE_COLS + Src::k_offset(f, xq);
            const int off = (t < n_valid && col < N && (K % TILE_COLS == 0 || k < K)) ? (col * K + k) * 2 : kOutOfRange;
            const uint32_t lds_base = (uint32_t)__builtin_amdgcn_readfirstlane(
                (int)(xs_lds + (uint32_t)(buf * STAGE_PIECES + j * 64) * 16u));
            issue_load_to_lds_b128<0>(x_rsrc, off, lds_base);
        }
    };

    const int b_piece = x_piece_of_lane(lane);
    float4_t acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        acc[nt] = (float4_t){0.f, 0.f, 0.f, 0.f};

    // xb: first piece of this k-tile's activations in LDS
    auto mma_pair = [&](const half8_t &a_even, const half8_t &a_odd, const u32x4 *xb, int p) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            half8_t b = bit_cast<half8_t>(xb[(nt * RUNS + 2 * p) * 64 + b_piece]);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_even, b, acc[nt], 0, 0, 0);
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            half8_t b = bit_cast<half8_t>(xb[(nt * RUNS + 2 * p + 1) * 64 + b_piece]);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_odd, b, acc[nt], 0, 0, 0);
        }
    };
    auto compute = [&](const typename Src::Tile &t, const u32x4 *xb) {
        static_for<RUNS / 2>([&](auto pc) {
            constexpr int p = decltype(pc)::value;
            half8_t a_even, a_odd;
            Src::template fragments<p>(t, a_even, a_odd);
            mma_pair(a_even, a_odd, xb, p);
        });
    };

    // ---- software pipeline.  Slot t % DEPTH of the register ring holds weight tile t of the slice; it is
    // requested DEPTH tiles ahead, right after the slot's previous tile has been consumed, so DEPTH-1 tiles
    // stay in flight while one is being computed.  The activation copies of stage s+1 are requested in the
    // first XSPREAD iterations of stage s, after that stage's barrier (by then every wave has finished
    // reading the buffer they overwrite).  Loads complete in order, so "at most n outstanding" with n = the
    // loads requested after the ones needed means those have arrived.  For the weights of tile t: n =
    // (DEPTH-1)*WLOADS plus the activation copies requested in the DEPTH-1 iterations in between (in every
    // iteration the copies are requested before the weights).  For the copies of a stage, needed at its first
    // iteration: the weights of the G - XSPREAD + 1 iterations since the last of them.  The first pass over
    // the ring has fewer copies behind it than the steady state (the prologue requests stage 0 before any
    // weights), so it waits for everything but the weights.  Tiles past the end of the slice read as zeros
    // through the buffer bounds check (no memory traffic), so the request pattern never varies.
    typename Src::Tile w[DEPTH];
    w_stream.bind_slots(w, xs_dyn + 2 * STAGE_PIECES + wave * (DEPTH * Src::kLdsTileBytes / 16), lane);
    x_issue(0, 0, XPER);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        w_stream.issue(w[d], d);
    const int n_tiles = n_stages * G;
    for (int t0 = 0; t0 < n_tiles; t0 += U) {
        static_for<U>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            constexpr int g = u % G, slot = u % DEPTH;
            constexpr int kWeightsAfter = (DEPTH - 1) * WLOADS + stream_copies_between(g, G, DEPTH, XSPREAD, XPART);
            constexpr int kCopiesAfter = (G - XSPREAD + 1) * WLOADS;
            constexpr int kAfter = g == 0 && kCopiesAfter < kWeightsAfter ? kCopiesAfter : kWeightsAfter;
            constexpr int kFirstPass = (DEPTH - 1) * WLOADS < kAfter ? (DEPTH - 1) * WLOADS : kAfter;
            static_assert(kAfter < 64, "more loads in flight than vmcnt can count");
            const int t = t0 + u;
            const int stage = t0 / G + u / G;
            if (t0 == 0)
                wait_loads<kFirstPass>();
            else
                wait_loads<kAfter>();
            Src::pin_tile(w[slot]);
            if (g == 0)
                __syncthreads();  // the copies of this stage by all waves have landed; the other buffer is no longer read
            if (g < XSPREAD)
                x_issue(stage + 1, g * XPART, (g + 1) * XPART);
            if (t < T)
                compute(w[slot], xs_dyn + (stage & 1) * STAGE_PIECES + g * (NT * RUNS * 64));
            w_stream.issue(w[slot], t + DEPTH);
        });
    }
    // drain: the look-ahead requests (weights out of range, activation copies into the unused buffer)
    // must land before the registers are reused and before the block gives up its LDS
    wait_loads<0>();
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        Src::pin_tile(w[d]);

    // ---- epilogue.  Lane L holds, per token tile, rows 4*(L/16)+i (i=0..3) of token column L%16.
    if (!active)
        return;  // no barrier follows the main loop
    const int n_in_tile = lane & 15;
    const int m0 = row_tile * kTileRows + 4 * (lane >> 4);
    auto finish = [&](const float4_t (&sum)[NT]) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int col = nt * 16 + n_in_tile;
            if (col < N)
                finish_rows<Src::kHasScale>(epi, scales, sum[nt], col, m0, M, Y);
        }
    };
    if (S == 1) {
        finish(acc);
        return;
    }

    // Split-K, one arrival counter per row tile: every wave is on its own from here (no barrier, so a wave
    // that finishes its stream early does not wait for the slowest wave of its block).  The partial tiles
    // are written and read with device-scope atomic (relaxed) accesses: such accesses are performed at the
    // point where all CUs of the device agree (they are not left in, nor served from, a non-coherent
    // cache), so no cache write-back or invalidate is needed.  Order: this wave's stores complete (vmcnt)
    // -> arrival count -> the last wave's loads; the signal fences keep the compiler from moving memory
    // operations across those two points.  The last wave adds the S partial tiles in split order, taking its
    // own from registers (the same bits it stored), so the sum does not depend on who is last.
    float *pf = reinterpret_cast<float *>(partials);
    auto slot = [&](int s_, int nt) { return pf + ((((int64_t)s_ * n_row_tiles + row_tile) * NT + nt) * 4) * 64 + lane; };
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        if (nt * 16 + n_in_tile < N) {
            float *dst = slot(split, nt);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __hip_atomic_store(dst + i * 64, acc[nt][i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's partial stores are done
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    int arrived = 0;
    if (lane == 0)
        arrived = __hip_atomic_fetch_add(&counters[row_tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    arrived = __builtin_amdgcn_readfirstlane(arrived);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    if (arrived != S - 1)
        return;
    // The partial tiles of kPartialBatch slices are requested together (one trip to memory per batch, not
    // per slice) and then added in slice order.  Every lane loads (lanes of token columns >= N read
    // words that nobody stored; their sums are never written).
    float4_t sum[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        sum[nt] = (float4_t){0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < S; s0 += kPartialBatch) {
        float4_t part[kPartialBatch][NT];
#pragma unroll
        for (int u = 0; u < kPartialBatch; ++u) {
            const int s_ = s0 + u < S ? s0 + u : S - 1;  // clamped: always an existing slot
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float *src = slot(s_, nt);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    part[u][nt][i] = __hip_atomic_load(src + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
#pragma unroll
        for (int u = 0; u < kPartialBatch; ++u) {
            const int s_ = s0 + u;
            if (s_ < S) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    sum[nt] += s_ == split ? acc[nt] : part[u][nt];
            }
        }
    }
    finish(sum);
    if (lane == 0)
        counters[row_tile] = 0;  // re-arm for the next call on this workspace
}

}  // namespace fp6
