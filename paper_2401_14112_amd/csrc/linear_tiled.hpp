// Tiled linear-layer kernel for prefill-sized token counts (N > 64), where the layer is bound by
// the matrix cores (Section 7.1 of the paper: all kernels become compute-bound beyond batch 128).
//
// A block is WM x WN waves; wave (wm, wn) owns RT 16-row tiles and NT 16-token tiles, i.e. a
// (16*RT) x (16*NT) piece of Y held in fp32 accumulators; the block covers (16*RT*WM) rows and
// (16*NT*WN) tokens.  Per 256-column k-tile a wave fetches its RT packed weight tiles straight into
// registers, de-quantizes four runs of 32 columns with one conversion and feeds every run to NT MFMAs (the
// conversion is amortised over 4*NT matrix instructions); every activation fragment read from LDS feeds RT
// MFMAs.  The activation tile (all tokens of the block x 256 columns) is shared by the block: it is
// copied global -> LDS without passing through registers, already in B-fragment order (the 64 lanes
// of one copy instruction fetch the 64 pieces that the 64 lanes of one MFMA will read), and is
// double-buffered.
//
// Pipeline (one k-tile of look-ahead, enough because a k-tile is RT*NT*8 MFMAs of work per wave and
// two waves share a SIMD): at the top of iteration t the wave waits for everything it requested for
// tile t, one barrier makes the whole activation tile visible (and guarantees that the other LDS
// buffer is no longer being read), then the requests for tile t+1 are issued - activation copies
// into the other LDS buffer, weights into the other register buffer - and tile t is computed.
//
// Split-K and the epilogue are those of the streaming kernel (linear_stream.hpp).
#pragma once
#include "fp6_device.hpp"

namespace fp6 {

template <class Src, int RT, int NT, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void linear_tiled_kernel(
    const void *__restrict__ weights, const half_t *__restrict__ scales, const half_t *__restrict__ X,
    half_t *Y, int M, int N, int K, int S, int n_blocks, float4_t *__restrict__ partials,
    int *__restrict__ counters, Epilogue epi)
{
    constexpr int WAVES = WM * WN;
    constexpr int BNT = WN * NT;             // 16-token tiles of the block
    constexpr int XCHUNKS = BNT * 512;       // 16-byte pieces of one activation tile
    constexpr int XBYTES = XCHUNKS * 16;
    constexpr int COPIES = BNT * 8;          // copy instructions per activation tile (one per token tile and run)
    static_assert(COPIES % WAVES == 0, "activation copies must split evenly over the waves");
    constexpr int XPER = COPIES / WAVES;

    extern __shared__ u32x4 xs_dyn[];  // [2][XCHUNKS]
    __shared__ int s_is_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int KT = K / kTileK;
    const int n_row_tiles = M / kTileRows;
    // block -> (row block, token block, k slice).  Consecutive block ids land on consecutive XCDs (8 of
    // them, each with its own L2).  The blocks of one XCD take row blocks congruent to the XCD index and,
    // running side by side, all token blocks / k slices of those row blocks: a weight tile is then fetched
    // from memory by one XCD only and the other token blocks hit it in that XCD's L2, while the (much
    // smaller) activations are the operand that every XCD reads in full.
    constexpr int kXcds = 8;
    const int combos = n_blocks * S;
    const int xcd = blockIdx.x % kXcds;
    const int rest = blockIdx.x / kXcds;
    const int combo = rest % combos;
    const int row_block = (rest / combos) * kXcds + xcd;  // may run past the last row block: handled as a ragged edge
    const int n_block = combo % n_blocks;
    const int split = combo / n_blocks;
    if (row_block * WM * RT >= n_row_tiles)
        return;  // padding block of the XCD round-robin (whole block, before any barrier)
    const int row_tile0 = (row_block * WM + wm) * RT;
    const int block_col0 = n_block * BNT * 16;
    const int col0 = block_col0 + wn * NT * 16;  // first token of this wave
    const int kt0 = (int)(((unsigned)KT * (unsigned)split) / (unsigned)S);
    const int kt1 = (int)(((unsigned)KT * (unsigned)(split + 1)) / (unsigned)S);
    const int n_valid = kt1 - kt0;

    typename Src::Stream w_stream[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const int rt = row_tile0 + r;
        w_stream[r].init(weights, scales, rt < n_row_tiles ? rt : n_row_tiles - 1, kt0, kt1, KT, K, lane);
    }
    const rsrc_t x_rsrc = make_rsrc(X, (uint32_t)N * (uint32_t)K * 2u);

    // Activation copies: copy j = wave + WAVES*i of a tile serves token tile nt = j/8 and run f = j%8;
    // lane p of the copy fetches X[block_col0 + 16*nt + n][k0 + k_offset(f, q) ..+8] for the (n, q) that
    // piece p of the 1 KB holds (see x_source_of_piece), and its 16 bytes land at piece 64*j + p.
    int xq, xn;
    x_source_of_piece(lane, xn, xq);
    const int b_piece = x_piece_of_lane(lane);
    // LDS byte address of the activation buffers (the low 32 bits of a shared-memory pointer)
    const uint32_t xs_lds = (uint32_t)reinterpret_cast<uintptr_t>(xs_dyn);
    // copies [i0, i1) of the XPER copies this wave contributes to the activation tile of k-tile t
    auto x_issue = [&](int t, int buf, int i0, int i1) {
#pragma unroll
        for (int i = 0; i < XPER; ++i) {
            if (i < i0 || i >= i1)
                continue;
            const int j = wave + WAVES * i;
            const int nt = j >> 3, f = j & 7;
            const int col = block_col0 + nt * 16 + xn;
            const int off = (t < n_valid && col < N)
                                ? (col * K + (kt0 + t) * kTileK + Src::k_offset(f, xq)) * 2
                                : kOutOfRange;
            const uint32_t lds_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(xs_lds + buf * XBYTES + j * 1024));
            issue_load_to_lds_b128<0>(x_rsrc, off, lds_base);
        }
    };

    float4_t acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            acc[r][nt] = (float4_t){0.f, 0.f, 0.f, 0.f};

    // One k-tile = 8 runs x NT token tiles = 8*NT steps of RT MFMAs.  B fragments travel through a small
    // ring of registers: the LDS read of step s+LOOK is issued when step s is consumed.  The A fragments of
    // runs 2g+2, 2g+3 are produced (conversion + register moves, VALU work) while the MFMAs of runs 2g, 2g+1
    // execute.  The sched_group_barrier sequence fixes the instruction order inside each group of two runs
    // to "1 LDS read, RT MFMAs, a few VALU" per step: a wave cannot issue anything else while one of its
    // MFMAs is being issued, so the VALU work is laid out in small pieces that the other waves of the SIMD
    // can cover with their own MFMAs, instead of bursts in which the matrix pipe idles.
    constexpr int LOOK = 4;
    constexpr int STEPS = 8 * NT;
#ifndef FP6_TILED_VALU
#define FP6_TILED_VALU 2  // VALU instructions the scheduler may place after the MFMAs of a step
#endif
#ifndef FP6_TILED_PARTS
#define FP6_TILED_PARTS 4
#endif
    constexpr int VALU_PER_STEP = FP6_TILED_VALU;
    auto ldb = [&](const u32x4 *xbuf, int st) {
        return bit_cast<half8_t>(xbuf[((wn * NT + (st % NT)) * 8 + st / NT) * 64 + b_piece]);
    };
    // `issue_part(g)`, g = 0..3, is called between the four groups: the requests for the next k-tile are
    // spread over the computation instead of being issued in one burst while the matrix pipe idles.
    auto compute = [&](const typename Src::Tile (&t)[RT], const u32x4 *xbuf, auto &&issue_part) {
        half8_t a[2][2][RT];  // [group parity][even/odd run][row tile]
        half8_t bq[LOOK];
#pragma unroll
        for (int i = 0; i < LOOK; ++i)
            bq[i] = ldb(xbuf, i);
#pragma unroll
        for (int r = 0; r < RT; ++r)
            Src::template fragments<0>(t[r], a[0][0][r], a[0][1][r]);
        __builtin_amdgcn_sched_barrier(0);
#define FP6_TILED_GROUP(G, NEXT)                                                                  \
    if (G < 3) {                                                                                  \
        _Pragma("unroll") for (int r = 0; r < RT; ++r)                                            \
            Src::template fragments<NEXT>(t[r], a[(G + 1) & 1][0][r], a[(G + 1) & 1][1][r]);      \
    }                                                                                             \
    _Pragma("unroll") for (int i = 0; i < 2 * NT; ++i) {                                          \
        const int st = 2 * G * NT + i;                                                            \
        const half8_t b = bq[st % LOOK];                                                          \
        if (st + LOOK < STEPS)                                                                    \
            bq[st % LOOK] = ldb(xbuf, st + LOOK);                                                 \
        _Pragma("unroll") for (int r = 0; r < RT; ++r)                                            \
            acc[r][st % NT] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[G & 1][i / NT][r], b, acc[r][st % NT], 0, 0, 0); \
    }                                                                                             \
    _Pragma("unroll") for (int i = 0; i < 2 * NT; ++i) {                                          \
        if (2 * G * NT + i + LOOK < STEPS)                                                        \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, RT, 0);                                       \
        __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_STEP, 0);                            \
    }                                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    issue_part(G);                                                                                \
    __builtin_amdgcn_sched_barrier(0);
        FP6_TILED_GROUP(0, 1)
        FP6_TILED_GROUP(1, 2)
        FP6_TILED_GROUP(2, 3)
        FP6_TILED_GROUP(3, 3)
#undef FP6_TILED_GROUP
    };

    typename Src::Tile w[2][RT];
    auto w_issue = [&](typename Src::Tile (&dst)[RT], int t, int r0, int r1) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
            if (r >= r0 && r < r1)
                w_stream[r].issue(dst[r], t);
    };
    auto arrive = [&](typename Src::Tile (&dst)[RT]) {
        wait_loads<0>();
#pragma unroll
        for (int r = 0; r < RT; ++r)
            Src::pin_tile(dst[r]);
    };
    // part g of the requests for k-tile t: a quarter of this wave's activation copies and (RT/4 or 1) weight tiles
    auto issue_part = [&](typename Src::Tile (&dst)[RT], int t, int buf, int g) {
        constexpr int PARTS = FP6_TILED_PARTS;  // the activation copies are spread over the first PARTS groups
        if (g < PARTS)
            x_issue(t, buf, g * XPER / PARTS, (g + 1) * XPER / PARTS);
        if (RT >= 4)
            w_issue(dst, t, g * RT / 4, (g + 1) * RT / 4);
        else if (g < RT)
            w_issue(dst, t, g, g + 1);
    };

    x_issue(0, 0, 0, XPER);
    w_issue(w[0], 0, 0, RT);
    // two tiles per trip so that the register / LDS buffer index is static; tiles past the slice are zeros
    for (int t = 0; t < n_valid; t += 2) {
        arrive(w[0]);
        __syncthreads();
        compute(w[0], xs_dyn, [&](int g) { issue_part(w[1], t + 1, 1, g); });

        arrive(w[1]);
        __syncthreads();
        compute(w[1], xs_dyn + XCHUNKS, [&](int g) { issue_part(w[0], t + 2, 0, g); });
    }
    arrive(w[0]);  // the last look-ahead requests (out of range: zeros) must land before the block ends

    // ---- epilogue.  Lane L holds, per (row tile, token tile), rows 4*(L/16)+i of token column L%16.
    const int n_in_tile = lane & 15;
    const int n_tiles_total = n_blocks * BNT;
    auto finish = [&](const float4_t (&sum)[NT], int r) {
        const int m0 = (row_tile0 + r) * kTileRows + 4 * (lane >> 4);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int col = col0 + nt * 16 + n_in_tile;
            if (col < N)
                finish_rows<Src::kHasScale>(epi, scales, sum[nt], col, m0, M, Y);
        }
    };

    if (S == 1) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
            if (row_tile0 + r < n_row_tiles)
                finish(acc[r], r);
        return;
    }

    // split-K: see linear_stream.hpp for the protocol (device-scope accesses, ordered sum)
    float *pf = reinterpret_cast<float *>(partials);
    auto partial_ptr = [&](int s, int r, int nt) {
        return pf
               + ((((int64_t)s * n_row_tiles + (row_tile0 + r)) * n_tiles_total + ((n_block * WN + wn) * NT + nt)) * 4) * 64
               + lane;
    };
#pragma unroll
    for (int r = 0; r < RT; ++r)
        if (row_tile0 + r < n_row_tiles) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (col0 + nt * 16 + n_in_tile < N) {
                    float *dst = partial_ptr(split, r, nt);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        __hip_atomic_store(dst + i * 64, acc[r][nt][i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
        }
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's partial stores are done
    __syncthreads();
    const int counter_index = row_block * n_blocks + n_block;
    if (tid == 0) {
        const int arrived = __hip_atomic_fetch_add(&counters[counter_index], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_is_last = (arrived == S - 1);
    }
    __syncthreads();
    if (!s_is_last)
        return;
    for (int r = 0; r < RT; ++r) {
        if (row_tile0 + r >= n_row_tiles)
            break;
        float4_t sum[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            sum[nt] = (float4_t){0.f, 0.f, 0.f, 0.f};
        // PB slices per trip to memory, added in slice order (see linear_stream.hpp); fewer with wide
        // wave tiles, whose partial tiles take more registers
        constexpr int PB = NT >= 8 ? kPartialBatch / 2 : kPartialBatch;
        for (int s0 = 0; s0 < S; s0 += PB) {
            float4_t part[PB][NT];
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const int s = s0 + u < S ? s0 + u : S - 1;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const float *src = partial_ptr(s, r, nt);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        part[u][nt][i] = __hip_atomic_load(src + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
#pragma unroll
            for (int u = 0; u < PB; ++u)
                if (s0 + u < S) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        sum[nt] += part[u][nt];
                }
        }
        finish(sum, r);
    }
    if (tid == 0)
        counters[counter_index] = 0;  // re-arm for the next call on this workspace
}

}  // namespace fp6
