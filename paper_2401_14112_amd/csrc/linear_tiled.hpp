// Tiled linear-layer kernel for prefill-sized token counts (N > 64), where the layer is bound by
// the matrix cores (Section 7.1 of the paper: all kernels become compute-bound beyond batch 128).
//
// A block is WM x WN waves; wave (wm, wn) owns RT 16-row tiles and NT 16-token tiles, i.e. a
// (16*RT) x (16*NT) piece of Y held in fp32 accumulators; the block covers (16*RT*WM) rows and
// (16*NT*WN) tokens.  Per 256-column k-tile a wave fetches its RT packed weight tiles straight into
// registers, de-quantizes four runs of 32 columns with one conversion and feeds every run to NT MFMAs (the
// conversion is amortised over 4*NT matrix instructions); every activation fragment read from LDS feeds RT
// MFMAs.  The activations (all tokens of the block) are shared by the block: they are copied
// global -> LDS without passing through registers, already in B-fragment order (the 64 lanes of one
// copy instruction fetch the 64 pieces that the 64 lanes of one MFMA will read), half a k-tile (128
// columns) at a time into a ring of four buffers, requested three half tiles ahead and made visible one
// half tile ahead; weights are double-buffered in registers, one k-tile ahead.
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
    // Activations are staged half a k-tile (128 columns = runs 0..3 or 4..7) at a time in a ring of XS
    // buffers; weights are double-buffered in registers (whole k-tiles).
    constexpr int XS = 4;
    constexpr int XHPIECES = BNT * 256;      // 16-byte pieces of one half tile of activations
    constexpr int XHBYTES = XHPIECES * 16;
    constexpr int HCOPIES = BNT * 4;         // copy instructions per half tile (one per token tile and run)
    static_assert(HCOPIES % WAVES == 0, "activation copies must split evenly over the waves");
    constexpr int XPERH = HCOPIES / WAVES;
    constexpr int WLOADS = RT * Src::kLoads; // weight loads of one wave per k-tile

    extern __shared__ u32x4 xs_dyn[];  // [XS][XHPIECES]
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
        w_stream[r].init(weights, scales, rt < n_row_tiles ? rt : n_row_tiles - 1, kt0, 1, n_valid, n_row_tiles, K, lane);
    }
    const rsrc_t x_rsrc = make_rsrc(X, (uint32_t)N * (uint32_t)K * 2u);

    // Activation copies: copy j = wave + WAVES*i of half tile h serves token tile nt = j/4 and run
    // f = j%4 + 4*(h%2) of k-tile h/2; lane p of the copy fetches
    // X[block_col0 + 16*nt + n][k0 + k_offset(f, q) ..+8] for the (n, q) that piece p of the 1 KB holds (see
    // x_source_of_piece), and its 16 bytes land at piece 64*j + p of the ring buffer.  Half tiles past the
    // end of the slice and token columns >= N get an offset outside the buffer: zeros land in LDS.
    int xq, xn;
    x_source_of_piece(lane, xn, xq);
    const int b_piece = x_piece_of_lane(lane);
    // LDS byte address of the activation buffers (the low 32 bits of a shared-memory pointer)
    const uint32_t xs_lds = (uint32_t)reinterpret_cast<uintptr_t>(xs_dyn);
    // copy i (of the XPERH this wave contributes) of half tile h into ring buffer buf
    auto x_issue_one = [&](int h, int buf, int i) {
        const int t = h >> 1;
        const int j = wave + WAVES * i;
        const int nt = j >> 2, f = (j & 3) + 4 * (h & 1);
        const int col = block_col0 + nt * 16 + xn;
        const int off = (t < n_valid && col < N)
                            ? (col * K + (kt0 + t) * kTileK + Src::k_offset(f, xq)) * 2
                            : kOutOfRange;
        const uint32_t lds_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(xs_lds + buf * XHBYTES + j * 1024));
        issue_load_to_lds_b128<0>(x_rsrc, off, lds_base);
    };
    auto x_issue = [&](int h, int buf) {
#pragma unroll
        for (int i = 0; i < XPERH; ++i)
            x_issue_one(h, buf, i);
    };

    float4_t acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            acc[r][nt] = (float4_t){0.f, 0.f, 0.f, 0.f};

    // One half tile = 4 runs x NT token tiles = 4*NT steps of RT MFMAs, in two groups of two runs.  B
    // fragments travel through a small ring of registers: the LDS read of step s+LOOK is issued when step s
    // is consumed, and the ring runs on across half tiles (the next half tile is already visible, see
    // below), so the matrix pipe does not drain at a boundary.  The A fragments of the next group are
    // produced (conversion + register moves, VALU work) while the MFMAs of the current group execute.  The
    // sched_group_barrier sequence fixes the instruction order inside a group to "1 LDS read, RT MFMAs, a few
    // VALU" per step: a wave cannot issue anything else while one of its MFMAs is being issued, so the VALU
    // work is laid out in small pieces that the other waves of the SIMD can cover with their own MFMAs.
    constexpr int LOOK = 4;
    constexpr int STEPS = 4 * NT;
    constexpr int VALU_PER_STEP = 2;  // VALU instructions the scheduler may place after the MFMAs of a step
    half8_t a[2][2][RT];  // [group parity][even/odd run][row tile]
    half8_t bq[LOOK];
    auto ldb = [&](const u32x4 *xbuf, int st) {
        return bit_cast<half8_t>(xbuf[((wn * NT + (st % NT)) * 4 + st / NT) * 64 + b_piece]);
    };
    // HP: which half of the k-tile t; xbuf: its activations; xnext: those of the following half tile;
    // request(step): called after each of the 4*NT steps of the half tile, issues the memory requests that the
    // schedule places there (the requests of a half step are spread over its matrix work: issued in one burst
    // after the barrier, the ten requests of each of the eight waves queue up in the CU's address unit and the
    // waves stand at the issue of their loads for a quarter of the half step with the matrix pipe idle)
    auto compute_half = [&](auto hp_c, const typename Src::Tile (&t)[RT], const u32x4 *xbuf, const u32x4 *xnext,
                            auto &&request) {
        constexpr int HP = decltype(hp_c)::value;
        static_for<2>([&](auto gh_c) {
            constexpr int GH = decltype(gh_c)::value;
            __builtin_amdgcn_sched_barrier(0);
            if (HP == 0 || GH == 0) {
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    Src::template fragments<(2 * HP + GH + 1 <= 3 ? 2 * HP + GH + 1 : 3)>(t[r], a[GH ^ 1][0][r], a[GH ^ 1][1][r]);
            }
            static_for<2 * NT>([&](auto i_c) {
                constexpr int i = decltype(i_c)::value;
                constexpr int st = 2 * GH * NT + i;
                const half8_t b = bq[st % LOOK];
                bq[st % LOOK] = st + LOOK < STEPS ? ldb(xbuf, st + LOOK) : ldb(xnext, st + LOOK - STEPS);
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    acc[r][st % NT] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[GH][i / NT][r], b, acc[r][st % NT], 0, 0, 0);
                request(std::integral_constant<int, st>{});
            });
#pragma unroll
            for (int i = 0; i < 2 * NT; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, RT, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_STEP, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // ---- software pipeline.  Half step h (k-tile t = h/2) computes half tile h.  At its top the wave waits
    // for the activations of half tile h+1 (its own copies of them, requested at half step h-2) and, when h
    // is even, for the weights of k-tile t (requested at half step h-2, before those copies); one barrier
    // then makes half tile h+1 visible to the whole block - half tile h became visible one step earlier,
    // which is what lets the B-fragment ring run across the boundary - and guarantees that half tile h-1 is
    // no longer being read, so its buffer takes the copies of half tile h+3, requested next, after the
    // weights of k-tile t+1 when h is even.  Loads complete in order, so "at most n outstanding" with n = the
    // loads requested after the ones needed (the copies of half step h-1, plus its weight loads when h is
    // odd) means they have arrived.
    typename Src::Tile w[2][RT];
    auto w_issue = [&](typename Src::Tile (&dst)[RT], int t) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
            w_stream[r].issue(dst[r], t);
    };
    auto pin_tiles = [&](typename Src::Tile (&dst)[RT]) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
            Src::pin_tile(dst[r]);
    };
    w_issue(w[0], 0);
#pragma unroll
    for (int i = 0; i < XS - 1; ++i)
        x_issue(i, i);
    // half tile 0 has to be visible before the ring is primed
    wait_loads<XPERH>();
    __syncthreads();
#pragma unroll
    for (int i = 0; i < LOOK; ++i)
        bq[i] = ldb(xs_dyn, i);
    const int n_half = 2 * n_valid;
    for (int h0 = 0; h0 < n_half; h0 += XS) {
        static_for<XS>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            constexpr int hp = u & 1, xb = u % XS, ws = (u / 2) % 2;
            constexpr int n_after = hp == 1 ? XPERH + WLOADS : XPERH;
            const int h = h0 + u;
            if (h < n_half) {  // the same for every wave of the block
                wait_loads<n_after>();
                if (hp == 0)
                    pin_tiles(w[ws]);
                __syncthreads();
                if (hp == 0) {
#pragma unroll
                    for (int r = 0; r < RT; ++r)
                        Src::template fragments<0>(w[ws][r], a[0][0][r], a[0][1][r]);
                }
                // the requests of this half step, unit by unit (the weights of one row tile of k-tile t+1 when h
                // is even, then one activation copy of half tile h+3 each), unit k after step (k+1)*STEPS/(units+1)
                constexpr int W_UNITS = hp == 0 ? RT : 0, UNITS = W_UNITS + XPERH;
                compute_half(std::integral_constant<int, hp>{}, w[ws], xs_dyn + xb * XHPIECES,
                             xs_dyn + ((xb + 1) % XS) * XHPIECES, [&](auto st_c) {
                                 constexpr int st = decltype(st_c)::value;
                                 static_for<UNITS>([&](auto k_c) {
                                     constexpr int k = decltype(k_c)::value;
                                     if constexpr ((k + 1) * STEPS / (UNITS + 1) - 1 == st) {
                                         if constexpr (k < W_UNITS)
                                             w_stream[k].issue(w[ws ^ 1][k], (h >> 1) + 1);
                                         else
                                             x_issue_one(h + XS - 1, (xb + XS - 1) % XS, k - W_UNITS);
                                     }
                                 });
                             });
            }
        });
    }
    // the look-ahead requests (out of range: zeros) must land before the registers are reused and before
    // the block gives up its LDS
    wait_loads<0>();
    pin_tiles(w[0]);
    pin_tiles(w[1]);

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
