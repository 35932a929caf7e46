// Weight-streaming linear-layer kernel for small token counts (N <= 32), where the
// layer is bound by reading the weights once from HBM (Section 3 and Section 7.1 of
// the paper: linear layers at batch < 128 are limited by weight traffic).
//
// Work split: one wave owns one 16-row tile and a contiguous range of its 256-column
// k-tiles (split-K slice); weights go HBM -> VGPR with three (packed) 128-bit loads
// per lane per tile, prefetched DEPTH tiles ahead, and are used by exactly one wave,
// so they never touch LDS.  The activation tile (16*NT tokens x 256 columns) is the
// only shared operand: the block stages it in LDS, already in MFMA B-fragment order,
// double-buffered with one barrier per k-tile.  fp32 accumulation in
// v_mfma_f32_16x16x32_f16; the row scale is applied once in the epilogue.
//
// Split-K: every block writes its fp32 partial tile, bumps an arrival counter of its
// row block, and the block that arrives last adds the S partials in split order
// (so the result does not depend on arrival order), scales, rounds and stores Y.
// The counter is reset by that block, so a zeroed workspace stays reusable.
#pragma once
#include "fp6_device.hpp"

namespace fp6 {

template <class Src, int NT, int WAVES, int DEPTH>
__global__ __launch_bounds__(WAVES * 64) void linear_stream_kernel(
    const void *__restrict__ weights, const half_t *__restrict__ scales, const half_t *__restrict__ X,
    half_t *__restrict__ Y, int M, int N, int K, int S, float4_t *__restrict__ partials,
    int *__restrict__ counters)
{
    constexpr int THREADS = WAVES * 64;
    constexpr int XCHUNKS = NT * 512;  // 16-byte pieces of one activation tile
    static_assert(XCHUNKS % THREADS == 0, "activation tile must split evenly over the block");
    constexpr int XPER = XCHUNKS / THREADS;

    __shared__ u32x4 xs[2][XCHUNKS];
    __shared__ int s_is_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int KT = K / kTileK;
    const int n_row_tiles = M / kTileRows;
    const int split = blockIdx.x % S;  // neighbouring blocks (one per XCD) take different k slices
    const int row_block = blockIdx.x / S;
    const int row_tile = row_block * WAVES + wave;
    const bool active = row_tile < n_row_tiles;
    const int kt0 = (int)(((int64_t)KT * split) / S);
    const int kt1 = (int)(((int64_t)KT * (split + 1)) / S);

    // ---- activation staging: piece c = nt*512 + f*64 + q*16 + n  <->  X[nt*16+n][k_tile*256 + k_offset(f,q) ..+8]
    u32x4 xr[XPER];
    auto x_fetch = [&](int k_tile) {
#pragma unroll
        for (int i = 0; i < XPER; ++i) {
            const int c = tid + i * THREADS;
            const int n = c & 15, q = (c >> 4) & 3, f = (c >> 6) & 7, nt = c >> 9;
            const int col = nt * 16 + n;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (col < N)
                v = *reinterpret_cast<const u32x4 *>(X + (int64_t)col * K + (int64_t)k_tile * kTileK
                                                     + Src::k_offset(f, q));
            xr[i] = v;
        }
    };
    auto x_commit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XPER; ++i)
            xs[buf][tid + i * THREADS] = xr[i];
    };

    float4_t acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        acc[nt] = (float4_t){0.f, 0.f, 0.f, 0.f};

    auto mma_pair = [&](const half8_t &a_even, const half8_t &a_odd, int buf, int g) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            half8_t b = bit_cast<half8_t>(xs[buf][nt * 512 + (2 * g) * 64 + lane]);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_even, b, acc[nt], 0, 0, 0);
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            half8_t b = bit_cast<half8_t>(xs[buf][nt * 512 + (2 * g + 1) * 64 + lane]);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_odd, b, acc[nt], 0, 0, 0);
        }
    };
    auto compute = [&](const typename Src::Tile &t, int buf) {
        half8_t a_even, a_odd;
        Src::template fragments<0>(t, a_even, a_odd);
        mma_pair(a_even, a_odd, buf, 0);
        Src::template fragments<1>(t, a_even, a_odd);
        mma_pair(a_even, a_odd, buf, 1);
        Src::template fragments<2>(t, a_even, a_odd);
        mma_pair(a_even, a_odd, buf, 2);
        Src::template fragments<3>(t, a_even, a_odd);
        mma_pair(a_even, a_odd, buf, 3);
    };

    // ---- prologue: DEPTH weight tiles in flight, first activation tile in LDS
    typename Src::Tile w[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (active && kt0 + d < kt1)
            w[d] = Src::load(weights, row_tile, kt0 + d, KT, K, lane);
    if (kt0 < kt1) {
        x_fetch(kt0);
        x_commit(0);
    }
    __syncthreads();

    // ---- main loop over the k-tiles of this split
    for (int kt = kt0; kt < kt1; kt += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int k = kt + d;
            if (k < kt1) {  // uniform over the block
                const int buf = (k - kt0) & 1;
                const bool more = (k + 1 < kt1);
                if (more)
                    x_fetch(k + 1);
                const typename Src::Tile cur = w[d];
                if (active && k + DEPTH < kt1)
                    w[d] = Src::load(weights, row_tile, k + DEPTH, KT, K, lane);
                if (active)
                    compute(cur, buf);
                if (more)
                    x_commit(buf ^ 1);
                __syncthreads();
            }
        }
    }

    // ---- epilogue.  Lane L holds, per n-tile, rows 4*(L/16)+i (i=0..3) of token column L%16.
    const int n_in_tile = lane & 15;
    const int m0 = row_tile * kTileRows + 4 * (lane >> 4);
    auto finish = [&](const float4_t (&sum)[NT]) {
        float sc[4] = {1.f, 1.f, 1.f, 1.f};
        if (Src::kHasScale) {
            const half4_t s4 = *reinterpret_cast<const half4_t *>(scales + m0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                sc[i] = (float)s4[i];
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int col = nt * 16 + n_in_tile;
            if (col < N) {
                half4_t y;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    y[i] = (half_t)(sum[nt][i] * sc[i]);
                *reinterpret_cast<half4_t *>(Y + (int64_t)col * M + m0) = y;
            }
        }
    };

    if (S == 1) {
        if (active)
            finish(acc);
        return;
    }

    if (active) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (nt * 16 + n_in_tile < N)
                partials[(((int64_t)split * n_row_tiles + row_tile) * NT + nt) * 64 + lane] = acc[nt];
    }
    __threadfence();  // publish the partial tile device-wide before signalling arrival
    __syncthreads();
    if (tid == 0) {
        __threadfence();
        const int arrived = atomicAdd(&counters[row_block], 1);
        s_is_last = (arrived == S - 1);
    }
    __syncthreads();
    if (!s_is_last)
        return;
    __threadfence();  // see the other blocks' partial tiles
    if (active) {
        float4_t sum[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            sum[nt] = (float4_t){0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < S; ++s) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (nt * 16 + n_in_tile < N)
                    sum[nt] += partials[(((int64_t)s * n_row_tiles + row_tile) * NT + nt) * 64 + lane];
        }
        finish(sum);
    }
    if (tid == 0)
        counters[row_block] = 0;  // re-arm for the next call on this workspace
}

}  // namespace fp6
