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

    extern __shared__ u32x4 xs_dyn[];  // [2][XCHUNKS]
    u32x4(*xs)[XCHUNKS] = reinterpret_cast<u32x4(*)[XCHUNKS]>(xs_dyn);
    __shared__ int s_is_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KT = K / kTileK;
    const int n_row_tiles = M / kTileRows;
    const int split = blockIdx.x % S;  // neighbouring blocks (one per XCD) take different k slices
    const int row_block = blockIdx.x / S;
    const int row_tile = row_block * WAVES + wave;
    const bool active = row_tile < n_row_tiles;
    const int kt0 = (int)(((unsigned)KT * (unsigned)split) / (unsigned)S);  // KT * S < 2^31 (host-checked)
    const int kt1 = (int)(((unsigned)KT * (unsigned)(split + 1)) / (unsigned)S);
    const int n_valid = kt1 - kt0;        // k-tiles of this slice
    const int T = (KT + S - 1) / S;       // loop trips: the same for every slice (>= n_valid)

    // Inactive waves (ragged last row block) stream the last valid row tile and drop the result,
    // so the main loop has no per-wave control flow.
    const rsrc_t w_rsrc = Src::slice_rsrc(weights, active ? row_tile : n_row_tiles - 1, kt0, kt1, KT, K);
    const rsrc_t x_rsrc = make_rsrc(X, (uint32_t)N * (uint32_t)K * 2u);

    // ---- activation staging: piece c = nt*512 + f*64 + p holds X[nt*16+n][k_tile*256 + k_offset(f,q) ..+8]
    // for the (n, q) given by x_source_of_piece(p).  Token columns >= N and k-tiles past the slice get an
    // offset outside the buffer and read as zeros.
    struct XRegs {
        u32x4 v[XPER];
    };
    int x_off[XPER];
#pragma unroll
    for (int i = 0; i < XPER; ++i) {
        const int c = tid + i * THREADS;
        const int f = (c >> 6) & 7, nt = c >> 9;
        int n, q;
        x_source_of_piece(c & 63, n, q);
        const int col = nt * 16 + n;
        x_off[i] = col < N ? (col * K + kt0 * kTileK + Src::k_offset(f, q)) * 2 : kOutOfRange;
    }
    auto x_issue = [&](XRegs &r, int t) {
#pragma unroll
        for (int i = 0; i < XPER; ++i) {
            const int off = (t < n_valid && x_off[i] != kOutOfRange) ? x_off[i] + t * (kTileK * 2) : kOutOfRange;
            r.v[i] = issue_load_b128<0, false>(x_rsrc, off);
        }
    };
    auto x_pin = [&](XRegs &r) {
#pragma unroll
        for (int i = 0; i < XPER; ++i)
            pin(r.v[i]);
    };
    auto x_commit = [&](const XRegs &r, int buf) {
#pragma unroll
        for (int i = 0; i < XPER; ++i)
            xs[buf][tid + i * THREADS] = r.v[i];
    };

    const int b_piece = x_piece_of_lane(lane);
    float4_t acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        acc[nt] = (float4_t){0.f, 0.f, 0.f, 0.f};

    auto mma_pair = [&](const half8_t &a_even, const half8_t &a_odd, int buf, int g) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            half8_t b = bit_cast<half8_t>(xs[buf][nt * 512 + (2 * g) * 64 + b_piece]);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_even, b, acc[nt], 0, 0, 0);
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            half8_t b = bit_cast<half8_t>(xs[buf][nt * 512 + (2 * g + 1) * 64 + b_piece]);
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

    // ---- software pipeline.  Slot d of the register ring holds tile i*DEPTH + d of the slice: its
    // weights and its share of the activation tile are requested DEPTH tiles ahead, right after the
    // slot's previous tile has been consumed, so the new data lands in the registers that just became
    // free and DEPTH-1 tiles stay in flight while one is being computed.  Every slot issues
    // kSlotLoads loads; loads return in order, so "at most (DEPTH-1)*kSlotLoads outstanding" means the
    // oldest slot has arrived.  The loop body has no branches: tiles past the end of the slice read
    // as zeros through the buffer bounds check.
    static_assert(DEPTH % 2 == 0, "the LDS double buffer is indexed by the ring slot");
    constexpr int kSlotLoads = XPER + Src::kLoads;
    typename Src::Tile w[DEPTH];
    XRegs xr[DEPTH];
    const int w_off = Src::lane_offset(lane, kt0, K);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        x_issue(xr[d], d);
        Src::issue(w[d], w_rsrc, w_off + d * Src::kTileStride);
    }
    for (int i = 0; i < T; i += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            wait_loads<(DEPTH - 1) * kSlotLoads>();
            x_pin(xr[d]);
            Src::pin_tile(w[d]);
            x_commit(xr[d], d & 1);
            __syncthreads();
            compute(w[d], d & 1);
            x_issue(xr[d], i + d + DEPTH);
            Src::issue(w[d], w_rsrc, w_off + (i + d + DEPTH) * Src::kTileStride);
        }
    }
    // drain: the look-ahead loads of the last DEPTH tiles (all out of range, zeros) must land before
    // their registers are reused
    wait_loads<0>();
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        x_pin(xr[d]);
        Src::pin_tile(w[d]);
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

#ifndef FP6_SPLITK_SYNC
#define FP6_SPLITK_SYNC 1
#endif
#if FP6_SPLITK_SYNC == 0
    // Release/acquire fences at device scope (write back and invalidate this XCD's L2).
    if (active) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (nt * 16 + n_in_tile < N)
                partials[(((int64_t)split * n_row_tiles + row_tile) * NT + nt) * 64 + lane] = acc[nt];
    }
    __syncthreads();  // every wave's partial stores have been issued and have completed
    if (tid == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        const int arrived = __hip_atomic_fetch_add(&counters[row_block], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_is_last = (arrived == S - 1);
    }
    __syncthreads();
    if (!s_is_last)
        return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
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
#else
    // The partial tiles are written and read with device-scope atomic (relaxed) accesses: such
    // accesses are performed at the point where all CUs of the device agree (they are not left
    // in, nor served from, a non-coherent cache), so no cache write-back or invalidate is needed.
    // Order: stores complete (the barrier waits for them) -> arrival count -> the last block's loads.
    float *pf = reinterpret_cast<float *>(partials);
    if (active) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (nt * 16 + n_in_tile < N) {
                float *dst = pf + ((((int64_t)split * n_row_tiles + row_tile) * NT + nt) * 4) * 64 + lane;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    __hip_atomic_store(dst + i * 64, acc[nt][i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's partial stores are done
    __syncthreads();
    if (tid == 0) {
        const int arrived = __hip_atomic_fetch_add(&counters[row_block], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_is_last = (arrived == S - 1);
    }
    __syncthreads();
    if (!s_is_last)
        return;
    if (active) {
        float4_t sum[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            sum[nt] = (float4_t){0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < S; ++s) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (nt * 16 + n_in_tile < N) {
                    const float *src = pf + ((((int64_t)s * n_row_tiles + row_tile) * NT + nt) * 4) * 64 + lane;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        sum[nt][i] += __hip_atomic_load(src + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
        }
        finish(sum);
    }
#endif
    if (tid == 0)
        counters[row_block] = 0;  // re-arm for the next call on this workspace
}

}  // namespace fp6
