// Bench-only build of the W6A16 kernels with the de-quantization of Section 5.3 of the paper in place of the
// chip's e3m2 -> fp16 conversion instruction: the head-to-head behind the library's choice of the conversion
// instruction for its one 6-bit path.  Nothing here is part of the library or of its boundary.
//
// The shift/mask variant needs a bit arrangement that word-parallel SIMT code can take apart, in the spirit of
// the paper's ahead-of-time bit-level pre-packing (Section 5.2).  Same tiles as the library (16 x 256 codes =
// three planes of 16 bytes per lane, k-tile major, lane (q, r) = row r, columns 8q..8q+7 of every run of 32),
// but inside a lane word g (0..3) of the three planes D0, D1, D2 holds the 16 codes of runs 2g and 2g+1:
// twelve sit in place as bytes "s..EEEMM" - bit 7 the sign, bits 4..0 exponent and mantissa, which is the top
// byte of the fp16 that Eq. 3 asks for - and the other four are spread over the free bits 6, 5 of those twelve
// bytes.  Unpack per 16 codes: 3 ANDs, a 4-term stitch, 8 byte permutes, 8 packed multiplies by 2^12 (Eq. 3).
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>

#include "paper_2401_14112_amd/csrc/fp6_device.hpp"
#include "paper_2401_14112_amd/csrc/linear_stream.hpp"
#include "paper_2401_14112_amd/csrc/linear_tiled.hpp"

namespace fp6 {

// two fp16 bit patterns "s00EEEMM 00000000" -> values (Eq. 3: the exponent field was copied without re-biasing,
// so the value is off by 2^(15-3); one packed multiply fixes both halves, subnormals included)
__device__ __forceinline__ uint32_t a6_rebias_pair(uint32_t pair)
{
    const half2_t h = bit_cast<half2_t>(pair) * (half2_t){(half_t)4096.0f, (half_t)4096.0f};
    return bit_cast<uint32_t>(h);
}

__device__ __forceinline__ void a6_bytes_to_halves(uint32_t b, uint32_t &lo, uint32_t &hi)
{
    lo = a6_rebias_pair(__builtin_amdgcn_perm(0u, b, 0x010c000cu));  // [b1 0 b0 0]
    hi = a6_rebias_pair(__builtin_amdgcn_perm(0u, b, 0x030c020cu));  // [b3 0 b2 0]
}

struct ShiftMaskFp6Source {
    typedef SimpleStream<ShiftMaskFp6Source> Stream;
    static constexpr bool kPackedConfigs = true;
    typedef PackedFp6Source::Tile Tile;
    static constexpr bool kHasScale = true;
    static constexpr int kLdsTileBytes = 0;
    static constexpr int kTileCols = kTileK;
    static constexpr bool kTallTile = true;
    static constexpr int kLoads = 3;
    __device__ static __forceinline__ int tile_stride(int64_t RT) { return PackedFp6Source::tile_stride(RT); }
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    __device__ static __forceinline__ rsrc_t slice_rsrc(const void *base, int64_t row_tile, int kt_first, int kt_step,
                                                        int n_tiles, int64_t RT, int64_t K)
    {
        return PackedFp6Source::slice_rsrc(base, row_tile, kt_first, kt_step, n_tiles, RT, K);
    }
    __device__ static __forceinline__ int lane_offset(int lane, int, int) { return lane * 16; }
    __device__ static __forceinline__ void issue(Tile &t, rsrc_t r, int off) { PackedFp6Source::issue(t, r, off); }
    __device__ static __forceinline__ void pin_tile(Tile &t) { PackedFp6Source::pin_tile(t); }
    // word G of the three planes -> the A fragments of runs 2G (even) and 2G+1 (odd)
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        const uint32_t d0 = t.p0[G], d1 = t.p1[G], d2 = t.p2[G];
        const uint32_t b0 = d0 & 0x9f9f9f9fu, b1 = d1 & 0x9f9f9f9fu, b2 = d2 & 0x9f9f9f9fu;
        uint32_t b3 = (d0 >> 5) & 0x03030303u;   // m1 m0 of the four spread codes
        b3 = ((d1 >> 3) & 0x0c0c0c0cu) | b3;     // e1 e0
        b3 = ((d2 << 1) & 0x80808080u) | b3;     // s
        b3 = ((d2 >> 1) & 0x10101010u) | b3;     // e2
        uint32_t h[8];
        a6_bytes_to_halves(b0, h[0], h[1]);
        a6_bytes_to_halves(b1, h[2], h[3]);
        a6_bytes_to_halves(b2, h[4], h[5]);
        a6_bytes_to_halves(b3, h[6], h[7]);
        even_run = bit_cast<half8_t>((u32x4){h[0], h[1], h[2], h[3]});
        odd_run = bit_cast<half8_t>((u32x4){h[4], h[5], h[6], h[7]});
    }
};

// The library's packed stream -> the arrangement above, one lane's 48 bytes at a time (same tile order).
__global__ void a6_repack_kernel(const uint32_t *__restrict__ in, uint32_t *__restrict__ out, size_t n_tiles)
{
    const size_t lane_slot = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // (tile, lane)
    if (lane_slot >= n_tiles * 64)
        return;
    const size_t tile = lane_slot / 64, lane = lane_slot % 64;
    const uint32_t *src = in + tile * 768 + lane * 4;
    uint32_t w[12];  // plane-major: the lane's two dense streams of 32 codes
    for (int p = 0; p < 3; ++p)
        for (int i = 0; i < 4; ++i)
            w[p * 4 + i] = src[p * 256 + i];
    uint8_t code[64];  // code[8 * run + j]
    for (int s = 0; s < 2; ++s)
        for (int i = 0; i < 32; ++i) {
            const int bit = 6 * i, word = 6 * s + bit / 32, sh = bit % 32;
            uint32_t v = w[word] >> sh;
            if (sh > 26)
                v |= w[word + 1] << (32 - sh);
            code[32 * s + i] = (uint8_t)(v & 63u);
        }
    uint32_t d[3][4];
    for (int g = 0; g < 4; ++g) {
        uint32_t d0 = 0, d1 = 0, d2 = 0;
        for (int k = 0; k < 4; ++k) {
            const uint32_t in0 = code[16 * g + k], in1 = code[16 * g + 4 + k], in2 = code[16 * g + 8 + k];
            const uint32_t sp = code[16 * g + 12 + k];  // the spread code: s e2 e1 e0 m1 m0
            const uint32_t byte0 = ((in0 & 32u) << 2) | (in0 & 31u) | ((sp & 3u) << 5);
            const uint32_t byte1 = ((in1 & 32u) << 2) | (in1 & 31u) | (((sp >> 2) & 3u) << 5);
            const uint32_t byte2 = ((in2 & 32u) << 2) | (in2 & 31u) | (((sp >> 5) & 1u) << 6) | (((sp >> 4) & 1u) << 5);
            d0 |= byte0 << (8 * k);
            d1 |= byte1 << (8 * k);
            d2 |= byte2 << (8 * k);
        }
        d[0][g] = d0;
        d[1][g] = d1;
        d[2][g] = d2;
    }
    uint32_t *dst = out + tile * 768 + lane * 4;
    for (int p = 0; p < 3; ++p)
        for (int i = 0; i < 4; ++i)
            dst[p * 256 + i] = d[p][i];
}

}  // namespace fp6

using namespace fp6;

namespace {

template <class Src, class Shape>
int launch_stream(const void *w, const void *sc, const void *X, void *Y, int64_t M, int64_t N, int64_t K, void *ws,
                  hipStream_t st)
{
    auto kernel = linear_stream_kernel<Src, Shape>;
    static bool done = false;
    if (!done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                Shape::template lds_bytes<Src>()) != hipSuccess)
            return 5;
        done = true;
    }
    const int64_t row_tiles = M / 16, rb = (row_tiles + Shape::WAVES - 1) / Shape::WAVES;
    int64_t S = 256 / rb;
    if (S < 1)
        S = 1;
    if (S > K / 512)
        S = K / 512;
    int *counters = static_cast<int *>(ws);
    float4_t *partials = reinterpret_cast<float4_t *>(static_cast<char *>(ws) + 65536);
    hipLaunchKernelGGL(kernel, dim3((unsigned)rb, (unsigned)S), dim3(Shape::kThreads), Shape::template lds_bytes<Src>(), st, w,
                       static_cast<const half_t *>(sc), static_cast<const half_t *>(X), static_cast<half_t *>(Y), (int)M,
                       (int)N, (int)K, (int)S, (int)(K / 256 / S), partials, counters, Epilogue{nullptr, nullptr, 0});
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

template <class Src>
int launch_tiled(const void *w, const void *sc, const void *X, void *Y, int64_t M, int64_t N, int64_t K, void *ws,
                 hipStream_t st)
{
    constexpr int RT = 2, NT = 8, WM = 8, WN = 1;
    auto kernel = linear_tiled_kernel<Src, RT, NT, WM, WN>;
    const size_t lds = (size_t)4 * NT * WN * 256 * 16;
    static bool done = false;
    if (!done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return 5;
        done = true;
    }
    const int rb = (int)((M + 255) / 256), nb = (int)((N + 127) / 128);
    int S = 256 / (rb * nb);
    if (S < 1)
        S = 1;
    if (S > 16)
        S = 16;
    int *counters = static_cast<int *>(ws);
    float4_t *partials = reinterpret_cast<float4_t *>(static_cast<char *>(ws) + 65536);
    hipLaunchKernelGGL(kernel, dim3((unsigned)((rb + 7) / 8 * 8 * nb * S)), dim3(WM * WN * 64), lds, st, w,
                       static_cast<const half_t *>(sc), static_cast<const half_t *>(X), static_cast<half_t *>(Y), (int)M,
                       (int)N, (int)K, S, nb, partials, counters, Epilogue{nullptr, nullptr, 0});
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

template <class Src>
int launch(const void *w, const void *sc, const void *X, void *Y, int64_t M, int64_t N, int64_t K, void *ws, hipStream_t st)
{
    if (N <= 16)
        return launch_stream<Src, StreamShape<1, 8, 2, 1, 1, true>>(w, sc, X, Y, M, N, K, ws, st);
    if (N <= 32)
        return launch_stream<Src, StreamShape<2, 8, 2, 1, 1, true>>(w, sc, X, Y, M, N, K, ws, st);
    if (N <= 64)
        return launch_stream<Src, StreamShape<4, 8, 2, 1, 1, true>>(w, sc, X, Y, M, N, K, ws, st);
    return launch_tiled<Src>(w, sc, X, Y, M, N, K, ws, st);
}

}  // namespace

extern "C" {

// bytes of workspace (zero-filled by the caller) that either variant needs: counters in the first 64 KB
size_t a6_workspace_bytes(int64_t M, int64_t N) { return 65536 + (size_t)16 * (size_t)M * (size_t)((N + 15) / 16 * 16) * 4; }

int a6_repack(const void *packed, void *out, int64_t M, int64_t K, void *stream)
{
    const size_t n_tiles = (size_t)(M / 16) * (size_t)(K / 256);
    hipLaunchKernelGGL(a6_repack_kernel, dim3((unsigned)((n_tiles * 64 + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint32_t *>(packed), static_cast<uint32_t *>(out),
                       n_tiles);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

// variant 0: the library's source (conversion instruction) on the library's stream; 1: shift/mask on the repacked one
int a6_linear(int variant, const void *packed, const void *scales, const void *X, void *Y, int64_t M, int64_t N, int64_t K,
              void *workspace, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    return variant == 0 ? launch<PackedFp6Source>(packed, scales, X, Y, M, N, K, workspace, st)
                        : launch<ShiftMaskFp6Source>(packed, scales, X, Y, M, N, K, workspace, st);
}

}  // extern "C"
