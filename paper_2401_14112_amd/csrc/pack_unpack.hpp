// fp6_quantize_pack and fp6_unpack kernels for gfx950.
//
// quantize_pack: a first launch finds the row maxima and the fp16 scales, a second
// one reads W tile by tile, rounds every weight to its code and writes whole tiles of
// the packed stream with 16-byte stores per lane and plane (the ahead-of-time re-layout
// of the paper's Section 5.2, in this library's order).
//
// unpack: one wave per tile; the same register-level decode as the GEMM, followed by
// the row scale and a single rounding to fp16.
#pragma once
#include "fp6_device.hpp"

namespace fp6 {

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// Magnitude code (0..31) of ratio = |w| / scale on the e3m2 grid, round to nearest,
// ties to the even code, saturating at 28.  The ratio is the correctly rounded fp32
// quotient of two 11-bit significands; it can only land on a grid midpoint when the
// exact quotient is that midpoint, so rounding it equals rounding the exact ratio.
__device__ __forceinline__ uint32_t e3m2_magnitude_code(float ratio)
{
    uint32_t g;
    if (ratio < 0.25f) {
        g = (uint32_t)__builtin_rintf(ratio * 16.0f);  // subnormal binade: multiples of 1/16
    } else {
        uint32_t u = bit_cast<uint32_t>(ratio);
        u += 0x000fffffu + ((u >> 21) & 1u);  // round the mantissa to 2 bits, half to even
        g = (u >> 21) - (124u << 2);          // exponent field - 127 + bias 3, then 2 mantissa bits
    }
    return g < 31u ? g : 31u;
}

// The row scale as the encoder needs it: the scale itself and its reciprocal (0 for a zero scale).
struct RowScale {
    float scale, inv;
};
__device__ __forceinline__ RowScale make_row_scale(float scale)
{
    RowScale r;
    r.scale = scale;
    r.inv = scale == 0.0f ? 0.0f : 1.0f / scale;
    return r;
}

// |w| / scale with one Newton correction on top of the reciprocal product.  When the exact quotient is a
// grid midpoint m (the only case where the last bit matters), q = m(1+e), the fused remainder a - q*scale
// is exact and the corrected value m(1+O(e^2)) rounds to m itself; everywhere else the exact quotient is
// at least 2^-16 (relative) away from every midpoint, far more than the error of q.
template <class Fmt>
__device__ __forceinline__ uint32_t quantize_code(uint32_t w_bits, RowScale rs)
{
    const uint32_t sign = (w_bits >> 15) & 1u;
    const float a = (float)bit_cast<half_t>((uint16_t)(w_bits & 0x7fffu));
    const float q = a * rs.inv;
    const float ratio = __builtin_fmaf(__builtin_fmaf(-q, rs.scale, a), rs.inv, q);
    return (sign << Fmt::kSignShift) | Fmt::magnitude_code(ratio);  // zero scale: inv = 0 -> ratio = 0 -> sign-only code
}

// ---- the two weight formats as the encoder sees them ---------------------------------------------
// magnitude_code(ratio): grid point of |w|/scale (round to nearest, ties to the even code, saturating);
// store_tile(): the lane's codes [run][j] (columns run*32 + 8q + j of its row) -> the lane's bytes of the tile.
struct E3M2Format {
    static constexpr float kMax = 28.0f;
    static constexpr int kSignShift = 5;
    static constexpr int kTileBytes = 3072;
    static constexpr bool kHalfTiles = false;
    __device__ static __forceinline__ uint32_t magnitude_code(float ratio) { return e3m2_magnitude_code(ratio); }
    __device__ static __forceinline__ void store_tile(const uint32_t (&code)[8][8], uint8_t *tile, int lane)
    {
        // two dense streams: code i = 8*(run%4) + j at bits [6i, 6i+6) of stream run/4
        uint32_t d[12];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            uint64_t a[4] = {0, 0, 0, 0};  // 192 bits (+ spill-over slot)
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const uint64_t cd = code[4 * c + i / 8][i % 8];
                const int pos = 6 * i, wd = pos >> 6, sh = pos & 63;
                a[wd] |= cd << sh;
                if (sh > 58)
                    a[wd + 1] |= cd >> (64 - sh);
            }
#pragma unroll
            for (int h = 0; h < 3; ++h) {
                d[6 * c + 2 * h] = (uint32_t)a[h];
                d[6 * c + 2 * h + 1] = (uint32_t)(a[h] >> 32);
            }
        }
        u32x4 *t = reinterpret_cast<u32x4 *>(tile) + lane;
        t[0] = (u32x4){d[0], d[1], d[2], d[3]};
        t[64] = (u32x4){d[4], d[5], d[6], d[7]};
        t[128] = (u32x4){d[8], d[9], d[10], d[11]};
    }
};

// e2m2: grid 0 .25 .5 .75 | 1 .. 1.75 | 2 .. 3.5 | 4 .. 7 (Eq. 1 with bias 1, subnormal E = 0 binade).
struct E2M2Format {
    static constexpr float kMax = 7.0f;
    static constexpr int kSignShift = 4;
    static constexpr int kTileBytes = 2560;
    static constexpr bool kHalfTiles = false;
    __device__ static __forceinline__ uint32_t magnitude_code(float ratio)
    {
        uint32_t g;
        if (ratio < 1.0f) {
            g = (uint32_t)__builtin_rintf(ratio * 4.0f);  // subnormal binade: multiples of 1/4
        } else {
            uint32_t u = bit_cast<uint32_t>(ratio);
            u += 0x000fffffu + ((u >> 21) & 1u);  // round the mantissa to 2 bits, half to even
            g = (u >> 21) - (126u << 2);          // exponent field - 127 + bias 1, then 2 mantissa bits
        }
        return g < 15u ? g : 15u;
    }
    // code s e1 e0 m1 m0 -> byte s 0 0 0 e1 e0 m1 m0
    __device__ static __forceinline__ uint32_t in_place(uint32_t c) { return ((c & 0x10u) << 3) | (c & 0x0fu); }
    __device__ static __forceinline__ void store_tile(const uint32_t (&code)[8][8], uint8_t *tile, int lane)
    {
        uint32_t d[10];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            uint32_t w[5] = {0, 0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 20; ++i)  // in place: byte i%4 of word i/4
                w[i / 4] |= in_place(code[4 * c + i / 8][i % 8]) << (8 * (i % 4));
#pragma unroll
            for (int b = 0; b < 4; ++b) {  // byte lane b of the three spread groups (codes 20+b, 24+b, 28+b)
                const uint32_t c0 = code[4 * c + 2][4 + b], c1 = code[4 * c + 3][b], c2 = code[4 * c + 3][4 + b];
                const int sh = 8 * b;
                // bits of a code: 4 = s, 3 = e1, 2 = e0, 1 = m1, 0 = m0
                w[0] |= ((((c0 >> 4) & 1u) << 6) | (((c0 >> 2) & 3u) << 4)) << sh;                       // s, e1 e0
                w[1] |= (((c0 & 3u) << 5) | (((c1 >> 4) & 1u) << 4)) << sh;                              // m1 m0 | s
                w[2] |= (((c1 >> 1) & 7u) << 4) << sh;                                                   // e1 e0 m1
                w[3] |= (((c1 & 1u) << 6) | (((c2 >> 4) & 1u) << 5) | (((c2 >> 3) & 1u) << 4)) << sh;    // m0 | s | e1
                w[4] |= ((c2 & 7u) << 4) << sh;                                                          // e0 m1 m0
            }
#pragma unroll
            for (int i = 0; i < 5; ++i)
                d[5 * c + i] = w[i];
        }
        u32x4 *t = reinterpret_cast<u32x4 *>(tile) + lane;
        t[0] = (u32x4){d[0], d[1], d[2], d[3]};
        t[64] = (u32x4){d[4], d[5], d[6], d[7]};
        reinterpret_cast<u32x2 *>(tile + 2048)[lane] = (u32x2){d[8], d[9]};
    }
};

// e2m1: grid 0 .5 | 1 1.5 | 2 3 | 4 6 (Eq. 1 with bias 1, subnormal E = 0 binade).
struct E2M1Format {
    static constexpr float kMax = 6.0f;
    static constexpr int kSignShift = 3;
    static constexpr int kTileBytes = 2048;
    static constexpr bool kHalfTiles = false;
    __device__ static __forceinline__ uint32_t magnitude_code(float ratio)
    {
        uint32_t g;
        if (ratio < 1.0f) {
            g = (uint32_t)__builtin_rintf(ratio * 2.0f);  // subnormal binade: multiples of 1/2
        } else {
            uint32_t u = bit_cast<uint32_t>(ratio);
            u += 0x001fffffu + ((u >> 22) & 1u);  // round the mantissa to 1 bit, half to even
            g = (u >> 22) - (126u << 1);          // exponent field - 127 + bias 1, then 1 mantissa bit
        }
        return g < 7u ? g : 7u;
    }
    __device__ static __forceinline__ void store_tile(const uint32_t (&code)[8][8], uint8_t *tile, int lane)
    {
        uint32_t d[8];
#pragma unroll
        for (int run = 0; run < 8; ++run) {
            uint32_t w = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                w |= code[run][j] << (4 * j);
            d[run] = w;
        }
        u32x4 *t = reinterpret_cast<u32x4 *>(tile) + lane;
        t[0] = (u32x4){d[0], d[1], d[2], d[3]};
        t[64] = (u32x4){d[4], d[5], d[6], d[7]};
    }
};

// e2m0: grid 0 | 1 | 2 | 4 (Eq. 1 with bias 1 and no mantissa bits; the E = 0 binade holds only 0).
struct E2M0Format {
    static constexpr float kMax = 4.0f;
    static constexpr int kSignShift = 2;
    static constexpr int kTileBytes = 3072;       // 16 rows x 512 columns: k-tile kt (256 columns) is half kt % 2 of tile kt / 2
    static constexpr bool kHalfTiles = true;
    __device__ static __forceinline__ uint32_t magnitude_code(float ratio)
    {
        uint32_t g;
        if (ratio < 1.0f) {
            g = (uint32_t)__builtin_rintf(ratio);  // 0 or 1, the midpoint 0.5 to the even code 0
        } else {
            uint32_t u = bit_cast<uint32_t>(ratio);
            u += 0x003fffffu + ((u >> 23) & 1u);  // round the mantissa away entirely, half to the even exponent code
            g = (u >> 23) - 126u;                 // exponent field - 127 + bias 1
        }
        return g < 3u ? g : 3u;
    }
    // the lane's bytes of one half of a tile: 16 in plane 0 (first half) or 2 (second half), 8 in the middle
    // plane; pad_other: the matrix ends with this half (K an odd multiple of 256) and the lane also writes the
    // zero padding of the other half
    __device__ static __forceinline__ void store_half(const uint32_t (&code)[8][8], uint8_t *tile, int half, bool pad_other,
                                                      int lane)
    {
        uint32_t d[6];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            uint32_t w[3] = {0, 0, 0};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    w[i] |= (code[4 * g + i][j] << 1) << (4 * j);  // in place: field "s e1 e0 ."
                const uint32_t c = code[4 * g + 3][j];             // spread over the free bits
#pragma unroll
                for (int b = 0; b < 3; ++b)
                    w[b] |= ((c >> b) & 1u) << (4 * j);
            }
#pragma unroll
            for (int i = 0; i < 3; ++i)
                d[3 * g + i] = w[i];
        }
        *(reinterpret_cast<u32x4 *>(tile + half * 2048) + lane) = (u32x4){d[0], d[1], d[2], d[3]};
        *(reinterpret_cast<u32x2 *>(tile + 1024) + 2 * lane + half) = (u32x2){d[4], d[5]};
        if (pad_other) {
            *(reinterpret_cast<u32x4 *>(tile + (half ^ 1) * 2048) + lane) = (u32x4){0, 0, 0, 0};
            *(reinterpret_cast<u32x2 *>(tile + 1024) + 2 * lane + (half ^ 1)) = (u32x2){0, 0};
        }
    }
};

// The lane's bytes of k-tile kt (256 columns) of row tile `row_tile` into the packed stream (tiles stored
// k-tile major; RT row tiles, KT k-tiles of 256 columns).
template <class Fmt, class = void>
struct KTileStore {
    __device__ static __forceinline__ void store(const uint32_t (&code)[8][8], uint8_t *packed, int64_t kt, int64_t row_tile,
                                                 int64_t RT, int /*KT*/, int lane)
    {
        Fmt::store_tile(code, packed + (kt * RT + row_tile) * Fmt::kTileBytes, lane);
    }
};
template <class Fmt>
struct KTileStore<Fmt, std::enable_if_t<Fmt::kHalfTiles>> {
    __device__ static __forceinline__ void store(const uint32_t (&code)[8][8], uint8_t *packed, int64_t kt, int64_t row_tile,
                                                 int64_t RT, int KT, int lane)
    {
        Fmt::store_half(code, packed + ((kt >> 1) * RT + row_tile) * Fmt::kTileBytes, (int)(kt & 1),
                        (kt & 1) == 0 && kt == KT - 1, lane);
    }
};

// ---- per-row scales: two launches ------------------------------------------------------------------
// row_scale_kernel: one wave per row finds max |W| and writes scale = fp16(max / Fmt::kMax) (a plain read of
// W at streaming rate).  quantize_tiles_kernel: one wave per 16 x 256 tile reads the tile once, rounds every
// weight with its row's scale and writes the packed tile.  The scales array is the only thing that passes
// between the two, so nothing is kept on chip across a row (a row of 22016 fp16 values is 44 KB and a row
// tile 0.7 MB - more than a CU can hold); W is read twice from memory and that is the algorithmic minimum
// for a per-row maximum unless rows fit on chip.
constexpr int kScaleWavesPerBlock = 4;

template <class Fmt>
__global__ __launch_bounds__(kScaleWavesPerBlock * 64) void row_scale_kernel(const half_t *__restrict__ W, int M, int K,
                                                                              half_t *__restrict__ scales)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = blockIdx.x * kScaleWavesPerBlock + wave;
    if (m >= M)
        return;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(W + (int64_t)m * K);
    const int n16 = K / 8;  // 16-byte pieces of the row (K % 256 == 0, so n16 % 32 == 0)
    ushort2_t mx = {0, 0};
    int i = lane;
    for (; i + 448 < n16; i += 512) {  // eight independent loads in flight
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = __builtin_nontemporal_load(row + i + 64 * u);
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                mx = __builtin_elementwise_max(mx, bit_cast<ushort2_t>(v[u][j] & 0x7fff7fffu));
    }
    for (; i < n16; i += 64) {
        const u32x4 v = row[i];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            mx = __builtin_elementwise_max(mx, bit_cast<ushort2_t>(v[j] & 0x7fff7fffu));
    }
    uint32_t amax = mx[0] > mx[1] ? mx[0] : mx[1];  // finite fp16 magnitudes order like integers
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t other = __shfl_xor(amax, off, 64);
        amax = other > amax ? other : amax;
    }
    if (lane == 0)
        scales[m] = (half_t)((float)bit_cast<half_t>((uint16_t)amax) / Fmt::kMax);  // fp32 quotient, one rounding
}

template <class Fmt>
__global__ __launch_bounds__(256) void quantize_tiles_kernel(const half_t *__restrict__ W, int M, int K,
                                                             uint8_t *__restrict__ packed,
                                                             const half_t *__restrict__ scales)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int KT = K / kTileK;
    const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
    if (tile >= (int64_t)(M / kTileRows) * KT)
        return;
    // the waves of a block take neighbouring k-tiles of one row tile (2 KB of every row of W between them);
    // in the packed stream tiles are stored k-tile major
    const int64_t RT = M / kTileRows, row_tile = tile / KT, kt = tile % KT;
    const int r = lane & 15, q = lane >> 4;  // lane (r, q) builds its bytes of the tile
    const half_t *row = W + (row_tile * kTileRows + r) * K + kt * kTileK + q * 8;
    u32x4 v[8];
#pragma unroll
    for (int f = 0; f < 8; ++f)
        v[f] = *reinterpret_cast<const u32x4 *>(row + f * 32);
    const RowScale scale = make_row_scale((float)scales[row_tile * kTileRows + r]);
    uint32_t code[8][8];
#pragma unroll
    for (int f = 0; f < 8; ++f)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            code[f][2 * j] = quantize_code<Fmt>(v[f][j] & 0xffffu, scale);
            code[f][2 * j + 1] = quantize_code<Fmt>(v[f][j] >> 16, scale);
        }
    KTileStore<Fmt>::store(code, packed, kt, row_tile, RT, KT, lane);
}

// Group-wise scales (one per row and per 128 columns): a group lies inside one tile and inside one of a
// lane's two streams, so row maxima need only a reduction over the four lanes (q = 0..3) that share a row:
// one pass over W, one wave per tile.  scales: fp16 [M][K/128].
__global__ __launch_bounds__(256) void quantize_pack_group_kernel(const half_t *__restrict__ W, int M, int K,
                                                                  uint8_t *__restrict__ packed,
                                                                  half_t *__restrict__ scales)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int KT = K / kTileK;
    const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
    if (tile >= (int64_t)(M / kTileRows) * KT)
        return;
    // the waves of a block take neighbouring k-tiles of one row tile (2 KB of every row of W between them);
    // in the packed stream tiles are stored k-tile major
    const int64_t RT = M / kTileRows, row_tile = tile / KT, kt = tile % KT, packed_tile = kt * RT + row_tile;
    const int r = lane & 15, q = lane >> 4;
    const half_t *row = W + (row_tile * kTileRows + r) * K + kt * kTileK + q * 8;
    u32x4 v[8];
#pragma unroll
    for (int f = 0; f < 8; ++f)
        v[f] = *reinterpret_cast<const u32x4 *>(row + f * 32);
    uint32_t code[8][8];
    uint32_t scale_bits[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        ushort2_t mx = {0, 0};
#pragma unroll
        for (int f = 4 * c; f < 4 * c + 4; ++f)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                mx = __builtin_elementwise_max(mx, bit_cast<ushort2_t>(v[f][j] & 0x7fff7fffu));
        uint32_t amax = mx[0] > mx[1] ? mx[0] : mx[1];  // finite fp16 magnitudes order like integers
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {        // the four lanes of a row
            const uint32_t other = __shfl_xor(amax, off, 64);
            amax = other > amax ? other : amax;
        }
        const half_t sc = (half_t)((float)bit_cast<half_t>((uint16_t)amax) / E3M2Format::kMax);
        scale_bits[c] = bit_cast<uint16_t>(sc);
        const RowScale scale = make_row_scale((float)sc);
#pragma unroll
        for (int f = 4 * c; f < 4 * c + 4; ++f)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                code[f][2 * j] = quantize_code<E3M2Format>(v[f][j] & 0xffffu, scale);
                code[f][2 * j + 1] = quantize_code<E3M2Format>(v[f][j] >> 16, scale);
            }
    }
    E3M2Format::store_tile(code, packed + packed_tile * E3M2Format::kTileBytes, lane);
    if (q == 0) {
        const int64_t groups = K / kGroupColumns;
        *reinterpret_cast<uint32_t *>(scales + (row_tile * kTileRows + r) * groups + 2 * kt) = scale_bits[0] | (scale_bits[1] << 16);
    }
}

template <class Src>
__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t *__restrict__ packed,
                                                     const half_t *__restrict__ scales, int M, int K,
                                                     half_t *__restrict__ W_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int KT = K / kTileK;
    const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
    if (tile >= (int64_t)(M / kTileRows) * KT)
        return;
    // the waves of a block take neighbouring k-tiles of one row tile (2 KB of every row of W between them);
    // in the packed stream tiles are stored k-tile major
    const int64_t RT = M / kTileRows, row_tile = tile / KT, kt = tile % KT;
    const int r = lane & 15, q = lane >> 4;
    typename Src::Stream stream;
    stream.init(packed, scales, row_tile, (int)kt, 1, 1, RT, K, lane);
    typename Src::Tile t;
    stream.issue(t, 0);
    wait_loads<0>();
    Src::pin_tile(t);
    const float scale = Src::kHasScale ? (float)scales[row_tile * kTileRows + r] : 1.0f;  // else already applied
    half_t *out = W_out + (row_tile * kTileRows + r) * K + kt * kTileK + q * 8;
    half8_t frag[8];
    Src::template fragments<0>(t, frag[0], frag[1]);
    Src::template fragments<1>(t, frag[2], frag[3]);
    Src::template fragments<2>(t, frag[4], frag[5]);
    Src::template fragments<3>(t, frag[6], frag[7]);
#pragma unroll
    for (int f = 0; f < 8; ++f) {
        half8_t y;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            y[j] = (half_t)((float)frag[f][j] * scale);  // exact product in fp32, one rounding
        *reinterpret_cast<half8_t *>(out + f * 32) = y;
    }
}

// ---- diagnostics: empirical ceilings of the device, with the request patterns of the linear kernels ------
// probe_read_kernel: the buffer is cut into pieces of 8 KB; in step s wave w of the W waves reads piece
// s * W + w, so that the grid sweeps the buffer front to back (the way the linear kernels sweep packed
// weights; one contiguous range per wave is 10 % slower), with the non-temporal 128-bit loads of the weight
// path, sixteen in flight per wave (two sets of eight).  Nothing is computed except the XOR of what was loaded.
__global__ __launch_bounds__(256) void probe_read_kernel(const uint8_t *__restrict__ buffer, size_t bytes,
                                                         uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * 4 + (size_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const size_t n_waves = (size_t)gridDim.x * 4;
    const size_t steps = bytes / (n_waves * 8192) / 2 * 2;  // whole double steps; the host sizes the grid for >= 2
    u32x4 a[8], b[8];
    auto issue8 = [&](u32x4 (&v)[8], size_t step) {
        // a step past the end gets an empty range: its loads return zeros and fetch nothing
        const rsrc_t r = make_rsrc(buffer + (step < steps ? step * n_waves + wave : 0) * 8192, step < steps ? 8192u : 0u);
        const int off = lane * 16;
        v[0] = issue_load_b128<0, true>(r, off);
        v[1] = issue_load_b128<1024, true>(r, off);
        v[2] = issue_load_b128<2048, true>(r, off);
        v[3] = issue_load_b128<3072, true>(r, off);
        v[4] = issue_load_b128<0, true>(r, off + 4096);  // the immediate offset is a 12-bit field
        v[5] = issue_load_b128<1024, true>(r, off + 4096);
        v[6] = issue_load_b128<2048, true>(r, off + 4096);
        v[7] = issue_load_b128<3072, true>(r, off + 4096);
    };
    u32x4 x = {0u, 0u, 0u, 0u};  // running XOR of everything loaded: the data is touched, and checkable
    auto pin8 = [&](u32x4 (&v)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            pin(v[i]);
            x ^= v[i];
        }
        pin(x);  // the set is consumed here, before its registers are the target of the next loads
    };
    issue8(a, 0);
    for (size_t s = 0; s < steps; s += 2) {
        issue8(b, s + 1);
        wait_loads<8>();
        pin8(a);
        issue8(a, s + 2);
        wait_loads<8>();
        pin8(b);
    }
    wait_loads<0>();
    pin8(a);  // the look-ahead past the last step: zeros
    uint32_t w = x[0] ^ x[1] ^ x[2] ^ x[3];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1)
        w ^= (uint32_t)__shfl_xor((int)w, m, 64);
    if (lane == 0)
        sink[wave] = w;  // XOR of all 32-bit words of the wave's pieces
}

// probe_mfma_kernel: every wave issues iters x 4 independent v_mfma_f32_32x32x16_f16 on register operands.
typedef float float16_t __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float *__restrict__ sink)
{
    const half_t one = (half_t)1.0f, tiny = (half_t)0.0009765625f;
    half8_t a = {one, tiny, one, tiny, one, tiny, one, tiny}, b = {tiny, one, tiny, one, tiny, one, tiny, one};
    float16_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            acc[i][j] = (float)(i + j);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            s += acc[i][j];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ void zero_fill_kernel(u32x4 *p, size_t n16)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n16)
        p[i] = (u32x4){0u, 0u, 0u, 0u};
}

}  // namespace fp6
