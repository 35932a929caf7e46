// Device-side building blocks shared by the gfx950 kernels: the packed tile layout,
// the register-level e3m2 -> fp16 de-quantization, and the two weight sources (packed
// 6-bit and plain fp16) that the linear-layer kernels are instantiated with.
//
// Packed layout, version 3 (this library's own; the paper's Section 5.2 only asks that
// the weights be reordered ahead of time so that each thread reads whole aligned words in
// the order the matrix cores consume them):
//   * the M x K code matrix is cut into tiles of 16 rows x 256 columns, 3072 bytes
//     each, stored k-tile major (tile (row tile r, k-tile t) is tile number t * M/16 + r): the
//     waves of a launch work on different row tiles at about the same depth t, so together
//     they sweep memory front to back instead of each following a stream of its own (a
//     read-only stream over a buffer of the benchmark layer's size takes 20.3 us swept this
//     way against 22.9 us with one contiguous piece per wave);
//   * a tile is three planes of 1024 bytes; lane L of a 64-wide wave owns bytes
//     [16L, 16L+16) of each plane = three 128-bit loads, each a contiguous 1 KB per
//     wave;
//   * lane L = 16*q + r holds row r of the tile and, of every run of 32 columns,
//     columns 8q..8q+7 - exactly the A operand of v_mfma_f32_16x16x32_f16;
//   * the lane's 12 words (plane-major) are two dense 192-bit streams: words 0..5 hold
//     the 32 codes of runs 0..3, words 6..11 those of runs 4..7; code i = 8*(run%4) + j
//     (column run*32 + 8q + j) occupies bits [6i, 6i+6) of its stream.
//
// De-quantization.  The paper (Section 5.3) builds fp16 values from 6-bit codes with SIMT
// shifts, masks and an exponent-bias multiply because its GPUs have no FP6 hardware.
// CDNA4 has: the e3m2 format of the paper is the "BF6" element type of the OCP
// microscaling formats, and v_cvt_scalef32_pk32_f16_bf6 turns a dense stream of 32 such
// codes (6 registers) into 32 fp16 values (16 registers) exactly - subnormal binade,
// signed zero and the 16..28 binade included - in one instruction.  A stream above is
// laid out so that the 32 results are, in order, the lane's A fragments of four
// consecutive MFMA steps.  (Layout version 1 kept 12 of 16 codes byte-aligned and
// re-assembled values with 27 VALU instructions per 16 weights; the conversion
// instruction made the kernels 4-7 % faster at every N and needs no layout tricks.)
#pragma once
#include <type_traits>
#include <utility>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp6 {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTileRows = 16;
constexpr int kTileK = 256;
constexpr int kTileBytes = 3072;
constexpr int kRunsPerTile = 8;  // runs of 32 columns = MFMA k-steps per tile

template <class To, class From>
__device__ __forceinline__ To bit_cast(const From &v)
{
    return __builtin_bit_cast(To, v);
}

typedef _Float16 half32_t __attribute__((ext_vector_type(32)));
typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));

// One dense stream of 32 e3m2 codes -> 32 fp16 values, exact (scale operand 1.0 = 2^0).
__device__ __forceinline__ half32_t dequant_stream(u32x6 codes)
{
    return __builtin_amdgcn_cvt_scalef32_pk32_f16_bf6(codes, 1.0f);
}

// ---- bounds-checked buffer loads -------------------------------------------
// A buffer resource lets the hardware range-check every load: an offset at or beyond
// num_bytes returns zeros and generates no memory traffic.  The streaming kernels use
// this so that their main loop has no branches (a tile past the end of a wave's slice
// simply reads as zero weights).  All four words must be wave-uniform.  Only the
// per-lane offset (plus the instruction's immediate) takes part in the range check,
// so every varying part of an address is put there and the scalar offset stays 0.
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef i32x4 rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t num_bytes)
{
    const uint64_t a = reinterpret_cast<uint64_t>(base);
    rsrc_t r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((a >> 32) & 0xffffu));  // stride 0: raw buffer
    r[2] = __builtin_amdgcn_readfirstlane((int)num_bytes);
    r[3] = 0x00020000;  // 32-bit data format, no swizzle
    return r;
}

constexpr int kPartialBatch = 4;  // split-K: partial tiles of this many k slices are fetched per trip to memory
constexpr int kOutOfRange = (int)0x80000000u;  // a lane offset no buffer here reaches: reads as zeros

// The pipelined kernels issue their loads from inline assembly and wait for them with explicit
// s_waitcnt: the compiler's own wait insertion cannot keep several tiles in flight across a loop
// back edge.  Rules that keep this sound: (1) a loaded value is only used after wait_loads<N>()
// followed by pin() on it, which orders the use after the wait; (2) every issued load is waited
// for (and pinned) before its registers die, so no late write lands in a reused register.  What the
// source cannot rule out is a compiler that moves an in-flight destination itself (a spill, or a copy
// of a loop-carried value it could not keep in place): the build refuses any kernel with scratch and
// scans the generated assembly for instructions that name a register with a load in flight.
template <int IMM, bool STREAMING>
__device__ __forceinline__ u32x4 issue_load_b128(rsrc_t rsrc, int lane_off)
{
    static_assert(IMM >= 0 && IMM < 4096, "the immediate offset of a buffer load is a 12-bit field");
    u32x4 r;
    if (STREAMING)  // "nt": read-once data, do not keep it in the caches
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:%3 nt"
                     : "=v"(r) : "v"(lane_off), "s"(rsrc), "n"(IMM) : "memory");
    else
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:%3"
                     : "=v"(r) : "v"(lane_off), "s"(rsrc), "n"(IMM) : "memory");
    return r;
}

// Wait until at most N of the loads issued so far are still outstanding (they return in order).
template <int N>
__device__ __forceinline__ void wait_loads()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

__device__ __forceinline__ void pin(u32x4 &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin(u32x2 &v) { asm volatile("" : "+v"(v)); }

// 32-bit load through the caches (data that several lanes and waves share, e.g. group scales).
template <int IMM>
__device__ __forceinline__ uint32_t issue_load_b32(rsrc_t rsrc, int lane_off)
{
    uint32_t r;
    asm volatile("buffer_load_dword %0, %1, %2, 0 offen offset:%3"
                 : "=v"(r) : "v"(lane_off), "s"(rsrc), "n"(IMM) : "memory");
    return r;
}
__device__ __forceinline__ void pin(uint32_t &v) { asm volatile("" : "+v"(v)); }

// 64-bit variant of issue_load_b128 (streaming policy), for planes that hold 8 bytes per lane.
template <int IMM>
__device__ __forceinline__ u32x2 issue_load_b64(rsrc_t rsrc, int lane_off)
{
    static_assert(IMM >= 0 && IMM < 4096, "the immediate offset of a buffer load is a 12-bit field");
    u32x2 r;
    asm volatile("buffer_load_dwordx2 %0, %1, %2, 0 offen offset:%3 nt"
                 : "=v"(r) : "v"(lane_off), "s"(rsrc), "n"(IMM) : "memory");
    return r;
}

// Global -> LDS copy without passing through registers: lane i's 16 bytes land at LDS byte address
// lds_base + IMM + 16*i (lds_base wave-uniform, placed in M0).  Counted by vmcnt like any other load;
// the data is in LDS once the wait has passed (other waves see it after the next barrier).  M0 is written
// inside the statement and cannot be named as clobbered: it is a reserved register for this compiler (which
// says so when it is listed), i.e. the compiler keeps no value in it across statements and sets it right
// before each instruction of its own that reads it.
template <int IMM, bool STREAMING = false>
__device__ __forceinline__ void issue_load_to_lds_b128(rsrc_t rsrc, int lane_off, uint32_t lds_base)
{
    static_assert(IMM >= 0 && IMM < 4096, "the immediate offset of a buffer load is a 12-bit field");
    if (STREAMING)  // "nt": read-once data, do not keep it in the caches
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen offset:%3 nt lds"
                     : : "s"(lds_base), "v"(lane_off), "s"(rsrc), "n"(IMM) : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen offset:%3 lds"
                     : : "s"(lds_base), "v"(lane_off), "s"(rsrc), "n"(IMM) : "memory");
}

// ---- activation tile layout in LDS -----------------------------------------
// One MFMA step needs, for its 16 token columns n and 4 lane groups q, the 8 consecutive columns
// X[n][k_offset(f, q) ..+8]: 64 pieces of 16 bytes = 1 KB per (token tile, run).  Inside that 1 KB,
// piece 4*n + (q ^ x_swizzle(n)) holds (n, q).  Reading side: the MFMA lane (q, n) = (L/16, L%16) reads
// that piece; the XOR with (n/2)%4 makes the 128-bit LDS read conflict-free (measured: same cost as the
// linear pattern, while 4*n + q and several other rotations cost extra passes).  Writing side: piece p is
// written by lane p of a 64-lane copy, which fetches row n = p/4, group q = (p%4) ^ x_swizzle(n) - so each
// quad of lanes reads 64 contiguous bytes of one row of X (the texture addresser merges such quads into
// one request; scattered 16-byte gathers are 4x slower).
__device__ __forceinline__ int x_swizzle(int n) { return (n >> 1) & 3; }
// piece read by MFMA lane L
__device__ __forceinline__ int x_piece_of_lane(int L)
{
    const int n = L & 15, q = L >> 4;
    return 4 * n + (q ^ x_swizzle(n));
}
// (token row, lane group) fetched by copy lane p
__device__ __forceinline__ void x_source_of_piece(int p, int &n, int &q)
{
    n = (p >> 2) & 15;
    q = (p & 3) ^ x_swizzle(n);
}

// ---- weight sources -------------------------------------------------------
// A source knows how one lane fetches its share of a 16 x 256 weight tile and how
// to turn it into the eight A fragments (one per run) of the tile.  k_offset(f, q)
// is the column, inside the tile, of the first of the 8 consecutive columns that
// lane group q feeds to MFMA step f; the activation staging uses the same map.
// slice_rsrc() describes the memory one wave may read for row tile `row_tile` and
// k-tiles kt_first + i * kt_step (i < n_tiles) of a matrix of RT row tiles (for a packed source: from the first
// tile of the slice to the end of its last; the tiles of other row tiles lie in between);
// issue() requests the tile at lane offset `off` (= lane_offset + t * tile_stride(RT) for
// tile t of the slice) with kLoads loads.  Offsets are 32-bit: the host admits only
// matrices whose packed size, plus the look-ahead of the pipelines, stays below 2^31.

// What one wave keeps to fetch the tiles of its slice: init() once, then issue(tile, t) requests tile t of
// the slice (t past the slice reads zeros).  A slice is the k-tiles kt_first, kt_first + kt_step, ... (n_tiles
// of them) of one row tile: kt_step = 1 is a contiguous range of k-tiles, kt_step = S deals the k-tiles of a
// row tile round-robin to S slices.  SimpleStream serves every source whose tile comes from one buffer; a
// source with a second input (per-group scales) defines its own.
template <class Src>
struct SimpleStream {
    rsrc_t rsrc;
    int off, stride;
    __device__ __forceinline__ void init(const void *weights, const half_t * /*scales*/, int64_t row_tile, int kt_first,
                                         int kt_step, int n_tiles, int64_t RT, int64_t K, int lane)
    {
        rsrc = Src::slice_rsrc(weights, row_tile, kt_first, kt_step, n_tiles, RT, K);
        off = Src::lane_offset(lane, kt_first, (int)K);
        stride = __builtin_amdgcn_readfirstlane(Src::tile_stride(RT) * kt_step);
    }
    __device__ __forceinline__ void issue(typename Src::Tile &tile, int t) const
    {
        Src::issue(tile, rsrc, off + t * stride);
    }
    // tiles live in registers: nothing to bind (see StagedFp16Source)
    template <int D>
    __device__ __forceinline__ void bind_slots(typename Src::Tile (&)[D], u32x4 *, int) const
    {
    }
};

// Packed sources: the slice of row tile `row_tile` over k-tiles kt_first + i * kt_step, i < n_tiles, tiles of
// TILE_BYTES stored k-tile major.  The range runs from the first tile of the slice to the end of its last (the
// tiles of other row tiles and slices lie in between); a tile past the slice lies past the range: it reads as
// zeros and fetches nothing.
template <int TILE_BYTES>
__device__ __forceinline__ rsrc_t packed_slice_rsrc(const void *base, int64_t row_tile, int kt_first, int kt_step,
                                                    int n_tiles, int64_t RT)
{
    return make_rsrc(static_cast<const uint8_t *>(base) + ((int64_t)kt_first * RT + row_tile) * TILE_BYTES,
                     (uint32_t)(((int64_t)(n_tiles - 1) * kt_step * RT + 1) * TILE_BYTES));
}

struct PackedFp6Source {
    typedef PackedFp6Source StreamSource;  // the source the streaming kernel uses for this format
    typedef SimpleStream<PackedFp6Source> Stream;
    static constexpr bool kPackedConfigs = true;  // which table of kernel configurations the host uses
    struct Tile {
        u32x4 p0, p1, p2;
    };
    static constexpr int kLdsTileBytes = 0;  // tiles in flight live in registers
    static constexpr int kTileCols = kTileK;  // columns of one weight tile in the streaming kernel
    static constexpr bool kHasScale = true;
    static constexpr bool kTallTile = true;  // a wave tile of 2 row tiles x 8 token tiles (64 accumulator registers) is affordable
    static constexpr int kLoads = 3;
    // bytes from one k-tile of the slice to the next
    __device__ static __forceinline__ int tile_stride(int64_t RT) { return (int)(RT * kTileBytes); }
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    __device__ static __forceinline__ rsrc_t slice_rsrc(const void *base, int64_t row_tile, int kt_first, int kt_step,
                                                        int n_tiles, int64_t RT, int64_t /*K*/)
    {
        return packed_slice_rsrc<kTileBytes>(base, row_tile, kt_first, kt_step, n_tiles, RT);
    }
    __device__ static __forceinline__ int lane_offset(int lane, int /*kt0*/, int /*K*/) { return lane * 16; }
    __device__ static __forceinline__ void issue(Tile &t, rsrc_t r, int off)
    {
        t.p0 = issue_load_b128<0, true>(r, off);
        t.p1 = issue_load_b128<1024, true>(r, off);
        t.p2 = issue_load_b128<2048, true>(r, off);
    }
    __device__ static __forceinline__ void pin_tile(Tile &t)
    {
        pin(t.p0);
        pin(t.p1);
        pin(t.p2);
    }
    // A fragments of runs 2G (even) and 2G+1 (odd).  Runs 0..3 come from the first stream of the lane
    // (words p0[0..3], p1[0..1]), runs 4..7 from the second (p1[2..3], p2[0..3]); the two calls that share
    // a stream (G = 0, 1 and G = 2, 3) are merged by the compiler into one conversion.
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        const u32x6 d = G < 2 ? (u32x6){t.p0[0], t.p0[1], t.p0[2], t.p0[3], t.p1[0], t.p1[1]}
                              : (u32x6){t.p1[2], t.p1[3], t.p2[0], t.p2[1], t.p2[2], t.p2[3]};
        const half32_t h = dequant_stream(d);
        constexpr int o = (G & 1) * 16;
        even_run = (half8_t){h[o + 0], h[o + 1], h[o + 2], h[o + 3], h[o + 4], h[o + 5], h[o + 6], h[o + 7]};
        odd_run = (half8_t){h[o + 8], h[o + 9], h[o + 10], h[o + 11], h[o + 12], h[o + 13], h[o + 14], h[o + 15]};
    }
};

// ---- 6-bit weights with one scale per row and per group of 128 columns --------------------------------
// Same packed stream as PackedFp6Source.  A group of 128 columns is exactly one of the two 32-code streams
// a lane holds per tile, so the scale multiplies the 32 converted values of a stream before they go to the
// matrix cores (the placement of Algorithm 1 of the paper); nothing is left for the epilogue.  The
// products decode(code) * scale are exact in fp32 and rounded once to fp16 by the packed multiply.
// scales: fp16 [M][K/128]; lane (r, q) fetches, with each tile, the two scales of its row for that tile.
constexpr int kGroupColumns = 128;

struct PackedFp6GroupSource {
    typedef PackedFp6GroupSource StreamSource;  // the source the streaming kernel uses for this format
    static constexpr bool kPackedConfigs = true;
    static constexpr int kLdsTileBytes = 0;  // tiles in flight live in registers
    static constexpr int kTileCols = kTileK;  // columns of one weight tile in the streaming kernel
    static constexpr bool kHasScale = false;  // no per-row factor in the epilogue
    static constexpr bool kTallTile = false;  // the scales and their multiplies leave no room for the 2 x 8 wave tile
    static constexpr int kLoads = 4;
    struct Tile {
        u32x4 p0, p1, p2;
        uint32_t sc;  // two fp16: the scales of groups 2*kt and 2*kt + 1 of the lane's row
    };
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    struct Stream {
        rsrc_t w_rsrc, s_rsrc;
        int w_off, w_stride, s_off;
        int s_stride;
        __device__ __forceinline__ void init(const void *weights, const half_t *scales, int64_t row_tile, int kt_first,
                                             int kt_step, int n_tiles, int64_t RT, int64_t K, int lane)
        {
            w_rsrc = PackedFp6Source::slice_rsrc(weights, row_tile, kt_first, kt_step, n_tiles, RT, K);
            w_off = lane * 16;
            w_stride = __builtin_amdgcn_readfirstlane(PackedFp6Source::tile_stride(RT) * kt_step);
            const int groups = (int)(K / kGroupColumns);  // per row; = 2 * KT
            // the scales of the 16 rows of the row tile; a tile past the slice reads other finite scales or
            // zeros, and its weights read as zeros
            s_rsrc = make_rsrc(scales + row_tile * kTileRows * groups, (uint32_t)(kTileRows * groups * 2));
            s_off = ((lane & 15) * groups + 2 * kt_first) * 2;
            s_stride = __builtin_amdgcn_readfirstlane(4 * kt_step);
        }
        __device__ __forceinline__ void issue(Tile &t, int i) const
        {
            const int off = w_off + i * w_stride;
            t.p0 = issue_load_b128<0, true>(w_rsrc, off);
            t.p1 = issue_load_b128<1024, true>(w_rsrc, off);
            t.p2 = issue_load_b128<2048, true>(w_rsrc, off);
            t.sc = issue_load_b32<0>(s_rsrc, s_off + i * s_stride);
        }
        template <int D>
        __device__ __forceinline__ void bind_slots(Tile (&)[D], u32x4 *, int) const
        {
        }
    };
    __device__ static __forceinline__ void pin_tile(Tile &t)
    {
        pin(t.p0);
        pin(t.p1);
        pin(t.p2);
        pin(t.sc);
    }
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        const u32x6 d = G < 2 ? (u32x6){t.p0[0], t.p0[1], t.p0[2], t.p0[3], t.p1[0], t.p1[1]}
                              : (u32x6){t.p1[2], t.p1[3], t.p2[0], t.p2[1], t.p2[2], t.p2[3]};
        const half32_t h = dequant_stream(d);
        const half2_t both = bit_cast<half2_t>(t.sc);
        const half_t s = G < 2 ? both[0] : both[1];
        constexpr int o = (G & 1) * 16;
        even_run = (half8_t){h[o + 0], h[o + 1], h[o + 2], h[o + 3], h[o + 4], h[o + 5], h[o + 6], h[o + 7]} * s;
        odd_run = (half8_t){h[o + 8], h[o + 9], h[o + 10], h[o + 11], h[o + 12], h[o + 13], h[o + 14], h[o + 15]} * s;
    }
};

// ---- 5-bit (e2m2) weights: the paper's scheme for a width the hardware cannot convert -------------
// The paper presents its pre-packing and its cast as independent of the bit-width (Sections 5.2, 5.3).
// CDNA4 has no conversion for e2m2, so this source de-quantizes the way Section 5.3 does, with shifts and
// masks on whole words (four codes per 32-bit operation) and the exponent-bias multiply of Eq. 3.
// Tile: 16 rows x 256 columns = 2560 bytes = two planes of 16 bytes per lane and one of 8 bytes per lane;
// lane L = 16q + r owns ten words, D0..D4 for runs 0..3 and another five for runs 4..7.  Of the 32 codes
// of four runs (index i = 8*(run%4) + j), the first twenty sit in place in byte i%4 of D[i/4] as
// "s...EEMM" - the top byte of the fp16 that Eq. 3 asks for - and the other twelve are spread over the
// free bits 6, 5, 4 of the twenty bytes:
//   codes 20..23:  s -> D0.6  e1 e0 -> D0.5 D0.4  m1 m0 -> D1.6 D1.5
//   codes 24..27:  s -> D1.4  e1 e0 m1 -> D2.6 D2.5 D2.4  m0 -> D3.6
//   codes 28..31:  s -> D3.5  e1 -> D3.4  e0 m1 m0 -> D4.6 D4.5 D4.4
// Unpack per 32 codes: 5 ANDs, 3 three-term stitches, then per four codes two byte permutes and two
// packed multiplies by 2^(15-1) (exact, the subnormal binade included).
__device__ __forceinline__ half8_t e2m2_bytes_to_fragment(uint32_t b_lo, uint32_t b_hi)
{
    const half2_t k = {(half_t)16384.0f, (half_t)16384.0f};
    u32x4 r;
    r[0] = bit_cast<uint32_t>(bit_cast<half2_t>(__builtin_amdgcn_perm(0u, b_lo, 0x010c000cu)) * k);  // [b1 0 b0 0]
    r[1] = bit_cast<uint32_t>(bit_cast<half2_t>(__builtin_amdgcn_perm(0u, b_lo, 0x030c020cu)) * k);  // [b3 0 b2 0]
    r[2] = bit_cast<uint32_t>(bit_cast<half2_t>(__builtin_amdgcn_perm(0u, b_hi, 0x010c000cu)) * k);
    r[3] = bit_cast<uint32_t>(bit_cast<half2_t>(__builtin_amdgcn_perm(0u, b_hi, 0x030c020cu)) * k);
    return bit_cast<half8_t>(r);
}

struct PackedFp5Source {
    typedef PackedFp5Source StreamSource;  // the source the streaming kernel uses for this format
    typedef SimpleStream<PackedFp5Source> Stream;
    static constexpr bool kPackedConfigs = true;  // which table of kernel configurations the host uses
    struct Tile {
        u32x4 p0, p1;
        u32x2 p2;
    };
    static constexpr int kLdsTileBytes = 0;  // tiles in flight live in registers
    static constexpr int kTileCols = kTileK;  // columns of one weight tile in the streaming kernel
    static constexpr bool kHasScale = true;
    static constexpr bool kTallTile = true;
    static constexpr int kLoads = 3;
    static constexpr int kTileBytes5 = 2560;
    __device__ static __forceinline__ int tile_stride(int64_t RT) { return (int)(RT * kTileBytes5); }
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    __device__ static __forceinline__ rsrc_t slice_rsrc(const void *base, int64_t row_tile, int kt_first, int kt_step,
                                                        int n_tiles, int64_t RT, int64_t /*K*/)
    {
        return packed_slice_rsrc<kTileBytes5>(base, row_tile, kt_first, kt_step, n_tiles, RT);
    }
    __device__ static __forceinline__ int lane_offset(int lane, int /*kt0*/, int /*K*/) { return lane * 16; }
    __device__ static __forceinline__ void issue(Tile &t, rsrc_t r, int off)
    {
        // the third plane holds 8 bytes per lane: its offset is the tile's base + 2048 + 8 * lane
        const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        t.p0 = issue_load_b128<0, true>(r, off);
        t.p1 = issue_load_b128<1024, true>(r, off);
        t.p2 = issue_load_b64<2048>(r, off - 8 * lane);
    }
    __device__ static __forceinline__ void pin_tile(Tile &t)
    {
        pin(t.p0);
        pin(t.p1);
        pin(t.p2);
    }
    // A fragments of runs 2G (even) and 2G+1 (odd).  Runs 0..3 come from D = (p0[0..3], p1[0]), runs 4..7
    // from D = (p1[1..3], p2[0..1]); inside a group of four runs, runs 0 and 1 are the in-place words
    // D0..D3, run 2 is D4 and the first stitched word, run 3 the other two stitched words.
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        uint32_t d0, d1, d2, d3, d4;
        if (G < 2) {
            d0 = t.p0[0], d1 = t.p0[1], d2 = t.p0[2], d3 = t.p0[3], d4 = t.p1[0];
        } else {
            d0 = t.p1[1], d1 = t.p1[2], d2 = t.p1[3], d3 = t.p2[0], d4 = t.p2[1];
        }
        constexpr uint32_t kInPlace = 0x8f8f8f8fu;
        if ((G & 1) == 0) {
            even_run = e2m2_bytes_to_fragment(d0 & kInPlace, d1 & kInPlace);
            odd_run = e2m2_bytes_to_fragment(d2 & kInPlace, d3 & kInPlace);
        } else {
            const uint32_t s0 = ((d0 << 1) & 0x80808080u) | ((d0 >> 2) & 0x0c0c0c0cu) | ((d1 >> 5) & 0x03030303u);
            const uint32_t s1 = ((d1 << 3) & 0x80808080u) | ((d2 >> 3) & 0x0e0e0e0eu) | ((d3 >> 6) & 0x01010101u);
            const uint32_t s2 = ((d3 << 2) & 0x80808080u) | ((d3 >> 1) & 0x08080808u) | ((d4 >> 4) & 0x07070707u);
            even_run = e2m2_bytes_to_fragment(d4 & kInPlace, s0);
            odd_run = e2m2_bytes_to_fragment(s1, s2);
        }
    }
};

// ---- 4-bit (e2m1) weights ------------------------------------------------------------------------
// e2m1 (bias 1, subnormal E = 0 binade: 0 .5 1 1.5 2 3 4 6) is the FP4 element type of the OCP microscaling
// formats; the chip converts two codes of a byte to two fp16 values with v_cvt_scalef32_pk_f16_fp4.
// Tile: 16 rows x 256 columns = 2048 bytes = two planes of 16 bytes per lane; lane L = 16q + r owns eight
// words, word d = run d (columns 32d + 8q + j), code j in bits [4j, 4j+4): one word is one A fragment.
__device__ __forceinline__ half8_t e2m1_word_to_fragment(uint32_t w)
{
    const half2_t a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 0);
    const half2_t b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 1);
    const half2_t c = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 2);
    const half2_t d = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 3);
    return (half8_t){a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

struct PackedFp4Source {
    typedef PackedFp4Source StreamSource;  // the source the streaming kernel uses for this format
    typedef SimpleStream<PackedFp4Source> Stream;
    static constexpr bool kPackedConfigs = true;  // which table of kernel configurations the host uses
    struct Tile {
        u32x4 p0, p1;
    };
    static constexpr int kLdsTileBytes = 0;  // tiles in flight live in registers
    static constexpr int kTileCols = kTileK;  // columns of one weight tile in the streaming kernel
    static constexpr bool kHasScale = true;
    static constexpr bool kTallTile = true;
    static constexpr int kLoads = 2;
    static constexpr int kTileBytes4 = 2048;
    __device__ static __forceinline__ int tile_stride(int64_t RT) { return (int)(RT * kTileBytes4); }
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    __device__ static __forceinline__ rsrc_t slice_rsrc(const void *base, int64_t row_tile, int kt_first, int kt_step,
                                                        int n_tiles, int64_t RT, int64_t /*K*/)
    {
        return packed_slice_rsrc<kTileBytes4>(base, row_tile, kt_first, kt_step, n_tiles, RT);
    }
    __device__ static __forceinline__ int lane_offset(int lane, int /*kt0*/, int /*K*/) { return lane * 16; }
    __device__ static __forceinline__ void issue(Tile &t, rsrc_t r, int off)
    {
        t.p0 = issue_load_b128<0, true>(r, off);
        t.p1 = issue_load_b128<1024, true>(r, off);
    }
    __device__ static __forceinline__ void pin_tile(Tile &t)
    {
        pin(t.p0);
        pin(t.p1);
    }
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        const u32x4 &p = G < 2 ? t.p0 : t.p1;
        even_run = e2m1_word_to_fragment(p[2 * (G & 1)]);
        odd_run = e2m1_word_to_fragment(p[2 * (G & 1) + 1]);
    }
};

// ---- 3-bit (e2m0) weights ------------------------------------------------------------------------
// e2m0 (bias 1, no mantissa bits: 0 1 2 4) has no conversion instruction of its own, but code s e1 e0 has
// the value of the e2m1 code s e1 e0 0, so a word of eight 4-bit fields "s e1 e0 0" goes through the FP4
// conversion.  The layout (the paper's ahead-of-time bit-level pre-packing, Section 5.2, with a 3+1 split)
// stores exactly such words.  Tile = 16 rows x 512 columns = 3072 bytes = three planes of 16 bytes per lane,
// so that the streaming kernel fetches a tile with three whole 128-bit loads (a 64-bit load costs the memory
// pipeline what a 128-bit one costs).  Each half of the tile (256 columns) gives the lane six words: the four
// of plane 0 (first half) or plane 2 (second half), then words 2h, 2h+1 of the middle plane.  Of those six,
// words 3g..3g+2 are runs 4g..4g+2 of the half in place with bit 0 of every field free, and those free bits
// carry run 4g+3: its bit b+1 of field j is bit 4j of word 3g+b.  Unpack: one AND per in-place run, three
// AND/shift/OR for the fourth.
// A fragments of runs 2G (even) and 2G+1 (odd) of one half, G = 0..3, from the half's six words
template <int G>
__device__ __forceinline__ void e2m0_half_fragments(const u32x4 &p0, uint32_t w4, uint32_t w5, half8_t &even_run,
                                                    half8_t &odd_run)
{
    constexpr uint32_t kFields = 0xeeeeeeeeu, kFree = 0x11111111u;
    const uint32_t a0 = G < 2 ? p0[0] : p0[3];
    const uint32_t a1 = G < 2 ? p0[1] : w4;
    const uint32_t a2 = G < 2 ? p0[2] : w5;
    if ((G & 1) == 0) {
        even_run = e2m1_word_to_fragment(a0 & kFields);
        odd_run = e2m1_word_to_fragment(a1 & kFields);
    } else {
        even_run = e2m1_word_to_fragment(a2 & kFields);
        odd_run = e2m1_word_to_fragment(((a0 & kFree) << 1) | ((a1 & kFree) << 2) | ((a2 & kFree) << 3));
    }
}
constexpr int kTileBytes3 = 3072;  // 16 rows x 512 columns of 3-bit codes

// The whole tile, for the streaming kernel: 512 columns per step.
struct PackedFp3WideSource {
    typedef SimpleStream<PackedFp3WideSource> Stream;
    typedef PackedFp3WideSource StreamSource;
    static constexpr bool kPackedConfigs = true;  // which table of kernel configurations the host uses
    struct Tile {
        u32x4 p0, p1, p2;
    };
    static constexpr int kLdsTileBytes = 0;  // tiles in flight live in registers
    static constexpr int kTileCols = 512;
    static constexpr bool kHasScale = true;
    static constexpr bool kTallTile = true;
    static constexpr int kLoads = 3;
    __device__ static __forceinline__ int tile_stride(int64_t RT) { return (int)(RT * kTileBytes3); }
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    __device__ static __forceinline__ rsrc_t slice_rsrc(const void *base, int64_t row_tile, int kt_first, int kt_step,
                                                        int n_tiles, int64_t RT, int64_t /*K*/)
    {
        return packed_slice_rsrc<kTileBytes3>(base, row_tile, kt_first, kt_step, n_tiles, RT);
    }
    __device__ static __forceinline__ int lane_offset(int lane, int /*kt0*/, int /*K*/) { return lane * 16; }
    __device__ static __forceinline__ void issue(Tile &t, rsrc_t r, int off)
    {
        t.p0 = issue_load_b128<0, true>(r, off);
        t.p1 = issue_load_b128<1024, true>(r, off);
        t.p2 = issue_load_b128<2048, true>(r, off);
    }
    __device__ static __forceinline__ void pin_tile(Tile &t)
    {
        pin(t.p0);
        pin(t.p1);
        pin(t.p2);
    }
    // A fragments of runs 2G and 2G+1 of the tile, G = 0..7
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        if (G < 4)
            e2m0_half_fragments<G % 4>(t.p0, t.p1[0], t.p1[1], even_run, odd_run);
        else
            e2m0_half_fragments<G % 4>(t.p2, t.p1[2], t.p1[3], even_run, odd_run);
    }
};

// One half of a tile (256 columns) at a time, for the kernels that step through k in units of 256 columns
// (the tiled kernel, unpack): k-tile kt is half kt % 2 of tile kt / 2, fetched with one 128-bit and one
// 64-bit load.
struct PackedFp3Source {
    typedef PackedFp3WideSource StreamSource;
    static constexpr bool kPackedConfigs = true;
    struct Tile {
        u32x4 p0;
        u32x2 p1;
    };
    static constexpr int kLdsTileBytes = 0;
    static constexpr int kTileCols = kTileK;
    static constexpr bool kHasScale = true;
    static constexpr bool kTallTile = true;
    static constexpr int kLoads = 2;
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    struct Stream {
        rsrc_t rsrc;
        int off, first, stride;  // lane offset, first k-tile, bytes from one tile of a row tile to the next
        // k-tiles kt_first .. kt_first + n_tiles - 1 of one row tile (contiguous: kt_step is 1 for every user)
        __device__ __forceinline__ void init(const void *weights, const half_t * /*scales*/, int64_t row_tile, int kt_first,
                                             int /*kt_step*/, int n_tiles, int64_t RT, int64_t /*K*/, int lane)
        {
            const int t0 = kt_first >> 1, t1 = (kt_first + n_tiles - 1) >> 1;  // first and last tile touched
            rsrc = make_rsrc(static_cast<const uint8_t *>(weights) + ((int64_t)t0 * RT + row_tile) * kTileBytes3,
                             (uint32_t)(((int64_t)(t1 - t0) * RT + 1) * kTileBytes3));
            off = lane * 16;
            first = kt_first;
            stride = __builtin_amdgcn_readfirstlane((int)(RT * kTileBytes3));
        }
        __device__ __forceinline__ void issue(Tile &tile, int t) const
        {
            const int kt = first + t, half = kt & 1;
            const int o = off + ((kt >> 1) - (first >> 1)) * stride;
            tile.p0 = issue_load_b128<0, true>(rsrc, o + half * 2048);
            tile.p1 = issue_load_b64<1024>(rsrc, o + half * 8);
        }
        template <int D>
        __device__ __forceinline__ void bind_slots(Tile (&)[D], u32x4 *, int) const
        {
        }
    };
    __device__ static __forceinline__ void pin_tile(Tile &t)
    {
        pin(t.p0);
        pin(t.p1);
    }
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        e2m0_half_fragments<G>(t.p0, t.p1[0], t.p1[1], even_run, odd_run);
    }
};

struct StagedFp16Source;
struct PlainFp16Source {
    typedef StagedFp16Source StreamSource;  // the source the streaming kernel uses for this format
    typedef SimpleStream<PlainFp16Source> Stream;
    static constexpr bool kPackedConfigs = false;  // which table of kernel configurations the host uses
    struct Tile {
        u32x4 v[8];
    };
    static constexpr int kLdsTileBytes = 0;  // tiles in flight live in registers
    static constexpr int kTileCols = kTileK;  // columns of one weight tile in the streaming kernel
    static constexpr bool kHasScale = false;
    static constexpr bool kTallTile = false;
    static constexpr int kLoads = 8;
    __device__ static __forceinline__ int tile_stride(int64_t /*RT*/) { return kTileK * 2; }  // row-major W
    // the four lane groups of a row read four adjacent 16-byte pieces (64 contiguous bytes per row
    // and load instruction); plain (cached) loads, so the other half of each line is an L1/L2 hit
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    // the 16 rows of the row tile; tiles past the slice are neutralised by zero activations
    __device__ static __forceinline__ rsrc_t slice_rsrc(const void *base, int64_t row_tile, int /*kt_first*/,
                                                        int /*kt_step*/, int /*n_tiles*/, int64_t /*RT*/, int64_t K)
    {
        return make_rsrc(static_cast<const half_t *>(base) + row_tile * kTileRows * K, (uint32_t)(kTileRows * K * 2));
    }
    __device__ static __forceinline__ int lane_offset(int lane, int kt0, int K)
    {
        const int r = lane & 15, q = lane >> 4;
        return (r * K + kt0 * kTileK + q * 8) * 2;
    }
    __device__ static __forceinline__ void issue(Tile &t, rsrc_t rs, int off)
    {
        t.v[0] = issue_load_b128<0, false>(rs, off);
        t.v[1] = issue_load_b128<64, false>(rs, off);
        t.v[2] = issue_load_b128<128, false>(rs, off);
        t.v[3] = issue_load_b128<192, false>(rs, off);
        t.v[4] = issue_load_b128<256, false>(rs, off);
        t.v[5] = issue_load_b128<320, false>(rs, off);
        t.v[6] = issue_load_b128<384, false>(rs, off);
        t.v[7] = issue_load_b128<448, false>(rs, off);
    }
    __device__ static __forceinline__ void pin_tile(Tile &t)
    {
#pragma unroll
        for (int f = 0; f < 8; ++f)
            pin(t.v[f]);
    }
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        even_run = bit_cast<half8_t>(t.v[2 * G]);
        odd_run = bit_cast<half8_t>(t.v[2 * G + 1]);
    }
};

// fp16 weights for the streaming kernel, staged through LDS.  Loading the A operand of a row-major fp16
// matrix straight into registers (PlainFp16Source) makes every load instruction touch 16 rows x 64 bytes:
// half a cache line per row and request.  Here a copy instruction (global -> LDS, no registers) fetches
// 8 rows x 128 bytes - eight whole lines - and the wave reads its A fragments back from LDS.  The region is
// private to the wave (its own copies, its own reads): the wait for the copies is all the synchronisation
// there is, no barrier.  The copies carry the streaming hint like every other weight load (measured on the
// 8192 x 22016 layer, N <= 16: 81 us without it, whole lines or not, 72 us with it).
//   Tile = 16 rows x 256 columns = eight blocks of 1 KB; block 2*seg + h holds rows 8h .. 8h+7, columns
// 64*seg .. 64*seg+63.  Copy lane i = 8*rho + pi lands at piece i of the block (16 bytes each) and fetches
// row 8h + rho, 8-column chunk pi ^ w_swizzle(row) of the segment: the eight lanes of a row fetch one whole
// line, a quad of lanes 64 contiguous bytes.  MFMA lane (q, r) of run f = 2*seg + e wants row r, chunk
// 4e + q: piece 8*(r%8) + ((4e + q) ^ w_swizzle(r)) of block 2*seg + r/8.  A 128-bit LDS read serves sixteen
// lanes at a time, and not sixteen consecutive ones: lanes {0-3, 12-15, 20-23, 24-27} of a half-wave go
// together, then {4-11, 16-19, 28-31} (the grouping under which the activation swizzle above is conflict-free
// and a first swizzle of this tile, which spread sixteen consecutive lanes, cost four extra cycles per read -
// both by SQ_LDS_BANK_CONFLICT).  In MFMA terms a group is rows {0-3, 12-15} of lane group q with rows
// {4-11} of lane group q ^ 1: with the chunk XORed by 2 * ((row / 2) % 4) their sixteen pieces fall into
// sixteen different 16-byte bank groups.
__device__ __forceinline__ int w_swizzle(int row) { return ((row >> 1) & 3) << 1; }

struct StagedFp16Source {
    typedef StagedFp16Source StreamSource;  // the source the streaming kernel uses for this format
    static constexpr bool kPackedConfigs = false;
    static constexpr bool kHasScale = false;
    static constexpr bool kTallTile = false;
    static constexpr int kLoads = 8;
    static constexpr int kLdsTileBytes = 8192;
    static constexpr int kTileCols = kTileK;
    struct Tile {
        const u32x4 *even, *odd;  // this lane's fragment of run 0 (even runs) and of run 1 (odd runs) in the slot
        uint32_t lds;             // LDS byte address of the slot (wave-uniform)
    };
    __device__ static __forceinline__ int k_offset(int f, int q) { return f * 32 + q * 8; }
    __device__ static __forceinline__ void pin_tile(Tile &) {}
    struct Stream {
        rsrc_t rsrc;
        int off0, off1, stride;  // lane offsets of the copies of rows 0..7 and of rows 8..15
        __device__ __forceinline__ void init(const void *weights, const half_t * /*scales*/, int64_t row_tile, int kt_first,
                                             int kt_step, int /*n_tiles*/, int64_t /*RT*/, int64_t K, int lane)
        {
            // the 16 rows of the row tile; tiles past the slice are neutralised by zero activations
            rsrc = make_rsrc(static_cast<const half_t *>(weights) + row_tile * kTileRows * K, (uint32_t)(kTileRows * K * 2));
            const int rho = lane >> 3, pi = lane & 7;
            off0 = (rho * (int)K + kt_first * kTileK + 8 * (pi ^ w_swizzle(rho))) * 2;
            off1 = ((rho + 8) * (int)K + kt_first * kTileK + 8 * (pi ^ w_swizzle(rho + 8))) * 2;
            stride = __builtin_amdgcn_readfirstlane(kTileK * 2 * kt_step);
        }
        template <int D>
        __device__ __forceinline__ void bind_slots(Tile (&w)[D], u32x4 *region, int lane) const
        {
            const int r = lane & 15, q = lane >> 4;
            const int piece = (r >> 3) * 64 + 8 * (r & 7) + (q ^ w_swizzle(r));
#pragma unroll
            for (int d = 0; d < D; ++d) {
                u32x4 *slot = region + d * (kLdsTileBytes / 16);
                w[d].even = slot + piece;
                w[d].odd = slot + (piece ^ 4);
                w[d].lds = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)reinterpret_cast<uintptr_t>(slot));
            }
        }
        __device__ __forceinline__ void issue(Tile &tile, int t) const
        {
            // the slot's previous contents have been read: every LDS read of this wave has returned
            asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
            const int o0 = off0 + t * stride, o1 = off1 + t * stride;
#pragma unroll
            for (int seg = 0; seg < 4; ++seg) {
                issue_load_to_lds_b128<0, true>(rsrc, o0 + seg * 128, tile.lds + (uint32_t)(2 * seg) * 1024u);
                issue_load_to_lds_b128<0, true>(rsrc, o1 + seg * 128, tile.lds + (uint32_t)(2 * seg + 1) * 1024u);
            }
        }
    };
    // A fragments of runs 2G (even) and 2G+1 (odd): segment G, chunks q and 4 + q
    template <int G>
    __device__ static __forceinline__ void fragments(const Tile &t, half8_t &even_run, half8_t &odd_run)
    {
        even_run = bit_cast<half8_t>(t.even[G * 128]);
        odd_run = bit_cast<half8_t>(t.odd[G * 128]);
    }
};

constexpr int stream_gcd(int a, int b) { return b == 0 ? a : stream_gcd(b, a % b); }

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a compile-time constant
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// ---- last step of the linear kernels ----------------------------------------------------------
// What happens between a finished fp32 sum and the stored fp16: the per-row scale (sources that
// have one), then the element-wise steps that a decoder block attaches to its projections
// (Section 7.3 of the paper runs whole decoders): an optional bias per weight row, optionally
// silu(gate) * up over row pairs, an optional residual, one rounding to fp16 at the very end.
struct Epilogue {
    const half_t *bias;      // fp16 [M] or nullptr
    const half_t *residual;  // fp16 laid out like the output, or nullptr; may be the output itself
    int gated;               // nonzero: weight rows 2i (gate), 2i+1 (up) give output row i of M/2
};

// Rows m0 .. m0+3 (m0 % 4 == 0) of token column `col`: the four sums one lane holds after the MFMAs.
// Y and the residual are [tokens][M] (or [tokens][M/2] when gated).
template <bool kHasScale>
__device__ __forceinline__ void finish_rows(const Epilogue &e, const half_t *__restrict__ scales, const float4_t &sum,
                                            int col, int m0, int M, half_t *Y)
{
    float v[4] = {sum[0], sum[1], sum[2], sum[3]};
    if (kHasScale) {
        const half4_t s4 = *reinterpret_cast<const half4_t *>(scales + m0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            v[i] *= (float)s4[i];
    }
    if (e.bias) {
        const half4_t b4 = *reinterpret_cast<const half4_t *>(e.bias + m0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            v[i] += (float)b4[i];
    }
    if (!e.gated) {
        const int64_t at = (int64_t)col * M + m0;
        if (e.residual) {
            const half4_t r4 = *reinterpret_cast<const half4_t *>(e.residual + at);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                v[i] += (float)r4[i];
        }
        half4_t y;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            y[i] = (half_t)v[i];
        *reinterpret_cast<half4_t *>(Y + at) = y;
    } else {
        const int64_t at = (int64_t)col * (M >> 1) + (m0 >> 1);
        float o[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
            o[i] = v[2 * i] / (1.0f + __expf(-v[2 * i])) * v[2 * i + 1];
        if (e.residual) {
            const half2_t r2 = *reinterpret_cast<const half2_t *>(e.residual + at);
            o[0] += (float)r2[0];
            o[1] += (float)r2[1];
        }
        half2_t y;
        y[0] = (half_t)o[0];
        y[1] = (half_t)o[1];
        *reinterpret_cast<half2_t *>(Y + at) = y;
    }
}

}  // namespace fp6
