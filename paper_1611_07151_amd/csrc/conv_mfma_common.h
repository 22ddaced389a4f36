// Shared pieces of the matrix-core convolution kernels (internal).
//
// On gfx950 the fp32 MFMA instructions do not overlap with ordinary vector-ALU
// instructions of the same SIMD (measured: every VALU instruction adds its four issue
// cycles to the MFMA time), so these kernels are written to keep the VALU instruction
// count per MFMA low: runtime divisions go through precomputed multipliers, every global
// access is "uniform base + 32-bit per-lane byte offset" with the per-lane part computed
// once per tile, and padding is applied with one select per staged element.
#pragma once

#include <stdint.h>

#include "sq_internal.h"

namespace sq {
namespace mfma {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kLdsBytes = 160 * 1024;

// Division of x < 2^31 by a runtime constant d >= 1:  q = (umulhi(x, mul) + (x & add)) >> shift.
// For d >= 2: l = ceil(log2 d), mul = ceil(2^(31+l) / d) (fits 32 bits), shift = l - 1, add = 0.
// For d == 1: mul = 0, add = all ones, shift = 0.
struct FastDiv {
    uint32_t mul, add, shift;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    if (d <= 1) {
        f.mul = 0; f.add = 0xffffffffu; f.shift = 0;
        return f;
    }
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    const unsigned long long num = 1ull << (31 + l);
    f.mul = (uint32_t)((num + d - 1) / d);
    f.add = 0;
    f.shift = l - 1;
    return f;
}

inline uint32_t fastdiv_host(uint32_t x, FastDiv f)
{
    const uint32_t hi = (uint32_t)(((unsigned long long)x * f.mul) >> 32);
    return (hi + (x & f.add)) >> f.shift;
}

__device__ __forceinline__ int fdiv(int x, FastDiv f)
{
    return (int)((__umulhi((uint32_t)x, f.mul) + ((uint32_t)x & f.add)) >> f.shift);
}

struct KParams {
    const float *in;
    const float *w;
    const float *b;
    float *out;
    int N, Cin, H, W, Cout, P, relu;
    int Ho, Wo, HoWo, HW, ldc, coff;
    int PT;      // N*Ho*Wo
    int VH;      // virtual rows per image
    int LW;      // patch columns staged
    int LWs;     // LDS row stride of the patch
    int PRcap;   // patch rows the LDS plane can hold
    int plane;   // LDS floats per input layer
    int mtiles;  // tiles along output layers
    int ntiles;  // tiles along pixels
    int nchunks;
    FastDiv dWo, dHo, dLW, dVH, dHW, dHoWo, dMtiles;
    uint32_t in_bytes, out_bytes, w_bytes;
    // fused expand (3x3 kernel that also produces the 1x1 expand of the same input)
    const float *w1;     // [Cout1][Cin] kernels of the 1x1 convolution
    const float *b1;     // [Cout1] or nullptr
    int Cout1, coff1;    // its layer count and first output layer
    uint32_t w1_bytes;
    int RG, CB;  // conv1-type kernel: tile grid per image (row groups, column blocks)
    FastDiv dRG, dCB;
    int T, TX, TXY;  // minimal-filtering kernel: 2x2-pixel tiles in all, per image row, per image
    FastDiv dTX, dTXY;
    const float *wu;     // its transformed kernels (written by wino_kernel_transform)
    uint32_t wu_bytes;
    int Win, HWin;       // 1x1 kernels with pooling on the way in: row length and plane size of the map in memory
    int avg_slots;       // averaging form of the 1x1 kernels: images a pixel tile can touch
    // pooling split between two layers (ColPool): geometry of the column-pooled map.  A 1x1 kernel that pools the rows
    // on the way in reads such a map; the conv1-type kernel and the autonomous minimal-filtering kernel write one
    // (p.out, rows of cpRS floats holding cpWp pooled columns and the seam slots; cpWp = 0 = plain map)
    int cpShift, cpSlotsRow, cpSlotsImage, cpWp, cpRS;
    // minimal-filtering kernel with autonomous wavefronts: how its workgroups are shared out over the layer blocks
    // (the first wa_big blocks have wa_cnt + 1 workgroups, the others wa_cnt), and tile groups per workgroup of a
    // block with wa_cnt (q0, remainder r0) or wa_cnt + 1 (q1, r1) workgroups
    int wa_big, wa_cnt, wa_q0, wa_r0, wa_q1, wa_r1;
};

// value of lane + n of the same row of 16 lanes (DPP row shift), zero past the row's end
template <int n> __device__ __forceinline__ float row_shl(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x100 + n, 0xf, 0xf, true));
}

template <int MT> struct Mfma;
template <> struct Mfma<32> {
    using Acc = f32x16;
    static constexpr int KQ = 2, NR = 16;
    static __device__ __forceinline__ Acc run(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    // output-layer row of accumulator register r in this lane = row_reg(r) + row_lane(lane)
    static __device__ __forceinline__ constexpr int row_reg(int r) { return 8 * (r >> 2) + (r & 3); }
    static __device__ __forceinline__ int row_lane(int lane) { return 4 * (lane >> 5); }
};
template <> struct Mfma<16> {
    using Acc = f32x4;
    static constexpr int KQ = 4, NR = 4;
    static __device__ __forceinline__ Acc run(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ constexpr int row_reg(int r) { return r; }
    static __device__ __forceinline__ int row_lane(int lane) { return 4 * (lane >> 4); }
};

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Renumber so
// that every XCD works on one contiguous range of tiles (neighbouring tiles share
// halo rows and the same kernels).
__device__ __forceinline__ int xcd_remap(int b, int total)
{
    const int q = total >> 3, r = total & 7;
    const int xcd = b & 7, idx = b >> 3;
    const int start = xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q;
    return start + idx;
}

// Share of a persistent workgroup in `total` work items such that the workgroups of one XCD (workgroup numbers
// equal modulo 8: they are dealt out round-robin) walk through one contiguous eighth of the items, side by side.
// Items that are neighbours in memory then meet in the same L2 instead of being fetched from HBM by several.
// The workgroup takes items first, first + step, ... below end.  The launch must have at least min(8, total) workgroups.
struct XcdShare {
    int first, step, end;
};
__device__ __forceinline__ XcdShare xcd_share(int block, int blocks, int total)
{
    const int xcd = block & 7, q = total >> 3, r = total & 7;
    const int lo = xcd * q + (xcd < r ? xcd : r), cnt = q + (xcd < r ? 1 : 0);
    const int step = (blocks - xcd + 7) >> 3;   // workgroups of this XCD
    return XcdShare{lo + (block >> 3), step, lo + cnt};
}

// Buffer addressing: a uniform 128-bit resource (base, size) + per-lane 32-bit byte offset
// + uniform 32-bit byte offset.  Needs no vector arithmetic per access, and the hardware
// range check does the zero padding: a lane whose offset is >= the buffer size reads 0 and
// its stores are dropped.  kOob is such an offset for every buffer this library describes
// (tensors handled through buffers are kept below 2 GiB).
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr uint32_t kOob = 0x80000000u;
constexpr long long kMaxBufferElems = 1ll << 29;

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    // word 3: DATA_FORMAT = 32-bit, raw (unstructured) buffer
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float buf_ld(rsrc_t r, uint32_t lane_off, uint32_t uni_off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_off, (int)uni_off, 0));
}
__device__ __forceinline__ void buf_st(rsrc_t r, uint32_t lane_off, uint32_t uni_off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)lane_off, (int)uni_off, 0);
}

// 8-byte store through a buffer resource, written as two adjacent 4-byte stores with the same
// lane offset register, which the compiler merges into one buffer_store_dwordx2.  (Its builtins
// for buffer accesses wider than four bytes are not used in this library: the ROCm 7.2 compiler
// lowers the wide loads to a single dword.  Writing the instruction out as inline assembly is
// not safe either: the compiler does not see which scalar registers the statement reads, so it
// leaves out the wait states the hardware needs between a vector instruction that writes a
// scalar register -- such as the re-load of a spilled one -- and a memory instruction that reads
// it, and the store then goes to a stale address.)
__device__ __forceinline__ void buf_st2(rsrc_t r, uint32_t lane_off, uint32_t uni_off, float v0, float v1)
{
    asm volatile("" : "+v"(lane_off));   // keeps the +4 an immediate of the second store
    buf_st(r, lane_off, uni_off, v0);
    buf_st(r, lane_off + 4u, uni_off, v1);
}

// Two fp32 values rounded to bfloat16 (nearest even), first in the low half of the word.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// Input element of type TIN as fp32: float as is, uint16_t = bfloat16 (upper half of binary32).
template <typename TIN> __device__ __forceinline__ float buf_ld_in(rsrc_t r, uint32_t lane_off, uint32_t uni_off);
template <> __device__ __forceinline__ float buf_ld_in<float>(rsrc_t r, uint32_t lane_off, uint32_t uni_off)
{
    return buf_ld(r, lane_off, uni_off);
}
template <> __device__ __forceinline__ float buf_ld_in<uint16_t>(rsrc_t r, uint32_t lane_off, uint32_t uni_off)
{
    const uint32_t h = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)lane_off, (int)uni_off, 0);
    return __builtin_bit_cast(float, h << 16);
}

// base + 32-bit byte offset: the addressing form that needs no per-lane 64-bit arithmetic
__device__ __forceinline__ float ld_f32(const float *base, uint32_t byte_off)
{
    return *(const float *)((const char *)base + byte_off);
}
__device__ __forceinline__ void st_f32(float *base, uint32_t byte_off, float v)
{
    *(float *)((char *)base + byte_off) = v;
}

// conv1-type layers (7x7, stride 2, three input layers, at most 96 output layers) have
// their own persistent kernel with NW autonomous wavefronts per workgroup (8 or 4).
typedef void (*KernelFn)(const KParams);

// Kernels of one tiling: plain, input layers not a multiple of CC, fused 1x1 expand, 1x1 with 3x3 stride-2
// max pooling on the way in, 1x1 writing per-image plane sums instead of its results, 1x1 pooling the rows of a
// column-pooled map on the way in.
struct KernelSet {
    KernelFn plain, tail, fused_e1, pooled, avg, rowpool;
};
extern const KernelSet conv_mfma_kernels_f32[], conv_mfma_kernels_bf16[];
// Both expands of a fire layer in one launch (expand_pair_kernel): the compiled expand1x1 tilings, each named
// like the stand-alone tiling it is.
typedef void (*PairFn)(const KParams, const KParams, int);
struct PairKernel {
    const char *e1_variant;   // name of the 1x1 tiling in the variant list
    const char *name;         // name of the pair in profiles
    PairFn fn;
    const char *e3_variant;   // name of the minimal-filtering tiling it runs
    PairFn fn_colpool;        // the form that writes a column-pooled map and its seam table, or nullptr
    const char *name_colpool;
};
extern const PairKernel expand_pair_kernels[];
extern const int num_expand_pair_kernels;
// TM = blocks of 32 output layers per workgroup: 3 (all 96), or 1 with the block chosen by blockIdx.y (NW = 4 only).
// colpool: the form that writes a column-pooled map and its seam table (fp32, 96 layers only), else nullptr.
KernelFn conv7s2c3_kernel_for(int NW, bool full_96_layers, bool bf16_inputs, int TM, bool colpool = false);

// Minimal-filtering F(2x2, 3x3) kernel: workgroup tile (output layers x tiles of 2x2 pixels),
// input layers per chunk, and the floats of the kernel image [16 positions][2][64][4] of one chunk.
constexpr int kWinoBM = 64, kWinoBT = 32, kWinoCC = 8;
constexpr int kWinoImage = 16 * 2 * 64 * 4;
constexpr int kWinoMaxJobs = 8;

// The same form with autonomous wavefronts (conv_wino_auto_kernel.h): output layers and tiles per wavefront
// item, wavefronts per workgroup, and the floats of the transformed kernels of one layer block and one step of
// four input layers, in LDS and in memory: [8 position pairs][64 lanes][4] with the 4 = (position parity, row
// block of 16 layers); lane = k * 16 + layer % 16.
constexpr int kWinoAutoLayers = 32, kWinoAutoTiles = 16, kWinoAutoWaves = 8;
constexpr int kWinoAutoStep = 8 * 64 * 4;

constexpr int kConv7TileRows = 2, kConv7TileCols = 16;   // output pixels per wavefront tile
size_t conv7s2c3_lds_bytes(int NW, int TM);

}  // namespace mfma
}  // namespace sq
