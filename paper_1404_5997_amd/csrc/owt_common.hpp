// Shared host/device definitions of libowt (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace owt {

// Exact unsigned division of any n < 2^31 by a fixed d >= 1 with one 64-bit
// multiply: l = ceil(log2 d), m = ceil(2^(31+l) / d) fits 32 bits and
// floor(n/d) == (n*m) >> (31+l)   (round-up method of Granlund & Montgomery).
struct FastDiv {
    uint32_t m, sh, d;
    __host__ void set(uint32_t dv)
    {
        d = dv;
        uint32_t l = 0;
        while ((1ull << l) < dv) l++;
        sh = 31 + l;
        m = (uint32_t)(((1ull << sh) + dv - 1) / dv);
    }
    __host__ __device__ __forceinline__ uint32_t div(uint32_t n) const
    {
        return (uint32_t)(((uint64_t)n * m) >> sh);
    }
};

// Geometry of one convolution seen as a GEMM.  Fully-connected layers are the
// H = W = R = S = 1 case.
struct Geom {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
    int bf16;                 // storage type of the tensors is bf16 (host-side planning only)
    int masked;               // the backward call applies a ReLU mask to dy itself (host-side planning only)
    FastDiv dC, dS, dK, dQ, dPQ, dW, dHW, dsh, dsw;
};

struct GemmParams {
    Geom g;
    int M, Ncols, Kd;        // GEMM extents of this pass
    const void *a, *b;       // tensors the A and B operands are gathered from
    const void *mask;        // forward output y (ReLU mask of the dz operand) or null
    const void *xmask;       // bwd-data only: the layer's input; dx is zeroed where it is <= 0 (or null)
    void *out;               // result tensor (used when splits == 1)
    float *partial;          // [splits][M][Ncols] fp32 (used when splits > 1)
    const float *bias;       // forward epilogue
    float alpha, beta;       // filter-gradient epilogue
    float *dbias;            // bias gradient (filter pass), may be null
    float *dbias_partial;    // [splits][M] fp32 when splits > 1
    int splits, ksteps, ksteps_per_split;
    int tiles_m, tiles_n;
    unsigned flags;
    // Direct (panel-resident) stride-1 kernel only: the gathered tensor is Hi x Wi x Cred per
    // image, the result Ho x Wo x Ncols; output pixel (ho,wo) reads input pixels
    // (ho-pah+r, wo-paw+s), r < R, s < S.
    int Hi, Wi, Ho, Wo, pah, paw, Cred;
    FastDiv dWo, dHoWo;
    // Direct filter-gradient kernel only: the input seen in zero-padded coordinates
    // (Hp = H + 2*pad_h rows of Wp = W + 2*pad_w pixels per image); taps are handled
    // `taps` at a time, either all R*S at once (groups == 1) or one filter row per group.
    int Hp, Wp, taps, groups, ctiles;
    FastDiv dWp, dHpWp;
    // Dense kernel of the fully-connected shard only: row pitches of the A and B operands, and the true
    // reduction length (the reduction runs over ksteps * 32 >= kvalid indices; A is zero beyond kvalid)
    int lda, ldb, kvalid;
    // cpi > 0: the pixel chunks never straddle two images (cpi chunks per image, the last one short)
    int cpi;
    FastDiv dCpi;
};

// chunks of 64 pixels one work-group of the streamed bf16 filter-gradient kernel may walk (its per-chunk LDS table)
constexpr int kDFilter16bMaxChunks = 256;

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even; NaN stays NaN.  gfx950 has the conversion in hardware
// (v_cvt_pk_bf16_f32, two values per instruction).
typedef __bf16 owt_bf16x2 __attribute__((ext_vector_type(2)));
typedef float owt_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    const owt_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, owt_bf16x2));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)(f32x2_to_bf16x2(f, 0.f) & 0xffffu); }

__device__ __forceinline__ float4 load4(const float *p, int off) { return *(const float4 *)(p + off); }
__device__ __forceinline__ float4 load4(const bf16_t *p, int off)
{
    const uint2 v = *(const uint2 *)(p + off);
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                       __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
}
// Work-group numbering of the filter-gradient kernels whose pixel range is split over work-groups.  The tiles of
// one split all read the same dz and x chunks (a dz chunk once per channel tile and filter row, an x chunk once per
// filter tile), so they should run at the same time behind the same L2.  The grid is one-dimensional with
// owt_split_major_grid(tiles, splits) work-groups, work-group L runs on XCD L % 8, and the (split, tile) pairs,
// split-major, are dealt to the XCDs in eight contiguous runs of equal length (+-1): an XCD works through whole
// splits, tile after tile.  (Numbered tile-major over a two-dimensional grid, the few tiles of a split land on
// different XCDs and every chunk is fetched once per tile: the counters showed 3-7 times the compulsory bytes.)
// Returns false for the padding work-groups at the end of the grid, which must exit before any barrier.
__host__ __device__ inline int owt_split_major_grid(int tiles, int splits) { return 8 * ((tiles * splits + 7) / 8); }
__device__ __forceinline__ bool owt_split_major_wg(int ntiles, int splits, int &tile, int &split)
{
    const int total = ntiles * splits, xcd = blockIdx.x & 7, jx = blockIdx.x >> 3;
    if (jx >= (total >> 3) + (xcd < (total & 7) ? 1 : 0)) return false;
    const int pair = xcd * (total >> 3) + min(xcd, total & 7) + jx;
    split = pair / ntiles;
    tile = pair - split * ntiles;
    return true;
}

// 16 bytes through a raw buffer descriptor: a byte offset outside [0, bytes) reads as zeros without touching
// memory, so bounds need no branch, no exec masking and no zeroing of the destination.
typedef unsigned int owt_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t owt_make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float4 buffer_load4(__amdgpu_buffer_rsrc_t rsrc, unsigned voffset_bytes)
{
    const owt_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voffset_bytes, 0, 0);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}

typedef int owt_i32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptor (base, byte count) in scalar registers.
__device__ __forceinline__ owt_i32x4 make_rsrc(const void *base, unsigned bytes)
{
    const unsigned long long a = (unsigned long long)base;
    owt_i32x4 r;
    r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r.y = __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu));
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);
    r.w = 0x00020000;
    return r;
}

// 16 bytes per lane from the buffer straight into LDS: lane l's piece lands at LDS byte address lds_base + 16 l;
// a lane whose offset is outside the descriptor's range writes zeros.  (m0 carries the LDS base; the s_nop is
// the wait state the hardware wants between a scalar write of m0 and the load that reads it.)
__device__ __forceinline__ void buffer_load16_to_lds(owt_i32x4 rsrc, unsigned voffset_bytes, unsigned lds_base)
{
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base);       // wave-uniform by construction
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
                 : : "v"(voffset_bytes), "s"(rsrc), "s"(m0v) : "memory", "m0");
}

__device__ __forceinline__ float load1(const float *p, int off) { return p[off]; }
__device__ __forceinline__ float load1(const bf16_t *p, int off) { return bf16_to_f32(p[off].bits); }

__device__ __forceinline__ void store1(float *p, size_t off, float v) { p[off] = v; }
__device__ __forceinline__ void store1(bf16_t *p, size_t off, float v) { p[off].bits = f32_to_bf16(v); }
__device__ __forceinline__ void store2(float *p, size_t off, float v0, float v1)
{
    *(float2 *)(p + off) = make_float2(v0, v1);
}
__device__ __forceinline__ void store2(bf16_t *p, size_t off, float v0, float v1)
{
    *(uint32_t *)(p + off) = f32x2_to_bf16x2(v0, v1);
}

}  // namespace owt
