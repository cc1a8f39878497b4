// Host-side helpers of libowt: error reporting, descriptor checks, tile planning.
#pragma once
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/owt.h"
#include "owt_common.hpp"

namespace owt {

owt_status fail(owt_status st, const char *fmt, ...);
void clear_error();

inline bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

// Tile shapes the implicit-GEMM kernel is instantiated for.
struct TileInfo { int id, WM, WN, BK; float eff; int BM; };
// ids 0..3 exist for the gather kernel; the stride-1 direct kernel has 128x128, 128x64, 256x64 and
// 128x64H (four wavefronts of 32x64 instead of two of 64x64: twice the wavefronts for small layers);
// 512x64 and 256x64P (four wavefronts of 128x64 / 64x64, 32-channel chunks) are the pipelined bf16-MFMA kernel only
enum { TILE_128x128 = 0, TILE_128x64 = 1, TILE_64x128 = 2, TILE_64x64 = 3, NUM_TILES = 4, TILE_256x64 = 4, TILE_128x64H = 5, TILE_128x128H = 6, TILE_512x64 = 7, TILE_256x64P = 8 };
extern const TileInfo kTiles[NUM_TILES + 5];

bool fill_geom(Geom &g, int N, int C, int H, int W, int K, int R, int S, int sh, int sw, int ph, int pw);

// One entry per (pass, storage type); defined in igemm_inst.hip, built once per pair.
typedef hipError_t (*LaunchFn)(int tile, int va, int vb, const GemmParams &p, hipStream_t s);
hipError_t owt_launch_fwd_f32(int, int, int, const GemmParams &, hipStream_t);
hipError_t owt_launch_fwd_bf16(int, int, int, const GemmParams &, hipStream_t);
hipError_t owt_launch_data_f32(int, int, int, const GemmParams &, hipStream_t);
hipError_t owt_launch_data_bf16(int, int, int, const GemmParams &, hipStream_t);
hipError_t owt_launch_filter_f32(int, int, int, const GemmParams &, hipStream_t);
hipError_t owt_launch_filter_bf16(int, int, int, const GemmParams &, hipStream_t);

// Panel-resident stride-1 kernel (dconv_inst.hip), forward and backward-data.
hipError_t owt_launch_dconv_fwd_f32(int tile, int pr, const GemmParams &, hipStream_t);
hipError_t owt_launch_dconv_fwd_bf16(int tile, int pr, const GemmParams &, hipStream_t);
hipError_t owt_launch_dconv_data_f32(int tile, int pr, const GemmParams &, hipStream_t);
hipError_t owt_launch_dconv_data_bf16(int tile, int pr, const GemmParams &, hipStream_t);

// Panel-resident stride-1 kernels on the bf16 MFMA (dconv_bf16_inst.hip, dconv_bf16p.hpp for the 512x64 tile).  The backward-data
// launcher first writes the flipped, transposed filters to the front of `ws`.
hipError_t owt_launch_dconv16_fwd(int tile, int pr, const GemmParams &, hipStream_t);
hipError_t owt_launch_dconv16_data(int tile, int pr, const GemmParams &, void *ws, hipStream_t);

// Direct filter-gradient kernel (dfilter_inst.hip): wavefront grid WK x WC (32 filters x 32
// channels each), exactly tmax taps per work-group, LDS panel of prf padded-image pixels.
// occ = work-groups per CU; aligned = the 32-pixel chunks are cut per image (taken only when the short
// last chunk of an image wastes under 4 %): no chunk then spans the padding rows between two images, so
// variant 3 gets by with a 64-row panel where variant 1 needs 192, and three work-groups fit a CU.
struct DFilterVariant { int WK, WC, tmax, prf, occ, aligned; };
constexpr int kNumDFilterVariants = 4;
constexpr DFilterVariant kDFilterVariants[kNumDFilterVariants] = {
    {4, 1, 9, 128, 2, 0}, {2, 2, 5, 192, 2, 0}, {2, 2, 9, 128, 2, 0}, {2, 2, 5, 64, 3, 1}};
hipError_t owt_launch_dfilter_f32(int variant, const GemmParams &, hipStream_t);
hipError_t owt_launch_dfilter_bf16(int variant, const GemmParams &, hipStream_t);

// Filter-gradient kernel with the pixel reduction split inside the work-group and operands streamed straight
// into LDS (dfilter2_inst.hip; fp32 storage, dz not masked by the call): WK filter blocks of 32 x WP pixel
// parts of 32 pixels, 32 channels, tmax taps per work-group, prows panel rows per LDS stage; one work-group of
// 8 wavefronts per CU.  SW > 0: all taps of an R x SW filter on padded rows exactly WPC pixels wide (both
// compile-time constants of the kernel); SW == 0: one filter row of tmax taps per work-group, any row width.
struct DFilter2Variant { int WK, WP, tmax, SW, WPC, prows; };
constexpr int kNumDFilter2Variants = 3;
constexpr DFilter2Variant kDFilter2Variants[kNumDFilter2Variants] = {
    {2, 4, 9, 3, 15, 256}, {4, 2, 9, 3, 15, 192}, {2, 4, 5, 0, 0, 320}};
constexpr int kDFilter2FirstTile = 10;      // owt_test_force_variant: tile numbers 10.. name these variants
hipError_t owt_launch_dfilter2_f32(int variant, const GemmParams &, hipStream_t);

// bf16-MFMA direct filter-gradient kernel (dfilter_bf16_inst.hip): work-group tile 32*KB*WK filters x
// 32*WC channels, 64-pixel chunks, tmax taps per work-group, prf panel rows, occ work-groups per CU.
// Variants 4 and 5 cover the tiles of 0 and 2 with twice the wavefronts of half the filter block each
// (two wavefronts per SIMD instead of one: more LDS reads per MFMA, but one wavefront's waits are
// filled by the other), variant 6 the tile of 3 with twelve wavefronts of one filter block, variant 7 a
// 128 x 192 tile (twelve wavefronts of two filter blocks; 192 channels in one tile, 156 KB of LDS).  Sixteen
// wavefronts of one block on the 128 x 128 tile were slower again: the LDS reads then bound the kernel.
struct DFilter16Variant { int WK, WC, KB, tmax, prf, occ; };
constexpr int kNumDFilter16Variants = 8;
constexpr DFilter16Variant kDFilter16Variants[kNumDFilter16Variants] = {
    {1, 4, 4, 3, 128, 1}, {2, 2, 2, 5, 224, 1}, {1, 2, 4, 3, 128, 2}, {3, 2, 2, 5, 224, 1}, {2, 4, 2, 3, 128, 1}, {2, 2, 2, 3, 128, 2},
    {6, 2, 1, 5, 224, 1}, {2, 6, 2, 3, 128, 1}};
constexpr int kDFilter16BP = 64;
hipError_t owt_launch_dfilter16(int variant, const GemmParams &, hipStream_t);

// The same filter gradient with the operands streamed straight into LDS (dfilter16b_inst.hip; unmasked dz, maps
// of at most 1024 padded positions, chunks that touch at most two images).  SW > 0: all R x SW taps per
// work-group on padded rows of WPC pixels; SW == 0: one filter row of tmax taps per work-group.  One work-group
// per CU.  The test hook numbers these variants from kDFilter16bFirstTile.
struct DFilter16bVariant { int WK, WC, KB, tmax, SW, WPC, prf; };
constexpr int kNumDFilter16bVariants = 7, kDFilter16bFirstTile = 30;
constexpr DFilter16bVariant kDFilter16bVariants[kNumDFilter16bVariants] = {
    {2, 4, 2, 3, 0, 0, 128}, {2, 6, 2, 3, 0, 0, 128}, {2, 4, 4, 3, 0, 0, 128}, {2, 2, 4, 3, 0, 0, 128},
    {6, 2, 1, 5, 0, 0, 224}, {3, 2, 2, 5, 0, 0, 224}, {2, 2, 3, 5, 0, 0, 224}};
hipError_t owt_launch_dfilter16b(int variant, const GemmParams &, hipStream_t);

// Dense GEMM kernel of the fully-connected shard (fcgemm_inst.hip; fp32 storage, reduction length a
// multiple of 32): WM x WN wavefronts of MB x NB accumulator blocks of 32 x 32, occ work-groups per CU.
// When the pass masks dy by y > 0 or wants the bias gradient, a small kernel first writes dz to `dz`
// ([N][O_local] floats of workspace) and the bias gradient to its place.
// NS = stages of the LDS ring ((BM + BN) * 128 bytes each).
struct FcTile { int WM, WN, MB, NB, NS, occ; };
constexpr int kNumFcTiles = 4;
constexpr FcTile kFcTiles[kNumFcTiles] = {{2, 2, 2, 2, 3, 1}, {2, 2, 1, 2, 3, 2}, {2, 2, 2, 1, 3, 2}, {2, 2, 1, 1, 3, 3}};
constexpr int kFcPairTile = 3;      // the tile of the launch that runs both backward products
hipError_t owt_launch_fcgemm(int pass, int tile, const GemmParams &, float *dz, hipStream_t);
// Both backward products on one dz (data pass params first): two launches, or one when `fused`
// (both with tile kFcPairTile, neither split).
hipError_t owt_launch_fcgemm_bwd(int tile_d, int tile_f, bool fused, const GemmParams &pd, const GemmParams &pf, float *dz,
                                 hipStream_t);

// bf16-MFMA small-channel strided forward kernel (sconv_bf16_inst.hip); w2 = K x KSLOTS bf16 values of workspace.
struct SConv16Geom;
hipError_t owt_launch_sconv16(const GemmParams &, const SConv16Geom &, int ktiles, int nwg, void *w2, hipStream_t);

// bf16-MFMA small-channel strided filter-gradient kernel (sfilter_bf16_inst.hip).
struct SFilter16Geom;
hipError_t owt_launch_sfilter16(const GemmParams &, const SFilter16Geom &, int ktiles, hipStream_t);

// Small-channel strided filter-gradient kernel (sfilter_inst.hip).
struct SFilterGeom;
hipError_t owt_launch_sfilter_f32(const GemmParams &, const SFilterGeom &, int ktiles, hipStream_t);
hipError_t owt_launch_sfilter_bf16(const GemmParams &, const SFilterGeom &, int ktiles, hipStream_t);

// Small-channel strided forward kernel (sconv_inst.hip); w2 is K x KSLOTS floats of workspace.
struct SConvGeom;
hipError_t owt_launch_sconv_f32(const GemmParams &, const SConvGeom &, int ktiles, int nwg, float *w2, hipStream_t);
hipError_t owt_launch_sfilter16b(const GemmParams &, const SFilter16Geom &, int ktiles, hipStream_t);
hipError_t owt_launch_sfilter2_f32(const GemmParams &, const SFilterGeom &, int ktiles, hipStream_t);
hipError_t owt_launch_sconv2_f32(const GemmParams &, const SConvGeom &, int ktiles, int nwg, float *w2, hipStream_t);
hipError_t owt_launch_sconv_bf16(const GemmParams &, const SConvGeom &, int ktiles, int nwg, float *w2, hipStream_t);

}  // namespace owt
