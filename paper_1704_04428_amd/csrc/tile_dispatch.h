// Host-side interface between the C ABI and the tile-kernel instantiations.  Every (operand type,
// kernel side) pair is compiled in a translation unit of its own (tile_f32_k3.hip, ...), so the
// library builds in parallel; this header is what they share.
#pragma once
#include <hip/hip_runtime.h>

#include "kn2row_tile.h"

namespace mcmk {

// Tile shapes every instantiation file provides: tile rows x columns, waves along the rows and along
// the positions, the number of channel groups (in-workgroup split of the contraction; fp32 only) and
// the 16-row blocks per wave (2: bf16 operands, unit stride, kernel sides up to 3).
// Index kGemmShape / kWideGemmShape are the plain-GEMM shapes (1 x 224 positions, 32-channel chunks)
// and exist for kernel side 1 only.  Stride 2 is instantiated for the first kStridedShapes entries
// (the 14 x 14 tiles without channel groups: the strided input tile of a larger output tile would not
// fit the LDS).
struct TileShapeDesc {
    int th, tw, wm, wp, kg, rb;
};
constexpr TileShapeDesc kTileShapes[] = {
    {14, 14, 4, 2, 1, 1}, {14, 14, 2, 4, 1, 1}, {14, 14, 1, 4, 1, 1}, {16, 16, 4, 2, 1, 1}, {16, 16, 2, 4, 1, 1}, {16, 16, 1, 4, 1, 1},
    {14, 14, 1, 4, 4, 1}, {1, 224, 4, 2, 1, 1},
    {14, 14, 4, 2, 1, 2}, {14, 14, 2, 4, 1, 2}, {14, 14, 4, 1, 1, 2}, {1, 224, 4, 2, 1, 2},
    // whole image rows of a 56-wide image: 224 positions = 14 blocks exactly, and a row of outputs is
    // one contiguous run in memory (what the [M][Q][P] output of the bf16 kernel, whose closing
    // write is a quarter of its time, gains from)
    {4, 56, 4, 2, 1, 2},
    // small images (a single 27 x 27 or 28 x 28 image has four 14 x 14 tiles): quarter tiles, one position
    // block per wave, so that a layer with few tiles still spreads over the chip
    {7, 7, 1, 4, 1, 1},
    // two 14 x 14 tiles side by side under sixteen waves (fp32 operands, kernel sides up to 3): 392 positions
    // are 24.5 blocks, so 2 % of the matrix work is padding where a single 14 x 14 tile (12.25 blocks in 13)
    // has 6 %; each SIMD gets one wave with 7 blocks and three with 6
    {14, 28, 4, 4, 1, 1},
    // the same pair with two channel groups of eight waves, 32 rows per workgroup: twice the workgroups for layers
    // that have too few pairs (28 x 28 images), and a SIMD carries 12.5 blocks per chunk where single tiles give it 13
    {14, 28, 2, 4, 2, 1},
    // quarter tiles with two channel groups of four waves: the split of the channel sum for single small images with
    // hundreds of channels, without the zero fill and the atomics of the two-workgroup split
    {7, 7, 1, 4, 2, 1},
    // bf16, two row blocks per wave, FOUR waves (128 rows x 112 positions = 7 blocks, all owned by every wave): a
    // workgroup is one wave per SIMD and needs under 256 registers, so two of them share a compute unit, each behind
    // its own barrier -- when one waits for its staged chunk the other has the matrix pipe.  8 x 14 for images whose
    // sides are multiples of 8 and 14 (56 x 56), 4 x 28 for 28-wide ones.
    {8, 14, 4, 1, 1, 2}, {4, 28, 4, 1, 1, 2},
};
constexpr int kConvShapes = 7;
constexpr int kGemmShape = 7;
constexpr int kStridedShapes = 3;
constexpr int kMaxKernelSide = 7;      // kernel sides 1..7 are instantiated
// shapes beyond the first seven (bf16 shapes with two row blocks per wave, quarter tiles): convolution shapes ...
constexpr int kWideConvShapes = 8;
constexpr int kWideConvShape[kWideConvShapes] = {8, 9, 10, 12, 13, 14, 15, 16};
constexpr int kWideGemmShape = 11;     // ... and the plain-GEMM shape
constexpr int kLaterConvShapes = 2;    // shapes added after those (their menu indices start at 30)
constexpr int kLaterConvShape[kLaterConvShapes] = {17, 18};
constexpr int kPairTileShape = 14;     // the 14 x 28 shapes: this one and the next (two channel groups)

struct TileRequest {
    TileArgs args;       // tiles_x, tiles_y and row_tiles are filled in by the launcher
    int shape;           // index into kTileShapes
    bool channels_last;  // input [n][h][w][c], output [n][q][p][rows] (kn2col); convolution shapes only
    int stride;          // 1, or 2 with a shape index below kStridedShapes
    bool lean;           // fp32, up to four channels, [C][H][W], odd kernel side >= 3, shapes 0 / 3 / 4 (stride 2: 0 / 1):
                         // the instantiation that stages and multiplies one channel quad per chunk instead of four
    hipStream_t stream;
};

// Return hipSuccess-or-not as 0 / 1; 2 when the shape index is not instantiated, 3 when the grid is too large.
int run_tile_f32_k1(const TileRequest &);
int run_tile_f32_k2(const TileRequest &);
int run_tile_f32_k3(const TileRequest &);
int run_tile_f32_k4(const TileRequest &);
int run_tile_f32_k5(const TileRequest &);
int run_tile_f32_k6(const TileRequest &);
int run_tile_f32_k7(const TileRequest &);
int run_tile_bf16_k1(const TileRequest &);
int run_tile_bf16_k2(const TileRequest &);
int run_tile_bf16_k3(const TileRequest &);
int run_tile_bf16_k4(const TileRequest &);
int run_tile_bf16_k5(const TileRequest &);
int run_tile_bf16_k6(const TileRequest &);
int run_tile_bf16_k7(const TileRequest &);

}  // namespace mcmk
