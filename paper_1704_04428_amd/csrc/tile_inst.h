// Body of one tile-kernel translation unit.  The including file defines
//   MCMK_KS    kernel side (1 to 7)
//   MCMK_BF16  0: fp32 operands, 1: bf16 operands
// and gets run_tile_<type>_k<KS>() with every tile shape of kTileShapes instantiated.
#include <atomic>

#include "tile_dispatch.h"
#if MCMK_BF16
#include "kn2row_tile_bf16.h"
#endif

// bf16 operands in [C][H][W] order with stride 2 and a kernel side of 5 or more: the staging gather
// of the large strided tile needs more registers than the two layouts with 7 position blocks per
// wave leave free, so only the 2 x 4 wave layout is built (the host never picks the others).
#define MCMK_STRIDED_BF16_NCHW_WIDE_ONLY (MCMK_BF16 && MCMK_KS >= 5)

namespace mcmk {
namespace {

template <int TH, int TW, int WM, int WP, int CCH = 16, bool CL = false, int KG = 1, int ST = 1, int RB = 1, int VQL = CCH / 4, bool V4 = false>
int launch_shape(const TileRequest &rq)
{
    TileArgs a = rq.args;
    a.tiles_x = (a.p + TW - 1) / TW;
    a.tiles_y = (a.q + TH - 1) / TH;
    a.row_tiles = (a.row_groups * a.mb_per_group + WM * RB - 1) / (WM * RB);
    a.div_row_tiles = make_fast_div((uint32_t)a.row_tiles);
    a.div_tiles_x = make_fast_div((uint32_t)a.tiles_x);
    a.div_tiles_y = make_fast_div((uint32_t)a.tiles_y);
    const long long blocks = (long long)a.n * a.tiles_x * a.tiles_y * a.row_tiles * a.csplit;
    if (blocks < 1 || blocks >= (1LL << 31) || (a.csplit & (a.csplit - 1)) != 0) return 3;
#if MCMK_BF16
    using S = TileShapeBf16<MCMK_KS, TH, TW, WM, WP, ST, KG>;
    constexpr size_t kLds = S::kLdsBytes;            // every channel group has its own pair of buffers
    static_assert(kLds <= 160 * 1024, "the tile does not fit the LDS of a compute unit");
    if (kLds > 65536) {
        // more than 64 KiB of dynamic LDS has to be allowed per kernel, once per device (two threads that both find
        // the flag clear both set the attribute, which is harmless; the flag itself is read and written atomically)
        static std::atomic<bool> allowed[64] = {};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 1;
        if (!allowed[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(&kn2row_tile_bf16<MCMK_KS, TH, TW, WM, WP, CL, ST, RB, KG>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds) != hipSuccess)
                return 1;
            allowed[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL((kn2row_tile_bf16<MCMK_KS, TH, TW, WM, WP, CL, ST, RB, KG>), dim3((unsigned)blocks), dim3(S::kThreads * KG),
                       kLds, rq.stream, a);
#else
    using S = TileShape<MCMK_KS, TH, TW, WM, WP, CCH, KG, ST, VQL, CL>;
    static_assert(S::kLdsBytes <= 160 * 1024, "the tile does not fit the LDS of a compute unit");
    if (S::kLdsBytes > 65536) {
        // more than 64 KiB of dynamic LDS has to be allowed per kernel, once per device (two threads that both find
        // the flag clear both set the attribute, which is harmless; the flag itself is read and written atomically)
        static std::atomic<bool> allowed[64] = {};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 1;
        if (!allowed[dev].load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(&kn2row_tile_f32<MCMK_KS, TH, TW, WM, WP, CCH, CL, KG, ST, VQL, V4>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::kLdsBytes) != hipSuccess)
                return 1;
            allowed[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL((kn2row_tile_f32<MCMK_KS, TH, TW, WM, WP, CCH, CL, KG, ST, VQL, V4>), dim3((unsigned)blocks), dim3(S::kThreads),
                       S::kLdsBytes, rq.stream, a);
#endif
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace

#define MCMK_CAT2(a, b, c) a##b##c
#define MCMK_CAT(a, b, c) MCMK_CAT2(a, b, c)
#if MCMK_BF16
#define MCMK_FN MCMK_CAT(run_tile_bf16, _k, MCMK_KS)
#else
#define MCMK_FN MCMK_CAT(run_tile_f32, _k, MCMK_KS)
#endif

int MCMK_FN(const TileRequest &rq)
{
    if (rq.stride == 2) {
        if (rq.shape < 0 || rq.shape >= kStridedShapes) return 2;
#if !MCMK_BF16 && MCMK_KS >= 3 && (MCMK_KS & 1)
        if (rq.lean) {
            // up to four channels (a strided RGB first layer): one staged channel quad instead of four
            switch (rq.shape) {
            case 0: return launch_shape<14, 14, 4, 2, 16, false, 1, 2, 1, 1>(rq);
            case 1: return launch_shape<14, 14, 2, 4, 16, false, 1, 2, 1, 1>(rq);
            default: return 2;
            }
        }
#endif
        switch (rq.shape + (rq.channels_last ? kStridedShapes : 0)) {
#if !MCMK_STRIDED_BF16_NCHW_WIDE_ONLY
        case 0: return launch_shape<14, 14, 4, 2, 16, false, 1, 2>(rq);
        case 2: return launch_shape<14, 14, 1, 4, 16, false, 1, 2>(rq);
#endif
        case 1: return launch_shape<14, 14, 2, 4, 16, false, 1, 2>(rq);
        case 3: return launch_shape<14, 14, 4, 2, 16, true, 1, 2>(rq);
        case 4: return launch_shape<14, 14, 2, 4, 16, true, 1, 2>(rq);
        case 5: return launch_shape<14, 14, 1, 4, 16, true, 1, 2>(rq);
        default: return 2;
        }
    }
    if (rq.stride != 1) return 2;
#if !MCMK_BF16 && MCMK_KS >= 3 && (MCMK_KS & 1)
    if (rq.lean) {
        // up to four channels, [C][H][W] input: one staged channel quad instead of four (kernel sides 3, 5, 7)
        switch (rq.shape) {
        case 0: return launch_shape<14, 14, 4, 2, 16, false, 1, 1, 1, 1>(rq);
        case 3: return launch_shape<16, 16, 4, 2, 16, false, 1, 1, 1, 1>(rq);
        case 4: return launch_shape<16, 16, 2, 4, 16, false, 1, 1, 1, 1>(rq);
        default: return 2;
        }
    }
#endif
    if (rq.channels_last) {
        switch (rq.shape) {
        case 0: return launch_shape<14, 14, 4, 2, 16, true>(rq);
        case 1: return launch_shape<14, 14, 2, 4, 16, true>(rq);
        case 2: return launch_shape<14, 14, 1, 4, 16, true>(rq);
        case 3: return launch_shape<16, 16, 4, 2, 16, true>(rq);
        case 4: return launch_shape<16, 16, 2, 4, 16, true>(rq);
        case 5: return launch_shape<16, 16, 1, 4, 16, true>(rq);
#if MCMK_KS <= 3
        case 6: return launch_shape<14, 14, 1, 4, 16, true, 4>(rq);
#endif
#if MCMK_KS == 1
        case 7: return launch_shape<1, 224, 4, 2, 32, true>(rq);
#endif
#if MCMK_KS <= 5
        case 13: return launch_shape<7, 7, 1, 4, 16, true>(rq);
#endif
#if !MCMK_BF16 && MCMK_KS <= 3
        case 14: return launch_shape<14, 28, 4, 4, 16, true>(rq);
        case 16: return launch_shape<7, 7, 1, 4, 16, true, 2>(rq);
#endif
#if MCMK_BF16 && MCMK_KS <= 3
        case 8: return launch_shape<14, 14, 4, 2, 16, true, 1, 1, 2>(rq);
        case 9: return launch_shape<14, 14, 2, 4, 16, true, 1, 1, 2>(rq);
        case 10: return launch_shape<14, 14, 4, 1, 16, true, 1, 1, 2>(rq);
        case 12: return launch_shape<4, 56, 4, 2, 16, true, 1, 1, 2>(rq);
        case 17: return launch_shape<8, 14, 4, 1, 16, true, 1, 1, 2>(rq);
        case 18: return launch_shape<4, 28, 4, 1, 16, true, 1, 1, 2>(rq);
#if MCMK_KS == 1
        case 11: return launch_shape<1, 224, 4, 2, 32, true, 1, 1, 2>(rq);
#endif
#endif
        default: return 2;
        }
    }
    switch (rq.shape) {
    case 0: return launch_shape<14, 14, 4, 2>(rq);
    case 1: return launch_shape<14, 14, 2, 4>(rq);
    case 2: return launch_shape<14, 14, 1, 4>(rq);
    case 3: return launch_shape<16, 16, 4, 2>(rq);
    case 4: return launch_shape<16, 16, 2, 4>(rq);
    case 5: return launch_shape<16, 16, 1, 4>(rq);
#if MCMK_KS <= 3
    case 6: return launch_shape<14, 14, 1, 4, 16, false, 4>(rq);   // four channel groups in the workgroup
#endif
#if MCMK_KS == 1
    case 7:                                                // plain GEMM: deeper chunks, fewer barriers
#if !MCMK_BF16
        // a plane of whole 16-byte vectors (the operand itself is 16-byte aligned): the vector staging plan
        if (rq.args.h == 1 && rq.args.w % 4 == 0 && (reinterpret_cast<uintptr_t>(rq.args.in) & 15u) == 0)
            return launch_shape<1, 224, 4, 2, 32, false, 1, 1, 1, 8, true>(rq);
#endif
        return launch_shape<1, 224, 4, 2, 32>(rq);
#endif
#if MCMK_KS <= 5
    case 13: return launch_shape<7, 7, 1, 4>(rq);                           // quarter tiles for small images
#endif
#if !MCMK_BF16 && MCMK_KS <= 3
    case 14: return launch_shape<14, 28, 4, 4>(rq);                         // a pair of tiles under sixteen waves
    case 16: return launch_shape<7, 7, 1, 4, 16, false, 2>(rq);             // quarter tiles, two channel groups
#if MCMK_KS != 2                // the 15 x 29 halo tile of a 2 x 2 kernel has no regular staging plan for 512 threads: it would spill
    case 15: return launch_shape<14, 28, 2, 4, 16, false, 2>(rq);           // ... split into two channel groups
#endif
#endif
#if MCMK_BF16 && MCMK_KS <= 3
    case 8: return launch_shape<14, 14, 4, 2, 16, false, 1, 1, 2>(rq);      // two row blocks per wave
    case 9: return launch_shape<14, 14, 2, 4, 16, false, 1, 1, 2>(rq);
    case 10: return launch_shape<14, 14, 4, 1, 16, false, 1, 1, 2>(rq);     // a wave owns every position block
    case 12: return launch_shape<4, 56, 4, 2, 16, false, 1, 1, 2>(rq);      // whole image rows
    case 17: return launch_shape<8, 14, 4, 1, 16, false, 1, 1, 2>(rq);      // four waves: two workgroups per compute unit
    case 18: return launch_shape<4, 28, 4, 1, 16, false, 1, 1, 2>(rq);
#if MCMK_KS == 1
    case 11: return launch_shape<1, 224, 4, 2, 32, false, 1, 1, 2>(rq);
#endif
#endif
    default: return 2;
    }
}

}  // namespace mcmk
