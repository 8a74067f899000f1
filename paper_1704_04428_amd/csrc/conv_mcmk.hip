// libconv_mcmk: C ABI and launch logic.  See include/conv_mcmk.h for the contract.
#include "../../include/conv_mcmk.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "aux_kernels.h"
#include "selector_constants.h"
#include "tile_dispatch.h"

namespace {

using namespace mcmk;

constexpr int kNumCU = 256;   // MI355X

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

struct Dims {
    int q, p, mb, taps;
};

int validate(const conv_mcmk_desc *d, int variant, Dims *out)
{
    if (!d) return CONV_MCMK_ERR_NULL;
    if (d->n < 1 || d->c < 1 || d->h < 1 || d->w < 1 || d->m < 1 || d->k < 1 || d->pad < 0 || d->stride < 1)
        return CONV_MCMK_ERR_SHAPE;
    if ((long long)d->h + 2LL * d->pad < d->k || (long long)d->w + 2LL * d->pad < d->k) return CONV_MCMK_ERR_SHAPE;
    const long long q = ((long long)d->h + 2LL * d->pad - d->k) / d->stride + 1;
    const long long p = ((long long)d->w + 2LL * d->pad - d->k) / d->stride + 1;
    // the tile kernel addresses one image through a 32-bit byte offset with 2 GiB kept free: the "outside the image"
    // offset of 2 GiB plus a staging slot's channel (below 32) plus the first chunk beyond the data (below C + 32)
    // must not wrap
    if (((long long)d->c + 64) * d->h * d->w >= (1LL << 29)) return CONV_MCMK_ERR_SHAPE;
    const long long lim = 1LL << 31;
    const long long kk = (long long)d->k * d->k;
    if ((long long)d->c * d->h * d->w >= lim || (long long)d->m * q * p >= lim ||
        (long long)d->m * d->c * kk >= lim || (long long)d->c * kk * q * p >= lim * 4 ||
        kk * d->m * d->h * d->w >= lim * 4 || q >= 65536 * 16 || p >= 65536 * 16)
        return CONV_MCMK_ERR_SHAPE;
    if (d->dtype != CONV_MCMK_F32 && d->dtype != CONV_MCMK_BF16) return CONV_MCMK_ERR_UNSUPPORTED;
    // bf16 input in [C][H][W] order is staged two positions at a time: a plane of a single element
    // (for im2col: a patch matrix with a single column) is not taken
    if (d->dtype == CONV_MCMK_BF16 &&
        (((variant == CONV_MCMK_KN2ROW || variant == CONV_MCMK_KN2ROW_2PASS) && (long long)d->h * d->w < 2) ||
         (variant == CONV_MCMK_IM2COL && q * p < 2)))
        return CONV_MCMK_ERR_UNSUPPORTED;
    switch (variant) {
    case CONV_MCMK_KN2ROW:
    case CONV_MCMK_KN2COL:
        if (d->k > kMaxKernelSide || d->stride > 2) return CONV_MCMK_ERR_UNSUPPORTED;
        if (d->pad > 65535) return CONV_MCMK_ERR_SHAPE;
        // channels-last input is read in aligned 16-byte channel vectors: 4 floats or 8 bfloat16
        if (variant == CONV_MCMK_KN2COL && d->c % (d->dtype == CONV_MCMK_BF16 ? 8 : 4) != 0) return CONV_MCMK_ERR_UNSUPPORTED;
        break;
    case CONV_MCMK_KN2ROW_2PASS:
        break;
    case CONV_MCMK_IM2COL:
    case CONV_MCMK_IM2ROW:
        // the GEMM reads the patch matrix of one image through the same 32-bit byte offsets
        if (((long long)d->c * kk + 64) * q * p >= (1LL << 29)) return CONV_MCMK_ERR_SHAPE;
        if (variant == CONV_MCMK_IM2ROW && d->c % (d->dtype == CONV_MCMK_BF16 ? 8 : 4) != 0) return CONV_MCMK_ERR_UNSUPPORTED;
        break;
    case CONV_MCMK_DIRECT:
        if (d->dtype != CONV_MCMK_F32) return CONV_MCMK_ERR_UNSUPPORTED;
        break;
    default:
        return CONV_MCMK_ERR_UNSUPPORTED;
    }
    if (out) {
        out->q = (int)q;
        out->p = (int)p;
        out->mb = ceil_div(d->m, 16);
        out->taps = d->k * d->k;
    }
    return CONV_MCMK_OK;
}

// Tuning overrides (conv_mcmk_force_tile / conv_mcmk_force_gemm_tile): -1 none, -2 not yet taken from the environment.
std::atomic<int> g_force_tile{-2}, g_force_gemm_tile{-2};

int forced_index(std::atomic<int> &slot, const char *env_name)
{
    int v = slot.load(std::memory_order_relaxed);
    if (v == -2) {
        const char *text = getenv(env_name);
        int from_env = (text && text[0] >= '0' && text[0] <= '9') ? atoi(text) : -1;
        slot.compare_exchange_strong(v, from_env, std::memory_order_relaxed);    // a concurrent force call wins
        v = slot.load(std::memory_order_relaxed);
    }
    return v;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int launch_status()
{
    return hipGetLastError() == hipSuccess ? CONV_MCMK_OK : CONV_MCMK_ERR_DEVICE;
}

// Grid for a streaming kernel whose threads take `per_thread` items each in one sweep: as many workgroups of 256 as
// the items need (the loop inside the kernel covers whatever the 2^31 limit cuts off).
int stream_grid(size_t items, int per_thread)
{
    const size_t g = (items + (size_t)256 * per_thread - 1) / ((size_t)256 * per_thread);
    return (int)(g < 1 ? 1 : (g > 0x7fffffffull ? 0x7fffffffull : g));
}

int grid_for(size_t total, int block)
{
    size_t g = (total + block - 1) / block;
    const size_t cap = (size_t)kNumCU * 64;
    return (int)(g < 1 ? 1 : (g > cap ? cap : g));
}

// ------------------------------------------------------------------------------------------
// Tile-shape menu for the fused kernel and the cost estimate that picks from it.
struct Candidate {
    int shape;     // index into kTileShapes
    int csplit;    // 1 or 2 (the flat shapes of a staged variant's matrix product: also 4, 8 and 16)
    int th, tw, wm, wp, kg, rb;
};

Candidate candidate(int shape, int csplit)
{
    const TileShapeDesc &t = kTileShapes[shape];
    return Candidate{shape, csplit, t.th, t.tw, t.wm, t.wp, t.kg, t.rb};
}

int run_tile(int dtype, int ks, const TileRequest &rq)
{
    int rc = 2;
    if (dtype == CONV_MCMK_F32) {
        switch (ks) {
        case 1: rc = run_tile_f32_k1(rq); break;
        case 2: rc = run_tile_f32_k2(rq); break;
        case 3: rc = run_tile_f32_k3(rq); break;
        case 4: rc = run_tile_f32_k4(rq); break;
        case 5: rc = run_tile_f32_k5(rq); break;
        case 6: rc = run_tile_f32_k6(rq); break;
        case 7: rc = run_tile_f32_k7(rq); break;
        }
    } else {
        switch (ks) {
        case 1: rc = run_tile_bf16_k1(rq); break;
        case 2: rc = run_tile_bf16_k2(rq); break;
        case 3: rc = run_tile_bf16_k3(rq); break;
        case 4: rc = run_tile_bf16_k4(rq); break;
        case 5: rc = run_tile_bf16_k5(rq); break;
        case 6: rc = run_tile_bf16_k6(rq); break;
        case 7: rc = run_tile_bf16_k7(rq); break;
        }
    }
    return rc == 0 ? CONV_MCMK_OK : rc == 1 ? CONV_MCMK_ERR_DEVICE : rc == 3 ? CONV_MCMK_ERR_SHAPE : CONV_MCMK_ERR_UNSUPPORTED;
}

// What a fused call may apply to the finished sums before storing them.
struct Epilogue {
    const float *bias = nullptr;   // [M], device
    int relu = 0;
    bool any() const { return bias != nullptr || relu != 0; }
};

// Layers of up to four channels (an RGB first layer) have a leaner instantiation of three tile shapes: one channel
// quad of the only chunk is staged and multiplied instead of four.
bool lean_applies(const conv_mcmk_desc *d, int ks, int shape, int csplit, bool channels_last, int stride, int row_groups)
{
    return d->dtype == CONV_MCMK_F32 && d->c <= 4 && !channels_last && row_groups == 1 && csplit == 1 &&
           (ks == 3 || ks == 5 || ks == 7) &&
           ((stride == 1 && (shape == 0 || shape == 3 || shape == 4)) || (stride == 2 && (shape == 0 || shape == 1)));
}

// Floats between the copies of a result that the parts of a split contraction store: the result, rounded up to whole
// 16-byte items.
size_t partial_floats(size_t total) { return (total + 3) / 4 * 4; }

// One launch of the tile kernel: a convolution (ks x ks taps, row_groups = 1) or a plain GEMM
// (ks = 1 over a 1 x cols image, row_groups row planes of m rows each).
int launch_tile(const conv_mcmk_desc *d, const Dims &dm, int ks, int shape, int csplit, const void *in,
                const void *apk, float *out, int in_c, int in_h, int in_w, int out_q, int out_p, int pad,
                int row_groups, hipStream_t st, bool channels_last = false, int stride = 1,
                const Epilogue &ep = Epilogue(), float *partials = nullptr)
{
    TileRequest rq;
    TileArgs &a = rq.args;
    a.in = static_cast<const float *>(in);
    a.apk = static_cast<const float *>(apk);
    a.out = out;
    a.n = d->n;  a.c = in_c;  a.h = in_h;  a.w = in_w;
    a.q = out_q;  a.p = out_p;  a.pad = pad;
    a.m = d->m;  a.mb_per_group = dm.mb;  a.row_groups = row_groups;
    a.cg = ceil_div(in_c, d->dtype == CONV_MCMK_BF16 ? 32 : 16);
    a.tiles_x = a.tiles_y = a.row_tiles = 0;
    a.csplit = csplit;
    a.bias = ep.bias;
    a.relu = ep.relu;
    if (csplit > 1 && ep.any()) return CONV_MCMK_ERR_UNSUPPORTED;   // partial sums cannot be rectified
    rq.shape = shape;
    rq.channels_last = channels_last;
    rq.stride = stride;
    rq.lean = in_c == d->c && lean_applies(d, ks, shape, csplit, channels_last, stride, row_groups);
    rq.stream = st;
    a.part_stride = 0;
    const size_t total = (size_t)a.n * row_groups * d->m * out_q * out_p;
    if (csplit > 1 && partials && (csplit == 2 || csplit == 4 || csplit == 8 || csplit == 16)) {
        // every part stores its sums into a copy of its own (partial_floats() each), and a streaming pass adds the
        // copies in a fixed order: no zero fill, no atomics, the same bits on every run
        a.out = partials;
        a.part_stride = (long long)partial_floats(total);
        if (int rc = run_tile(d->dtype, ks, rq)) return rc;
        const dim3 grid(stream_grid(total / 4 + 1, 1)), block(256);
        const size_t stride = (size_t)a.part_stride;
        if (csplit == 2) hipLaunchKernelGGL(sum_parts_kernel<2>, grid, block, 0, st, partials, out, total, stride);
        else if (csplit == 4) hipLaunchKernelGGL(sum_parts_kernel<4>, grid, block, 0, st, partials, out, total, stride);
        else if (csplit == 8) hipLaunchKernelGGL(sum_parts_kernel<8>, grid, block, 0, st, partials, out, total, stride);
        else hipLaunchKernelGGL(sum_parts_kernel<16>, grid, block, 0, st, partials, out, total, stride);
        return launch_status();
    }
    if (csplit > 1) {
        // partial sums are added into the output, so it starts from zero (a fill kernel, not a
        // memset node, so the call can be captured into a graph)
        hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(total / 4 + 1, 256)), dim3(256), 0, st, out, total);
        if (int rc = launch_status()) return rc;
    }
    return run_tile(d->dtype, ks, rq);
}

// Estimated run time of a candidate in microseconds; the constants were fitted to measurements of
// every candidate on the benchmark layers, the layers of the networks the paper draws from and several hundred
// random layers per precision and layout.
//   - a block-step is one 16x16x4 MFMA, 32 cycles of a SIMD's matrix pipe (13.9 ns at 2.3 GHz);
//   - a workgroup's waves are dealt round-robin to the 4 SIMDs, its time is that of the SIMD with
//     the most position blocks; the busiest CU runs ceil(workgroups / 256) of them;
//   - a SIMD with a single resident wave cannot hide LDS and global latency (70 % pipe use
//     against 90 % with two or more);
//   - each launch pays a fixed prologue / epilogue; the channel split pays a zero fill plus two
//     device-scope atomic adds per output element.
long long workgroups(const conv_mcmk_desc *d, const Dims &dm, const Candidate &c)
{
    return (long long)d->n * ceil_div(dm.p, c.tw) * ceil_div(dm.q, c.th) * ceil_div(dm.mb, c.wm * c.rb) * c.csplit;
}

double tile_cost(const conv_mcmk_desc *d, const Dims &dm, const Candidate &c, int ks, bool channels_last = true)
{
    const bool bf16 = d->dtype == CONV_MCMK_BF16;
    // one set of constants per operand type and layout (selector_constants.h; fitted to timings of every menu entry
    // on random layers and on the layers of the networks the paper draws from: paper_1704_04428_amd/tuning)
    const CostParams &P = kCost[(bf16 ? 2 : 0) + (channels_last ? 1 : 0)];
    const long long wgs = workgroups(d, dm, c);
    const int npb = ceil_div(c.th * c.tw, 16);
    const int group_waves = c.wm * c.wp;
    const int waves = group_waves * c.kg;
    int simd_blocks[4] = {0, 0, 0, 0};
    for (int w = 0; w < waves; ++w) {
        const int g = w / group_waves;                                  // channel group, rotated by g
        const int wp = ((w % group_waves + g * c.wm) % group_waves) / c.wm;
        const int rem = npb % c.wp, pbw = ceil_div(npb, c.wp);
        simd_blocks[w % 4] += c.rb * ((rem == 0 || wp < rem) ? pbw : pbw - 1);
    }
    int simd_load = 0, simd_sum = 0;
    for (int i = 0; i < 4; ++i) {
        simd_load = simd_blocks[i] > simd_load ? simd_blocks[i] : simd_load;
        simd_sum += simd_blocks[i];
    }
    // chunks each wave works through (the channel groups of a workgroup share them out)
    const int chunks = ceil_div(ceil_div(ceil_div(d->c, bf16 ? 32 : 16), c.csplit), c.kg);
    // fp32: 4 MFMAs of 32 cycles per tap and 16-channel chunk (1 in the lean form); bf16: 1 MFMA of 16 cycles per tap
    // and 32-channel chunk
    const bool lean = ks == d->k && lean_applies(d, ks, c.shape, c.csplit, channels_last, d->stride, 1);
    const double steps = (double)chunks * ks * ks * (bf16 ? 0.5 : lean ? 1.0 : 4.0);
    const long long per_cu = (wgs + kNumCU - 1) / kNumCU;
    // workgroups a CU can hold (VGPRs: the bf16 kernels need more than 128 registers, so 8 waves per CU; fp32: the two
    // double-buffered halo tiles of 16 channels in 160 KB of LDS)
    int can_hold = (bf16 ? 8 : 16) / waves;        // sixteen-wave workgroups (channel groups, tile pairs): one
    if (can_hold < 1) can_hold = 1;
    // (the four-wave bf16 shape whose waves own all thirteen blocks of a 14 x 14 tile twice over needs 300 registers)
    if (bf16 && c.rb == 2 && c.wp == 1 && c.th * c.tw > 128) can_hold = 1;
    const int halo = ((c.th - 1) * d->stride + ks) * ((c.tw - 1) * d->stride + ks);
    if (!bf16) {
        const int fit = 163840 / (2 * c.kg * 16 * (((halo + 15) / 32) * 32 + 16) * 4);
        can_hold = can_hold < fit ? can_hold : fit;
        if (can_hold < 1) can_hold = 1;
    }
    const long long held = per_cu < can_hold ? per_cu : can_hold;
    const double waves_per_simd = (double)held * waves / 4.0;
    // a SIMD with a single resident wave cannot hide LDS and global latency
    double pipe_use = (waves_per_simd >= 2.0 ? P.pipe_multi : P.pipe_single) * P.type_scale;
    // bf16: the product is four times shorter than the fp32 one while a B fragment is four times larger, so LDS
    // reads, operand loads and the per-chunk hand-over weigh more.  An A fragment (1 KB from L1/L2 per wave) is reused
    // for the wave's position blocks, the staged tile for the workgroup's rows: few blocks per wave or few rows per
    // workgroup leave the load path, not the matrix pipe, as the limit
    if (bf16) {
        const double reuse_a = P.reuse_a0 + P.reuse_a1 * ceil_div(npb, c.wp);
        const double rows = 16.0 * c.wm * c.rb;
        const double reuse_b = rows / (rows + 16.0) / P.reuse_b;
        pipe_use *= (reuse_a < P.reuse_a_cap ? reuse_a : P.reuse_a_cap) * (reuse_b < 1.0 ? reuse_b : 1.0);
    }
    // a chunk of a large kernel is many taps long, so the hand-over between chunks weighs less
    if (ks > 3) pipe_use *= 1.0 + P.taps_gain * (1.0 - 9.0 / (ks * ks));
    if (pipe_use > 1.0) pipe_use = 1.0;
    // a ragged deal of blocks loads one SIMD more than the others; workgroups that share a CU even that out in part
    const double blocks = (!bf16 && held >= 2) ? 0.5 * simd_load + 0.125 * simd_sum : (double)simd_load;
    // (a block-step is one fp32 16x16x4 MFMA, 32 cycles of a SIMD's matrix pipe: 13.9 ns at 2.3 GHz)
    double us = (double)per_cu * blocks * steps * 0.0139 / pipe_use;
    // a wave has one chunk of staging loads in flight, so a workgroup cannot finish a chunk faster than a round trip to
    // memory allows, however little matrix work it holds (workgroups that share a CU walk their chains side by side;
    // quarter tiles stage a fifth of a 14 x 14 tile's positions per chunk, and their round trips are shorter)
    const double floor_us = ceil_div(per_cu, can_hold) * chunks * P.floor_chunk * (c.th == 7 ? P.floor_small : 1.0);
    if (us < floor_us) us = floor_us;
    // staging-heavy cases: a 1 x 1 kernel uses every staged value once instead of k*k times, a
    // strided tile stages four input values per output position (both measured)
    // (less so for the 16 x 16 tile, whose 256 positions per channel give every thread one position to stage)
    if (ks == 1 && c.shape != kGemmShape && c.shape != kWideGemmShape) us *= c.th * c.tw == 256 ? P.k1_tile256 : P.k1_other;
    if (d->stride == 2) us *= P.stride2;
    // bf16: staging the halo tile is serial with the matrix work of a workgroup that has a CU to itself
    if (bf16) us += (double)per_cu * chunks * halo * c.kg / waves * (P.stage / 64.0);
    us += P.fixed;          // launch, first loads, output write
    // fp32: every workgroup stages its halo tile of every channel, so workgroups of few rows re-read the input once
    // per group of rows (from L2 when the rows of one tile run side by side; tile rows that are no whole 64-byte lines
    // cost more): what decides between many small and few large workgroups, and what a 1 x 1 layer on a large image
    // is bound by (2 x 768 x 224 x 224, M 128: 16 rows per workgroup 287 us, 64 rows 212 us)
    if (!bf16)
        us += P.stage * (double)wgs * halo * ((double)d->c / c.csplit) * 4.0e-6 * ((c.tw % 16 == 0 || c.tw >= 28) ? 1.0 : P.stage_partial);
    // every further workgroup a CU works through brings its own prologue and closing write, hidden in part behind
    // the workgroups resident beside it
    if (!bf16 && per_cu > 1) us += (double)(per_cu - 1) * P.extra_wg / can_hold;
    if (bf16 && per_cu > 1) us += (double)(per_cu - 1) * (waves == 16 ? P.extra_wg_16 : can_hold == 1 ? P.extra_wg_alone : P.extra_wg);
    // [M][Q][P] output of a bf16 call: tile rows of 14 or 7 floats are partial cache lines, and with so little
    // matrix time per output the write shows (tiles 16 wide or whole image rows: nothing)
    // (rows: M, or k*k*M when the rows of a staged variant's matrix product are (tap, kernel) pairs)
    const double out_rows = (double)d->m * (dm.mb / ceil_div(d->m, 16));
    const double out_mb = (double)d->n * out_rows * dm.q * dm.p * 4.0e-6;
    const bool partial_lines = !channels_last && c.tw % 16 != 0 && c.tw < 28;
    if (bf16 && partial_lines) us += P.partial_out * out_mb;
    // what of the closing write the matrix work does not hide (layers of few channels and many kernels are bound by it)
    us += (P.out_write + (c.rb == 2 ? P.out_write_rb2 : 0.0)) * out_mb;
    // with one channel quad there is so little matrix work that the output write shows: half of it at 5 TB/s
    // when the tile rows are whole 64-byte lines, at 3.3 TB/s when they are not (fitted to the first-layer shapes)
    if (lean) us += 0.5 * 4.0 * (double)d->n * d->m * dm.q * dm.p / (c.tw % 16 == 0 ? 5.0e6 : 3.3e6);
    // the zero fill and two atomic adds per output: per MB of output ([M][Q][P]: tile rows of whole or partial lines)
    // (a split into more parts -- the flat shapes of a staged variant's matrix product -- adds its parts' worth of atomics)
    if (c.csplit > 1) us += P.split_fixed + (partial_lines ? P.split_mb_partial : P.split_mb) * out_mb * (c.csplit / 2.0);
    // the closing exchange of channel groups through LDS (quarter tiles: a seventh of the data)
    if (c.kg > 1) us += c.kg == 4 ? P.kg4 : waves == 16 ? P.kg2_16 : P.kg2;
    return us;
}

// The candidate the cost estimate prefers for the fused kernel (or the one CONV_MCMK_TILE forces:
// tuning aid, menu index = shape + 7 * (csplit - 1) for the seven common shapes, then
// 14 + further shape + 8 * (csplit - 1) for the eight further shapes: bf16 with two row blocks per wave, quarter tiles,
// tile pairs, quarter tiles with two channel groups; then 30 + later shape + count * (csplit - 1) for the shapes added
// since: the bf16 four-wave workgroups).
Candidate search_fused(const conv_mcmk_desc *d, const Dims &dm, bool channels_last, bool epilogue, int force, bool gemm = false);

constexpr int kGemmAtomics = 1, kGemmCopies = 2;   // how the parts of a split matrix product meet (choose_fused)

// The tile a staged variant's matrix product runs on unless one is forced: a flat shape (64 rows, or for bf16 also 128
// rows with two row blocks per wave, x 224 columns of the plane taken as one row, 32-channel chunks), with the
// contraction split 1, 2, 4, 8 or 16 ways.  A split buys workgroups for a product with few tiles (two per compute unit hide
// each other's staging; below one per unit the chip is idle in proportion) and pays for the way its parts meet: a copy
// of the result per part plus a streaming pass that adds the copies (im2col, im2row: room in their workspace), or a
// zero fill plus one atomic add per part and output element.  The rates are what the kernel sustained when every
// shape and split was timed on the benchmark layers' three staged variants, both precisions (the pick then loses 1 %
// on average and 13 % at worst against the fastest entry; the 2-D tiles of the fused kernel stage too little per
// barrier for a product whose every value is used once, and were never the fastest there).
double flat_gemm_us(const conv_mcmk_desc *d, const Dims &dm, bool channels_last, int shape, int cs, bool copies)
{
    const bool bf16 = d->dtype == CONV_MCMK_BF16;
    const long long cols = (long long)dm.q * dm.p;
    const TileShapeDesc &t = kTileShapes[shape];
    const long long col_tiles = ceil_div(cols, t.tw);
    const long long w = (long long)d->n * col_tiles * ceil_div(dm.mb, t.wm * t.rb) * cs;
    // (the rows a workgroup's waves cover whether the product has them or not: 64, or 128 with two row blocks per wave)
    const double rows = 16.0 * t.wm * t.rb * ceil_div(dm.mb, t.wm * t.rb);
    const double flop = 2.0 * d->n * rows * cols * d->c;
    const double out_mb = (double)d->n * (dm.mb * 16.0) * cols * 4.0e-6;
    // Fraction of the matrix peak to count with two workgroups per compute unit (full) and with one (single).  These
    // are fitted to the time of whole calls, in which the tail of one kernel overlaps the head of the next, together
    // with the cost of the parts' meeting below: for bf16 with two row blocks per wave they are not the kernel's own
    // rate (0.19 - 0.24 of the peak in a trace: cfg5b's product split four ways, 62 us).  bf16 with one row block per
    // wave reads a B fragment from LDS per product and is bound by that; two row blocks per wave halve the reads but
    // need the second workgroup to cover their latency.  Channels last, the staging gather and its transposing LDS
    // stores cost a fifth to a third (im2row's products).
    double full, single;
    if (!bf16)           { full = channels_last ? 0.55 : 0.69;   single = channels_last ? 0.50 : 0.60; }
    else if (t.rb == 2)  { full = channels_last ? 0.26 : 0.40;   single = channels_last ? 0.15 : 0.18; }
    else                 { full = channels_last ? 0.125 : 0.17;  single = channels_last ? 0.08 : 0.09; }
    const double eff = w >= 448 ? full : w >= kNumCU ? single : single * (double)w / kNumCU;
    const double compute = flop / ((bf16 ? 2500.0e6 : 157.3e6) * eff);
    // reading the right operand and writing the result (every part's copy of it), at 3.5 TB/s: what bounds a product
    // with a short contraction (the two-pass form's, whose result is k k times the output)
    const double moved_mb = (double)d->n * d->c * cols * (bf16 ? 2.0e-6 : 4.0e-6) + out_mb * (copies && cs > 1 ? cs : 1);
    const double memory = moved_mb / 3.5;
    double us = (compute > memory ? compute : memory) + 0.1 * (compute > memory ? memory : compute);
    // the parts' meeting: the pass that reads the copies and writes their sum (counted at 4.5 TB/s), or the zero fill and the
    // atomics (channels last, a lane's four rows are 16 bytes of one position: four scattered atomics where [M][Q][P]
    // output has runs of sixteen -- measured at several times the cost per MB)
    if (cs > 1) us += copies ? 3.0 + (cs + 1.0) * out_mb / 4.5 : 3.0 + (channels_last ? 9.0 : 1.6) * out_mb * (cs / 2.0);
    return us;
}

Candidate flat_gemm_candidate(const conv_mcmk_desc *d, const Dims &dm, bool channels_last, bool copies)
{
    const int chunks = ceil_div(d->c, 32);
    const int shapes[2] = {kGemmShape, kWideGemmShape};
    Candidate best = candidate(kGemmShape, 1);
    double best_us = -1.0;
    for (int s = 0; s < (d->dtype == CONV_MCMK_BF16 ? 2 : 1); ++s)
        for (int cs = 1; cs <= 16 && (cs == 1 || chunks >= cs); cs *= 2) {       // every part has a chunk to work on
            const double us = flat_gemm_us(d, dm, channels_last, shapes[s], cs, copies);
            if (best_us < 0.0 || us < best_us) { best = candidate(shapes[s], cs); best_us = us; }
        }
    return best;
}

// The search walks the whole menu, a few microseconds of host time -- as long as the smallest layers
// run on the GPU -- so the last few answers are remembered (per layer, layout, epilogue and override).
// gemm: 0 a convolution; 1 the matrix product of a staged variant whose split parts add into the result with
// atomics; 2 one whose parts each store a copy of the result (kGemmCopies).
Candidate choose_fused(const conv_mcmk_desc *d, const Dims &dm, bool channels_last, bool epilogue = false, int gemm = 0)
{
    const int force = gemm ? forced_index(g_force_gemm_tile, "CONV_MCMK_GEMM_TILE") : forced_index(g_force_tile, "CONV_MCMK_TILE");
    struct Key {
        conv_mcmk_desc d;
        int flags, forced, mb;
    };
    Key key;
    memset(&key, 0, sizeof(key));
    key.d = *d;
    key.flags = (channels_last ? 1 : 0) | (epilogue ? 2 : 0) | (gemm << 2);
    key.forced = force;
    key.mb = dm.mb;                       // a matrix product's rows may be (tap, kernel) pairs
    constexpr int kSlots = 32;
    static std::mutex mu;
    static Key keys[kSlots];
    static Candidate vals[kSlots];
    static int used = 0, next = 0;
    {
        std::lock_guard<std::mutex> lock(mu);
        for (int i = 0; i < used; ++i)
            if (memcmp(&keys[i], &key, sizeof(Key)) == 0) return vals[i];
    }
    const Candidate best = (gemm && force < 0) ? flat_gemm_candidate(d, dm, channels_last, gemm == kGemmCopies)
                                               : search_fused(d, dm, channels_last, epilogue, force, gemm != 0);
    {
        std::lock_guard<std::mutex> lock(mu);
        keys[next] = key;
        vals[next] = best;
        next = (next + 1) % kSlots;
        if (used < kSlots) ++used;
    }
    return best;
}

// gemm: the layer is the matrix product of a staged variant seen as a 1 x 1 convolution (d->k == 1, no padding, unit
// stride; the channels are the contraction index, the plane is the patch matrix's or the two-pass product's).  The
// whole menu applies, and after it come the two flat shapes (1 x 224 columns of the plane taken as one row, 32-channel
// chunks), each with the channels unsplit and split two, four, eight and sixteen ways: indices 100 .. 109.
Candidate search_fused(const conv_mcmk_desc *d, const Dims &dm, bool channels_last, bool epilogue, int force, bool gemm)
{
    Candidate best{};
    double best_cost = -1.0;
    // (the flat shapes also with the contraction split four, eight and sixteen ways: a staged variant's product over C k k
    // channels on a small plane has few tiles, and unlike the fused kernel's two-way split more than two partial sums
    // meet at the atomics, so the last bits of such a result depend on the order they arrive in)
    // Menu passes and the index their first entry has: the seven common shapes (0), the eight further ones (14), the
    // shapes added after those (30), and, for a matrix product only, the two flat shapes (100).
    struct Pass { const int *shapes; int count, first_index, max_split; };
    static const int kCommon[kConvShapes] = {0, 1, 2, 3, 4, 5, 6};
    static const int kFlat[2] = {kGemmShape, kWideGemmShape};
    const Pass passes[4] = {{kCommon, kConvShapes, 0, 2}, {kWideConvShape, kWideConvShapes, 14, 2},
                            {kLaterConvShape, kLaterConvShapes, 30, 2}, {kFlat, 2, 100, 16}};
    for (int pass = 0; pass < (gemm ? 4 : 3); ++pass)
    for (int cs = 1, index = passes[pass].first_index; cs <= passes[pass].max_split; cs *= 2)
        for (int pos = 0; pos < passes[pass].count; ++pos, ++index) {
            const int sh = passes[pass].shapes[pos];
            const Candidate c = candidate(sh, cs);
            if (sh == kWideGemmShape && d->dtype != CONV_MCMK_BF16) continue;
            // two row blocks per wave: bf16 operands, unit stride
            if (c.rb > 1 && (d->dtype != CONV_MCMK_BF16 || d->stride > 1 || d->k > 3)) continue;
            if (c.th == 7 && (d->stride > 1 || d->k > 5)) continue;
            // the 14 x 28 pairs under sixteen waves: fp32 operands, unit stride (excluded below), kernel sides up to 3
            if (sh >= kPairTileShape && sh <= kPairTileShape + 2 && (d->dtype == CONV_MCMK_BF16 || d->k > 3)) continue;
            // the two-group pair is not built for 2 x 2 kernels, nor for channels-last operands (measured slower there
            // than single tiles: the 16-byte gathers of eight waves fill a 30-column tile less evenly)
            if (sh == kPairTileShape + 1 && (d->k == 2 || channels_last)) continue;    // quarter tiles: unit stride, kernel sides up to 5
            // channel groups exist for kernel sides up to 3 only (four groups of double-buffered 5x5 halo
            // tiles would not fit the 160 KB of LDS); they combine with the two-way split (each workgroup's groups
            // share its half of the chunks: 1 x 512 x 28 x 28, M 512 runs 43.7 us that way, 48.2 us on quarter tiles)
            if (c.kg > 1 && d->k > 3) continue;
            // nor for a 1 x 1 kernel, whose chunks are too short to pay for the closing exchange (never the fastest
            // candidate on any 1 x 1 layer timed, either precision)
            // (a staged variant's product contracts over C k k: thousands of channels on the deep layers, and
            // there the groups are what fills the chip)
            if (c.kg > 1 && d->k == 1 && (d->c < 256 || d->dtype == CONV_MCMK_BF16) && force != index) continue;
            if (d->stride > 1 && sh >= kStridedShapes) continue;       // strided input tiles: 14 x 14 outputs only
            if (epilogue && cs > 1) continue;                          // partial sums cannot take the epilogue
            // strided bf16 tiles gathered from [C][H][W] with a kernel side of 5 or more exist for the
            // 2 x 4 wave layout only (register budget of the staging gather)
            if (d->stride > 1 && d->dtype == CONV_MCMK_BF16 && !channels_last && d->k >= 5 && sh != 1) continue;
            double cost;
            if (force == index) cost = 0.0;
            else if (sh == kGemmShape || sh == kWideGemmShape) {
                // the flat shapes see the plane as a single row of H W columns
                conv_mcmk_desc flat = *d;
                flat.h = 1;  flat.w = dm.q * dm.p;
                const Dims fdm{1, dm.q * dm.p, dm.mb, 1};
                cost = 1.2 * tile_cost(&flat, fdm, c, 1, channels_last);
            } else cost = tile_cost(d, dm, c, d->k, channels_last);
            // equal estimates (layers that sit on a latency floor): the candidate with more workgroups keeps more
            // loads in flight
            const bool tie = best_cost >= 0 && cost <= best_cost + 1e-6 && cost >= best_cost - 1e-6;
            if (best_cost < 0 || (tie ? workgroups(d, dm, c) > workgroups(d, dm, best) : cost < best_cost)) {
                best_cost = cost;
                best = c;
            }
        }
    return best;
}

// ------------------------------------------------------------------------------------------
// Estimated run time in microseconds of a whole variant (the per-layer choice among algorithms the
// paper's conclusion calls for).  Pieces: the tile-kernel estimate above for the matrix work; the
// memory-bound passes at the 6 TB/s they were measured to sustain plus a launch; the direct loop
// nest at its measured 3 TFLOP/s.
// The matrix product of a staged variant as the tile kernels see it: a 1 x 1 convolution of `kc` channels over a
// ph x pw plane per image (im2col / im2row: the patch matrix, plane = the output's; two-pass: the input itself), rows =
// row_groups x M.
struct GemmView {
    conv_mcmk_desc d;
    Dims dm;
};

GemmView gemm_view(const conv_mcmk_desc *d, long long kc, int ph, int pw, int row_groups)
{
    GemmView v;
    v.d = *d;
    v.d.c = (int)kc;  v.d.h = ph;  v.d.w = pw;  v.d.k = 1;  v.d.pad = 0;  v.d.stride = 1;
    v.dm = Dims{ph, pw, ceil_div(d->m, 16) * row_groups, 1};
    return v;
}

// im2row's product: channels last, the patch rows of all images are one [N Q P] x [C k k] matrix and the outputs one
// [N Q P] x [M] matrix, so the batch folds into the plane (one image of N Q P positions) and small planes fill whole
// 224-column tiles -- unless a 2-D tile is forced, which wants the plane's own shape, or the folded plane would pass
// the 32-bit offsets of one image.
void im2row_plane(const conv_mcmk_desc *d, const Dims &dm, conv_mcmk_desc *view, int *ph, int *pw)
{
    *view = *d;
    *ph = dm.q;
    *pw = dm.p;
    const long long positions = (long long)d->n * dm.q * dm.p;
    if (forced_index(g_force_gemm_tile, "CONV_MCMK_GEMM_TILE") < 0 && ((long long)d->c * dm.taps + 64) * positions < (1LL << 29)) {
        view->n = 1;
        *ph = 1;
        *pw = (int)positions;
    }
}

double gemm_cost(const conv_mcmk_desc *d, long long kc, int ph, int pw, int row_groups, bool channels_last = false, int mode = kGemmAtomics)
{
    const GemmView v = gemm_view(d, kc, ph, pw, row_groups);
    const Candidate c = choose_fused(&v.d, v.dm, channels_last, false, mode);
    // the flat shapes: the rates the kernel was measured to sustain, plus a launch; a forced 2-D tile: the fused
    // kernel's estimate for a 1 x 1 layer
    if (c.shape == kGemmShape || c.shape == kWideGemmShape) return flat_gemm_us(&v.d, v.dm, channels_last, c.shape, c.csplit, mode == kGemmCopies) + 5.0;
    return tile_cost(&v.d, v.dm, c, 1, channels_last);
}

// How a fused call runs.  A 1 x 1 kernel without padding or stride makes the layer a plain matrix product over the
// plane (section III-A), with no tile edges inside the image: where the flat shape's estimate beats the best 2-D
// tile's by a tenth, the call runs as that product.  ([C][H][W] input only: with channels last the flat shape measured
// 3 - 8 % slower than the tiles on the layers where its estimate won.)  The product may split its contraction two ways
// at most, as the tiles do: two parts at the atomics keep the result independent of their order.
struct FusedPlan {
    Candidate c;
    double cost;
    bool as_product;
    conv_mcmk_desc view;   // as_product: the layer the product's launch sees ...
    int ph, pw;            // ... and its plane
};

FusedPlan plan_fused(const conv_mcmk_desc *d, const Dims &dm, bool channels_last, bool epilogue)
{
    FusedPlan f;
    f.c = choose_fused(d, dm, channels_last, epilogue);
    f.cost = tile_cost(d, dm, f.c, d->k, channels_last);
    f.as_product = false;
    f.view = *d;  f.ph = d->h;  f.pw = d->w;
    if (d->k != 1 || d->pad != 0 || d->stride != 1 || channels_last) return f;
    if (forced_index(g_force_tile, "CONV_MCMK_TILE") >= 0 || forced_index(g_force_gemm_tile, "CONV_MCMK_GEMM_TILE") >= 0) return f;
    const conv_mcmk_desc view = *d;
    const int ph = d->h, pw = d->w;
    if ((long long)ph * pw >= (1LL << 31)) return f;
    const GemmView v = gemm_view(&view, d->c, ph, pw, 1);
    const Candidate g = choose_fused(&v.d, v.dm, channels_last, false, kGemmAtomics);
    if ((g.shape != kGemmShape && g.shape != kWideGemmShape) || g.csplit > (epilogue ? 1 : 2)) return f;
    const double cost = flat_gemm_us(&v.d, v.dm, channels_last, g.shape, g.csplit, false) + 5.0;
    if (cost < 0.9 * f.cost) {
        f.c = g;  f.cost = cost;  f.as_product = true;
        f.view = view;  f.ph = ph;  f.pw = pw;
    }
    return f;
}

// a memory-bound pass before or after the matrix kernel: its bytes, its launch, and the drain / fill
// between two dependent kernels
// (the streaming forms for unit stride and kernel sides 3 and 5 sustain 6 TB/s; the general kernels, which also pay
// 64-bit index arithmetic per item, 3.5 TB/s and a longer tail)
double stream_cost(double bytes, bool streaming_form) { return streaming_form ? bytes / 6.0e6 + 4.0 : bytes / 3.5e6 + 12.0; }

double variant_cost(const conv_mcmk_desc *d, const Dims &dm, int variant)
{
    const double elt = d->dtype == CONV_MCMK_BF16 ? 2.0 : 4.0;
    const double in_elems = (double)d->n * d->c * d->h * d->w;
    const double patch_elems = (double)d->n * d->c * dm.taps * dm.q * dm.p;
    switch (variant) {
    case CONV_MCMK_KN2ROW:
    case CONV_MCMK_KN2COL:
        return plan_fused(d, dm, variant == CONV_MCMK_KN2COL, false).cost;
    case CONV_MCMK_KN2ROW_2PASS: {
        const double planes = (double)d->n * d->m * d->h * d->w;
        return gemm_cost(d, d->c, d->h, d->w, dm.taps) +
               stream_cost(4.0 * (dm.taps * planes + (double)d->n * d->m * dm.q * dm.p), d->stride == 1 && (d->k == 3 || d->k == 5));
    }
    case CONV_MCMK_IM2COL:
    case CONV_MCMK_IM2ROW:
    {
        const double build = stream_cost(elt * (in_elems + patch_elems), variant == CONV_MCMK_IM2ROW || (d->stride == 1 && (d->k == 3 || d->k == 5)));
        if (variant == CONV_MCMK_IM2COL) return build + gemm_cost(d, (long long)d->c * dm.taps, dm.q, dm.p, 1, false, kGemmCopies);
        conv_mcmk_desc folded;
        int ph, pw;
        im2row_plane(d, dm, &folded, &ph, &pw);
        return build + gemm_cost(&folded, (long long)d->c * dm.taps, ph, pw, 1, true, kGemmCopies);
    }
    default: {
        // one thread per output walks its C*k*k terms one after the other (0.12 us each when the chip
        // is not full); a full chip sustains 3 TFLOP/s
        const double serial = 0.12 * d->c * dm.taps;
        const double bulk = 2.0 * d->n * d->m * (double)d->c * dm.taps * dm.q * dm.p / 3.0e6;
        return (serial > bulk ? serial : bulk) + 5.0;
    }
    }
}

int launch_product(const conv_mcmk_desc *d, const Candidate &c, const void *bmat, const void *apk, float *cmat, long long kc,
                   int ph, int pw, int row_groups, hipStream_t st, bool channels_last, const Epilogue &ep, float *partials);

int launch_fused(const conv_mcmk_desc *d, const Dims &dm, const void *in, const void *apk, float *out,
                 hipStream_t st, bool channels_last, const Epilogue &ep = Epilogue())
{
    const FusedPlan plan = plan_fused(d, dm, channels_last, ep.any());
    if (plan.as_product)
        return launch_product(&plan.view, plan.c, in, apk, out, d->c, plan.ph, plan.pw, 1, st, channels_last, ep, nullptr);
    const Candidate &best = plan.c;
    return launch_tile(d, dm, d->k, best.shape, best.csplit, in, apk, out, d->c, d->h, d->w, dm.q, dm.p, d->pad, 1, st,
                       channels_last, d->stride, ep);
}

// Plain matrix product [row_groups M x kc] . [kc x ph pw] per image on the tile kernels: a 1 x 1 "convolution" over
// the ph x pw plane, with the tile shape (2-D tiles, channel groups, channel split, or the flat 1 x 224 shape over the
// plane taken as one row) chosen by the same estimate that serves the fused kernel.
// mode kGemmCopies: `spare` (spare_bytes of device memory, 16-byte aligned, or null) takes one copy of the result per
// part of a split contraction; a buffer too small for them sends the parts back to atomics on a zeroed result.
int launch_gemm(const conv_mcmk_desc *d, const void *bmat, const void *apk, float *cmat,
                long long kc, int ph, int pw, int row_groups, hipStream_t st, bool channels_last = false,
                int mode = kGemmAtomics, void *spare = nullptr, size_t spare_bytes = 0)
{
    if ((long long)ph * pw >= (1LL << 31) || kc >= (1LL << 31)) return CONV_MCMK_ERR_SHAPE;
    const GemmView v = gemm_view(d, kc, ph, pw, row_groups);
    const Candidate c = choose_fused(&v.d, v.dm, channels_last, false, mode);
    const size_t result = (size_t)d->n * row_groups * d->m * ph * pw;
    float *partials = nullptr;
    if (mode == kGemmCopies && c.csplit > 1 && spare && spare_bytes >= partial_floats(result) * sizeof(float) * c.csplit)
        partials = static_cast<float *>(spare);
    return launch_product(d, c, bmat, apk, cmat, kc, ph, pw, row_groups, st, channels_last, Epilogue(), partials);
}

// The launch of a matrix product on candidate c: the flat shapes see the plane as one row of ph pw columns.
int launch_product(const conv_mcmk_desc *d, const Candidate &c, const void *bmat, const void *apk, float *cmat, long long kc,
                   int ph, int pw, int row_groups, hipStream_t st, bool channels_last, const Epilogue &ep, float *partials)
{
    const bool flat = c.shape == kGemmShape || c.shape == kWideGemmShape;
    const int h = flat ? 1 : ph, w = flat ? ph * pw : pw;
    const Dims dm{ph, pw, ceil_div(d->m, 16), 1};          // launch_tile takes the blocks of one row group
    return launch_tile(d, dm, 1, c.shape, c.csplit, bmat, apk, cmat, (int)kc, h, w, h, w, 0, row_groups, st, channels_last, 1,
                       ep, partials);
}

int common_ptr_checks(const void *I, const void *K, const void *O)
{
    if (!I || !K || !O) return CONV_MCMK_ERR_NULL;
    if (misaligned(I) || misaligned(K) || misaligned(O)) return CONV_MCMK_ERR_ALIGN;
    return CONV_MCMK_OK;
}

// The matrix a staged variant builds or fills: the part of its workspace it cannot do without.
size_t workspace_matrix_bytes(const conv_mcmk_desc *d, const Dims &dm, int variant)
{
    const size_t elt = d->dtype == CONV_MCMK_BF16 ? 2 : 4;
    switch (variant) {
    case CONV_MCMK_KN2ROW_2PASS: return (size_t)d->n * dm.taps * d->m * d->h * d->w * sizeof(float);
    case CONV_MCMK_IM2COL:
    case CONV_MCMK_IM2ROW: return (size_t)d->n * d->c * dm.taps * dm.q * dm.p * elt;
    default: return 0;
    }
}

// Where the copies of the result start behind that matrix, and how many bytes they take: one copy per part when the
// product of im2col / im2row splits its contraction, none otherwise.
size_t workspace_copies_offset(size_t matrix_bytes) { return (matrix_bytes + 255) / 256 * 256; }

size_t workspace_copies_bytes(const conv_mcmk_desc *d, const Dims &dm, int variant)
{
    if (variant != CONV_MCMK_IM2COL && variant != CONV_MCMK_IM2ROW) return 0;
    conv_mcmk_desc view = *d;
    int ph = dm.q, pw = dm.p;
    if (variant == CONV_MCMK_IM2ROW) im2row_plane(d, dm, &view, &ph, &pw);
    const long long kc = (long long)d->c * dm.taps;
    if ((long long)ph * pw >= (1LL << 31) || kc >= (1LL << 31)) return 0;
    const GemmView v = gemm_view(&view, kc, ph, pw, 1);
    const Candidate c = choose_fused(&v.d, v.dm, variant == CONV_MCMK_IM2ROW, false, kGemmCopies);
    if (c.csplit < 2) return 0;
    return partial_floats((size_t)d->n * d->m * dm.q * dm.p) * sizeof(float) * c.csplit;
}

int workspace_check(const conv_mcmk_desc *d, int variant, const void *ws, size_t ws_bytes)
{
    Dims dm;
    if (int rc = validate(d, variant, &dm)) return rc;
    const size_t need = workspace_matrix_bytes(d, dm, variant);
    if (need == 0) return CONV_MCMK_OK;
    if (!ws || ws_bytes < need) return CONV_MCMK_ERR_WORKSPACE;
    if (misaligned(ws)) return CONV_MCMK_ERR_ALIGN;
    return CONV_MCMK_OK;
}

int fused_entry(const conv_mcmk_desc *d, int variant, const void *I_dev, const void *Kp_dev, void *O_dev, void *stream,
                const Epilogue &ep = Epilogue())
{
    Dims dm;
    int rc = validate(d, variant, &dm);
    if (rc) return rc;
    if ((rc = common_ptr_checks(I_dev, Kp_dev, O_dev))) return rc;
    if (ep.bias && (reinterpret_cast<uintptr_t>(ep.bias) & 3u) != 0) return CONV_MCMK_ERR_ALIGN;
    return launch_fused(d, dm, I_dev, Kp_dev, static_cast<float *>(O_dev), static_cast<hipStream_t>(stream),
                        variant == CONV_MCMK_KN2COL, ep);
}

// The two passes of section III-A on a product buffer T of N * k*k*M * H*W floats.
int two_pass(const conv_mcmk_desc *d, const Dims &dm, const void *I_dev, const void *Kp_dev, void *O_dev, float *T, hipStream_t st)
{
    int rc;
    // pass 1: T[n][t*M+m][HW] = Kp[k*k*M x C] . I[n][C x HW]
    rc = launch_gemm(d, I_dev, Kp_dev, T, d->c, d->h, d->w, dm.taps, st);
    if (rc) return rc;
    // pass 2: shift-add of the k*k planes
    const int vec = dm.p % 4 == 0 ? 4 : dm.p % 2 == 0 ? 2 : 1;
    if (d->stride == 1 && (d->k == 3 || d->k == 5) && (size_t)dm.taps * d->m * d->h * d->w * sizeof(float) < (1ull << 31)) {
        // the common case: the streaming form (one item per thread, images along the grid's second dimension)
        const dim3 grid(stream_grid((size_t)d->m * dm.q * (dm.p / vec), 1), d->n < 65535 ? d->n : 65535);
        auto launch = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, grid, dim3(256), 0, st, T, static_cast<float *>(O_dev), d->n, d->m, d->h, d->w, d->pad, dm.q, dm.p);
        };
        if (d->k == 3) { if (vec == 4) launch(shift_add_fast_kernel<4, 3>); else if (vec == 2) launch(shift_add_fast_kernel<2, 3>); else launch(shift_add_fast_kernel<1, 3>); }
        else           { if (vec == 4) launch(shift_add_fast_kernel<4, 5>); else if (vec == 2) launch(shift_add_fast_kernel<2, 5>); else launch(shift_add_fast_kernel<1, 5>); }
        return launch_status();
    }
    const int gvec = vec == 4 ? 4 : 1;
    const size_t total = (size_t)d->n * d->m * dm.q * (dm.p / gvec);
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, T, static_cast<float *>(O_dev), d->n, d->m,
                           d->h, d->w, d->k, d->pad, d->stride, dm.q, dm.p);
    };
    if (gvec == 4 && d->k == 3) launch(shift_add_f32_kernel<4, 3>);
    else if (gvec == 4) launch(shift_add_f32_kernel<4, 0>);
    else if (d->k == 3) launch(shift_add_f32_kernel<1, 3>);
    else launch(shift_add_f32_kernel<1, 0>);
    return launch_status();
}

// ------------------------------------------------------------------------------------------
// Product buffer of conv_mcmk_kn2row_2pass_static: device memory that belongs to the library's code object, so that
// the call needs no allocation by anyone.  Every GPU the library runs on holds its own copy (at its own address) until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address it yields
// for the current device is what kernels are given.
constexpr size_t kStaticScratchBytes = CONV_MCMK_STATIC_SCRATCH_BYTES;
}  // namespace (closed so that the array is declared at file scope)

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

int static_scratch_address(void **out)
{
    static std::mutex mu;
    static void *address[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CONV_MCMK_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CONV_MCMK_ERR_DEVICE;
        address[dev] = p;
    }
    *out = address[dev];
    return CONV_MCMK_OK;
}

}  // namespace

extern "C" {

const char *conv_mcmk_strerror(int code)
{
    switch (code) {
    case CONV_MCMK_OK: return "ok";
    case CONV_MCMK_ERR_NULL: return "a required pointer is NULL";
    case CONV_MCMK_ERR_SHAPE: return "invalid shape (dimension < 1, negative pad, empty output or tensor too large)";
    case CONV_MCMK_ERR_UNSUPPORTED: return "unsupported stride, dtype, variant, kernel size or channel count for this variant";
    case CONV_MCMK_ERR_WORKSPACE: return "workspace missing or too small";
    case CONV_MCMK_ERR_DEVICE: return "the HIP runtime refused a launch";
    case CONV_MCMK_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    default: return "unknown error code";
    }
}

int conv_mcmk_check(const conv_mcmk_desc *desc, int variant) { return validate(desc, variant, nullptr); }

int conv_mcmk_output_dims(const conv_mcmk_desc *desc, int *q, int *p)
{
    Dims dm;
    // the staged two-pass variant takes every shape the library takes at all
    const int rc = validate(desc, CONV_MCMK_KN2ROW_2PASS, &dm);
    if (rc) return rc;
    if (q) *q = dm.q;
    if (p) *p = dm.p;
    return CONV_MCMK_OK;
}

void conv_mcmk_force_tile(int index) { g_force_tile.store(index < 0 ? -1 : index, std::memory_order_relaxed); }
void conv_mcmk_force_gemm_tile(int index) { g_force_gemm_tile.store(index < 0 ? -1 : index, std::memory_order_relaxed); }

int conv_mcmk_probe_mfma(int dtype, int blocks, int iters, float *sink_dev, void *stream)
{
    if (!sink_dev) return CONV_MCMK_ERR_NULL;
    if (misaligned(sink_dev)) return CONV_MCMK_ERR_ALIGN;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return CONV_MCMK_ERR_SHAPE;
    if (dtype != CONV_MCMK_F32 && dtype != CONV_MCMK_BF16) return CONV_MCMK_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == CONV_MCMK_BF16) hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(blocks), dim3(256), 0, st, sink_dev, iters);
    else hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(blocks), dim3(256), 0, st, sink_dev, iters);
    return launch_status();
}

int conv_mcmk_probe_copy(const void *src_dev, void *dst_dev, size_t bytes, void *stream)
{
    if (!src_dev || !dst_dev) return CONV_MCMK_ERR_NULL;
    if (misaligned(src_dev) || misaligned(dst_dev)) return CONV_MCMK_ERR_ALIGN;
    if (bytes % 16 != 0) return CONV_MCMK_ERR_SHAPE;
    if (bytes == 0) return CONV_MCMK_OK;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(stream_grid(bytes / 16, 1)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const float4 *>(src_dev), static_cast<float4 *>(dst_dev), bytes / 16);
    return launch_status();
}

int conv_mcmk_describe_plan(const conv_mcmk_desc *d, int variant, char *buf, size_t n)
{
    Dims dm;
    int rc = validate(d, variant, &dm);
    if (rc) return rc;
    if (!buf || n == 0) return CONV_MCMK_ERR_NULL;
    const char *type = d->dtype == CONV_MCMK_BF16 ? "bf16" : "f32";
    // the tile the matrix product of a staged variant would run on
    auto gemm_text = [&](long long kc, int ph, int pw, int row_groups, bool cl, int mode, char *out, size_t len) {
        const GemmView v = gemm_view(d, kc, ph, pw, row_groups);
        const Candidate c = choose_fused(&v.d, v.dm, cl, false, mode);
        const bool flat = c.shape == kGemmShape || c.shape == kWideGemmShape;
        const long long cols = flat ? ceil_div((long long)ph * pw, c.tw) : (long long)ceil_div(pw, c.tw) * ceil_div(ph, c.th);
        snprintf(out, len, "tile %dx%d%s, waves %dx%d, row blocks %d, channel groups %d, channel split %d, %lld workgroups",
                 c.th, c.tw, flat ? " over the flattened plane" : "", c.wm, c.wp, c.rb, c.kg, c.csplit,
                 (long long)d->n * cols * ceil_div(v.dm.mb, c.wm * c.rb) * c.csplit);
    };
    char tile[160];
    switch (variant) {
    case CONV_MCMK_KN2ROW:
    case CONV_MCMK_KN2COL: {
        const FusedPlan plan = plan_fused(d, dm, variant == CONV_MCMK_KN2COL, false);
        const Candidate &c = plan.c;
        const long long wgs = plan.as_product
            ? (long long)plan.view.n * ceil_div((long long)plan.ph * plan.pw, c.tw) * ceil_div(dm.mb, c.wm * c.rb) * c.csplit
            : (long long)d->n * ceil_div(dm.p, c.tw) * ceil_div(dm.q, c.th) * ceil_div(dm.mb, c.wm * c.rb) * c.csplit;
        const bool lean = !plan.as_product && lean_applies(d, d->k, c.shape, c.csplit, variant == CONV_MCMK_KN2COL, d->stride, 1);
        snprintf(buf, n, "%s fused %s: tile %dx%d%s, waves %dx%d, row blocks %d, channel groups %d, channel split %d, %lld workgroups%s, est %.1f us",
                 variant == CONV_MCMK_KN2COL ? "kn2col" : "kn2row", type, c.th, c.tw,
                 !plan.as_product ? "" : plan.view.n == 1 && d->n > 1 ? " over the flattened planes of the batch" : " over the flattened plane",
                 c.wm, c.wp, c.rb, c.kg, c.csplit, wgs, lean ? ", one channel quad" : "", plan.cost);
        break;
    }
    case CONV_MCMK_KN2ROW_2PASS:
        gemm_text(d->c, d->h, d->w, dm.taps, false, kGemmAtomics, tile, sizeof(tile));
        snprintf(buf, n, "kn2row two-pass %s: GEMM [%d x %d].[%d x %d] per image (%s), then shift-add, est %.1f us",
                 type, dm.taps * d->m, d->c, d->c, d->h * d->w, tile, variant_cost(d, dm, variant));
        break;
    case CONV_MCMK_IM2COL:
        gemm_text((long long)d->c * dm.taps, dm.q, dm.p, 1, false, kGemmCopies, tile, sizeof(tile));
        snprintf(buf, n, "im2col %s: patch matrix [%d x %d] per image, GEMM [%d x %d].[%d x %d] (%s), est %.1f us",
                 type, d->c * dm.taps, dm.q * dm.p, d->m, d->c * dm.taps, d->c * dm.taps, dm.q * dm.p, tile,
                 variant_cost(d, dm, variant));
        break;
    case CONV_MCMK_IM2ROW:
        {
            conv_mcmk_desc folded;
            int ph, pw;
            im2row_plane(d, dm, &folded, &ph, &pw);
            const GemmView v = gemm_view(&folded, (long long)d->c * dm.taps, ph, pw, 1);
            const Candidate c = choose_fused(&v.d, v.dm, true, false, kGemmCopies);
            const bool flat = c.shape == kGemmShape || c.shape == kWideGemmShape;
            const long long cols = flat ? ceil_div((long long)ph * pw, c.tw) : (long long)ceil_div(pw, c.tw) * ceil_div(ph, c.th);
            snprintf(tile, sizeof(tile), "tile %dx%d%s, waves %dx%d, row blocks %d, channel groups %d, channel split %d, %lld workgroups",
                     c.th, c.tw, flat ? (folded.n == 1 && d->n > 1 ? " over the flattened planes of the batch" : " over the flattened plane") : "",
                     c.wm, c.wp, c.rb, c.kg, c.csplit, (long long)folded.n * cols * ceil_div(v.dm.mb, c.wm * c.rb) * c.csplit);
        }
        snprintf(buf, n, "im2row %s: patch matrix [%d x %d] per image (channels last), GEMM [%d x %d].[%d x %d] (%s), est %.1f us",
                 type, dm.q * dm.p, d->c * dm.taps, dm.q * dm.p, d->c * dm.taps, d->c * dm.taps, d->m, tile,
                 variant_cost(d, dm, variant));
        break;
    default:
        snprintf(buf, n, "direct f32: one thread per output element, %lld outputs, est %.1f us",
                 (long long)d->n * d->m * dm.q * dm.p, variant_cost(d, dm, variant));
        break;
    }
    return CONV_MCMK_OK;
}

size_t conv_mcmk_workspace_bytes(const conv_mcmk_desc *d, int variant)
{
    Dims dm;
    if (validate(d, variant, &dm) != CONV_MCMK_OK) return 0;
    const size_t matrix = workspace_matrix_bytes(d, dm, variant);
    const size_t copies = workspace_copies_bytes(d, dm, variant);
    return copies ? workspace_copies_offset(matrix) + copies : matrix;
}

size_t conv_mcmk_packed_kernel_bytes(const conv_mcmk_desc *d, int variant)
{
    Dims dm;
    if (validate(d, variant, &dm) != CONV_MCMK_OK) return 0;
    const int group = d->dtype == CONV_MCMK_BF16 ? 32 : 16;
    const size_t elt = d->dtype == CONV_MCMK_BF16 ? 2 : 4;
    switch (variant) {
    case CONV_MCMK_KN2ROW:
    case CONV_MCMK_KN2ROW_2PASS:
    case CONV_MCMK_KN2COL:
        return (size_t)dm.taps * dm.mb * ceil_div(d->c, group) * 16 * group * elt;
    case CONV_MCMK_IM2COL:
    case CONV_MCMK_IM2ROW:
        return (size_t)dm.mb * ceil_div((long long)d->c * dm.taps, group) * 16 * group * elt;
    default: return 0;
    }
}

int conv_mcmk_prepack(const conv_mcmk_desc *d, int variant, const void *K_dev, void *Kp_dev, void *stream)
{
    Dims dm;
    int rc = validate(d, variant, &dm);
    if (rc) return rc;
    if (variant == CONV_MCMK_DIRECT) return CONV_MCMK_ERR_UNSUPPORTED;
    if (!K_dev || !Kp_dev) return CONV_MCMK_ERR_NULL;
    if (misaligned(K_dev) || misaligned(Kp_dev)) return CONV_MCMK_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int order = variant == CONV_MCMK_IM2COL ? 1 : variant == CONV_MCMK_IM2ROW ? 2 : 0;
    const bool bf16 = d->dtype == CONV_MCMK_BF16;
    const int group = bf16 ? 32 : 16;
    const int taps = order ? 1 : dm.taps;
    const int cg = order ? ceil_div((long long)d->c * dm.taps, group) : ceil_div(d->c, group);
    const size_t total = (size_t)taps * dm.mb * cg * 16 * group;
    if (bf16)
        hipLaunchKernelGGL(prepack_bf16_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st,
                           static_cast<const float *>(K_dev), static_cast<uint16_t *>(Kp_dev),
                           d->m, d->c, d->k, dm.mb, cg, taps, order);
    else
        hipLaunchKernelGGL(prepack_f32_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st,
                           static_cast<const float *>(K_dev), static_cast<float *>(Kp_dev),
                           d->m, d->c, d->k, dm.mb, cg, taps, order);
    return launch_status();
}

int conv_mcmk_kn2row(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream)
{
    (void)ws; (void)ws_bytes;
    return fused_entry(d, CONV_MCMK_KN2ROW, I_dev, Kp_dev, O_dev, stream);
}

int conv_mcmk_kn2col(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream)
{
    (void)ws; (void)ws_bytes;
    return fused_entry(d, CONV_MCMK_KN2COL, I_dev, Kp_dev, O_dev, stream);
}

int conv_mcmk_kn2row_bias_relu(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, const float *bias_dev,
                               int relu, void *O_dev, void *stream)
{
    Epilogue ep;
    ep.bias = bias_dev;
    ep.relu = relu != 0;
    return fused_entry(d, CONV_MCMK_KN2ROW, I_dev, Kp_dev, O_dev, stream, ep);
}

int conv_mcmk_kn2col_bias_relu(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, const float *bias_dev,
                               int relu, void *O_dev, void *stream)
{
    Epilogue ep;
    ep.bias = bias_dev;
    ep.relu = relu != 0;
    return fused_entry(d, CONV_MCMK_KN2COL, I_dev, Kp_dev, O_dev, stream, ep);
}

int conv_mcmk_1x1(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, void *O_dev, void *stream)
{
    Dims dm;
    int rc = validate(d, CONV_MCMK_KN2ROW, &dm);
    if (rc) return rc;
    if (d->k != 1) return CONV_MCMK_ERR_UNSUPPORTED;
    if ((rc = common_ptr_checks(I_dev, Kp_dev, O_dev))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // without padding or stride the image is just H*W columns of the matrix [C x HW] (section III-A): the fused
    // path runs it as a plain product with no tile edges inside the image where that is the faster of the two
    return launch_fused(d, dm, I_dev, Kp_dev, static_cast<float *>(O_dev), st, false);
}

int conv_mcmk_kn2row_2pass(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, void *O_dev,
                           void *ws, size_t ws_bytes, void *stream)
{
    Dims dm;
    int rc = validate(d, CONV_MCMK_KN2ROW_2PASS, &dm);
    if (rc) return rc;
    if ((rc = common_ptr_checks(I_dev, Kp_dev, O_dev))) return rc;
    if ((rc = workspace_check(d, CONV_MCMK_KN2ROW_2PASS, ws, ws_bytes))) return rc;
    return two_pass(d, dm, I_dev, Kp_dev, O_dev, static_cast<float *>(ws), static_cast<hipStream_t>(stream));
}

int conv_mcmk_kn2row_2pass_static(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, void *O_dev, void *stream)
{
    Dims dm;
    int rc = validate(d, CONV_MCMK_KN2ROW_2PASS, &dm);
    if (rc) return rc;
    if ((rc = common_ptr_checks(I_dev, Kp_dev, O_dev))) return rc;
    if (conv_mcmk_workspace_bytes(d, CONV_MCMK_KN2ROW_2PASS) > kStaticScratchBytes) return CONV_MCMK_ERR_WORKSPACE;
    void *T = nullptr;
    if ((rc = static_scratch_address(&T))) return rc;
    // nothing in the array has to start from zero: the matrix product writes every element of its k*k*M x H*W result
    // (or clears it with a fill kernel first, where it splits the contraction) before the post pass reads it
    return two_pass(d, dm, I_dev, Kp_dev, O_dev, static_cast<float *>(T), static_cast<hipStream_t>(stream));
}

int conv_mcmk_im2col(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream)
{
    Dims dm;
    int rc = validate(d, CONV_MCMK_IM2COL, &dm);
    if (rc) return rc;
    if ((rc = common_ptr_checks(I_dev, Kp_dev, O_dev))) return rc;
    if ((rc = workspace_check(d, CONV_MCMK_IM2COL, ws, ws_bytes))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf16 = d->dtype == CONV_MCMK_BF16;
    if (d->stride == 1 && (d->k == 3 || d->k == 5)) {
        // the common case: the streaming form; the widest store the row length allows, up to 16 bytes
        const int vmax = bf16 ? 8 : 4;
        int vec = vmax;
        while (dm.p % vec != 0) vec /= 2;
        const dim3 grid(stream_grid((size_t)d->c * dm.q * (dm.p / vec), 1), d->n < 65535 ? d->n : 65535), block(256);
#define MCMK_IM2COL_FAST(T, V, KS)                                                                            \
    hipLaunchKernelGGL((im2col_build_fast_kernel<T, V, KS>), grid, block, 0, st, static_cast<const T *>(I_dev), \
                       static_cast<T *>(ws), d->n, d->c, d->h, d->w, d->pad, dm.q, dm.p)
#define MCMK_IM2COL_FAST_K(T, V) do { if (d->k == 3) MCMK_IM2COL_FAST(T, V, 3); else MCMK_IM2COL_FAST(T, V, 5); } while (0)
        if (bf16) {
            if (vec == 8) MCMK_IM2COL_FAST_K(uint16_t, 8); else if (vec == 4) MCMK_IM2COL_FAST_K(uint16_t, 4);
            else if (vec == 2) MCMK_IM2COL_FAST_K(uint16_t, 2); else MCMK_IM2COL_FAST_K(uint16_t, 1);
        } else {
            if (vec == 4) MCMK_IM2COL_FAST_K(float, 4); else if (vec == 2) MCMK_IM2COL_FAST_K(float, 2); else MCMK_IM2COL_FAST_K(float, 1);
        }
#undef MCMK_IM2COL_FAST_K
#undef MCMK_IM2COL_FAST
    } else {
        // any kernel side and stride: 16-byte stores when P is a multiple of 4 (fp32) / 8 (bf16)
        const int vec = bf16 ? (dm.p % 8 == 0 ? 8 : 1) : (dm.p % 4 == 0 ? 4 : 1);
        const size_t total = (size_t)d->n * d->c * dm.q * (dm.p / vec);
        const dim3 grid(grid_for(total, 256)), block(256);
#define MCMK_IM2COL(T, V)                                                                             \
    hipLaunchKernelGGL((im2col_build_kernel<T, V>), grid, block, 0, st, static_cast<const T *>(I_dev), \
                       static_cast<T *>(ws), d->n, d->c, d->h, d->w, d->k, d->pad, d->stride, dm.q, dm.p)
        if (bf16) { if (vec == 8) MCMK_IM2COL(uint16_t, 8); else MCMK_IM2COL(uint16_t, 1); }
        else      { if (vec == 4) MCMK_IM2COL(float, 4);    else MCMK_IM2COL(float, 1); }
#undef MCMK_IM2COL
    }
    if ((rc = launch_status())) return rc;
    const size_t copies_at = workspace_copies_offset(workspace_matrix_bytes(d, dm, CONV_MCMK_IM2COL));
    return launch_gemm(d, ws, Kp_dev, static_cast<float *>(O_dev), (long long)d->c * dm.taps, dm.q, dm.p, 1, st, false, kGemmCopies,
                       ws_bytes > copies_at ? static_cast<char *>(ws) + copies_at : nullptr, ws_bytes > copies_at ? ws_bytes - copies_at : 0);
}

int conv_mcmk_im2row(const conv_mcmk_desc *d, const void *I_dev, const void *Kp_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream)
{
    Dims dm;
    int rc = validate(d, CONV_MCMK_IM2ROW, &dm);
    if (rc) return rc;
    if ((rc = common_ptr_checks(I_dev, Kp_dev, O_dev))) return rc;
    if ((rc = workspace_check(d, CONV_MCMK_IM2ROW, ws, ws_bytes))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf16 = d->dtype == CONV_MCMK_BF16;
    const int vec = bf16 ? 8 : 4;
    const int images = d->n < 65535 ? d->n : 65535;
    if (d->stride == 1 && (d->k == 3 || d->k == 5)) {
        // the common case: all k*k taps of a channel vector per thread
        const dim3 grid(stream_grid((size_t)dm.q * dm.p * (d->c / vec), 1), images), block(256);
#define MCMK_IM2ROW_FAST(T, V, KS)                                                                            \
    hipLaunchKernelGGL((im2row_build_fast_kernel<T, V, KS>), grid, block, 0, st, static_cast<const T *>(I_dev), \
                       static_cast<T *>(ws), d->n, d->c, d->h, d->w, d->pad, dm.q, dm.p)
        if (bf16) { if (d->k == 3) MCMK_IM2ROW_FAST(uint16_t, 8, 3); else MCMK_IM2ROW_FAST(uint16_t, 8, 5); }
        else      { if (d->k == 3) MCMK_IM2ROW_FAST(float, 4, 3);    else MCMK_IM2ROW_FAST(float, 4, 5); }
#undef MCMK_IM2ROW_FAST
    } else {
        const dim3 grid(stream_grid((size_t)dm.q * dm.p * dm.taps * (d->c / vec), 1), images), block(256);
        if (bf16)
            hipLaunchKernelGGL((im2row_build_kernel<uint16_t, 8>), grid, block, 0, st, static_cast<const uint16_t *>(I_dev),
                               static_cast<uint16_t *>(ws), d->n, d->c, d->h, d->w, d->k, d->pad, d->stride, dm.q, dm.p);
        else
            hipLaunchKernelGGL((im2row_build_kernel<float, 4>), grid, block, 0, st, static_cast<const float *>(I_dev),
                               static_cast<float *>(ws), d->n, d->c, d->h, d->w, d->k, d->pad, d->stride, dm.q, dm.p);
    }
    if ((rc = launch_status())) return rc;
    // O[n][q*P+p][m] = rows[n][q*P+p][:] . Khat[:][m]: the channels-last GEMM
    conv_mcmk_desc folded;
    int ph, pw;
    im2row_plane(d, dm, &folded, &ph, &pw);
    const size_t copies_at = workspace_copies_offset(workspace_matrix_bytes(d, dm, CONV_MCMK_IM2ROW));
    return launch_gemm(&folded, ws, Kp_dev, static_cast<float *>(O_dev), (long long)d->c * dm.taps, ph, pw, 1, st, true, kGemmCopies,
                       ws_bytes > copies_at ? static_cast<char *>(ws) + copies_at : nullptr, ws_bytes > copies_at ? ws_bytes - copies_at : 0);
}

int conv_mcmk_direct(const conv_mcmk_desc *d, const void *I_dev, const void *K_dev, void *O_dev,
                     void *ws, size_t ws_bytes, void *stream)
{
    (void)ws; (void)ws_bytes;
    Dims dm;
    int rc = validate(d, CONV_MCMK_DIRECT, &dm);
    if (rc) return rc;
    if ((rc = common_ptr_checks(I_dev, K_dev, O_dev))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t total = (size_t)d->n * d->m * dm.q * dm.p;
    hipLaunchKernelGGL(direct_f32_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st,
                       static_cast<const float *>(I_dev), static_cast<const float *>(K_dev),
                       static_cast<float *>(O_dev), d->n, d->c, d->h, d->w, d->m, d->k, d->pad, d->stride, dm.q, dm.p);
    return launch_status();
}

int conv_mcmk_select(const conv_mcmk_desc *d, int channels_last, size_t ws_limit_bytes, int *variant, double *est_us)
{
    if (!d || !variant) return CONV_MCMK_ERR_NULL;
    static const int kFirst[] = {CONV_MCMK_KN2ROW, CONV_MCMK_KN2ROW_2PASS, CONV_MCMK_IM2COL, CONV_MCMK_DIRECT};
    static const int kLast[] = {CONV_MCMK_KN2COL, CONV_MCMK_IM2ROW};
    const int *menu = channels_last ? kLast : kFirst;
    const int count = channels_last ? 2 : 4;
    int best = -1, worst_rc = CONV_MCMK_OK;
    double best_cost = 0.0;
    bool over_limit = false;
    for (int i = 0; i < count; ++i) {
        Dims dm;
        const int rc = validate(d, menu[i], &dm);
        if (rc) {
            // a malformed descriptor fails every variant the same way; remember the reason
            if (worst_rc == CONV_MCMK_OK || rc == CONV_MCMK_ERR_SHAPE) worst_rc = rc;
            continue;
        }
        if (conv_mcmk_workspace_bytes(d, menu[i]) > ws_limit_bytes) { over_limit = true; continue; }
        const double cost = variant_cost(d, dm, menu[i]);
        if (best < 0 || cost < best_cost) { best = menu[i]; best_cost = cost; }
    }
    if (best < 0) return over_limit ? CONV_MCMK_ERR_WORKSPACE : worst_rc ? worst_rc : CONV_MCMK_ERR_UNSUPPORTED;
    *variant = best;
    if (est_us) *est_us = best_cost;
    return CONV_MCMK_OK;
}

int conv_mcmk_run(const conv_mcmk_desc *d, int variant, const void *I_dev, const void *K_dev, void *O_dev,
                  void *ws, size_t ws_bytes, void *stream)
{
    switch (variant) {
    case CONV_MCMK_KN2ROW: return conv_mcmk_kn2row(d, I_dev, K_dev, O_dev, ws, ws_bytes, stream);
    case CONV_MCMK_KN2ROW_2PASS: return conv_mcmk_kn2row_2pass(d, I_dev, K_dev, O_dev, ws, ws_bytes, stream);
    case CONV_MCMK_IM2COL: return conv_mcmk_im2col(d, I_dev, K_dev, O_dev, ws, ws_bytes, stream);
    case CONV_MCMK_DIRECT: return conv_mcmk_direct(d, I_dev, K_dev, O_dev, ws, ws_bytes, stream);
    case CONV_MCMK_KN2COL: return conv_mcmk_kn2col(d, I_dev, K_dev, O_dev, ws, ws_bytes, stream);
    case CONV_MCMK_IM2ROW: return conv_mcmk_im2row(d, I_dev, K_dev, O_dev, ws, ws_bytes, stream);
    default: return d ? CONV_MCMK_ERR_UNSUPPORTED : CONV_MCMK_ERR_NULL;
    }
}

int conv_mcmk_cvt_f32_bf16(const void *src_dev, void *dst_dev, size_t count, void *stream)
{
    if (!src_dev || !dst_dev) return CONV_MCMK_ERR_NULL;
    if (misaligned(src_dev) || misaligned(dst_dev)) return CONV_MCMK_ERR_ALIGN;
    if (count == 0) return CONV_MCMK_OK;
    hipLaunchKernelGGL(cvt_f32_bf16_kernel, dim3(grid_for(count, 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const float *>(src_dev),
                       static_cast<uint16_t *>(dst_dev), count);
    return launch_status();
}

}  // extern "C"
