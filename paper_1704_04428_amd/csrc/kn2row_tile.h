// Workgroup-tile kernel shared by every matrix-core variant (fp32 operands).
//
// One workgroup produces a tile of [16*WM rows] x [TH x TW output positions] of one image.
// The contraction runs over (tap, channel): for every tap (i, j) of the KS x KS kernel the tile
// receives the 1x1-convolution product  A_t[rows x C] . I[C x positions displaced by the tap]
// (paper section III-A), accumulated in the same registers for all taps -- the shift-add of
// kn2row happens as an address offset into the input tile held in LDS, so the k*k partial planes
// never exist in memory.  With KS = 1 and TH = 1 the same kernel is a plain GEMM
// [rows x C] . [C x columns], which is what the staged variants (kn2row two-pass, im2col) call.
//
// Operands
//   A (kernel): pre-ordered in global memory exactly as v_mfma_f32_16x16x4_f32 takes it, so a wave
//     loads its fragments with one coalesced 16-byte load per lane and tap, straight into VGPRs
//     (a register queue two to eight taps deep, the deeper the fewer position blocks a wave has).
//     No LDS traffic for A.
//   B (input): a halo tile of 16 channels x (TH+KS-1) x (TW+KS-1), zero-filled outside the image,
//     staged global -> registers -> LDS one 16-channel chunk ahead through two buffers, or two
//     chunks ahead through four with a barrier after every second chunk.
//     Each lane keeps the LDS address of its output position; a tap is an immediate offset.
//
// MFMA 16x16x4 f32 layouts (lane l of 64):  A[row l%16][k l/16],  B[k l/16][col l%16],
//   D[row 4*(l/16) + v][col l%16] for accumulator register v = 0..3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace mcmk {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kXcds = 8;   // accelerator complex dies on MI355X

// Division of a workgroup index by a launch constant: the host turns the divisor d into a multiplier and a shift,
// floor(n / d) == (n * mul) >> shift for every n below 2^31 (mul = ceil(2^shift / d), shift = 31 + ceil(log2 d): the
// error of the rounded-up reciprocal, below d / 2^shift per unit of n, stays under 1 / d).  Three scalar instructions
// where the compiler's division by a runtime value is thirty-odd dependent ones.
struct FastDiv {
    uint32_t mul, shift;
};

inline FastDiv make_fast_div(uint32_t d)
{
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    return FastDiv{(uint32_t)((((uint64_t)1 << (31 + l)) + d - 1) / d), 31 + l};
}

__device__ inline uint32_t fast_div(uint32_t n, const FastDiv &f) { return (uint32_t)(((uint64_t)n * f.mul) >> f.shift); }

struct TileArgs {
    const float *in;      // [n][c][h][w]
    const float *apk;     // packed A: [taps][mb_per_tap][cg][64][4]
    float *out;           // [n][out_rows][q][p]
    int n, c, h, w;       // input
    int q, p;             // output plane
    int pad;
    int m;                // valid rows per row group
    int mb_per_group;     // 16-row blocks per row group (= ceil(m/16))
    int row_groups;       // 1 for a convolution; k*k when the rows are (tap, m) pairs
    int cg;               // 16-channel groups (= ceil(c/16)) == number of chunks
    int tiles_x, tiles_y; // spatial tiles per image
    int row_tiles;        // ceil(row_groups*mb_per_group / WM)
    FastDiv div_row_tiles, div_tiles_x, div_tiles_y;   // the reciprocals of the three counts above (set by the launcher)
    int csplit;           // 1, or 2: two workgroups share a tile, each takes half the chunks and
                          // adds its partial sums into a zeroed output (a + b is order-independent)
    long long part_stride; // 0: the parts of a split add into `out` with atomics.  Otherwise part i stores its sums
                          // plainly into the copy of the output that starts part_stride * i floats into `out`
                          // (the caller adds the copies up in a fixed order afterwards: no zero fill, no atomics)
    const float *bias;    // [row_groups * m] added to every output of its row, or nullptr (csplit == 1 only)
    int relu;             // nonzero: negative results are stored as zero (csplit == 1 only)
};

template <int KS, int TH, int TW, int WM, int WP, int CCH = 16, int KG = 1, int ST = 1, int VQL = CCH / 4, bool CL = false>
struct TileShape {
    static constexpr int kCC = CCH;                      // channels per chunk, a multiple of 16
    static constexpr int kSC = 4 * VQL;                  // channels of a chunk that are staged and multiplied
    static constexpr int kGroupThreads = 64 * WM * WP;   // one channel group: WM x WP waves
    static constexpr int kThreads = kGroupThreads * KG;
    static constexpr int kHT = (TH - 1) * ST + KS;       // input rows under a tile of TH output rows
    static constexpr int kWT = (TW - 1) * ST + KS;
    static constexpr int kPos = kHT * kWT;               // halo-tile positions per channel
    // Staging deals the tile's elements to the group's threads channel by channel.  When the thread count is
    // a multiple of the positions per channel, a thread keeps one position and walks the channels: one
    // offset pair serves all its slots.  A tile that misses that by less than a tenth is staged as if it
    // had kPosStage positions (the few threads beyond kPos load nothing and store zeros into the padding
    // behind their channel), which frees the registers of the per-slot offsets.
    static constexpr int kPerPass = kGroupThreads / kPos;                // whole channels per pass of the group
    static constexpr bool kPadStage = kPerPass >= 1 && kGroupThreads % kPos != 0 && kGroupThreads % kPerPass == 0 &&
                                      (kGroupThreads / kPerPass) * 10 <= kPos * 11;
    static constexpr int kPosStage = kPadStage ? kGroupThreads / kPerPass : kPos;
    // channel stride in LDS words, >= kPos.  Unit stride: == 16 mod 32, so the four channels one B
    // fragment touches start 16 banks apart.  Stride 2: the 16 positions of a fragment sit on every
    // second bank, and an odd channel stride puts the next channel on the banks between them.
    static constexpr int kCHS = ST == 1 ? ((kPosStage + 15) / 32) * 32 + 16 : (kPosStage | 1);
    // Channels-last input at unit stride keeps the tile position-major instead: the staged channels of one position
    // side by side (what a 16-byte load of four channels brings is one 16-byte LDS store), positions kPS words apart.
    // kPS = channels + 4: a multiple of 4 for the 16-byte stores, and 4 (mod 16) so that the 16 consecutive positions
    // of a B fragment fall on every fourth bank, its four channels on the banks between: two lanes per bank, the least
    // 64 lanes can have.
    static constexpr bool kPosMajor = CL && ST == 1;
    static constexpr int kPS = kSC + 4;
    static constexpr int kBuf = kPosMajor ? kPos * kPS : kSC * kCHS;   // words per LDS buffer
    static constexpr int kNPB = (TH * TW + 15) / 16;     // 16-position blocks per tile
    static constexpr int kPBW = (kNPB + WP - 1) / WP;    // blocks per wave
    static constexpr int kSlots = (kSC * kPosStage + kGroupThreads - 1) / kGroupThreads;
    // LDS buffers per channel group: two (staging one chunk ahead, a barrier per chunk), or four (staging
    // two chunks ahead, a barrier every second chunk) where four buffers for every workgroup that the
    // wave count lets share a compute unit still fit its 160 KB
    static constexpr int kNBuf =
        (KG == 1 && 4 * (size_t)kBuf * sizeof(float) * (16 / (WM * WP) > 0 ? 16 / (WM * WP) : 1) <= 160 * 1024) ? 4 : 2;
    static constexpr size_t kLdsBytes = (size_t)kNBuf * KG * kBuf * sizeof(float);
};

// CL = false: input [n][c][h][w], output [n][rows][q][p] (kn2row).
// CL = true : channels last (c a multiple of 4), input [n][h][w][c], output [n][q][p][rows] -- the layout of the paper's
//             kn2col variant (section III-A, last paragraph); the packed kernel and the whole
//             accumulation are the same, only the staging gather and the final store differ.
// ST: stride of the convolution (1 or 2).  Output position (y, x) reads the input tile at
//     (ST*y + tap row, ST*x + tap column); the paper treats unit stride only (section II-A), the
//     kn2row sum itself does not change.
// KG > 1: the workgroup holds KG channel groups of WM x WP waves each.  Group g takes the chunks
//         g, g+KG, g+2KG, ... of the tile (its own LDS buffers, its own staging), and the groups'
//         partial sums are added through LDS at the end in a fixed order.  This is the split of the
//         contraction for layers with too few tiles to fill the chip (small images, deep channels):
//         no atomics, no zero fill, and -- because group g's waves are rotated by g along the position
//         axis -- every SIMD ends up with the same number of position blocks.
// VQL: channel quads of a chunk that are staged and multiplied: all CCH / 4 of them, or 1 for layers of up to
//      four channels (an RGB first layer), whose single chunk would otherwise be three quarters zeros: a
//      quarter of the loads, the LDS and the products.  The packed kernel is the same.
// V4: the flat plain-product shape (1 x 224 positions, 32-channel chunks, 512 threads) on a plane whose length is a
//     multiple of 4: a tile row is then whole aligned 16-byte vectors of memory, so a thread stages four 16-byte
//     loads and four 16-byte LDS stores per chunk where the element-wise plan takes fourteen of each.
template <int KS, int TH, int TW, int WM, int WP, int CCH = 16, bool CL = false, int KG = 1, int ST = 1, int VQL = CCH / 4, bool V4 = false>
__global__ __launch_bounds__(64 * WM * WP * KG) void kn2row_tile_f32(const TileArgs a)
{
    static_assert(!V4 || (!CL && KS == 1 && TH == 1 && TW == 224 && KG == 1 && ST == 1 && CCH == 32 && VQL == 8 && WM * WP == 8),
                  "the vector staging plan is built for the flat shape");
    using S = TileShape<KS, TH, TW, WM, WP, CCH, KG, ST, VQL, CL>;
    static_assert(VQL == CCH / 4 || (!CL && KG == 1 && CCH == 16), "the lean form exists for [C][H][W] input without channel groups");
    static_assert(CCH % 16 == 0, "a chunk is a whole number of packed 16-channel groups");
    constexpr int NQ = CCH / 16;                   // packed A vectors per tap and chunk
    constexpr int CC = S::kCC, SC = S::kSC, NT = S::kGroupThreads, WT = S::kWT, POS = S::kPos, POSS = S::kPosStage, CHS = S::kCHS;
    constexpr int PBW = S::kPBW, NPB = S::kNPB, SLOTS = S::kSlots, BUF = S::kBuf, NBUF = S::kNBuf;
    constexpr bool PM = S::kPosMajor;              // position-major tile (channels last, unit stride)
    constexpr int PS = S::kPS;
    // position blocks are dealt evenly to the WP waves: the first REM waves own PBW blocks, the
    // others PBW-1 (all own PBW when the split is exact)
    constexpr int REM = NPB % WP;
    constexpr bool kRagged = REM != 0;
    static_assert(NPB >= WP, "every wave needs at least one position block");

    extern __shared__ float lds_all[];

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kg = wave_all / (WM * WP);                          // channel group of this wave
    // waves go to SIMD (wave index % 4); rotating the group's waves by kg along the position axis
    // gives each SIMD one wave of every position share
    const int wave = (wave_all % (WM * WP) + kg * WM) % (WM * WP);
    const int tid = wave * 64 + lane;                             // thread index inside the group
    const int wm = wave % WM;
    const int wp = wave / WM;
    float *const lds = lds_all + (size_t)kg * NBUF * BUF;         // this group's buffers

    // ---- which tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so
    // the launch index is re-mapped to give every XCD a contiguous run of tiles: the row tiles that
    // share one input tile, and spatially adjacent tiles that share halo columns and output cache
    // lines, then meet in the same L2.
    int bid = blockIdx.x;
    {
        const int per_xcd = gridDim.x / kXcds;
        if (bid < per_xcd * kXcds) bid = (bid % kXcds) * per_xcd + bid / kXcds;
    }
    // (a division by a launch constant is thirty-odd dependent scalar instructions: the counts come with their
    // reciprocals, and the number of parts is a power of two)
    unsigned ubid = (unsigned)bid;
    int part = 0;
    if (a.csplit > 1) { part = (int)(ubid & (unsigned)(a.csplit - 1));  ubid >>= __builtin_ctz((unsigned)a.csplit); }
    unsigned quot = fast_div(ubid, a.div_row_tiles);
    const int rt = (int)(ubid - quot * (unsigned)a.row_tiles);  ubid = quot;
    quot = fast_div(ubid, a.div_tiles_x);
    const int tx = (int)(ubid - quot * (unsigned)a.tiles_x);    ubid = quot;
    quot = fast_div(ubid, a.div_tiles_y);
    const int ty = (int)(ubid - quot * (unsigned)a.tiles_y);    ubid = quot;
    const int img = (int)ubid;
    const int x0 = tx * TW, y0 = ty * TH;                         // first output position of the tile
    const int ix0 = x0 * ST - a.pad, iy0 = y0 * ST - a.pad;       // input position under halo-tile element (0, 0)

    const int total_rb = a.row_groups * a.mb_per_group;
    int rb = rt * WM + wm;                       // this wave's 16-row block
    const bool rb_valid = rb < total_rb;
    if (!rb_valid) rb = total_rb - 1;            // keep loads in bounds; nothing is stored
    // row group (tap index when rows are (tap, m)): a convolution has one
    const int grp = a.row_groups > 1 ? (int)((unsigned)rb / (unsigned)a.mb_per_group) : 0;
    const int mbi = rb - grp * a.mb_per_group;

    // ---- staging plan: element e = tid + s*NT of the [CC][POS] halo tile.
    // The image is read through a raw buffer descriptor whose range check returns 0 for any offset
    // at or beyond its size: positions outside the image get an offset of 2 GiB (never valid, and
    // adding a chunk's channel offset cannot wrap it), channels beyond C fall off the end by
    // themselves.  No branch and no select sits between a load and its use.
    const size_t plane = (size_t)a.h * a.w;
    const float *in_img = a.in + (size_t)img * a.c * plane;
    const __amdgpu_buffer_rsrc_t in_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(in_img), 0, (int)((size_t)a.c * plane * sizeof(float)), 0x00020000);
    const uint32_t chunk_bytes = (uint32_t)(CC * plane * sizeof(float));
    const int chunks_total = (a.cg + NQ - 1) / NQ;
    // When the thread count is a multiple of the (staged) positions per channel every thread keeps one
    // position and walks the channels in steps of NT/POSS: one offset pair serves all its slots.
    constexpr bool kRegular = (NT % POSS) == 0;
    constexpr int NOFF = kRegular ? 1 : SLOTS;
    constexpr int CSTEP = kRegular ? NT / POSS : 0;
    uint32_t g_off[NOFF];  // byte offset of the element in chunk 0, or 2 GiB when outside the image
    int l_off[NOFF];       // word offset inside an LDS buffer, or -1 when the slot is unused
#pragma unroll
    for (int s = 0; s < NOFF; ++s) {
        const int e = tid + s * NT;
        const int cl = e / POSS, pos = e % POSS;
        const int r = pos / WT, col = pos % WT;
        const int gy = iy0 + r, gx = ix0 + col;
        const bool used = e < SC * POSS;
        // (unsigned compares fold the two-sided range checks; bitwise and 32-bit, so that the compiler selects
        // instead of branching around a 64-bit product: an image has fewer than 2^29 elements)
        const bool inside = used & (pos < POS) & ((unsigned)gy < (unsigned)a.h) & ((unsigned)gx < (unsigned)a.w);
        const uint32_t elem = (uint32_t)cl * (uint32_t)plane + (uint32_t)gy * (uint32_t)a.w + (uint32_t)gx;
        g_off[s] = inside ? elem * (uint32_t)sizeof(float) : 0x80000000u;
        l_off[s] = used ? cl * CHS + pos : -1;          // pos == r * WT + col; beyond POS: the padding, CHS >= POSS
    }
    static_assert(!kRegular || SLOTS * CSTEP == SC, "regular staging must cover the staged channels exactly");

    // channels last: an item is (channel quad, position): one 16-byte load of four consecutive channels
    // (the host requires C to be a multiple of 4, so every quad is aligned and whole), stored as four
    // words CHS apart.  CHS is 16 mod 32, so channels four apart share their banks: a wave that held all
    // the quads of 16 positions would put four lanes on every bank it touches.  Instead the 64 lanes of
    // one store are two neighbouring quads of 32 consecutive positions (two lanes per bank, the least 64
    // lanes can have), and the next 64 items are the next two quads of the same positions.
    // Offsets are recomputed per chunk (an opaque copy of tid keeps the compiler from
    // hoisting them into more live registers).
    // (With the position-major tile of unit stride the quads of one position are neighbouring lanes instead: a wave's
    // load is whole 64- or 128-byte runs of memory, and its store one 16-byte write per lane.)
    constexpr int QPC = CC / 4;                                   // channel quads per chunk
    constexpr int QH = QPC / 2 > 0 ? QPC / 2 : 1;                 // 64-item groups per 32 positions
    constexpr int VITEMS = PM ? POS * QPC : 64 * QH * ((POS + 31) / 32);
    constexpr int VSLOTS = (VITEMS + NT - 1) / NT;                // items per thread
    auto cl_item = [](int e, int &quad, int &pos) {
        if constexpr (PM) {
            quad = e % QPC;
            pos = e / QPC;
        } else {
            const int grp64 = e >> 6, l = e & 63;
            quad = (l & 1) + 2 * (grp64 % QH);
            pos = 32 * (grp64 / QH) + (l >> 1);
        }
    };
    constexpr int NSTAGE = V4 ? 16 : CL ? 4 * VSLOTS : SLOTS;
    float stage[NSTAGE];
    // vector plan: 64 lanes per channel row (56 vectors in use), 8 channel rows per pass, 4 passes per chunk
    const int v4_p = tid & 63, v4_ch = tid >> 6;
    const bool v4_used = v4_p < TW / 4;
    const uint32_t v4_goff = (V4 && v4_used && x0 + 4 * v4_p < a.w)
        ? ((uint32_t)v4_ch * (uint32_t)plane + (uint32_t)(x0 + 4 * v4_p)) * (uint32_t)sizeof(float) : 0x80000000u;
    const int v4_loff = v4_ch * CHS + 4 * v4_p;
    auto load_chunk = [&](int chunk) {
        if constexpr (CL) {
            int t = tid;
            asm volatile("" : "+v"(t));
#pragma unroll
            for (int s = 0; s < VSLOTS; ++s) {
                int quad, pos;
                cl_item(t + s * NT, quad, pos);
                const int r = pos / WT, col = pos % WT;
                const int gy = iy0 + r, gx = ix0 + col;
                const int ch = chunk * CC + quad * 4;
                const bool ok = pos < POS && gy >= 0 && gy < a.h && gx >= 0 && gx < a.w;
                const uint32_t base = (uint32_t)((((size_t)gy * a.w + gx) * a.c + ch) * sizeof(float));
                const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                    in_rsrc, (int)((ok && ch < a.c) ? base : 0x80000000u), 0, 0));
#pragma unroll
                for (int u = 0; u < 4; ++u) stage[4 * s + u] = v[u];
            }
        } else if constexpr (V4) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                    in_rsrc, (int)(v4_goff + (uint32_t)(8 * s) * (uint32_t)(plane * sizeof(float)) +
                                   (uint32_t)min(chunk, chunks_total) * chunk_bytes), 0, 0));
#pragma unroll
                for (int u = 0; u < 4; ++u) stage[4 * s + u] = v[u];
            }
        } else {
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) {
                const uint32_t off = kRegular ? g_off[0] + (uint32_t)(s * CSTEP) * (uint32_t)(plane * sizeof(float))
                                              : g_off[kRegular ? 0 : s];
                // prefetches run past the last chunk; clamped to the first chunk index beyond the data,
                // they stay out of range (zeros, never used) without the offset growing any further
                stage[s] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                    in_rsrc, (int)(off + (uint32_t)min(chunk, chunks_total) * chunk_bytes), 0, 0));
            }
        }
    };
    auto store_chunk = [&](float *buf) {
        if constexpr (CL) {
            int t = tid;
            asm volatile("" : "+v"(t));
#pragma unroll
            for (int s = 0; s < VSLOTS; ++s) {
                int quad, pos;
                cl_item(t + s * NT, quad, pos);
                if (pos < POS) {
                    if constexpr (PM) {
                        *reinterpret_cast<f32x4 *>(buf + pos * PS + quad * 4) =
                            f32x4{stage[4 * s], stage[4 * s + 1], stage[4 * s + 2], stage[4 * s + 3]};
                    } else {
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            buf[(quad * 4 + u) * CHS + (pos / WT) * WT + (pos % WT)] = stage[4 * s + u];
                    }
                }
            }
        } else if constexpr (V4) {
            if (v4_used) {
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    *reinterpret_cast<f32x4 *>(buf + v4_loff + 8 * s * CHS) =
                        f32x4{stage[4 * s], stage[4 * s + 1], stage[4 * s + 2], stage[4 * s + 3]};
            }
        } else {
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) {
                if (kRegular) buf[l_off[0] + s * CSTEP * CHS] = stage[s];
                else if (l_off[kRegular ? 0 : s] >= 0) buf[l_off[kRegular ? 0 : s]] = stage[s];
            }
        }
    };

    // ---- per-lane LDS offsets of this wave's output positions (B operand: k = lane/16, col = lane%16)
    const int nb_wave = (!kRagged || wp < REM) ? PBW : PBW - 1;                  // wave-uniform
    const int first_pb = kRagged ? wp * (PBW - 1) + min(wp, REM) : wp * PBW;     // first block owned
    int b_off[PBW];
#pragma unroll
    for (int b = 0; b < PBW; ++b) {
        int pp = (first_pb + b) * 16 + (lane & 15);
        if (pp >= TH * TW) pp = 0;
        b_off[b] = PM ? (lane >> 4) + ((pp / TW) * WT + (pp % TW)) * PS : (lane >> 4) * CHS + (pp / TW) * ST * WT + (pp % TW) * ST;
    }

    // ---- A fragments: one f32x4 per lane per tap covers a 16-channel chunk.  They are fetched
    // straight from global memory kDepth taps ahead of use and handed down a short register queue.
    constexpr int T = KS * KS;                   // taps per chunk
    // taps: the fragment has to cross the L2's latency while the wave works through kDepth taps of PBW blocks
    // each, so waves with few blocks look further ahead (a quarter tile's tap is four products, 128 cycles)
    // (not with a 1 x 1 kernel, whose next taps are the next chunks, nor with channel groups: both measured slower)
    constexpr int kDepth = (PBW >= 6 || (KG > 1 && PBW > 1) || T < 4) ? 2 : PBW >= 3 ? 3 : 8;
    const int nchunks = (a.cg + NQ - 1) / NQ;
    // this part's share of the chunks (nchunks * csplit stays far below 2^31: no 64-bit division)
    const int chunk_lo = a.csplit > 1 ? (int)((unsigned)(nchunks * part) / (unsigned)a.csplit) : 0;
    const int chunk_hi = a.csplit > 1 ? (int)((unsigned)(nchunks * (part + 1)) / (unsigned)a.csplit) : nchunks;
    const f32x4 *apk = reinterpret_cast<const f32x4 *>(a.apk);
    struct AFrag { f32x4 q[NQ]; };
    auto load_a = [&](int chunk, int t) {
        // conv: tap planes are [tap][mb][cg]; row-group GEMM: KS == 1 and grp picks the plane
        const size_t tap = (size_t)t + grp;
        const int c0 = min(chunk, nchunks - 1) * NQ;
        AFrag f;
#pragma unroll
        for (int qq = 0; qq < NQ; ++qq) {
            // a chunk may reach past the last packed group: read the last one again (it is zeroed where it is used:
            // a select here, on the value just asked for, makes the wave wait for the load on the spot, and with
            // it for every staging load issued before it)
            const int g16 = min(c0 + qq, a.cg - 1);
            f.q[qq] = apk[((tap * a.mb_per_group + mbi) * a.cg + g16) * 64 + lane];
        }
        return f;
    };

    f32x4 acc[PBW];
#pragma unroll
    for (int b = 0; b < PBW; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};

    AFrag a_queue[kDepth];
    const int chunk_first = chunk_lo + kg;                        // this group's chunks: first, +KG, +2KG, ...
    const int nsteps = (chunk_hi - chunk_lo + KG - 1) / KG;       // the same for every group: barriers match
    // With four buffers and enough chunks to repay a second staged chunk before the first product, the
    // input is staged two chunks ahead and the workgroup meets at a barrier only after every second
    // chunk.  The SIMD serves its oldest ready wave first, so the waves of a chunk finish one after the
    // other and the last one runs its final stretch alone, with nobody to cover its LDS latency, before
    // the barrier lets anyone go on: half as many barriers, half as many such tails.
    const bool deep = NBUF == 4 && nsteps >= 8;                   // the same for the whole workgroup
    const int ahead = deep ? 2 : 1;
    load_chunk(chunk_first);
#pragma unroll
    for (int d = 0; d < kDepth; ++d) a_queue[d] = load_a(chunk_first + KG * (d / T), d % T);
    store_chunk(lds);
    if (deep) {
        load_chunk(chunk_first + KG);
        store_chunk(lds + BUF);
    }
    __syncthreads();

    // One chunk of matrix-core work for NB position blocks (NB is PBW, or PBW-1 for the wave that
    // owns the ragged last share); straight-line code, every LDS offset an immediate.
    auto compute_chunk = [&](auto nb_tag, int chunk) {
        constexpr int NB = decltype(nb_tag)::value;
        constexpr int VQ = VQL;                    // channel quads per chunk
        constexpr int G = T * VQ;                  // steps per chunk: (tap, channel quad)
        const float *bsrc = lds + (((chunk - chunk_first) / KG) & (NBUF - 1)) * BUF;
        float bq[2][NB];                           // B fragments: this step's and the next one's
#pragma unroll
        for (int b = 0; b < NB; ++b) bq[0][b] = bsrc[b_off[b]];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            AFrag a_cur = a_queue[0];
            if constexpr (NQ > 1) {
#pragma unroll
                for (int qq = 1; qq < NQ; ++qq)
                    if (chunk * NQ + qq >= a.cg) a_cur.q[qq] = f32x4{0.f, 0.f, 0.f, 0.f};   // wave-uniform
            }
#pragma unroll
            for (int d = 0; d + 1 < kDepth; ++d) a_queue[d] = a_queue[d + 1];
            a_queue[kDepth - 1] = load_a(chunk + KG * ((t + kDepth) / T), (t + kDepth) % T);
#pragma unroll
            for (int v = 0; v < VQ; ++v) {
                const int g = t * VQ + v;          // step number inside the chunk
                // fetch the next step's fragments while this step's products run
                const int t1 = (g + 1) / VQ, v1 = (g + 1) % VQ;
                if (g + 1 < G) {
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        bq[(g + 1) & 1][b] = PM ? bsrc[b_off[b] + 4 * v1 + ((t1 / KS) * WT + (t1 % KS)) * PS]
                                                : bsrc[b_off[b] + (4 * v1) * CHS + (t1 / KS) * WT + (t1 % KS)];
                }
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur.q[v / 4][v % 4], bq[g & 1][b], acc[b], 0, 0, 0);
                // pin the order: one LDS read of step g+1 between consecutive products of step g,
                // and nothing drifts across steps
                if (g + 1 < G) {
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read ...
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // ... then one MFMA
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // The loop body has no data-dependent branch around its loads: the prefetches for "the next
    // chunk" are issued in the last iteration too (A from the last chunk again, input from beyond
    // the last channel, which the buffer range check turns into zeros) and simply go unused.
    // Step s reads buffer s and refills buffer s + ahead (both modulo NBUF), which was last read in step
    // s + ahead - NBUF: before the last barrier in either mode.  What step s + 1 reads was stored in step
    // s + 1 - ahead, and a barrier lies between the two: after every step, or after every odd one.
    for (int step = 0; step < nsteps; ++step) {
        const int chunk = chunk_first + step * KG;
        load_chunk(chunk + ahead * KG);
        if (KG == 1 || chunk < chunk_hi) {                        // wave-uniform
            if (kRagged && nb_wave != PBW) compute_chunk(std::integral_constant<int, kRagged ? PBW - 1 : PBW>{}, chunk);
            else compute_chunk(std::integral_constant<int, PBW>{}, chunk);
        }
        store_chunk(lds + ((step + ahead) & (NBUF - 1)) * BUF);
        if (!deep || (step & 1)) __syncthreads();
    }

    // ---- add the channel groups' partial sums: groups 1.. park theirs in LDS (the staging buffers
    // are free now), group 0 adds them in group order and goes on to write the tile
    if constexpr (KG > 1) {
        static_assert((size_t)(KG - 1) * WM * WP * PBW * 64 * sizeof(f32x4) <= S::kLdsBytes, "parked sums must fit the staging buffers");
        f32x4 *park = reinterpret_cast<f32x4 *>(lds_all);
        const int slot = (wm + WM * wp) * PBW;                    // same (wm, wp) in every group
        if (kg > 0) {
#pragma unroll
            for (int b = 0; b < PBW; ++b) park[(((kg - 1) * WM * WP * PBW) + slot + b) * 64 + lane] = acc[b];
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int g = 1; g < KG; ++g)
#pragma unroll
            for (int b = 0; b < PBW; ++b) {
                const f32x4 other = park[(((g - 1) * WM * WP * PBW) + slot + b) * 64 + lane];
                acc[b] += other;
            }
    }

    // ---- write the tile: accumulator register v of lane l is row 4*(l/16)+v, position l%16
    if (!rb_valid) return;
    const size_t oplane = (size_t)a.q * a.p;
    const int out_rows = a.row_groups * a.m;
    float *out_img = a.out + (size_t)part * (size_t)a.part_stride + (size_t)img * out_rows * oplane;
    const bool plain = a.csplit == 1 || a.part_stride != 0;       // this workgroup owns what it writes
    if (a.bias != nullptr || a.relu) {
        // layer epilogue on the finished sums: per-row offset, then the rectifier
        const int mrow0 = mbi * 16 + 4 * (lane >> 4);
        f32x4 bv = {0.f, 0.f, 0.f, 0.f};
        if (a.bias != nullptr) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (mrow0 + v < a.m) bv[v] = a.bias[(size_t)grp * a.m + mrow0 + v];
        }
#pragma unroll
        for (int b = 0; b < PBW; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float r = acc[b][v] + bv[v];
                acc[b][v] = (a.relu && r < 0.0f) ? 0.0f : r;      // a NaN stays a NaN
            }
    }
#pragma unroll
    for (int b = 0; b < PBW; ++b) {
        if (b >= nb_wave) continue;
        const int pp = (first_pb + b) * 16 + (lane & 15);
        const int y = y0 + pp / TW, x = x0 + pp % TW;
        if (pp >= TH * TW || y >= a.q || x >= a.p) continue;
        const int mrow0 = mbi * 16 + 4 * (lane >> 4);
        if constexpr (CL) {
            // channels last: the lane's four rows are four consecutive floats of one output position
            float *dst = out_img + ((size_t)y * a.p + x) * out_rows + (size_t)grp * a.m + mrow0;
            if (plain && (out_rows & 3) == 0 && mrow0 + 3 < a.m) {
                *reinterpret_cast<f32x4 *>(dst) = acc[b];
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (mrow0 + v >= a.m) continue;
                    if (plain) dst[v] = acc[b][v];
                    else unsafeAtomicAdd(dst + v, acc[b][v]);
                }
            }
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int mrow = mrow0 + v;
                if (mrow >= a.m) continue;
                float *dst = out_img + (size_t)(grp * a.m + mrow) * oplane + (size_t)y * a.p + x;
                if (plain) *dst = acc[b][v];
                else unsafeAtomicAdd(dst, acc[b][v]);      // hardware fp32 add at the L2
            }
        }
    }
}

}  // namespace mcmk
