// Workgroup-tile kernel for bfloat16 operands with fp32 accumulation: the same decomposition as
// kn2row_tile_f32 (one workgroup = 16*WM*RB rows x a TH x TW output tile; all k*k taps of the kn2row
// sum, paper section III-A, accumulate into the same registers; a tap is an address offset into the
// input tile in LDS), re-shaped for v_mfma_f32_16x16x32_bf16:
//
//   - a chunk is 32 channels, one MFMA per (tap, position block, chunk);
//   - the B operand wants 8 consecutive channels of ONE position per lane, so the halo tile lives in
//     LDS as [channel octet][row][column][8 channels]: the 16 lanes that share an octet read 16
//     bytes each from consecutive columns, i.e. one contiguous 256-byte run -- the only pattern a
//     probe of ds_read_b128 on gfx950 showed to run at full rate.  A 16-position block of a tile
//     that is TW wide continues on the next tile row; the row stride is chosen congruent to
//     16*TW modulo 256 bytes, so the continued part falls on exactly the banks the first part
//     left free.  Global memory stays [C][H][W]; the staging pass transposes: a thread fetches 8
//     channels of two neighbouring positions with eight 4-byte loads, separates the positions with
//     byte permutes and writes two 16-byte LDS entries (see the staging plan in the kernel);
//   - the A operand is again pre-ordered in global memory: one 16-byte load per lane gives the
//     fragment of a (tap, 16-row block, 32-channel chunk).
//
// MFMA 16x16x32 bf16 layouts (lane l of 64):  A[row l%16][k 8*(l/16) + e],  B[k 8*(l/16) + e][col l%16],
//   e = 0..7;  D[row 4*(l/16) + v][col l%16], v = 0..3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "kn2row_tile.h"

namespace mcmk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int KS, int TH, int TW, int WM, int WP, int ST = 1, int KG = 1>
struct TileShapeBf16 {
    static constexpr int kCC = 32;                       // channels per chunk
    static constexpr int kThreads = 64 * WM * WP;
    static constexpr int kHT = (TH - 1) * ST + KS;
    static constexpr int kWT = (TW - 1) * ST + KS;
    static constexpr int kPos = kHT * kWT;
    // bytes between tile rows: >= 16 per column; for unit stride == 16*TW (mod 256), see above; the
    // strided tile is four times the size, and with channel groups there are KG pairs of buffers: both
    // are packed tight to stay inside the LDS (bank conflicts matter little where they are used)
    static constexpr int kRowBytes =
        (ST == 1 && KG == 1) ? ((kWT * 16 - (TW * 16) % 256 + 255) / 256) * 256 + (TW * 16) % 256 : kWT * 16;
    static constexpr int kPlaneBytes = ((kHT * kRowBytes + 255) / 256) * 256;   // one channel octet
    static constexpr int kBufBytes = 4 * kPlaneBytes;
    static constexpr int kNPB = (TH * TW + 15) / 16;
    static constexpr int kPBW = (kNPB + WP - 1) / WP;
    static constexpr int kItems = 4 * kPos;              // (position, channel octet) pairs per chunk
    static constexpr int kSlots = (kItems + kThreads - 1) / kThreads;
    static constexpr size_t kLdsBytes = 2 * (size_t)KG * kBufBytes;
};

// TileArgs is shared with the fp32 kernel; `in` and `apk` point at bf16 data, cg counts 32-channel groups.
// CL = true: channels last (input [n][h][w][c], output [n][q][p][rows], the kn2col layout); needs
// c % 8 == 0 so that a channel octet of one position is one aligned 16-byte load -- the staging
// transpose disappears.
// ST: stride of the convolution (1 or 2), as in kn2row_tile_f32.
// RB: 16-row blocks per wave.  A B fragment read from LDS (1 KB per wave) feeds RB products, and the
//     bf16 product is so short (16 cycles) that one read per product would keep the LDS, not the matrix
//     pipe, busy: four SIMDs x one 1 KB read per 16 cycles is the whole LDS bandwidth of a compute unit.
//     The workgroup covers 16*WM*RB rows.
// KG: channel groups inside the workgroup, as in kn2row_tile_f32: group g (WM x WP waves, its own pair of LDS
//     buffers) takes chunks g, g+KG, ...; the partial sums meet in LDS at the end in a fixed order.  For
//     the short bf16 chunks the gain is not matrix work but latency: a wave can keep only one chunk of
//     staging loads in flight (its loads complete in order, and it also has to wait for its A
//     fragments), so a small-image layer with many channels is a chain of memory round trips, and KG
//     groups walk KG such chains side by side.
template <int KS, int TH, int TW, int WM, int WP, bool CL = false, int ST = 1, int RB = 1, int KG = 1>
__global__ __launch_bounds__(64 * WM * WP * KG) void kn2row_tile_bf16(const TileArgs a)
{
    using S = TileShapeBf16<KS, TH, TW, WM, WP, ST, KG>;
    constexpr int CC = S::kCC, NT = S::kThreads, WT = S::kWT, POS = S::kPos, RSB = S::kRowBytes, PLB = S::kPlaneBytes;
    static_assert(RSB >= WT * 16 && (ST != 1 || KG != 1 || (RSB - TW * 16) % 256 == 0), "row stride rule");
    constexpr int PBW = S::kPBW, NPB = S::kNPB, SLOTS = S::kSlots, BUF = S::kBufBytes;
    constexpr int REM = NPB % WP;
    constexpr bool kRagged = REM != 0;
    static_assert(NPB >= WP, "every wave needs at least one position block");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kg = KG == 1 ? 0 : wave_all / (WM * WP);            // channel group of this wave
    // waves go to SIMD (wave index % 4); rotating the group's waves by kg along the position axis
    // gives each SIMD one wave of every position share
    const int wave = (wave_all % (WM * WP) + kg * WM) % (WM * WP);
    const int tid = wave * 64 + lane;                             // thread index inside the group
    const int wm = wave % WM;
    const int wp = wave / WM;
    unsigned char *const lds_raw = lds_all + (size_t)kg * 2 * BUF;    // this group's two buffers

    // ---- which tile (XCD-aware order, see kn2row_tile_f32)
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
    bool rb_valid[RB];
    int grp[RB], mbi[RB];                        // row group (tap plane of a row-group GEMM) and block inside it
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        int rb = (rt * WM + wm) * RB + r;
        rb_valid[r] = rb < total_rb;
        if (!rb_valid[r]) rb = total_rb - 1;     // keep loads in bounds; nothing is stored
        grp[r] = a.row_groups > 1 ? (int)((unsigned)rb / (unsigned)a.mb_per_group) : 0;
        mbi[r] = rb - grp[r] * a.mb_per_group;
    }

    // ---- staging plan for [C][H][W] input.  The tile wants 8 channels of one position side by side,
    // memory has the positions of one channel side by side: an item is (channel octet, tile row, PAIR
    // of columns), fetched with eight 4-byte loads (one per channel, two positions each) and turned
    // into the two 16-byte LDS entries by eight byte permutes.  Half the loads of a 2-byte gather per
    // element, and the texture addresser, which takes a wave's gather a few lanes at a time, is
    // what this path waits for.  The loads go through a range-checked buffer descriptor: an
    // offset of 2 GiB (pair outside the image) and channels beyond C return 0.  A pair with only
    // one element inside the image (left / right border) reads a dword that lies wholly inside the
    // plane -- at the element, or one element earlier when it is the last of its plane -- and the
    // permute selector of the slot picks the half that holds it (or zeros).  Needs H*W >= 2.
    // A dword at an odd element index costs the texture addresser 16 cycles per wave where an aligned
    // one costs 6 (measured), and the gathers of a chunk queue up behind it: so the pairs of a row start
    // at an even image column when the image width is even (every row and plane then starts at an even
    // element), even if the tile's own first column is odd -- one more pair per row, whose outer halves
    // fall outside the tile and are dropped.  Built where the extra pairs need no further staging slot
    // (a slot more for everyone costs the 14 x 14 tiles more than the alignment of every second tile gains).
    // With channels-last input (CL) an item is simply (channel octet, position): one 16-byte load.
    constexpr int HT = S::kHT;
    constexpr int kPairsPlain = (WT + 1) / 2, kPairsEven = (WT + 2) / 2;
    constexpr bool kEvenPairs = (4 * HT * kPairsEven + NT - 1) / NT == (4 * HT * kPairsPlain + NT - 1) / NT;
    constexpr int PW = kEvenPairs ? kPairsEven : kPairsPlain;   // column pairs per tile row
    constexpr int PITEMS = 4 * HT * PW;
    constexpr int PSLOTS = (PITEMS + NT - 1) / NT;
    constexpr uint32_t kSelLo = 0x05040100u, kSelHi = 0x07060302u, kSelZero = 0x0c0c0c0cu;
    const size_t plane = (size_t)a.h * a.w;
    const uint16_t *in_img = reinterpret_cast<const uint16_t *>(a.in) + (size_t)img * a.c * plane;
    const __amdgpu_buffer_rsrc_t in_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(in_img), 0, (int)((size_t)a.c * plane * sizeof(uint16_t)), 0x00020000);
    const uint32_t plane_bytes = (uint32_t)(plane * sizeof(uint16_t));
    const uint32_t chunk_bytes = (uint32_t)CC * plane_bytes;
    const int nchunks = a.cg;
    // this part's share of the chunks (nchunks * csplit stays far below 2^31: no 64-bit division)
    const int chunk_lo = a.csplit > 1 ? (int)((unsigned)(nchunks * part) / (unsigned)a.csplit) : 0;
    const int chunk_hi = a.csplit > 1 ? (int)((unsigned)(nchunks * (part + 1)) / (unsigned)a.csplit) : nchunks;
    // a chunk index at or beyond chunk_hi (the prefetch past the end, or the step a channel group sits out when the
    // chunks do not divide among the groups) is staged as zeros: its offset is moved beyond the data
    auto staged_chunk = [&](int chunk) { return chunk < chunk_hi ? chunk : a.cg; };
    constexpr int NSEL = CL ? 1 : PSLOTS;
    uint32_t g_off[NSEL];    // byte offset of the slot's dword in the first channel of its octet, chunk 0, or 2 GiB
    uint32_t sel_a[NSEL];    // permute selector for the first column of the pair, ...
    uint32_t sel_b[NSEL];    // ... and for the second
    int l_off[NSEL];         // byte offset of the pair's first column inside an LDS buffer (one entry before the row when that column is -1)
    bool put_a[NSEL];        // the tile row has the pair's first column, ...
    bool put_b[NSEL];        // ... its second column
    if constexpr (!CL) {
        const int shift = (kEvenPairs && (a.w & 1) == 0) ? (ix0 & 1) : 0;      // the same for the whole workgroup
#pragma unroll
        for (int s = 0; s < PSLOTS; ++s) {
            const int e = tid + s * NT;
            const int oct = e / (HT * PW), rem = e % (HT * PW);
            const int r = rem / PW, col = 2 * (rem % PW) - shift;              // -1: only the pair's second column is in the tile
            const int gy = iy0 + r, gx = ix0 + col;
            const bool used = e < PITEMS;
            const bool in_row = used && gy >= 0 && gy < a.h;
            const bool c0 = used && col >= 0 && col < WT, c1 = used && col + 1 < WT;
            const bool v0 = in_row && c0 && gx >= 0 && gx < a.w;
            const bool v1 = in_row && c1 && gx + 1 >= 0 && gx + 1 < a.w;
            long long p = (long long)gy * a.w + gx;         // element index of the dword's lower half inside a plane
            uint32_t sa = kSelZero, sb = kSelZero;
            if (v0 && v1) {
                sa = kSelLo;  sb = kSelHi;
            } else if (v0 || v1) {
                // a single element: the aligned dword that holds it if that lies inside the plane, else the other one
                const long long el = v0 ? p : p + 1;
                const bool low = (el & 1) == 0 ? el + 1 < (long long)plane : el == 0;
                p = low ? el : el - 1;
                (v0 ? sa : sb) = low ? kSelLo : kSelHi;
            }
            g_off[s] = (v0 || v1) ? (uint32_t)(oct * 8) * plane_bytes + (uint32_t)p * 2u : 0x80000000u;
            sel_a[s] = sa;
            sel_b[s] = sb;
            l_off[s] = oct * PLB + r * RSB + col * 16;
            put_a[s] = c0;
            put_b[s] = c1;
        }
    }

    uint32_t stage[NSEL][8];       // channels first: eight 4-byte loads per item (two positions of one channel each)
    u32x4 stage_cl[SLOTS];         // channels last: one 16-byte load per item
    auto load_chunk = [&](int chunk) {
        if constexpr (CL) {
            // item e = tid + s*NT is (channel octet e % 4, position e / 4): 4 lanes read one 64-byte run
            int t = tid;
            asm volatile("" : "+v"(t));
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) {
                const int e = t + s * NT;
                const int oct = e % 4, pos = e / 4;
                const int r = pos / WT, col = pos % WT;
                const int gy = iy0 + r, gx = ix0 + col;
                const int ch = chunk * CC + oct * 8;
                const bool ok = e < S::kItems && gy >= 0 && gy < a.h && gx >= 0 && gx < a.w && ch < a.c && chunk < chunk_hi;
                const uint32_t off = ok ? (uint32_t)((((size_t)gy * a.w + gx) * a.c + ch) * sizeof(uint16_t)) : 0x80000000u;
                stage_cl[s] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(in_rsrc, (int)off, 0, 0));
            }
        } else {
#pragma unroll
            for (int s = 0; s < PSLOTS; ++s)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    stage[s][e] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(
                        in_rsrc, (int)(g_off[s] + (uint32_t)e * plane_bytes + (uint32_t)staged_chunk(chunk) * chunk_bytes), 0, 0);
        }
    };
    auto store_chunk = [&](unsigned char *buf) {
        if constexpr (CL) {
            int t = tid;
            asm volatile("" : "+v"(t));
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) {
                const int e = t + s * NT;
                const int oct = e % 4, pos = e / 4;
                if (e < S::kItems)
                    *reinterpret_cast<u32x4 *>(buf + oct * PLB + (pos / WT) * RSB + (pos % WT) * 16) = stage_cl[s];
            }
        } else {
#pragma unroll
            for (int s = 0; s < PSLOTS; ++s) {
                u32x4 first, second;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // channels 2e and 2e+1 of the octet side by side, for the pair's first and second column
                    first[e] = __builtin_amdgcn_perm(stage[s][2 * e + 1], stage[s][2 * e], sel_a[s]);
                    second[e] = __builtin_amdgcn_perm(stage[s][2 * e + 1], stage[s][2 * e], sel_b[s]);
                }
                if (put_a[s]) *reinterpret_cast<u32x4 *>(buf + l_off[s]) = first;
                if (put_b[s]) *reinterpret_cast<u32x4 *>(buf + l_off[s] + 16) = second;
            }
        }
    };

    // ---- per-lane LDS byte offsets of this wave's output positions (B operand: k octet = lane/16)
    const int nb_wave = (!kRagged || wp < REM) ? PBW : PBW - 1;
    const int first_pb = kRagged ? wp * (PBW - 1) + min(wp, REM) : wp * PBW;
    int b_off[PBW];
#pragma unroll
    for (int b = 0; b < PBW; ++b) {
        int pp = (first_pb + b) * 16 + (lane & 15);
        if (pp >= TH * TW) pp = 0;
        b_off[b] = (lane >> 4) * PLB + (pp / TW) * ST * RSB + (pp % TW) * ST * 16;
    }

    // ---- A fragments, fetched one tap row ahead: a ring of D = KS registers whose slot for tap t is
    // t % D -- static, because D divides the taps per chunk -- refilled right after use with the
    // fragment D taps further on.  (A ring a whole chunk deep measured slower: it costs 24 more
    // VGPRs in a kernel that is already register-bound.)
    constexpr int T = KS * KS;
    constexpr int D = KS;
    static_assert(T % D == 0, "ring slots must be static");
    const u32x4 *apk = reinterpret_cast<const u32x4 *>(a.apk);
    struct AFrag { u32x4 r[RB]; };
    auto load_a = [&](int chunk, int t) {
        AFrag f;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const size_t tap = (size_t)t + grp[r];
            f.r[r] = apk[((tap * a.mb_per_group + mbi[r]) * a.cg + min(chunk, nchunks - 1)) * 64 + lane];
        }
        return f;
    };

    f32x4 acc[RB][PBW];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int b = 0; b < PBW; ++b) acc[r][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    AFrag a_ring[D];
    const int chunk_first = chunk_lo + kg;                        // this group's chunks: first, +KG, +2KG, ...
    load_chunk(chunk_first);
#pragma unroll
    for (int d = 0; d < D; ++d) a_ring[d] = load_a(chunk_first + KG * (d / T), d % T);
    store_chunk(lds_raw);
    __syncthreads();

    // One chunk of matrix-core work.  The (tap, position block) pairs form one sequence of B
    // fragments; each is read from LDS kAhead fragments before its RB products are issued and waits
    // in a short register ring (a ring a whole tap deep costs 2 * NB * 4 registers and pushed the
    // kernel over its budget once a wave held two row blocks).
    auto compute_chunk = [&](auto nb_tag, int chunk, int step) {
        constexpr int NB = decltype(nb_tag)::value;
        constexpr int NF = T * NB;                                 // fragments per chunk
        // with two products per fragment three reads ahead cover the LDS latency; sixteen-wave workgroups (channel
        // groups) have 128 registers per lane and four waves per SIMD to cover it instead
        constexpr int kWant = KG > 1 ? 2 : RB > 1 ? 3 : 4;
        constexpr int kAhead = NF > kWant ? kWant : NF - 1;
        constexpr int R = kAhead + 1;
        const unsigned char *bsrc = lds_raw + (step & 1) * BUF;
        const uint32_t a_keep = (KG > 1 && chunk >= chunk_hi) ? 0u : ~0u;          // wave-uniform
        auto read_frag = [&](int s) {
            const int t = s / NB, b = s % NB;
            return *reinterpret_cast<const u32x4 *>(bsrc + b_off[b] + (t / KS) * RSB + (t % KS) * 16);
        };
        u32x4 ring[R];
#pragma unroll
        for (int s = 0; s < kAhead; ++s) ring[s % R] = read_frag(s);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            AFrag a_cur = a_ring[t % D];
            if constexpr (KG > 1) {
                // the step a group sits out: its A fragments count as zeros (and so was its chunk staged), so the
                // products add nothing and no branch around the chunk's work stands between a load and its use
#pragma unroll
                for (int r = 0; r < RB; ++r) a_cur.r[r] &= a_keep;
            }
            a_ring[t % D] = load_a(chunk + KG * ((t + D) / T), (t + D) % T);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int s = t * NB + b;                                             // position in the fragment sequence
                if (s + kAhead < NF) ring[(s + kAhead) % R] = read_frag(s + kAhead);
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    acc[r][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a_cur.r[r]),
                                                                        __builtin_bit_cast(bf16x8, ring[s % R]),
                                                                        acc[r][b], 0, 0, 0);
                if (s + kAhead < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read ...
                __builtin_amdgcn_sched_group_barrier(0x008, RB, 0);                       // ... then the products of one fragment
            }
            __builtin_amdgcn_sched_barrier(0);                                            // nothing drifts across taps
        }
    };

    const int nsteps = (chunk_hi - chunk_lo + KG - 1) / KG;       // the same for every group: barriers match
    // The wave's share of the position blocks (PBW, or PBW - 1 for the ragged last shares) picks one of two copies of the
    // whole loop, not of a chunk's work inside one loop, and a channel group works through the step it sits out with
    // zeros instead of branching around it: where two paths meet again the compiler pins the A ring and the
    // accumulators to fixed registers with copies, and a copy of a register that a load issued two products ago is
    // still filling waits for that load -- once per chunk, with one or two waves per SIMD to cover it.  (The fp32
    // kernel keeps the choice inside its loop: with four waves per SIMD the wait costs it nothing, and the same
    // change measured 3 - 4 % slower on its channel-group shapes.)
    auto run_steps = [&](auto nb_tag) {
        for (int step = 0; step < nsteps; ++step) {
            const int chunk = chunk_first + step * KG;
            load_chunk(chunk + KG);
            if constexpr (decltype(nb_tag)::value < 0) {
                if (kRagged && nb_wave != PBW) compute_chunk(std::integral_constant<int, kRagged ? PBW - 1 : PBW>{}, chunk, step);
                else compute_chunk(std::integral_constant<int, PBW>{}, chunk, step);
            } else {
                compute_chunk(nb_tag, chunk, step);
            }
            store_chunk(lds_raw + ((step + 1) & 1) * BUF);
            __syncthreads();
        }
    };
    if constexpr (ST == 1) {
        if (kRagged && nb_wave != PBW) run_steps(std::integral_constant<int, kRagged ? PBW - 1 : PBW>{});
        else run_steps(std::integral_constant<int, PBW>{});
    } else {
        // (the strided kernels keep the choice inside the loop: with two copies of their larger loop the compiler
        // spilled the 1 x 4 wave layouts to scratch)
        run_steps(std::integral_constant<int, -1>{});
    }

    // ---- add the channel groups' partial sums: groups 1.. park theirs in LDS (the staging buffers
    // are free now), group 0 adds them in group order and goes on to write the tile
    if constexpr (KG > 1) {
        static_assert((size_t)(KG - 1) * WM * WP * RB * PBW * 1024 <= 2 * (size_t)KG * BUF, "parked sums must fit the staging buffers");
        f32x4 *park = reinterpret_cast<f32x4 *>(lds_all);
        const int slot = (wm + WM * wp) * RB * PBW;               // same (wm, wp) in every group
        if (kg > 0) {
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int b = 0; b < PBW; ++b)
                    park[(((kg - 1) * WM * WP * RB * PBW) + slot + r * PBW + b) * 64 + lane] = acc[r][b];
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int g = 1; g < KG; ++g)
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int b = 0; b < PBW; ++b)
                    acc[r][b] += park[(((g - 1) * WM * WP * RB * PBW) + slot + r * PBW + b) * 64 + lane];
    }

    const size_t oplane = (size_t)a.q * a.p;
    const int out_rows = a.row_groups * a.m;
    float *out_img = a.out + (size_t)part * (size_t)a.part_stride + (size_t)img * out_rows * oplane;
    const bool plain = a.csplit == 1 || a.part_stride != 0;       // this workgroup owns what it writes
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        if (!rb_valid[r]) continue;
        const int mrow0 = mbi[r] * 16 + 4 * (lane >> 4);
        if (a.bias != nullptr || a.relu) {
            // layer epilogue on the finished sums: per-row offset, then the rectifier
            f32x4 bv = {0.f, 0.f, 0.f, 0.f};
            if (a.bias != nullptr) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (mrow0 + v < a.m) bv[v] = a.bias[(size_t)grp[r] * a.m + mrow0 + v];
            }
#pragma unroll
            for (int b = 0; b < PBW; ++b)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = acc[r][b][v] + bv[v];
                    acc[r][b][v] = (a.relu && x < 0.0f) ? 0.0f : x;      // a NaN stays a NaN
                }
        }
#pragma unroll
        for (int b = 0; b < PBW; ++b) {
            if (b >= nb_wave) continue;
            const int pp = (first_pb + b) * 16 + (lane & 15);
            const int y = y0 + pp / TW, x = x0 + pp % TW;
            if (pp >= TH * TW || y >= a.q || x >= a.p) continue;
            if constexpr (CL) {
                float *dst = out_img + ((size_t)y * a.p + x) * out_rows + (size_t)grp[r] * a.m + mrow0;
                if (plain && (out_rows & 3) == 0 && mrow0 + 3 < a.m) {
                    *reinterpret_cast<f32x4 *>(dst) = acc[r][b];
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        if (mrow0 + v >= a.m) continue;
                        if (plain) dst[v] = acc[r][b][v];
                        else unsafeAtomicAdd(dst + v, acc[r][b][v]);
                    }
                }
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int mrow = mrow0 + v;
                    if (mrow >= a.m) continue;
                    float *dst = out_img + (size_t)(grp[r] * a.m + mrow) * oplane + (size_t)y * a.p + x;
                    if (plain) *dst = acc[r][b][v];
                    else unsafeAtomicAdd(dst, acc[r][b][v]);
                }
            }
        }
    }
}

}  // namespace mcmk
