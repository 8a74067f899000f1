// Memory-bound helper kernels: kernel re-ordering, the im2col matrix build, the kn2row
// shift-add post pass, the direct loop nest and the fp32 -> bf16 conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mcmk {

// ---------------------------------------------------------------------------------------------
// float -> bfloat16, round to nearest even; NaN stays a quiet NaN.
__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---------------------------------------------------------------------------------------------
// Kernel re-ordering (section III-A: done once, ahead of time).
// Output element index e decodes as [t][mb][cg][lane][v]; see conv_mcmk.h for the layout.
//   order 0 (kn2row, kn2col): A_t[m][c] = K[m][c][i][j], t = i*k + j, contraction length kc = C
//   order 1 (im2col): t = 0,   A[m][(c*k+i)*k+j] = K[m][c][i][j], contraction length kc = C*k*k
//   order 2 (im2row): t = 0,   A[m][(i*k+j)*C+c] = K[m][c][i][j], contraction length kc = C*k*k
__device__ inline float packed_source(const float *__restrict__ K, int m, int c, int k, int order, int t,
                                      int row, int kk)
{
    if (row >= m) return 0.0f;
    if (order == 0) return kk < c ? K[((size_t)row * c + kk) * k * k + t] : 0.0f;
    if (kk >= c * k * k) return 0.0f;
    if (order == 1) return K[(size_t)row * c * k * k + kk];
    return K[((size_t)row * c + kk % c) * k * k + kk / c];
}

__global__ void prepack_f32_kernel(const float *__restrict__ K, float *__restrict__ Kp,
                                   int m, int c, int k, int mb, int cg, int taps, int order)
{
    const size_t total = (size_t)taps * mb * cg * 256;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int v = e & 3;
        const int lane = (e >> 2) & 63;
        size_t rest = e >> 8;
        const int icg = rest % cg;  rest /= cg;
        const int imb = rest % mb;  rest /= mb;
        const int t = (int)rest;
        const int row = imb * 16 + (lane & 15);
        const int kk = icg * 16 + 4 * v + (lane >> 4);
        Kp[e] = packed_source(K, m, c, k, order, t, row, kk);
    }
}

// bfloat16 form: element index e decodes as [t][mb][cg][lane][e8]; 32-channel groups,
//   Kp = bf16(A_t[mb*16 + lane%16][cg*32 + 8*(lane/16) + e8]).
__global__ void prepack_bf16_kernel(const float *__restrict__ K, uint16_t *__restrict__ Kp,
                                    int m, int c, int k, int mb, int cg, int taps, int order)
{
    const size_t total = (size_t)taps * mb * cg * 512;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int e8 = e & 7;
        const int lane = (e >> 3) & 63;
        size_t rest = e >> 9;
        const int icg = rest % cg;  rest /= cg;
        const int imb = rest % mb;  rest /= mb;
        const int t = (int)rest;
        const int row = imb * 16 + (lane & 15);
        const int kk = icg * 32 + 8 * (lane >> 4) + e8;
        Kp[e] = f32_to_bf16_rne(packed_source(K, m, c, k, order, t, row, kk));
    }
}

// ---------------------------------------------------------------------------------------------
// Input-patch-matrix of section II-B for one batch: Ihat[n][(c*k+i)*k+j][q*P+p]; T is float, or
// uint16_t for bfloat16 bit patterns (zero is all-bits-zero in both).
// One thread owns VEC consecutive output columns of one (image, channel, output row) and writes
// them for all k*k taps, so the input patch is read once (through L1/L2) and every store is a
// full VEC-wide, coalesced row segment of one of the k*k matrix rows -- the k*k-fold replication
// is pure write traffic.  VEC > 1 needs P % VEC == 0 (16-byte aligned stores); the host picks.
// With a stride only the patches of the outputs that exist are built: column (q, p) is centred on
// input (stride*q, stride*p).
template <typename T, int VEC>
__global__ void im2col_build_kernel(const T *__restrict__ I, T *__restrict__ cols,
                                    int n, int c, int h, int w, int k, int pad, int stride, int q, int p)
{
    struct alignas(sizeof(T) * VEC) Pack { T v[VEC]; };
    const int pv = p / VEC;                                   // column groups per row
    const size_t qp = (size_t)q * p;
    const size_t total = (size_t)n * c * q * pv;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int xg = (int)(e % pv);
        size_t rest = e / pv;
        const int oq = (int)(rest % q);
        const size_t nc = rest / q;                           // image * C + channel
        const T *src = I + nc * (size_t)h * w;
        T *dst = cols + nc * (size_t)k * k * qp + (size_t)oq * p + (size_t)xg * VEC;
        const int x0 = xg * VEC * stride - pad;
        for (int i = 0; i < k; ++i) {
            const int y = oq * stride - pad + i;
            const bool row_ok = y >= 0 && y < h;
            for (int j = 0; j < k; ++j) {
                Pack out;
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    const int x = x0 + j + u * stride;
                    out.v[u] = (row_ok && x >= 0 && x < w) ? src[(size_t)y * w + x] : T(0);
                }
                *reinterpret_cast<Pack *>(dst + (size_t)(i * k + j) * qp) = out;
            }
        }
    }
}

// The same matrix for the common case -- unit stride, kernel side KS known at compile time, P a multiple of VEC --
// arranged for memory throughput (the build is k*k-fold write traffic and nothing else): one item per thread and a
// grid as large as the work (no loop-carried index arithmetic; measured faster than several items per thread or a
// grid capped to the chip), 32-bit indices inside one image (images along the grid's second dimension), every load
// of an item issued before its first store, loads through a range-checked buffer descriptor (zero padding = an
// offset beyond the image, no branches), stores marked non-temporal (written once, read by the next kernel).
template <typename T, int VEC, int KS>
__global__ __launch_bounds__(256) void im2col_build_fast_kernel(const T *__restrict__ I, T *__restrict__ cols,
                                                                int n, int c, int h, int w, int pad, int q, int p)
{
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    const unsigned pv = (unsigned)p / VEC;
    const unsigned hw = (unsigned)h * w, qp = (unsigned)q * p;
    const unsigned per_image = (unsigned)c * q * pv;
    for (unsigned in = blockIdx.y; in < (unsigned)n; in += gridDim.y) {
        const T *In = I + (size_t)in * c * hw;
        T *Cn = cols + (size_t)in * c * (KS * KS) * qp;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(In), 0, (int)((size_t)c * hw * sizeof(T)), 0x00020000);
        for (unsigned e = blockIdx.x * 256u + threadIdx.x; e < per_image; e += gridDim.x * 256u) {
            const unsigned xg = e % pv, rest = e / pv;
            const unsigned oq = rest % (unsigned)q, ch = rest / (unsigned)q;
            T in_px[KS][VEC + KS - 1];               // the input patch under VEC neighbouring outputs
#pragma unroll
            for (int r = 0; r < KS; ++r) {
                const int y = (int)oq - pad + r;
#pragma unroll
                for (int u = 0; u < VEC + KS - 1; ++u) {
                    const int x = (int)(xg * VEC) - pad + u;
                    const bool ok = (unsigned)y < (unsigned)h && (unsigned)x < (unsigned)w;
                    const int off = ok ? (int)((ch * hw + (unsigned)y * w + (unsigned)x) * (unsigned)sizeof(T)) : (int)0x80000000u;
                    if constexpr (sizeof(T) == 4) in_px[r][u] = __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 0));
                    else in_px[r][u] = __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b16(rs, off, 0, 0));
                }
            }
            T *dst0 = Cn + (size_t)ch * (KS * KS) * qp + (size_t)oq * p + xg * VEC;
#pragma unroll
            for (int i = 0; i < KS; ++i)
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    vec_t out;
#pragma unroll
                    for (int u = 0; u < VEC; ++u) out[u] = in_px[i][j + u];
                    __builtin_nontemporal_store(out, reinterpret_cast<vec_t *>(dst0 + (size_t)(i * KS + j) * qp));
                }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// im2row (section II-B, last paragraph): patches unrolled into ROWS, from a channels-last input:
//   rows[n][q*P+p][(i*k+j)*C + c] = I[n][stride*q-pad+i][stride*p-pad+j][c]  (zero outside the image).
// One thread copies one VEC-wide channel vector (VEC elements = 16 bytes; C % VEC == 0), so both the
// read and the write are contiguous runs of C elements.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void im2row_build_kernel(const T *__restrict__ I, T *__restrict__ rows,
                                                           int n, int c, int h, int w, int k, int pad, int stride, int q, int p)
{
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    const unsigned cv = (unsigned)c / VEC;
    const unsigned per_image = (unsigned)q * p * k * k * cv;          // below 2^29: 32-bit indices inside an image
    for (unsigned in = blockIdx.y; in < (unsigned)n; in += gridDim.y) {
        const T *In = I + (size_t)in * h * w * c;
        T *Rn = rows + (size_t)in * per_image * VEC;
        for (unsigned e = blockIdx.x * 256u + threadIdx.x; e < per_image; e += gridDim.x * 256u) {
            const unsigned ic = e % cv;
            unsigned rest = e / cv;
            const int j = (int)(rest % (unsigned)k);  rest /= (unsigned)k;
            const int i = (int)(rest % (unsigned)k);  rest /= (unsigned)k;
            const int op = (int)(rest % (unsigned)p);
            const int oq = (int)(rest / (unsigned)p);
            const int y = oq * stride - pad + i, x = op * stride - pad + j;
            vec_t out;
#pragma unroll
            for (int u = 0; u < VEC; ++u) out[u] = T(0);
            if ((unsigned)y < (unsigned)h && (unsigned)x < (unsigned)w)
                out = *reinterpret_cast<const vec_t *>(In + ((size_t)y * w + x) * c + (size_t)ic * VEC);
            __builtin_nontemporal_store(out, reinterpret_cast<vec_t *>(Rn + (size_t)e * VEC));
        }
    }
}

// The same rows for the common case (unit stride, kernel side KS known at compile time), arranged like
// im2col_build_fast_kernel: a thread owns one channel vector of one output position and copies it for all KS*KS taps,
// every load issued before the first store (KS*KS loads in flight per thread instead of one, and one index
// decomposition per KS*KS stores); a wave's stores of one tap are one contiguous run of the row.
template <typename T, int VEC, int KS>
__global__ __launch_bounds__(256) void im2row_build_fast_kernel(const T *__restrict__ I, T *__restrict__ rows,
                                                                int n, int c, int h, int w, int pad, int q, int p)
{
    typedef T vec_t __attribute__((ext_vector_type(VEC)));
    const unsigned cv = (unsigned)c / VEC;
    const unsigned per_image = (unsigned)q * p * cv;
    const unsigned row_elems = (unsigned)(KS * KS) * c;                   // elements of one patch row
    for (unsigned in = blockIdx.y; in < (unsigned)n; in += gridDim.y) {
        const T *In = I + (size_t)in * h * w * c;
        T *Rn = rows + (size_t)in * q * p * row_elems;
        for (unsigned e = blockIdx.x * 256u + threadIdx.x; e < per_image; e += gridDim.x * 256u) {
            const unsigned ic = e % cv, pos = e / cv;
            const int op = (int)(pos % (unsigned)p), oq = (int)(pos / (unsigned)p);
            vec_t v[KS][KS];
#pragma unroll
            for (int i = 0; i < KS; ++i)
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    const int y = oq - pad + i, x = op - pad + j;
#pragma unroll
                    for (int u = 0; u < VEC; ++u) v[i][j][u] = T(0);
                    if ((unsigned)y < (unsigned)h && (unsigned)x < (unsigned)w)
                        v[i][j] = *reinterpret_cast<const vec_t *>(In + ((size_t)y * w + x) * c + (size_t)ic * VEC);
                }
            T *dst = Rn + (size_t)pos * row_elems + (size_t)ic * VEC;
#pragma unroll
            for (int i = 0; i < KS; ++i)
#pragma unroll
                for (int j = 0; j < KS; ++j)
                    __builtin_nontemporal_store(v[i][j], reinterpret_cast<vec_t *>(dst + (size_t)(i * KS + j) * c));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Shift-add post pass of section III-A: O[n][m][q][p] = sum over taps of T[n][t*M+m][s*q+di][s*p+dj]
// (s = stride, 1 in the paper), offsets taken in the 2-D plane; positions outside the H x W plane are discarded.
// One thread owns VEC consecutive columns of one output row (VEC > 1 needs P % VEC == 0).
// KS > 0: the kernel side is a compile-time constant (the tap loops unroll, so every load of the k*k planes is in
// flight before the first add: the pass is a pure memory sweep and waits for nothing else); KS == 0: any side.
template <int VEC, int KS>
__global__ void shift_add_f32_kernel(const float *__restrict__ T, float *__restrict__ O,
                                     int n, int m, int h, int w, int k_arg, int pad, int stride, int q, int p)
{
    const int k = KS > 0 ? KS : k_arg;
    struct alignas(sizeof(float) * VEC) Pack { float v[VEC]; };
    const int pv = p / VEC;
    const size_t hw = (size_t)h * w;
    const size_t total = (size_t)n * m * q * pv;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int xg = (int)(e % pv);
        size_t rest = e / pv;
        const int oq = (int)(rest % q);
        const size_t nm = rest / q;
        const int im = (int)(nm % m);
        const size_t in = nm / m;
        const float *Tn = T + in * (size_t)k * k * m * hw;
        Pack acc;
#pragma unroll
        for (int u = 0; u < VEC; ++u) acc.v[u] = 0.0f;
#pragma unroll
        for (int i = 0; i < k; ++i) {
            const int y = oq * stride - pad + i;
            if (y < 0 || y >= h) continue;
#pragma unroll
            for (int j = 0; j < k; ++j) {
                const float *row = Tn + ((size_t)(i * k + j) * m + im) * hw + (size_t)y * w;
                const int x0 = xg * VEC * stride - pad + j;
#pragma unroll
                for (int u = 0; u < VEC; ++u) {
                    const int x = x0 + u * stride;
                    if (x >= 0 && x < w) acc.v[u] += row[x];
                }
            }
        }
        *reinterpret_cast<Pack *>(O + (nm * q + oq) * (size_t)p + (size_t)xg * VEC) = acc;
    }
}

// The same post pass for the common case -- unit stride, kernel side KS known at compile time, P a multiple of VEC,
// one image's product matrix below 2 GiB -- arranged for memory throughput like im2col_build_fast_kernel: one item per
// thread, a grid as large as the work, 32-bit indices inside an image, all k*k loads of an item in flight before the
// first add.  Each tap contributes one VEC-wide load at the tap's column offset (4-byte aligned, not 16): a vector
// that crosses a row end of the plane picks up the neighbouring row's values, which the column test below drops, and
// a row outside the plane gets an offset beyond the buffer, which the range check answers with zeros.  Only the
// vectors that reach before the first or beyond the last element of the whole matrix are fetched element by
// element instead (how a partly out-of-range vector load is answered is not relied on).
template <int VEC, int KS>
__global__ __launch_bounds__(256) void shift_add_fast_kernel(const float *__restrict__ T, float *__restrict__ O,
                                                             int n, int m, int h, int w, int pad, int q, int p)
{
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    const unsigned pv = (unsigned)p / VEC;
    const unsigned hw = (unsigned)h * w;
    const unsigned per_image = (unsigned)m * q * pv;
    const int t_elems = (int)((unsigned)(KS * KS) * m * hw);                 // below 2^29
    for (unsigned in = blockIdx.y; in < (unsigned)n; in += gridDim.y) {
        const float *Tn = T + (size_t)in * t_elems;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(Tn), 0, t_elems * 4, 0x00020000);
        for (unsigned e = blockIdx.x * 256u + threadIdx.x; e < per_image; e += gridDim.x * 256u) {
            const unsigned xg = e % pv, rest = e / pv;
            const unsigned oq = rest % (unsigned)q, im = rest / (unsigned)q;
            vec_t v[KS][KS];
#pragma unroll
            for (int i = 0; i < KS; ++i)
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    const int y = (int)oq - pad + i;
                    const int x0 = (int)(xg * VEC) - pad + j;
                    const bool row_ok = (unsigned)y < (unsigned)h;
                    const int off = (int)(((unsigned)(i * KS + j) * m + im) * hw) + y * w + x0;      // element index in the matrix
                    const int boff = row_ok ? off * 4 : (int)0x80000000u;
                    if constexpr (VEC == 4) v[i][j] = __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b128(rs, boff, 0, 0));
                    else if constexpr (VEC == 2) v[i][j] = __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b64(rs, boff, 0, 0));
                    else v[i][j] = __builtin_bit_cast(vec_t, __builtin_amdgcn_raw_buffer_load_b32(rs, boff, 0, 0));
                    if (VEC > 1 && row_ok && (off < 0 || off + VEC > t_elems)) {
#pragma unroll
                        for (int u = 0; u < VEC; ++u) v[i][j][u] = (off + u >= 0 && off + u < t_elems) ? Tn[off + u] : 0.0f;
                    }
                }
            vec_t acc;
#pragma unroll
            for (int u = 0; u < VEC; ++u) acc[u] = 0.0f;
#pragma unroll
            for (int i = 0; i < KS; ++i)
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    const int x0 = (int)(xg * VEC) - pad + j;
#pragma unroll
                    for (int u = 0; u < VEC; ++u)
                        if ((unsigned)(x0 + u) < (unsigned)w) acc[u] += v[i][j][u];
                }
            *reinterpret_cast<vec_t *>(O + ((size_t)in * m * q + (size_t)im * q + oq) * p + xg * VEC) = acc;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Direct loop nest (Eq. 1-3): one output element per thread, plain fp32 FMA.
__global__ void direct_f32_kernel(const float *__restrict__ I, const float *__restrict__ K,
                                  float *__restrict__ O, int n, int c, int h, int w, int m, int k,
                                  int pad, int stride, int q, int p)
{
    const size_t qp = (size_t)q * p;
    const size_t total = (size_t)n * m * qp;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int op = (int)(e % qp);
        const size_t nm = e / qp;
        const int im = (int)(nm % m);
        const size_t in = nm / m;
        const int oq = op / p, ox = op % p;
        const float *img = I + in * (size_t)c * h * w;
        const float *ker = K + (size_t)im * c * k * k;
        float acc = 0.0f;
        for (int ch = 0; ch < c; ++ch)
            for (int i = 0; i < k; ++i) {
                const int y = oq * stride - pad + i;
                if (y < 0 || y >= h) continue;
                for (int j = 0; j < k; ++j) {
                    const int x = ox * stride - pad + j;
                    if (x < 0 || x >= w) continue;
                    acc = fmaf(img[((size_t)ch * h + y) * w + x], ker[(ch * k + i) * k + j], acc);
                }
            }
        O[e] = acc;
    }
}

// ---------------------------------------------------------------------------------------------
// Zero `count` floats (count a multiple of 4 is not required; dst 16-byte aligned).
__global__ void fill_zero_kernel(float *__restrict__ dst, size_t count)
{
    const size_t vec = count / 4;
    float4 *d4 = reinterpret_cast<float4 *>(dst);
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < vec; e += (size_t)gridDim.x * blockDim.x)
        d4[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (blockIdx.x == 0 && threadIdx.x < count - vec * 4) dst[vec * 4 + threadIdx.x] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// Add up the PARTS copies of a result that the parts of a split contraction stored one after the other
// (copy i starts stride * i floats into src; stride a multiple of 4, both pointers 16-byte aligned):
// dst[e] = ((src[0][e] + src[1][e]) + src[2][e]) + ...  -- always in this order, so the sum does not depend on
// which workgroup finished first.  One 16-byte item per thread, every load issued before the first add.
template <int PARTS>
__global__ __launch_bounds__(256) void sum_parts_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                        size_t count, size_t stride)
{
    typedef float vec_t __attribute__((ext_vector_type(4)));
    const size_t vec = count / 4;
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e < vec) {
        vec_t v[PARTS];
#pragma unroll
        for (int i = 0; i < PARTS; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(src + (size_t)i * stride) + e);
        vec_t sum = v[0];
#pragma unroll
        for (int i = 1; i < PARTS; ++i) sum += v[i];
        __builtin_nontemporal_store(sum, reinterpret_cast<vec_t *>(dst) + e);
    }
    if (blockIdx.x == 0 && threadIdx.x < count - vec * 4) {
        const size_t t = vec * 4 + threadIdx.x;
        float sum = src[t];
#pragma unroll
        for (int i = 1; i < PARTS; ++i) sum += src[(size_t)i * stride + t];
        dst[t] = sum;
    }
}

// ---------------------------------------------------------------------------------------------
// Measurement aids: the machine rates the benchmark compares the kernels with.
//
// Register-only matrix-core loop: 16 independent accumulators per wave, operands fixed in registers, no memory
// access inside the loop.  The instruction is written out so that operands and accumulators stay where they are
// (the compiler's own allocation for the builtin moves accumulators between the two register files).
template <bool BF16>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float *__restrict__ sink, int iters)
{
    typedef float v4f __attribute__((ext_vector_type(4)));
    constexpr int NACC = 16;
    v4f acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = v4f{0.f, 0.f, 0.f, 0.f};
    // operand bit patterns that are ordinary small numbers in either type (0x3c003c00: two bf16 of 2^-7)
    const unsigned lane = threadIdx.x & 63u;
    v4f a4, b4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        a4[e] = __uint_as_float(0x3c003c00u + ((lane & 7u) << 16));
        b4[e] = __uint_as_float(0x3c003c00u + ((lane >> 3) << 16));
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NACC; ++i) {
            if constexpr (BF16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a4), "v"(b4));
            else asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a4[0]), "v"(b4[0]));
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i) sum += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}

// Plain copy, 16 bytes per thread, non-temporal (the form that measured fastest: more accesses per thread or a grid
// capped to the chip are slower).
__global__ __launch_bounds__(256) void probe_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t count)
{
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f *s = reinterpret_cast<const v4f *>(src);
    v4f *d = reinterpret_cast<v4f *>(dst);
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (size_t)gridDim.x * 256)
        __builtin_nontemporal_store(__builtin_nontemporal_load(s + e), d + e);
}

__global__ void cvt_f32_bf16_kernel(const float *__restrict__ src, uint16_t *__restrict__ dst, size_t count)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count;
         e += (size_t)gridDim.x * blockDim.x)
        dst[e] = f32_to_bf16_rne(src[e]);
}

}  // namespace mcmk
