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

// ---------------------------------------------------------------------------------------------
// im2row (section II-B, last paragraph): patches unrolled into ROWS, from a channels-last input:
//   rows[n][q*P+p][(i*k+j)*C + c] = I[n][stride*q-pad+i][stride*p-pad+j][c]  (zero outside the image).
// One thread copies one VEC-wide channel vector (VEC elements = 16 bytes; C % VEC == 0), so both the
// read and the write are contiguous runs of C elements.
template <typename T, int VEC>
__global__ void im2row_build_kernel(const T *__restrict__ I, T *__restrict__ rows,
                                    int n, int c, int h, int w, int k, int pad, int stride, int q, int p)
{
    struct alignas(sizeof(T) * VEC) Pack { T v[VEC]; };
    const int cv = c / VEC;
    const size_t total = (size_t)n * q * p * k * k * cv;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int ic = (int)(e % cv);
        size_t rest = e / cv;
        const int j = (int)(rest % k);  rest /= k;
        const int i = (int)(rest % k);  rest /= k;
        const int op = (int)(rest % p); rest /= p;
        const int oq = (int)(rest % q);
        const size_t in = rest / q;
        const int y = oq * stride - pad + i, x = op * stride - pad + j;
        Pack out;
#pragma unroll
        for (int u = 0; u < VEC; ++u) out.v[u] = T(0);
        if (y >= 0 && y < h && x >= 0 && x < w)
            out = *reinterpret_cast<const Pack *>(I + ((in * h + y) * w + x) * (size_t)c + (size_t)ic * VEC);
        *reinterpret_cast<Pack *>(rows + e * VEC) = out;
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

__global__ void cvt_f32_bf16_kernel(const float *__restrict__ src, uint16_t *__restrict__ dst, size_t count)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count;
         e += (size_t)gridDim.x * blockDim.x)
        dst[e] = f32_to_bf16_rne(src[e]);
}

}  // namespace mcmk
