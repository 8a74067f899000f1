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
//   im2col = false: A_t[m][c] = K[m][c][i][j], t = i*k + j, contraction length kc = C
//   im2col = true : t = 0,   A[m][(c*k+i)*k+j] = K[m][c][i][j], contraction length kc = C*k*k
__global__ void prepack_f32_kernel(const float *__restrict__ K, float *__restrict__ Kp,
                                   int m, int c, int k, int mb, int cg, int taps, bool im2col)
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
        float val = 0.0f;
        if (row < m) {
            if (im2col) {
                if (kk < c * k * k) val = K[(size_t)row * c * k * k + kk];
            } else if (kk < c) {
                val = K[((size_t)row * c + kk) * k * k + t];
            }
        }
        Kp[e] = val;
    }
}

// bfloat16 form: element index e decodes as [t][mb][cg][lane][e8]; 32-channel groups,
//   Kp = bf16(A_t[mb*16 + lane%16][cg*32 + 8*(lane/16) + e8]).
__global__ void prepack_bf16_kernel(const float *__restrict__ K, uint16_t *__restrict__ Kp,
                                    int m, int c, int k, int mb, int cg, int taps, bool im2col)
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
        float val = 0.0f;
        if (row < m) {
            if (im2col) {
                if (kk < c * k * k) val = K[(size_t)row * c * k * k + kk];
            } else if (kk < c) {
                val = K[((size_t)row * c + kk) * k * k + t];
            }
        }
        Kp[e] = f32_to_bf16_rne(val);
    }
}

// ---------------------------------------------------------------------------------------------
// Input-patch-matrix of section II-B for one batch: Ihat[n][(c*k+i)*k+j][q*P+p]; T is float, or
// uint16_t for bfloat16 bit patterns (zero is all-bits-zero in both).
template <typename T>
__global__ void im2col_build_kernel(const T *__restrict__ I, T *__restrict__ cols,
                                    int n, int c, int h, int w, int k, int pad, int q, int p)
{
    const size_t qp = (size_t)q * p;
    const size_t total = (size_t)n * c * k * k * qp;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int op = (int)(e % qp);
        size_t row = e / qp;                           // n*(c*k*k) + (c*k+i)*k+j
        const int j = row % k;  row /= k;
        const int i = row % k;  row /= k;              // row = n*c + channel
        const int y = op / p - pad + i;
        const int x = op % p - pad + j;
        T v = T(0);
        if (y >= 0 && y < h && x >= 0 && x < w) v = I[(row * h + y) * w + x];
        cols[e] = v;
    }
}

// ---------------------------------------------------------------------------------------------
// Shift-add post pass of section III-A: O[n][m][q][p] = sum over taps of T[n][t*M+m][q+di][p+dj],
// offsets taken in the 2-D plane; positions outside the H x W plane are discarded.
__global__ void shift_add_f32_kernel(const float *__restrict__ T, float *__restrict__ O,
                                     int n, int m, int h, int w, int k, int pad, int q, int p)
{
    const size_t qp = (size_t)q * p, hw = (size_t)h * w;
    const size_t total = (size_t)n * m * qp;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const int op = (int)(e % qp);
        const size_t nm = e / qp;
        const int im = (int)(nm % m);
        const size_t in = nm / m;
        const int oq = op / p, ox = op % p;
        const float *Tn = T + in * (size_t)k * k * m * hw;
        float acc = 0.0f;
        for (int i = 0; i < k; ++i) {
            const int y = oq - pad + i;
            if (y < 0 || y >= h) continue;
            for (int j = 0; j < k; ++j) {
                const int x = ox - pad + j;
                if (x < 0 || x >= w) continue;
                acc += Tn[((size_t)(i * k + j) * m + im) * hw + (size_t)y * w + x];
            }
        }
        O[e] = acc;
    }
}

// ---------------------------------------------------------------------------------------------
// Direct loop nest (Eq. 1-3): one output element per thread, plain fp32 FMA.
__global__ void direct_f32_kernel(const float *__restrict__ I, const float *__restrict__ K,
                                  float *__restrict__ O, int n, int c, int h, int w, int m, int k,
                                  int pad, int q, int p)
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
                const int y = oq - pad + i;
                if (y < 0 || y >= h) continue;
                for (int j = 0; j < k; ++j) {
                    const int x = ox - pad + j;
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
