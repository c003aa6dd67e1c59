// The comparator of Section 3.1: im2col lowering followed by a dense matrix product on the
// matrix cores (the only dense contraction of the path, hence the only MFMA user).
//
//   lowered[(c*kh + l)*kw + w][y*Ow + x] = padded input at (c, y*stride + l, x*stride + w)
//   out[k][y*Ow + x] = sum_q W[k][q] * lowered[q][y*Ow + x],  W = weights seen as K x (C*kh*kw)
//
// fp32: v_mfma_f32_32x32x2_f32.  bf16: operands rounded to nearest-even bf16 (the lowered
// matrix is stored in bf16), v_mfma_f32_32x32x8_bf16_1k, fp32 accumulation.
#include "common.hpp"

namespace cpoconv {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((b >> 16) | 0x40u);  // NaN
    b += 0x7fffu + ((b >> 16) & 1u);  // round to nearest, ties to even
    return static_cast<uint16_t>(b >> 16);
}

template <typename T> __device__ __forceinline__ T lowered_cast(float v);
template <> __device__ __forceinline__ float lowered_cast<float>(float v) { return v; }
template <> __device__ __forceinline__ uint16_t lowered_cast<uint16_t>(float v) { return to_bf16(v); }

constexpr int kLowThreads = 256;
constexpr int kLowCols = 1024;  // lowered-matrix columns per workgroup

template <typename T>
__global__ __launch_bounds__(kLowThreads) void im2col_lower_kernel(const Geometry g, const float *__restrict__ act,
                                                                  T *__restrict__ lowered)
{
    const int N = g.Oh * g.Ow;
    const int chunks = (N + kLowCols - 1) / kLowCols;
    const int row = blockIdx.x / chunks;                  // (c*kh + l)*kw + w
    const int col0 = (blockIdx.x - row * chunks) * kLowCols;
    const int w = row % g.kw, l = (row / g.kw) % g.kh, c = row / (g.kw * g.kh);
    const float *chan = act + static_cast<int64_t>(c) * g.H * g.W;
    for (int col = col0 + threadIdx.x; col < min(col0 + kLowCols, N); col += kLowThreads) {
        const int y = col / g.Ow, x = col - y * g.Ow;
        const int hr = y * g.stride + l - g.pad, jr = x * g.stride + w - g.pad;
        const float v = (hr >= 0 && hr < g.H && jr >= 0 && jr < g.W) ? chan[hr * g.W + jr] : 0.0f;
        lowered[static_cast<int64_t>(row) * N + col] = lowered_cast<T>(v);
    }
}

// ---- matrix product: C[M x N] = A[M x Kd] * B[Kd x N], all row-major --------------------
constexpr int kGemmThreads = 256;  // 4 wavefronts as 2 x 2, each a 32 x 32 MFMA tile
constexpr int kBM = 64, kBN = 64;

// fp32 operands.  LDS: As[m][k] (row stride odd: the 32 lanes of an operand column hit 32
// banks), Bs[k][n].
constexpr int kBK32 = 16;

__global__ __launch_bounds__(kGemmThreads) void gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ B,
                                                               float *__restrict__ C, int M, int N, int Kd)
{
    __shared__ float As[kBM][kBK32 + 1];
    __shared__ float Bs[kBK32][kBN + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * kBM, n0 = blockIdx.x * kBN;
    const int li = lane & 31, lk = lane >> 5;
    floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    for (int k0 = 0; k0 < Kd; k0 += kBK32) {
        // A tile 64 x 16: thread -> row tid/4, four consecutive k
        {
            const int r = tid >> 2, kq = (tid & 3) * 4;
            const int gm = m0 + r;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int gk = k0 + kq + u;
                As[r][kq + u] = (gm < M && gk < Kd) ? A[static_cast<int64_t>(gm) * Kd + gk] : 0.0f;
            }
        }
        // B tile 16 x 64: thread -> k row tid/16, four consecutive n
        {
            const int r = tid >> 4, nq = (tid & 15) * 4;
            const int gk = k0 + r;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int gn = n0 + nq + u;
                Bs[r][nq + u] = (gk < Kd && gn < N) ? B[static_cast<int64_t>(gk) * N + gn] : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kBK32; kk += 2) {
            const float a = As[wm * 32 + li][kk + lk];
            const float b = Bs[kk + lk][wn * 32 + li];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    // accumulator register r of lane: row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        const int gn = n0 + wn * 32 + li;
        if (gm < M && gn < N) C[static_cast<int64_t>(gm) * N + gn] = acc[r];
    }
}

// bf16 operands: A (fp32 in memory) is rounded while staged, B is the bf16 lowered matrix.
// LDS holds both with k fastest so that the four consecutive k of an MFMA operand are one
// 8-byte read: As[m][k], Bt[n][k].
constexpr int kBK16 = 32;
constexpr int kPad16 = 4;

__global__ __launch_bounds__(kGemmThreads) void gemm_bf16_kernel(const float *__restrict__ A,
                                                                const uint16_t *__restrict__ B,
                                                                float *__restrict__ C, int M, int N, int Kd)
{
    __shared__ __attribute__((aligned(8))) uint16_t As[kBM][kBK16 + kPad16];
    __shared__ __attribute__((aligned(8))) uint16_t Bt[kBN][kBK16 + kPad16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * kBM, n0 = blockIdx.x * kBN;
    const int li = lane & 31, lk = lane >> 5;
    floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    for (int k0 = 0; k0 < Kd; k0 += kBK16) {
        // A tile 64 x 32: thread -> row tid/4, eight consecutive k
        {
            const int r = tid >> 2, kq = (tid & 3) * 8;
            const int gm = m0 + r;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int gk = k0 + kq + u;
                As[r][kq + u] = (gm < M && gk < Kd) ? to_bf16(A[static_cast<int64_t>(gm) * Kd + gk]) : uint16_t{0};
            }
        }
        // B tile 32 x 64, read along n, stored transposed: thread -> k row tid/8, eight n
        {
            const int r = tid >> 3, nq = (tid & 7) * 8;
            const int gk = k0 + r;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int gn = n0 + nq + u;
                Bt[nq + u][r] = (gk < Kd && gn < N) ? B[static_cast<int64_t>(gk) * N + gn] : uint16_t{0};
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kBK16; kk += 8) {
            const shortx4 a = *reinterpret_cast<const shortx4 *>(&As[wm * 32 + li][kk + 4 * lk]);
            const shortx4 b = *reinterpret_cast<const shortx4 *>(&Bt[wn * 32 + li][kk + 4 * lk]);
            acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        const int gn = n0 + wn * 32 + li;
        if (gm < M && gn < N) C[static_cast<int64_t>(gm) * N + gn] = acc[r];
    }
}

}  // namespace

int launch_im2col_conv(const float *act, const Geometry &g, const float *w, void *lowered, float *out,
                       int precision, hipStream_t stream)
{
    const int N = g.Oh * g.Ow, Kd = g.C * g.kh * g.kw, M = g.K;
    const int chunks = (N + kLowCols - 1) / kLowCols;
    const dim3 lgrid(static_cast<unsigned>(Kd) * chunks);
    const dim3 ggrid((N + kBN - 1) / kBN, (M + kBM - 1) / kBM);
    if (precision == 0) {
        {
            KernelTimer timer("im2col_lower_f32", stream);
            hipLaunchKernelGGL(im2col_lower_kernel<float>, lgrid, dim3(kLowThreads), 0, stream, g, act,
                               static_cast<float *>(lowered));
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("gemm_f32", stream);
        hipLaunchKernelGGL(gemm_f32_kernel, ggrid, dim3(kGemmThreads), 0, stream, w,
                           static_cast<const float *>(lowered), out, M, N, Kd);
    } else {
        {
            KernelTimer timer("im2col_lower_bf16", stream);
            hipLaunchKernelGGL(im2col_lower_kernel<uint16_t>, lgrid, dim3(kLowThreads), 0, stream, g, act,
                               static_cast<uint16_t *>(lowered));
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("gemm_bf16", stream);
        hipLaunchKernelGGL(gemm_bf16_kernel, ggrid, dim3(kGemmThreads), 0, stream, w,
                           static_cast<const uint16_t *>(lowered), out, M, N, Kd);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

}  // namespace cpoconv
