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
__global__ __launch_bounds__(kLowThreads) void im2col_lower_kernel(const Geometry g, const float *__restrict__ act_all,
                                                                  const Producer prod, T *__restrict__ lowered_all, const int ldb,
                                                                  const int64_t image_stride)
{
    // image blockIdx.y: its own lowered matrix, image_stride elements after the previous one
    const float *__restrict__ act = act_all + static_cast<int64_t>(blockIdx.y) * g.C * g.H * g.W;
    T *__restrict__ lowered = lowered_all + blockIdx.y * image_stride;
    const int N = g.Oh * g.Ow;
    const int chunks = (N + kLowCols - 1) / kLowCols;
    const int row = blockIdx.x / chunks;                  // (c*kh + l)*kw + w
    const int col0 = (blockIdx.x - row * chunks) * kLowCols;
    const int w = row % g.kw, l = (row / g.kw) % g.kh, c = row / (g.kw * g.kh);
    const float *chan = act + static_cast<int64_t>(c) * g.H * g.W;
    const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;
    for (int col = col0 + threadIdx.x; col < min(col0 + kLowCols, N); col += kLowThreads) {
        const int y = col / g.Ow, x = col - y * g.Ow;
        const int hr = y * g.stride + l - g.pad_h, jr = x * g.stride + w - g.pad_w;
        const float v = (hr >= 0 && hr < g.H && jr >= 0 && jr < g.W) ? produced(chan[hr * g.W + jr], prod, bias_c) : 0.0f;
        lowered[static_cast<int64_t>(row) * ldb + col] = lowered_cast<T>(v);
    }
}

// bf16 lowered matrix, laid out for the matrix cores: [ceil(Kd/4)][ldb][4], i.e. the four
// consecutive contraction indices one MFMA lane consumes sit next to each other (8 bytes) and
// consecutive output positions follow each other.  Rows beyond Kd are zero.
__global__ __launch_bounds__(kLowThreads) void im2col_lower_bf16_kernel(const Geometry g,
                                                                       const float *__restrict__ act_all, const Producer prod,
                                                                       uint16_t *__restrict__ lowered_all, const int ldb,
                                                                       const int64_t image_stride)
{
    const float *__restrict__ act = act_all + static_cast<int64_t>(blockIdx.y) * g.C * g.H * g.W;
    uint16_t *__restrict__ lowered = lowered_all + blockIdx.y * image_stride;
    const int N = g.Oh * g.Ow, Kd = g.C * g.kh * g.kw;
    const int chunks = (N + kLowCols - 1) / kLowCols;
    const int k4 = blockIdx.x / chunks;
    const int col0 = (blockIdx.x - k4 * chunks) * kLowCols;
    for (int col = col0 + threadIdx.x; col < min(col0 + kLowCols, N); col += kLowThreads) {
        const int y = col / g.Ow, x = col - y * g.Ow;
        uint16_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = 4 * k4 + u;
            float f = 0.0f;
            if (row < Kd) {
                const int w = row % g.kw, l = (row / g.kw) % g.kh, c = row / (g.kw * g.kh);
                const int hr = y * g.stride + l - g.pad_h, jr = x * g.stride + w - g.pad_w;
                if (hr >= 0 && hr < g.H && jr >= 0 && jr < g.W)
                    f = produced(act[(static_cast<int64_t>(c) * g.H + hr) * g.W + jr], prod,
                                 (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f);
            }
            v[u] = to_bf16(f);
        }
        uint2 packed;
        packed.x = v[0] | (static_cast<uint32_t>(v[1]) << 16);
        packed.y = v[2] | (static_cast<uint32_t>(v[3]) << 16);
        *reinterpret_cast<uint2 *>(lowered + (static_cast<int64_t>(k4) * ldb + col) * 4) = packed;
    }
}

// ---- matrix product: C[M x N] = A[M x Kd] * B[Kd x N], row-major, B with row stride ldb ------
constexpr int kGemmThreads = 256;  // 4 wavefronts as 2 x 2, each a 32 x 32 MFMA tile
constexpr int kBM = 64, kBN = 64;
constexpr int kMaxSplitK = 16;

// fp32 operands, v_mfma_f32_32x32x2_f32.  A workgroup owns a 64 x 64 tile of C and one slice
// of the contraction index (split-K: these layers have too few output tiles to fill the chip).
// The next 64x32 / 32x64 operand tiles travel global -> registers while the matrix cores work
// on the current ones in LDS (two LDS stages, one barrier per step).  LDS layouts make both
// MFMA operand reads unit-stride across lanes: At[k][m], Bs[k][n].
constexpr int kBK32 = 32;

template <bool kVecA>
__global__ __launch_bounds__(kGemmThreads) void gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ B_all,
                                                               float *__restrict__ C_all, int M, int N, int Kd, int ldb,
                                                               int k_per_split, int64_t split_stride, int ntn,
                                                               int64_t b_image_stride)
{
    // batched: blockIdx.x = image * ntn + column tile; every image has its own B and its own M x N C
    const int image = blockIdx.x / ntn;
    const float *__restrict__ B = B_all + image * b_image_stride;
    float *__restrict__ C = C_all + static_cast<int64_t>(image) * M * N;
    __shared__ __attribute__((aligned(16))) float At[2][kBK32][kBM];
    __shared__ __attribute__((aligned(16))) float Bs[2][kBK32][kBN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * kBM, n0 = (blockIdx.x % ntn) * kBN;
    const int k_begin = blockIdx.z * k_per_split, k_end = min(Kd, k_begin + k_per_split);
    const int li = lane & 31, lk = lane >> 5;
    floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    // operand tiles in flight: two float4 of A (row = tid % 64: lanes of a wavefront take
    // different rows, so the transposed LDS store is conflict free) and two float4 of B
    float4 ra[2], rb[2];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + u * kGemmThreads;
            {
                const int r = idx & 63, c4 = idx >> 6;          // row, group of four k
                const int gm = m0 + r, gk = k0 + 4 * c4;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (gm < M) {
                    const float *src = A + static_cast<int64_t>(gm) * Kd + gk;
                    if (kVecA && gk + 3 < k_end) v = *reinterpret_cast<const float4 *>(src);
                    else {
                        if (gk + 0 < k_end) v.x = src[0];
                        if (gk + 1 < k_end) v.y = src[1];
                        if (gk + 2 < k_end) v.z = src[2];
                        if (gk + 3 < k_end) v.w = src[3];
                    }
                }
                ra[u] = v;
            }
            {
                const int kr = idx >> 4, n4 = idx & 15;          // k row, group of four n
                const int gk = k0 + kr, gn = n0 + 4 * n4;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                // rows of B are padded to a multiple of four columns: a float4 never leaves its row
                if (gk < k_end && gn < ldb) v = *reinterpret_cast<const float4 *>(B + static_cast<int64_t>(gk) * ldb + gn);
                rb[u] = v;
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + u * kGemmThreads;
            const int r = idx & 63, c4 = idx >> 6;
            At[buf][4 * c4 + 0][r] = ra[u].x;
            At[buf][4 * c4 + 1][r] = ra[u].y;
            At[buf][4 * c4 + 2][r] = ra[u].z;
            At[buf][4 * c4 + 3][r] = ra[u].w;
            const int kr = idx >> 4, n4 = idx & 15;
            *reinterpret_cast<float4 *>(&Bs[buf][kr][4 * n4]) = rb[u];
        }
    };

    fetch(k_begin);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = k_begin; k0 < k_end; k0 += kBK32) {
        const bool more = k0 + kBK32 < k_end;
        if (more) fetch(k0 + kBK32);
#pragma unroll
        for (int kk = 0; kk < kBK32; kk += 2) {
            const float a = At[buf][kk + lk][wm * 32 + li];
            const float b = Bs[buf][kk + lk][wn * 32 + li];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        if (more) stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    // accumulator register r of lane: row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
    float *dst = C + blockIdx.z * split_stride;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        const int gn = n0 + wn * 32 + li;
        if (gm < M && gn < N) dst[static_cast<int64_t>(gm) * N + gn] = acc[r];
    }
}

// C = sum over the split-K slices, ascending (fixed order: repeatable results).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, float *__restrict__ C,
                                                           int64_t total, int splits)
{
    const int64_t i = (blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x) * 4;
    if ((total & 3) == 0 && i + 3 < total) {   // slices stay 16-byte aligned only then
        float4 s = *reinterpret_cast<const float4 *>(partial + i);
        for (int k = 1; k < splits; ++k) {
            const float4 v = *reinterpret_cast<const float4 *>(partial + k * total + i);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        *reinterpret_cast<float4 *>(C + i) = s;
    } else {
        for (int64_t j = i; j < min(i + 4, total); ++j) {
            float s = partial[j];
            for (int k = 1; k < splits; ++k) s += partial[k * total + j];
            C[j] = s;
        }
    }
}

// bf16 operands, v_mfma_f32_32x32x8_bf16_1k, fp32 accumulation; same tiling, split-K and
// software pipeline as the fp32 kernel.  A (fp32 in memory) is rounded to nearest-even while it
// is staged; B is the k-interleaved bf16 lowered matrix, so an MFMA operand is one 8-byte read
// for both: As[m][k], Bs[k/4][n][4].
constexpr int kBK16 = 32;
constexpr int kPad16 = 8;   // keeps rows 8-byte aligned and spreads the 32 operand rows over the banks

template <bool kVecA>
__global__ __launch_bounds__(kGemmThreads) void gemm_bf16_kernel(const float *__restrict__ A,
                                                                const uint16_t *__restrict__ B_all,
                                                                float *__restrict__ C_all, int M, int N, int Kd, int ldb,
                                                                int k_per_split, int64_t split_stride, int ntn,
                                                                int64_t b_image_stride)
{
    const int image = blockIdx.x / ntn;   // batched as in the fp32 kernel
    const uint16_t *__restrict__ B = B_all + image * b_image_stride;
    float *__restrict__ C = C_all + static_cast<int64_t>(image) * M * N;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][kBM][kBK16 + kPad16];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][kBK16 / 4][kBN][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * kBM, n0 = (blockIdx.x % ntn) * kBN;
    const int k_begin = blockIdx.z * k_per_split, k_end = min(Kd, k_begin + k_per_split);
    const int li = lane & 31, lk = lane >> 5;
    floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    float4 ra[2];
    uint4 rb;
    auto fetch = [&](int k0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + u * kGemmThreads;
            const int r = idx & 63, c4 = idx >> 6;
            const int gm = m0 + r, gk = k0 + 4 * c4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gm < M) {
                const float *src = A + static_cast<int64_t>(gm) * Kd + gk;
                if (kVecA && gk + 3 < k_end) v = *reinterpret_cast<const float4 *>(src);
                else {
                    if (gk + 0 < k_end) v.x = src[0];
                    if (gk + 1 < k_end) v.y = src[1];
                    if (gk + 2 < k_end) v.z = src[2];
                    if (gk + 3 < k_end) v.w = src[3];
                }
            }
            ra[u] = v;
        }
        {
            // 8 groups of four k  x  64 columns x 8 bytes: one 16-byte piece (two columns) per thread
            const int kq = tid >> 5, n2 = tid & 31;
            const int gk4 = (k0 >> 2) + kq, gn = n0 + 2 * n2;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            // rows are padded to an even column count and k_begin, k_end are multiples of 4 or Kd
            if (4 * gk4 < k_end && gn < ldb) v = *reinterpret_cast<const uint4 *>(B + (static_cast<int64_t>(gk4) * ldb + gn) * 4);
            rb = v;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + u * kGemmThreads;
            const int r = idx & 63, c4 = idx >> 6;
            uint2 p;
            p.x = to_bf16(ra[u].x) | (static_cast<uint32_t>(to_bf16(ra[u].y)) << 16);
            p.y = to_bf16(ra[u].z) | (static_cast<uint32_t>(to_bf16(ra[u].w)) << 16);
            *reinterpret_cast<uint2 *>(&As[buf][r][4 * c4]) = p;
        }
        const int kq = tid >> 5, n2 = tid & 31;
        *reinterpret_cast<uint4 *>(&Bs[buf][kq][2 * n2][0]) = rb;
    };

    fetch(k_begin);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = k_begin; k0 < k_end; k0 += kBK16) {
        const bool more = k0 + kBK16 < k_end;
        if (more) fetch(k0 + kBK16);
#pragma unroll
        for (int kk = 0; kk < kBK16; kk += 8) {
            const shortx4 a = *reinterpret_cast<const shortx4 *>(&As[buf][wm * 32 + li][kk + 4 * lk]);
            const shortx4 b = *reinterpret_cast<const shortx4 *>(&Bs[buf][kk / 4 + lk][wn * 32 + li][0]);
            acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b, acc, 0, 0, 0);
        }
        if (more) stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    float *dst = C + blockIdx.z * split_stride;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        const int gn = n0 + wn * 32 + li;
        if (gm < M && gn < N) dst[static_cast<int64_t>(gm) * N + gn] = acc[r];
    }
}

}  // namespace

int im2col_ldb(const Geometry &g) { return (g.Oh * g.Ow + 3) / 4 * 4; }

int im2col_splits(const Geometry &g)
{
    const int N = g.Oh * g.Ow, Kd = g.C * g.kh * g.kw, M = g.K;
    const int tiles = ((N + kBN - 1) / kBN) * ((M + kBM - 1) / kBM) * g.N;
    int s = (384 + tiles / 2) / tiles;
    const int cap = Kd / 128;                       // at least four 32-deep steps per slice
    if (s > cap) s = cap;
    if (s > kMaxSplitK) s = kMaxSplitK;
    if (s < 1) s = 1;
    return s;
}

// bytes of one image's lowered matrix (the bf16 variant rounds Kd up to 4), 256-byte aligned
static int64_t lowered_image_bytes(const Geometry &g)
{
    const int64_t Kd = static_cast<int64_t>(g.C) * g.kh * g.kw;
    return ((Kd + 3) * im2col_ldb(g) * 4 + 255) / 256 * 256;
}

int64_t im2col_scratch_bytes(const Geometry &g)
{
    const int64_t partial = static_cast<int64_t>(g.N == 1 ? kMaxSplitK : im2col_splits(g)) * g.N * g.K * g.Oh * g.Ow * 4;
    return lowered_image_bytes(g) * g.N + partial;
}

int launch_im2col_conv(const float *act, const Producer &prod, const Geometry &g, const float *w, void *lowered, float *out,
                       int precision, hipStream_t stream)
{
    const int N = g.Oh * g.Ow, Kd = g.C * g.kh * g.kw, M = g.K;
    const int ldb = im2col_ldb(g);
    const int chunks = (N + kLowCols - 1) / kLowCols;
    const int splits = im2col_splits(g);
    const int k_per_split = ((Kd + splits - 1) / splits + kBK32 - 1) / kBK32 * kBK32;
    const int nsplit = (Kd + k_per_split - 1) / k_per_split;
    const int64_t low_bytes = lowered_image_bytes(g);
    float *partial = reinterpret_cast<float *>(static_cast<char *>(lowered) + low_bytes * g.N);
    float *dst = nsplit > 1 ? partial : out;
    const int ntn = (N + kBN - 1) / kBN;
    const dim3 ggrid(ntn * g.N, (M + kBM - 1) / kBM, nsplit);
    const bool vec_a = Kd % 4 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0;
    const int64_t mn = static_cast<int64_t>(M) * N * g.N;   // the whole batch: one split-K slice
    if (precision == 0) {
        {
            KernelTimer timer("im2col_lower_f32", stream);
            hipLaunchKernelGGL(im2col_lower_kernel<float>, dim3(static_cast<unsigned>(Kd) * chunks, g.N), dim3(kLowThreads),
                               0, stream, g, act, prod, static_cast<float *>(lowered), ldb, low_bytes / 4);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("gemm_f32", stream);
        if (vec_a)
            hipLaunchKernelGGL(gemm_f32_kernel<true>, ggrid, dim3(kGemmThreads), 0, stream, w,
                               static_cast<const float *>(lowered), dst, M, N, Kd, ldb, k_per_split, mn, ntn, low_bytes / 4);
        else
            hipLaunchKernelGGL(gemm_f32_kernel<false>, ggrid, dim3(kGemmThreads), 0, stream, w,
                               static_cast<const float *>(lowered), dst, M, N, Kd, ldb, k_per_split, mn, ntn, low_bytes / 4);
    } else {
        {
            KernelTimer timer("im2col_lower_bf16", stream);
            hipLaunchKernelGGL(im2col_lower_bf16_kernel, dim3(static_cast<unsigned>((Kd + 3) / 4) * chunks, g.N),
                               dim3(kLowThreads), 0, stream, g, act, prod, static_cast<uint16_t *>(lowered), ldb, low_bytes / 2);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("gemm_bf16", stream);
        if (vec_a)
            hipLaunchKernelGGL(gemm_bf16_kernel<true>, ggrid, dim3(kGemmThreads), 0, stream, w,
                               static_cast<const uint16_t *>(lowered), dst, M, N, Kd, ldb, k_per_split, mn, ntn, low_bytes / 2);
        else
            hipLaunchKernelGGL(gemm_bf16_kernel<false>, ggrid, dim3(kGemmThreads), 0, stream, w,
                               static_cast<const uint16_t *>(lowered), dst, M, N, Kd, ldb, k_per_split, mn, ntn, low_bytes / 2);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    if (nsplit > 1) {
        KernelTimer timer("splitk_reduce", stream);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(static_cast<unsigned>((mn / 4 + 256) / 256)), dim3(256), 0, stream,
                           partial, out, mn, nsplit);
        CPOCONV_HIP_TRY(hipGetLastError());
    }
    return CPOCONV_OK;
}

}  // namespace cpoconv
