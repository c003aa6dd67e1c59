// The comparator of Section 3.1: im2col lowering followed by a dense matrix product on the
// matrix cores (the only dense contraction of the path, hence the only MFMA user).
//
//   lowered[(c*kh + l)*kw + w][y*Ow + x] = padded input at (c, y*stride + l, x*stride + w)
//   out[k][y*Ow + x] = sum_q W[k][q] * lowered[q][y*Ow + x],  W = weights seen as K x (C*kh*kw)
//
// fp32: v_mfma_f32_32x32x2_f32.  bf16: operands rounded to nearest-even bf16 (the lowered
// matrix is stored in bf16, the kernel matrix is converted once by a prepare call or on every
// call), v_mfma_f32_32x32x16_bf16, fp32 accumulation.
#include "common.hpp"

#include <algorithm>

namespace cpoconv {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// two floats -> two bf16, round to nearest even (v_cvt_pk_bf16_f32), low half first
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// ---- lowering ------------------------------------------------------------------------------
// A workgroup takes eight channels and a band of whole output rows.  The padded input rows the
// band needs go through LDS once (zeros where the padding is, bias and ReLU of a producing layer
// applied on the way in); every lowered row of those channels - eight channels are kh*kw groups
// of eight rows - is then read back from LDS with an offset that is the same for the whole
// workgroup, and the band's columns, which are consecutive in the lowered matrix, leave as
// contiguous stores.
//   fp32: lowered[Kd][ldb].
//   bf16: lowered[ceil(Kd/8)][ldb][8], the eight consecutive contraction indices one lane hands
//         to v_mfma_f32_32x32x16_bf16 next to each other (16 bytes); rows beyond Kd are zero.
constexpr int kLowThreads = 256;
constexpr int kLowChannels = 8;
constexpr int kLowUnroll = 6;
constexpr int kLowBandCols = 256;   // output positions per band, rounded down to whole rows (at least one)

template <bool kBf16>
__global__ __launch_bounds__(kLowThreads) void im2col_lower_kernel(const Geometry g, const float *__restrict__ act_all,
                                                                  const Producer prod, void *__restrict__ lowered_all,
                                                                  const int ldb, const int64_t image_bytes, const int band_rows,
                                                                  const int parts)
{
    // blockIdx.x = band * parts + part: where a launch has few bands and channel groups, the
    // groups of eight lowered rows of a channel group are shared out over `parts` workgroups
    extern __shared__ float tile[];   // [channel][input row of the band][padded column]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int band = blockIdx.x / parts, part = blockIdx.x - band * parts;
    const int y0 = band * band_rows, rows_out = min(band_rows, g.Oh - y0);
    const int c0 = blockIdx.y * kLowChannels, nc = min(kLowChannels, g.C - c0);
    const float *__restrict__ act = act_all + static_cast<int64_t>(blockIdx.z) * g.C * g.H * g.W;
    const int rows_max = (band_rows - 1) * g.stride + g.kh, rows_in = (rows_out - 1) * g.stride + g.kh;
    const int wp = (g.Ow - 1) * g.stride + g.kw;

    // units of 64 consecutive columns of one (channel, input row); a wavefront takes kLowUnroll of
    // them at a time so that their loads are in flight together
    const int xchunks = (wp + 63) / 64, units = nc * rows_in * xchunks;
    for (int u0 = wave; u0 < units; u0 += (kLowThreads / 64) * kLowUnroll) {
        float v[kLowUnroll];
        int at[kLowUnroll];
#pragma unroll
        for (int q = 0; q < kLowUnroll; ++q) {
            const int u = u0 + (kLowThreads / 64) * q;
            v[q] = 0.0f;
            at[q] = -1;
            if (u < units) {
                const int line = u / xchunks, x = (u - line * xchunks) * 64 + lane;
                const int c = line / rows_in, r = line - c * rows_in;
                const int hr = y0 * g.stride + r - g.pad_h, jr = x - g.pad_w;
                if (x < wp) {
                    at[q] = (c * rows_max + r) * wp + x;
                    if (hr >= 0 && hr < g.H && jr >= 0 && jr < g.W)
                        v[q] = produced(act[map_index(g, c0 + c, hr, jr)], prod,
                                        (prod.relu && prod.bias != nullptr) ? prod.bias[c0 + c] : 0.0f);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < kLowUnroll; ++q)
            if (at[q] >= 0) tile[at[q]] = v[q];
    }
    __syncthreads();

    const int ncols = rows_out * g.Ow, khkw = g.kh * g.kw;
    const int groups = (nc * khkw + 7) / 8, per_part = (groups + parts - 1) / parts;
    const int j_begin = part * per_part, j_end = min(groups, j_begin + per_part);
    const int c_begin = 8 * j_begin / khkw, l_begin = (8 * j_begin - c_begin * khkw) / g.kw,
              w_begin = 8 * j_begin - c_begin * khkw - l_begin * g.kw;
    char *out = static_cast<char *>(lowered_all) + blockIdx.z * image_bytes;
    for (int t = tid; t < ncols; t += kLowThreads) {
        const int y = t / g.Ow, x = t - y * g.Ow;
        const float *mine = tile + y * g.stride * wp + x * g.stride;
        const int col = y0 * g.Ow + t;
        // lowered rows of the channel group in order: (channel, kernel row, kernel column) by counting
        int c = c_begin, l = l_begin, w = w_begin;
        if (kBf16) {
            uint4 *dst = reinterpret_cast<uint4 *>(out) + static_cast<int64_t>(blockIdx.y) * khkw * ldb + col;
            for (int j = j_begin; j < j_end; ++j) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    v[u] = c < nc ? mine[(c * rows_max + l) * wp + w] : 0.0f;
                    if (++w == g.kw) {
                        w = 0;
                        if (++l == g.kh) { l = 0; ++c; }
                    }
                }
                dst[static_cast<int64_t>(j) * ldb] = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]),
                                                                pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
            }
        } else {
            float *dst = reinterpret_cast<float *>(out) + static_cast<int64_t>(c0) * khkw * ldb + col;
            for (int k = 8 * j_begin; k < min(8 * j_end, nc * khkw); ++k) {
                dst[static_cast<int64_t>(k) * ldb] = mine[(c * rows_max + l) * wp + w];
                if (++w == g.kw) {
                    w = 0;
                    if (++l == g.kh) { l = 0; ++c; }
                }
            }
        }
    }
}

// Lowering without the LDS stage, for launches too small to fill the chip with band workgroups
// (a single image): a workgroup takes kDirectCols columns of one lowered row (fp32) or of one
// group of eight rows (bf16) and reads the input directly; neighbouring workgroups re-read the
// same input lines from the caches.
constexpr int kDirectCols = 1024;
constexpr int kLowStagedImages = 8;   // launches of fewer images take the direct kernel (measured: equal at 8, direct faster at 4)

template <bool kBf16>
__global__ __launch_bounds__(kLowThreads) void im2col_lower_direct_kernel(const Geometry g, const float *__restrict__ act_all,
                                                                         const Producer prod, void *__restrict__ lowered_all,
                                                                         const int ldb, const int64_t image_bytes)
{
    const float *__restrict__ act = act_all + static_cast<int64_t>(blockIdx.y) * g.C * g.H * g.W;
    char *out = static_cast<char *>(lowered_all) + blockIdx.y * image_bytes;
    const int N = g.Oh * g.Ow, Kd = g.C * g.kh * g.kw;
    const int chunks = (N + kDirectCols - 1) / kDirectCols;
    const int first = blockIdx.x / chunks;   // the lowered row, or the group of eight
    const int col0 = (blockIdx.x - first * chunks) * kDirectCols;
    const int row0 = kBf16 ? 8 * first : first;
    const int w0 = row0 % g.kw, l0 = (row0 / g.kw) % g.kh, c0 = row0 / (g.kw * g.kh);
    for (int col = col0 + threadIdx.x; col < min(col0 + kDirectCols, N); col += kLowThreads) {
        const int y = col / g.Ow, x = col - y * g.Ow;
        const int hr0 = y * g.stride - g.pad_h, jr0 = x * g.stride - g.pad_w;
        float v[8];
        int w = w0, l = l0, c = c0;
#pragma unroll
        for (int u = 0; u < (kBf16 ? 8 : 1); ++u) {
            const int hr = hr0 + l, jr = jr0 + w;
            v[u] = 0.0f;
            if (row0 + u < Kd && hr >= 0 && hr < g.H && jr >= 0 && jr < g.W)
                v[u] = produced(act[map_index(g, c, hr, jr)], prod,
                                (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f);
            if (++w == g.kw) {
                w = 0;
                if (++l == g.kh) { l = 0; ++c; }
            }
        }
        if (kBf16)
            reinterpret_cast<uint4 *>(out)[static_cast<int64_t>(first) * ldb + col] =
                make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
        else
            reinterpret_cast<float *>(out)[static_cast<int64_t>(first) * ldb + col] = v[0];
    }
}

// The kernel matrix K x Kd (fp32, row-major) in the operand layout of the bf16 product:
// [ceil(Kd/8)][round_up(K,64)][8], rounded to nearest-even bf16, zero filled.
__global__ __launch_bounds__(256) void prepare_weights_bf16_kernel(const float *__restrict__ w, uint16_t *__restrict__ wb,
                                                                  const int M, const int Mp, const int Kd, const int K8)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;   // one 16-byte group: (k8, m)
    if (idx >= K8 * Mp) return;
    const int k8 = idx / Mp, m = idx - k8 * Mp;
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int k = 8 * k8 + u;
        v[u] = (m < M && k < Kd) ? w[static_cast<int64_t>(m) * Kd + k] : 0.0f;
    }
    reinterpret_cast<uint4 *>(wb)[idx] = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]),
                                                    pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
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

// bf16 operands, v_mfma_f32_32x32x16_bf16, fp32 accumulation.  Both operands arrive in the
// 16-byte-group layouts above (A = prepared weights [K8][Mp][8], B = lowered [K8][ldb][8]), so a
// lane's MFMA operand is one 16-byte LDS read and global -> LDS is a straight copy.  Four
// wavefronts as 2 x 2; a wavefront owns TM x TN accumulator tiles of 32 x 32, so the workgroup
// tile is 64*TM x 64*TN.  64 contraction indices per step; the next step's operands travel
// global -> registers while the matrix cores work on the current ones (one LDS stage: several
// workgroups share a compute unit and fill each other's barrier gaps).
constexpr int kBK16 = 64;
constexpr int kG16 = kBK16 / 8;   // 16-byte groups per step along the contraction index

template <int TM, int TN>
__global__ __launch_bounds__(kGemmThreads) void gemm_bf16_kernel(const uint16_t *__restrict__ A,
                                                                const uint16_t *__restrict__ B_all,
                                                                float *__restrict__ C_all, int M, int Mp, int N, int K8, int ldb,
                                                                int g_per_split, int64_t split_stride, int ntn,
                                                                int64_t b_image_stride)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int PA = kG16 * BM / kGemmThreads, PB = kG16 * BN / kGemmThreads;   // 16-byte pieces per thread and step
    const int image = blockIdx.x / ntn;   // batched as in the fp32 kernel
    const uint4 *__restrict__ Ag = reinterpret_cast<const uint4 *>(A);
    const uint4 *__restrict__ Bg = reinterpret_cast<const uint4 *>(B_all + image * b_image_stride);
    float *__restrict__ C = C_all + static_cast<int64_t>(image) * M * N;
    __shared__ uint4 As[kG16][BM];
    __shared__ uint4 Bs[kG16][BN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = (blockIdx.x % ntn) * BN;
    const int g_begin = blockIdx.z * g_per_split, g_end = min(K8, g_begin + g_per_split);
    const int li = lane & 31, lk = lane >> 5;
    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    uint4 ra[PA], rb[PB];
    auto fetch = [&](int g0) {
#pragma unroll
        for (int u = 0; u < PA; ++u) {
            const int idx = tid + u * kGemmThreads;
            const int kq = idx / BM, m = idx % BM;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (g0 + kq < g_end && m0 + m < Mp) v = Ag[static_cast<int64_t>(g0 + kq) * Mp + m0 + m];
            ra[u] = v;
        }
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const int idx = tid + u * kGemmThreads;
            const int kq = idx / BN, n = idx % BN;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (g0 + kq < g_end && n0 + n < ldb) v = Bg[static_cast<int64_t>(g0 + kq) * ldb + n0 + n];
            rb[u] = v;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int u = 0; u < PA; ++u) (&As[0][0])[tid + u * kGemmThreads] = ra[u];
#pragma unroll
        for (int u = 0; u < PB; ++u) (&Bs[0][0])[tid + u * kGemmThreads] = rb[u];
    };

    fetch(g_begin);
    for (int g0 = g_begin; g0 < g_end; g0 += kG16) {
        stage();
        __syncthreads();
        if (g0 + kG16 < g_end) fetch(g0 + kG16);
#pragma unroll
        for (int kk = 0; kk < kG16; kk += 2) {
            // a lane hands over contraction indices 8*(kk + lane/32) ... + 7 of row (column) lane%32
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = __builtin_bit_cast(bf16x8, As[kk + lk][(wm * TM + i) * 32 + li]);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = __builtin_bit_cast(bf16x8, Bs[kk + lk][(wn * TN + j) * 32 + li]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }
    float *dst = C + blockIdx.z * split_stride;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int gm = m0 + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                const int gn = n0 + (wn * TN + j) * 32 + li;
                if (gm < M && gn < N) dst[static_cast<int64_t>(gm) * N + gn] = acc[i][j][r];
            }
}

// Tile shape and contraction split of the bf16 product: the largest workgroup tile that still
// gives every compute unit work, split-K only where even the smallest does not.
struct Bf16Plan {
    int tm, tn, splits;
};

Bf16Plan bf16_plan(const Geometry &g)
{
    const int N = g.Oh * g.Ow, M = g.K, K8 = (g.C * g.kh * g.kw + 7) / 8;
    auto tiles = [&](int tm, int tn) {
        return static_cast<int64_t>((N + 64 * tn - 1) / (64 * tn)) * ((M + 64 * tm - 1) / (64 * tm)) * g.N;
    };
    if (M > 64 && tiles(2, 4) >= 384) return {2, 4, 1};
    if (M > 64 && tiles(2, 2) >= 256) return {2, 2, 1};
    if (tiles(1, 2) >= 256) return {1, 2, 1};
    const int64_t t = tiles(1, 1);
    int s = static_cast<int>((512 + t / 2) / t);
    const int cap = K8 / (2 * kG16);                // at least two 64-deep steps per slice
    if (s > cap) s = cap;
    if (s > kMaxSplitK) s = kMaxSplitK;
    if (s < 1) s = 1;
    return {1, 1, s};
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

// bytes of one image's lowered matrix (the bf16 variant rounds Kd up to 8), 256-byte aligned
static int64_t lowered_image_bytes(const Geometry &g)
{
    const int64_t Kd = static_cast<int64_t>(g.C) * g.kh * g.kw;
    return ((Kd + 7) * im2col_ldb(g) * 4 + 255) / 256 * 256;
}

int64_t im2col_weights_bf16_len(const Geometry &g)
{
    const int64_t K8 = (static_cast<int64_t>(g.C) * g.kh * g.kw + 7) / 8;
    return K8 * ((g.K + 63) / 64 * 64) * 8;
}

static int64_t partial_bytes(const Geometry &g)
{
    const int splits = g.N == 1 ? kMaxSplitK : max(im2col_splits(g), bf16_plan(g).splits);
    return (static_cast<int64_t>(splits) * g.N * g.K * g.Oh * g.Ow * 4 + 255) / 256 * 256;
}

static int64_t weights_region_bytes(const Geometry &g) { return (im2col_weights_bf16_len(g) * 2 + 255) / 256 * 256; }

int64_t im2col_scratch_bytes(const Geometry &g)
{
    // the bf16 kernel matrix of a precision-1 call, then the lowered matrices and the split-K partial sums
    return weights_region_bytes(g) + lowered_image_bytes(g) * g.N + partial_bytes(g);
}

int launch_prepare_weights_bf16(const float *w, const Geometry &g, uint16_t *wb, hipStream_t stream)
{
    const int Kd = g.C * g.kh * g.kw, K8 = (Kd + 7) / 8, Mp = (g.K + 63) / 64 * 64;
    KernelTimer timer("prepare_weights_bf16", stream);
    hipLaunchKernelGGL(prepare_weights_bf16_kernel, dim3((K8 * Mp + 255) / 256), dim3(256), 0, stream, w, wb, g.K, Mp, Kd, K8);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

template <bool kBf16>
static int launch_lower(const float *act, const Producer &prod, const Geometry &g, void *lowered, hipStream_t stream)
{
    if (g.N < kLowStagedImages) {
        const int N = g.Oh * g.Ow, Kd = g.C * g.kh * g.kw;
        const unsigned firsts = kBf16 ? (Kd + 7) / 8 : Kd;
        KernelTimer timer(kBf16 ? "im2col_lower_bf16" : "im2col_lower_f32", stream);
        hipLaunchKernelGGL(im2col_lower_direct_kernel<kBf16>, dim3(firsts * ((N + kDirectCols - 1) / kDirectCols), g.N),
                           dim3(kLowThreads), 0, stream, g, act, prod, lowered, im2col_ldb(g), lowered_image_bytes(g));
        CPOCONV_HIP_TRY(hipGetLastError());
        return CPOCONV_OK;
    }
    int band_rows = kLowBandCols / g.Ow;
    if (band_rows < 1) band_rows = 1;
    if (band_rows > g.Oh) band_rows = g.Oh;
    const int nc = g.C < kLowChannels ? g.C : kLowChannels;
    const int wp = (g.Ow - 1) * g.stride + g.kw;
    auto lds_bytes = [&](int rows) { return static_cast<size_t>(nc) * ((rows - 1) * g.stride + g.kh) * wp * sizeof(float); };
    while (band_rows > 1 && lds_bytes(band_rows) > (48u << 10)) --band_rows;
    const size_t lds = lds_bytes(band_rows);   // one row of output: at most 8 * 11 * 256 floats
    if (lds > (64u << 10))
        CPOCONV_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&im2col_lower_kernel<kBf16>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
    const int bands = (g.Oh + band_rows - 1) / band_rows, cgroups = (g.C + kLowChannels - 1) / kLowChannels;
    // few workgroups: share the kh*kw groups of eight lowered rows of a channel group out
    int parts = static_cast<int>((512 + static_cast<int64_t>(bands) * cgroups * g.N - 1) / (static_cast<int64_t>(bands) * cgroups * g.N));
    parts = std::min(parts, (nc * g.kh * g.kw + 7) / 8);
    const dim3 grid(bands * parts, cgroups, g.N);
    KernelTimer timer(kBf16 ? "im2col_lower_bf16" : "im2col_lower_f32", stream);
    hipLaunchKernelGGL(im2col_lower_kernel<kBf16>, grid, dim3(kLowThreads), lds, stream, g, act, prod, lowered, im2col_ldb(g),
                       lowered_image_bytes(g), band_rows, parts);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

template <int TM, int TN>
static void launch_gemm_bf16(const Geometry &g, const uint16_t *wb, const uint16_t *lowered, float *dst, int g_per_split,
                             int nsplit, int64_t image_stride, hipStream_t stream)
{
    const int N = g.Oh * g.Ow, K8 = (g.C * g.kh * g.kw + 7) / 8, M = g.K, Mp = (M + 63) / 64 * 64;
    const int ntn = (N + 64 * TN - 1) / (64 * TN);
    const dim3 grid(ntn * g.N, (M + 64 * TM - 1) / (64 * TM), nsplit);
    hipLaunchKernelGGL((gemm_bf16_kernel<TM, TN>), grid, dim3(kGemmThreads), 0, stream, wb, lowered, dst, M, Mp, N, K8,
                       im2col_ldb(g), g_per_split, static_cast<int64_t>(M) * N * g.N, ntn, image_stride);
}

int launch_im2col_conv(const float *act, const Producer &prod, const Geometry &g, const void *w, void *scratch, float *out,
                       int precision, hipStream_t stream)
{
    // precision 1: fp32 kernel matrix, brought into the operand layout here, on every call;
    // precision 2: the caller did that once (launch_prepare_weights_bf16)
    if (precision == 1) {
        const int rc = launch_prepare_weights_bf16(static_cast<const float *>(w), g, static_cast<uint16_t *>(scratch), stream);
        if (rc != CPOCONV_OK) return rc;
        w = scratch;
    }
    void *lowered = static_cast<char *>(scratch) + weights_region_bytes(g);
    const int N = g.Oh * g.Ow, Kd = g.C * g.kh * g.kw, M = g.K;
    const int ldb = im2col_ldb(g);
    const int64_t low_bytes = lowered_image_bytes(g);
    float *partial = reinterpret_cast<float *>(static_cast<char *>(lowered) + low_bytes * g.N);
    const int64_t mn = static_cast<int64_t>(M) * N * g.N;   // the whole batch: one split-K slice
    int nsplit = 1;
    if (precision == 0) {
        const int splits = im2col_splits(g);
        const int k_per_split = ((Kd + splits - 1) / splits + kBK32 - 1) / kBK32 * kBK32;
        nsplit = (Kd + k_per_split - 1) / k_per_split;
        float *dst = nsplit > 1 ? partial : out;
        const int ntn = (N + kBN - 1) / kBN;
        const dim3 ggrid(ntn * g.N, (M + kBM - 1) / kBM, nsplit);
        const float *wf = static_cast<const float *>(w);
        const bool vec_a = Kd % 4 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0;
        const int lrc = launch_lower<false>(act, prod, g, lowered, stream);
        if (lrc != CPOCONV_OK) return lrc;
        KernelTimer timer("gemm_f32", stream);
        if (vec_a)
            hipLaunchKernelGGL(gemm_f32_kernel<true>, ggrid, dim3(kGemmThreads), 0, stream, wf,
                               static_cast<const float *>(lowered), dst, M, N, Kd, ldb, k_per_split, mn, ntn, low_bytes / 4);
        else
            hipLaunchKernelGGL(gemm_f32_kernel<false>, ggrid, dim3(kGemmThreads), 0, stream, wf,
                               static_cast<const float *>(lowered), dst, M, N, Kd, ldb, k_per_split, mn, ntn, low_bytes / 4);
    } else {
        const uint16_t *wb = static_cast<const uint16_t *>(w);
        const int lrc = launch_lower<true>(act, prod, g, lowered, stream);
        if (lrc != CPOCONV_OK) return lrc;
        const Bf16Plan plan = bf16_plan(g);
        const int K8 = (Kd + 7) / 8;
        const int g_per_split = ((K8 + plan.splits - 1) / plan.splits + kG16 - 1) / kG16 * kG16;
        nsplit = (K8 + g_per_split - 1) / g_per_split;
        float *dst = nsplit > 1 ? partial : out;
        const uint16_t *low = static_cast<const uint16_t *>(lowered);
        KernelTimer timer("gemm_bf16", stream);
        if (plan.tn == 4)
            launch_gemm_bf16<2, 4>(g, wb, low, dst, g_per_split, nsplit, low_bytes / 2, stream);
        else if (plan.tm == 2)
            launch_gemm_bf16<2, 2>(g, wb, low, dst, g_per_split, nsplit, low_bytes / 2, stream);
        else if (plan.tn == 2)
            launch_gemm_bf16<1, 2>(g, wb, low, dst, g_per_split, nsplit, low_bytes / 2, stream);
        else
            launch_gemm_bf16<1, 1>(g, wb, low, dst, g_per_split, nsplit, low_bytes / 2, stream);
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
