// Internal declarations shared by the translation units of libcpoconv.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "cpoconv.h"

namespace cpoconv {

constexpr int kMaxTypes = CPOCONV_MAX_K;   // overlap types 0 .. kw-1
constexpr int kMaxCols = CPOCONV_MAX_I;    // padded columns
constexpr int kLanes = 64;                 // wavefront width on CDNA

// Partition / overlap-type table of a layer (Sections 3.1-3.2), built on the host once per
// call and passed to kernels by value.  "Columns" are the encoded ones (covered by a
// partition and part of the unpadded map) in stream order: overlap type ascending, then
// padded column ascending (which is also first-partition ascending).
struct Geometry {
    int32_t C, H, W, K, kh, kw, stride, pad_h, pad_w;
    int32_t Ih, Iw, Oh, Ow;
    int32_t n_cols;                  // encoded columns
    int32_t n_types;                 // present overlap types
    int32_t nop3;                    // NOP type is the 3-entry segment (no column padding, stride 1)
    int32_t top;                     // overlap type CPS packs, -1 if none
    int32_t top_slot;                // its slot in type_id, -1 if none
    int32_t Kpad;                    // K rounded up to a multiple of 64
    int32_t N;                       // images in the launch (1 unless a batched entry point)
    int32_t channel_last;            // the dense input map is H x W x C instead of C x H x W
    uint8_t type_id[kMaxTypes];      // present types, ascending
    uint16_t type_begin[kMaxTypes + 1];  // column range of each present type
    uint8_t col_j[kMaxCols];         // padded column
    uint8_t col_p0[kMaxCols];        // first partition holding it
    uint8_t col_what[kMaxCols];      // column inside that partition
};

// Where element (channel c, row hr, column jr) of one image's dense input map sits.
__device__ __forceinline__ int64_t map_index(const Geometry &g, int c, int hr, int jr)
{
    return g.channel_last ? (static_cast<int64_t>(hr) * g.W + jr) * g.C + c
                          : (static_cast<int64_t>(c) * g.H + hr) * g.W + jr;
}

// Element strides between consecutive images of a batched launch (image 0 is at the base pointers).
struct BatchStrides {
    int64_t ptr, da, in;   // streams and side band: the per-image capacities of the map
    int64_t indices;       // what the convolution reads as IN: the stream itself or the rebuilt CPS indices (entries)
    int64_t mtab, partial, out;
    int64_t columns;       // entries of the column table per image (column-run kernel)
    int32_t map_in16;      // the map's IN stream holds int16 entries
    int32_t indices16;     // so does what the convolution reads as IN (the rebuilt CPS indices always do)
    const int32_t *hdr;    // the map's header (8 ints per image)
    int32_t algo;          // the algorithm the call expects the map to hold
};

// What the column-run kernel knows of one padded column of one channel: where the column's run of
// NZEs starts in DA and which padded rows hold one (maps of at most 64 padded rows).
struct ColumnEntry {
    int32_t begin;             // absolute offset of the run in DA
    int32_t count;             // its length (= set bits)
    uint32_t rows_lo, rows_hi; // bit r: padded row r holds an NZE
};

// A map the convolution must not read: its encoder gave up (hdr[7] equals the header's stamp), or it holds the other
// algorithm's streams (hdr[3]).  Every kernel on the convolution side leaves its outputs alone then.
__device__ __forceinline__ bool map_unusable(const BatchStrides &bs, int image)
{
    const int32_t *h = bs.hdr + static_cast<int64_t>(image) * 8;
    const int failed_in = h[7];   // stamp of the call in which an encoder unit gave up; hdr[6] >> 8: stamp of the header
    return (failed_in != 0 && failed_in == (h[6] >> 8)) || h[3] != bs.algo;
}

// IN entries: int32, or int16 in a compact map (same values).  The stream pointer is typed int32
// either way; offsets count entries.
__device__ __forceinline__ int load_index(const int32_t *in, int64_t n, int in16)
{
    return in16 ? static_cast<int>(reinterpret_cast<const int16_t *>(in)[n]) : in[n];
}
__device__ __forceinline__ void store_index(int32_t *in, int64_t n, int v, int in16)
{
    if (in16) reinterpret_cast<int16_t *>(in)[n] = static_cast<int16_t>(v);
    else in[n] = v;
}
template <typename P> __device__ __forceinline__ P *index_advance(P *in, int64_t entries, int in16)
{
    using Byte = typename std::conditional<std::is_const<P>::value, const char, char>::type;
    return reinterpret_cast<P *>(reinterpret_cast<Byte *>(in) + entries * (in16 ? 2 : 4));
}

// What a kernel that reads a dense map applies to every value on the way in: the end of the layer
// that produced the map (its bias, then the ReLU that makes the input of Eq. 1 sparse), so the
// activated map itself is never stored.
struct Producer {
    const float *bias;   // one float per channel of the map, or nullptr
    int32_t relu;        // 0: the map is taken as it is (bias unused)
};

// value of a map element of a channel with bias b: z = v + b (one fp32 addition, none without a
// bias), then z if z > 0, else +0.  The test is on the bit pattern (0 < bits <= +inf), so negative
// values, both zeros and NaN give +0 whatever the denormal mode of the comparison would be.
__device__ __forceinline__ float produced(float v, const Producer &prod, float b)
{
    if (prod.relu) {
        if (prod.bias != nullptr) v += b;
        v = (__float_as_uint(v) - 1u) < 0x7f800000u ? v : 0.0f;
    }
    return v;
}

int check_shape(const cpoconv_shape *s);           // CPOCONV_OK or CPOCONV_ERR_SHAPE
int build_geometry(const cpoconv_shape *s, Geometry *g);
int64_t max_ptr_len(const Geometry &g);
int64_t scratch_bytes_for(const Geometry &g);

void set_hip_error(hipError_t e);

#define CPOCONV_HIP_TRY(expr)                         \
    do {                                              \
        hipError_t e__ = (expr);                      \
        if (e__ != hipSuccess) {                      \
            ::cpoconv::set_hip_error(e__);            \
            return CPOCONV_ERR_HIP;                   \
        }                                             \
    } while (0)

// Measurement aid: while kernel timing is enabled (cpoconv_kernel_timing), every kernel launch is
// bracketed by two HIP events on its own stream.
class KernelTimer {
public:
    KernelTimer(const char *name, hipStream_t stream);
    ~KernelTimer();
    KernelTimer(const KernelTimer &) = delete;
    KernelTimer &operator=(const KernelTimer &) = delete;

private:
    hipStream_t stream_;
    void *stop_;
};

// launchers (defined next to their kernels)
int launch_encode(const float *act, const Producer &prod, const Geometry &g, const cpoconv_map &map, int algo,
                  void *scratch, hipStream_t stream, bool write_table = false, bool write_indices = false);
bool encode_uses_channel_kernel(const Geometry &g); // the workgroup-per-channel encoder takes the layer
bool encode_writes_columns(const Geometry &g);      // with write_table: does the encoder also leave the column table?
int64_t encode_fixed_bytes();                        // look-back words every scratch buffer starts with
int64_t encode_call_flags_bytes(const Geometry &g);  // look-back words of a call that takes two launches
int launch_prepare_weights(const float *w, const Geometry &g, float *wt, hipStream_t stream);
int launch_zero_fill(void *buffer, int64_t bytes, hipStream_t stream);
int launch_sparse_conv(const cpoconv_map &map, const Geometry &g, int algo, const float *wt,
                       float *out, void *scratch, hipStream_t stream, bool table_ready = false,
                       bool indices_ready = false, bool columns_ready = false);
bool sparse_conv_uses_prologue(const Geometry &g);
int64_t lds_kernel_partial_bytes(const Geometry &g);   // general kernel (spmv_conv.hip)
// register-tile SpMV kernel (spmv_conv_tile.hip)
bool tile_kernel_supports(const Geometry &g);
int64_t tile_kernel_partial_bytes(const Geometry &g);
int launch_sparse_conv_tile(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g, const float *wt,
                            float *out, float *partial, BatchStrides bs, hipStream_t stream);
// strip SpMV kernel (spmv_conv_strip.hip)
bool strip_kernel_supports(const Geometry &g);
bool strip_kernel_preferred(const Geometry &g);
int64_t strip_kernel_partial_bytes(const Geometry &g);
int launch_sparse_conv_strip(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g,
                             const float *wt, float *out, float *partial, BatchStrides bs, hipStream_t stream);
// column-run SpMV kernel (spmv_conv_runs.hip)
bool runs_kernel_supports(const Geometry &g);
bool runs_kernel_preferred(const Geometry &g);
int64_t runs_kernel_partial_bytes(const Geometry &g);
int64_t runs_kernel_columns_bytes(const Geometry &g);
int launch_column_table(const cpoconv_map &map, const int32_t *mtab, ColumnEntry *columns, const Geometry &g, BatchStrides bs,
                        bool cps, hipStream_t stream);
int launch_sparse_conv_runs(const cpoconv_map &map, const ColumnEntry *columns, const Geometry &g, const float *wt, float *out,
                            float *partial, BatchStrides bs, hipStream_t stream);
// byte offsets of the regions of the caller's scratch buffer
int64_t scratch_counts_bytes(const Geometry &g);
int64_t scratch_indices_bytes(const Geometry &g);
int64_t scratch_mtab_bytes(const Geometry &g);
int64_t scratch_columns_offset(const Geometry &g);   // the column table comes last
// per-image strides inside those regions, in 4-byte elements
int64_t indices_stride(const Geometry &g);
int64_t mtab_stride(const Geometry &g);
int64_t columns_stride(const Geometry &g);           // in entries
// out[k][y][x] = sum over channel slices of partial[slice][y][x][k] (spmv_conv.hip)
int launch_reduce_transpose(const Geometry &g, const float *partial, int slices, int Ypad, int Xpad, float *out,
                            const BatchStrides &bs, hipStream_t stream);   // per image: partial advances by slices*Ypad*Xpad*Kpad, out by K*Oh*Ow

// Sum over the channel slices of one output element: four interleaved running sums, then
// pairwise.  Every kernel that adds slices uses this order, so they agree bit for bit.
__device__ inline float sum_slices(const float *src, int64_t slice_stride, int slices)
{
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    int sl = 0;
    for (; sl + 3 < slices; sl += 4) {
        s0 += src[sl * slice_stride];
        s1 += src[(sl + 1) * slice_stride];
        s2 += src[(sl + 2) * slice_stride];
        s3 += src[(sl + 3) * slice_stride];
    }
    for (; sl < slices; ++sl) s0 += src[sl * slice_stride];
    return (s0 + s1) + (s2 + s3);
}
int64_t im2col_scratch_bytes(const Geometry &g);
int64_t im2col_weights_bf16_len(const Geometry &g);
int launch_prepare_weights_bf16(const float *w, const Geometry &g, uint16_t *wb, hipStream_t stream);
int launch_im2col_conv(const float *act, const Producer &prod, const Geometry &g, const void *w, void *lowered,
                       float *out, int precision, hipStream_t stream);

}  // namespace cpoconv
