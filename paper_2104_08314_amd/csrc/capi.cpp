// C ABI of libcpoconv: argument validation, layer geometry, host-only calls.  Every device
// step is queued by the launch_* functions next to the kernels.
#include <string.h>

#include <algorithm>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "common.hpp"

namespace cpoconv {

static thread_local int g_last_hip_error = 0;

void set_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }

namespace {
struct TimingRecord {
    std::string name;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
};
std::mutex g_timing_mutex;
bool g_timing_enabled = false;
std::vector<TimingRecord> g_timing;

void timing_clear()
{
    for (auto &rec : g_timing)
        for (auto &ev : rec.events) {
            hipEventDestroy(ev.first);
            hipEventDestroy(ev.second);
        }
    g_timing.clear();
}
}  // namespace

KernelTimer::KernelTimer(const char *name, hipStream_t stream) : stream_(stream), stop_(nullptr)
{
    if (!g_timing_enabled) return;
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    hipEvent_t start, stop;
    if (hipEventCreate(&start) != hipSuccess) return;
    if (hipEventCreate(&stop) != hipSuccess) { hipEventDestroy(start); return; }
    TimingRecord *rec = nullptr;
    for (auto &r : g_timing)
        if (r.name == name) rec = &r;
    if (!rec) {
        g_timing.push_back(TimingRecord{name, {}});
        rec = &g_timing.back();
    }
    rec->events.emplace_back(start, stop);
    hipEventRecord(start, stream_);
    stop_ = stop;
}

KernelTimer::~KernelTimer()
{
    if (stop_) hipEventRecord(static_cast<hipEvent_t>(stop_), stream_);
}

int check_shape(const cpoconv_shape *s)
{
    if (s->C < 1 || s->H < 1 || s->W < 1 || s->K < 1) return CPOCONV_ERR_SHAPE;
    if (s->kh < 1 || s->kw < 1 || s->kh > CPOCONV_MAX_K || s->kw > CPOCONV_MAX_K)
        return CPOCONV_ERR_SHAPE;
    if (s->stride < 1 || s->pad_h < 0 || s->pad_h > CPOCONV_MAX_I || s->pad_w < 0 || s->pad_w > CPOCONV_MAX_I)
        return CPOCONV_ERR_SHAPE;
    if (s->H > CPOCONV_MAX_I || s->W > CPOCONV_MAX_I) return CPOCONV_ERR_SHAPE;
    if (s->layout != CPOCONV_LAYOUT_CHW && s->layout != CPOCONV_LAYOUT_HWC) return CPOCONV_ERR_SHAPE;
    const int Ih = s->H + 2 * s->pad_h, Iw = s->W + 2 * s->pad_w;
    if (Ih > CPOCONV_MAX_I || Iw > CPOCONV_MAX_I) return CPOCONV_ERR_SHAPE;
    if (Ih < s->kh || Iw < s->kw) return CPOCONV_ERR_SHAPE;
    if (static_cast<int64_t>(s->C) * s->H * s->W >= (int64_t{1} << 31)) return CPOCONV_ERR_SHAPE;
    if (static_cast<int64_t>(s->K) * s->C * s->kh * s->kw >= (int64_t{1} << 31))
        return CPOCONV_ERR_SHAPE;
    return CPOCONV_OK;
}

// A padded column j lies in partitions p with p*stride <= j <= p*stride + kw - 1, 0 <= p < Ow
// (Section 3.1: Ow partitions of width kw separated by the stride).  Its overlap type is the
// number of such partitions minus one; the first of them indexes the column (Section 3.2).
int build_geometry(const cpoconv_shape *s, Geometry *g)
{
    const int rc = check_shape(s);
    if (rc != CPOCONV_OK) return rc;
    memset(g, 0, sizeof(*g));
    g->C = s->C; g->H = s->H; g->W = s->W; g->K = s->K;
    g->channel_last = s->layout == CPOCONV_LAYOUT_HWC ? 1 : 0;
    g->kh = s->kh; g->kw = s->kw; g->stride = s->stride; g->pad_h = s->pad_h; g->pad_w = s->pad_w;
    g->Ih = s->H + 2 * s->pad_h;
    g->Iw = s->W + 2 * s->pad_w;
    g->Oh = (g->Ih - s->kh) / s->stride + 1;
    g->Ow = (g->Iw - s->kw) / s->stride + 1;
    g->Kpad = (s->K + 63) / 64 * 64;
    g->N = 1;

    int type_of[kMaxCols], p0_of[kMaxCols];
    int count[kMaxTypes] = {0};
    for (int j = 0; j < g->Iw; ++j) {
        type_of[j] = -1;
        const int lo_num = j - s->kw + 1;
        const int p_lo = lo_num <= 0 ? 0 : (lo_num + s->stride - 1) / s->stride;
        int p_hi = j / s->stride;
        if (p_hi > g->Ow - 1) p_hi = g->Ow - 1;
        const int m = p_hi - p_lo + 1;
        const bool real = j >= s->pad_w && j < s->pad_w + s->W;
        if (m < 1 || !real) continue;
        type_of[j] = m - 1;
        p0_of[j] = p_lo;
        ++count[m - 1];
    }
    int n = 0;
    for (int t = 0; t < s->kw; ++t) {
        if (count[t] == 0) continue;
        g->type_id[g->n_types] = static_cast<uint8_t>(t);
        g->type_begin[g->n_types] = static_cast<uint16_t>(n);
        for (int j = 0; j < g->Iw; ++j) {
            if (type_of[j] != t) continue;
            g->col_j[n] = static_cast<uint8_t>(j);
            g->col_p0[n] = static_cast<uint8_t>(p0_of[j]);
            g->col_what[n] = static_cast<uint8_t>(j - p0_of[j] * s->stride);
            ++n;
        }
        ++g->n_types;
    }
    g->type_begin[g->n_types] = static_cast<uint16_t>(n);
    g->n_cols = n;
    g->nop3 = (s->stride == 1 && s->pad_w == 0 && s->kw >= 2 && g->Ow >= 2) ? 1 : 0;
    g->top = -1;
    g->top_slot = -1;
    const int top = (s->kw + s->stride - 1) / s->stride - 1;
    if (top >= 1) {
        for (int i = 0; i < g->n_types; ++i)
            if (g->type_id[i] == top) { g->top = top; g->top_slot = i; }
    }
    return CPOCONV_OK;
}

int64_t max_ptr_len(const Geometry &g)
{
    int64_t per_channel = 0;
    for (int i = 0; i < g.n_types; ++i)
        per_channel += (g.nop3 && g.type_id[i] == 0) ? 3 : 1 + g.Ow;
    if (per_channel < 1) per_channel = 1;
    return per_channel * g.C;
}

// Scratch layout: the encoder's look-back words (epochs, per-band stream lengths) | the convolution's
// table of resolved ptr offsets | one int16 per NZE for the indices cps_conv rebuilds | partial
// sums of the convolution | the column table of the column-run convolution.
// (each region holds g.N images back to back, with the per-image strides below)
int64_t indices_stride(const Geometry &g) { return static_cast<int64_t>(g.C) * g.H * g.W; }                 // entries
int64_t mtab_stride(const Geometry &g) { return static_cast<int64_t>(g.C) * std::max(g.n_types, 1) * (g.Ow + 1); }   // ints
int64_t columns_stride(const Geometry &g) { return static_cast<int64_t>(g.C) * g.Iw; }                       // entries

// encoder look-back words: the fixed region every scratch buffer starts with (its place and size do
// not depend on the call, so calls of any shape and batch size may share a buffer), then the words
// of a call that takes two launches
int64_t scratch_counts_bytes(const Geometry &g) { return encode_fixed_bytes() + encode_call_flags_bytes(g); }
int64_t scratch_indices_bytes(const Geometry &g) { return (2 * indices_stride(g) * g.N + 255) / 256 * 256; }   // int16 each
int64_t scratch_mtab_bytes(const Geometry &g) { return (4 * mtab_stride(g) * g.N + 255) / 256 * 256; }

int64_t scratch_columns_offset(const Geometry &g)
{
    const int64_t partial = std::max(std::max(tile_kernel_partial_bytes(g), strip_kernel_partial_bytes(g)),
                                     std::max(runs_kernel_partial_bytes(g), lds_kernel_partial_bytes(g)));
    return scratch_counts_bytes(g) + scratch_mtab_bytes(g) + scratch_indices_bytes(g) + (partial + 255) / 256 * 256;
}

int64_t scratch_bytes_for(const Geometry &g) { return scratch_columns_offset(g) + runs_kernel_columns_bytes(g); }

}  // namespace cpoconv

using namespace cpoconv;

extern "C" {

static const Producer kAsStored = {nullptr, 0};

static int batch_geometry(const cpoconv_shape *shape, int n_images, Geometry *g)
{
    const int rc = build_geometry(shape, g);
    if (rc != CPOCONV_OK) return rc;
    if (n_images < 1 || n_images > CPOCONV_MAX_BATCH) return CPOCONV_ERR_SHAPE;
    g->N = n_images;
    return CPOCONV_OK;
}

int cpoconv_sizes(const cpoconv_shape *shape, cpoconv_sizes_t *sizes)
{
    return cpoconv_batch_sizes(shape, 1, sizes);
}

int cpoconv_batch_sizes(const cpoconv_shape *shape, int n_images, cpoconv_sizes_t *sizes)
{
    if (!shape || !sizes) return CPOCONV_ERR_NULL;
    Geometry g;
    const int rc = batch_geometry(shape, n_images, &g);
    if (rc != CPOCONV_OK) return rc;
    const int64_t chw = static_cast<int64_t>(g.C) * g.H * g.W;
    sizes->ptr_cap = max_ptr_len(g);
    sizes->da_cap = chw;
    sizes->in_cap = chw;
    sizes->chan_off_len = 3 * static_cast<int64_t>(g.C + 1);
    sizes->wt_len = static_cast<int64_t>(g.C) * g.kh * g.kw * g.Kpad;
    sizes->out_len = static_cast<int64_t>(g.N) * g.K * g.Oh * g.Ow;
    sizes->lowered_bytes = im2col_scratch_bytes(g);
    sizes->scratch_bytes = scratch_bytes_for(g);
    sizes->wb_len = im2col_weights_bf16_len(g);
    sizes->Oh = g.Oh;
    sizes->Ow = g.Ow;
    return CPOCONV_OK;
}

static int encode_common(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *map,
                         void *scratch, int64_t scratch_bytes, void *stream, int algo, const Producer &prod = kAsStored)
{
    if (!act || !shape || !map || !scratch) return CPOCONV_ERR_NULL;
    if (!map->ptr || !map->da || !map->in || !map->chan_off || !map->hdr) return CPOCONV_ERR_NULL;
    if (map->in_bits != 0 && map->in_bits != 16 && map->in_bits != 32) return CPOCONV_ERR_ALGO;
    Geometry g;
    const int rc = batch_geometry(shape, n_images, &g);
    if (rc != CPOCONV_OK) return rc;
    const int64_t chw = static_cast<int64_t>(g.C) * g.H * g.W;
    if (map->ptr_cap < max_ptr_len(g) || map->da_cap < chw || map->in_cap < chw)
        return CPOCONV_ERR_SMALL;
    if (scratch_bytes < scratch_bytes_for(g)) return CPOCONV_ERR_SMALL;
    return launch_encode(act, prod, g, *map, algo, scratch, static_cast<hipStream_t>(stream));
}

// ---- an encoder entry point that takes no scratch buffer from the caller ---------------------------
// The encoder's look-back words live in a file-scope device array (zero at load time, which is the
// state cpoconv_scratch_init leaves).  Host code never uses the array's name as an address: the
// device address is asked for once per device and kept.
namespace {
constexpr int64_t kStaticScratchBytes = int64_t{2} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_static_scratch[kMaxDevices] = {nullptr};
std::mutex g_static_scratch_mutex;

int static_scratch_of_current_device(void **ptr)
{
    int dev = -1;
    CPOCONV_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CPOCONV_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (g_static_scratch[dev] == nullptr) {
        void *p = nullptr;
        CPOCONV_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));   // this device's copy of the array
        g_static_scratch[dev] = p;
    }
    *ptr = g_static_scratch[dev];
    return CPOCONV_OK;
}
}  // namespace

int cpo_encode_static_scratch(const float *act, const cpoconv_shape *shape, const cpoconv_map *map, void *stream)
{
    if (!act || !shape || !map) return CPOCONV_ERR_NULL;
    if (!map->ptr || !map->da || !map->in || !map->chan_off || !map->hdr) return CPOCONV_ERR_NULL;
    if (map->in_bits != 0 && map->in_bits != 16 && map->in_bits != 32) return CPOCONV_ERR_ALGO;
    Geometry g;
    const int rc = build_geometry(shape, &g);
    if (rc != CPOCONV_OK) return rc;
    const int64_t chw = static_cast<int64_t>(g.C) * g.H * g.W;
    if (map->ptr_cap < max_ptr_len(g) || map->da_cap < chw || map->in_cap < chw) return CPOCONV_ERR_SMALL;
    // the encoder's part of a scratch buffer is all this call needs; layers whose look-back words
    // do not fit the array (very many channels: the two-launch encoder's own words) are refused
    if (scratch_counts_bytes(g) > kStaticScratchBytes) return CPOCONV_ERR_SMALL;
    void *buffer = nullptr;
    const int src = static_scratch_of_current_device(&buffer);
    if (src != CPOCONV_OK) return src;
    return launch_encode(act, kAsStored, g, *map, CPOCONV_ALGO_CPO, buffer, static_cast<hipStream_t>(stream));
}

int cpoconv_scratch_init(void *scratch, int64_t bytes, void *stream)
{
    if (!scratch) return CPOCONV_ERR_NULL;
    if (bytes < 0) return CPOCONV_ERR_SHAPE;
    return launch_zero_fill(scratch, bytes, static_cast<hipStream_t>(stream));
}

int cpo_encode(const float *act, const cpoconv_shape *shape, const cpoconv_map *map,
               void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_common(act, shape, 1, map, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPO);
}

int cps_encode(const float *act, const cpoconv_shape *shape, const cpoconv_map *map,
               void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_common(act, shape, 1, map, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPS);
}

int cpoconv_prepare_weights(const float *weights, const cpoconv_shape *shape, float *wt,
                            void *stream)
{
    if (!weights || !shape || !wt) return CPOCONV_ERR_NULL;
    Geometry g;
    const int rc = build_geometry(shape, &g);
    if (rc != CPOCONV_OK) return rc;
    return launch_prepare_weights(weights, g, wt, static_cast<hipStream_t>(stream));
}

static int conv_common(const cpoconv_map *map, const cpoconv_shape *shape, int n_images, const float *wt,
                       float *out, void *scratch, int64_t scratch_bytes, void *stream, int algo)
{
    if (!map || !shape || !wt || !out || !scratch) return CPOCONV_ERR_NULL;
    if (!map->ptr || !map->da || !map->in || !map->chan_off || !map->hdr) return CPOCONV_ERR_NULL;
    if (map->in_bits != 0 && map->in_bits != 16 && map->in_bits != 32) return CPOCONV_ERR_ALGO;
    Geometry g;
    const int rc = batch_geometry(shape, n_images, &g);
    if (rc != CPOCONV_OK) return rc;
    const int64_t chw = static_cast<int64_t>(g.C) * g.H * g.W;
    if (g.N > 1 && (map->ptr_cap < max_ptr_len(g) || map->da_cap < chw || map->in_cap < chw))
        return CPOCONV_ERR_SMALL;   // the capacities are the strides between images
    if (scratch_bytes < scratch_bytes_for(g)) return CPOCONV_ERR_SMALL;
    return launch_sparse_conv(*map, g, algo, wt, out, scratch, static_cast<hipStream_t>(stream));
}

int cpo_conv(const cpoconv_map *map, const cpoconv_shape *shape, const float *wt, float *out,
             void *scratch, int64_t scratch_bytes, void *stream)
{
    return conv_common(map, shape, 1, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPO);
}

int cps_conv(const cpoconv_map *map, const cpoconv_shape *shape, const float *wt, float *out,
             void *scratch, int64_t scratch_bytes, void *stream)
{
    return conv_common(map, shape, 1, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPS);
}

static int encode_conv_common(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *map,
                              const float *wt, float *out, void *scratch, int64_t scratch_bytes, void *stream, int algo,
                              const Producer &prod = kAsStored)
{
    if (!act || !shape || !map || !wt || !out || !scratch) return CPOCONV_ERR_NULL;
    if (!map->ptr || !map->da || !map->in || !map->chan_off || !map->hdr) return CPOCONV_ERR_NULL;
    if (map->in_bits != 0 && map->in_bits != 16 && map->in_bits != 32) return CPOCONV_ERR_ALGO;
    Geometry g;
    const int rc = batch_geometry(shape, n_images, &g);
    if (rc != CPOCONV_OK) return rc;
    const int64_t chw = static_cast<int64_t>(g.C) * g.H * g.W;
    if (map->ptr_cap < max_ptr_len(g) || map->da_cap < chw || map->in_cap < chw) return CPOCONV_ERR_SMALL;
    if (scratch_bytes < scratch_bytes_for(g)) return CPOCONV_ERR_SMALL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the encoder also leaves the table of resolved ptr offsets: the convolution needs no prologue
    // of its own; for a CPS map it also leaves there the plain index of every NZE (16 bits each: what
    // Algorithm 4 rebuilds from the packed IN stream, which the map itself holds as after cps_encode)
    // (not where the column-run convolution follows: the column table is all it reads, and where the
    // encoder does not leave it, it is rebuilt from the packed stream itself)
    const bool table = sparse_conv_uses_prologue(g);
    const bool columns = table && encode_writes_columns(g);
    const bool indices = algo == CPOCONV_ALGO_CPS && g.top_slot >= 0 && !runs_kernel_preferred(g);
    const int erc = launch_encode(act, prod, g, *map, algo, scratch, st, table, indices);
    if (erc != CPOCONV_OK) return erc;
    return launch_sparse_conv(*map, g, algo, wt, out, scratch, st, table, indices, columns);
}

int cpo_encode_conv(const float *act, const cpoconv_shape *shape, const cpoconv_map *map, const float *wt,
                    float *out, void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_conv_common(act, shape, 1, map, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPO);
}

int cps_encode_conv(const float *act, const cpoconv_shape *shape, const cpoconv_map *map, const float *wt,
                    float *out, void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_conv_common(act, shape, 1, map, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPS);
}

int cpo_encode_conv_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                          const float *wt, float *out, void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_conv_common(act, shape, n_images, maps, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPO);
}

int cps_encode_conv_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                          const float *wt, float *out, void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_conv_common(act, shape, n_images, maps, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPS);
}

int cpo_encode_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                     void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_common(act, shape, n_images, maps, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPO);
}

int cps_encode_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                     void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_common(act, shape, n_images, maps, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPS);
}

int cpo_conv_batch(const cpoconv_map *maps, const cpoconv_shape *shape, int n_images, const float *wt,
                   float *out, void *scratch, int64_t scratch_bytes, void *stream)
{
    return conv_common(maps, shape, n_images, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPO);
}

int cps_conv_batch(const cpoconv_map *maps, const cpoconv_shape *shape, int n_images, const float *wt,
                   float *out, void *scratch, int64_t scratch_bytes, void *stream)
{
    return conv_common(maps, shape, n_images, wt, out, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPS);
}

int im2col_conv(const float *act, const cpoconv_shape *shape, const void *weights, void *lowered,
                float *out, int precision, void *stream)
{
    return im2col_conv_batch(act, shape, 1, weights, lowered, out, precision, stream);
}

int im2col_prepare_weights_bf16(const float *weights, const cpoconv_shape *shape, void *wb, void *stream)
{
    if (!weights || !shape || !wb) return CPOCONV_ERR_NULL;
    Geometry g;
    const int rc = batch_geometry(shape, 1, &g);
    if (rc != CPOCONV_OK) return rc;
    if (reinterpret_cast<uintptr_t>(wb) % 16 != 0) return CPOCONV_ERR_SHAPE;
    return launch_prepare_weights_bf16(weights, g, static_cast<uint16_t *>(wb), static_cast<hipStream_t>(stream));
}

static int im2col_common(const float *act, const cpoconv_shape *shape, int n_images, const void *weights,
                         void *lowered, float *out, int precision, void *stream, const Producer &prod)
{
    if (!act || !shape || !weights || !lowered || !out) return CPOCONV_ERR_NULL;
    Geometry g;
    const int rc = batch_geometry(shape, n_images, &g);
    if (rc != CPOCONV_OK) return rc;
    if (precision < 0 || precision > 2) return CPOCONV_ERR_ALGO;
    if (reinterpret_cast<uintptr_t>(lowered) % 16 != 0) return CPOCONV_ERR_SHAPE;   // vector accesses
    if (precision == 2 && reinterpret_cast<uintptr_t>(weights) % 16 != 0) return CPOCONV_ERR_SHAPE;
    return launch_im2col_conv(act, prod, g, weights, lowered, out, precision,
                              static_cast<hipStream_t>(stream));
}

int im2col_conv_batch(const float *act, const cpoconv_shape *shape, int n_images, const void *weights,
                      void *lowered, float *out, int precision, void *stream)
{
    return im2col_common(act, shape, n_images, weights, lowered, out, precision, stream, kAsStored);
}

// ---- a layer's input produced on the way in: bias and ReLU of the layer before it ----------------
int cpo_encode_relu(const float *pre, const float *bias, const cpoconv_shape *shape, int n_images,
                    const cpoconv_map *maps, void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_common(pre, shape, n_images, maps, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPO, Producer{bias, 1});
}

int cps_encode_relu(const float *pre, const float *bias, const cpoconv_shape *shape, int n_images,
                    const cpoconv_map *maps, void *scratch, int64_t scratch_bytes, void *stream)
{
    return encode_common(pre, shape, n_images, maps, scratch, scratch_bytes, stream, CPOCONV_ALGO_CPS, Producer{bias, 1});
}

int im2col_conv_relu(const float *pre, const float *bias, const cpoconv_shape *shape, int n_images,
                     const void *weights, void *lowered, float *out, int precision, void *stream)
{
    return im2col_common(pre, shape, n_images, weights, lowered, out, precision, stream, Producer{bias, 1});
}

// ---- chained layers -------------------------------------------------------------------------------
static int chain_check(const cpoconv_chain_layer *layers, int n_layers, int n_images)
{
    if (!layers) return CPOCONV_ERR_NULL;
    if (n_layers < 1 || n_layers > CPOCONV_MAX_CHAIN) return CPOCONV_ERR_SHAPE;
    Geometry g, prev;
    for (int i = 0; i < n_layers; ++i) {
        const cpoconv_chain_layer &l = layers[i];
        const int rc = batch_geometry(&l.shape, n_images, &g);
        if (rc != CPOCONV_OK) return rc;
        if (l.method != CPOCONV_ALGO_IM2COL && l.method != CPOCONV_ALGO_CPO && l.method != CPOCONV_ALGO_CPS)
            return CPOCONV_ERR_ALGO;
        if (l.method == CPOCONV_ALGO_IM2COL && (l.precision < 0 || l.precision > 2)) return CPOCONV_ERR_ALGO;
        if (l.relu_in != 0 && l.relu_in != 1) return CPOCONV_ERR_ALGO;
        if (!l.relu_in && l.bias_in) return CPOCONV_ERR_ALGO;      // a bias is only applied in front of the ReLU
        // a layer reads what the layer before it wrote: K x Oh x Ow, channel-first
        if (i > 0 && (g.C != prev.K || g.H != prev.Oh || g.W != prev.Ow || g.channel_last)) return CPOCONV_ERR_SHAPE;
        prev = g;
    }
    return CPOCONV_OK;
}

int cpoconv_chain_sizes(const cpoconv_chain_layer *layers, int n_layers, int n_images, cpoconv_sizes_t *sizes)
{
    if (!sizes) return CPOCONV_ERR_NULL;
    const int rc = chain_check(layers, n_layers, n_images);
    if (rc != CPOCONV_OK) return rc;
    memset(sizes, 0, sizeof(*sizes));
    for (int i = 0; i < n_layers; ++i) {
        cpoconv_sizes_t one;
        const int src = cpoconv_batch_sizes(&layers[i].shape, n_images, &one);
        if (src != CPOCONV_OK) return src;
        sizes->ptr_cap = std::max(sizes->ptr_cap, one.ptr_cap);
        sizes->da_cap = std::max(sizes->da_cap, one.da_cap);
        sizes->in_cap = std::max(sizes->in_cap, one.in_cap);
        sizes->chan_off_len = std::max(sizes->chan_off_len, one.chan_off_len);
        sizes->wt_len = std::max(sizes->wt_len, one.wt_len);
        sizes->out_len = std::max(sizes->out_len, one.out_len);
        sizes->lowered_bytes = std::max(sizes->lowered_bytes, one.lowered_bytes);
        sizes->scratch_bytes = std::max(sizes->scratch_bytes, one.scratch_bytes);
        sizes->wb_len = std::max(sizes->wb_len, one.wb_len);
        sizes->Oh = one.Oh;
        sizes->Ow = one.Ow;
    }
    return CPOCONV_OK;
}

int cpoconv_chain_forward(const float *act, const cpoconv_chain_layer *layers, int n_layers, int n_images,
                          const cpoconv_map *maps, void *scratch, int64_t scratch_bytes, void *lowered,
                          int64_t lowered_bytes, void *stream)
{
    if (!act) return CPOCONV_ERR_NULL;
    const int rc = chain_check(layers, n_layers, n_images);
    if (rc != CPOCONV_OK) return rc;
    // every buffer is checked before the first launch, so a chain runs whole or not at all
    for (int i = 0; i < n_layers; ++i) {
        const cpoconv_chain_layer &l = layers[i];
        if (!l.weights || !l.out) return CPOCONV_ERR_NULL;
        cpoconv_sizes_t one;
        const int src = cpoconv_batch_sizes(&l.shape, n_images, &one);
        if (src != CPOCONV_OK) return src;
        if (l.method == CPOCONV_ALGO_IM2COL) {
            if (!lowered) return CPOCONV_ERR_NULL;
            if (lowered_bytes < one.lowered_bytes) return CPOCONV_ERR_SMALL;
            if (reinterpret_cast<uintptr_t>(lowered) % 16 != 0) return CPOCONV_ERR_SHAPE;
        } else {
            if (!maps || !scratch) return CPOCONV_ERR_NULL;
            if (!maps->ptr || !maps->da || !maps->in || !maps->chan_off || !maps->hdr) return CPOCONV_ERR_NULL;
            if (maps->in_bits != 0 && maps->in_bits != 16 && maps->in_bits != 32) return CPOCONV_ERR_ALGO;
            if (maps->ptr_cap < one.ptr_cap || maps->da_cap < one.da_cap || maps->in_cap < one.in_cap) return CPOCONV_ERR_SMALL;
            if (scratch_bytes < one.scratch_bytes) return CPOCONV_ERR_SMALL;
        }
    }
    const float *x = act;
    for (int i = 0; i < n_layers; ++i) {
        const cpoconv_chain_layer &l = layers[i];
        const Producer prod{l.relu_in ? l.bias_in : nullptr, l.relu_in};
        int lrc;
        if (l.method == CPOCONV_ALGO_IM2COL)
            lrc = im2col_common(x, &l.shape, n_images, l.weights, lowered, l.out, l.precision, stream, prod);
        else
            lrc = encode_conv_common(x, &l.shape, n_images, maps, l.weights, l.out, scratch, scratch_bytes, stream,
                                     l.method, prod);
        if (lrc != CPOCONV_OK) return lrc;
        x = l.out;
    }
    return CPOCONV_OK;
}

int select_layer_algo(const double *t_im2col, const double *t_cpo, const double *t_cps,
                      int m_inputs, int mode, int *algo_out)
{
    if (!algo_out || !t_im2col) return CPOCONV_ERR_NULL;
    if (mode != 0 && mode != 1) return CPOCONV_ERR_ALGO;
    const double *t_sparse = mode == 0 ? t_cpo : t_cps;
    if (!t_sparse) return CPOCONV_ERR_NULL;
    if (m_inputs < 1) return CPOCONV_ERR_SHAPE;
    double total_dense = 0.0, total_sparse = 0.0;
    for (int i = 0; i < m_inputs; ++i) {
        total_dense += t_im2col[i];
        total_sparse += t_sparse[i];
    }
    if (total_sparse < total_dense)
        *algo_out = mode == 0 ? CPOCONV_ALGO_CPO : CPOCONV_ALGO_CPS;
    else
        *algo_out = CPOCONV_ALGO_IM2COL;
    return CPOCONV_OK;
}

int cpoconv_map_header_to_host(const cpoconv_map *map, int32_t hdr_host[8], void *stream)
{
    if (!map || !map->hdr || !hdr_host) return CPOCONV_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    CPOCONV_HIP_TRY(hipMemcpyAsync(hdr_host, map->hdr, 8 * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    CPOCONV_HIP_TRY(hipStreamSynchronize(st));
    // on the device hdr[6] also carries the stamp of the call that wrote the header and hdr[7] the stamp
    // of the call in which an encoder unit gave up: the caller gets the width and a plain 0 / 1
    const int32_t stamp = hdr_host[6] >> 8, failed_in = hdr_host[7];
    hdr_host[6] &= 0xFF;
    hdr_host[7] = (failed_in != 0 && failed_in == stamp) ? 1 : 0;
    return hdr_host[7] != 0 ? CPOCONV_ERR_MAP : CPOCONV_OK;
}

int cpoconv_geometry(const cpoconv_shape *shape, int32_t info[8], int32_t *col_j,
                     int32_t *col_type, int32_t *col_p0, int32_t *col_what)
{
    if (!shape || !info || !col_j || !col_type || !col_p0 || !col_what) return CPOCONV_ERR_NULL;
    Geometry g;
    const int rc = build_geometry(shape, &g);
    if (rc != CPOCONV_OK) return rc;
    info[0] = g.Ih; info[1] = g.Iw; info[2] = g.Oh; info[3] = g.Ow;
    info[4] = g.n_cols; info[5] = g.n_types; info[6] = g.nop3; info[7] = g.top;
    for (int i = 0; i < g.n_types; ++i)
        for (int n = g.type_begin[i]; n < g.type_begin[i + 1]; ++n) {
            col_j[n] = g.col_j[n];
            col_type[n] = g.type_id[i];
            col_p0[n] = g.col_p0[n];
            col_what[n] = g.col_what[n];
        }
    return CPOCONV_OK;
}

int cpoconv_kernel_timing(int enable)
{
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    if (enable) timing_clear();
    g_timing_enabled = enable != 0;
    return CPOCONV_OK;
}

int cpoconv_kernel_timing_read(int index, char *name_out, int name_cap, double *avg_us, int *calls)
{
    if (!name_out || !avg_us || !calls) return CPOCONV_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    if (index < 0 || index >= static_cast<int>(g_timing.size()) || name_cap < 1) return CPOCONV_ERR_SHAPE;
    const TimingRecord &rec = g_timing[index];
    double total_ms = 0.0;
    for (const auto &ev : rec.events) {
        CPOCONV_HIP_TRY(hipEventSynchronize(ev.second));
        float ms = 0.0f;
        CPOCONV_HIP_TRY(hipEventElapsedTime(&ms, ev.first, ev.second));
        total_ms += ms;
    }
    strncpy(name_out, rec.name.c_str(), static_cast<size_t>(name_cap) - 1);
    name_out[name_cap - 1] = '\0';
    *calls = static_cast<int>(rec.events.size());
    *avg_us = rec.events.empty() ? 0.0 : total_ms * 1000.0 / rec.events.size();
    return CPOCONV_OK;
}

const char *cpoconv_strerror(int code)
{
    switch (code) {
    case CPOCONV_OK: return "ok";
    case CPOCONV_ERR_NULL: return "a required pointer is NULL";
    case CPOCONV_ERR_SHAPE: return "shape outside the supported limits or inconsistent";
    case CPOCONV_ERR_SMALL: return "a caller buffer is smaller than required";
    case CPOCONV_ERR_HIP: return "a HIP call failed (see cpoconv_last_hip_error)";
    case CPOCONV_ERR_ALGO: return "unknown algorithm, precision or mode value";
    case CPOCONV_ERR_MAP: return "the map's encoder gave up (scratch buffer not prepared, or overwritten): no valid streams";
    default: return "unknown error code";
    }
}

int cpoconv_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
