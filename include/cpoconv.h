/*
 * cpoconv — convolution of sparse post-ReLU activation maps with Compressed Pattern Overlap
 * (CPO) and Compressed Pattern Sets (CPS) on AMD MI355X (gfx950), after arXiv 2104.08314
 * ("High Performance Convolution Using Sparsity and Patterns for Inference in Deep CNNs").
 *
 * C ABI.  Conventions shared by every call unless a call says otherwise:
 *   - Tensors are DEVICE pointers owned by the caller; the library never allocates or frees
 *     device memory and never synchronises unless stated.  Work is queued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) of the current device.
 *   - Batch 1, fp32, one stride for both directions; pad_h zero rows above and below the map,
 *     pad_w zero columns left and right of it (Algorithm 1 takes the column padding as an input
 *     of its own; the 1 x n and n x 1 layers of the SI's layer tables pad one direction only).
 *     act is C x H x W row-major; weights are K x C x kh x kw row-major; out is K x Oh x Ow
 *     row-major with Oh = (H + 2 pad_h - kh) / stride + 1, Ow = (W + 2 pad_w - kw) / stride + 1
 *     (floor).
 *   - Every call returns CPOCONV_OK (0) or a negative CPOCONV_ERR_* code.  Arguments are
 *     validated on the host before anything is queued: a call that returns an error other
 *     than CPOCONV_ERR_HIP has launched nothing.
 *   - Limits: 1 <= kh, kw <= CPOCONV_MAX_K; H + 2 pad_h, W + 2 pad_w <= CPOCONV_MAX_I;
 *     C * H * W < 2^31.
 */
#ifndef CPOCONV_H
#define CPOCONV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CPOCONV_MAX_K 11
#define CPOCONV_MAX_I 256

/* Skip flags stored in ptr (Section 3.3 names them; the numeric values are this library's). */
#define CPOCONV_NPF (-2) /* No Ptr Flag: an overlap type of a live channel holds no NZE */
#define CPOCONV_NPC (-3) /* No Ptr Channel: the whole channel holds no NZE              */

#define CPOCONV_OK 0
#define CPOCONV_ERR_NULL (-1)        /* a required pointer is NULL                         */
#define CPOCONV_ERR_SHAPE (-2)       /* shape outside the limits above or inconsistent     */
#define CPOCONV_ERR_SMALL (-3)       /* a caller buffer is smaller than required           */
#define CPOCONV_ERR_HIP (-4)         /* a HIP call failed: see cpoconv_last_hip_error()    */
#define CPOCONV_ERR_ALGO (-5)        /* unknown algorithm / precision / mode value         */
#define CPOCONV_ERR_MAP (-6)         /* the map's encoder gave up (hdr[7] != 0): the map    */
                                     /* holds no valid streams                              */

#define CPOCONV_ALGO_IM2COL 0
#define CPOCONV_ALGO_CPO 1
#define CPOCONV_ALGO_CPS 2

typedef struct {
    int32_t C, H, W;     /* input channels, unpadded map height and width */
    int32_t K;           /* output kernels                                */
    int32_t kh, kw;      /* kernel height and width                       */
    int32_t stride;      /* both directions                               */
    int32_t pad_h, pad_w; /* zero rows above and below, zero columns left and right */
    int32_t layout;      /* of the input map `act` / `pre`: CPOCONV_LAYOUT_CHW (0) or _HWC (1)  */
} cpoconv_shape;

/*
 * Layout of the dense input map of a call (the "N x H x W x C" input of Table 1's I_n beside the
 * channel-first one): CHW = C x H x W (N x C x H x W for a batch), HWC = H x W x C (N x H x W x C).
 * Only the readers of `act` / `pre` look at it - the encoders and the im2col lowering; the encoded
 * streams, the weights and every output (K x Oh x Ow) are the same for both.  In a chain only the
 * first layer may be HWC: the others read what a convolution wrote.
 */
#define CPOCONV_LAYOUT_CHW 0
#define CPOCONV_LAYOUT_HWC 1

/*
 * An encoded activation map: the three streams of Section 3.3 in caller-allocated device
 * buffers, plus a small side band.
 *   ptr, da, in  ptr (int32), DA (fp32 NZE values), IN (int32 indices) as Algorithms 1 and 3
 *                define them, for channels in order; inside a channel for the overlap types
 *                present in the layer, ascending (NOP, overlap2, .., overlap-kw); inside a
 *                type for partitions, then columns, then rows ascending.
 *                ptr per channel: CPOCONV_NPC if the channel has no NZE, else per type
 *                CPOCONV_NPF if the type has no NZE, else [pType, e_0 .. e_{Ow-1}] with e_p
 *                the cumulative NZE count of the type after partition p or -1 if partition
 *                p shows no new column of the type; with pad_w = 0 and stride 1 the NOP type
 *                is [0, n_first_column, n_first_column + n_last_column] instead.
 *                IN: index = column inside the first partition holding the cell +
 *                padded row * kw.  CPS differs in the overlap-kw type only: per column and
 *                group of four padded rows, 3-4 NZEs -> {index of the first, 4-bit row
 *                pattern}, 2 -> both indices negated, 1 -> the index negated (Section 3.4).
 *   *_cap        capacities in elements; required: ptr_cap >= cpoconv_sizes().ptr_cap,
 *                da_cap and in_cap >= C*H*W.
 *   chan_off     3*(C+1) int32: offset of every channel in ptr, then in da, then in in, each
 *                list closed by the total.  Side band for parallel readers (Algorithm 2
 *                is written without the per-channel offsets into the streams).
 *   hdr          8 int32: |ptr|, |DA|, |IN|, algorithm (CPOCONV_ALGO_CPO / _CPS), C, Ow, the width
 *                of an IN entry in bits (32 or 16), and a failure flag (0, or 1 if the encoder
 *                gave up: see cpo_encode) - as cpoconv_map_header_to_host returns them.  In
 *                device memory the last two words are the library's: the width shares its word
 *                with a stamp of the encoding call, and the flag is raised by storing that stamp.
 *   in_bits      width of the IN entries: 0 or 32 for int32; 16 for a compact map whose `in`
 *                points at int16 entries (in_cap still counts entries).  Every IN entry is an
 *                index below (H + 2 pad_h) * kw <= 2816, the negative of one, or a row pattern
 *                below 16, so the narrow stream holds exactly the same values; the paper counts
 *                the size of the structure in elements (SI, space complexity), the narrow
 *                entries shrink it in bytes.  Encoders write, convolutions read, the width the
 *                map declares.  Any other value: CPOCONV_ERR_ALGO.
 */
typedef struct {
    int32_t *ptr;
    int64_t ptr_cap;
    float *da;
    int64_t da_cap;
    int32_t *in;
    int64_t in_cap;
    int32_t *chan_off;
    int32_t *hdr;
    int32_t in_bits;
} cpoconv_map;

/* Buffer sizes for one layer shape (elements unless named bytes). */
typedef struct {
    int64_t ptr_cap;       /* largest possible |ptr|                                      */
    int64_t da_cap;        /* C*H*W                                                        */
    int64_t in_cap;        /* C*H*W                                                        */
    int64_t chan_off_len;  /* 3*(C+1)                                                      */
    int64_t wt_len;        /* prepared weights: C*kh*kw*round_up(K,64) floats              */
    int64_t out_len;       /* K*Oh*Ow                                                      */
    int64_t lowered_bytes; /* im2col scratch: lowered matrix (rows padded to 4 columns),   */
                           /* split-K partial sums of the matrix product, the bf16 kernel  */
                           /* matrix of a precision-1 call                                 */
    int64_t scratch_bytes; /* scratch for encode and conv calls (prepare once with          */
                           /* cpoconv_scratch_init)                                         */
    int64_t wb_len;        /* bf16 kernel matrix of im2col_prepare_weights_bf16, in 16-bit  */
                           /* elements: ceil(C*kh*kw/8) * round_up(K,64) * 8                */
    int32_t Oh, Ow;
} cpoconv_sizes_t;

/* Host only.  Fills *sizes for the shape.  Errors: NULL, SHAPE. */
int cpoconv_sizes(const cpoconv_shape *shape, cpoconv_sizes_t *sizes);

/*
 * Prepares a scratch buffer (zero fill by a kernel queued on stream).  Required once after the buffer is
 * allocated and before its first use by any call below; after that the library keeps what it
 * needs in it consistent from call to call, provided nothing else writes to the buffer and the
 * calls that share it are ordered (one stream, or explicit dependencies).  The encoders keep an
 * epoch counter and the per-channel stream lengths of the running call there (Algorithm 1 appends
 * channel after channel: a channel's position is the sum of the lengths before it).
 * Errors: NULL, SHAPE (bytes < 0), HIP.
 */
int cpoconv_scratch_init(void *scratch, int64_t bytes, void *stream);

/*
 * CPO encoding of one activation map (Algorithm 1; partition / overlap-type geometry of
 * Sections 3.1-3.2).  Reads act, writes every stream of *map, chan_off and hdr.  scratch:
 * device memory of at least sizes.scratch_bytes bytes prepared by cpoconv_scratch_init; its
 * other contents are clobbered.  Streams, counts and indices are bit-exact functions of act and
 * shape.  With a scratch buffer that was never prepared (or was overwritten by something else)
 * the encoder gives up: every wait inside it is bounded, and a workgroup whose wait runs out, or
 * whose stream offsets would leave the map's capacities, writes no stream and sets hdr[7] to 1
 * (otherwise 0); cpoconv_map_header_to_host reports it, convolutions skip such a map.
 * Errors: NULL, SHAPE, SMALL (a capacity or scratch_bytes below the requirement), HIP.
 */
int cpo_encode(const float *act, const cpoconv_shape *shape, const cpoconv_map *map,
               void *scratch, int64_t scratch_bytes, void *stream);

/*
 * cpo_encode for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): the same encoding, bit for bit, with the encoder's
 * look-back words kept in a device array of the library instead of a caller's scratch buffer.  The
 * call allocates nothing and needs no cpoconv_scratch_init.  The array is CPOCONV_STATIC_SCRATCH_BYTES
 * (2 MiB) per GPU the library runs on, held until the process ends, shared by every call of this
 * entry point on that GPU and keeping state from call to call: calls that overlap on one GPU race -
 * order them (one stream, or explicit dependencies).  Layers whose look-back words do not fit the
 * array (more than 512 channels with so many that the two-launch encoder's words exceed it) are
 * refused with CPOCONV_ERR_SMALL.  Errors otherwise as cpo_encode; SHAPE also for a device ordinal
 * of 64 or more.
 */
#define CPOCONV_STATIC_SCRATCH_BYTES (2 << 20)
int cpo_encode_static_scratch(const float *act, const cpoconv_shape *shape, const cpoconv_map *map, void *stream);

/* CPS encoding (Algorithm 3): as cpo_encode, with the overlap-kw indices packed in set4
 * patterns. */
int cps_encode(const float *act, const cpoconv_shape *shape, const cpoconv_map *map,
               void *scratch, int64_t scratch_bytes, void *stream);

/*
 * Re-lays weights K x C x kh x kw as C x kh x kw x round_up(K,64) (kernel index fastest,
 * zero filled) for cpo_conv / cps_conv: Section 3.3 flattens each kernel row by row into a
 * vector; here that happens once per layer, for all kernels.  wt: sizes.wt_len floats.
 * Errors: NULL, SHAPE, HIP.
 */
int cpoconv_prepare_weights(const float *weights, const cpoconv_shape *shape, float *wt,
                            void *stream);

/*
 * Convolution as sparse matrix-vector products over a CPO map (Algorithm 2): every NZE
 * meets kh * (pType+1) kernel cells, for all K kernels.  map must come from cpo_encode with
 * the same shape and stream order must place that call before this one.  out is overwritten
 * (no accumulation into previous contents).  fp32 multiply-add, fp32 accumulation; the order
 * of additions is fixed, so results are bitwise repeatable.  scratch as in cpo_encode.
 * Errors: NULL, SHAPE, SMALL, HIP.
 */
int cpo_conv(const cpoconv_map *map, const cpoconv_shape *shape, const float *wt, float *out,
             void *scratch, int64_t scratch_bytes, void *stream);

/* Convolution over a CPS map (Algorithm 4): indices of the overlap-kw type are rebuilt
 * from singletons and {first index, pattern} pairs, then as cpo_conv. */
int cps_conv(const cpoconv_map *map, const cpoconv_shape *shape, const float *wt, float *out,
             void *scratch, int64_t scratch_bytes, void *stream);

/*
 * Encoding and convolution of one layer in one call: exactly cpo_encode (cps_encode) followed by
 * cpo_conv (cps_conv) on the same map, scratch buffer and stream - same streams, same output -
 * which is how a layer runs at inference time and what the per-layer selection of Section 3.5
 * times against im2col.  Knowing that the convolution follows, the encoder also leaves the
 * resolved partition offsets in the scratch buffer, so the convolution starts without a pass
 * over ptr of its own; for a CPS map it also leaves there the plain index of every NZE, 16 bits
 * each (what Algorithm 4 rebuilds from the packed IN stream), while map->in holds the packed stream
 * exactly as after cps_encode.  Arguments, layouts and errors as the separate calls.
 */
int cpo_encode_conv(const float *act, const cpoconv_shape *shape, const cpoconv_map *map, const float *wt,
                    float *out, void *scratch, int64_t scratch_bytes, void *stream);
int cps_encode_conv(const float *act, const cpoconv_shape *shape, const cpoconv_map *map, const float *wt,
                    float *out, void *scratch, int64_t scratch_bytes, void *stream);

/*
 * The comparator of Section 3.1: im2col lowering (lowered matrix C*kh*kw x Oh*Ow, row
 * (c*kh + l)*kw + w, column y*Ow + x, holds the padded input at (c, y*stride + l,
 * x*stride + w)) followed by a dense matrix product with the K x C*kh*kw kernel matrix on
 * the matrix cores.  precision 0: fp32 operands; 1: operands rounded to bf16 (nearest even),
 * fp32 accumulation; 2: as 1 with the kernel matrix already converted - weights then points to
 * the sizes.wb_len 16-bit elements im2col_prepare_weights_bf16 wrote (same result, bit for bit,
 * without the conversion launch of every precision-1 call).  lowered: scratch of
 * sizes.lowered_bytes bytes (lowered matrix, then the partial sums of the product when the
 * contraction is split over workgroups; slices are added in a fixed order).  weights for
 * precision 0 and 1: fp32 in the K x C x kh x kw layout.  lowered must be 16-byte aligned, and so
 * must precision-2 weights.
 * Errors: NULL, SHAPE (also a misaligned lowered), ALGO (precision), HIP.
 */
int im2col_conv(const float *act, const cpoconv_shape *shape, const void *weights,
                void *lowered, float *out, int precision, void *stream);

/*
 * The kernel matrix of Section 3.1's product (K x C*kh*kw, from weights K x C x kh x kw) rounded to
 * nearest-even bf16 and laid out as the matrix cores read it: groups of eight consecutive
 * contraction indices, [ceil(C*kh*kw/8)][round_up(K,64)][8], zero filled.  Done once per layer;
 * wb (device, 16-byte aligned, sizes.wb_len 16-bit elements) then serves every im2col_conv call
 * with precision 2.  Errors: NULL, SHAPE (also a misaligned wb), HIP.
 */
int im2col_prepare_weights_bf16(const float *weights, const cpoconv_shape *shape, void *wb, void *stream);

/*
 * Batched variants: n_images activation maps of one shape in one launch (the "I_n" of the
 * paper's Table 1; Section 3.3 encodes "one input image", so a batch is one independent encoding
 * per image).  Layouts: act is N x C x H x W, out is N x K x Oh x Ow.  *maps describes image 0;
 * image n uses the same struct with every buffer advanced by its per-image capacity:
 * ptr + n * ptr_cap, da + n * da_cap, in + n * in_cap, chan_off + n * 3*(C+1), hdr + n * 8
 * (so each buffer holds n_images consecutive regions and *_cap are per-image capacities with the
 * single-image minimum sizes).  Every image's streams, side band and header are exactly what
 * the single-image call produces for that image.  scratch / lowered: sizes from
 * cpoconv_batch_sizes.  Errors as the single-image calls, plus SHAPE for n_images < 1 or
 * n_images > CPOCONV_MAX_BATCH.
 */
#define CPOCONV_MAX_BATCH 1024

/* Host only.  As cpoconv_sizes for a batch: ptr_cap, da_cap, in_cap, chan_off_len and wt_len are
 * per image (unchanged); out_len, lowered_bytes and scratch_bytes cover the whole batch. */
int cpoconv_batch_sizes(const cpoconv_shape *shape, int n_images, cpoconv_sizes_t *sizes);

int cpo_encode_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                     void *scratch, int64_t scratch_bytes, void *stream);
int cps_encode_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                     void *scratch, int64_t scratch_bytes, void *stream);
int cpo_conv_batch(const cpoconv_map *maps, const cpoconv_shape *shape, int n_images, const float *wt,
                   float *out, void *scratch, int64_t scratch_bytes, void *stream);
int cps_conv_batch(const cpoconv_map *maps, const cpoconv_shape *shape, int n_images, const float *wt,
                   float *out, void *scratch, int64_t scratch_bytes, void *stream);
int im2col_conv_batch(const float *act, const cpoconv_shape *shape, int n_images, const void *weights,
                      void *lowered, float *out, int precision, void *stream);
int cpo_encode_conv_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                          const float *wt, float *out, void *scratch, int64_t scratch_bytes, void *stream);
int cps_encode_conv_batch(const float *act, const cpoconv_shape *shape, int n_images, const cpoconv_map *maps,
                          const float *wt, float *out, void *scratch, int64_t scratch_bytes, void *stream);

/*
 * A layer's input taken from the layer before it without storing the activated map.  The input I
 * of Eq. 1 is the output max(0, z) of a ReLU (Section 3.1); here `pre` holds z before the bias
 * (N x C x H x W, e.g. the `out` of the previous convolution) and every kernel that reads the
 * map applies, element by element, z = pre + bias[c] (one fp32 addition; none when bias is NULL)
 * and then takes z if z > 0, else +0 (negative values, both zeros and NaN give +0).  The streams
 * are bit for bit those of cpo_encode / cps_encode on that activated map, the convolution that of
 * im2col_conv on it.  bias: device, C floats, or NULL.  n_images, maps, scratch, lowered: as the
 * batched calls (n_images = 1 for one map).  Errors as the calls they extend.
 */
int cpo_encode_relu(const float *pre, const float *bias, const cpoconv_shape *shape, int n_images,
                    const cpoconv_map *maps, void *scratch, int64_t scratch_bytes, void *stream);
int cps_encode_relu(const float *pre, const float *bias, const cpoconv_shape *shape, int n_images,
                    const cpoconv_map *maps, void *scratch, int64_t scratch_bytes, void *stream);
int im2col_conv_relu(const float *pre, const float *bias, const cpoconv_shape *shape, int n_images,
                     const void *weights, void *lowered, float *out, int precision, void *stream);

/*
 * The conv layers of a network run one after the other, each with the method the offline
 * selection chose for it (Section 3.5: at inference time the selected method is used at the
 * layer).  Layer i reads layers[i-1].out (layer 0 reads `act`), which must have its input shape:
 * C = previous K, H x W = previous Oh x Ow.  With relu_in = 1 the input is max(0, that + bias_in)
 * applied on the way in, as in the *_relu calls (bias_in may be NULL); with relu_in = 0 it is
 * taken as stored and bias_in must be NULL.  method: CPOCONV_ALGO_CPO / _CPS (weights = the
 * prepared layout of cpoconv_prepare_weights; the layer runs as cpo_/cps_encode_conv_batch) or
 * CPOCONV_ALGO_IM2COL (precision 0 fp32 or 1 bf16: weights K x C x kh x kw; precision 2: the bf16
 * kernel matrix of im2col_prepare_weights_bf16, passed through the same pointer).  out: device,
 * n_images x K x Oh x Ow, written by the layer and read by the next one; it holds the sums before
 * any bias or ReLU.  One map, scratch and lowered buffer serve all layers in turn: sizes from
 * cpoconv_chain_sizes (the largest any layer needs; *maps is image 0's struct, capacities =
 * strides between images as in the batched calls); maps / scratch may be NULL if no layer uses
 * CPO or CPS, lowered if none uses im2col.  After the call the map holds the encoding of the last
 * CPO / CPS layer.  All arguments are checked before the first launch.
 * Errors: NULL, SHAPE (also layers that do not fit each other, n_layers outside 1..CPOCONV_MAX_CHAIN),
 * ALGO (method, precision, relu_in, bias without ReLU), SMALL, HIP.
 */
#define CPOCONV_MAX_CHAIN 1024
typedef struct {
    cpoconv_shape shape;
    int32_t method;
    int32_t precision;
    int32_t relu_in;
    const float *bias_in;
    const float *weights;
    float *out;
} cpoconv_chain_layer;

/* Host only.  ptr_cap .. chan_off_len, wt_len, out_len, lowered_bytes, scratch_bytes: the largest
 * over the layers (per image where cpoconv_batch_sizes is per image); Oh, Ow: of the last layer.
 * Pointer members of the layers are not read. */
int cpoconv_chain_sizes(const cpoconv_chain_layer *layers, int n_layers, int n_images, cpoconv_sizes_t *sizes);
int cpoconv_chain_forward(const float *act, const cpoconv_chain_layer *layers, int n_layers, int n_images,
                          const cpoconv_map *maps, void *scratch, int64_t scratch_bytes, void *lowered,
                          int64_t lowered_bytes, void *stream);

/*
 * Offline per-layer selection (Section 3.5).  Host only.  t_*: times of the three methods on
 * the same m_inputs offline inputs, any common unit.  mode 0 "favour time": the smaller total
 * of im2col and CPO; mode 1 "favour space": the smaller total of im2col and CPS; im2col keeps
 * a tie.  *algo_out receives CPOCONV_ALGO_*.  The array of the method not compared may be NULL.
 * Errors: NULL, SHAPE (m_inputs < 1), ALGO (mode).
 */
int select_layer_algo(const double *t_im2col, const double *t_cpo, const double *t_cps,
                      int m_inputs, int mode, int *algo_out);

/* Copies map->hdr to the host and waits for the stream: the only synchronising call.  hdr_host is
 * filled in any case; the call returns CPOCONV_ERR_MAP if the header says that the encoder gave up
 * (hdr[7] != 0, see cpo_encode): such a map holds no valid streams, and every convolution call
 * given it (or given a map that holds the other algorithm's streams, hdr[3]) leaves `out`
 * untouched - the kernels read the header themselves, so this also holds for the calls that encode
 * and convolve in one go, which cannot report it.
 * Errors: NULL, HIP, MAP. */
int cpoconv_map_header_to_host(const cpoconv_map *map, int32_t hdr_host[8], void *stream);

/* Host only: partition / overlap-type table of a layer, as the encoders use it.
 * info: 8 int32 = Ih, Iw, Oh, Ow, number of encoded columns, number of present types,
 * nop3 (NOP uses the three-entry segment), top (the type CPS packs, or -1).
 * col_j / col_type / col_p0 / col_what: CPOCONV_MAX_I int32 each, one entry per encoded
 * column in stream order: padded column, overlap type (0 = NOP), first partition holding the
 * column, column inside that partition.  Errors: NULL, SHAPE. */
int cpoconv_geometry(const cpoconv_shape *shape, int32_t info[8], int32_t *col_j,
                     int32_t *col_type, int32_t *col_p0, int32_t *col_what);

/*
 * Measurement aid (not part of the method).  cpoconv_kernel_timing(1) clears earlier records
 * and makes every later kernel launch of the library bracket itself with two HIP events on the
 * stream it runs on; cpoconv_kernel_timing(0) stops that.  cpoconv_kernel_timing_read returns
 * record `index` (0, 1, .. until it returns CPOCONV_ERR_SHAPE): kernel name (NUL-terminated,
 * at most name_cap bytes), average duration in microseconds and number of launches; it waits
 * for the recorded launches to finish.  Host-side events only: no device memory is allocated.
 * Errors: NULL, SHAPE (index out of range), HIP.
 */
int cpoconv_kernel_timing(int enable);
int cpoconv_kernel_timing_read(int index, char *name_out, int name_cap, double *avg_us, int *calls);

/* Text for an error code (static storage). */
const char *cpoconv_strerror(int code);

/* hipError_t value of the last failed HIP call made by this library in this thread (0 if none). */
int cpoconv_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CPOCONV_H */
