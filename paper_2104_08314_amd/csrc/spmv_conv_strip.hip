// Strip SpMV convolution over a CPO map (Algorithm 2) for the common kernel shapes.
//
// CPO streams are column-major: inside a channel and overlap type the NZEs follow the
// partitions (columns) and, inside a column, the rows.  ptr therefore delimits exactly the NZEs
// of a strip of output columns, for all rows at once.  A workgroup owns such a strip (XT*TX
// output columns, all or up to 16/XT * TY output rows) for 64*KPL output kernels (KPL per lane)
// and one slice of the input channels; its wavefronts are TY x TX tiles of the strip: row bands, XT tiles side by side.
// Wide strips (XT > 1) are for small maps: the whole map is then decoded once per workgroup and
// the staged weights serve up to sixteen wavefronts.  Maps so small that a strip has fewer than
// eight tiles share a workgroup between several images of the launch: each image has its own
// table and patches, the staged weights serve all of them.
//
// Per group of G channels
//   decode   the wavefronts share the NZE chunks (64 NZEs each) of the group's channels: load
//            value and index, find the partition from the position in DA (ptr used as CSR row
//            pointers), split the index into padded row and column inside the partition, and
//            drop the value at its cell of the channel's LDS patch of the padded input;
//   apply    every wavefront reads the cells behind its TY x TX tile one per lane, takes a ballot
//            of the non-zero ones and walks them in a fully unrolled loop: a clear bit costs a
//            scalar bit test and an untaken branch, a set bit broadcasts the value from its lane
//            (lanes are output kernels, so the NZE is a scalar operand) and issues the
//            kh*(pType+1) FMAs of convSpMv that land in the tile, KPL times, with compile-time
//            registers for sums and weights.
// No two wavefronts add to the same output, so there is no reduction inside the workgroup.  The
// tile's sums go to partial[slice][y][x][k] (k fastest: coalesced); a second kernel adds the
// channel slices in a fixed order and transposes to K x Oh x Ow (one slice: written directly).

#include <algorithm>

#include "common.hpp"
#include "resolve_ptr.hpp"

namespace cpoconv {

namespace {

constexpr int kMaxBands = 16;        // wavefronts (row bands) per workgroup
constexpr int kStripTabBytes = 6 * 1024;
constexpr int kMaxSlices = 32;
constexpr size_t kLdsBytes = 160 * 1024;   // LDS of a compute unit

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

struct StripArgs {
    const float *da;
    const int32_t *in;        // one index per NZE, laid out like DA
    const int32_t *mtab;      // [C][n_types][Ow+1] absolute DA offsets (prologue kernel), or null:
    const int32_t *ptr;       //   then the kernel resolves ptr itself, with the
    const int32_t *chan_off;  //   channel offsets of the map's side band
    const float *wt;          // [C][kh*kw][Kpad]
    float *partial;           // [slices][Ypad][Xpad][Kpad]
    float *out;               // K x Oh x Ow
    int32_t slices;           // channel slices across workgroups
    BatchStrides bs;          // image n of the launch: every buffer advanced n strides
    int32_t Ypad, Xpad;
    int32_t bands;            // row bands per workgroup (wavefronts: bands * XT * imgs)
    int32_t imgs;             // images sharing a workgroup
    int32_t n_images;         // images of the launch
    int32_t batch;            // channels per table refill (multiple of G)
    int32_t chunks;           // upper bound of 64-NZE chunks of one channel's strip
    int32_t chunks_magic;     // ceil(2^16 / chunks): item / chunks == (item * magic) >> 16 for item < 1024
};

template <int KH, int KW, int S, int TY, int TX, int G, int KPL, int XT>
__global__ __launch_bounds__(kMaxBands *kLanes) void spmv_conv_strip_kernel(const Geometry g, const StripArgs a_launch)
{
    constexpr int RH = (TY - 1) * S + KH;      // rows of the padded input behind one tile
    constexpr int RWT = (TX - 1) * S + KW;     // columns behind one tile
    constexpr int RW = (XT * TX - 1) * S + KW; // columns behind the strip
    constexpr int NCELL = RH * RWT;
    constexpr int NDREG = (NCELL + kLanes - 1) / kLanes;
    constexpr int TAPS = KH * KW;
    constexpr int SPAN = XT * TX + KW + 1;     // table slots per (channel, type): partitions p_lo-1 ..
    constexpr int IT = 4;                      // decode items whose loads are in flight together

    const int ngroups = g.Kpad / (kLanes * KPL);   // a wavefront holds KPL kernels per lane
    const int tid = threadIdx.x, lane = lane_id();
    const int wave_wg = uni(tid / kLanes);           // in a scalar register: everything derived from it stays scalar
    const int nwaves = a_launch.bands * XT;          // wavefronts of one image
    const int img_l = wave_wg / nwaves;              // which of the workgroup's images this wavefront works on
    const int wave = wave_wg - img_l * nwaves;       // wavefront inside the image
    const int image_raw = (blockIdx.z / (ngroups * a_launch.slices)) * a_launch.imgs + img_l;
    // past the launch's last image, or an image whose map must not be read: only barriers and shared staging
    const bool live = image_raw < a_launch.n_images && !map_unusable(a_launch.bs, image_raw);
    const int image = live ? image_raw : 0;
    StripArgs a = a_launch;
    a.da += image * a.bs.da;
    a.in = index_advance(a.in, image * a.bs.indices, a.bs.indices16);
    if (a.mtab != nullptr) a.mtab += image * a.bs.mtab;
    a.ptr += image * a.bs.ptr;
    a.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    a.partial += image * a.bs.partial;
    a.out += image * a.bs.out;

    extern __shared__ int32_t smem[];
    // layout: tab[imgs][batch][n_types][SPAN] | stage[imgs][wavefronts][kStageInts] | wl[G][TAPS][KPL*64] |
    //         patch[imgs][G][RW][PH]
    const int PH = (a.bands * TY - 1) * S + KH;             // patch height: rows behind the workgroup
    int32_t *tab = smem + img_l * (a.batch * g.n_types * SPAN);
    int32_t *stage = smem + a.imgs * (a.batch * g.n_types * SPAN) + img_l * (nwaves * kStageInts);
    float *wl = reinterpret_cast<float *>(smem + a.imgs * (a.batch * g.n_types * SPAN + nwaves * kStageInts));
    float *patch_all = wl + G * TAPS * KPL * kLanes;
    float *patch = patch_all + img_l * (G * RW * PH);

    const int nthreads = nwaves * kLanes;                   // threads of one image
    const int tid_img = wave * kLanes + lane;
    const int nwaves_wg = nwaves * a.imgs;
    const int xt = XT == 1 ? 0 : wave / a.bands, band = wave - xt * a.bands;   // this wavefront's tile of the strip
    const int x0 = blockIdx.x * (TX * XT);                  // first output column of the strip
    const int xw0 = x0 + xt * TX;                           // first output column of this wavefront
    const int yb = blockIdx.y * a.bands * TY;               // first output row of the workgroup
    const int y0 = yb + band * TY;                          // first output row of this wavefront
    const int kg = blockIdx.z % ngroups, slice = (blockIdx.z / ngroups) % a.slices;
    const int kbase = kg * kLanes * KPL;
    const int per_slice = (g.C + a.slices - 1) / a.slices;
    const int c_begin = slice * per_slice, c_end = min(g.C, c_begin + per_slice);

    float acc[TY][TX][KPL];
#pragma unroll
    for (int y = 0; y < TY; ++y)
#pragma unroll
        for (int x = 0; x < TX; ++x)
#pragma unroll
            for (int kk = 0; kk < KPL; ++kk) acc[y][x][kk] = 0.0f;

    // one NZE -> its cell of the patch.  n is its position in DA; the partition is the number of
    // table boundaries at or below n.
    auto scatter = [&](int idx, float v, int n, const int (&bound)[SPAN], int p_lo, float *pt) {
        int prel = 0;
#pragma unroll
        for (int e = 1; e < SPAN; ++e) prel += (n >= bound[e]) ? 1 : 0;
        const int h = idx / KW, wh = idx - h * KW;   // padded row, column inside the partition
        const int r = h - yb * S;
        const int q = (p_lo + prel - x0) * S + wh;
        if (idx >= 0 && r >= 0 && r < PH && q >= 0 && q < RW) pt[q * PH + r] = v;
    };

    const int main_slot = g.n_types - 1;   // the highest overlap type holds most NZEs
    for (int cb = c_begin; cb < c_end; cb += a.batch) {
        const int nb = min(a.batch, c_end - cb);
        __syncthreads();   // previous batch's table no longer in use
        // table: DA offset after partition p for the partitions that reach the strip; slot e of
        // (channel, type) holds partition p_lo - 1 + e (clamped: later slots repeat the end)
        if (!live) {
            // nothing to resolve
        } else if (a.mtab != nullptr) {
            for (int idx = tid_img; idx < nb * g.n_types * SPAN; idx += nthreads) {
                const int e = idx % SPAN;
                const int i = (idx / SPAN) % g.n_types;
                const int c = cb + idx / (SPAN * g.n_types);
                const int p = min(max(0, x0 - static_cast<int>(g.type_id[i])) - 1 + e, g.Ow - 1);
                tab[idx] = a.mtab[(static_cast<int64_t>(c) * g.n_types + i) * (g.Ow + 1) + p + 1];
            }
        } else {
            resolve_ptr_rows<SPAN>(g, a.ptr, a.chan_off, cb, nb, x0, tab, stage, wave, nwaves, lane);
        }

        for (int g0 = 0; g0 < nb; g0 += G) {
            const int ng = min(G, nb - g0);
            // ---- clear the patches of the group (all readers of the previous group are done) ----
            __syncthreads();
            for (int i = tid_img; i < ng * RW * PH; i += nthreads) patch[i] = 0.0f;
            // weights of the group's channels for this workgroup's 64 kernels (coalesced rows of 64)
            for (int row = wave_wg; row < ng * TAPS; row += nwaves_wg)
#pragma unroll
                for (int kk = 0; kk < KPL; ++kk)
                    wl[(row * KPL + kk) * kLanes + lane] =
                        a.wt[(static_cast<int64_t>(cb + g0) * TAPS + row) * g.Kpad + kbase + kk * kLanes + lane];
            __syncthreads();

            // ---- decode: work item = (channel of the group, 64-NZE chunk of its main-type range);
            // the loads of IT items are issued before any of them is used ------------------------
            const int nitems = live ? ng * a.chunks : 0;
            for (int it0 = wave; it0 < nitems; it0 += nwaves * IT) {
                int idxv[IT], nv[IT];
                float valv[IT];
                const int t_main = g.type_id[main_slot];
                const int plo_main = max(0, x0 - t_main), phi = min(g.Ow - 1, x0 + XT * TX - 1);
#pragma unroll
                for (int u = 0; u < IT; ++u) {
                    const int item = it0 + u * nwaves;
                    idxv[u] = -1; valv[u] = 0.0f; nv[u] = 0;
                    if (item < nitems) {
                        const int gi = (item * a.chunks_magic) >> 16, ch = item - gi * a.chunks;
                        const int32_t *row = tab + ((g0 + gi) * g.n_types + main_slot) * SPAN;
                        const int first = uni(row[0]), last = uni(row[phi - plo_main + 1]);
                        const int n = first + ch * kLanes + lane;
                        nv[u] = n;
                        if (n < last) { idxv[u] = load_index(a.in, n, a.bs.indices16); valv[u] = a.da[n]; }
                    }
                }
#pragma unroll
                for (int u = 0; u < IT; ++u) {
                    const int item = it0 + u * nwaves;
                    if (item >= nitems) continue;
                    const int gi = (item * a.chunks_magic) >> 16, ch = item - gi * a.chunks;
                    float *pt = patch + gi * RW * PH;
                    const int32_t *rows = tab + ((g0 + gi) * g.n_types) * SPAN;
                    int bound[SPAN];
#pragma unroll
                    for (int e = 0; e < SPAN; ++e) bound[e] = uni(rows[main_slot * SPAN + e]);
                    // chunks past the strip's last NZE of the channel hold nothing
                    const int last_main = uni(rows[main_slot * SPAN + phi - plo_main + 1]);
                    if (bound[0] + ch * kLanes < last_main) scatter(idxv[u], valv[u], nv[u], bound, plo_main, pt);
                    if (ch != 0) continue;
                    // the lower overlap types (edge columns): few NZEs, loaded on demand
                    for (int i = 0; i < main_slot; ++i) {
                        const int t = g.type_id[i];
                        const int p_lo = max(0, x0 - t);
                        const int f = uni(rows[i * SPAN]), l = uni(rows[i * SPAN + phi - p_lo + 1]);
                        if (l == f) continue;
#pragma unroll
                        for (int e = 0; e < SPAN; ++e) bound[e] = uni(rows[i * SPAN + e]);
                        for (int n0 = f; n0 < l; n0 += kLanes) {
                            const int n = n0 + lane;
                            const bool ok = n < l;
                            scatter(ok ? load_index(a.in, n, a.bs.indices16) : -1, ok ? a.da[n] : 0.0f, n, bound, p_lo, pt);
                        }
                    }
                }
            }
            __syncthreads();

            // ---- apply: every wavefront walks the cells behind its own tile --------------------
            if (live && y0 < g.Oh && xw0 < g.Ow) {
#pragma unroll 1
                for (int gi = 0; gi < ng; ++gi) {
                    const float *pt = patch + gi * RW * PH + xt * (TX * S) * PH + band * TY * S;   // first cell behind the tile
                    float cell[NDREG];
                    unsigned long long bits[NDREG];
                    bool any = false;
#pragma unroll
                    for (int d = 0; d < NDREG; ++d) {
                        const int i = d * kLanes + lane;
                        const int q = i / RH, r = i - q * RH;
                        cell[d] = i < NCELL ? pt[q * PH + r] : 0.0f;
                        bits[d] = __ballot((__float_as_uint(cell[d]) & 0x7fffffffu) != 0u);
                        any = any || bits[d] != 0ull;
                    }
                    if (!any) continue;
                    float w[TAPS][KPL];
#pragma unroll
                    for (int tp = 0; tp < TAPS; ++tp)
#pragma unroll
                        for (int kk = 0; kk < KPL; ++kk) w[tp][kk] = wl[((gi * TAPS + tp) * KPL + kk) * kLanes + lane];
#pragma unroll
                    for (int q = 0; q < RWT; ++q) {
#pragma unroll
                        for (int r = 0; r < RH; ++r) {
                            const int cellno = q * RH + r;
                            // (tested on 32-bit halves: a single scalar bit-compare per cell)
                            const unsigned half = (cellno % kLanes) < 32 ? static_cast<unsigned>(bits[cellno / kLanes])
                                                                          : static_cast<unsigned>(bits[cellno / kLanes] >> 32);
                            if ((half >> (cellno % 32)) & 1u) {
                                const float v = __int_as_float(
                                    __builtin_amdgcn_readlane(__float_as_int(cell[cellno / kLanes]), cellno % kLanes));
#pragma unroll
                                for (int l = 0; l < KH; ++l) {
                                    if ((r - l) < 0 || (r - l) % S != 0 || (r - l) / S >= TY) continue;
#pragma unroll
                                    for (int ww = 0; ww < KW; ++ww) {
                                        if ((q - ww) < 0 || (q - ww) % S != 0 || (q - ww) / S >= TX) continue;
#pragma unroll
                                        for (int kk = 0; kk < KPL; ++kk)
                                            acc[(r - l) / S][(q - ww) / S][kk] =
                                                fmaf(v, w[l * KW + ww][kk], acc[(r - l) / S][(q - ww) / S][kk]);
                                    }
                                }
                            }
                        }
                    }
                }
            }
        }
    }

    if (!live) return;
    if (a.slices == 1) {
#pragma unroll
        for (int kk = 0; kk < KPL; ++kk) {
            const int k = kbase + kk * kLanes + lane;
            if (k < g.K)
#pragma unroll
                for (int y = 0; y < TY; ++y)
#pragma unroll
                    for (int x = 0; x < TX; ++x)
                        if (y0 + y < g.Oh && xw0 + x < g.Ow)
                            a.out[(static_cast<int64_t>(k) * g.Oh + y0 + y) * g.Ow + xw0 + x] = acc[y][x][kk];
        }
        return;
    }
    // partial sums of this channel slice, kernel index fastest
    if (y0 < g.Oh && xw0 < g.Ow) {
        float *dst = a.partial + ((static_cast<int64_t>(slice) * a.Ypad + y0) * a.Xpad + xw0) * g.Kpad + kbase + lane;
#pragma unroll
        for (int y = 0; y < TY; ++y)
#pragma unroll
            for (int x = 0; x < TX; ++x)
#pragma unroll
                for (int kk = 0; kk < KPL; ++kk)
                    dst[(static_cast<int64_t>(y) * a.Xpad + x) * g.Kpad + kk * kLanes] = acc[y][x][kk];
    }
}

struct StripPlan {
    int bands, row_blocks, slices, batch, chunks, Ypad, imgs;
    size_t lds;
};

template <int KH, int KW, int S, int TY, int TX, int G, int KPL, int XT>
StripPlan strip_plan(const Geometry &g)
{
    constexpr int RW = (XT * TX - 1) * S + KW, SPAN = XT * TX + KW + 1;
    constexpr int kBandsMax = kMaxBands / XT;
    StripPlan p;
    const int bands_all = (g.Oh + TY - 1) / TY;
    p.row_blocks = (bands_all + kBandsMax - 1) / kBandsMax;
    p.bands = (bands_all + p.row_blocks - 1) / p.row_blocks;
    const int PH = (p.bands * TY - 1) * S + KH;
    p.Ypad = p.row_blocks * p.bands * TY;
    p.chunks = (RW * g.Ih + kLanes - 1) / kLanes;   // a strip's partitions hold at most RW columns of Ih rows
    // images per workgroup: fill the sixteen wavefronts when a strip of the map has few tiles
    p.imgs = 1;
    if (XT > 1 && p.bands * XT * 2 <= kMaxBands) p.imgs = std::min(kMaxBands / (p.bands * XT), g.N);
    int batch = kStripTabBytes / (g.n_types * SPAN * 4);
    batch = batch / G * G;
    if (batch < G) batch = G;
    if (batch > 64) batch = 64;
    p.batch = batch;
    auto lds_bytes = [&](int imgs) {
        return (imgs * (static_cast<size_t>(batch) * g.n_types * SPAN + static_cast<size_t>(p.bands) * XT * kStageInts +
                        static_cast<size_t>(G) * RW * PH) +
                static_cast<size_t>(G) * KH * KW * KPL * kLanes) * 4;
    };
    while (p.imgs > 1 && lds_bytes(p.imgs) > kLdsBytes) --p.imgs;   // everything has to fit the compute unit's LDS
    const int wgs = ((g.Ow + TX * XT - 1) / (TX * XT)) * p.row_blocks * (g.Kpad / (kLanes * KPL)) * ((g.N + p.imgs - 1) / p.imgs);
    // channel slices: one workgroup of fourteen wavefronts or more per compute unit, or as many
    // smaller ones as give fourteen wavefronts (measured best), each slice keeping four channels or more
    const int nw = p.bands * XT * p.imgs;
    int s = (256 * std::max(14, nw)) / (wgs * nw);
    const int cap = (g.C + 3) / 4;
    if (s > cap) s = cap;
    if (s > kMaxSlices) s = kMaxSlices;
    if (s < 1) s = 1;
    // no empty slices: with ceil(C / s) channels each, fewer slices may already cover the layer
    const int per_slice = (g.C + s - 1) / s;
    p.slices = (g.C + per_slice - 1) / per_slice;
    p.lds = lds_bytes(p.imgs);
    return p;
}

template <int KH, int KW, int S, int TY, int TX, int G, int KPL, int XT>
int launch_strip(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g,
                 const float *wt, float *out, float *partial, BatchStrides bs, hipStream_t stream)
{
    const StripPlan p = strip_plan<KH, KW, S, TY, TX, G, KPL, XT>(g);
    const int ntx = (g.Ow + TX * XT - 1) / (TX * XT);
    StripArgs a;
    a.da = map.da; a.in = indices; a.mtab = mtab; a.ptr = map.ptr; a.chan_off = map.chan_off; a.wt = wt;
    a.partial = partial; a.out = out;
    a.slices = p.slices; a.Ypad = p.row_blocks * p.bands * TY; a.Xpad = ntx * TX * XT;
    a.bands = p.bands; a.batch = p.batch; a.chunks = p.chunks; a.imgs = p.imgs; a.n_images = g.N;
    a.chunks_magic = (65536 + p.chunks - 1) / p.chunks;
    bs.partial = static_cast<int64_t>(p.slices) * a.Ypad * a.Xpad * g.Kpad;
    a.bs = bs;
    if (p.lds > kLdsBytes) return CPOCONV_ERR_SHAPE;   // no launch shape of the dispatch asks for more than a compute unit has
    {
        KernelTimer timer("spmv_conv_strip", stream);
        hipLaunchKernelGGL((spmv_conv_strip_kernel<KH, KW, S, TY, TX, G, KPL, XT>),
                           dim3(ntx, p.row_blocks, (g.Kpad / (kLanes * KPL)) * p.slices * ((g.N + p.imgs - 1) / p.imgs)),
                           dim3(p.bands * XT * p.imgs * kLanes), p.lds, stream,
                           g, a);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    if (p.slices > 1) return launch_reduce_transpose(g, partial, p.slices, a.Ypad, a.Xpad, out, bs, stream);
    return CPOCONV_OK;
}

}  // namespace

// Images per launch from which the batched launch shapes below are taken.
constexpr int kBatchedFromImages = 4;

// 1 x n and n x 1 kernels at stride 1 (n = 3, 7): the layers of that kind in the SI's layer tables.
inline bool line_kernel(const Geometry &g)
{
    return g.stride == 1 && ((g.kh == 1 && (g.kw == 3 || g.kw == 7)) || (g.kw == 1 && (g.kh == 3 || g.kh == 7)));
}

// Column tiles per workgroup.  With several images per launch there are workgroups enough, and the
// small 3 x 3 maps gain from wide strips: 14 x 14 outputs are one strip of four tiles by four bands
// (every NZE decoded once per workgroup, weights staged once for sixteen wavefronts), 28 x 28
// outputs strips of two tiles by seven bands.
int strip_xt(const Geometry &g)
{
    if (g.N < kBatchedFromImages || g.C < 32) return 1;
    const int bands_all = (g.Oh + 3) / 4;
    if (line_kernel(g)) {
        // 1 x 7 and 7 x 1 layers (17 x 17 maps in the SI's tables): one strip of three six-column
        // tiles covers up to 18 columns; 1 x 3 and 3 x 1 layers (8 x 8 maps): two four-column tiles
        if (g.kh == 7 || g.kw == 7) return (g.Ow > 12 && g.Ow <= 18 && bands_all * 3 <= kMaxBands) ? 3 : 1;
        if (g.Ow <= 4 || g.Ow > 8 || bands_all * 2 > kMaxBands) return 1;
        return (bands_all * 2 < 8 && g.N < 8) ? 1 : 2;
    }
    if (g.kh != 3 || g.kw != 3) return 1;
    int xt = 1;
    if (bands_all * 4 <= kMaxBands && g.Ow > 8) xt = 4;
    else if (bands_all * 2 <= kMaxBands && g.Ow > 4) xt = 2;
    // a strip of fewer than eight tiles shares its workgroup between images: that pays from
    // eight images on (measured: 512 x 7 x 7 at 4 images 11.0 against 9.7 us per image, at 8 images 6.1 against 8.1)
    if (bands_all * xt < 8 && g.N < 8) return 1;
    return xt;
}

// Tiles of eight columns (measured with 32 images per launch): on 56 x 56 stride-1 maps the wider
// tile visits fewer halo cells per output (15.7 -> 13.8 us per image at 128 channels).
inline int strip_wide_xt(const Geometry &g)   // 0: four-column tiles, else the strip's number of eight-column tiles
{
    if (g.N < kBatchedFromImages || g.kh != 3 || g.kw != 3) return 0;
    if (g.stride == 1 && g.Oh * g.Ow >= 2048) return 1;
    return 0;
}

// Four kernels per lane (256 per wavefront): a visited cell then feeds four times the FMAs of its
// scalar work, and half as many workgroups decode the same NZEs.  It needs 256 kernels or a
// multiple, several images per launch and at least eight workgroups before any channel slicing
// (measured per image, 2 -> 4 kernels per lane: 32 images, 256 x 14 x 14 3.6 -> 3.0 us, 512 x 7 x 7
// 4.0 -> 3.1, 128 x 56 x 56 stride 2 with 256 kernels 12.3 -> 8.8; with fewer than eight workgroups
// it loses, e.g. 256 x 14 x 14 at four images 8.7 -> 10.3).
inline bool strip_four_kernels_per_lane(const Geometry &g)
{
    if (g.Kpad % 256 != 0 || g.N < kBatchedFromImages || g.kh != 3 || g.kw != 3 || strip_wide_xt(g) != 0) return false;
    const int xt = strip_xt(g), bands_all = (g.Oh + 3) / 4;
    const int row_blocks = (bands_all + kMaxBands / xt - 1) / (kMaxBands / xt);
    const int bands = (bands_all + row_blocks - 1) / row_blocks;
    int imgs = 1;
    if (xt > 1 && bands * xt * 2 <= kMaxBands) imgs = std::min(kMaxBands / (bands * xt), static_cast<int>(g.N));
    const int wgs = ((g.Ow + 4 * xt - 1) / (4 * xt)) * row_blocks * (g.Kpad / 256) * ((g.N + imgs - 1) / imgs);
    return wgs >= 8;
}

bool strip_kernel_supports(const Geometry &g)
{
    if (g.n_types < 1) return false;
    if (line_kernel(g)) return strip_xt(g) > 1;   // only in their batched launch shapes
    return (g.kh == 3 && g.kw == 3 && (g.stride == 1 || g.stride == 2)) ||
           (g.kh == 5 && g.kw == 5 && g.stride == 1) || (g.kh == 7 && g.kw == 7 && g.stride == 2);
}

// Measured on MI355X over the workload layers: the strip kernel wins where one channel slice
// would leave the register-tile kernel few workgroups with long serial channel loops or where
// its shared patch saves decoding: layers of few channels, 5 x 5 kernels, and wide 3 x 3 maps
// (stride 1 from 2048 outputs, or 784 when images are batched; stride 2 from 784 outputs with 128
// kernels or more).  Elsewhere the register-tile kernel is as fast or faster.
bool strip_kernel_preferred(const Geometry &g)
{
    if (!strip_kernel_supports(g)) return false;
    if (strip_xt(g) > 1 || strip_wide_xt(g) > 0) return true;   // several images: wide strips or wide tiles
    if (g.C <= 16 || g.kh == 5) return true;
    if (g.stride == 2) return g.Oh * g.Ow >= 784 && g.Kpad >= 128;   // 3 x 3 stride 2 from a 56 x 56 map: 46 -> 34 us
    // stride 1: from 56 x 56 maps on; with several images per launch already from 28 x 28
    return g.stride == 1 && g.Oh * g.Ow >= (g.N >= 4 ? 784 : 2048);
}

// 3 x 3 layers whose padded kernel count is a multiple of 128 keep two kernels per lane: the
// scalar work of a visited cell (bit test, broadcast) then feeds twice the FMAs
// (seven columns where they divide the map's width: 56-wide maps, 13.9 -> 12.7 us per image at 128
// channels and 32 images, 6.0 -> 5.6 at 64 channels)
// Groups of sixteen channels in these wide-tile variants: half the barriers per channel
// (12.7 -> 12.2 and 5.6 -> 5.3; in the strips of several tiles larger groups gain nothing, and with
// four kernels per lane they cost images per workgroup: 3.1 -> 5.9 on 7 x 7 maps)
#define CPOCONV_STRIP_TX7(CALL)                                                      \
    if (g.kh == 3 && g.kw == 3 && g.stride == 1 && strip_wide_xt(g) == 1 && g.Ow % 7 == 0) { \
        if (g.Kpad % 128 == 0) return CALL(3, 3, 1, 4, 7, 16, 2, 1);                  \
        return CALL(3, 3, 1, 4, 7, 16, 1, 1);                                         \
    }
#define CPOCONV_STRIP_WIDE(CALL, S, XTW)                                             \
    CPOCONV_STRIP_TX7(CALL)                                                          \
    if (g.kh == 3 && g.kw == 3 && g.stride == S && strip_wide_xt(g) == XTW) {        \
        if (g.Kpad % 128 == 0) return CALL(3, 3, S, 4, 8, 16, 2, XTW);                \
        return CALL(3, 3, S, 4, 8, 16, 1, XTW);                                       \
    }
// (28-wide outputs without four kernels per lane: two seven-column tiles per strip divide the map
// exactly: 128 x 28 x 28 4.6 -> 4.1 us per image at 32 images)
#define CPOCONV_TX7X2_CASES(CALL, S)                                                 \
        if (xt == 2 && g.Ow % 14 == 0 && !strip_four_kernels_per_lane(g)) {          \
            if (g.Kpad % 128 == 0) return CALL(3, 3, S, 4, 7, 8, 2, 2);              \
            return CALL(3, 3, S, 4, 7, 8, 1, 2);                                     \
        }
#define CPOCONV_STRIP_3X3(CALL, S)                                                   \
    if (g.kh == 3 && g.kw == 3 && g.stride == S) {                                   \
        const int xt = strip_xt(g);                                                  \
        CPOCONV_TX7X2_CASES(CALL, S)                                                 \
        if (strip_four_kernels_per_lane(g)) {                                        \
            if (xt == 4) return CALL(3, 3, S, 4, 4, 8, 4, 4);                        \
            if (xt == 2) return CALL(3, 3, S, 4, 4, 8, 4, 2);                        \
            return CALL(3, 3, S, 4, 4, 8, 4, 1);                                     \
        }                                                                            \
        if (g.Kpad % 192 == 0 && g.N >= kBatchedFromImages) {                        \
            if (xt == 4) return CALL(3, 3, S, 4, 4, 8, 3, 4);                        \
            if (xt == 2) return CALL(3, 3, S, 4, 4, 8, 3, 2);                        \
            return CALL(3, 3, S, 4, 4, 8, 3, 1);                                     \
        }                                                                            \
        if (g.Kpad % 128 == 0) {                                                     \
            if (xt == 4) return CALL(3, 3, S, 4, 4, 8, 2, 4);                        \
            if (xt == 2) return CALL(3, 3, S, 4, 4, 8, 2, 2);                        \
            return CALL(3, 3, S, 4, 4, 8, 2, 1);                                     \
        }                                                                            \
        if (xt == 4) return CALL(3, 3, S, 4, 4, 8, 1, 4);                            \
        if (xt == 2) return CALL(3, 3, S, 4, 4, 8, 1, 2);                            \
        return CALL(3, 3, S, 4, 4, 8, 1, 1);                                         \
    }
// (kernels per lane: 160 and 192 kernels, frequent in these layers, pad to 192 = 3 x 64)
#define CPOCONV_STRIP_LINE(CALL, KH, KW, TXW, XTW)                                   \
    if (g.kh == KH && g.kw == KW && g.stride == 1 && strip_xt(g) == XTW) {           \
        if (g.Kpad % 192 == 0) return CALL(KH, KW, 1, 4, TXW, 8, 3, XTW);            \
        if (g.Kpad % 128 == 0) return CALL(KH, KW, 1, 4, TXW, 8, 2, XTW);            \
        return CALL(KH, KW, 1, 4, TXW, 8, 1, XTW);                                   \
    }
#define CPOCONV_STRIP_DISPATCH(CALL)                                                 \
    CPOCONV_STRIP_LINE(CALL, 1, 7, 6, 3)                                             \
    CPOCONV_STRIP_LINE(CALL, 7, 1, 6, 3)                                             \
    CPOCONV_STRIP_LINE(CALL, 1, 3, 4, 2)                                             \
    CPOCONV_STRIP_LINE(CALL, 3, 1, 4, 2)                                             \
    CPOCONV_STRIP_WIDE(CALL, 1, 1)                                                   \
    CPOCONV_STRIP_3X3(CALL, 1)                                                       \
    CPOCONV_STRIP_3X3(CALL, 2)                                                       \
    if (g.kh == 5 && g.kw == 5 && g.stride == 1) {                                   \
        if (g.N >= kBatchedFromImages && g.Kpad % 192 == 0) return CALL(5, 5, 1, 4, 4, 4, 3, 1); \
        if (g.N >= kBatchedFromImages && g.Kpad % 128 == 0) return CALL(5, 5, 1, 4, 4, 4, 2, 1); \
        return CALL(5, 5, 1, 4, 4, 8, 1, 1);                                         \
    }                                                                                \
    if (g.kh == 7 && g.kw == 7 && g.stride == 2) return CALL(7, 7, 2, 4, 4, 4, 1, 1);

int64_t strip_kernel_partial_bytes(const Geometry &g)
{
    if (!strip_kernel_supports(g)) return 0;
#define CPOCONV_STRIP_BYTES(KH, KW, S, TY, TX, G, KPL, XT)                                      \
    [&]() -> int64_t {                                                                          \
        const StripPlan p = strip_plan<KH, KW, S, TY, TX, G, KPL, XT>(g);                       \
        return 4 * static_cast<int64_t>(p.slices) * p.Ypad * ((g.Ow + TX * XT - 1) / (TX * XT) * (TX * XT)) * g.Kpad * g.N; \
    }()
    CPOCONV_STRIP_DISPATCH(CPOCONV_STRIP_BYTES)
#undef CPOCONV_STRIP_BYTES
    return 0;
}

int launch_sparse_conv_strip(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g,
                             const float *wt, float *out, float *partial, BatchStrides bs, hipStream_t stream)
{
#define CPOCONV_STRIP_LAUNCH(KH, KW, S, TY, TX, G, KPL, XT) \
    launch_strip<KH, KW, S, TY, TX, G, KPL, XT>(map, indices, mtab, g, wt, out, partial, bs, stream)
    CPOCONV_STRIP_DISPATCH(CPOCONV_STRIP_LAUNCH)
#undef CPOCONV_STRIP_LAUNCH
    return CPOCONV_ERR_SHAPE;
}

}  // namespace cpoconv
