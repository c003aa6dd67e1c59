// Register-tile SpMV convolution over a CPO map (Algorithm 2) for the common kernel shapes.
//
// Work split: a workgroup owns one TY x TX tile of output positions for 64*KPL output
// kernels and one slice of the input channels; its four wavefronts split that slice again and
// add their accumulators through LDS in a fixed order.  Lanes are output kernels, so the NZE
// being applied is wavefront-uniform (a scalar operand of the FMA) and the weights of the
// current channel sit in registers, one register per kernel cell.
//
// Per channel a wavefront
//   1. takes from a small LDS table the DA / IN range of every partition that reaches its
//      tile (ptr's cumulative counts with the "-1 = previous entry" rule already applied),
//   2. loads those NZEs with lane = position in the column, keeps the rows that reach the
//      tile and drops each value at its (column, row) cell of a private LDS patch of the
//      padded input (index / kw = padded row, index % kw = column inside the partition),
//   3. reads the patch back one cell per lane; a ballot gives the bitmap of non-zero cells,
//   4. walks the cells in a fully unrolled loop: a cell whose bit is clear costs two scalar
//      instructions; a set bit broadcasts the value from its lane and issues the kh*(pType+1)
//      FMAs of convSpMv that land inside the tile, all with compile-time register indices.
// With several channel slices the tile's partial sums go to a [slice][y][x][k] buffer (k fastest:
// coalesced) and a second kernel adds the slices in a fixed order and transposes to the
// K x Oh x Ow output; with one slice the output is written directly.
#include "common.hpp"

namespace cpoconv {

namespace {

constexpr int kTabBytes = 8 * 1024;  // LDS budget of the per-channel range table
constexpr int kGroup = 4;
// 64-NZE chunks of a channel whose loads are issued ahead.  The scatter of every such chunk is
// compiled branch-free (predicated), so chunks past the channel's NZEs still cost their arithmetic:
// two instead of four took 1.5 us off the 14 x 14 and 28 x 28 layers at batch 1; further chunks
// of dense channels are loaded on demand.
constexpr int kChunksAhead = 2;
constexpr int kMaxSlices = 16;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

struct TileArgs {
    const float *da;
    const int32_t *in;        // one index per NZE, laid out like DA
    const int32_t *mtab;      // [C][n_types][Ow+1] absolute DA offsets (prologue kernel)
    const float *wt;          // [C][kh*kw][Kpad]
    float *partial;           // [slices][Ypad][Xpad][Kpad]
    float *out;               // K x Oh x Ow, written directly when there is one slice
    int32_t slices;           // channel slices across workgroups
    BatchStrides bs;          // image n of the launch: every buffer advanced n strides
    int32_t Ypad, Xpad;
    int32_t batch;            // channels per table refill
};

template <int KH, int KW, int S, int TY, int TX, int KPL, int NW>
__global__ __launch_bounds__(NW *kLanes) void spmv_conv_tile_kernel(const Geometry g, const TileArgs a_launch)
{
    constexpr int kWavesPerWg = NW;
    constexpr int RH = (TY - 1) * S + KH;      // rows of the input patch behind the tile
    constexpr int RW = (TX - 1) * S + KW;      // columns of it
    constexpr int NCELL = RH * RW;
    constexpr int NDREG = (NCELL + kLanes - 1) / kLanes;
    constexpr int TAPS = KH * KW;
    constexpr int SPAN_MAX = TX + KW + 1;      // table entries per (channel, type): M[p_lo-1 .. p_hi]
    constexpr int G = kGroup;                  // channels whose loads are in flight together
    constexpr int MAXC = kChunksAhead;         // 64-NZE chunks of a channel loaded ahead

    extern __shared__ int32_t smem[];
    // layout: tab[batch][n_types][SPAN_MAX] | patch[NW][G][NCELL] ; the reduction buffers
    // overlay all of it after the channel loop
    int32_t *tab = smem;
    float *patch_all = reinterpret_cast<float *>(tab + a_launch.batch * g.n_types * SPAN_MAX);

    const int tid = threadIdx.x, lane = lane_id();
    const int wave = uni(tid / kLanes);   // in a scalar register: everything derived from it stays scalar
    const int x0 = blockIdx.x * TX, y0 = blockIdx.y * TY;
    const int ngroups = g.Kpad / (kLanes * KPL);
    const int kg = blockIdx.z % ngroups, slice = (blockIdx.z / ngroups) % a_launch.slices;
    const int image = blockIdx.z / (ngroups * a_launch.slices);
    if (map_unusable(a_launch.bs, image)) return;
    TileArgs a = a_launch;
    a.da += image * a.bs.da;
    a.in = index_advance(a.in, image * a.bs.indices, a.bs.indices16);
    a.mtab += image * a.bs.mtab;
    a.partial += image * a.bs.partial;
    a.out += image * a.bs.out;
    const int kbase = kg * kLanes * KPL;
    float *patch = patch_all + wave * (G * NCELL);   // G private patches per wavefront

    // channel range of this workgroup
    const int per_slice = (g.C + a.slices - 1) / a.slices;
    const int c_begin = slice * per_slice, c_end = min(g.C, c_begin + per_slice);
    float acc[TY][TX][KPL];
#pragma unroll
    for (int y = 0; y < TY; ++y)
#pragma unroll
        for (int x = 0; x < TX; ++x)
#pragma unroll
            for (int k = 0; k < KPL; ++k) acc[y][x][k] = 0.0f;

    for (int i = lane; i < G * NCELL; i += kLanes) patch[i] = 0.0f;

    for (int cb = c_begin; cb < c_end; cb += a.batch) {
        const int nb = min(a.batch, c_end - cb);
        __syncthreads();   // previous batch's table no longer in use
        // ---- table: DA offset after partition p for the partitions that reach the tile; slot e
        // of (channel, type) holds partition p_lo - 1 + e (clamped: later slots repeat the end)
        for (int idx = tid; idx < nb * g.n_types * SPAN_MAX; idx += blockDim.x) {
            const int e = idx % SPAN_MAX;
            const int i = (idx / SPAN_MAX) % g.n_types;
            const int c = cb + idx / (SPAN_MAX * g.n_types);
            const int p = min(max(0, x0 - static_cast<int>(g.type_id[i])) - 1 + e, g.Ow - 1);
            tab[idx] = a.mtab[(static_cast<int64_t>(c) * g.n_types + i) * (g.Ow + 1) + p + 1];
        }
        __syncthreads();

        // ---- this wavefront's channels of the batch (wave, wave+NW, ..), G at a time ----------
        // The DA / IN loads of G channels are issued back to back before any of them is used,
        // so their latency is paid once per group and not once per partition.
        const int main_slot = g.n_types - 1;   // the highest overlap type holds most NZEs
        for (int j0 = wave; j0 < nb; j0 += kWavesPerWg * G) {
            int idxr[G][MAXC];
            float valr[G][MAXC];
            int first[G], last[G];
            {
                const int t = g.type_id[main_slot];
                const int span = min(g.Ow - 1, x0 + TX - 1) - max(0, x0 - t) + 1;
#pragma unroll
                for (int gi = 0; gi < G; ++gi) {
                    const int cl = j0 + gi * kWavesPerWg;
                    first[gi] = 0;
                    last[gi] = 0;
                    if (cl < nb) {
                        const int32_t *row = tab + (cl * g.n_types + main_slot) * SPAN_MAX;
                        first[gi] = uni(row[0]);
                        last[gi] = uni(row[span]);
                    }
#pragma unroll
                    for (int ch = 0; ch < MAXC; ++ch) {
                        const int n = first[gi] + ch * kLanes + lane;
                        const bool ok = n < last[gi];
                        idxr[gi][ch] = ok ? load_index(a.in, n, a.bs.indices16) : -1;
                        valr[gi][ch] = ok ? a.da[n] : 0.0f;
                    }
                }
            }
            // weights of the group's first channel
            float w[TAPS][KPL];
            {
                const float *wc = a.wt + static_cast<int64_t>(cb + j0) * TAPS * g.Kpad + kbase + lane;
#pragma unroll
                for (int tp = 0; tp < TAPS; ++tp)
#pragma unroll
                    for (int k = 0; k < KPL; ++k) w[tp][k] = wc[tp * g.Kpad + k * kLanes];
            }

            // one NZE -> its cell of the patch.  n is its position in DA; the partition is the
            // number of table boundaries at or below n (ptr used as in CSR).
            auto scatter = [&](int idx, float v, int n, const int (&bound)[SPAN_MAX], int p_lo, float *pt) {
                int prel = 0;
#pragma unroll
                for (int e = 1; e < SPAN_MAX; ++e) prel += (n >= bound[e]) ? 1 : 0;
                const int h = idx / KW, wh = idx - h * KW;   // padded row, column inside the partition
                const int r = h - y0 * S;
                const int q = (p_lo + prel - x0) * S + wh;
                if (idx >= 0 && r >= 0 && r < RH && q >= 0 && q < RW) pt[q * RH + r] = v;
            };

#pragma unroll
            for (int gi = 0; gi < G; ++gi) {
                const int cl = j0 + gi * kWavesPerWg;
                if (cl >= nb) continue;
                float *pt = patch + gi * NCELL;
                {
                    const int t = g.type_id[main_slot];
                    const int p_lo = max(0, x0 - t);
                    const int32_t *row = tab + (cl * g.n_types + main_slot) * SPAN_MAX;
                    int bound[SPAN_MAX];
#pragma unroll
                    for (int e = 0; e < SPAN_MAX; ++e) bound[e] = uni(row[e]);
#pragma unroll
                    for (int ch = 0; ch < MAXC; ++ch)
                        if (first[gi] + ch * kLanes < last[gi])
                            scatter(idxr[gi][ch], valr[gi][ch], first[gi] + ch * kLanes + lane, bound, p_lo, pt);
                    // columns with more NZEs than the prefetched chunks hold
                    for (int n0 = first[gi] + MAXC * kLanes; n0 < last[gi]; n0 += kLanes) {
                        const int n = n0 + lane;
                        const bool ok = n < last[gi];
                        scatter(ok ? load_index(a.in, n, a.bs.indices16) : -1, ok ? a.da[n] : 0.0f, n, bound, p_lo, pt);
                    }
                }
                // the lower overlap types (edge columns): few NZEs, loaded on demand
                for (int i = 0; i < main_slot; ++i) {
                    const int t = g.type_id[i];
                    const int p_lo = max(0, x0 - t), p_hi = min(g.Ow - 1, x0 + TX - 1);
                    const int32_t *row = tab + (cl * g.n_types + i) * SPAN_MAX;
                    const int f = uni(row[0]), l = uni(row[p_hi - p_lo + 1]);
                    if (l == f) continue;
                    int bound[SPAN_MAX];
#pragma unroll
                    for (int e = 0; e < SPAN_MAX; ++e) bound[e] = uni(row[e]);
                    for (int n0 = f; n0 < l; n0 += kLanes) {
                        const int n = n0 + lane;
                        const bool ok = n < l;
                        scatter(ok ? load_index(a.in, n, a.bs.indices16) : -1, ok ? a.da[n] : 0.0f, n, bound, p_lo, pt);
                    }
                }
            }
#pragma unroll 1
            for (int gi = 0; gi < G; ++gi) {
                const int cl = j0 + gi * kWavesPerWg;
                if (cl >= nb) break;
                float *pt = patch + gi * NCELL;
                // weights of the next channel of the group, in flight during this channel's FMAs
                float wn[TAPS][KPL];
                {
                    const int cn = min(cb + cl + kWavesPerWg, g.C - 1);
                    const float *wc = a.wt + static_cast<int64_t>(cn) * TAPS * g.Kpad + kbase + lane;
#pragma unroll
                    for (int tp = 0; tp < TAPS; ++tp)
#pragma unroll
                        for (int k = 0; k < KPL; ++k) wn[tp][k] = wc[tp * g.Kpad + k * kLanes];
                }
                // ---- patch -> lanes, bitmap of non-zero cells, clear the patch ------------------
                float cell[NDREG];
                unsigned long long bits[NDREG];
#pragma unroll
                for (int d = 0; d < NDREG; ++d) {
                    const int i = d * kLanes + lane;
                    cell[d] = i < NCELL ? pt[i] : 0.0f;
                    bits[d] = __ballot((__float_as_uint(cell[d]) & 0x7fffffffu) != 0u);
                }
#pragma unroll
                for (int d = 0; d < NDREG; ++d) {
                    const int i = d * kLanes + lane;
                    if (i < NCELL) pt[i] = 0.0f;
                }
                // ---- convSpMv over the patch: compile-time cells, registers and weights ---------
#pragma unroll
                for (int q = 0; q < RW; ++q) {
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
                                    for (int k = 0; k < KPL; ++k)
                                        acc[(r - l) / S][(q - ww) / S][k] =
                                            fmaf(v, w[l * KW + ww][k], acc[(r - l) / S][(q - ww) / S][k]);
                                }
                            }
                        }
                    }
                }
#pragma unroll
                for (int tp = 0; tp < TAPS; ++tp)
#pragma unroll
                    for (int k = 0; k < KPL; ++k) w[tp][k] = wn[tp][k];
            }
        }
    }

    // ---- add the wavefronts' accumulators.  Every wavefront parks its registers in LDS (16 bytes
    // per lane and access); after one barrier wavefront w adds, always in wavefront order, the
    // copies of accumulator group w and stores that part of the tile itself, so the stores are
    // spread over the workgroup too.
    constexpr int KW64 = KPL * kLanes;
    constexpr int A = TY * TX * KPL;           // accumulators per lane
    static_assert(A % 4 == 0, "tile accumulators must pack into float4");
    constexpr int A4 = A / 4;
    float4 *red4 = reinterpret_cast<float4 *>(smem);
    float *red = reinterpret_cast<float *>(smem);
    auto acc_at = [&](int n) -> float & { return acc[n / (TX * KPL)][(n / KPL) % TX][n % KPL]; };
    __syncthreads();   // table and patches are no longer in use: the parking area overlays them
    {
        float4 *dst = red4 + wave * A4 * kLanes + lane;
#pragma unroll
        for (int j = 0; j < A4; ++j)
            dst[j * kLanes] = make_float4(acc_at(4 * j), acc_at(4 * j + 1), acc_at(4 * j + 2), acc_at(4 * j + 3));
    }
    __syncthreads();
    constexpr int LDT = KW64 + 1;              // row stride of the transposed tile (bank conflicts)
    float4 sums[(A4 + kWavesPerWg - 1) / kWavesPerWg];
#pragma unroll
    for (int jj = 0; jj < (A4 + kWavesPerWg - 1) / kWavesPerWg; ++jj) {
        const int j = wave + jj * kWavesPerWg;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < A4) {
            t = red4[j * kLanes + lane];
#pragma unroll
            for (int w2 = 1; w2 < kWavesPerWg; ++w2) {
                const float4 v = red4[(w2 * A4 + j) * kLanes + lane];
                t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
            }
        }
        sums[jj] = t;
    }
    if (a.slices > 1) {
        // partial sums of this channel slice, kernel index fastest
#pragma unroll
        for (int jj = 0; jj < (A4 + kWavesPerWg - 1) / kWavesPerWg; ++jj) {
            const int j = wave + jj * kWavesPerWg;
            if (j >= A4) continue;
            const float e[4] = {sums[jj].x, sums[jj].y, sums[jj].z, sums[jj].w};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int n = 4 * j + u, y = n / (TX * KPL), x = (n / KPL) % TX, k = n % KPL;
                a.partial[((static_cast<int64_t>(slice) * a.Ypad + y0 + y) * a.Xpad + x0 + x) * g.Kpad + kbase + k * kLanes + lane] = e[u];
            }
        }
        return;   // a second kernel adds the slices
    }
    // one slice: transpose through LDS and store the K x Oh x Ow output directly, TX consecutive x
    // per kernel and row
    __syncthreads();   // every wavefront has read the parked copies: the area is free again
#pragma unroll
    for (int jj = 0; jj < (A4 + kWavesPerWg - 1) / kWavesPerWg; ++jj) {
        const int j = wave + jj * kWavesPerWg;
        if (j >= A4) continue;
        const float e[4] = {sums[jj].x, sums[jj].y, sums[jj].z, sums[jj].w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int n = 4 * j + u, y = n / (TX * KPL), x = (n / KPL) % TX, k = n % KPL;
            red[(y * TX + x) * LDT + k * kLanes + lane] = e[u];
        }
    }
    __syncthreads();
    for (int i = tid; i < TY * TX * KW64; i += kWavesPerWg * kLanes) {
        const int x = i % TX, k = (i / TX) % KW64, y = i / (TX * KW64);
        if (kbase + k < g.K && y0 + y < g.Oh && x0 + x < g.Ow)
            a.out[(static_cast<int64_t>(kbase + k) * g.Oh + y0 + y) * g.Ow + x0 + x] = red[(y * TX + x) * LDT + k];
    }
}

// Launch shape of the register kernel for a layer.
struct TilePlan {
    int ty, tx, kpl, nw, slices;
};

TilePlan plan_for(const Geometry &g)
{
    // Measured on MI355X over the workload layers: 4 x 8 tiles with 64 kernels per wavefront and
    // eight wavefronts per workgroup win or tie everywhere; the channel slices are chosen so that
    // about 1.5 workgroups per compute unit exist while each wavefront keeps a channel or more.
    TilePlan p;
    p.ty = 4; p.tx = 8; p.kpl = 1; p.nw = 8;
    const int ntiles = ((g.Ow + p.tx - 1) / p.tx) * ((g.Oh + p.ty - 1) / p.ty);
    const int wgs = ntiles * (g.Kpad / (kLanes * p.kpl)) * g.N;
    int s = (512 + wgs / 2) / wgs;
    const int cap = (g.C + 7) / 8;
    if (s > cap) s = cap;
    if (s > kMaxSlices) s = kMaxSlices;
    if (s < 1) s = 1;
    // no empty slices: with ceil(C / s) channels each, fewer slices may already cover the layer
    const int per_slice = (g.C + s - 1) / s;
    p.slices = (g.C + per_slice - 1) / per_slice;
    return p;
}

template <int KH, int KW, int S, int TY, int TX, int KPL, int NW>
int launch_tile(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g,
                const float *wt, float *out, float *partial, int slices, BatchStrides bs, hipStream_t stream)
{
    constexpr int RH = (TY - 1) * S + KH, RW = (TX - 1) * S + KW, NCELL = RH * RW;
    constexpr int SPAN_MAX = TX + KW + 1;
    const int ntx = (g.Ow + TX - 1) / TX, nty = (g.Oh + TY - 1) / TY;
    const int ngroups = g.Kpad / (kLanes * KPL);
    int batch = kTabBytes / (g.n_types * SPAN_MAX * 4);
    if (batch > 128) batch = 128;
    if (batch < NW) batch = NW;
    TileArgs a;
    a.da = map.da; a.in = indices; a.mtab = mtab; a.wt = wt;
    a.partial = partial; a.out = out; a.slices = slices; a.Ypad = nty * TY; a.Xpad = ntx * TX; a.batch = batch;
    bs.partial = static_cast<int64_t>(slices) * a.Ypad * a.Xpad * g.Kpad;
    a.bs = bs;
    const size_t work = (static_cast<size_t>(g.n_types) * SPAN_MAX * batch + NW * kGroup * NCELL) * 4;
    const size_t park = static_cast<size_t>(NW) * TY * TX * KPL * kLanes * 4;   // every wavefront's accumulators
    const size_t transpose = static_cast<size_t>(TY) * TX * (KPL * kLanes + 1) * 4;
    size_t lds = work;
    if (park > lds) lds = park;
    if (transpose > lds) lds = transpose;
    {
        KernelTimer timer("spmv_conv_tile", stream);
        hipLaunchKernelGGL((spmv_conv_tile_kernel<KH, KW, S, TY, TX, KPL, NW>), dim3(ntx, nty, ngroups * slices * g.N),
                           dim3(NW * kLanes), lds, stream, g, a);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    if (slices > 1) return launch_reduce_transpose(g, partial, slices, a.Ypad, a.Xpad, out, bs, stream);
    return CPOCONV_OK;
}

}  // namespace

bool tile_kernel_supports(const Geometry &g)
{
    if (g.n_types < 1) return false;
    if ((g.kh == 3 && g.kw == 3 && (g.stride == 1 || g.stride == 2)) ||
        (g.kh == 5 && g.kw == 5 && g.stride == 1) || (g.kh == 7 && g.kw == 7 && g.stride == 2))
        return true;
    // the 1 x n and n x 1 layers of the SI's layer tables (K_h = 1: the general algorithm; K_w = 1:
    // a single overlap type, the SI's special case)
    return g.stride == 1 && ((g.kh == 1 && (g.kw == 3 || g.kw == 7)) || (g.kw == 1 && (g.kh == 3 || g.kh == 7)));
}

int64_t tile_kernel_partial_bytes(const Geometry &g)
{
    if (!tile_kernel_supports(g)) return 0;
    const TilePlan p = plan_for(g);
    const int64_t Ypad = (g.Oh + p.ty - 1) / p.ty * p.ty, Xpad = (g.Ow + p.tx - 1) / p.tx * p.tx;
    return 4 * Ypad * Xpad * g.Kpad * p.slices * g.N;
}

int launch_sparse_conv_tile(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g,
                            const float *wt, float *out, float *partial, BatchStrides bs, hipStream_t stream)
{
    const TilePlan p = plan_for(g);
#define CPOCONV_TILE(KH, KW, S)                    \
    if (g.kh == KH && g.kw == KW && g.stride == S) \
        return launch_tile<KH, KW, S, 4, 8, 1, 8>(map, indices, mtab, g, wt, out, partial, p.slices, bs, stream);
    CPOCONV_TILE(3, 3, 1)
    CPOCONV_TILE(3, 3, 2)
    CPOCONV_TILE(5, 5, 1)
    CPOCONV_TILE(7, 7, 2)
    CPOCONV_TILE(1, 7, 1)
    CPOCONV_TILE(7, 1, 1)
    CPOCONV_TILE(1, 3, 1)
    CPOCONV_TILE(3, 1, 1)
#undef CPOCONV_TILE
    return CPOCONV_ERR_SHAPE;
}

}  // namespace cpoconv
