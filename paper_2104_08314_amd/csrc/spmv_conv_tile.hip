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
// The tile's partial sums go to a [slice][y][x][k] buffer (k fastest: coalesced); a second
// kernel adds the slices in order and transposes to the K x Oh x Ow output.
#include "common.hpp"

namespace cpoconv {

namespace {

constexpr int kWavesPerWg = 4;
constexpr int kTabBytes = 8 * 1024;  // LDS budget of the per-channel range table

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

struct TileArgs {
    const int32_t *ptr;
    const float *da;
    const int32_t *in;        // one index per NZE, laid out like DA
    const int32_t *chan_off;  // 3*(C+1)
    const float *wt;          // [C][kh*kw][Kpad]
    float *partial;           // [slices][Ypad][Xpad][Kpad]
    int32_t slices;           // channel slices across workgroups
    int32_t Ypad, Xpad;
    int32_t batch;            // channels per table refill
};

template <int KH, int KW, int S, int TY, int TX, int KPL>
__global__ __launch_bounds__(kWavesPerWg *kLanes) void spmv_conv_tile_kernel(const Geometry g, const TileArgs a)
{
    constexpr int RH = (TY - 1) * S + KH;      // rows of the input patch behind the tile
    constexpr int RW = (TX - 1) * S + KW;      // columns of it
    constexpr int NCELL = RH * RW;
    constexpr int NDREG = (NCELL + kLanes - 1) / kLanes;
    constexpr int TAPS = KH * KW;
    constexpr int SPAN_MAX = TX + KW + 1;      // table entries per (channel, type): M[p_lo-1 .. p_hi]

    extern __shared__ int32_t smem[];
    // layout: lastp[n_types][SPAN_MAX] | tab[batch][n_types][SPAN_MAX] | patch[4][NCELL] ; the
    // reduction buffer (TY*TX*KPL*64 floats) overlays all of it after the channel loop
    int32_t *lastp = smem;
    int32_t *tab = lastp + g.n_types * SPAN_MAX;
    float *patch_all = reinterpret_cast<float *>(tab + a.batch * g.n_types * SPAN_MAX);

    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kLanes;
    const int x0 = blockIdx.x * TX, y0 = blockIdx.y * TY;
    const int ngroups = g.Kpad / (kLanes * KPL);
    const int kg = blockIdx.z % ngroups, slice = blockIdx.z / ngroups;
    const int kbase = kg * kLanes * KPL;
    float *patch = patch_all + wave * NCELL;

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

    for (int i = lane; i < NCELL; i += kLanes) patch[i] = 0.0f;

    // ---- geometry only: for every type and table slot, the last partition <= p that shows a
    // column of the type (binary search in the type's ascending first-partition list) ----------
    for (int idx = tid; idx < g.n_types * SPAN_MAX; idx += blockDim.x) {
        const int i = idx / SPAN_MAX, e = idx - i * SPAN_MAX;
        const int t = g.type_id[i];
        const int p = max(0, x0 - t) - 1 + e;                 // slot e holds partition p_lo - 1 + e
        int lo = g.type_begin[i], hi = g.type_begin[i + 1];   // columns [lo, hi)
        const int first = lo;
        while (lo < hi) {                                     // first column with p0 > p
            const int mid = (lo + hi) >> 1;
            if (static_cast<int>(g.col_p0[mid]) <= p) lo = mid + 1; else hi = mid;
        }
        // slot of ptr's segment to read: column index inside the type for the 3-entry NOP
        // segment, else the partition number; -1: nothing of this type up to p
        int v = -1;
        if (lo > first) v = (g.nop3 && t == 0) ? (lo - first - 1) : static_cast<int>(g.col_p0[lo - 1]);
        lastp[idx] = v;
    }

    for (int cb = c_begin; cb < c_end; cb += a.batch) {
        const int nb = min(a.batch, c_end - cb);
        __syncthreads();   // lastp ready / previous batch's table no longer in use
        // ---- table: absolute DA offset after partition p, for the partitions that reach the tile
        for (int idx = tid; idx < nb * g.n_types * SPAN_MAX; idx += blockDim.x) {
            const int e = idx % SPAN_MAX;
            const int i = (idx / SPAN_MAX) % g.n_types;
            const int c = cb + idx / (SPAN_MAX * g.n_types);
            int seg = a.chan_off[c];
            int off = a.chan_off[(g.C + 1) + c];
            int val = off;
            if (a.ptr[seg] != CPOCONV_NPC) {
                // walk the segments of the types before i: NPF = 1 entry, else 1+Ow (3 for NOP3);
                // a live type's NZE count is its last cumulative entry
                for (int ii = 0; ii < i; ++ii) {
                    const bool three = g.nop3 && g.type_id[ii] == 0;
                    if (three) { off += a.ptr[seg + 2]; seg += 3; }
                    else if (a.ptr[seg] == CPOCONV_NPF) seg += 1;
                    else {
                        const int last_col = g.type_begin[ii + 1] - 1;
                        off += a.ptr[seg + 1 + g.col_p0[last_col]];
                        seg += 1 + g.Ow;
                    }
                }
                const bool three = g.nop3 && g.type_id[i] == 0;
                const int lp = lastp[i * SPAN_MAX + e];
                val = off;
                if (lp >= 0 && (three || a.ptr[seg] != CPOCONV_NPF)) val = off + a.ptr[seg + 1 + lp];
            }
            tab[idx] = val;
        }
        __syncthreads();

        // ---- this wavefront's channels of the batch: wave, wave+4, ... ---------------------
        for (int cl = wave; cl < nb; cl += kWavesPerWg) {
            const int c = cb + cl;
            // weights of channel c for this lane's kernels
            float w[TAPS][KPL];
            const float *wc = a.wt + static_cast<int64_t>(c) * TAPS * g.Kpad + kbase + lane;
#pragma unroll
            for (int tp = 0; tp < TAPS; ++tp)
#pragma unroll
                for (int k = 0; k < KPL; ++k) w[tp][k] = wc[tp * g.Kpad + k * kLanes];

            bool any = false;
            for (int i = 0; i < g.n_types; ++i) {
                const int t = g.type_id[i];
                const int p_lo = max(0, x0 - t), p_hi = min(g.Ow - 1, x0 + TX - 1);
                const int32_t *row = tab + (cl * g.n_types + i) * SPAN_MAX;
                const int first = uni(row[0]), last = uni(row[p_hi - p_lo + 1]);
                if (last == first) continue;                       // nothing of this type reaches the tile
                for (int p = p_lo; p <= p_hi; ++p) {
                    const int beg = uni(row[p - p_lo]), end = uni(row[p - p_lo + 1]);
                    for (int n0 = beg; n0 < end; n0 += kLanes) {
                        const int n = n0 + lane;
                        if (n < end) {
                            const int idx = a.in[n];
                            const float v = a.da[n];
                            const int h = idx / KW, wh = idx - h * KW;
                            const int r = h - y0 * S;                 // row inside the patch
                            const int q = (p - x0) * S + wh;          // column inside the patch
                            if (r >= 0 && r < RH && q >= 0 && q < RW) patch[q * RH + r] = v;
                        }
                    }
                    any = true;
                }
            }
            if (!any) continue;

            // ---- patch -> lanes, bitmap of non-zero cells, clear the patch ------------------
            float cell[NDREG];
            unsigned long long bits[NDREG];
#pragma unroll
            for (int d = 0; d < NDREG; ++d) {
                const int i = d * kLanes + lane;
                cell[d] = i < NCELL ? patch[i] : 0.0f;
                bits[d] = __ballot((__float_as_uint(cell[d]) & 0x7fffffffu) != 0u);
            }
#pragma unroll
            for (int d = 0; d < NDREG; ++d) {
                const int i = d * kLanes + lane;
                if (i < NCELL) patch[i] = 0.0f;
            }

            // ---- convSpMv over the patch: compile-time cells, registers and weights ---------
#pragma unroll
            for (int q = 0; q < RW; ++q) {
#pragma unroll
                for (int r = 0; r < RH; ++r) {
                    const int cellno = q * RH + r;
                    if (bits[cellno / kLanes] & (1ull << (cellno % kLanes))) {
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
        }
    }

    // ---- add the four wavefronts' accumulators in a fixed order: 3 -> 2 -> 1 -> 0 -----------
    float *red = reinterpret_cast<float *>(smem);   // TY*TX*KPL*64 floats, overlays the tables
    for (int src = kWavesPerWg - 1; src >= 1; --src) {
        __syncthreads();
        if (wave == src) {
#pragma unroll
            for (int y = 0; y < TY; ++y)
#pragma unroll
                for (int x = 0; x < TX; ++x)
#pragma unroll
                    for (int k = 0; k < KPL; ++k) red[((y * TX + x) * KPL + k) * kLanes + lane] = acc[y][x][k];
        }
        __syncthreads();
        if (wave == src - 1) {
#pragma unroll
            for (int y = 0; y < TY; ++y)
#pragma unroll
                for (int x = 0; x < TX; ++x)
#pragma unroll
                    for (int k = 0; k < KPL; ++k) acc[y][x][k] += red[((y * TX + x) * KPL + k) * kLanes + lane];
        }
    }
    if (wave == 0) {
        float *dst = a.partial + ((static_cast<int64_t>(slice) * a.Ypad + y0) * a.Xpad + x0) * g.Kpad + kbase + lane;
#pragma unroll
        for (int y = 0; y < TY; ++y)
#pragma unroll
            for (int x = 0; x < TX; ++x)
#pragma unroll
                for (int k = 0; k < KPL; ++k)
                    dst[(static_cast<int64_t>(y) * a.Xpad + x) * g.Kpad + k * kLanes] = acc[y][x][k];
    }
}

// out[k][y][x] = sum over slices (ascending) of partial[slice][y][x][k]; one workgroup per
// (output row, 64 kernels): reads coalesced along k, writes coalesced along x via an LDS tile.
__global__ __launch_bounds__(256) void reduce_transpose_kernel(const Geometry g, const float *__restrict__ partial,
                                                              int slices, int Ypad, int Xpad, float *__restrict__ out)
{
    extern __shared__ float t[];            // 64 x (Ow + 1)
    const int y = blockIdx.x, kb = blockIdx.y * kLanes;
    const int tid = threadIdx.x, lane = tid & (kLanes - 1), wave = tid / kLanes;
    const int ld = g.Ow + 1;
    const int64_t slice_stride = static_cast<int64_t>(Ypad) * Xpad * g.Kpad;
    for (int x = wave; x < g.Ow; x += 4) {
        const float *src = partial + (static_cast<int64_t>(y) * Xpad + x) * g.Kpad + kb + lane;
        float s = src[0];
        for (int sl = 1; sl < slices; ++sl) s += src[sl * slice_stride];
        t[lane * ld + x] = s;
    }
    __syncthreads();
    for (int i = tid; i < kLanes * g.Ow; i += 256) {
        const int k = i / g.Ow, x = i - k * g.Ow;
        if (kb + k < g.K) out[(static_cast<int64_t>(kb + k) * g.Oh + y) * g.Ow + x] = t[k * ld + x];
    }
}

template <int KH, int KW, int S, int TY, int TX, int KPL>
int launch_tile(const cpoconv_map &map, const int32_t *indices, const Geometry &g, const float *wt, float *out,
                float *partial, int slices, hipStream_t stream)
{
    constexpr int RH = (TY - 1) * S + KH, RW = (TX - 1) * S + KW, NCELL = RH * RW;
    constexpr int SPAN_MAX = TX + KW + 1;
    const int ntx = (g.Ow + TX - 1) / TX, nty = (g.Oh + TY - 1) / TY;
    const int ngroups = g.Kpad / (kLanes * KPL);
    int batch = kTabBytes / (g.n_types * SPAN_MAX * 4);
    if (batch > 64) batch = 64;
    if (batch < kWavesPerWg) batch = kWavesPerWg;
    TileArgs a;
    a.ptr = map.ptr; a.da = map.da; a.in = indices; a.chan_off = map.chan_off; a.wt = wt;
    a.partial = partial; a.slices = slices; a.Ypad = nty * TY; a.Xpad = ntx * TX; a.batch = batch;
    const size_t work = (static_cast<size_t>(g.n_types) * SPAN_MAX * (1 + batch) + kWavesPerWg * NCELL) * 4;
    const size_t red = static_cast<size_t>(TY) * TX * KPL * kLanes * 4;
    const size_t lds = work > red ? work : red;
    hipLaunchKernelGGL((spmv_conv_tile_kernel<KH, KW, S, TY, TX, KPL>), dim3(ntx, nty, ngroups * slices),
                       dim3(kWavesPerWg * kLanes), lds, stream, g, a);
    CPOCONV_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(reduce_transpose_kernel, dim3(g.Oh, g.Kpad / kLanes), dim3(256),
                       static_cast<size_t>(kLanes) * (g.Ow + 1) * 4, stream, g, partial, slices, a.Ypad, a.Xpad, out);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

}  // namespace

// Tile geometry of the register kernel, shared with the scratch-size computation.
constexpr int kTileY = 8, kTileX = 8;

bool tile_kernel_supports(const Geometry &g)
{
    const bool shape = (g.kh == 3 && g.kw == 3 && (g.stride == 1 || g.stride == 2)) ||
                       (g.kh == 5 && g.kw == 5 && g.stride == 1) || (g.kh == 7 && g.kw == 7 && g.stride == 2);
    return shape;
}

int tile_kernel_slices(const Geometry &g)
{
    // enough workgroups to fill the chip (about 2 per CU), each keeping >= 8 channels
    const int ntiles = ((g.Ow + kTileX - 1) / kTileX) * ((g.Oh + kTileY - 1) / kTileY);
    const int kpl = (g.Kpad % 128 == 0 && g.kh * g.kw <= 9) ? 2 : 1;
    const int wgs = ntiles * (g.Kpad / (kLanes * kpl));
    int s = (512 + wgs - 1) / wgs;
    const int cap = (g.C + 7) / 8;
    if (s > cap) s = cap;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    return s;
}

int64_t tile_kernel_partial_bytes(const Geometry &g)
{
    if (!tile_kernel_supports(g)) return 0;
    const int64_t Ypad = (g.Oh + kTileY - 1) / kTileY * kTileY, Xpad = (g.Ow + kTileX - 1) / kTileX * kTileX;
    return 4 * Ypad * Xpad * g.Kpad * tile_kernel_slices(g);
}

int launch_sparse_conv_tile(const cpoconv_map &map, const int32_t *indices, const Geometry &g, const float *wt,
                            float *out, float *partial, hipStream_t stream)
{
    const int slices = tile_kernel_slices(g);
    const bool kpl2 = (g.Kpad % 128 == 0 && g.kh * g.kw <= 9);
#define CPOCONV_TILE(KH, KW, S)                                                                         \
    if (g.kh == KH && g.kw == KW && g.stride == S) {                                                    \
        if (kpl2) return launch_tile<KH, KW, S, kTileY, kTileX, 2>(map, indices, g, wt, out, partial, slices, stream); \
        return launch_tile<KH, KW, S, kTileY, kTileX, 1>(map, indices, g, wt, out, partial, slices, stream);           \
    }
    CPOCONV_TILE(3, 3, 1)
    CPOCONV_TILE(3, 3, 2)
    CPOCONV_TILE(5, 5, 1)
    CPOCONV_TILE(7, 7, 2)
#undef CPOCONV_TILE
    return CPOCONV_ERR_SHAPE;
}

}  // namespace cpoconv
