// Column-run SpMV convolution over a CPO map (Algorithm 2): the work is driven by the NZE lists.
//
// CPO streams are column-major: inside a channel and overlap type the NZEs follow the partitions
// and, inside a partition's new column, the padded rows, ascending.  ptr therefore delimits the
// run of NZEs of every padded column (with one new column per overlap type and partition, which
// holds for every kernel shape taken here), and inside a run the NZEs that reach a band of output
// rows are one contiguous piece, because the run is sorted by row.
//
// Work split: a workgroup owns one TY x TX tile of output positions for 64*KPL output kernels
// (lanes are kernels, KPL per lane); its wavefronts split the input channels and add their sums
// through LDS in a fixed order when the channels are done - no barrier before that.  Per channel
// a wavefront
//   1. reads the bounds of the runs of the (TX-1)*S+KW padded columns behind its tile from the
//      table of resolved ptr offsets (wavefront-uniform);
//   2. loads every run with lane = position in the run (value and index, coalesced; lanes past the
//      run repeat its last NZE);
//   3. sends every NZE whose row lies inside the input window behind the tile to the lane of that
//      row (index - first index of the window, divided by kw; one forward permute per column), so a
//      window column is a dense vector in one register, and takes the ballot of its non-zero lanes;
//   4. walks the set bits: the value is read from its (compile-time) lane into a scalar register
//      and the kh*(pType+1) multiply-adds of convSpMv that land in the tile are issued with
//      compile-time registers for sums and weights.
// An empty cell costs one scalar bit test and an untaken branch; loads, permutes and multiply-adds
// follow the number of NZEs and runs, not the map size.
// Loads of the next channel (bounds, runs, weights) are issued before the current one is applied.
// With several channel slices across workgroups the tile's sums go to partial[slice][y][x][k] and a
// second kernel adds the slices in a fixed order; with one slice the output is written directly.

#include <algorithm>

#include "common.hpp"

namespace cpoconv {

namespace {

constexpr int kMaxWaves = 16;              // wavefronts (channel slices) per workgroup
constexpr int kRunsMaxSlices = 16;         // channel slices across workgroups
constexpr int kEmptyIndex = 0x7fffffff;    // index of a lane past the end of its run

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

struct RunsArgs {
    int32_t slices;          // channel slices across workgroups
    int32_t Ypad, Xpad;      // extents of the partial-sum planes
    BatchStrides bs;         // image n of the launch: every buffer advanced n strides
};

// The multiply-adds of one NZE at row R, column Q of the input window behind the tile: kernel row l
// and column ww meet it for output (R - l) / S, (Q - ww) / S when that lies inside the tile.
template <int KH, int KW, int S, int TY, int TX, int KPL, int Q, int R>
__device__ __forceinline__ void apply_nze(float (&acc)[TY][TX][KPL], const float (&w)[KH * KW][KPL], const float v)
{
#pragma unroll
    for (int l = 0; l < KH; ++l) {
        if ((R - l) < 0 || (R - l) % S != 0 || (R - l) / S >= TY) continue;
#pragma unroll
        for (int ww = 0; ww < KW; ++ww) {
            if ((Q - ww) < 0 || (Q - ww) % S != 0 || (Q - ww) / S >= TX) continue;
#pragma unroll
            for (int kk = 0; kk < KPL; ++kk)
                acc[(R - l) / S][(Q - ww) / S][kk] = fmaf(v, w[l * KW + ww][kk], acc[(R - l) / S][(Q - ww) / S][kk]);
        }
    }
}

// One window column.  Lane k of idx / val is the k-th NZE of the column's run (lanes past the run
// hold kEmptyIndex).  The NZEs whose rows lie inside the window are sent to the lane of their window
// row with one cross-lane move (a forward permute: it uses the LDS crossbar, no LDS memory; lanes
// that receive nothing read zero), so the column segment sits in a register as a dense vector.  A
// ballot of its non-zero lanes is the bitmap of occupied rows; the walk over the rows is unrolled: a
// clear bit costs a scalar bit test and an untaken branch, a set bit broadcasts the value from its
// (compile-time) lane and issues the multiply-adds of that row.
template <int KH, int KW, int S, int TY, int TX, int KPL, int Q, int R>
__device__ __forceinline__ void apply_rows(float (&acc)[TY][TX][KPL], const float (&w)[KH * KW][KPL], const int col,
                                           const unsigned mask)
{
    constexpr int RH = (TY - 1) * S + KH;
    if constexpr (R < RH) {
        if (__builtin_expect((mask >> R) & 1u, 1)) {
            const float v = __int_as_float(__builtin_amdgcn_readlane(col, R));
            apply_nze<KH, KW, S, TY, TX, KPL, Q, R>(acc, w, v);
        }
        apply_rows<KH, KW, S, TY, TX, KPL, Q, R + 1>(acc, w, col, mask);
    }
}

template <int KH, int KW, int S, int TY, int TX, int KPL, int Q>
__device__ __forceinline__ void walk_columns(float (&acc)[TY][TX][KPL], const float (&w)[KH * KW][KPL],
                                             const int (&col)[(TX - 1) * S + KW], const unsigned (&mask)[(TX - 1) * S + KW])
{
    constexpr int RW = (TX - 1) * S + KW;
    if constexpr (Q < RW) {
        apply_rows<KH, KW, S, TY, TX, KPL, Q, 0>(acc, w, col[Q], mask[Q]);
        walk_columns<KH, KW, S, TY, TX, KPL, Q + 1>(acc, w, col, mask);
    }
}

// One channel's loads: per window column the run's indices and values, lane k = k-th NZE of the run
// (lanes past the run repeat its last NZE: harmless, they land on the same lane with the same value),
// the scalar bound that tells rows inside the window from the rest (0 for a column without a run:
// then nothing is inside), and the channel's weights for this lane's KPL kernels.
template <int TAPS, int KPL, int RW>
struct ChannelSet {
    int idx[RW];
    float val[RW];
    unsigned lim[RW];
    float w[TAPS][KPL];
};

template <int KH, int KW, int S, int TY, int TX, int KPL>
__device__ __forceinline__ void apply_columns(float (&acc)[TY][TX][KPL], ChannelSet<KH * KW, KPL, (TX - 1) * S + KW> &cs,
                                              const int lo)
{
    constexpr int RH = (TY - 1) * S + KH;
    constexpr int RW = (TX - 1) * S + KW;
    static_assert(RH < kLanes - 1, "the window's rows must leave the last lane free");
    static_assert(RH * KW < (1 << 12), "the multiply-shift below is exact for small operands only");
    int col[RW];
    unsigned mask[RW];
    // The weights are the youngest loads of this channel's set and loads complete in order: one
    // wait on the last weight register here covers every register the walk below reads, instead
    // of a wait in front of each multiply-add.
    asm volatile("" : "+v"(cs.w[KH * KW - 1][KPL - 1]));
    // every column's cross-lane move is issued before the first one is used
#pragma unroll
    for (int q = 0; q < RW; ++q) {
        // index = column in partition + padded row * kw: d / kw is the row inside the window
        const unsigned d = static_cast<unsigned>(cs.idx[q] - lo);
        const bool inside = d < cs.lim[q];
        const unsigned row = KW == 1 ? d : __umul24(d, (1u << 16) / KW + 1u) >> 16;
        const int dst = inside ? static_cast<int>(row) : kLanes - 1;   // the last lane collects the rest and is never read
        col[q] = __builtin_amdgcn_ds_permute(dst << 2, __float_as_int(cs.val[q]));
    }
#pragma unroll
    for (int q = 0; q < RW; ++q) mask[q] = static_cast<unsigned>(__ballot(col[q] != 0));
    walk_columns<KH, KW, S, TY, TX, KPL, 0>(acc, cs.w, col, mask);
}

// KPL consecutive floats as one load
template <int KPL> struct WeightVec;
template <> struct WeightVec<1> { typedef float type; };
template <> struct WeightVec<2> { typedef float2 type; };
template <> struct WeightVec<3> { struct type { float x, y, z; }; };
template <> struct WeightVec<4> { typedef float4 type; };

typedef const __attribute__((address_space(4))) int32_t *TablePtr;   // read-only for the kernel: scalar loads

template <int KH, int KW, int S, int TY, int TX, int KPL, int NW, bool IN16>
__global__ __launch_bounds__(NW *kLanes) void spmv_conv_runs_kernel(
    const Geometry g, const RunsArgs a, const float *__restrict__ da_all, const int32_t *__restrict__ in_all,
    const int32_t *__restrict__ mtab_all, const float *__restrict__ wt, float *__restrict__ partial_all,
    float *__restrict__ out_all)
{
    constexpr int RH = (TY - 1) * S + KH;      // rows of the padded input behind the tile
    constexpr int RW = (TX - 1) * S + KW;      // columns of it
    constexpr int TAPS = KH * KW;
    constexpr int A = TY * TX * KPL;           // accumulators per lane
    using Set = ChannelSet<TAPS, KPL, RW>;

    extern __shared__ float red[];             // [wavefront][accumulator][lane], used after the channel loop

    const int lane = lane_id();
    const int wave = uni(threadIdx.x / kLanes), nwaves = blockDim.x / kLanes;
    const int ngroups = g.Kpad / (kLanes * KPL);
    const int kg = blockIdx.z % ngroups, slice = (blockIdx.z / ngroups) % a.slices;
    const int image = blockIdx.z / (ngroups * a.slices);
    if (map_unusable(a.bs, image)) return;
    const int x0 = blockIdx.x * TX, y0 = blockIdx.y * TY;
    const int kbase = kg * kLanes * KPL;       // this lane holds kernels kbase + lane * KPL .. + KPL - 1
    const char *__restrict__ da = reinterpret_cast<const char *>(da_all + image * a.bs.da);
    const char *__restrict__ in = reinterpret_cast<const char *>(index_advance(in_all, image * a.bs.indices, IN16 ? 1 : 0));
    const TablePtr mtab = (TablePtr)(mtab_all + image * a.bs.mtab);

    // where the bounds of every window column's run sit inside a channel's block of the table:
    // row of its overlap type, entry of its first partition (Section 3.2); -1: no encoded column
    int toff[RW];
#pragma unroll
    for (int q = 0; q < RW; ++q) {
        const int j = x0 * S + q;
        const int lo_num = j - KW + 1;
        const int p_lo = lo_num <= 0 ? 0 : (lo_num + S - 1) / S;
        const int p_hi = min(j / S, g.Ow - 1);
        const int t = p_hi - p_lo;               // overlap type: partitions holding the column, minus one
        int slot = -1;
        for (int i = 0; i < g.n_types; ++i)
            if (static_cast<int>(g.type_id[i]) == t) slot = i;
        const bool real = j >= g.pad_w && j < g.pad_w + g.W;
        toff[q] = (real && t >= 0 && slot >= 0) ? slot * (g.Ow + 1) + p_lo : -1;
    }
    const int lo = y0 * S * KW;                  // indices below it lie above the window
    const int tab_block = g.n_types * (g.Ow + 1);
    const unsigned lane4 = static_cast<unsigned>(lane) * 4u;
    const unsigned lane_w = static_cast<unsigned>(lane) * (KPL * 4u);

    // channels of this wavefront: c_begin + wave, + nwaves, ..
    const int per_slice = (g.C + a.slices - 1) / a.slices;
    const int c_begin = slice * per_slice, c_end = min(g.C, c_begin + per_slice);

    float acc[TY][TX][KPL];
#pragma unroll
    for (int y = 0; y < TY; ++y)
#pragma unroll
        for (int x = 0; x < TX; ++x)
#pragma unroll
            for (int kk = 0; kk < KPL; ++kk) acc[y][x][kk] = 0.0f;

    // bounds of a channel's runs: scalar loads, (begin, end) pairs side by side in the table
    auto load_bounds = [&](int c, int (&beg)[RW], int (&end)[RW]) {
        const TablePtr blk = mtab + static_cast<int64_t>(min(c, c_end - 1)) * tab_block;
#pragma unroll
        for (int q = 0; q < RW; ++q) {
            const int at = max(toff[q], 0);
            beg[q] = blk[at];
            end[q] = (toff[q] >= 0 && c < c_end) ? blk[at + 1] : beg[q];   // no column, no channel: an empty run
        }
    };
    auto load_set = [&](int c, const int (&beg)[RW], const int (&end)[RW], Set &cs) {
#pragma unroll
        for (int q = 0; q < RW; ++q) {
            const int cnt = end[q] - beg[q];
            cs.lim[q] = cnt > 0 ? static_cast<unsigned>(RH * KW) : 0u;
            // lane k reads NZE min(k, cnt - 1) of the run (NZE 0 of the stream for an empty run: never used)
            const unsigned last4 = static_cast<unsigned>(max(end[q], 1) - 1) * 4u;
            const unsigned at = min(static_cast<unsigned>(beg[q]) * 4u + lane4, last4);
            cs.idx[q] = IN16 ? static_cast<int>(*reinterpret_cast<const int16_t *>(in + at / 2))   // compact map: same values
                             : *reinterpret_cast<const int32_t *>(in + at);
            cs.val[q] = *reinterpret_cast<const float *>(da + at);
        }
        const float *wc = wt + static_cast<int64_t>(min(c, g.C - 1)) * TAPS * g.Kpad + kbase;
#pragma unroll
        for (int tp = 0; tp < TAPS; ++tp) {
            typedef typename WeightVec<KPL>::type Vec;
            const Vec v = *reinterpret_cast<const Vec *>(reinterpret_cast<const char *>(wc + tp * g.Kpad) + lane_w);
            const float *f = reinterpret_cast<const float *>(&v);
#pragma unroll
            for (int kk = 0; kk < KPL; ++kk) cs.w[tp][kk] = f[kk];
        }
    };

    // two register sets in turn: the loads of one channel are in flight while the other is applied,
    // and the bounds are fetched one channel further ahead
    {
        Set sa, sb;
        int beg_a[RW], end_a[RW], beg_b[RW], end_b[RW];
        const int c0 = c_begin + wave;
        load_bounds(c0, beg_a, end_a);
        load_bounds(c0 + nwaves, beg_b, end_b);
        load_set(c0, beg_a, end_a, sa);
#pragma unroll 1
        for (int c = c0; c < c_end; c += 2 * nwaves) {
            load_set(c + nwaves, beg_b, end_b, sb);
            load_bounds(c + 2 * nwaves, beg_a, end_a);
            apply_columns<KH, KW, S, TY, TX, KPL>(acc, sa, lo);
            load_set(c + 2 * nwaves, beg_a, end_a, sa);
            load_bounds(c + 3 * nwaves, beg_b, end_b);
            apply_columns<KH, KW, S, TY, TX, KPL>(acc, sb, lo);
        }
    }

    // ---- add the wavefronts' sums: every wavefront parks its registers in LDS; after one barrier
    // wavefront w adds, always in wavefront order, accumulators w, w + nwaves, .. and stores them
    auto acc_at = [&](int n) -> float & { return acc[n / (TX * KPL)][(n / KPL) % TX][n % KPL]; };
#pragma unroll
    for (int n = 0; n < A; ++n) red[(wave * A + n) * kLanes + lane] = acc_at(n);
    __syncthreads();
    float *partial = partial_all + image * a.bs.partial;
    float *out = out_all + image * a.bs.out;
    for (int n = wave; n < A; n += nwaves) {
        float s = red[n * kLanes + lane];
        for (int w2 = 1; w2 < nwaves; ++w2) s += red[(w2 * A + n) * kLanes + lane];
        const int y = y0 + n / (TX * KPL), x = x0 + (n / KPL) % TX, k = kbase + lane * KPL + n % KPL;
        if (a.slices > 1) {
            // partial sums of this channel slice, kernel index fastest (tiles past the map's edge included)
            partial[((static_cast<int64_t>(slice) * a.Ypad + y) * a.Xpad + x) * g.Kpad + k] = s;
        } else if (y < g.Oh && x < g.Ow && k < g.K) {
            out[(static_cast<int64_t>(k) * g.Oh + y) * g.Ow + x] = s;
        }
    }
}

struct RunsPlan {
    int ty, tx, kpl, waves, slices;
};

// Launch shape (measured on MI355X at one to three images per launch, where this kernel is used):
// 4 x 4 tiles, two kernels per lane where the padded kernel count allows, sixteen wavefronts per
// workgroup - fewer when that would leave a wavefront less than two channels - and channel slices
// across workgroups only while the tiles alone leave compute units without a workgroup (config 2:
// 196 workgroups, one slice, 31 against 35 us for the strip kernel and its slice sum).
RunsPlan runs_plan(const Geometry &g)
{
    RunsPlan p;
    p.ty = 4; p.tx = 4;
    p.kpl = g.Kpad % 128 == 0 ? 2 : 1;
    const int tiles = ((g.Ow + p.tx - 1) / p.tx) * ((g.Oh + p.ty - 1) / p.ty) * (g.Kpad / (kLanes * p.kpl)) * g.N;
    p.waves = kMaxWaves;
    while (p.waves > 1 && g.C < 2 * p.waves) p.waves /= 2;
    int s = 256 / std::max(tiles, 1);
    s = std::min(std::min(s, std::max(1, g.C / (2 * p.waves))), kRunsMaxSlices);
    s = std::max(s, 1);
    const int per_slice = (g.C + s - 1) / s;
    p.slices = (g.C + per_slice - 1) / per_slice;
    return p;
}

template <int KH, int KW, int S, int TY, int TX, int KPL, int NW>
int launch_runs(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g, const float *wt,
                float *out, float *partial, const RunsPlan &p, BatchStrides bs, hipStream_t stream)
{
    const int ntx = (g.Ow + TX - 1) / TX, nty = (g.Oh + TY - 1) / TY;
    const int ngroups = g.Kpad / (kLanes * KPL);
    RunsArgs a;
    a.slices = p.slices; a.Ypad = nty * TY; a.Xpad = ntx * TX;
    bs.partial = static_cast<int64_t>(p.slices) * a.Ypad * a.Xpad * g.Kpad;
    a.bs = bs;
    const size_t lds = static_cast<size_t>(p.waves) * TY * TX * KPL * kLanes * sizeof(float);
    if (lds > 160 * 1024 || p.waves > NW) return CPOCONV_ERR_SHAPE;
    {
        KernelTimer timer("spmv_conv_runs", stream);
        const dim3 grid(ntx, nty, ngroups * p.slices * g.N), block(p.waves * kLanes);
        if (bs.indices16)
            hipLaunchKernelGGL((spmv_conv_runs_kernel<KH, KW, S, TY, TX, KPL, NW, true>), grid, block, lds, stream, g, a, map.da,
                               indices, mtab, wt, partial, out);
        else
            hipLaunchKernelGGL((spmv_conv_runs_kernel<KH, KW, S, TY, TX, KPL, NW, false>), grid, block, lds, stream, g, a, map.da,
                               indices, mtab, wt, partial, out);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    if (p.slices > 1) return launch_reduce_transpose(g, partial, p.slices, a.Ypad, a.Xpad, out, bs, stream);
    return CPOCONV_OK;
}

}  // namespace

// Shapes the kernel is instantiated for, maps whose column runs fit a wavefront (one lane per
// padded row), and geometries with one new column per overlap type and partition (a stride that
// does not divide the padded width leaves a last column that shares its partition with another).
bool runs_kernel_supports(const Geometry &g)
{
    if (g.n_types < 1 || g.Ih > kLanes) return false;
    if (!(g.kh == 3 && g.kw == 3 && g.stride == 1)) return false;
    for (int i = 0; i < g.n_types; ++i)
        for (int n = g.type_begin[i] + 1; n < g.type_begin[i + 1]; ++n)
            if (g.col_p0[n] == g.col_p0[n - 1]) return false;
    return true;
}

// Measured over the workload layers at one to three images per launch: where the tiles alone give
// every compute unit a workgroup (one channel slice: no partial sums, no second kernel) the kernel
// is 3 us faster per layer than the strip kernel with its slice sum (config 2: 44 against 47 us for
// the layer, 64 x 56 x 56: 32 against 35); on the smaller maps, which need channel slices across
// workgroups either way, it ties with the register-tile kernel, which keeps them.  From four images
// on the strip kernel's shared decode wins (config 2 at 32 images: 12.6 against 15.3 us per image).
bool runs_kernel_preferred(const Geometry &g)
{
    return runs_kernel_supports(g) && g.N < 4 && runs_plan(g).slices == 1;
}

int64_t runs_kernel_partial_bytes(const Geometry &g)
{
    if (!runs_kernel_supports(g)) return 0;
    const RunsPlan p = runs_plan(g);
    if (p.slices == 1) return 0;
    const int64_t Ypad = (g.Oh + p.ty - 1) / p.ty * p.ty, Xpad = (g.Ow + p.tx - 1) / p.tx * p.tx;
    return 4 * Ypad * Xpad * g.Kpad * p.slices * g.N;
}

int launch_sparse_conv_runs(const cpoconv_map &map, const int32_t *indices, const int32_t *mtab, const Geometry &g,
                            const float *wt, float *out, float *partial, BatchStrides bs, hipStream_t stream)
{
    const RunsPlan p = runs_plan(g);
    if (p.kpl == 2) {
        if (p.waves > 8) return launch_runs<3, 3, 1, 4, 4, 2, 16>(map, indices, mtab, g, wt, out, partial, p, bs, stream);
        return launch_runs<3, 3, 1, 4, 4, 2, 8>(map, indices, mtab, g, wt, out, partial, p, bs, stream);
    }
    if (p.waves > 8) return launch_runs<3, 3, 1, 4, 4, 1, 16>(map, indices, mtab, g, wt, out, partial, p, bs, stream);
    return launch_runs<3, 3, 1, 4, 4, 1, 8>(map, indices, mtab, g, wt, out, partial, p, bs, stream);
}

}  // namespace cpoconv
