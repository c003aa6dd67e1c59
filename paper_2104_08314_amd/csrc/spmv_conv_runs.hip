// Column-run SpMV convolution over a CPO map (Algorithm 2): the work is driven by the NZE lists.
//
// CPO streams are column-major: inside a channel and overlap type the NZEs follow the partitions
// and, inside a partition's new column, the padded rows, ascending.  ptr therefore delimits the
// run of NZEs of every padded column (with one new column per overlap type and partition, which
// holds for every kernel shape taken here), and a run is sorted by row.  What the kernel needs of
// a column is then two things: where its run starts in DA, and which padded rows hold an NZE - a
// 64-bit row bitmap (maps up to 64 padded rows).  Both sit in a table of one 16-byte entry per
// (channel, padded column), written by the encoder when it runs in the same call (it has the
// bitmaps in hand: they are how it counts) or rebuilt from ptr and IN by column_table_kernel.
// With the table the indices of a run never have to be read: the k-th set bit of the bitmap is the
// row of the run's k-th NZE.
//
// Work split: a workgroup owns one TY x TX tile of output positions for 64*KPL output kernels
// (lanes are kernels, KPL per lane); its wavefronts split the input channels and add their sums
// through LDS in a fixed order when the channels are done - no barrier before that.  Per channel
// a wavefront
//   1. reads the table entries of the (TX-1)*S+KW padded columns behind its tile (scalar loads) and
//      cuts the rows of the input window behind the tile out of every bitmap: the window's bits, and
//      the number of NZEs of the run above the window (a population count);
//   2. loads the window's NZEs with ONE vector load, lane = 8 * window column + window row: the
//      lane of a set bit reads DA[run start + NZEs above the window + set bits below its own];
//   3. walks the window bits, which are scalar registers: a clear bit costs a scalar bit test and an
//      untaken branch, a set bit reads the value from its (compile-time) lane into a scalar register
//      and issues the kh*(pType+1) multiply-adds of convSpMv that land in the tile, with
//      compile-time registers for sums and weights.
// Loads and multiply-adds follow the number of NZEs, not the map size.  The entries of the channel
// after next and the values and weights of the next channel are in flight while the current one is
// applied.  With several channel slices across workgroups the tile's sums go to
// partial[slice][y][x][k] and a second kernel adds the slices in a fixed order; with one slice the
// output is written directly.

#include <algorithm>

#include "common.hpp"
#include "resolve_ptr.hpp"

namespace cpoconv {

namespace {

constexpr int kMaxWaves = 16;              // wavefronts (channel slices) per workgroup
constexpr int kRunsMaxSlices = 16;         // channel slices across workgroups
constexpr int kRowsPerColumn = 8;          // lanes a window column takes in the value register
constexpr int kXcds = 8;                   // accelerator dies, each with an L2 of its own

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

// The walk over the window, unrolled: bit 8 * Q + R of `cells` says whether row R of window column Q
// holds an NZE; its value sits in the lane of that number.
template <int KH, int KW, int S, int TY, int TX, int KPL, int Q, int R>
__device__ __forceinline__ void apply_rows(float (&acc)[TY][TX][KPL], const float (&w)[KH * KW][KPL], const float values,
                                           const unsigned long long cells)
{
    constexpr int RH = (TY - 1) * S + KH;
    if constexpr (R < RH) {
        if (__builtin_expect((cells >> (Q * kRowsPerColumn + R)) & 1ull, 1)) {
            const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(values), Q * kRowsPerColumn + R));
            apply_nze<KH, KW, S, TY, TX, KPL, Q, R>(acc, w, v);
        }
        apply_rows<KH, KW, S, TY, TX, KPL, Q, R + 1>(acc, w, values, cells);
    }
}

template <int KH, int KW, int S, int TY, int TX, int KPL, int Q>
__device__ __forceinline__ void walk_columns(float (&acc)[TY][TX][KPL], const float (&w)[KH * KW][KPL], const float values,
                                             const unsigned long long cells)
{
    constexpr int RW = (TX - 1) * S + KW;
    if constexpr (Q < RW) {
        apply_rows<KH, KW, S, TY, TX, KPL, Q, 0>(acc, w, values, cells);
        walk_columns<KH, KW, S, TY, TX, KPL, Q + 1>(acc, w, values, cells);
    }
}

// One channel's window: which of its cells hold an NZE (bit 8 * column + row, wavefront-uniform),
// the NZEs themselves (in the lane of that number; other lanes hold zero) and the channel's weights
// for this lane's KPL kernels.
template <int TAPS, int KPL>
struct ChannelSet {
    unsigned long long cells;
    float values;
    float w[TAPS][KPL];
};

// KPL consecutive floats as one load
template <int KPL> struct WeightVec;
template <> struct WeightVec<1> { typedef float type; };
template <> struct WeightVec<2> { typedef float2 type; };
template <> struct WeightVec<3> { struct type { float x, y, z; }; };
template <> struct WeightVec<4> { typedef float4 type; };

static_assert(sizeof(ColumnEntry) == 16, "an entry is read as four ints");

template <int KH, int KW, int S, int TY, int TX, int KPL, int NW>
__global__ __launch_bounds__(NW *kLanes) void spmv_conv_runs_kernel(
    const Geometry g, const RunsArgs a, const float *__restrict__ da_all, const ColumnEntry *__restrict__ columns_all,
    const float *__restrict__ wt, float *__restrict__ partial_all, float *__restrict__ out_all)
{
    constexpr int RH = (TY - 1) * S + KH;      // rows of the padded input behind the tile
    constexpr int RW = (TX - 1) * S + KW;      // columns of it
    constexpr int TAPS = KH * KW;
    constexpr int A = TY * TX * KPL;           // accumulators per lane
    static_assert(RH <= kRowsPerColumn && RW * kRowsPerColumn <= kLanes, "the window must fit one register, 8 lanes per column");
    using Set = ChannelSet<TAPS, KPL>;

    extern __shared__ float red[];             // [wavefront][accumulator][lane], used after the channel loop

    const int lane = lane_id();
    const int wave = uni(threadIdx.x / kLanes), nwaves = blockDim.x / kLanes;
    const int ngroups = g.Kpad / (kLanes * KPL);
    const int kg = blockIdx.z % ngroups, slice = (blockIdx.z / ngroups) % a.slices;
    const int image = blockIdx.z / (ngroups * a.slices);
    if (map_unusable(a.bs, image)) return;
    // Tile of this workgroup.  Workgroups go to the eight XCDs in turn by their linear number, and an
    // XCD's L2 fetches what its workgroups read: the tiles are numbered down the tile columns and the
    // numbers dealt so that an XCD holds a stretch of neighbouring tile columns - its L2 then fetches
    // the runs of those columns only, not the whole of DA and the table.
    const int n_tiles = gridDim.x * gridDim.y, issued = blockIdx.x + gridDim.x * blockIdx.y;
    const int xcd = issued % kXcds, nth = issued / kXcds;
    const int tile = xcd * (n_tiles / kXcds) + min(xcd, n_tiles % kXcds) + nth;
    const int x0 = (tile / static_cast<int>(gridDim.y)) * TX, y0 = (tile % static_cast<int>(gridDim.y)) * TY;
    const int kbase = kg * kLanes * KPL;       // this lane holds kernels kbase + lane * KPL .. + KPL - 1
    const float *__restrict__ da = da_all + image * a.bs.da;
    // the window's first padded column and row; lane 8 * q + r stands for row r of window column q; a
    // column past the padded width (a tile that hangs over the map's edge) reads the row's last entry
    // and counts as empty
    const int j0 = x0 * S, top = y0 * S;
    const int my_q = lane / kRowsPerColumn, my_r = lane % kRowsPerColumn;
    const bool my_cell = my_q < RW && my_r < RH && j0 + my_q < g.Iw;
    const int4 *__restrict__ my_entries =
        reinterpret_cast<const int4 *>(columns_all + image * a.bs.columns) + min(j0 + my_q, g.Iw - 1);
    const unsigned long long above = (1ull << top) - 1ull;        // top <= 63: the map has at most 64 padded rows
    const unsigned above_lo = static_cast<unsigned>(above), above_hi = static_cast<unsigned>(above >> 32);
    const unsigned below_mine = (1u << my_r) - 1u;
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

    // every lane reads the table entry of its own window column (begin, count, rows_lo, rows_hi): one
    // 16-byte load, the eight lanes of a column the same address
    auto load_entries = [&](int c, int4 &e) { e = my_entries[static_cast<int64_t>(min(c, c_end - 1)) * g.Iw]; };
    auto load_weights = [&](int c, Set &cs) {
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
    // the lane's cell: its bit of the column's rows; the NZE's place in DA is the run's start + the
    // NZEs of the run above the window + those of the window above the lane's row
    auto load_values = [&](int c, const int4 &e, Set &cs) {
        const unsigned rows_lo = static_cast<unsigned>(e.z), rows_hi = static_cast<unsigned>(e.w);
        const unsigned window = static_cast<unsigned>(((static_cast<unsigned long long>(rows_hi) << 32) | rows_lo) >> top);
        const bool has = my_cell && c < c_end && ((window >> my_r) & 1u);
        const int at = e.x + __popc(rows_lo & above_lo) + __popc(rows_hi & above_hi) + __popc(window & below_mine);
        cs.cells = __ballot(has);
        cs.values = has ? da[at] : 0.0f;
    };
    // values first: the weights are then the youngest loads of the set (see apply)
    auto load_set = [&](int c, const int4 &e, Set &cs) {
        load_values(c, e, cs);
        if (c < c_end) load_weights(c, cs);   // (wavefront-uniform) past the last channel the walk finds no bit set
    };
    auto apply = [&](Set &cs) {
        // The weights are the youngest loads of the set and loads complete in order: one wait on
        // the last weight register covers every register the walk reads, instead of a wait in
        // front of each multiply-add.
        asm volatile("" : "+v"(cs.w[TAPS - 1][KPL - 1]));
        if (cs.cells != 0ull) walk_columns<KH, KW, S, TY, TX, KPL, 0>(acc, cs.w, cs.values, cs.cells);
    };

    // two register sets in turn: the loads of one channel are in flight while the other is applied,
    // and the table entries are fetched one channel further ahead
    {
        Set sa = {}, sb = {};
        int4 ea, eb;
        const int c0 = c_begin + wave;
        load_entries(c0, ea);
        load_entries(c0 + nwaves, eb);
        load_weights(c0, sa);    // on their way before the first entries are back
        load_values(c0, ea, sa);
#pragma unroll 1
        for (int c = c0; c < c_end; c += 2 * nwaves) {
            load_set(c + nwaves, eb, sb);
            load_entries(c + 2 * nwaves, ea);
            apply(sa);
            load_set(c + 2 * nwaves, ea, sa);
            load_entries(c + 3 * nwaves, eb);
            apply(sb);
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
    if (TX == 4 && a.slices == 1 && g.Ow % 4 == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
        // direct output, four columns wide: a wavefront adds the four sums of a tile row for one of the
        // lane's kernels (same order of additions as below) and stores them as one 16-byte piece
        for (int pair = wave; pair < TY * KPL; pair += nwaves) {
            const int ty = pair / KPL, kk = pair % KPL;
            float s[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int n = (ty * TX + x) * KPL + kk;
                s[x] = red[n * kLanes + lane];
                for (int w = 1; w < nwaves; ++w) s[x] += red[(w * A + n) * kLanes + lane];
            }
            const int y = y0 + ty, k = kbase + lane * KPL + kk;
            if (y < g.Oh && x0 < g.Ow && k < g.K)   // Ow is a multiple of four: the whole piece lies inside the map
                *reinterpret_cast<float4 *>(out + (static_cast<int64_t>(k) * g.Oh + y) * g.Ow + x0) = make_float4(s[0], s[1], s[2], s[3]);
        }
        return;
    }
    for (int n = wave; n < A; n += nwaves) {
        float s = red[n * kLanes + lane];
        for (int w = 1; w < nwaves; ++w) s += red[(w * A + n) * kLanes + lane];
        const int y = y0 + n / (TX * KPL), x = x0 + (n / KPL) % TX, k = kbase + lane * KPL + n % KPL;
        if (a.slices > 1) {
            // partial sums of this channel slice, kernel index fastest (tiles past the map's edge included)
            partial[((static_cast<int64_t>(slice) * a.Ypad + y) * a.Xpad + x) * g.Kpad + k] = s;
        } else if (y < g.Oh && x < g.Ow && k < g.K) {
            out[(static_cast<int64_t>(k) * g.Oh + y) * g.Ow + x] = s;
        }
    }
}

// inclusive running sum over the 64 lanes (same moves as wave_running_max)
__device__ __forceinline__ int wave_running_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
    return v;
}

// The table of column entries rebuilt from the streams, for a convolution whose encoder ran in an
// earlier call: one workgroup per (channel, image).  First the channel's ptr segments become
// absolute DA offsets after every partition (Algorithm 2's forward fill, a running maximum: one
// wavefront, one lane per partition - or they are copied from the table of resolved offsets when a
// kernel before this one has left it).  Then one wavefront per stream column in turn: entries p0 and
// p0 + 1 of its type's row delimit the NZEs of the column's partition, which holds its columns one
// after the other (mostly just one; two at the map's edge when the stride is 2); every lane takes
// one NZE, index / kw is its padded row and index mod kw its column inside the partition: the NZEs
// of earlier columns give the start of this column's run, the rows of its own are or-ed into the
// bitmap through LDS.
//
// A CPS map (cps_top = slot of the overlap-kw type, else -1) is decoded here, straight from the
// packed stream: below the top type IN_cps holds one plain index per NZE, at the channel's IN
// offset plus the NZE's rank in the channel; the top type's entries are parsed as Algorithm 4 reads
// them, in parallel: an entry < 0 is a single NZE with the index negated; a run of entries >= 0
// alternates {index of the set's first NZE, pattern}, so an entry's role is the parity of its
// distance to the last negative entry before it (a running maximum), and the NZE an entry starts
// at is the running sum of the NZEs of the entries before it.  The pattern's bits from its first
// set bit up are the rows of the set's NZEs from the first one's row up; the column is the
// partition whose DA range holds the entry's first NZE (a search over the resolved offsets).
// Nothing is written per NZE.
constexpr int kTableThreads = 1024;                       // at most; the launch sizes the workgroup to the map
constexpr int kTableWaves = kTableThreads / kLanes;

__global__ __launch_bounds__(kTableThreads) void column_table_kernel(const Geometry g, const int32_t *__restrict__ ptr_all,
                                                                    const int32_t *__restrict__ chan_off_all,
                                                                    const int32_t *__restrict__ indices_all,
                                                                    const int32_t *__restrict__ mtab_all,
                                                                    ColumnEntry *__restrict__ columns_all, const BatchStrides bs,
                                                                    const int cps_top)
{
    __shared__ unsigned long long rows[kMaxCols];
    __shared__ int32_t offsets[kMaxTypes][kLanes + 1];   // Ow <= 62 for the maps taken here
    __shared__ int32_t run_begin[kMaxCols];              // start of every padded column's run in DA (count = set bits)
    __shared__ int32_t top_col[kLanes];                  // CPS: padded column of every partition of the top type
    __shared__ int32_t wave_neg[kTableWaves], wave_out[kTableWaves];
    const int c = blockIdx.x, image = blockIdx.y;
    if (map_unusable(bs, image)) return;
    const int lane = lane_id(), wave = threadIdx.x / kLanes;
    const int nthreads = blockDim.x, nwaves = nthreads / kLanes;
    const int32_t *indices = index_advance(indices_all, image * bs.indices, bs.indices16);
    const int32_t *chan_off = chan_off_all + static_cast<int64_t>(image) * 3 * (g.C + 1);
    ColumnEntry *out = columns_all + image * bs.columns + static_cast<int64_t>(c) * g.Iw;
    // CPS: IN entry of a lower-type NZE = the channel's IN offset + the NZE's rank in the channel
    const int da0 = chan_off[(g.C + 1) + c];
    const int in_shift = cps_top >= 0 ? chan_off[2 * (g.C + 1) + c] - da0 : 0;
    const int in_end = cps_top >= 0 ? chan_off[2 * (g.C + 1) + c + 1] : 0;
    for (int j = threadIdx.x; j < g.Iw; j += nthreads) { rows[j] = 0ull; run_begin[j] = 0; }
    if (threadIdx.x < kLanes) top_col[threadIdx.x] = 0;
    if (mtab_all != nullptr) {
        const int32_t *table = mtab_all + image * bs.mtab + static_cast<int64_t>(c) * g.n_types * (g.Ow + 1);
        for (int n = threadIdx.x; n < g.n_types * (g.Ow + 1); n += nthreads)
            offsets[n / (g.Ow + 1)][n % (g.Ow + 1)] = table[n];
    } else if (wave == 0) {
        const int32_t *ptr = ptr_all + image * bs.ptr;
        int seg = chan_off[c], at = chan_off[(g.C + 1) + c];
        const bool npc = ptr[seg] == CPOCONV_NPC;
        for (int i = 0; i < g.n_types; ++i) {
            int live = 0;   // 0: no NZE, 1: [pType, e_0 .. e_{Ow-1}], 2: the three-entry NOP segment
            if (!npc) live = (g.nop3 && g.type_id[i] == 0) ? 2 : (ptr[seg] == CPOCONV_NPF ? 0 : 1);
            int e = -1;
            if (lane < g.Ow) {
                if (live == 1) e = ptr[seg + 1 + lane];
                else if (live == 2) e = lane < g.Ow - 1 ? ptr[seg + 1] : ptr[seg + 2];
            }
            const int m = max(wave_running_max(e), 0);
            if (lane < g.Ow) offsets[i][1 + lane] = at + m;
            if (lane == 0) offsets[i][0] = at;
            at += __builtin_amdgcn_readlane(m, kLanes - 1);
            seg += npc ? 0 : (live == 2 ? 3 : (live == 1 ? 1 + g.Ow : 1));
        }
    }
    __syncthreads();
    for (int i = 0; i < g.n_types; ++i) {
        for (int vi = g.type_begin[i] + wave; vi < g.type_begin[i + 1]; vi += nwaves) {
            const int p0 = g.col_p0[vi], j = g.col_j[vi], what = g.col_what[vi];
            const int begin = offsets[i][p0], end = offsets[i][p0 + 1];   // the partition's NZEs: its columns in turn
            if (i == cps_top) {   // (one column per partition in this type)
                if (lane == 0) { run_begin[j] = begin; top_col[p0] = j; }
                continue;
            }
            int before = 0;       // NZEs of the partition's columns before this one
            for (int n0 = begin; n0 < end; n0 += kLanes) {
                const int index = n0 + lane < end ? load_index(indices, n0 + lane + in_shift, bs.indices16) : -1;
                const int row = index / g.kw, column = index - row * g.kw;
                before += __popcll(__ballot(index >= 0 && column < what));
                if (index >= 0 && column == what) atomicOr(&rows[j], 1ull << row);
            }
            if (lane == 0) run_begin[j] = begin + before;
        }
    }
    if (cps_top >= 0) {
        __syncthreads();   // top_col complete
        const int32_t *bound = offsets[cps_top];
        const int top_base = bound[0];
        const int e0 = top_base + in_shift;                           // first IN entry of the top type
        const int n_entries = in_end - e0;                            // the top type closes the channel
        int carry_neg = -1;   // position (from e0) of the last negative entry so far
        int carry_out = 0;    // NZEs of the entries so far
        // a lane's entry and the one behind it (the pattern, if the lane's entry leads a pair); the
        // next round's are in flight while this round's are parsed
        auto fetch = [&](int e, int &entry, int &after) {
            entry = e < n_entries ? load_index(indices, e0 + e, bs.indices16) : -1;
            after = e + 1 < n_entries ? load_index(indices, e0 + e + 1, bs.indices16) : 0;
        };
        int entry_next, after_next;
        fetch(threadIdx.x, entry_next, after_next);
        for (int first = 0; first < n_entries; first += nthreads) {
            const int e = first + threadIdx.x;
            const bool valid = e < n_entries;
            const int entry = entry_next, after = after_next;
            if (first + nthreads < n_entries) fetch(e + nthreads, entry_next, after_next);
            const int m = wave_running_max(entry < 0 ? e : -1);
            if (lane == kLanes - 1) wave_neg[wave] = m;
            __syncthreads();
            int before_neg = carry_neg;
            for (int w = 0; w < wave; ++w) before_neg = max(before_neg, wave_neg[w]);
            const int last_neg = max(m, before_neg);
            const bool leads = valid && entry >= 0 && ((e - last_neg - 1) & 1) == 0;   // the index of a {index, pattern} pair
            const int pattern = leads ? after : 0;
            const int emits = !valid ? 0 : (entry < 0 ? 1 : (leads ? __popc(pattern) : 0));
            const int s = wave_running_sum(emits);
            if (lane == kLanes - 1) wave_out[wave] = s;
            __syncthreads();
            int before_out = carry_out;
            for (int w = 0; w < wave; ++w) before_out += wave_out[w];
            if (emits > 0) {
                const int at = top_base + before_out + s - emits;   // DA position of the entry's first NZE
                int lo = 0, hi = g.Ow - 1;                          // smallest partition whose range ends past it
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (bound[mid + 1] > at) hi = mid; else lo = mid + 1;
                }
                const int index = entry < 0 ? -entry : entry;
                const unsigned long long set = entry < 0 ? 1ull : static_cast<unsigned long long>(pattern >> (__ffs(pattern) - 1));
                atomicOr(&rows[top_col[lo]], set << (index / g.kw));
            }
            int all_neg = carry_neg, all_out = carry_out;
            for (int w = 0; w < nwaves; ++w) { all_neg = max(all_neg, wave_neg[w]); all_out += wave_out[w]; }
            carry_neg = all_neg;
            carry_out = all_out;
            __syncthreads();   // wave_neg / wave_out free for the next round
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < g.Iw; j += nthreads) {   // padding columns: no run, no rows
        ColumnEntry entry;
        entry.begin = run_begin[j];
        entry.count = __popcll(rows[j]);
        entry.rows_lo = static_cast<uint32_t>(rows[j]);
        entry.rows_hi = static_cast<uint32_t>(rows[j] >> 32);
        out[j] = entry;
    }
}

struct RunsPlan {
    int ty, tx, kpl, waves, slices;
};

// The instantiations: kernel shape, stride, output tile.  The window of padded cells behind a tile,
// ((ty - 1) s + kh) x ((tx - 1) s + kw), takes a lane per cell, eight lanes per window column.
struct RunsShape {
    int kh, kw, stride, ty, tx, max_kpl;
};
constexpr RunsShape kRunsShapes[] = {
    {3, 3, 1, 4, 4, 2},   // 6 x 6 window
    {3, 3, 2, 3, 3, 2},   // 7 x 7
    {5, 5, 1, 4, 4, 1},   // 8 x 8; 25 weights per kernel: one kernel's worth of registers
    {1, 7, 1, 8, 2, 2},   // 8 x 8
    {7, 1, 1, 2, 8, 2},
    {1, 3, 1, 4, 4, 2},   // 4 x 6
    {3, 1, 1, 4, 4, 2},
};

const RunsShape *runs_shape(const Geometry &g)
{
    for (const RunsShape &r : kRunsShapes)
        if (r.kh == g.kh && r.kw == g.kw && r.stride == g.stride) return &r;
    return nullptr;
}

// Launch shape (measured on MI355X at one to three images per launch, where this kernel is used):
// the tile of the kernel shape (4 x 4 for 3 x 3 stride 1; larger and smaller tiles were slower), two
// kernels per lane where the padded kernel count allows, sixteen wavefronts per
// workgroup - fewer when that would leave a wavefront less than two channels - and channel slices
// across workgroups only while the tiles alone leave compute units without a workgroup.
RunsPlan runs_plan(const Geometry &g)
{
    RunsPlan p;
    const RunsShape *shape = runs_shape(g);
    p.ty = shape ? shape->ty : 4;
    p.tx = shape ? shape->tx : 4;
    p.kpl = (shape && g.Kpad % 128 == 0) ? shape->max_kpl : 1;
    const int tiles = ((g.Ow + p.tx - 1) / p.tx) * ((g.Oh + p.ty - 1) / p.ty) * (g.Kpad / (kLanes * p.kpl)) * g.N;
    p.waves = kMaxWaves;
    while (p.waves > 1 && g.C < 2 * p.waves) p.waves /= 2;
    int s = 256 / std::max(tiles, 1);
    // (a slice leaves every wavefront at least one channel; layers of few channels: two, measured on 16 -> 16 at 28 x 28)
    s = std::min(std::min(s, std::max(1, g.C / ((g.C < 64 ? 2 : 1) * p.waves))), kRunsMaxSlices);
    s = std::max(s, 1);
    const int per_slice = (g.C + s - 1) / s;
    p.slices = (g.C + per_slice - 1) / per_slice;
    return p;
}

template <int KH, int KW, int S, int TY, int TX, int KPL, int NW>
int launch_runs(const cpoconv_map &map, const ColumnEntry *columns, const Geometry &g, const float *wt, float *out,
                float *partial, const RunsPlan &p, BatchStrides bs, hipStream_t stream)
{
    const int ntx = (g.Ow + TX - 1) / TX, nty = (g.Oh + TY - 1) / TY;
    const int ngroups = g.Kpad / (kLanes * KPL);
    RunsArgs a;
    a.slices = p.slices; a.Ypad = nty * TY; a.Xpad = ntx * TX;
    bs.partial = static_cast<int64_t>(p.slices) * a.Ypad * a.Xpad * g.Kpad;
    a.bs = bs;
    const size_t lds = static_cast<size_t>(p.waves) * TY * TX * KPL * kLanes * sizeof(float);
    if (lds > 160 * 1024 || p.waves > NW || p.ty != TY || p.tx != TX || p.kpl != KPL) return CPOCONV_ERR_SHAPE;
    {
        KernelTimer timer("spmv_conv_runs", stream);
        const dim3 grid(ntx, nty, ngroups * p.slices * g.N), block(p.waves * kLanes);
        hipLaunchKernelGGL((spmv_conv_runs_kernel<KH, KW, S, TY, TX, KPL, NW>), grid, block, lds, stream, g, a, map.da, columns,
                           wt, partial, out);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    if (p.slices > 1) return launch_reduce_transpose(g, partial, p.slices, a.Ypad, a.Xpad, out, bs, stream);
    return CPOCONV_OK;
}

}  // namespace

// Shapes the kernel is instantiated for, maps of at most 64 padded rows (a column's rows are one
// 64-bit bitmap) and 64 partitions (one lane per partition where the table is rebuilt).
bool runs_kernel_supports(const Geometry &g)
{
    if (g.n_types < 1 || g.Ih > kLanes || g.Ow > kLanes) return false;
    if (runs_shape(g) == nullptr) return false;
    const RunsPlan p = runs_plan(g);
    if (static_cast<size_t>(p.waves) * p.ty * p.tx * p.kpl * kLanes * sizeof(float) > 160 * 1024) return false;   // the sums' LDS
    // every column of the map itself lies under some kernel position: then all columns outside the
    // streams are padding, and the table holds an empty entry for each of them
    if ((g.Ow - 1) * g.stride + g.kw < g.pad_w + g.W) return false;
    return true;
}

// Measured over the workload layers at one to three images per launch: where the tiles alone give
// every compute unit a workgroup (one channel slice: no partial sums, no second kernel) the kernel
// beats the strip kernel with its slice sum (config 2: 19 against 25 + 5.5 us); with channel slices
// and the slice sum it still beats the register-tile and strip kernels where the encoder of a
// one-call layer leaves the column table - the workgroup-per-channel encoder, which at these batch
// sizes takes every layer this kernel supports (one-call layers: 128 @ 28 30.5 -> 23.5 us,
// 256 @ 14 28.7 -> 23.4, 3 x 3 stride 2 128 @ 56 39.7 -> 27.5, 5 x 5 38.3 -> 27.3).  From four images
// on the strip kernel's shared decode wins.
bool runs_kernel_preferred(const Geometry &g)
{
    return runs_kernel_supports(g) && g.N < 4 && (runs_plan(g).slices == 1 || encode_uses_channel_kernel(g));
}

int64_t runs_kernel_partial_bytes(const Geometry &g)
{
    if (!runs_kernel_supports(g)) return 0;
    const RunsPlan p = runs_plan(g);
    if (p.slices == 1) return 0;
    const int64_t Ypad = (g.Oh + p.ty - 1) / p.ty * p.ty, Xpad = (g.Ow + p.tx - 1) / p.tx * p.tx;
    return 4 * Ypad * Xpad * g.Kpad * p.slices * g.N;
}

int64_t runs_kernel_columns_bytes(const Geometry &g)
{
    if (!runs_kernel_preferred(g)) return 0;
    return (static_cast<int64_t>(sizeof(ColumnEntry)) * columns_stride(g) * g.N + 255) / 256 * 256;
}

// mtab: the table of resolved ptr offsets if a kernel before this one has left it, else nullptr
// (then the kernel resolves ptr itself)
// cps: the map's IN stream is the packed one of Algorithm 3 (decoded in the kernel)
int launch_column_table(const cpoconv_map &map, const int32_t *mtab, ColumnEntry *columns, const Geometry &g, BatchStrides bs,
                        bool cps, hipStream_t stream)
{
    bs.indices = map.in_cap;
    bs.indices16 = bs.map_in16;
    // a lane per packed entry / a wavefront per column: enough wavefronts for one or two rounds
    const int threads = std::min(kTableThreads, std::max(256, (g.H * g.W / 2 + kLanes - 1) / kLanes * kLanes));
    KernelTimer timer("column_table", stream);
    hipLaunchKernelGGL(column_table_kernel, dim3(g.C, g.N), dim3(threads), 0, stream, g, map.ptr, map.chan_off, map.in,
                       mtab, columns, bs, cps ? g.top_slot : -1);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

int launch_sparse_conv_runs(const cpoconv_map &map, const ColumnEntry *columns, const Geometry &g, const float *wt, float *out,
                            float *partial, BatchStrides bs, hipStream_t stream)
{
    const RunsPlan p = runs_plan(g);
    const RunsShape *shape = runs_shape(g);
    if (shape == nullptr) return CPOCONV_ERR_SHAPE;
#define CPOCONV_RUNS(KH, KW, S, TY, TX)                                                                                  \
    if (g.kh == KH && g.kw == KW && g.stride == S)                                                                      \
        return p.kpl == 2 ? launch_runs<KH, KW, S, TY, TX, 2, kMaxWaves>(map, columns, g, wt, out, partial, p, bs, stream) \
                          : launch_runs<KH, KW, S, TY, TX, 1, kMaxWaves>(map, columns, g, wt, out, partial, p, bs, stream);
    CPOCONV_RUNS(3, 3, 1, 4, 4)
    CPOCONV_RUNS(3, 3, 2, 3, 3)
    CPOCONV_RUNS(1, 7, 1, 8, 2)
    CPOCONV_RUNS(7, 1, 1, 2, 8)
    CPOCONV_RUNS(1, 3, 1, 4, 4)
    CPOCONV_RUNS(3, 1, 1, 4, 4)
#undef CPOCONV_RUNS
    if (g.kh == 5) return launch_runs<5, 5, 1, 4, 4, 1, kMaxWaves>(map, columns, g, wt, out, partial, p, bs, stream);
    return CPOCONV_ERR_SHAPE;
}

}  // namespace cpoconv
