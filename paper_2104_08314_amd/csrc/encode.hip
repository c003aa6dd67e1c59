// CPO / CPS encoders (Algorithms 1 and 3) as a stream compaction.
//
// The sequential algorithms append NZEs while walking channel -> overlap type -> partition ->
// column -> row, so the position of every NZE in DA / IN is "number of NZEs visited before
// it".  Here one workgroup owns one channel and stages it in LDS with coalesced row reads.
//   counts   one thread per column (in stream order) walks its column down the rows and builds
//            the column's NZE bitmap: its popcount is the column count; for CPS columns of the
//            overlap-kw type, min(NZEs, 2) per group of four rows is the number of IN entries.
//   offsets  a prefix sum over the columns in stream order gives every column's start in DA
//            and IN, the cumulative entries of ptr and the channel totals.
//   scatter  each wavefront takes whole columns with lane = padded row: a ballot rebuilds the
//            bitmap, the popcount of the lower lanes is the rank of an NZE inside its column,
//            so a column is written as one contiguous, coalesced run.
// One launch: a channel's position in the packed streams is the sum of the lengths of the
// channels before it, so every workgroup publishes its three lengths in the scratch buffer and
// reads those of its predecessors (a look-back over individual lengths, not a chain).  The
// lengths travel inside 64-bit atomics tagged with the call's epoch - no other memory is
// communicated, so no fence is needed - and the wait on a predecessor is bounded: a workgroup
// that gives up writes nothing and raises hdr[7].  Workgroups only ever wait for lower block
// indices, which the hardware dispatches first.  All of it is integer / bit work on the fp32 bit
// patterns: outputs are exact.
#include "common.hpp"

#include <algorithm>

namespace cpoconv {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kLanes;
// Padded rows handled per pass (lane = row inside the chunk): 64, a multiple of 4, so a set4 never
// straddles chunks.  The widest map's chunk (64 rows of 257 floats) takes 66 KB of LDS; chunks of 32
// rows for wide maps kept the tile within 40 KB but made the 224 x 224 map twice as many passes
// (104 -> 72 us at three channels).
constexpr int kMaxChunks = (CPOCONV_MAX_I + kLanes - 1) / kLanes;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x / kLanes; }

__device__ __forceinline__ bool is_nze(float v)
{
    // +0 and -0 are zeros; denormals and NaN are not (bit test: no flush-to-zero dependence)
    return (__float_as_uint(v) & 0x7fffffffu) != 0u;
}

// inclusive sum over the 64 lanes: shifts inside rows of 16 lanes, then the last lane of a row
// added to the rows after it
__device__ __forceinline__ int wave_inclusive_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
    return v;
}

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int d = kLanes / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kLanes);
    return v;
}

// IN entries of one column chunk under Algorithm 3: per group of four rows min(NZEs, 2).
__device__ __forceinline__ int set4_entries(unsigned long long mask)
{
    int n = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) n += min(__popc(static_cast<unsigned>(mask >> (4 * q)) & 0xFu), 2);
    return n;
}

// Scratch words of the look-back (unsigned 64-bit): [8 + n] the epoch of image slot n,
// incremented by the workgroup of the last channel once its own look-back is complete (every
// channel before it has then published, hence started and read the epoch); from word kCtrlWords
// on, two words per (image, channel): {tag, |DA|} and {tag, |IN| + (|ptr| << 17)}, at a position
// that does not depend on the layer (image * 512 + channel), so a word is only ever tagged from
// one epoch counter.  tag = epoch % (2^32 - 2) + 1 of the call that wrote the word: never 0, the
// initial state, and never 2^32 - 1, which marks lengths published by a separate launch.
constexpr int kCtrlWords = 8 + CPOCONV_MAX_BATCH;
constexpr unsigned long long kTagTwoLaunches = 0xFFFFFFFFull;
// Every workgroup reads C/2 lengths past the caches, C*C/2 loads in all: up to 512 channels that is
// cheaper than a second launch (measured: 4 us saved at 128 channels, 1.5 us at 512).  Beyond, a
// first launch only publishes the lengths and the second reads them as ordinary data.
constexpr int kSinglePassChannels = 512;
enum EncodeMode { kSinglePass = 0, kPublishOnly = 1, kPublished = 2 };
constexpr int kSpinLimit = 1 << 14;   // polls of one predecessor before the encoder gives up

__device__ __forceinline__ unsigned long long peek(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void poke(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int kMode>
__global__ __launch_bounds__(kThreads) void encode_kernel(const Geometry g, const float *__restrict__ act_all,
                                                         const Producer prod, const int cps, const int kChunk,
                                                         unsigned long long *__restrict__ ctrl, const cpoconv_map maps,
                                                         int32_t *__restrict__ mtab_all, const int64_t mtab_stride,
                                                         int32_t *__restrict__ full_all, const int64_t full_stride)
{
    // image blockIdx.y of the launch: its map is image 0's advanced by the per-image capacities
    const int image = blockIdx.y;
    const float *__restrict__ act = act_all + static_cast<int64_t>(image) * g.C * g.H * g.W;
    const unsigned long long epoch = kMode == kSinglePass ? peek(ctrl + 8 + image) : 0ull;
    const unsigned long long tag = kMode == kSinglePass ? epoch % 0xFFFFFFFEull + 1ull : kTagTwoLaunches;
    unsigned long long *flags = ctrl + kCtrlWords +
                                2 * static_cast<int64_t>(image) * (kMode == kSinglePass ? kSinglePassChannels : g.C);
    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    const int in16 = maps.in_bits == 16 ? 1 : 0;
    map.in = index_advance(maps.in, image * maps.in_cap, in16);
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;
    // for a CPS convolution launched by the same call: the plain index of every NZE, laid out like DA
    int32_t *__restrict__ full = full_all != nullptr ? full_all + image * full_stride : nullptr;

    extern __shared__ float tile[];                    // kChunk x Wt, Wt odd: conflict-free column reads
    __shared__ uint16_t cnt_q[kMaxChunks][kMaxCols];   // NZEs per (row chunk, column), then their
    __shared__ uint16_t ecnt_q[kMaxChunks][kMaxCols];  //   exclusive sums over the chunks; same for IN
    __shared__ int32_t col_excl[kMaxCols + 1];         // NZEs of the channel before each column
    __shared__ int32_t ecol_excl[kMaxCols + 1];        // IN entries of the channel before each column
    __shared__ uint8_t col_jr[kMaxCols], col_p0[kMaxCols], col_wh[kMaxCols];  // geometry, per column
    __shared__ int32_t tbl[kMaxCols];                  // one ptr segment under construction
    __shared__ int32_t type_base[kMaxTypes + 1];       // NZEs of the channel before each type
    __shared__ int32_t wave_tot[2][kWaves];
    __shared__ uint8_t mask_part[kMaxCols][kWaves];    // a column's row bitmap in pieces, one per wavefront
    __shared__ int32_t chan_base[4];                   // ptr / DA / IN start of the channel, look-back failures

    const int c = blockIdx.x;
    const int lane = lane_id(), wave = wave_id(), tid = threadIdx.x;
    const int Wt = g.W | 1;
    const int nchunks = (g.Ih + kChunk - 1) / kChunk;
    const int top_begin = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot] : kMaxCols + 1;
    const int top_end = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot + 1] : 0;
    const float *chan = act + static_cast<int64_t>(c) * g.H * g.W;
    const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;

    auto load_tile = [&](int q) {
        for (int r = wave; r < kChunk; r += kWaves) {
            const int hr = q * kChunk + r - g.pad_h;
            if (hr < 0 || hr >= g.H) continue;
            for (int jr = lane; jr < g.W; jr += kLanes) tile[r * Wt + jr] = produced(chan[hr * g.W + jr], prod, bias_c);
        }
    };

    // the tile's loads first, then everything that does not depend on them
    load_tile(0);
    if (tid < g.n_cols) {
        col_jr[tid] = static_cast<uint8_t>(g.col_j[tid] - g.pad_w);
        col_p0[tid] = g.col_p0[tid];
        col_wh[tid] = g.col_what[tid];
    }
    if (tid < 4) chan_base[tid] = 0;
    if (kMode != kPublishOnly && tid == 0 && c == 0) map.hdr[7] = 0;   // raised by a workgroup that gives up its look-back
    __syncthreads();

    // ---- counts: every wavefront takes kChunk / 8 rows of the chunk (lane = column in stream
    // order) and leaves its part of every column's row bitmap in LDS; one thread per column then
    // puts the eight parts together ------------------------------------------------------------
    const int rows_per_wave = kChunk / kWaves;   // 8
    for (int q = 0; q < nchunks; ++q) {
        if (q > 0) {
            __syncthreads();   // every thread is done with the previous chunk
            load_tile(q);
            __syncthreads();
        }
        for (int vi = lane; vi < g.n_cols; vi += kLanes) {
            const int jr = col_jr[vi];
            unsigned bits = 0;
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) {
                const int r = wave * rows_per_wave + rr, hr = q * kChunk + r - g.pad_h;
                if (rr < rows_per_wave && hr >= 0 && hr < g.H) bits |= static_cast<unsigned>(is_nze(tile[r * Wt + jr])) << rr;
            }
            mask_part[vi][wave] = static_cast<uint8_t>(bits);
        }
        __syncthreads();
        if (tid < g.n_cols) {
            unsigned long long mask = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w)
                mask |= static_cast<unsigned long long>(mask_part[tid][w]) << (w * rows_per_wave);
            cnt_q[q][tid] = static_cast<uint16_t>(__popcll(mask));
            ecnt_q[q][tid] = static_cast<uint16_t>((tid >= top_begin && tid < top_end) ? set4_entries(mask)
                                                                                      : __popcll(mask));
        }
    }

    // ---- offsets: exclusive sums over the chunks of a column, then over the columns ------------
    {
        int n = 0, e = 0;
        if (tid < g.n_cols)
            for (int q = 0; q < nchunks; ++q) {
                const int cn = cnt_q[q][tid], ce = ecnt_q[q][tid];
                cnt_q[q][tid] = static_cast<uint16_t>(n);
                ecnt_q[q][tid] = static_cast<uint16_t>(e);
                n += cn;
                e += ce;
            }
        const int ni = wave_inclusive_sum(n), ei = wave_inclusive_sum(e);
        if (lane == kLanes - 1) { wave_tot[0][wave] = ni; wave_tot[1][wave] = ei; }
        __syncthreads();
        int nb = 0, eb = 0;
        for (int w = 0; w < wave; ++w) { nb += wave_tot[0][w]; eb += wave_tot[1][w]; }
        if (tid < kMaxCols) { col_excl[tid + 1] = nb + ni; ecol_excl[tid + 1] = eb + ei; }
        if (tid == 0) { col_excl[0] = 0; ecol_excl[0] = 0; }
    }
    __syncthreads();
    if (tid <= g.n_types) type_base[tid] = col_excl[g.type_begin[tid]];
    __syncthreads();
    const int nnz_c = col_excl[g.n_cols];
    const int in_c = ecol_excl[g.n_cols];
    int ptr_c = 1;  // NPC
    if (nnz_c > 0) {
        ptr_c = 0;
        for (int i = 0; i < g.n_types; ++i) {
            if (g.nop3 && g.type_id[i] == 0) ptr_c += 3;
            else ptr_c += (type_base[i + 1] > type_base[i]) ? 1 + g.Ow : 1;
        }
    }

    // ---- look-back: publish this channel's lengths, add up those of the channels before it --------
    if (kMode != kPublished && tid == 0) {
        poke(flags + 2 * c, (tag << 32) | static_cast<unsigned>(nnz_c));
        poke(flags + 2 * c + 1, (tag << 32) | static_cast<unsigned>(in_c) | (static_cast<unsigned>(ptr_c) << 17));
    }
    if (kMode == kPublishOnly) return;
    {
        int a0 = 0, a1 = 0, a2 = 0, failed = 0;
        for (int cc = tid; cc < c; cc += kThreads) {
            unsigned long long w0, w1;
            if (kMode == kPublished) {   // written by the launch before this one: ordinary loads
                w0 = flags[2 * cc];
                w1 = flags[2 * cc + 1];
            } else {
                w0 = peek(flags + 2 * cc);
                w1 = peek(flags + 2 * cc + 1);
                for (int spin = 0; ((w0 >> 32) != tag || (w1 >> 32) != tag) && spin < kSpinLimit; ++spin) {
                    __builtin_amdgcn_s_sleep(8);
                    w0 = peek(flags + 2 * cc);
                    w1 = peek(flags + 2 * cc + 1);
                }
            }
            if ((w0 >> 32) != tag || (w1 >> 32) != tag) { failed = 1; break; }
            a1 += static_cast<int>(w0 & 0xFFFFFFFFull);
            a2 += static_cast<int>(w1 & 0x1FFFFull);
            a0 += static_cast<int>((w1 >> 17) & 0x7FFFull);
        }
        a0 = wave_sum(a0); a1 = wave_sum(a1); a2 = wave_sum(a2); failed = wave_sum(failed);
        if (lane == 0) {
            atomicAdd(&chan_base[0], a0);
            atomicAdd(&chan_base[1], a1);
            atomicAdd(&chan_base[2], a2);
            atomicAdd(&chan_base[3], failed);
        }
    }
    __syncthreads();
    // the last channel has seen every other channel's lengths, so all of them have read the epoch:
    // it may move on (one writer per image; the next call is ordered after this launch)
    if (kMode == kSinglePass && tid == 0 && c == g.C - 1 && chan_base[3] == 0) poke(ctrl + 8 + image, epoch + 1ull);
    if (chan_base[3] != 0) {   // a predecessor never showed up (scratch not initialised?): write nothing
        if (tid == 0) atomicOr(&map.hdr[7], 1);
        return;
    }

    const int ptr_off = chan_base[0], da_off = chan_base[1], in_off = chan_base[2];
    if (tid == 0) {
        map.chan_off[c] = ptr_off;
        map.chan_off[(g.C + 1) + c] = da_off;
        map.chan_off[2 * (g.C + 1) + c] = in_off;
        if (c == g.C - 1) {
            map.chan_off[g.C] = ptr_off + ptr_c;
            map.chan_off[(g.C + 1) + g.C] = da_off + nnz_c;
            map.chan_off[2 * (g.C + 1) + g.C] = in_off + in_c;
            map.hdr[0] = ptr_off + ptr_c;
            map.hdr[1] = da_off + nnz_c;
            map.hdr[2] = in_off + in_c;
            map.hdr[3] = cps ? CPOCONV_ALGO_CPS : CPOCONV_ALGO_CPO;
            map.hdr[4] = g.C;
            map.hdr[5] = g.Ow;
            map.hdr[6] = in16 ? 16 : 32;
        }
    }

    // ---- for a convolution that follows in the same call: the table of absolute DA offsets after
    // every partition (what Algorithm 2 gets by forward-filling ptr), per present type ----------
    if (mtab_all != nullptr) {
        for (int i = 0; i < g.n_types; ++i) {
            int32_t *row = mtab_all + image * mtab_stride + (static_cast<int64_t>(c) * g.n_types + i) * (g.Ow + 1);
            const int cb = g.type_begin[i], ce = g.type_begin[i + 1];
            const int base = type_base[i], at = da_off + base;
            const int p_first = cb < ce ? col_p0[cb] : g.Ow;        // partitions before it hold nothing of the type
            for (int k = tid; k <= p_first; k += kThreads) row[k] = at;
            for (int vi = cb + tid; vi < ce; vi += kThreads) {
                const int p_end = vi + 1 < ce ? col_p0[vi + 1] : g.Ow;
                const int upto = at + col_excl[vi + 1] - base;
                for (int pp = col_p0[vi]; pp < p_end; ++pp) row[1 + pp] = upto;
            }
        }
    }

    // ---- ptr of this channel -------------------------------------------------------------
    if (nnz_c == 0) {
        if (tid == 0) map.ptr[ptr_off] = CPOCONV_NPC;
        return;  // nothing to write to DA / IN
    }
    {
        int seg = ptr_off;
        for (int i = 0; i < g.n_types; ++i) {
            const int cb = g.type_begin[i], ce = g.type_begin[i + 1];
            const int base = type_base[i];
            if (g.nop3 && g.type_id[i] == 0) {
                // [0, NZEs of the first column, NZEs of first + last column]
                if (tid == 0) map.ptr[seg] = 0;
                if (tid >= 1 && tid <= 2) map.ptr[seg + tid] = col_excl[min(cb + tid, ce)] - base;
                seg += 3;
                continue;
            }
            if (type_base[i + 1] == base) {
                if (tid == 0) map.ptr[seg] = CPOCONV_NPF;
                seg += 1;
                continue;
            }
            for (int p = tid; p < g.Ow; p += kThreads) tbl[p] = -1;
            __syncthreads();
            // cumulative count after the last column first seen in each partition
            for (int vi = cb + tid; vi < ce; vi += kThreads)
                if (vi + 1 == ce || col_p0[vi + 1] != col_p0[vi]) tbl[col_p0[vi]] = col_excl[vi + 1] - base;
            __syncthreads();
            if (tid == 0) map.ptr[seg] = g.type_id[i];
            for (int p = tid; p < g.Ow; p += kThreads) map.ptr[seg + 1 + p] = tbl[p];
            __syncthreads();
            seg += 1 + g.Ow;
        }
    }

    // ---- scatter DA and IN: one wavefront per column, lane = padded row -----------------------
    for (int q = nchunks - 1; q >= 0; --q) {   // the last chunk is still in LDS
        if (q != nchunks - 1) {
            __syncthreads();
            load_tile(q);
            __syncthreads();
        }
        const int hr = q * kChunk + lane - g.pad_h;
        const bool row_ok = lane < kChunk && hr >= 0 && hr < g.H;
        const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll 2
        for (int vi = wave; vi < g.n_cols; vi += kWaves) {
            const float v = row_ok ? tile[lane * Wt + col_jr[vi]] : 0.0f;
            const bool nz = is_nze(v);
            const unsigned long long mask = __ballot(nz);
            const int rank = __popcll(mask & below);
            const int da_at = da_off + col_excl[vi] + cnt_q[q][vi];
            const int in_at = in_off + ecol_excl[vi] + ecnt_q[q][vi];
            const int index = static_cast<int>(col_wh[vi]) + (q * kChunk + lane) * g.kw;
            if (nz) map.da[da_at + rank] = v;
            if (nz && full != nullptr) full[da_at + rank] = index;
            if (vi >= top_begin && vi < top_end) {
                // set4 of Algorithm 3: the four padded rows 4*(h/4) .. +3
                const int pattern = static_cast<int>((mask >> (lane & ~3)) & 0xFull);
                const int r = __popc(pattern & ((1 << (lane & 3)) - 1));   // rank inside the set
                const bool emit = nz && r < 2;
                const int erank = __popcll(__ballot(emit) & below);
                // first NZE of the set: its index (negated unless a pattern follows);
                // second NZE: the pattern, or its own negated index
                const int entry = __popc(pattern) >= 3 ? (r == 0 ? index : pattern) : -index;
                if (emit) store_index(map.in, in_at + erank, entry, in16);
            } else {
                if (nz) store_index(map.in, in_at + rank, index, in16);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The same encoder for small maps (padded height and width up to 64, the unpadded map within 4 KiB):
// one WAVEFRONT per channel, eight channels per workgroup.  A 14 x 14 or 7 x 7 map keeps a
// 512-thread workgroup idle almost everywhere; here every step of a channel is a wavefront-wide
// operation without workgroup barriers (column bitmaps with lane = column, prefix sums and type
// bases by lane exchange, scatter with several columns per pass when the map has 32 or 16 rows).
// Only the look-back is shared: the workgroup publishes its eight channels' lengths, all 512
// threads read the channels before the group, and each wavefront adds its neighbours' lengths.
// ---------------------------------------------------------------------------------------------
constexpr int kSmallTileBytes = 4096;
// padded maps up to this many elements always take the one-wavefront-per-channel kernel; larger
// ones from this many channel-images on (four 512-thread workgroups fit a compute unit, 256 units)
constexpr int kSmallAlways = 18 * 18;
constexpr int64_t kSmallFromChannels = 1024;

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int kMode>
__global__ __launch_bounds__(kThreads) void encode_small_kernel(const Geometry g, const float *__restrict__ act_all,
                                                               const Producer prod, const int cps,
                                                               unsigned long long *__restrict__ ctrl,
                                                               const cpoconv_map maps, int32_t *__restrict__ mtab_all,
                                                               const int64_t mtab_stride, int32_t *__restrict__ full_all,
                                                               const int64_t full_stride)
{
    extern __shared__ float tiles[];                   // per wavefront: H x Wt floats, then 64 ints of ptr staging
    __shared__ int32_t grp[kWaves][3];                 // the group's lengths: ptr, DA, IN per channel
    __shared__ int32_t grp_base[4];                    // lengths of the channels before the group; failures

    const int image = blockIdx.y;
    const int lane = lane_id(), tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(wave_id());
    const int c0 = blockIdx.x * kWaves, c = c0 + wave;
    const bool live = c < g.C;                         // wavefronts past the last channel only help with the look-back
    const float *__restrict__ act = act_all + static_cast<int64_t>(image) * g.C * g.H * g.W;
    const unsigned long long epoch = kMode == kSinglePass ? peek(ctrl + 8 + image) : 0ull;
    const unsigned long long tag = kMode == kSinglePass ? epoch % 0xFFFFFFFEull + 1ull : kTagTwoLaunches;
    unsigned long long *flags = ctrl + kCtrlWords +
                                2 * static_cast<int64_t>(image) * (kMode == kSinglePass ? kSinglePassChannels : g.C);
    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    const int in16 = maps.in_bits == 16 ? 1 : 0;
    map.in = index_advance(maps.in, image * maps.in_cap, in16);
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;
    int32_t *__restrict__ full = full_all != nullptr ? full_all + image * full_stride : nullptr;

    const int Wt = g.W | 1;
    const int per_wave = g.H * Wt + kLanes;            // floats of LDS per wavefront
    float *tile = tiles + wave * per_wave;
    int32_t *tblw = reinterpret_cast<int32_t *>(tile + g.H * Wt);
    const int top_begin = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot] : kMaxCols + 1;
    const int top_end = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot + 1] : 0;

    if (tid < 4) grp_base[tid] = 0;
    if (kMode != kPublishOnly && tid == 0 && c0 == 0) map.hdr[7] = 0;

    // ---- the channel into LDS (coalesced), then its column bitmaps: lane = column in stream order ----
    if (live) {
        const float *chan = act + static_cast<int64_t>(c) * g.H * g.W;
        const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;
        for (int i = lane; i < g.H * g.W; i += kLanes) {
            const int r = i / g.W;
            tile[r * Wt + (i - r * g.W)] = produced(chan[i], prod, bias_c);
        }
    }
    wave_lds_fence();
    const bool col_ok = live && lane < g.n_cols;
    const int my_jr = col_ok ? static_cast<int>(g.col_j[lane]) - g.pad_w : 0;
    const int my_p0 = col_ok ? static_cast<int>(g.col_p0[lane]) : 0;
    const int next_p0 = (live && lane + 1 < g.n_cols) ? static_cast<int>(g.col_p0[lane + 1]) : -1;
    unsigned long long colmask = 0;
    if (col_ok)
        for (int r = 0; r < g.H; ++r)
            colmask |= static_cast<unsigned long long>(is_nze(tile[r * Wt + my_jr])) << (r + g.pad_h);   // bit = padded row
    const int cnt = __popcll(colmask);
    const int ecnt = (lane >= top_begin && lane < top_end) ? set4_entries(colmask) : cnt;
    const int incl = wave_inclusive_sum(cnt), eincl = wave_inclusive_sum(ecnt);
    const int excl = incl - cnt, eexcl = eincl - ecnt;
    const int nnz_c = __builtin_amdgcn_readlane(incl, kLanes - 1), in_c = __builtin_amdgcn_readlane(eincl, kLanes - 1);
    int type_base[kMaxTypes + 1];
#pragma unroll
    for (int i = 0; i <= kMaxTypes; ++i) {
        type_base[i] = nnz_c;
        if (i <= g.n_types) {
            const int b = g.type_begin[i];
            if (b < g.n_cols) type_base[i] = __builtin_amdgcn_readlane(excl, b);
        }
    }
    int ptr_c = 1;  // NPC
    if (nnz_c > 0) {
        ptr_c = 0;
#pragma unroll
        for (int i = 0; i < kMaxTypes; ++i) {
            if (i >= g.n_types) continue;
            if (g.nop3 && g.type_id[i] == 0) ptr_c += 3;
            else ptr_c += (type_base[i + 1] > type_base[i]) ? 1 + g.Ow : 1;
        }
    }

    // ---- look-back, shared by the workgroup -----------------------------------------------------
    if (lane == 0) {
        grp[wave][0] = live ? ptr_c : 0;
        grp[wave][1] = live ? nnz_c : 0;
        grp[wave][2] = live ? in_c : 0;
        if (kMode != kPublished && live) {
            poke(flags + 2 * c, (tag << 32) | static_cast<unsigned>(nnz_c));
            poke(flags + 2 * c + 1, (tag << 32) | static_cast<unsigned>(in_c) | (static_cast<unsigned>(ptr_c) << 17));
        }
    }
    if (kMode == kPublishOnly) return;
    __syncthreads();   // grp and grp_base written
    {
        int a0 = 0, a1 = 0, a2 = 0, failed = 0;
        for (int cc = tid; cc < c0; cc += kThreads) {
            unsigned long long w0, w1;
            if (kMode == kPublished) {
                w0 = flags[2 * cc];
                w1 = flags[2 * cc + 1];
            } else {
                w0 = peek(flags + 2 * cc);
                w1 = peek(flags + 2 * cc + 1);
                for (int spin = 0; ((w0 >> 32) != tag || (w1 >> 32) != tag) && spin < kSpinLimit; ++spin) {
                    __builtin_amdgcn_s_sleep(8);
                    w0 = peek(flags + 2 * cc);
                    w1 = peek(flags + 2 * cc + 1);
                }
            }
            if ((w0 >> 32) != tag || (w1 >> 32) != tag) { failed = 1; break; }
            a1 += static_cast<int>(w0 & 0xFFFFFFFFull);
            a2 += static_cast<int>(w1 & 0x1FFFFull);
            a0 += static_cast<int>((w1 >> 17) & 0x7FFFull);
        }
        a0 = wave_sum(a0); a1 = wave_sum(a1); a2 = wave_sum(a2); failed = wave_sum(failed);
        if (lane == 0) {
            atomicAdd(&grp_base[0], a0);
            atomicAdd(&grp_base[1], a1);
            atomicAdd(&grp_base[2], a2);
            atomicAdd(&grp_base[3], failed);
        }
    }
    __syncthreads();
    const bool failed = grp_base[3] != 0;
    // the last channel's group has seen every other channel's lengths: the epoch may move on
    if (kMode == kSinglePass && tid == 0 && c0 + kWaves >= g.C && !failed) poke(ctrl + 8 + image, epoch + 1ull);
    if (failed) {
        if (tid == 0) atomicOr(&map.hdr[7], 1);
        return;
    }
    if (!live) return;
    int ptr_off = grp_base[0], da_off = grp_base[1], in_off = grp_base[2];
    for (int w = 0; w < wave; ++w) { ptr_off += grp[w][0]; da_off += grp[w][1]; in_off += grp[w][2]; }

    if (lane == 0) {
        map.chan_off[c] = ptr_off;
        map.chan_off[(g.C + 1) + c] = da_off;
        map.chan_off[2 * (g.C + 1) + c] = in_off;
        if (c == g.C - 1) {
            map.chan_off[g.C] = ptr_off + ptr_c;
            map.chan_off[(g.C + 1) + g.C] = da_off + nnz_c;
            map.chan_off[2 * (g.C + 1) + g.C] = in_off + in_c;
            map.hdr[0] = ptr_off + ptr_c;
            map.hdr[1] = da_off + nnz_c;
            map.hdr[2] = in_off + in_c;
            map.hdr[3] = cps ? CPOCONV_ALGO_CPS : CPOCONV_ALGO_CPO;
            map.hdr[4] = g.C;
            map.hdr[5] = g.Ow;
            map.hdr[6] = in16 ? 16 : 32;
        }
    }

    // ---- the table of absolute DA offsets after every partition, for a convolution of the same call ----
    if (mtab_all != nullptr) {
#pragma unroll
        for (int i = 0; i < kMaxTypes; ++i) {
            if (i >= g.n_types) continue;
            int32_t *row = mtab_all + image * mtab_stride + (static_cast<int64_t>(c) * g.n_types + i) * (g.Ow + 1);
            const int cb = g.type_begin[i], ce = g.type_begin[i + 1];
            const int at = da_off + type_base[i];
            const int p_first = cb < ce ? static_cast<int>(g.col_p0[cb]) : g.Ow;
            for (int k = lane; k <= p_first; k += kLanes) row[k] = at;
            if (lane >= cb && lane < ce) {
                const int p_end = lane + 1 < ce ? next_p0 : g.Ow;
                const int upto = da_off + incl;
                for (int pp = my_p0; pp < p_end; ++pp) row[1 + pp] = upto;
            }
        }
    }

    // ---- ptr ----------------------------------------------------------------------------------------
    if (nnz_c == 0) {
        if (lane == 0) map.ptr[ptr_off] = CPOCONV_NPC;
        return;
    }
    {
        int seg = ptr_off;
#pragma unroll
        for (int i = 0; i < kMaxTypes; ++i) {
            if (i >= g.n_types) continue;
            const int cb = g.type_begin[i], ce = g.type_begin[i + 1];
            const int base = type_base[i];
            if (g.nop3 && g.type_id[i] == 0) {
                // [0, NZEs of the first column, NZEs of first + last column]
                const int n1 = __builtin_amdgcn_readlane(incl, min(cb, kLanes - 1)) - base;
                const int n2 = __builtin_amdgcn_readlane(incl, min(max(ce - 1, cb), kLanes - 1)) - base;
                if (lane == 0) { map.ptr[seg] = 0; map.ptr[seg + 1] = n1; map.ptr[seg + 2] = n2; }
                seg += 3;
                continue;
            }
            if (type_base[i + 1] == base) {
                if (lane == 0) map.ptr[seg] = CPOCONV_NPF;
                seg += 1;
                continue;
            }
            tblw[lane] = -1;
            wave_lds_fence();
            // cumulative count after the last column first seen in each partition
            if (lane >= cb && lane < ce && (lane + 1 == ce || next_p0 != my_p0)) tblw[my_p0] = incl - base;
            wave_lds_fence();
            if (lane == 0) map.ptr[seg] = g.type_id[i];
            if (lane < g.Ow) map.ptr[seg + 1 + lane] = tblw[lane];
            wave_lds_fence();
            seg += 1 + g.Ow;
        }
    }

    // ---- scatter DA and IN: lane = (column of the pass, padded row); 1, 2 or 4 columns per pass -----
    const int rows_pass = g.Ih <= 16 ? 16 : (g.Ih <= 32 ? 32 : 64);
    const int cols_pass = kLanes / rows_pass;
    const int sub = lane / rows_pass, h = lane - sub * rows_pass;     // h: padded row
    const unsigned long long sub_bits = rows_pass == 64 ? ~0ull : ((1ull << rows_pass) - 1ull);
    const unsigned long long below = (1ull << h) - 1ull;
    const int hr = h - g.pad_h;
    const bool row_ok = hr >= 0 && hr < g.H;
    for (int v0 = 0; v0 < g.n_cols; v0 += cols_pass) {
        const int vi = v0 + sub;
        const bool on = vi < g.n_cols;
        const int src = on ? vi : 0;
        const int jr = __shfl(my_jr, src, kLanes);
        const int at_da = da_off + __shfl(excl, src, kLanes), at_in = in_off + __shfl(eexcl, src, kLanes);
        const int what = on ? static_cast<int>(g.col_what[vi]) : 0;
        const float v = (on && row_ok) ? tile[hr * Wt + jr] : 0.0f;
        const bool nz = is_nze(v);
        const unsigned long long all = __ballot(nz);
        const unsigned long long mask = (all >> (sub * rows_pass)) & sub_bits;
        const int rank = __popcll(mask & below);
        const int index = what + h * g.kw;
        if (nz) map.da[at_da + rank] = v;
        if (nz && full != nullptr) full[at_da + rank] = index;
        const bool packed = on && vi >= top_begin && vi < top_end;
        // set4 of Algorithm 3: the four padded rows 4*(h/4) .. +3
        const int pattern = static_cast<int>((mask >> (h & ~3)) & 0xFull);
        const int r = __popc(pattern & ((1 << (h & 3)) - 1));   // rank inside the set
        const bool emit = packed && nz && r < 2;
        const unsigned long long emits = (__ballot(emit) >> (sub * rows_pass)) & sub_bits;
        const int erank = __popcll(emits & below);
        const int entry = __popc(pattern) >= 3 ? (r == 0 ? index : pattern) : -index;
        if (packed) {
            if (emit) store_index(map.in, at_in + erank, entry, in16);
        } else if (nz) {
            store_index(map.in, at_in + rank, index, in16);
        }
    }
}

// zero fill of a scratch buffer (a kernel rather than a memset node, so that a caller may capture
// the call in a graph)
__global__ __launch_bounds__(256) void zero_fill_kernel(uint32_t *__restrict__ words, const int64_t n_words,
                                                       unsigned char *__restrict__ tail, const int n_tail)
{
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < n_words;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x)
        words[i] = 0u;
    if (blockIdx.x == 0 && static_cast<int>(threadIdx.x) < n_tail) tail[threadIdx.x] = 0;
}

__global__ __launch_bounds__(256) void prepare_weights_kernel(const Geometry g, const float *__restrict__ w,
                                                             float *__restrict__ wt)
{
    // wt[c][l][x][k] = w[k][c][l][x], kernel index fastest, zero beyond K
    const int64_t total = static_cast<int64_t>(g.C) * g.kh * g.kw * g.Kpad;
    const int taps = g.C * g.kh * g.kw;
    for (int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int k = static_cast<int>(i % g.Kpad);
        const int tap = static_cast<int>(i / g.Kpad);
        wt[i] = k < g.K ? w[static_cast<int64_t>(k) * taps + tap] : 0.0f;
    }
}

}  // namespace

int launch_encode(const float *act, const Producer &prod, const Geometry &g, const cpoconv_map &map, int algo,
                  void *scratch, hipStream_t stream, bool write_table, bool write_indices)
{
    // the plain per-NZE indices, for a CPS convolution launched by the same call (same place and
    // layout as the convolution's own reconstruction would leave them)
    int32_t *full = write_indices ? reinterpret_cast<int32_t *>(static_cast<char *>(scratch) + scratch_counts_bytes(g) +
                                                                scratch_mtab_bytes(g))
                                  : nullptr;
    const int64_t fstride = indices_stride(g);
    // the table of resolved ptr offsets, for a convolution launched by the same call
    int32_t *mtab = write_table ? reinterpret_cast<int32_t *>(static_cast<char *>(scratch) + scratch_counts_bytes(g)) : nullptr;
    const int64_t mstride = mtab_stride(g);
    const int cps = algo == CPOCONV_ALGO_CPS ? 1 : 0;
    const size_t row_bytes = static_cast<size_t>(g.W | 1) * sizeof(float);
    const int chunk = kLanes;
    const size_t lds = chunk * row_bytes;
    unsigned long long *ctrl = static_cast<unsigned long long *>(scratch);
    const size_t small_tile = static_cast<size_t>(g.H) * (g.W | 1) * sizeof(float);
    // A wavefront walks its channel's rows alone, which costs latency on the larger of the small maps:
    // those take the path only once workgroups of the other kernel would queue for a compute unit.
    const bool worth = g.Ih * g.Iw <= kSmallAlways || static_cast<int64_t>(g.N) * g.C >= kSmallFromChannels;
    if (g.Ih <= kLanes && g.Iw <= kLanes && small_tile <= kSmallTileBytes && worth) {
        // small maps: one wavefront per channel
        const size_t lds_small = kWaves * (small_tile + kLanes * sizeof(float));
        const dim3 grid((g.C + kWaves - 1) / kWaves, g.N);
        if (g.C <= kSinglePassChannels) {
            KernelTimer timer("encode", stream);
            hipLaunchKernelGGL(encode_small_kernel<kSinglePass>, grid, dim3(kThreads), lds_small, stream, g, act, prod, cps, ctrl,
                               map, mtab, mstride, full, fstride);
        } else {
            {
                KernelTimer timer("encode_count", stream);
                hipLaunchKernelGGL(encode_small_kernel<kPublishOnly>, grid, dim3(kThreads), lds_small, stream, g, act, prod, cps,
                                   ctrl, map, static_cast<int32_t *>(nullptr), mstride, static_cast<int32_t *>(nullptr), fstride);
            }
            CPOCONV_HIP_TRY(hipGetLastError());
            KernelTimer timer("encode", stream);
            hipLaunchKernelGGL(encode_small_kernel<kPublished>, grid, dim3(kThreads), lds_small, stream, g, act, prod, cps, ctrl,
                               map, mtab, mstride, full, fstride);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        return CPOCONV_OK;
    }
    if (g.C <= kSinglePassChannels) {
        KernelTimer timer("encode", stream);
        hipLaunchKernelGGL(encode_kernel<kSinglePass>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, prod, cps, chunk, ctrl, map,
                           mtab, mstride, full, fstride);
    } else {
        {
            KernelTimer timer("encode_count", stream);
            hipLaunchKernelGGL(encode_kernel<kPublishOnly>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, prod, cps, chunk,
                               ctrl, map, static_cast<int32_t *>(nullptr), mstride, static_cast<int32_t *>(nullptr), fstride);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("encode", stream);
        hipLaunchKernelGGL(encode_kernel<kPublished>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, prod, cps, chunk, ctrl, map,
                           mtab, mstride, full, fstride);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

int launch_zero_fill(void *buffer, int64_t bytes, hipStream_t stream)
{
    if (bytes == 0) return CPOCONV_OK;
    // leading bytes up to 4-byte alignment and trailing bytes are written one by one
    unsigned char *p = static_cast<unsigned char *>(buffer);
    const int64_t head = std::min<int64_t>(bytes, (4 - reinterpret_cast<uintptr_t>(p) % 4) % 4);
    const int64_t n_words = (bytes - head) / 4;
    const int n_tail = static_cast<int>(bytes - head - 4 * n_words);
    if (head > 0) {
        hipLaunchKernelGGL(zero_fill_kernel, dim3(1), dim3(256), 0, stream, nullptr, 0, p, static_cast<int>(head));
        CPOCONV_HIP_TRY(hipGetLastError());
    }
    const int64_t want = (n_words + 255) / 256;
    const int blocks = static_cast<int>(want < 1 ? 1 : (want > 2048 ? 2048 : want));
    hipLaunchKernelGGL(zero_fill_kernel, dim3(blocks), dim3(256), 0, stream, reinterpret_cast<uint32_t *>(p + head), n_words,
                       p + head + 4 * n_words, n_tail);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

int launch_prepare_weights(const float *w, const Geometry &g, float *wt, hipStream_t stream)
{
    const int64_t total = static_cast<int64_t>(g.C) * g.kh * g.kw * g.Kpad;
    const int blocks = static_cast<int>((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
    {
        KernelTimer timer("prepare_weights", stream);
        hipLaunchKernelGGL(prepare_weights_kernel, dim3(blocks), dim3(256), 0, stream, g, w, wt);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

}  // namespace cpoconv
