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
// A first launch only counts (per-channel lengths of ptr / DA / IN); the second launch
// recomputes the counts from LDS, sums the lengths of the channels before its own and writes
// the streams.  All of it is integer / bit work on the fp32 bit patterns: outputs are exact.
#include "common.hpp"

namespace cpoconv {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kLanes;
// Padded rows handled per pass (lane = row inside the chunk): 64, or 32 for maps so wide that
// 64 rows would not fit the LDS tile.  Both are multiples of 4, so a set4 never straddles chunks.
constexpr int kChunkWide = 32;
constexpr int kMaxChunks = (CPOCONV_MAX_I + kChunkWide - 1) / kChunkWide;
constexpr size_t kTileBytesMax = 40 * 1024;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x / kLanes; }

__device__ __forceinline__ bool is_nze(float v)
{
    // +0 and -0 are zeros; denormals and NaN are not (bit test: no flush-to-zero dependence)
    return (__float_as_uint(v) & 0x7fffffffu) != 0u;
}

__device__ __forceinline__ int wave_inclusive_sum(int v)
{
#pragma unroll
    for (int d = 1; d < kLanes; d <<= 1) {
        const int n = __shfl_up(v, d, kLanes);
        if (lane_id() >= d) v += n;
    }
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

template <bool kCountOnly>
__global__ __launch_bounds__(kThreads) void encode_kernel(const Geometry g, const float *__restrict__ act_all,
                                                         const int cps, const int kChunk,
                                                         int32_t *__restrict__ counts_all, const cpoconv_map maps)
{
    // image blockIdx.y of the launch: its map is image 0's advanced by the per-image capacities
    const int image = blockIdx.y;
    const float *__restrict__ act = act_all + static_cast<int64_t>(image) * g.C * g.H * g.W;
    int32_t *__restrict__ counts = counts_all + static_cast<int64_t>(image) * 4 * (g.C + 1);
    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    map.in += image * maps.in_cap;
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;

    extern __shared__ float tile[];                    // kChunk x Wt, Wt odd: conflict-free column reads
    __shared__ uint16_t cnt_q[kMaxChunks][kMaxCols];   // NZEs per (row chunk, column), then their
    __shared__ uint16_t ecnt_q[kMaxChunks][kMaxCols];  //   exclusive sums over the chunks; same for IN
    __shared__ int32_t col_excl[kMaxCols + 1];         // NZEs of the channel before each column
    __shared__ int32_t ecol_excl[kMaxCols + 1];        // IN entries of the channel before each column
    __shared__ uint8_t col_jr[kMaxCols], col_p0[kMaxCols], col_wh[kMaxCols];  // geometry, per column
    __shared__ int32_t tbl[kMaxCols];                  // one ptr segment under construction
    __shared__ int32_t type_base[kMaxTypes + 1];       // NZEs of the channel before each type
    __shared__ int32_t wave_tot[2][kWaves];
    __shared__ int32_t chan_base[3];

    const int c = blockIdx.x;
    const int lane = lane_id(), wave = wave_id(), tid = threadIdx.x;
    const int Wt = g.W | 1;
    const int nchunks = (g.Ih + kChunk - 1) / kChunk;
    const int top_begin = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot] : kMaxCols + 1;
    const int top_end = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot + 1] : 0;
    const float *chan = act + static_cast<int64_t>(c) * g.H * g.W;

    auto load_tile = [&](int q) {
        for (int r = wave; r < kChunk; r += kWaves) {
            const int hr = q * kChunk + r - g.pad;
            if (hr < 0 || hr >= g.H) continue;
            for (int jr = lane; jr < g.W; jr += kLanes) tile[r * Wt + jr] = chan[hr * g.W + jr];
        }
    };

    // the tile's loads first, then everything that does not depend on them
    load_tile(0);
    if (tid < g.n_cols) {
        col_jr[tid] = static_cast<uint8_t>(g.col_j[tid] - g.pad);
        col_p0[tid] = g.col_p0[tid];
        col_wh[tid] = g.col_what[tid];
    }
    int a0 = 0, a1 = 0, a2 = 0;
    if (!kCountOnly) {
        // start of this channel in the three streams: lengths of the channels before it
        for (int cc = tid; cc < c; cc += kThreads) {
            a0 += counts[4 * cc + 0];
            a1 += counts[4 * cc + 1];
            a2 += counts[4 * cc + 2];
        }
        if (tid < 3) chan_base[tid] = 0;
    }
    __syncthreads();

    // ---- counts: one thread per column ---------------------------------------------------------
    for (int q = 0; q < nchunks; ++q) {
        if (q > 0) {
            __syncthreads();   // every thread is done with the previous chunk
            load_tile(q);
            __syncthreads();
        }
        if (tid < g.n_cols) {
            const int jr = col_jr[tid];
            const int r_lo = max(0, g.pad - q * kChunk), r_hi = min(kChunk, g.pad + g.H - q * kChunk);
            unsigned long long mask = 0;
            for (int r = r_lo; r < r_hi; ++r)
                mask |= static_cast<unsigned long long>(is_nze(tile[r * Wt + jr])) << r;
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
        if (!kCountOnly) {
            a0 = wave_sum(a0); a1 = wave_sum(a1); a2 = wave_sum(a2);
        }
        __syncthreads();
        int nb = 0, eb = 0;
        for (int w = 0; w < wave; ++w) { nb += wave_tot[0][w]; eb += wave_tot[1][w]; }
        if (tid < kMaxCols) { col_excl[tid + 1] = nb + ni; ecol_excl[tid + 1] = eb + ei; }
        if (tid == 0) { col_excl[0] = 0; ecol_excl[0] = 0; }
        if (!kCountOnly && lane == 0) {
            atomicAdd(&chan_base[0], a0);
            atomicAdd(&chan_base[1], a1);
            atomicAdd(&chan_base[2], a2);
        }
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

    if (kCountOnly) {
        if (tid == 0) {
            counts[4 * c + 0] = ptr_c;
            counts[4 * c + 1] = nnz_c;
            counts[4 * c + 2] = in_c;
            counts[4 * c + 3] = 0;
        }
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
            map.hdr[6] = 0;
            map.hdr[7] = 0;
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
        const int hr = q * kChunk + lane - g.pad;
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
            if (vi >= top_begin && vi < top_end) {
                // set4 of Algorithm 3: the four padded rows 4*(h/4) .. +3
                const int pattern = static_cast<int>((mask >> (lane & ~3)) & 0xFull);
                const int r = __popc(pattern & ((1 << (lane & 3)) - 1));   // rank inside the set
                const bool emit = nz && r < 2;
                const int erank = __popcll(__ballot(emit) & below);
                // first NZE of the set: its index (negated unless a pattern follows);
                // second NZE: the pattern, or its own negated index
                const int entry = __popc(pattern) >= 3 ? (r == 0 ? index : pattern) : -index;
                if (emit) map.in[in_at + erank] = entry;
            } else {
                if (nz) map.in[in_at + rank] = index;
            }
        }
    }
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

int launch_encode(const float *act, const Geometry &g, const cpoconv_map &map, int algo, void *scratch,
                  hipStream_t stream)
{
    const int cps = algo == CPOCONV_ALGO_CPS ? 1 : 0;
    const size_t row_bytes = static_cast<size_t>(g.W | 1) * sizeof(float);
    const int chunk = kLanes * row_bytes <= kTileBytesMax ? kLanes : kChunkWide;   // 32 rows always fit: W <= 256
    const size_t lds = chunk * row_bytes;
    int32_t *counts = static_cast<int32_t *>(scratch);
    {
        KernelTimer timer("encode_count", stream);
        hipLaunchKernelGGL(encode_kernel<true>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, cps, chunk, counts, map);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    {
        KernelTimer timer("encode_write", stream);
        hipLaunchKernelGGL(encode_kernel<false>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, cps, chunk, counts, map);
    }
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
