// CPO / CPS encoders (Algorithms 1 and 3) as a stream compaction.
//
// The sequential algorithms append NZEs while walking channel -> overlap type -> partition ->
// column -> row, so the position of every NZE in DA / IN is "number of NZEs visited before
// it".  Here one workgroup owns one channel: it stages the channel in LDS (coalesced row
// reads), then each wavefront takes whole columns with lane = padded row, so that a ballot
// gives the column's NZE bitmap, its popcount the column count, and the popcount of the
// lower lanes the rank of an NZE inside its column.  A prefix sum over the columns in stream
// order gives the column starts, the cumulative entries of ptr and the channel totals.
// A first launch only counts (per-channel lengths of ptr / DA / IN); the second launch
// recomputes the counts from LDS, sums the lengths of the channels before its own and writes
// the streams.  All of it is integer / bit work on the fp32 bit patterns: outputs are exact.
#include "common.hpp"

namespace cpoconv {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kLanes;
// Padded rows handled per pass (lane = row inside the chunk): 64, or 32 for maps so wide that
// 64 rows would not fit the LDS tile.  Both are multiples of 4, so a set4 never straddles chunks.
constexpr int kChunkWide = 32;
constexpr int kMaxChunks = (CPOCONV_MAX_I + kChunkWide - 1) / kChunkWide;
constexpr size_t kTileBytesMax = 48 * 1024;

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

// Inclusive prefix sum over the kThreads values held one per thread.
__device__ __forceinline__ int block_inclusive_sum(int v, int *wave_totals)
{
    v = wave_inclusive_sum(v);
    if (lane_id() == kLanes - 1) wave_totals[wave_id()] = v;
    __syncthreads();
    int add = 0;
    for (int w = 0; w < wave_id(); ++w) add += wave_totals[w];
    __syncthreads();
    return v + add;
}

struct ColumnBits {
    float v;                  // this lane's cell
    bool nz;
    unsigned long long mask;  // NZE bitmap of the 64 rows of this chunk
};

template <bool kCountOnly>
__global__ __launch_bounds__(kThreads) void encode_kernel(const Geometry g, const float *__restrict__ act,
                                                         const int cps, const int kChunk,
                                                         int32_t *__restrict__ counts, const cpoconv_map map)
{
    extern __shared__ float tile[];                   // kChunk x Wt, Wt odd: conflict-free column reads
    __shared__ uint8_t cnt_q[kMaxChunks][kMaxCols];   // NZEs per (row chunk, column)
    __shared__ uint8_t ecnt_q[kMaxChunks][kMaxCols];  // IN entries per (row chunk, column)
    __shared__ int32_t col_incl[kMaxCols];            // inclusive prefix of NZE counts, stream order
    __shared__ int32_t ecol_incl[kMaxCols];           // same for IN entries
    __shared__ int32_t tbl[kMaxCols];                 // one ptr segment under construction
    __shared__ int32_t type_base[kMaxTypes + 1];      // NZEs of the channel before each type
    __shared__ int32_t wave_totals[kWaves];
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
    auto column_bits = [&](int q, int vi) {
        ColumnBits b;
        const int hr = q * kChunk + lane - g.pad;
        const int jr = static_cast<int>(g.col_j[vi]) - g.pad;
        b.v = (lane < kChunk && hr >= 0 && hr < g.H) ? tile[lane * Wt + jr] : 0.0f;
        b.nz = is_nze(b.v);
        b.mask = __ballot(b.nz);
        return b;
    };
    // set4 of Algorithm 3: the four padded rows 4*(h/4) .. +3; chunks start at multiples of 64,
    // so a set never straddles two chunks.
    auto set4 = [&](const ColumnBits &b, int &pattern, int &rank_in_set) {
        pattern = static_cast<int>((b.mask >> (lane & ~3)) & 0xFull);
        rank_in_set = __popc(pattern & ((1 << (lane & 3)) - 1));
    };

    // ---- pass A: NZE and IN-entry counts per (chunk, column) -----------------------------
    for (int q = 0; q < nchunks; ++q) {
        load_tile(q);
        __syncthreads();
        for (int vi = wave; vi < g.n_cols; vi += kWaves) {
            const ColumnBits b = column_bits(q, vi);
            int entries = __popcll(b.mask);
            if (vi >= top_begin && vi < top_end) {
                int pattern, r;
                set4(b, pattern, r);
                entries = __popcll(__ballot(b.nz && r < 2));  // min(NZEs of the set, 2) per set
            }
            if (lane == 0) {
                cnt_q[q][vi] = static_cast<uint8_t>(__popcll(b.mask));
                ecnt_q[q][vi] = static_cast<uint8_t>(entries);
            }
        }
        if (nchunks > 1) __syncthreads();  // the next chunk overwrites the tile
    }
    __syncthreads();

    // ---- prefix sums over the columns in stream order -----------------------------------
    {
        int n = 0, e = 0;
        if (tid < g.n_cols)
            for (int q = 0; q < nchunks; ++q) { n += cnt_q[q][tid]; e += ecnt_q[q][tid]; }
        const int ni = block_inclusive_sum(n, wave_totals);
        const int ei = block_inclusive_sum(e, wave_totals);
        if (tid < kMaxCols) { col_incl[tid] = ni; ecol_incl[tid] = ei; }
    }
    __syncthreads();
    if (tid <= g.n_types) {
        const int first_col = g.type_begin[tid];
        type_base[tid] = first_col > 0 ? col_incl[first_col - 1] : 0;
    }
    __syncthreads();
    const int nnz_c = g.n_cols > 0 ? col_incl[g.n_cols - 1] : 0;
    const int in_c = g.n_cols > 0 ? ecol_incl[g.n_cols - 1] : 0;
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

    // ---- start of this channel in the three streams: sum over the channels before it ----
    {
        int a0 = 0, a1 = 0, a2 = 0;
        for (int cc = tid; cc < c; cc += kThreads) {
            a0 += counts[4 * cc + 0];
            a1 += counts[4 * cc + 1];
            a2 += counts[4 * cc + 2];
        }
        a0 = wave_sum(a0); a1 = wave_sum(a1); a2 = wave_sum(a2);
        if (tid < 3) chan_base[tid] = 0;
        __syncthreads();
        if (lane == 0) {
            atomicAdd(&chan_base[0], a0);
            atomicAdd(&chan_base[1], a1);
            atomicAdd(&chan_base[2], a2);
        }
        __syncthreads();
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
                if (tid >= 1 && tid <= 2) map.ptr[seg + tid] = col_incl[min(cb + tid - 1, ce - 1)] - base;
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
                if (vi + 1 == ce || g.col_p0[vi + 1] != g.col_p0[vi]) tbl[g.col_p0[vi]] = col_incl[vi] - base;
            __syncthreads();
            if (tid == 0) map.ptr[seg] = g.type_id[i];
            for (int p = tid; p < g.Ow; p += kThreads) map.ptr[seg + 1 + p] = tbl[p];
            __syncthreads();
            seg += 1 + g.Ow;
        }
    }

    // ---- pass B: scatter DA and IN -----------------------------------------------------------
    for (int q = 0; q < nchunks; ++q) {
        if (nchunks > 1) {
            __syncthreads();
            load_tile(q);
            __syncthreads();
        }
        for (int vi = wave; vi < g.n_cols; vi += kWaves) {
            const ColumnBits b = column_bits(q, vi);
            int da_start = vi > 0 ? col_incl[vi - 1] : 0;
            int in_start = vi > 0 ? ecol_incl[vi - 1] : 0;
            for (int qq = 0; qq < q; ++qq) { da_start += cnt_q[qq][vi]; in_start += ecnt_q[qq][vi]; }
            const unsigned long long below = (1ull << lane) - 1ull;
            const int rank = __popcll(b.mask & below);
            const int index = static_cast<int>(g.col_what[vi]) + (q * kChunk + lane) * g.kw;
            if (b.nz) map.da[da_off + da_start + rank] = b.v;
            if (vi >= top_begin && vi < top_end) {
                int pattern, r;
                set4(b, pattern, r);
                const bool emit = b.nz && r < 2;
                const unsigned long long emask = __ballot(emit);
                const int erank = __popcll(emask & below);
                const bool packed = __popc(pattern) >= 3;
                // first NZE of the set: its index (negated unless a pattern follows);
                // second NZE: the pattern, or its own negated index
                const int entry = packed ? (r == 0 ? index : pattern) : -index;
                if (emit) map.in[in_off + in_start + erank] = entry;
            } else {
                if (b.nz) map.in[in_off + in_start + rank] = index;
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
    const int chunk = kLanes * row_bytes <= kTileBytesMax ? kLanes : kChunkWide;
    const size_t lds = chunk * row_bytes;
    int32_t *counts = static_cast<int32_t *>(scratch);
    hipLaunchKernelGGL(encode_kernel<true>, dim3(g.C), dim3(kThreads), lds, stream, g, act, cps, chunk, counts, map);
    CPOCONV_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(encode_kernel<false>, dim3(g.C), dim3(kThreads), lds, stream, g, act, cps, chunk, counts, map);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

int launch_prepare_weights(const float *w, const Geometry &g, float *wt, hipStream_t stream)
{
    const int64_t total = static_cast<int64_t>(g.C) * g.kh * g.kw * g.Kpad;
    const int blocks = static_cast<int>((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
    hipLaunchKernelGGL(prepare_weights_kernel, dim3(blocks), dim3(256), 0, stream, g, w, wt);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

}  // namespace cpoconv
