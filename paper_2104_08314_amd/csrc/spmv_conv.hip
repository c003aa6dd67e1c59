// Convolution as sparse matrix-vector products over a CPO / CPS map (Algorithms 2 and 4).
//
// Mapping to the GPU: the 64 lanes of a wavefront are 64 output kernels k, so one NZE
// (value, index) is wavefront-uniform and skipping zeros costs no divergence; the
// kh * (pType+1) multiply-adds of convSpMv become that many 64-wide FMAs against weights
// laid out kernel-index-fastest.  A workgroup owns a tile of output rows x columns (and 64
// kernels); ptr's per-partition cumulative counts give exactly the DA / IN ranges of the
// partitions that reach the tile's columns, and since a column's NZEs are sorted by row, the
// rows that reach a wavefront's output rows form one contiguous lane range found by a
// ballot.  No two wavefronts add to the same output and every output adds its terms in
// stream order, so results are bitwise repeatable.

#include "common.hpp"
#include "resolve_ptr.hpp"

namespace cpoconv {

namespace {

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }

__device__ __forceinline__ int wave_inclusive_max(int v)
{
#pragma unroll
    for (int d = 1; d < kLanes; d <<= 1) {
        const int n = __shfl_up(v, d, kLanes);
        if (lane_id() >= d) v = max(v, n);
    }
    return v;
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

__device__ __forceinline__ int bcast_i(int v, int src) { return __builtin_amdgcn_readlane(v, src); }
__device__ __forceinline__ float bcast_f(float v, int src)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}

// ---------------------------------------------------------------------------------------
// Prologue of every convolution call, one workgroup per channel.
//  (1) ptr -> table of absolute DA offsets: mtab[c][type][0] = first NZE of the type in DA,
//      mtab[c][type][1+p] = one past the last NZE of partitions 0..p.  This is Algorithm 2's
//      rule that an entry of -1 stands for the entry before it, applied once for all readers (a running
//      maximum, since live entries are cumulative counts), with NPC / NPF resolved to empty
//      ranges.
//  (2) CPS only - index reconstruction of Algorithm 4: IN_cps -> one index per NZE, laid out
//      like DA.  In the overlap-kw type an entry < 0 is a singleton; a run of entries >= 0
//      alternates {first index, pattern}, so an entry's role is the parity of its distance to
//      the last negative entry before it.
// ---------------------------------------------------------------------------------------
constexpr int kExpThreads = 256;

__global__ __launch_bounds__(kExpThreads) void conv_prologue_kernel(const Geometry g, const int32_t *__restrict__ ptr_all,
                                                                  const int32_t *__restrict__ in_all,
                                                                  const int32_t *__restrict__ chan_off_all,
                                                                  int32_t *__restrict__ mtab_all,
                                                                  int32_t *__restrict__ in_full_all, const BatchStrides bs)
{
    __shared__ int32_t wave_a[kExpThreads / kLanes], wave_b[kExpThreads / kLanes];
    const int image = blockIdx.y;
    if (map_unusable(bs, image)) return;
    const int32_t *__restrict__ ptr = ptr_all + image * bs.ptr;
    const int32_t *__restrict__ in = index_advance(in_all, image * bs.in, bs.map_in16);
    const int32_t *__restrict__ chan_off = chan_off_all + static_cast<int64_t>(image) * 3 * (g.C + 1);
    int32_t *__restrict__ mtab = mtab_all + image * bs.mtab;
    int16_t *__restrict__ in_full = in_full_all ? reinterpret_cast<int16_t *>(in_full_all) + image * bs.indices : nullptr;   // every index fits 16 bits
    const int c = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wave = tid / kLanes;
    const int da0 = chan_off[(g.C + 1) + c], da1 = chan_off[(g.C + 1) + c + 1];
    const int in0 = chan_off[2 * (g.C + 1) + c], in1 = chan_off[2 * (g.C + 1) + c + 1];

    // Segments of the channel: NPC = none; per present type NPF (1 entry), the 3-entry NOP form,
    // or [pType, e_0 .. e_{Ow-1}].  Every thread walks them (uniform loads); a type's NZE count is
    // the running maximum of its entries.
    int seg = chan_off[c], base = da0, top_base = da1;
    const bool npc = ptr[seg] == CPOCONV_NPC;
    for (int i = 0; i < g.n_types; ++i) {
        int32_t *row = mtab + (static_cast<int64_t>(c) * g.n_types + i) * (g.Ow + 1);
        int live = 0;
        if (!npc) live = (g.nop3 && g.type_id[i] == 0) ? 2 : (ptr[seg] == CPOCONV_NPF ? 0 : 1);
        int e = -1;   // Ow <= 256 = workgroup size: one entry per thread
        if (tid < g.Ow) {
            if (live == 1) e = ptr[seg + 1 + tid];
            else if (live == 2) e = tid < g.Ow - 1 ? ptr[seg + 1] : ptr[seg + 2];
        }
        int m = wave_inclusive_max(e);
        if (lane == kLanes - 1) wave_a[wave] = m;
        __syncthreads();
        int total = 0;
        for (int w = 0; w < kExpThreads / kLanes; ++w) {
            total = max(total, wave_a[w]);
            if (w < wave) m = max(m, wave_a[w]);
        }
        if (tid < g.Ow) row[1 + tid] = base + max(m, 0);
        if (tid == 0) row[0] = base;
        if (i == g.top_slot) top_base = base;
        base += total;
        seg += npc ? 0 : (live == 2 ? 3 : (live == 1 ? 1 + g.Ow : 1));
        __syncthreads();
    }
    if (in_full == nullptr) return;

    const int nnz = da1 - da0;
    if (nnz == 0) return;
    // NZEs of the overlap-kw type: it is the highest type, so it closes the channel
    const int top_count = da1 - top_base;
    const int lower = nnz - top_count;  // NZEs of the other types: their IN entries are plain
    for (int i = tid; i < lower; i += kExpThreads) in_full[da0 + i] = static_cast<int16_t>(load_index(in, in0 + i, bs.map_in16));
    if (top_count == 0) return;

    const int e0 = in0 + lower, n_entries = in1 - e0;
    int carry_neg = -1;   // position (relative to e0) of the last negative entry seen so far
    int carry_out = 0;    // NZEs emitted so far
    for (int base = 0; base < n_entries; base += kExpThreads) {
        const int e = base + tid;
        const bool valid = e < n_entries;
        const int entry = valid ? load_index(in, e0 + e, bs.map_in16) : -1;
        // inclusive max scan of "position if negative"
        int m = wave_inclusive_max(entry < 0 ? e : -1);
        if (lane == kLanes - 1) wave_a[wave] = m;
        __syncthreads();
        int prev = carry_neg;
        for (int w = 0; w < wave; ++w) prev = max(prev, wave_a[w]);
        const int last_neg = max(m, prev);
        const bool is_index = valid && entry >= 0 && (((e - last_neg - 1) & 1) == 0);
        const int pattern = (is_index && e + 1 < n_entries) ? load_index(in, e0 + e + 1, bs.map_in16) : 0;
        const int emits = !valid ? 0 : (entry < 0 ? 1 : (is_index ? __popc(pattern) : 0));
        int s = wave_inclusive_sum(emits);
        if (lane == kLanes - 1) wave_b[wave] = s;
        __syncthreads();
        int before = carry_out;
        for (int w = 0; w < wave; ++w) before += wave_b[w];
        const int at = da0 + lower + before + s - emits;
        if (valid && entry < 0) {
            in_full[at] = static_cast<int16_t>(-entry);
        } else if (is_index) {
            // NZEs of the set: first index, then + kw per row after the first set bit
            const int first = __ffs(pattern) - 1;
            int k = 0;
            for (int b = first; b < 4; ++b)
                if (pattern & (1 << b)) in_full[at + k++] = static_cast<int16_t>(entry + g.kw * (b - first));
        }
        int tot_neg = carry_neg, tot_out = carry_out;
        for (int w = 0; w < kExpThreads / kLanes; ++w) { tot_neg = max(tot_neg, wave_a[w]); tot_out += wave_b[w]; }
        __syncthreads();
        carry_neg = tot_neg;
        carry_out = tot_out;
    }
}

// ---------------------------------------------------------------------------------------
// General SpMV convolution (any kh, kw, stride): accumulators of a TY x TX output tile for 64
// kernels live in LDS, [row][col][k] with k fastest (conflict-free).  Wavefront w of the
// workgroup owns the tile rows w*RW .. w*RW+RW-1.  Where the tiles alone leave compute units
// idle the input channels are cut into slices across workgroups; the slices' sums go to
// partial[slice][y][x][k] and reduce_transpose_kernel adds them in a fixed order.
// ---------------------------------------------------------------------------------------
constexpr int kConvThreads = 256;
constexpr int kConvWaves = kConvThreads / kLanes;
constexpr int kTY = 8, kTX = 8;
constexpr int kRW = kTY / kConvWaves;              // output rows per wavefront
constexpr int kMspan = kTX + kMaxTypes + 1;        // partitions a tile can reach, plus one

__global__ __launch_bounds__(kConvThreads) void spmv_conv_lds_kernel(const Geometry g, const int32_t *__restrict__ ptr_all,
                                                                    const float *__restrict__ da_all,
                                                                    const int32_t *__restrict__ in_all,
                                                                    const int32_t *__restrict__ chan_off_all,
                                                                    const float *__restrict__ wt,
                                                                    float *__restrict__ out_all,
                                                                    float *__restrict__ partial_all, const int slices,
                                                                    const BatchStrides bs)
{
    const int ngroups = g.Kpad / kLanes;
    const int slice = (blockIdx.z / ngroups) % slices;
    const int image = blockIdx.z / (ngroups * slices);
    if (map_unusable(bs, image)) return;
    const int per_slice = (g.C + slices - 1) / slices;
    const int c_begin = slice * per_slice, c_end = min(g.C, c_begin + per_slice);
    const int32_t *__restrict__ ptr = ptr_all + image * bs.ptr;
    const float *__restrict__ da = da_all + image * bs.da;
    const int32_t *__restrict__ in = index_advance(in_all, image * bs.indices, bs.indices16);
    const int32_t *__restrict__ chan_off = chan_off_all + static_cast<int64_t>(image) * 3 * (g.C + 1);
    float *__restrict__ out = out_all + image * bs.out;
    extern __shared__ float smem[];
    float *acc = smem;                               // kTY*kTX*64
    float *wl = smem + kTY * kTX * kLanes;           // kh*kw*64: weights of the current channel
    __shared__ int32_t Mtab[kMaxTypes][kMspan];      // running NZE count at the tile's partitions
    __shared__ int32_t type_da0[kMaxTypes];          // DA start of each type inside the channel

    const int tid = threadIdx.x, lane = lane_id(), wave = tid / kLanes;
    const int x0 = blockIdx.x * kTX, y0 = blockIdx.y * kTY, k0 = (blockIdx.z % ngroups) * kLanes;
    const int ylo = y0 + wave * kRW;                       // this wavefront's output rows
    const int yhi = min(min(ylo + kRW, y0 + kTY), g.Oh);
    const int taps = g.kh * g.kw;
    const int s = g.stride;

    for (int i = tid; i < kTY * kTX * kLanes; i += kConvThreads) acc[i] = 0.0f;
    __syncthreads();

    for (int c = c_begin; c < c_end; ++c) {
        const int pbase = chan_off[c];
        if (ptr[pbase] == CPOCONV_NPC) continue;       // skip channel (uniform)
        __syncthreads();                                 // previous channel done with wl / Mtab
        for (int i = tid; i < taps * kLanes; i += kConvThreads)
            wl[i] = wt[(static_cast<int64_t>(c) * taps + i / kLanes) * g.Kpad + k0 + (i & (kLanes - 1))];
        if (wave == 0) {
            // walk the channel's ptr: one segment per present type
            int seg = pbase, da_run = chan_off[(g.C + 1) + c];
            for (int i = 0; i < g.n_types; ++i) {
                const int t = g.type_id[i];
                const int p_lo = max(0, x0 - t), p_hi = min(g.Ow - 1, x0 + kTX - 1);
                const int span = p_hi - p_lo + 2;          // entries M[p_lo-1 .. p_hi]
                int count = 0;
                if (g.nop3 && t == 0) {
                    const int n_first = ptr[seg + 1], n_both = ptr[seg + 2];
                    // running count after partition p: n_first for p < Ow-1, n_both for the last
                    if (lane < span) {
                        const int p = p_lo - 1 + lane;
                        Mtab[i][lane] = p < 0 ? 0 : (p < g.Ow - 1 ? n_first : n_both);
                    }
                    count = n_both;
                    seg += 3;
                } else if (ptr[seg] == CPOCONV_NPF) {
                    if (lane < span) Mtab[i][lane] = 0;
                    seg += 1;
                } else {
                    // running maximum of the cumulative entries = count after each partition,
                    // the "-1 takes the previous entry" rule of Algorithm 2 without writing ptr
                    int carry = 0;
                    for (int b = 0; b < g.Ow; b += kLanes) {
                        const int p = b + lane;
                        const int e = p < g.Ow ? ptr[seg + 1 + p] : -1;
                        const int m = max(wave_inclusive_max(e), carry);
                        if (p < g.Ow && p >= p_lo - 1 && p <= p_hi) Mtab[i][p - (p_lo - 1)] = m;
                        carry = bcast_i(m, kLanes - 1);
                    }
                    if (p_lo == 0 && lane == 0) Mtab[i][0] = 0;
                    count = carry;
                    seg += 1 + g.Ow;
                }
                if (lane == 0) type_da0[i] = da_run;
                da_run += count;
            }
        }
        __syncthreads();

        for (int i = 0; i < g.n_types; ++i) {
            const int t = g.type_id[i];
            const int p_lo = max(0, x0 - t), p_hi = min(g.Ow - 1, x0 + kTX - 1);
            const int base = type_da0[i];
            for (int p = p_lo; p <= p_hi; ++p) {
                const int beg = Mtab[i][p - p_lo], end = Mtab[i][p - p_lo + 1];
                for (int n0 = beg; n0 < end; n0 += kLanes) {
                    const int n = n0 + lane;
                    const bool valid = n < end;
                    const int idx = valid ? load_index(in, base + n, bs.indices16) : 0;
                    const float v = valid ? da[base + n] : 0.0f;
                    const int h = idx / g.kw, wh = idx - h * g.kw;   // padded row, column in partition
                    const int qh = h / s, rh = h - qh * s;
                    // rows of the map that reach output rows [ylo, yhi)
                    const bool hit = valid && h >= ylo * s && h <= (yhi - 1) * s + g.kh - 1;
                    unsigned long long bits = __ballot(hit);
                    while (bits) {
                        const int src = __ffsll(static_cast<long long>(bits)) - 1;
                        bits &= bits - 1;
                        const float sv = bcast_f(v, src);
                        const int swh = bcast_i(wh, src), sqh = bcast_i(qh, src), srh = bcast_i(rh, src);
                        // kernel rows l = rh, rh+s, ..: output row (h-l)/s = qh, qh-1, ..
                        for (int l = srh, y = sqh; l < g.kh; l += s, --y) {
                            if (y < ylo) break;
                            if (y >= yhi) continue;
                            for (int ii = 0; ii <= t; ++ii) {
                                const int x = p + ii - x0;
                                if (x < 0 || x >= kTX) continue;
                                const int wcol = swh - ii * s;
                                acc[((y - y0) * kTX + x) * kLanes + lane] += sv * wl[(l * g.kw + wcol) * kLanes + lane];
                            }
                        }
                    }
                }
            }
        }
    }
    // each wavefront stores its own rows
    const int k = k0 + lane;
    if (slices > 1) {
        // partial sums of this channel slice, kernel index fastest; rows and columns past the map's edge hold zeros
        const int Ypad = gridDim.y * kTY, Xpad = gridDim.x * kTX;
        float *partial = partial_all + image * bs.partial;
        for (int y = ylo; y < min(ylo + kRW, y0 + kTY); ++y)
            for (int x = 0; x < kTX; ++x)
                partial[((static_cast<int64_t>(slice) * Ypad + y) * Xpad + x0 + x) * g.Kpad + k] =
                    acc[((y - y0) * kTX + x) * kLanes + lane];
    } else if (k < g.K) {
        for (int y = ylo; y < yhi; ++y)
            for (int x = 0; x < kTX && x0 + x < g.Ow; ++x)
                out[(static_cast<int64_t>(k) * g.Oh + y) * g.Ow + x0 + x] = acc[((y - y0) * kTX + x) * kLanes + lane];
    }
}

// Channel slices of the general kernel: about 512 workgroups per launch, at least four channels a slice.
static int lds_kernel_slices(const Geometry &g)
{
    const int64_t tiles = static_cast<int64_t>((g.Ow + kTX - 1) / kTX) * ((g.Oh + kTY - 1) / kTY) * (g.Kpad / kLanes) * g.N;
    int s = static_cast<int>(std::min<int64_t>(16, 512 / std::max<int64_t>(tiles, 1)));
    s = std::min(s, g.C / 4);
    s = std::max(s, 1);
    const int per_slice = (g.C + s - 1) / s;
    return (g.C + per_slice - 1) / per_slice;
}


// The table of conv_prologue_kernel for layers whose ptr segments of one channel fit a wavefront's
// stage (resolve_in_kernel_ok): one wavefront per channel, the channel's ptr entries loaded at
// once, so the chain of dependent loads is side band -> ptr -> table.
constexpr int kProWaves = 4;

__global__ __launch_bounds__(kProWaves *kLanes) void conv_prologue_wave_kernel(const Geometry g,
                                                                              const int32_t *__restrict__ ptr_all,
                                                                              const int32_t *__restrict__ chan_off_all,
                                                                              int32_t *__restrict__ mtab_all,
                                                                              const BatchStrides bs)
{
    __shared__ int32_t stage_all[kProWaves * kStageInts];
    const int image = blockIdx.y;
    if (map_unusable(bs, image)) return;
    const int32_t *__restrict__ ptr = ptr_all + image * bs.ptr;
    const int32_t *__restrict__ chan_off = chan_off_all + static_cast<int64_t>(image) * 3 * (g.C + 1);
    int32_t *__restrict__ mtab = mtab_all + image * bs.mtab;
    const int lane = lane_id(), wave = threadIdx.x / kLanes;
    const int c = blockIdx.x * kProWaves + wave;
    if (c >= g.C) return;   // the whole wavefront leaves; the kernel has no workgroup barrier
    int32_t *stage = stage_all + wave * kStageInts;
    const int seg = __builtin_amdgcn_readfirstlane(chan_off[c]);
    const int len = __builtin_amdgcn_readfirstlane(chan_off[c + 1]) - seg;
    int at = __builtin_amdgcn_readfirstlane(chan_off[(g.C + 1) + c]);
#pragma unroll
    for (int k = 0; k < kStageInts / kLanes; ++k)
        stage[k * kLanes + lane] = k * kLanes + lane < len ? ptr[seg + k * kLanes + lane] : 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const bool npc = stage[0] == CPOCONV_NPC;
    int pos = 0;
    for (int i = 0; i < g.n_types; ++i) {
        int live = 0;   // 0: no NZE, 1: [pType, e_0 .. e_{Ow-1}], 2: the three-entry NOP segment
        if (!npc) live = (g.nop3 && g.type_id[i] == 0) ? 2 : (stage[pos] == CPOCONV_NPF ? 0 : 1);
        int e = -1;
        if (lane < g.Ow) {
            if (live == 1) e = stage[pos + 1 + lane];
            else if (live == 2) e = lane < g.Ow - 1 ? stage[pos + 1] : stage[pos + 2];
        }
        const int m = max(wave_running_max(e), 0);
        int32_t *row = mtab + (static_cast<int64_t>(c) * g.n_types + i) * (g.Ow + 1);
        if (lane < g.Ow) row[1 + lane] = at + m;
        if (lane == 0) row[0] = at;
        at += __builtin_amdgcn_readlane(m, kLanes - 1);
        pos += npc ? 0 : (live == 2 ? 3 : (live == 1 ? 1 + g.Ow : 1));
    }
}

// out[k][y][x] = sum over slices of partial[slice][y][x][k]; one workgroup per (output row,
// 64 kernels, 16 columns): reads coalesced along k, writes runs along x via LDS.
constexpr int kEpiCols = 4;

__global__ __launch_bounds__(256) void reduce_transpose_kernel(const Geometry g, const float *__restrict__ partial_all,
                                                              int slices, int Ypad, int Xpad, float *__restrict__ out_all,
                                                              const BatchStrides bs)
{
    __shared__ float t[kLanes][kEpiCols + 1];
    const int ngroups = g.Kpad / kLanes, image = blockIdx.y / ngroups;
    if (map_unusable(bs, image)) return;
    const int y = blockIdx.x, kb = (blockIdx.y % ngroups) * kLanes, xb = blockIdx.z * kEpiCols;
    const int tid = threadIdx.x, lane = tid & (kLanes - 1), wave = tid / kLanes;
    const int64_t slice_stride = static_cast<int64_t>(Ypad) * Xpad * g.Kpad;
    const float *__restrict__ partial = partial_all + image * slices * slice_stride;
    float *__restrict__ out = out_all + static_cast<int64_t>(image) * g.K * g.Oh * g.Ow;
#pragma unroll
    for (int u = 0; u < kEpiCols / 4; ++u) {
        const int x = xb + wave * (kEpiCols / 4) + u;
        const float *src = partial + (static_cast<int64_t>(y) * Xpad + min(x, Xpad - 1)) * g.Kpad + kb + lane;
        t[lane][wave * (kEpiCols / 4) + u] = sum_slices(src, slice_stride, slices);
    }
    __syncthreads();
    for (int i = tid; i < kLanes * kEpiCols; i += 256) {
        const int k = i / kEpiCols, x = i % kEpiCols;
        if (kb + k < g.K && xb + x < g.Ow) out[(static_cast<int64_t>(kb + k) * g.Oh + y) * g.Ow + xb + x] = t[k][x];
    }
}

}  // namespace

int64_t lds_kernel_partial_bytes(const Geometry &g)
{
    const int s = lds_kernel_slices(g);
    if (s == 1) return 0;
    const int64_t Ypad = (g.Oh + kTY - 1) / kTY * kTY, Xpad = (g.Ow + kTX - 1) / kTX * kTX;
    return 4 * Ypad * Xpad * g.Kpad * s * g.N;
}

int launch_reduce_transpose(const Geometry &g, const float *partial, int slices, int Ypad, int Xpad, float *out,
                            const BatchStrides &bs, hipStream_t stream)
{
    KernelTimer timer("reduce_transpose", stream);
    hipLaunchKernelGGL(reduce_transpose_kernel, dim3(g.Oh, (g.Kpad / kLanes) * g.N, (g.Ow + kEpiCols - 1) / kEpiCols), dim3(256),
                       0, stream, g, partial, slices, Ypad, Xpad, out, bs);
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

// Would a CPO convolution of this layer run conv_prologue first?  (Then an encoder that runs in
// the same call can leave the table instead; the strip kernel mostly resolves ptr itself.)
bool sparse_conv_uses_prologue(const Geometry &g)
{
    if (runs_kernel_preferred(g)) return true;
    const bool strip = strip_kernel_preferred(g) || (strip_kernel_supports(g) && !tile_kernel_supports(g));
    const bool tile = strip || tile_kernel_supports(g);
    return tile && !(strip && resolve_in_kernel_ok(g));
}

int launch_sparse_conv(const cpoconv_map &map, const Geometry &g, int algo, const float *wt, float *out,
                       void *scratch, hipStream_t stream, bool table_ready, bool indices_ready, bool columns_ready)
{
    char *base = static_cast<char *>(scratch);
    int32_t *mtab = reinterpret_cast<int32_t *>(base + scratch_counts_bytes(g));
    const int64_t after_mtab = scratch_counts_bytes(g) + scratch_mtab_bytes(g);
    int32_t *in_full = nullptr;
    const int32_t *indices = map.in;
    BatchStrides bs;
    bs.ptr = map.ptr_cap; bs.da = map.da_cap; bs.in = map.in_cap; bs.indices = map.in_cap;
    bs.mtab = mtab_stride(g); bs.partial = 0; bs.out = static_cast<int64_t>(g.K) * g.Oh * g.Ow;
    bs.columns = columns_stride(g);
    bs.map_in16 = map.in_bits == 16 ? 1 : 0;
    bs.indices16 = bs.map_in16;
    bs.hdr = map.hdr;
    bs.algo = algo;
    if (algo == CPOCONV_ALGO_CPS && g.top_slot >= 0) {
        in_full = reinterpret_cast<int32_t *>(base + after_mtab);
        indices = in_full;
        bs.indices = indices_stride(g);
        bs.indices16 = 1;
    }
    const bool runs = runs_kernel_preferred(g);
    const bool strip = !runs && (strip_kernel_preferred(g) || (strip_kernel_supports(g) && !tile_kernel_supports(g)));
    const bool tile = runs || strip || tile_kernel_supports(g);
    // The strip kernel resolves ptr itself for CPO maps whose segments fit a wavefront (measured:
    // 1-4 us faster than a prologue launch; in the register-tile kernel, where many more workgroups
    // would repeat the work, it was slower).  Otherwise, and for the index reconstruction of CPS,
    // a prologue kernel runs first.
    // (table_ready / indices_ready / columns_ready: the encoder of the same call left the table / the
    // plain CPS indices / the column table of the column-run kernel in the scratch buffer)
    ColumnEntry *columns = reinterpret_cast<ColumnEntry *>(base + scratch_columns_offset(g));
    float *partial = reinterpret_cast<float *>(base + after_mtab + scratch_indices_bytes(g));
    if (runs && columns_ready) return launch_sparse_conv_runs(map, columns, g, wt, out, partial, bs, stream);
    if (runs) {
        // the column table from ptr and IN (a CPS map's packed stream is decoded there), then the
        // convolution: nothing is written per NZE
        const int rc = launch_column_table(map, table_ready ? mtab : static_cast<const int32_t *>(nullptr), columns, g, bs,
                                           in_full != nullptr, stream);
        if (rc != CPOCONV_OK) return rc;
        return launch_sparse_conv_runs(map, columns, g, wt, out, partial, bs, stream);
    }
    const bool expand = in_full != nullptr && !indices_ready;
    const bool in_kernel = strip && !expand && !table_ready && resolve_in_kernel_ok(g);
    if (in_kernel) mtab = nullptr;
    if ((tile && !in_kernel && !table_ready) || expand) {
        KernelTimer timer("conv_prologue", stream);
        if (!expand && resolve_in_kernel_ok(g))
            hipLaunchKernelGGL(conv_prologue_wave_kernel, dim3((g.C + kProWaves - 1) / kProWaves, g.N),
                               dim3(kProWaves * kLanes), 0, stream, g, map.ptr, map.chan_off, mtab, bs);
        else
            hipLaunchKernelGGL(conv_prologue_kernel, dim3(g.C, g.N), dim3(kExpThreads), 0, stream, g, map.ptr, map.in,
                               map.chan_off, mtab, expand ? in_full : static_cast<int32_t *>(nullptr), bs);
        CPOCONV_HIP_TRY(hipGetLastError());
    }
    if (strip) return launch_sparse_conv_strip(map, indices, mtab, g, wt, out, partial, bs, stream);
    if (tile) return launch_sparse_conv_tile(map, indices, mtab, g, wt, out, partial, bs, stream);
    const int slices = lds_kernel_slices(g);
    const dim3 grid((g.Ow + kTX - 1) / kTX, (g.Oh + kTY - 1) / kTY, (g.Kpad / kLanes) * slices * g.N);
    const size_t lds = (static_cast<size_t>(kTY) * kTX + static_cast<size_t>(g.kh) * g.kw) * kLanes * sizeof(float);
    const int Ypad = grid.y * kTY, Xpad = grid.x * kTX;
    bs.partial = static_cast<int64_t>(slices) * Ypad * Xpad * g.Kpad;
    {
        KernelTimer timer("spmv_conv_lds", stream);
        hipLaunchKernelGGL(spmv_conv_lds_kernel, grid, dim3(kConvThreads), lds, stream, g, map.ptr, map.da, indices,
                           map.chan_off, wt, out, partial, slices, bs);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    if (slices > 1) return launch_reduce_transpose(g, partial, slices, Ypad, Xpad, out, bs, stream);
    return CPOCONV_OK;
}

}  // namespace cpoconv
