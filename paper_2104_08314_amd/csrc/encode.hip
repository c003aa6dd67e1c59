// CPO / CPS encoders (Algorithms 1 and 3) as a stream compaction.
//
// The sequential algorithms append NZEs while walking channel -> overlap type -> partition ->
// column -> row, so the position of every NZE in DA / IN is "number of NZEs visited before it".
// Here the unit of work is a band: a run of at most 64 columns of one channel, consecutive in
// stream order, that is either a set of whole overlap types or a piece of one type.  One
// wavefront encodes one band and needs no workgroup barrier:
//   load     rows of the band are read coalesced with lane = (row phase, column); every lane keeps
//            the bitmap of the non-zero rows of its column in registers and drops the values into
//            an LDS tile transposed (column-major), for the scatter below;
//   counts   the bitmap's population count is the column's NZE count; for CPS columns of the
//            overlap-kw type, min(NZEs, 2) per group of four rows is the number of IN entries;
//   offsets  prefix sums over the lanes (columns in stream order) give every column's start in
//            DA and IN and the cumulative entries of ptr;
//   look-back the band publishes its lengths in the scratch buffer and reads those of every band
//            before it and of the other bands of its channel (its position in the packed streams,
//            and whether its overlap type and channel hold an NZE at all: NPF / NPC);
//   scatter  lane = padded row: the rank of an NZE inside its column is the population count of
//            the bitmap below its row, so a column is written as one contiguous, coalesced run.
// The lengths travel inside 64-bit atomics tagged with the call's epoch - no other memory is
// communicated, so no fence is needed - and every wait is bounded: a band that gives up, or whose
// offsets would leave the map's buffers, writes nothing and raises hdr[7].  Bands wait for bands
// with lower unit numbers (dispatched first) and for the later bands of their own channel (at
// most 31 units ahead, far fewer than the device holds at once).  All of it is integer / bit work
// on the fp32 bit patterns: outputs are exact.
#include "common.hpp"

#include <string.h>

#include <algorithm>

namespace cpoconv {

namespace {

constexpr int kEncWaves = 4;                       // bands per workgroup
constexpr int kEncThreads = kEncWaves * kLanes;
constexpr int kMaxBands = 32;                      // bands per channel
constexpr int kWholeTypes = 0xFF;                  // band_slot of a band that holds whole overlap types
constexpr int kBandLdsBytes = 16 * 1024;           // transposed tile of one band
constexpr int kMaskWords = CPOCONV_MAX_I / kLanes; // 64-bit words of a column's row bitmap

// How the columns of a channel are cut into bands (host, once per call).
struct EncodePlan {
    int32_t B;                            // bands per channel
    uint16_t band_begin[kMaxBands + 1];   // stream-order columns of band b: [band_begin[b], band_begin[b + 1])
    uint8_t band_slot[kMaxBands];         // a piece of one type: the type's slot; whole types: kWholeTypes
    uint8_t band_head[kMaxBands];         // first band of that type (the band itself for whole types)
};

// Look-back words (unsigned 64-bit) at the start of every scratch buffer, at positions that do
// not depend on the call: [8 + n] the epoch of image slot n, then two words per unit,
// {tag, |DA|} and {tag, |IN| + (ptr part << 17)}, unit = image * kUnitsPerImage + channel * B + band.
// A word is only ever tagged from the epoch counter of its image slot.  tag = epoch % (2^32 - 2) + 1
// of the call that wrote the word: never 0, the initial state, and never 2^32 - 1, which marks
// lengths published by a separate launch.  The last unit of an image advances its epoch once its
// own look-back is over (every other unit has then published, hence read the epoch).
// Calls with more than kSinglePassImages images or kUnitsPerImage units per image publish in a
// first launch and read in a second; their words lie behind the fixed region, in the part of the
// scratch buffer that belongs to the call.
constexpr int kCtrlWords = 8 + CPOCONV_MAX_BATCH;
constexpr int kUnitsPerImage = 512;
constexpr int kSinglePassImages = 128;
constexpr int64_t kFixedWords = kCtrlWords + 2 * static_cast<int64_t>(kUnitsPerImage) * kSinglePassImages;
constexpr unsigned long long kTagTwoLaunches = 0xFFFFFFFFull;
enum EncodeMode { kSinglePass = 0, kPublishOnly = 1, kPublished = 2 };
constexpr int kSpinLimit = 1 << 14;   // polls of one unit before the encoder gives up

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kLanes - 1); }

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

__device__ __forceinline__ int wave_inclusive_max(int v)
{
    constexpr int kLow = static_cast<int>(0x80000000u);   // identity of max
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x111, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x112, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x114, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x118, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x142, 0xa, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x143, 0xc, 0xf, false));
    return v;
}

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int d = kLanes / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kLanes);
    return v;
}

__device__ __forceinline__ int bcast(int v, int src) { return __builtin_amdgcn_readlane(v, src); }

// IN entries of one 64-row piece of a column under Algorithm 3: per group of four rows min(NZEs, 2).
// Counts per group by pairwise sums inside every nibble, then a group counts twice if it holds two
// NZEs or more and once if it holds one.
__device__ __forceinline__ int set4_entries(unsigned long long mask)
{
    unsigned long long c = mask - ((mask >> 1) & 0x5555555555555555ull);
    c = (c & 0x3333333333333333ull) + ((c >> 2) & 0x3333333333333333ull);   // 0 .. 4 in every nibble
    const unsigned long long two = ((c >> 1) | (c >> 2)) & 0x1111111111111111ull;
    const unsigned long long one = c & 0x1111111111111111ull & ~two;
    return 2 * __popcll(two) + __popcll(one);
}

__device__ __forceinline__ unsigned long long peek(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void poke(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Lengths one unit published: NZEs, IN entries, and the ptr entries of the whole overlap types it
// holds (counted as for a live channel).  ok: the words carried the call's tag.
struct UnitLengths {
    int nnz, in, ptr_part;
    bool ok;
};

template <int kMode>
__device__ __forceinline__ UnitLengths read_unit(const unsigned long long *flags, int unit, unsigned long long tag)
{
    unsigned long long w0, w1;
    if (kMode == kPublished) {   // written by the launch before this one: ordinary loads
        w0 = flags[2 * unit];
        w1 = flags[2 * unit + 1];
    } else {
        w0 = peek(flags + 2 * unit);
        w1 = peek(flags + 2 * unit + 1);
        for (int spin = 0; ((w0 >> 32) != tag || (w1 >> 32) != tag) && spin < kSpinLimit; ++spin) {
            __builtin_amdgcn_s_sleep(8);
            w0 = peek(flags + 2 * unit);
            w1 = peek(flags + 2 * unit + 1);
        }
    }
    UnitLengths r;
    r.ok = (w0 >> 32) == tag && (w1 >> 32) == tag;
    r.nnz = static_cast<int>(w0 & 0xFFFFFFFFull);
    r.in = static_cast<int>(w1 & 0x1FFFFull);
    r.ptr_part = static_cast<int>((w1 >> 17) & 0x7FFFull);
    return r;
}

// ptr entries of an overlap type's segment in a live channel: the three-entry NOP form, a lone
// NPF, or [pType, e_0 .. e_{Ow-1}].
__device__ __forceinline__ int segment_length(const Geometry &g, int slot, int type_nnz)
{
    if (g.nop3 && g.type_id[slot] == 0) return 3;
    return type_nnz > 0 ? 1 + g.Ow : 1;
}

template <int kMode>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(const Geometry g, const EncodePlan plan,
                                                            const float *__restrict__ act_all, const Producer prod,
                                                            const int cps, const int tile_floats,
                                                            unsigned long long *__restrict__ ctrl,
                                                            unsigned long long *__restrict__ flags_all, const int units_stride,
                                                            const cpoconv_map maps, int32_t *__restrict__ mtab_all,
                                                            const int64_t mtab_stride)
{
    extern __shared__ float lds[];   // per wavefront: tile_floats (band columns x (Ih | 1), column-major), then 64 ints

    const int image = blockIdx.y;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
    const int B = plan.B;
    const int unit = blockIdx.x * (blockDim.x / kLanes) + wave;   // band `unit % B` of channel `unit / B`
    if (unit >= g.C * B) return;                          // the kernel has no workgroup barrier
    const int c = unit / B, b = unit - c * B;
    const int vb = plan.band_begin[b], ve = plan.band_begin[b + 1], nb = ve - vb;
    const int my_slot = plan.band_slot[b];

    const unsigned long long epoch = kMode == kSinglePass ? peek(ctrl + 8 + image) : 0ull;
    const unsigned long long tag = kMode == kSinglePass ? epoch % 0xFFFFFFFEull + 1ull : kTagTwoLaunches;
    unsigned long long *flags = flags_all + 2 * static_cast<int64_t>(image) * units_stride;

    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    const int in16 = maps.in_bits == 16 ? 1 : 0;
    map.in = index_advance(maps.in, image * maps.in_cap, in16);
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;
    if (kMode != kPublishOnly && unit == 0 && lane == 0) map.hdr[7] = 0;   // raised by a band that gives up

    // ---- load: lane = (row phase rp, column col); CW columns side by side, 64 / CW rows per pass ------
    int cw_log2 = 0;
    while ((1 << cw_log2) < nb) ++cw_log2;
    const int CW = 1 << cw_log2, RP = kLanes >> cw_log2;
    const int col = lane & (CW - 1), rp = lane >> cw_log2;
    const bool col_ok = col < nb;
    const int vi = vb + (col_ok ? col : 0);               // this lane's column in stream order
    const int jr = static_cast<int>(g.col_j[vi]) - g.pad_w;
    const int IhP = g.Ih | 1;                             // odd column stride: conflict-free rows
    float *tile = lds + wave * (tile_floats + kLanes);
    int32_t *tblw = reinterpret_cast<int32_t *>(tile + tile_floats);
    const float *chan = act_all + (static_cast<int64_t>(image) * g.C + c) * g.H * g.W;
    const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;

    unsigned long long m[kMaskWords];   // bit h % 64 of word h / 64: padded row h of this lane's column holds an NZE
#pragma unroll
    for (int w = 0; w < kMaskWords; ++w) {
        m[w] = 0ull;
        if (w * kLanes >= g.Ih) continue;
        const int h_end = min(g.Ih, (w + 1) * kLanes);
#pragma unroll 4
        for (int h0 = w * kLanes; h0 < h_end; h0 += RP) {
            const int h = h0 + rp, hr = h - g.pad_h;
            const bool ok = col_ok && h < h_end && hr >= 0 && hr < g.H;
            const float v = ok ? produced(chan[hr * g.W + jr], prod, bias_c) : 0.0f;
            if (ok) tile[col * IhP + h] = v;
            m[w] |= static_cast<unsigned long long>(is_nze(v)) << (h & (kLanes - 1));
        }
        // the row phases of a column put their bits together: every lane of the column ends up with all of them
        for (int d = CW; d < kLanes; d <<= 1) m[w] |= __shfl_xor(m[w], d, kLanes);
    }
    wave_lds_fence();

    // ---- counts and offsets: lanes 0 .. nb-1 are the band's columns in stream order -------------------
    const int top_begin = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot] : kMaxCols + 1;
    const int top_end = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot + 1] : 0;
    int cnt = 0, ecnt = 0;
    if (lane < nb) {
        const bool packed = vb + lane >= top_begin && vb + lane < top_end;
#pragma unroll
        for (int w = 0; w < kMaskWords; ++w) {
            cnt += __popcll(m[w]);
            ecnt += packed ? set4_entries(m[w]) : __popcll(m[w]);
        }
    }
    const int incl = wave_inclusive_sum(cnt), eincl = wave_inclusive_sum(ecnt);
    const int excl = incl - cnt, eexcl = eincl - ecnt;
    const int nnz_u = bcast(incl, kLanes - 1), in_u = bcast(eincl, kLanes - 1);
    // whole types inside the band: their ptr entries, as if the channel were live
    int ptr_part = 0;
    if (my_slot == kWholeTypes) {
        for (int i = 0; i < g.n_types; ++i) {
            const int tb = g.type_begin[i], te = g.type_begin[i + 1];
            if (tb < vb || te > ve) continue;
            const int upto = te == ve ? nnz_u : bcast(excl, te - vb);
            ptr_part += segment_length(g, i, upto - bcast(excl, tb - vb));
        }
    }

    // ---- look-back -------------------------------------------------------------------------------------
    if (kMode != kPublished && lane == 0) {
        poke(flags + 2 * unit, (tag << 32) | static_cast<unsigned>(nnz_u));
        poke(flags + 2 * unit + 1, (tag << 32) | static_cast<unsigned>(in_u) | (static_cast<unsigned>(ptr_part) << 17));
    }
    if (kMode == kPublishOnly) return;

    int failed = 0;
    // channels before this one: one lane per channel adds up its bands
    int ptr_off = 0, da_off = 0, in_off = 0;
    for (int cc = lane; cc < c; cc += kLanes) {
        int tot_n = 0, tot_i = 0, tot_p = 0, cur = kWholeTypes, cur_n = 0;
        for (int bb = 0; bb < B; ++bb) {
            const UnitLengths u = read_unit<kMode>(flags, cc * B + bb, tag);
            if (!u.ok) failed = 1;
            const int slot = plan.band_slot[bb];
            if (slot != cur) {
                if (cur != kWholeTypes) tot_p += segment_length(g, cur, cur_n);
                cur = slot;
                cur_n = 0;
            }
            if (slot != kWholeTypes) cur_n += u.nnz;
            tot_n += u.nnz;
            tot_i += u.in;
            tot_p += u.ptr_part;
        }
        if (cur != kWholeTypes) tot_p += segment_length(g, cur, cur_n);
        ptr_off += tot_n > 0 ? tot_p : 1;   // a channel without an NZE is one NPC entry
        da_off += tot_n;
        in_off += tot_i;
    }
    ptr_off = wave_sum(ptr_off);
    da_off = wave_sum(da_off);
    in_off = wave_sum(in_off);
    // the bands of this channel: lane bb holds band bb
    int sib_n = 0, sib_i = 0, sib_p = 0;
    if (lane < B) {
        if (lane == b) {
            sib_n = nnz_u; sib_i = in_u; sib_p = ptr_part;
        } else {
            const UnitLengths u = read_unit<kMode>(flags, c * B + lane, tag);
            if (!u.ok) failed = 1;
            sib_n = u.nnz; sib_i = u.in; sib_p = u.ptr_part;
        }
    }
    failed = __ballot(failed != 0) != 0ull ? 1 : 0;
    // channel totals, what lies before this band, and this band's type when it is a piece of one
    int chan_nnz = 0, chan_in = 0, chan_ptr = 0;       // chan_ptr: entries of a live channel
    int da_before = 0, in_before = 0, ptr_start = 0;   // ptr_start: where the segment of the band's first type begins
    int type_before = 0, type_total = 0;
    {
        const int head = plan.band_head[b];
        int cur = kWholeTypes, cur_n = 0;
        for (int bb = 0; bb < B; ++bb) {
            const int n = bcast(sib_n, bb), e = bcast(sib_i, bb), pp = bcast(sib_p, bb);
            const int slot = plan.band_slot[bb];
            if (slot != cur) {
                if (cur != kWholeTypes) chan_ptr += segment_length(g, cur, cur_n);
                cur = slot;
                cur_n = 0;
            }
            if (bb == head) ptr_start = chan_ptr;      // segments of everything before the band's (first) type
            if (slot != kWholeTypes) cur_n += n;
            if (slot != kWholeTypes && slot == my_slot) {
                type_total += n;
                if (bb < b) type_before += n;
            }
            if (bb < b) { da_before += n; in_before += e; }
            chan_nnz += n;
            chan_in += e;
            chan_ptr += pp;
        }
        if (cur != kWholeTypes) chan_ptr += segment_length(g, cur, cur_n);
    }
    const bool live = chan_nnz > 0;
    const int ptr_len = live ? chan_ptr : 1;
    // offsets that would leave the caller's buffers (a scratch buffer overwritten by something else) count as a failure
    if (ptr_off + ptr_len > maps.ptr_cap || da_off + chan_nnz > maps.da_cap || in_off + chan_in > maps.in_cap) failed = 1;
    const bool last_unit = unit == g.C * B - 1;
    // the last unit has seen every other unit's lengths, so all of them have read the epoch: it moves on
    // (one writer per image; the next call is ordered after this launch), also after a failure, so that
    // the words of this call are never taken for the next one's
    if (kMode == kSinglePass && last_unit && lane == 0) poke(ctrl + 8 + image, epoch + 1ull);
    if (failed) {
        if (lane == 0) atomicOr(&map.hdr[7], 1);
        return;
    }

    if (lane == 0 && b == 0) {
        map.chan_off[c] = ptr_off;
        map.chan_off[(g.C + 1) + c] = da_off;
        map.chan_off[2 * (g.C + 1) + c] = in_off;
    }
    if (lane == 0 && last_unit) {
        map.chan_off[g.C] = ptr_off + ptr_len;
        map.chan_off[(g.C + 1) + g.C] = da_off + chan_nnz;
        map.chan_off[2 * (g.C + 1) + g.C] = in_off + chan_in;
        map.hdr[0] = ptr_off + ptr_len;
        map.hdr[1] = da_off + chan_nnz;
        map.hdr[2] = in_off + chan_in;
        map.hdr[3] = cps ? CPOCONV_ALGO_CPS : CPOCONV_ALGO_CPO;
        map.hdr[4] = g.C;
        map.hdr[5] = g.Ow;
        map.hdr[6] = in16 ? 16 : 32;
    }

    // ---- ptr of the band's types and, for a convolution of the same call, the table of absolute DA
    // offsets after every partition (what Algorithm 2 gets by forward-filling ptr) ------------------------
    if (!live && b == 0 && lane == 0) map.ptr[ptr_off] = CPOCONV_NPC;
    {
        const int my_p0 = static_cast<int>(g.col_p0[vb + min(lane, nb - 1)]);
        const int next_p0 = lane + 1 < nb ? static_cast<int>(g.col_p0[vb + lane + 1]) : -1;
        int seg = ptr_off + ptr_start;
        for (int i = 0; i < g.n_types; ++i) {
            const int tb = g.type_begin[i], te = g.type_begin[i + 1];
            const int cb = max(tb, vb), ce = min(te, ve);
            if (cb >= ce) continue;                                   // no column of the type in this band
            const bool has_first = cb == tb, has_last = ce == te;
            const int local_before = bcast(excl, cb - vb);            // NZEs of the band before the type's columns
            const int local = (ce == ve ? nnz_u : bcast(excl, ce - vb)) - local_before;
            const int t_before = my_slot == kWholeTypes ? 0 : type_before;
            const int t_total = my_slot == kWholeTypes ? local : type_total;
            const int type_start = da_off + da_before + local_before - t_before;   // first NZE of the type in DA
            const int p_begin = has_first ? 0 : static_cast<int>(g.col_p0[cb]);
            const int p_end = has_last ? g.Ow : static_cast<int>(g.col_p0[ce]);
            int32_t *row = mtab_all != nullptr
                               ? mtab_all + image * mtab_stride + (static_cast<int64_t>(c) * g.n_types + i) * (g.Ow + 1)
                               : nullptr;
            if (row != nullptr && has_first && lane == 0) row[0] = type_start;
            const bool nop3 = g.nop3 && g.type_id[i] == 0;
            const bool entries = live && t_total > 0 && !nop3;        // the segment has its Ow cumulative entries
            if (live && has_first && lane == 0) {
                if (nop3) {
                    // [0, NZEs of the first column, NZEs of first + last column]
                    map.ptr[seg] = 0;
                } else {
                    map.ptr[seg] = t_total > 0 ? static_cast<int>(g.type_id[i]) : CPOCONV_NPF;
                }
            }
            if (live && nop3) {
                const int n1 = bcast(incl, cb - vb) - local_before, n2 = bcast(incl, ce - 1 - vb) - local_before;
                if (lane == 0) { map.ptr[seg + 1] = n1; map.ptr[seg + 2] = n2; }
            }
            // partitions p_begin .. p_end-1, 64 at a time: cumulative count of the type after the last
            // column first seen in the partition, -1 where no column of the type is first seen
            int carry = t_before;                                      // count after the partitions before p_begin
            for (int p0 = p_begin; p0 < p_end; p0 += kLanes) {
                tblw[lane] = -1;
                wave_lds_fence();
                const int at = vb + lane;
                if (lane < nb && at >= cb && at < ce && my_p0 >= p0 && my_p0 < p0 + kLanes &&
                    (at + 1 == ce || next_p0 != my_p0))
                    tblw[my_p0 - p0] = t_before + incl - local_before;
                wave_lds_fence();
                const int e = tblw[lane], p = p0 + lane;
                if (entries && p < p_end) map.ptr[seg + 1 + p] = e;
                const int filled = max(wave_inclusive_max(e), carry);
                if (row != nullptr && p < p_end) row[1 + p] = type_start + filled;
                carry = bcast(filled, kLanes - 1);
                wave_lds_fence();
            }
            seg += live ? segment_length(g, i, t_total) : 0;
        }
    }
    if (!live) return;   // nothing to write to DA / IN

    // ---- scatter DA and IN: lane = (column of the pass, padded row); 1, 2 or 4 columns per pass -----------
    const int rows_pass = g.Ih <= 16 ? 16 : (g.Ih <= 32 ? 32 : kLanes);
    const int cols_pass = kLanes / rows_pass;
    const int sub = lane / rows_pass, hl = lane - sub * rows_pass;    // hl: padded row inside the 64-row piece
    const unsigned long long below = (1ull << hl) - 1ull;
    const int da_base = da_off + da_before, in_base = in_off + in_before;
    for (int v0 = 0; v0 < nb; v0 += cols_pass) {
        const int k = v0 + sub;                                        // column of the band
        const bool on = k < nb;
        const int src = on ? k : 0;
        int at_da = da_base + __shfl(excl, src, kLanes), at_in = in_base + __shfl(eexcl, src, kLanes);
        const int what = static_cast<int>(g.col_what[vb + src]);
        const bool packed = on && vb + k >= top_begin && vb + k < top_end;
#pragma unroll
        for (int w = 0; w < kMaskWords; ++w) {
            if (w * kLanes >= g.Ih) continue;
            // (read by every lane: a cross-lane read under a partial mask would not see the masked-off lanes)
            const unsigned long long fetched = __shfl(m[w], src, kLanes);
            const unsigned long long mask = on ? fetched : 0ull;
            if (__ballot(mask != 0ull) == 0ull) continue;              // no NZE in these rows of the pass's columns
            const int h = w * kLanes + hl;
            const bool nz = (mask >> hl) & 1ull;
            const int rank = __popcll(mask & below);
            const int index = what + h * g.kw;
            if (nz) map.da[at_da + rank] = tile[src * IhP + h];
            if (packed) {
                // set4 of Algorithm 3: the four padded rows 4*(h/4) .. +3
                const int pattern = static_cast<int>((mask >> (hl & ~3)) & 0xFull);
                const int r = __popc(pattern & ((1 << (hl & 3)) - 1));   // rank inside the set
                const bool emit = nz && r < 2;
                // entries before this one: two per earlier set with two or more NZEs, one per set with one
                const unsigned long long lower = mask & ((1ull << (hl & ~3)) - 1ull);
                const int erank = set4_entries(lower) + r;
                // first NZE of the set: its index (negated unless a pattern follows);
                // second NZE: the pattern, or its own negated index
                const int entry = __popc(pattern) >= 3 ? (r == 0 ? index : pattern) : -index;
                if (emit) store_index(map.in, at_in + erank, entry, in16);
                at_in += set4_entries(mask);
            } else {
                if (nz) store_index(map.in, at_in + rank, index, in16);
                at_in += __popcll(mask);
            }
            at_da += __popcll(mask);
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

// Cuts the columns of a channel into bands.  A band has at most `cpb` columns, never splits columns
// that share a first partition, and is either a run of whole overlap types or a piece of one type.
bool build_bands(const Geometry &g, int cpb, EncodePlan *plan)
{
    EncodePlan p;
    memset(&p, 0, sizeof(p));
    int nbands = 0;
    int whole_begin = -1, whole_end = -1;   // the run of whole types being collected
    auto flush_whole = [&]() {
        if (whole_begin < 0) return true;
        if (nbands >= kMaxBands) return false;
        p.band_begin[nbands] = static_cast<uint16_t>(whole_begin);
        p.band_slot[nbands] = kWholeTypes;
        p.band_head[nbands] = static_cast<uint8_t>(nbands);
        ++nbands;
        p.band_begin[nbands] = static_cast<uint16_t>(whole_end);
        whole_begin = -1;
        return true;
    };
    for (int i = 0; i < g.n_types; ++i) {
        const int tb = g.type_begin[i], te = g.type_begin[i + 1], n = te - tb;
        if (n <= cpb) {
            if (whole_begin >= 0 && te - whole_begin <= cpb) { whole_end = te; continue; }
            if (!flush_whole()) return false;
            whole_begin = tb;
            whole_end = te;
            continue;
        }
        if (!flush_whole()) return false;
        const int parts = (n + cpb - 1) / cpb, size = (n + parts - 1) / parts;
        const int head = nbands;
        for (int start = tb; start < te;) {
            int end = std::min(te, start + size);
            while (end < te && g.col_p0[end] == g.col_p0[end - 1]) ++end;
            if (end - start > kLanes || nbands >= kMaxBands) return false;
            p.band_begin[nbands] = static_cast<uint16_t>(start);
            p.band_slot[nbands] = static_cast<uint8_t>(i);
            p.band_head[nbands] = static_cast<uint8_t>(head);
            ++nbands;
            p.band_begin[nbands] = static_cast<uint16_t>(end);
            start = end;
        }
    }
    if (!flush_whole()) return false;
    p.B = nbands;
    *plan = p;
    return nbands >= 1;
}

// Columns per band: at most 64 (one lane each) and what fits the wavefront's LDS tile; with few
// channel-images in the launch, narrower bands, so that about 768 bands exist (three per compute
// unit) while a band keeps eight columns or more; one launch needs at most kUnitsPerImage bands per
// image.  `single_pass`: the look-back words of the call fit the fixed region.
EncodePlan plan_encode(const Geometry &g, bool *single_pass)
{
    const int IhP = g.Ih | 1;
    int group = 1;   // columns sharing a first partition stay in one band: leave room for the largest group
    for (int i = 0; i < g.n_types; ++i)
        for (int n = g.type_begin[i] + 1, run = 1; n < g.type_begin[i + 1]; ++n) {
            run = g.col_p0[n] == g.col_p0[n - 1] ? run + 1 : 1;
            group = std::max(group, run);
        }
    // fewest bands first (widest bands the LDS budget allows; if those are too many, up to a full
    // wavefront of columns, with fewer wavefronts per workgroup): if even they do not fit the fixed
    // look-back region, two launches it is
    int cap = std::max(1, std::min(kLanes, kBandLdsBytes / (4 * IhP)) - (group - 1));
    EncodePlan widest;
    if (!build_bands(g, cap, &widest)) {
        cap = kLanes - (group - 1);
        if (!build_bands(g, cap, &widest)) {   // cannot happen within the library's shape limits
            memset(&widest, 0, sizeof(widest));
            *single_pass = false;
            return widest;
        }
    }
    *single_pass = g.N <= kSinglePassImages && static_cast<int64_t>(g.C) * widest.B <= kUnitsPerImage;
    if (!*single_pass) return widest;
    const int64_t channel_images = static_cast<int64_t>(g.N) * g.C;
    const int bands_wanted = static_cast<int>(std::max<int64_t>(1, (768 + channel_images - 1) / channel_images));
    EncodePlan plan;
    for (int cpb = std::min(cap, std::max(8, (g.n_cols + bands_wanted - 1) / bands_wanted)); cpb < cap; ++cpb)
        if (build_bands(g, cpb, &plan) && static_cast<int64_t>(g.C) * plan.B <= kUnitsPerImage) return plan;
    return widest;
}

int64_t fixed_scratch_bytes() { return (8 * kFixedWords + 255) / 256 * 256; }

}  // namespace

// look-back words of a call that takes two launches (behind the fixed region)
int64_t encode_call_flags_bytes(const Geometry &g)
{
    bool single_pass;
    const EncodePlan plan = plan_encode(g, &single_pass);
    if (single_pass) return 0;
    return (16 * static_cast<int64_t>(g.N) * g.C * plan.B + 255) / 256 * 256;
}

int64_t encode_fixed_bytes() { return fixed_scratch_bytes(); }

int launch_encode(const float *act, const Producer &prod, const Geometry &g, const cpoconv_map &map, int algo,
                  void *scratch, hipStream_t stream, bool write_table)
{
    bool single_pass;
    const EncodePlan plan = plan_encode(g, &single_pass);
    if (plan.B < 1) return CPOCONV_ERR_SHAPE;
    // the table of resolved ptr offsets, for a convolution launched by the same call
    int32_t *mtab = write_table ? reinterpret_cast<int32_t *>(static_cast<char *>(scratch) + scratch_counts_bytes(g)) : nullptr;
    const int64_t mstride = mtab_stride(g);
    const int cps = algo == CPOCONV_ALGO_CPS ? 1 : 0;
    unsigned long long *ctrl = static_cast<unsigned long long *>(scratch);
    int widest = 1;
    for (int b = 0; b < plan.B; ++b) widest = std::max(widest, plan.band_begin[b + 1] - plan.band_begin[b]);
    const int tile_floats = widest * (g.Ih | 1);
    const size_t lds_wave = static_cast<size_t>(tile_floats + kLanes) * sizeof(float);
    const int waves = static_cast<int>(std::max<size_t>(1, std::min<size_t>(kEncWaves, (144 * 1024) / lds_wave)));
    const size_t lds = waves * lds_wave;
    const int units = g.C * plan.B;
    const dim3 grid((units + waves - 1) / waves, g.N), block(waves * kLanes);
    if (single_pass) {
        KernelTimer timer("encode", stream);
        hipLaunchKernelGGL(encode_kernel<kSinglePass>, grid, block, lds, stream, g, plan, act, prod, cps, tile_floats,
                           ctrl, ctrl + kCtrlWords, kUnitsPerImage, map, mtab, mstride);
    } else {
        unsigned long long *call_flags = reinterpret_cast<unsigned long long *>(static_cast<char *>(scratch) + fixed_scratch_bytes());
        {
            KernelTimer timer("encode_count", stream);
            hipLaunchKernelGGL(encode_kernel<kPublishOnly>, grid, block, lds, stream, g, plan, act, prod, cps,
                               tile_floats, ctrl, call_flags, units, map, static_cast<int32_t *>(nullptr), mstride);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("encode", stream);
        hipLaunchKernelGGL(encode_kernel<kPublished>, grid, block, lds, stream, g, plan, act, prod, cps, tile_floats,
                           ctrl, call_flags, units, map, mtab, mstride);
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
