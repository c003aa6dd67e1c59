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

// Failure flag of a map.  hdr[6] carries, above the width of the IN entries, a stamp of the call that
// wrote the header (derived from the image slot's epoch, which every call advances); a unit that gives
// up stores the same stamp in hdr[7].  A map is failed when the two agree.  Nothing has to be reset when
// a call starts - a reset would race with units that give up at once - and a stamp left by an
// earlier failed call never equals a later call's; the last unit clears such a leftover all the same.
__device__ __forceinline__ int call_stamp(unsigned long long epoch) { return static_cast<int>(epoch % 0x7FFFFFull) + 1; }
__device__ __forceinline__ void close_header(int32_t *hdr, int stamp, int in16)   // the last unit, also when it gives up
{
    hdr[6] = (in16 ? 16 : 32) | (stamp << 8);
    const int old = __hip_atomic_load(&hdr[7], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old != 0 && old != stamp) atomicCAS(&hdr[7], old, 0);
}
__device__ __forceinline__ void raise_failure(int32_t *hdr, int stamp) { atomicExch(&hdr[7], stamp); }

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A published length is at most one map's worth of elements; anything larger is not a length (a
// scratch buffer overwritten by something else) and makes the reader give up before it adds offsets.
constexpr unsigned kMaxUnitLength = CPOCONV_MAX_I * CPOCONV_MAX_I;
__device__ __forceinline__ bool lengths_plausible(unsigned long long w0, unsigned long long w1)
{
    return (w0 & 0xFFFFFFFFull) <= kMaxUnitLength && (w1 & 0x1FFFFull) <= kMaxUnitLength;
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
    r.ok = (w0 >> 32) == tag && (w1 >> 32) == tag && lengths_plausible(w0, w1);
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
                                                            const int64_t mtab_stride, int16_t *__restrict__ full_all,
                                                            const int64_t full_stride)
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

    const unsigned long long epoch = peek(ctrl + 8 + image);   // one launch: the tag of its words; always: the call's stamp
    const int stamp = call_stamp(epoch);
    const unsigned long long tag = kMode == kSinglePass ? epoch % 0xFFFFFFFEull + 1ull : kTagTwoLaunches;
    unsigned long long *flags = flags_all + 2 * static_cast<int64_t>(image) * units_stride;

    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    const int in16 = maps.in_bits == 16 ? 1 : 0;
    map.in = index_advance(maps.in, image * maps.in_cap, in16);
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;
    // for a CPS convolution launched by the same call: the plain index of every NZE, laid out like DA
    int16_t *__restrict__ full = full_all != nullptr ? full_all + image * full_stride : nullptr;

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
    const float *map_in = act_all + static_cast<int64_t>(image) * g.C * g.H * g.W;
    const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;

    unsigned long long m[kMaskWords];   // bit h % 64 of word h / 64: padded row h of this lane's column holds an NZE
    constexpr int kInFlight = 16;       // row loads issued before the first one is used
#pragma unroll
    for (int w = 0; w < kMaskWords; ++w) {
        m[w] = 0ull;
        if (w * kLanes >= g.Ih) continue;
        const int h_end = min(g.Ih, (w + 1) * kLanes);
        for (int h0 = w * kLanes; h0 < h_end; h0 += RP * kInFlight) {
            float v[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int h = h0 + u * RP + rp, hr = h - g.pad_h;
                const bool ok = col_ok && h < h_end && hr >= 0 && hr < g.H;
                v[u] = ok ? map_in[map_index(g, c, hr, jr)] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int h = h0 + u * RP + rp, hr = h - g.pad_h;
                const bool ok = col_ok && h < h_end && hr >= 0 && hr < g.H;
                const float x = ok ? produced(v[u], prod, bias_c) : 0.0f;
                if (ok) tile[col * IhP + h] = x;
                m[w] |= static_cast<unsigned long long>(is_nze(x)) << (h & (kLanes - 1));
            }
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
    // channels before this one: one lane per channel (64 at a time) adds up its bands; the words of
    // eight (channel, band) pairs are requested before the first is looked at, so a lane waits for
    // one round trip per eight pairs and not for one per pair
    int ptr_off = 0, da_off = 0, in_off = 0;
    {
        constexpr int kPairs = 8;
        const int items = (c + kLanes - 1) / kLanes * B;   // (pass over 64 channels, band), band fastest
        int tot_n = 0, tot_i = 0, tot_p = 0, cur = kWholeTypes, cur_n = 0;
        for (int t0 = 0; t0 < items; t0 += kPairs) {
            unsigned long long w0[kPairs], w1[kPairs];
#pragma unroll
            for (int j = 0; j < kPairs; ++j) {
                const int t = t0 + j, pass = t / B, bb = t - pass * B, cc = pass * kLanes + lane;
                const int u = (t < items && cc < c) ? cc * B + bb : unit;
                if (kMode == kPublished) { w0[j] = flags[2 * u]; w1[j] = flags[2 * u + 1]; }
                else { w0[j] = peek(flags + 2 * u); w1[j] = peek(flags + 2 * u + 1); }
            }
#pragma unroll
            for (int j = 0; j < kPairs; ++j) {
                const int t = t0 + j, pass = t / B, bb = t - pass * B, cc = pass * kLanes + lane;
                if (t >= items) break;
                if (cc < c) {
                    UnitLengths u;
                    if ((w0[j] >> 32) == tag && (w1[j] >> 32) == tag) {
                        u.ok = lengths_plausible(w0[j], w1[j]);
                        u.nnz = static_cast<int>(w0[j] & 0xFFFFFFFFull);
                        u.in = static_cast<int>(w1[j] & 0x1FFFFull);
                        u.ptr_part = static_cast<int>((w1[j] >> 17) & 0x7FFFull);
                    } else {
                        u = read_unit<kMode>(flags, cc * B + bb, tag);   // not there yet: wait for it
                    }
                    if (!u.ok) failed = 1;
                    const int slot = plan.band_slot[bb];
                    if (bb == 0) { tot_n = 0; tot_i = 0; tot_p = 0; cur = kWholeTypes; cur_n = 0; }
                    if (slot != cur) {
                        if (cur != kWholeTypes) tot_p += segment_length(g, cur, cur_n);
                        cur = slot;
                        cur_n = 0;
                    }
                    if (slot != kWholeTypes) cur_n += u.nnz;
                    tot_n += u.nnz;
                    tot_i += u.in;
                    tot_p += u.ptr_part;
                    if (bb == B - 1) {
                        if (cur != kWholeTypes) tot_p += segment_length(g, cur, cur_n);
                        ptr_off += tot_n > 0 ? tot_p : 1;   // a channel without an NZE is one NPC entry
                        da_off += tot_n;
                        in_off += tot_i;
                    }
                }
            }
        }
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
    if (last_unit && lane == 0) {
        poke(ctrl + 8 + image, epoch + 1ull);
        close_header(map.hdr, stamp, in16);
    }
    if (failed) {
        if (lane == 0) raise_failure(map.hdr, stamp);
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
            if (nz && full != nullptr) full[at_da + rank] = static_cast<int16_t>(index);
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

// ---------------------------------------------------------------------------------------------
// One workgroup per channel: the encoder for launches with many channel-images (every channel then
// has a workgroup's worth of parallelism and the chip is full anyway).  The channel is staged in
// LDS with coalesced row reads; one thread per column builds the column bitmaps; prefix sums over
// the columns; a look-back over the channels before it (same words as above, one unit per channel,
// its second word carrying the channel's actual number of ptr entries); scatter with lane = row.
// ---------------------------------------------------------------------------------------------
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kLanes;
constexpr int64_t kNarrowFrom = 2048;   // channel-images from which the 64 x 64 encoder runs four wavefronts per workgroup
// Padded rows handled per pass (lane = row inside the chunk): 64, a multiple of 4, so a set4 never
// straddles chunks.
constexpr int kMaxChunks = (CPOCONV_MAX_I + kLanes - 1) / kLanes;
__device__ __forceinline__ int wave_id() { return threadIdx.x / kLanes; }

template <int kMode>
__global__ __launch_bounds__(kThreads) void encode_channel_kernel(const Geometry g, const float *__restrict__ act_all,
                                                         const Producer prod, const int cps, const int kChunk,
                                                         unsigned long long *__restrict__ ctrl,
                                                         unsigned long long *__restrict__ flags_all, const int units_stride,
                                                         const cpoconv_map maps, int32_t *__restrict__ mtab_all,
                                                         const int64_t mtab_stride, int16_t *__restrict__ full_all,
                                                         const int64_t full_stride, ColumnEntry *__restrict__ columns_all,
                                                         const int64_t columns_stride)
{
    // image blockIdx.y of the launch: its map is image 0's advanced by the per-image capacities
    const int image = blockIdx.y;
    const float *__restrict__ act = act_all + static_cast<int64_t>(image) * g.C * g.H * g.W;
    const unsigned long long epoch = peek(ctrl + 8 + image);   // one launch: the tag of its words; always: the call's stamp
    const int stamp = call_stamp(epoch);
    const unsigned long long tag = kMode == kSinglePass ? epoch % 0xFFFFFFFEull + 1ull : kTagTwoLaunches;
    unsigned long long *flags = flags_all + 2 * static_cast<int64_t>(image) * units_stride;
    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    const int in16 = maps.in_bits == 16 ? 1 : 0;
    map.in = index_advance(maps.in, image * maps.in_cap, in16);
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;
    int16_t *__restrict__ full = full_all != nullptr ? full_all + image * full_stride : nullptr;   // as in the band kernel

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
    const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;

    // rows wave, wave + 8, .. of the chunk: all of a wavefront's row loads are in flight before the
    // first value is stored (one memory round trip per 64 columns instead of one per row)
    auto load_tile = [&](int q) {
        constexpr int kRowsPerWave = kLanes / kWaves;   // the chunk has at most 64 rows
        for (int j0 = 0; j0 < g.W; j0 += kLanes) {
            const int jr = j0 + lane;
            float v[kRowsPerWave];
#pragma unroll
            for (int i = 0; i < kRowsPerWave; ++i) {
                const int r = wave + i * kWaves, hr = q * kChunk + r - g.pad_h;
                v[i] = (r < kChunk && hr >= 0 && hr < g.H && jr < g.W) ? act[map_index(g, c, hr, jr)] : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < kRowsPerWave; ++i) {
                const int r = wave + i * kWaves, hr = q * kChunk + r - g.pad_h;
                if (r < kChunk && hr >= 0 && hr < g.H && jr < g.W) tile[r * Wt + jr] = produced(v[i], prod, bias_c);
            }
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
    __syncthreads();

    // ---- counts: every wavefront takes kChunk / 8 rows of the chunk (lane = column in stream
    // order) and leaves its part of every column's row bitmap in LDS; one thread per column then
    // puts the eight parts together ------------------------------------------------------------
    const int rows_per_wave = kChunk / kWaves;   // 8
    unsigned long long rows_first = 0;           // column tid: the bitmap of its first 64 padded rows
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
            if (q == 0) rows_first = mask;
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
            if ((w0 >> 32) != tag || (w1 >> 32) != tag || !lengths_plausible(w0, w1)) { failed = 1; break; }
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
    // (also after a failure, so that the words of this call are never taken for the next one's)
    if (tid == 0 && c == g.C - 1) {
        poke(ctrl + 8 + image, epoch + 1ull);
        close_header(map.hdr, stamp, in16);
    }
    // a predecessor never showed up (scratch not initialised?), or the offsets would leave the map's
    // buffers (a scratch buffer overwritten by something else): write nothing
    if (chan_base[3] != 0 || chan_base[0] + ptr_c > maps.ptr_cap || chan_base[1] + nnz_c > maps.da_cap ||
        chan_base[2] + in_c > maps.in_cap) {
        if (tid == 0) raise_failure(map.hdr, stamp);
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

    // ---- and, for the column-run convolution (maps of at most 64 padded rows: one chunk): where every
    // padded column's run starts in DA and which padded rows it holds; padding columns hold nothing
    if (columns_all != nullptr) {
        ColumnEntry *row = columns_all + image * columns_stride + static_cast<int64_t>(c) * g.Iw;
        if (tid < g.n_cols) {
            ColumnEntry e;
            e.begin = da_off + col_excl[tid];
            e.count = col_excl[tid + 1] - col_excl[tid];
            e.rows_lo = static_cast<uint32_t>(rows_first);
            e.rows_hi = static_cast<uint32_t>(rows_first >> 32);
            row[g.col_j[tid]] = e;
        }
        for (int j = tid; j < g.Iw; j += kThreads)
            if (j < g.pad_w || j >= g.pad_w + g.W) row[j] = ColumnEntry{0, 0, 0u, 0u};
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
            if (nz && full != nullptr) full[da_at + rank] = static_cast<int16_t>(index);
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
// The workgroup-per-channel encoder for maps of at most 64 padded rows and 64 padded columns (every
// layer of the workloads but the stems): the eight wavefronts share the channel's loads, the column
// bitmaps and the scatter, and in between EVERY wavefront does the channel's bookkeeping for itself,
// lane = column in stream order - counts, prefix sums, type bases, offsets; only the look-back over
// the channels before it is shared out (its words are read past the caches).  Almost nothing has to
// be handed from wavefront to wavefront then, so the kernel has three workgroup barriers (tile
// loaded, bitmaps built, look-back added up) where the general one has about fifteen, and a
// workgroup lives two thirds as long.  The tables of a convolution that follows and the ptr segments
// are written by the wavefront whose number the overlap type has (mod 8).
// ---------------------------------------------------------------------------------------------
template <int kMode, int NW>
__global__ __launch_bounds__(NW *kLanes, 8) void encode_channel64_kernel(const Geometry g, const float *__restrict__ act_all,
                                                                   const Producer prod, const int cps,
                                                                   unsigned long long *__restrict__ ctrl,
                                                                   unsigned long long *__restrict__ flags_all,
                                                                   const int units_stride, const cpoconv_map maps,
                                                                   int32_t *__restrict__ mtab_all, const int64_t mtab_stride,
                                                                   int16_t *__restrict__ full_all, const int64_t full_stride,
                                                                   ColumnEntry *__restrict__ columns_all,
                                                                   const int64_t columns_stride)
{
    extern __shared__ float tile[];                              // Ih x Wt, Wt odd: conflict-free column reads
    __shared__ unsigned long long parts[kLanes];                 // a column's row bitmap: piece w (64 / NW bits) from wavefront w
    constexpr int kT = NW * kLanes;                              // threads of the workgroup
    __shared__ int32_t stage[NW][kLanes];                        // one ptr segment under construction, per wavefront
    __shared__ int32_t chan_base[4];                             // ptr / DA / IN start of the channel, look-back failures

    const int image = blockIdx.y, c = blockIdx.x;
    const int lane = lane_id(), tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(wave_id());
    const float *__restrict__ act = act_all + static_cast<int64_t>(image) * g.C * g.H * g.W;
    unsigned long long *flags = flags_all + 2 * static_cast<int64_t>(image) * units_stride;
    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    const int in16 = maps.in_bits == 16 ? 1 : 0;
    map.in = index_advance(maps.in, image * maps.in_cap, in16);
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;
    int16_t *__restrict__ full = full_all != nullptr ? full_all + image * full_stride : nullptr;

    const int Wt = g.W | 1;
    const int top_begin = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot] : kMaxCols + 1;
    const int top_end = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot + 1] : 0;
    const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;
    constexpr int kRowsPerWave = kLanes / NW;   // 8 or 16: padded rows wave * kRowsPerWave .. belong to the wavefront

    // ---- the channel into LDS: all of a wavefront's row loads in flight before the first store -----
    {
        float v[kRowsPerWave];
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            const int hr = wave * kRowsPerWave + i - g.pad_h;
            v[i] = (hr >= 0 && hr < g.H && lane < g.W) ? act[map_index(g, c, hr, lane)] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            const int hr = wave * kRowsPerWave + i - g.pad_h;
            if (hr >= 0 && hr < g.H && lane < g.W) tile[hr * Wt + lane] = produced(v[i], prod, bias_c);
        }
    }
    // (read behind the tile's loads: loads complete in order, and this one goes past the caches)
    const unsigned long long epoch = peek(ctrl + 8 + image);   // one launch: the tag of its words; always: the call's stamp
    const int stamp = call_stamp(epoch);
    const unsigned long long tag = kMode == kSinglePass ? epoch % 0xFFFFFFFEull + 1ull : kTagTwoLaunches;
    const bool col_ok = lane < g.n_cols;
    const int my_jr = col_ok ? static_cast<int>(g.col_j[lane]) - g.pad_w : 0;
    const int my_p0 = col_ok ? static_cast<int>(g.col_p0[lane]) : 0;
    const int next_p0 = lane + 1 < g.n_cols ? static_cast<int>(g.col_p0[lane + 1]) : -1;
    if (tid < 4) chan_base[tid] = 0;
    __syncthreads();

    // ---- column bitmaps: the wavefront's eight rows of every column (lane = column), one byte each ---
    {
        unsigned bits = 0;
        if (col_ok) {
#pragma unroll
            for (int i = 0; i < kRowsPerWave; ++i) {
                const int hr = wave * kRowsPerWave + i - g.pad_h;
                if (hr >= 0 && hr < g.H) bits |= static_cast<unsigned>(is_nze(tile[hr * Wt + my_jr])) << i;
            }
        }
        if constexpr (NW == 8) reinterpret_cast<uint8_t *>(parts)[lane * NW + wave] = static_cast<uint8_t>(bits);
        else reinterpret_cast<uint16_t *>(parts)[lane * NW + wave] = static_cast<uint16_t>(bits);
    }
    __syncthreads();

    // ---- from here on every wavefront keeps the channel's books itself: lane = column ---------------
    const unsigned long long colmask = col_ok ? parts[lane] : 0ull;      // bit = padded row
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

    // ---- look-back: one wavefront publishes, every wavefront adds up the channels before this one ---
    if (kMode != kPublished && tid == 0) {
        poke(flags + 2 * c, (tag << 32) | static_cast<unsigned>(nnz_c));
        poke(flags + 2 * c + 1, (tag << 32) | static_cast<unsigned>(in_c) | (static_cast<unsigned>(ptr_c) << 17));
    }
    if (kMode == kPublishOnly) return;
    // the channels before this one are shared out over the threads (at most 512 channels take this
    // path in one launch, so a thread has at most kPolls of them); the first reads go out now ...
    // (a launch that follows a publish-only launch may have more channels: it reads them as ordinary data below)
    constexpr int kPolls = kUnitsPerImage / kT;
    unsigned long long w0 = 0, w1 = 0;   // (the first of them)
    if (kMode == kSinglePass && tid < c) {
        w0 = peek(flags + 2 * tid);
        w1 = peek(flags + 2 * tid + 1);
    }

    // ... and while they travel, the scatter's items are prepared: columns wave, wave + 8, .. of the
    // wavefront, lane = padded row; value, rank among the column's NZEs, and the IN entry with its rank
    constexpr int kColsPerWave = kLanes / NW;   // n_cols <= 64
    const int hr = lane - g.pad_h;
    const bool row_ok = hr >= 0 && hr < g.H;
    const unsigned long long below = (1ull << lane) - 1ull;
    // (an item's integers share a register: rank in bits 0-6, rank of the IN entry + 1 in bits 7-13 -
    // 0: no IN entry from this lane -, the entry itself, which fits 16 bits, above)
    float item_v[kColsPerWave];
    int item_n[kColsPerWave];
#pragma unroll
    for (int n = 0; n < kColsPerWave; ++n) {
        const int vi = wave + n * NW;
        item_v[n] = 0.0f;
        item_n[n] = 0;
        if (vi < g.n_cols) {
            int entry, erank = -1;
            const int jr = __builtin_amdgcn_readlane(my_jr, vi);
            const float v = row_ok ? tile[hr * Wt + jr] : 0.0f;
            const bool nz = is_nze(v);
            const unsigned long long mask = __ballot(nz);
            const int rank = __popcll(mask & below);
            const int index = static_cast<int>(g.col_what[vi]) + lane * g.kw;
            item_v[n] = v;
            if (vi >= top_begin && vi < top_end) {
                // set4 of Algorithm 3: the four padded rows 4*(h/4) .. +3
                const int pattern = static_cast<int>((mask >> (lane & ~3)) & 0xFull);
                const int r = __popc(pattern & ((1 << (lane & 3)) - 1));   // rank inside the set
                const bool emit = nz && r < 2;
                const int among = __popcll(__ballot(emit) & below);
                // first NZE of the set: its index (negated unless a pattern follows);
                // second NZE: the pattern, or its own negated index
                entry = __popc(pattern) >= 3 ? (r == 0 ? index : pattern) : -index;
                if (emit) erank = among;
            } else {
                entry = index;
                if (nz) erank = rank;
            }
            item_n[n] = rank | ((erank + 1) << 7) | (entry << 16);
        }
    }

    {
        int a0 = 0, a1 = 0, a2 = 0, bad = 0;
#pragma unroll
        for (int p = 0; p < kPolls; ++p) {
            if (!(kMode == kSinglePass && tid + p * kT < c)) continue;
            unsigned long long v0 = w0, v1 = w1;
            if (p > 0) {
                v0 = peek(flags + 2 * (tid + p * kT));
                v1 = peek(flags + 2 * (tid + p * kT) + 1);
            }
            for (int spin = 0; ((v0 >> 32) != tag || (v1 >> 32) != tag) && spin < kSpinLimit; ++spin) {
                __builtin_amdgcn_s_sleep(8);
                v0 = peek(flags + 2 * (tid + p * kT));
                v1 = peek(flags + 2 * (tid + p * kT) + 1);
            }
            if ((v0 >> 32) != tag || (v1 >> 32) != tag || !lengths_plausible(v0, v1)) bad = 1;
            else {
                a1 += static_cast<int>(v0 & 0xFFFFFFFFull);
                a2 += static_cast<int>(v1 & 0x1FFFFull);
                a0 += static_cast<int>((v1 >> 17) & 0x7FFFull);
            }
        }
        if (kMode == kPublished)
            for (int cc = tid; cc < c; cc += kT) {
                const unsigned long long p0 = flags[2 * cc], p1 = flags[2 * cc + 1];
                if ((p0 >> 32) != tag || (p1 >> 32) != tag || !lengths_plausible(p0, p1)) { bad = 1; break; }
                a1 += static_cast<int>(p0 & 0xFFFFFFFFull);
                a2 += static_cast<int>(p1 & 0x1FFFFull);
                a0 += static_cast<int>((p1 >> 17) & 0x7FFFull);
            }
        a0 = wave_sum(a0); a1 = wave_sum(a1); a2 = wave_sum(a2); bad = wave_sum(bad);
        if (lane == 0 && (a0 | a1 | a2 | bad) != 0) {
            atomicAdd(&chan_base[0], a0);
            atomicAdd(&chan_base[1], a1);
            atomicAdd(&chan_base[2], a2);
            atomicAdd(&chan_base[3], bad);
        }
    }
    __syncthreads();
    const int ptr_off = chan_base[0], da_off = chan_base[1], in_off = chan_base[2], failed = chan_base[3];
    // the last channel has seen every other channel's lengths, so all of them have read the epoch:
    // it may move on (also after a failure, so that the words of this call are never taken for the next one's)
    if (tid == 0 && c == g.C - 1) {
        poke(ctrl + 8 + image, epoch + 1ull);
        close_header(map.hdr, stamp, in16);
    }
    // a predecessor never showed up, or the offsets would leave the map's buffers: write nothing
    if (failed != 0 || ptr_off + ptr_c > maps.ptr_cap || da_off + nnz_c > maps.da_cap || in_off + in_c > maps.in_cap) {
        if (tid == 0) raise_failure(map.hdr, stamp);
        return;
    }

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
        }
    }

    // ---- for a convolution of the same call: the table of absolute DA offsets after every partition
    // (overlap type i by wavefront i mod 8) and the column table of the column-run kernel -----------
    if (mtab_all != nullptr) {
#pragma unroll
        for (int i = 0; i < kMaxTypes; ++i) {
            if (i >= g.n_types || (i & (NW - 1)) != wave) continue;
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
    if (columns_all != nullptr && wave == NW - 1) {
        ColumnEntry *row = columns_all + image * columns_stride + static_cast<int64_t>(c) * g.Iw;
        if (col_ok)
            row[g.col_j[lane]] = ColumnEntry{da_off + excl, cnt, static_cast<uint32_t>(colmask), static_cast<uint32_t>(colmask >> 32)};
        if (lane < g.Iw && (lane < g.pad_w || lane >= g.pad_w + g.W)) row[lane] = ColumnEntry{0, 0, 0u, 0u};
    }

    // ---- ptr: overlap type i by wavefront i mod 8 ----------------------------------------------------
    if (nnz_c == 0) {
        if (tid == 0) map.ptr[ptr_off] = CPOCONV_NPC;
        return;  // nothing to write to DA / IN
    }
    {
        int seg = ptr_off;
#pragma unroll
        for (int i = 0; i < kMaxTypes; ++i) {
            if (i >= g.n_types) continue;
            const int cb = g.type_begin[i], ce = g.type_begin[i + 1];
            const int base = type_base[i];
            const bool mine = (i & (NW - 1)) == wave;
            if (g.nop3 && g.type_id[i] == 0) {
                // [0, NZEs of the first column, NZEs of first + last column]
                const int n1 = __builtin_amdgcn_readlane(incl, min(cb, kLanes - 1)) - base;
                const int n2 = __builtin_amdgcn_readlane(incl, min(max(ce - 1, cb), kLanes - 1)) - base;
                if (mine && lane == 0) { map.ptr[seg] = 0; map.ptr[seg + 1] = n1; map.ptr[seg + 2] = n2; }
                seg += 3;
                continue;
            }
            if (type_base[i + 1] == base) {
                if (mine && lane == 0) map.ptr[seg] = CPOCONV_NPF;
                seg += 1;
                continue;
            }
            if (mine) {
                int32_t *tblw = stage[wave];
                tblw[lane] = -1;
                wave_lds_fence();
                // cumulative count after the last column first seen in each partition
                if (lane >= cb && lane < ce && (lane + 1 == ce || next_p0 != my_p0)) tblw[my_p0] = incl - base;
                wave_lds_fence();
                if (lane == 0) map.ptr[seg] = g.type_id[i];
                if (lane < g.Ow) map.ptr[seg + 1 + lane] = tblw[lane];
                wave_lds_fence();
            }
            seg += 1 + g.Ow;
        }
    }

    // ---- scatter DA and IN from the prepared items ------------------------------------------------------
#pragma unroll
    for (int n = 0; n < kColsPerWave; ++n) {
        const int vi = wave + n * NW;
        if (vi < g.n_cols) {
            const int da_at = da_off + __builtin_amdgcn_readlane(excl, vi), in_at = in_off + __builtin_amdgcn_readlane(eexcl, vi);
            const bool nz = is_nze(item_v[n]);
            const int rank = item_n[n] & 127, erank = ((item_n[n] >> 7) & 127) - 1, entry = item_n[n] >> 16;
            if (nz) map.da[da_at + rank] = item_v[n];
            if (nz && full != nullptr)
                full[da_at + rank] = static_cast<int16_t>(static_cast<int>(g.col_what[vi]) + lane * g.kw);
            if (erank >= 0) store_index(map.in, in_at + erank, entry, in16);
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

template <int kMode>
__global__ __launch_bounds__(kThreads) void encode_small_kernel(const Geometry g, const float *__restrict__ act_all,
                                                               const Producer prod, const int cps,
                                                               unsigned long long *__restrict__ ctrl,
                                                               unsigned long long *__restrict__ flags_all, const int units_stride,
                                                               const cpoconv_map maps, int32_t *__restrict__ mtab_all,
                                                               const int64_t mtab_stride, int16_t *__restrict__ full_all,
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
    const unsigned long long epoch = peek(ctrl + 8 + image);   // one launch: the tag of its words; always: the call's stamp
    const int stamp = call_stamp(epoch);
    const unsigned long long tag = kMode == kSinglePass ? epoch % 0xFFFFFFFEull + 1ull : kTagTwoLaunches;
    unsigned long long *flags = flags_all + 2 * static_cast<int64_t>(image) * units_stride;
    cpoconv_map map = maps;
    map.ptr += image * maps.ptr_cap;
    map.da += image * maps.da_cap;
    const int in16 = maps.in_bits == 16 ? 1 : 0;
    map.in = index_advance(maps.in, image * maps.in_cap, in16);
    map.chan_off += static_cast<int64_t>(image) * 3 * (g.C + 1);
    map.hdr += image * 8;
    int16_t *__restrict__ full = full_all != nullptr ? full_all + image * full_stride : nullptr;

    const int Wt = g.W | 1;
    const int per_wave = g.H * Wt + kLanes;            // floats of LDS per wavefront
    float *tile = tiles + wave * per_wave;
    int32_t *tblw = reinterpret_cast<int32_t *>(tile + g.H * Wt);
    const int top_begin = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot] : kMaxCols + 1;
    const int top_end = (cps && g.top_slot >= 0) ? g.type_begin[g.top_slot + 1] : 0;

    if (tid < 4) grp_base[tid] = 0;

    // ---- the channel into LDS (coalesced), then its column bitmaps: lane = column in stream order ----
    if (live) {
        const float bias_c = (prod.relu && prod.bias != nullptr) ? prod.bias[c] : 0.0f;
        // eight loads of the wavefront in flight before the first value is stored
        constexpr int kInFlight = 8;
        for (int i0 = lane; i0 < g.H * g.W; i0 += kInFlight * kLanes) {
            float v[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int i = i0 + u * kLanes, r = i / g.W;
                v[u] = i < g.H * g.W ? act[map_index(g, c, r, i - r * g.W)] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int i = i0 + u * kLanes, r = i / g.W;
                if (i < g.H * g.W) tile[r * Wt + (i - r * g.W)] = produced(v[u], prod, bias_c);
            }
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
            if ((w0 >> 32) != tag || (w1 >> 32) != tag || !lengths_plausible(w0, w1)) { failed = 1; break; }
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
    // the last channel's group has seen every other channel's lengths: the epoch may move on (also
    // after a failure, so that the words of this call are never taken for the next one's)
    if (tid == 0 && c0 + kWaves >= g.C) {
        poke(ctrl + 8 + image, epoch + 1ull);
        close_header(map.hdr, stamp, in16);
    }
    int group_ptr = 0, group_da = 0, group_in = 0;
    for (int w = 0; w < kWaves; ++w) { group_ptr += grp[w][0]; group_da += grp[w][1]; group_in += grp[w][2]; }
    // a predecessor never showed up, or the offsets would leave the map's buffers: write nothing
    const bool failed = grp_base[3] != 0 || grp_base[0] + group_ptr > maps.ptr_cap || grp_base[1] + group_da > maps.da_cap ||
                        grp_base[2] + group_in > maps.in_cap;
    if (failed) {
        if (tid == 0) raise_failure(map.hdr, stamp);
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
        if (nz && full != nullptr) full[at_da + rank] = static_cast<int16_t>(index);
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

// Which encoder a launch takes.  Bands (one wavefront per run of columns) pay when the launch has
// few channel-images and large maps - a workgroup per channel would leave most compute units idle
// (the 3 x 224 x 224 stem: 3 workgroups, 74 us; in bands 39 us) - ; everywhere else a workgroup per
// channel is faster (measured: 128 x 56 x 56 at one image 12 against 27 us, at 32 images the same).
static bool use_bands(const Geometry &g)
{
    const int64_t channel_images = static_cast<int64_t>(g.N) * g.C;
    // (maps from 128 x 128 on keep the bands up to 2048 channel-images: 32 stem images 1.6 against 3.1 us per image)
    return g.H * g.W >= 128 * 128 ? channel_images < 2048 : (channel_images < 32 && g.H * g.W >= 64 * 64);
}

static bool channels_single_pass(const Geometry &g) { return g.C <= kUnitsPerImage && g.N <= kSinglePassImages; }

// look-back words of a call that takes two launches (behind the fixed region)
int64_t encode_call_flags_bytes(const Geometry &g)
{
    if (!use_bands(g)) return channels_single_pass(g) ? 0 : (16 * static_cast<int64_t>(g.N) * g.C + 255) / 256 * 256;
    bool single_pass;
    const EncodePlan plan = plan_encode(g, &single_pass);
    if (single_pass) return 0;
    return (16 * static_cast<int64_t>(g.N) * g.C * plan.B + 255) / 256 * 256;
}

int64_t encode_fixed_bytes() { return fixed_scratch_bytes(); }

static int launch_encode_bands(const float *act, const Producer &prod, const Geometry &g, const cpoconv_map &map, int cps,
                               void *scratch, hipStream_t stream, int32_t *mtab, int64_t mstride, int16_t *full, int64_t fstride)
{
    bool single_pass;
    const EncodePlan plan = plan_encode(g, &single_pass);
    if (plan.B < 1) return CPOCONV_ERR_SHAPE;
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
                           ctrl, ctrl + kCtrlWords, kUnitsPerImage, map, mtab, mstride, full, fstride);
    } else {
        unsigned long long *call_flags = reinterpret_cast<unsigned long long *>(static_cast<char *>(scratch) + fixed_scratch_bytes());
        {
            KernelTimer timer("encode_count", stream);
            hipLaunchKernelGGL(encode_kernel<kPublishOnly>, grid, block, lds, stream, g, plan, act, prod, cps,
                               tile_floats, ctrl, call_flags, units, map, static_cast<int32_t *>(nullptr), mstride,
                               static_cast<int16_t *>(nullptr), fstride);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("encode", stream);
        hipLaunchKernelGGL(encode_kernel<kPublished>, grid, block, lds, stream, g, plan, act, prod, cps, tile_floats,
                           ctrl, call_flags, units, map, mtab, mstride, full, fstride);
    }
    CPOCONV_HIP_TRY(hipGetLastError());
    return CPOCONV_OK;
}

// A wavefront walks its channel's rows alone, which costs latency on the larger of the small maps:
// those take the one-wavefront-per-channel kernel only once workgroups of the other kernel would
// queue for a compute unit.
static bool use_small(const Geometry &g)
{
    // Where the column-run convolution can follow (fewer than four images, a shape it is instantiated for) the
    // workgroup-per-channel encoder takes the small maps too: it leaves the column table, and the
    // layer gains more from that kernel than the encoder loses (256 x 14 x 14: 28.8 -> 24.5 us for
    // the one-call layer, 512 x 7 x 7: 28.4 -> 26.6, the encoder alone 9.7 -> 12.0).
    if (g.N < 4 && runs_kernel_supports(g)) return false;
    const size_t small_tile = static_cast<size_t>(g.H) * (g.W | 1) * sizeof(float);
    const bool worth = g.Ih * g.Iw <= kSmallAlways || static_cast<int64_t>(g.N) * g.C >= kSmallFromChannels;
    return g.Ih <= kLanes && g.Iw <= kLanes && small_tile <= kSmallTileBytes && worth;
}

// The workgroup-per-channel kernel is the one that leaves the column table (for layers the
// column-run convolution takes); after the other two the convolution rebuilds it from the streams.
bool encode_uses_channel_kernel(const Geometry &g) { return !use_bands(g) && !use_small(g); }
bool encode_writes_columns(const Geometry &g) { return runs_kernel_preferred(g) && encode_uses_channel_kernel(g); }

int launch_encode(const float *act, const Producer &prod, const Geometry &g, const cpoconv_map &map, int algo,
                  void *scratch, hipStream_t stream, bool write_table, bool write_indices)
{
    // the plain per-NZE indices, for a CPS convolution launched by the same call (same place and
    // layout as the convolution's own reconstruction would leave them)
    int16_t *full = write_indices ? reinterpret_cast<int16_t *>(static_cast<char *>(scratch) + scratch_counts_bytes(g) +
                                                                scratch_mtab_bytes(g))
                                  : nullptr;
    const int64_t fstride = indices_stride(g);
    // the table of resolved ptr offsets, for a convolution launched by the same call
    int32_t *mtab = write_table ? reinterpret_cast<int32_t *>(static_cast<char *>(scratch) + scratch_counts_bytes(g)) : nullptr;
    const int64_t mstride = mtab_stride(g);
    const int cps = algo == CPOCONV_ALGO_CPS ? 1 : 0;
    if (use_bands(g)) return launch_encode_bands(act, prod, g, map, cps, scratch, stream, mtab, mstride, full, fstride);
    // the column table of the column-run convolution, where that kernel takes the layer
    ColumnEntry *columns = (write_table && encode_writes_columns(g))
                               ? reinterpret_cast<ColumnEntry *>(static_cast<char *>(scratch) + scratch_columns_offset(g))
                               : nullptr;
    const int64_t cstride = columns_stride(g);
    if (columns != nullptr) mtab = nullptr;   // the column-run convolution reads the column table only

    unsigned long long *ctrl = static_cast<unsigned long long *>(scratch);
    const bool single = channels_single_pass(g);
    // one launch: the words of the fixed region, 512 channel slots per image; two launches: the call's own words
    unsigned long long *flags = single ? ctrl + kCtrlWords
                                       : reinterpret_cast<unsigned long long *>(static_cast<char *>(scratch) + fixed_scratch_bytes());
    const int units_stride = single ? kUnitsPerImage : g.C;
    const size_t row_bytes = static_cast<size_t>(g.W | 1) * sizeof(float);
    const int chunk = kLanes;
    const size_t lds = chunk * row_bytes;
    const size_t small_tile = static_cast<size_t>(g.H) * (g.W | 1) * sizeof(float);
    if (use_small(g)) {
        // small maps: one wavefront per channel
        const size_t lds_small = kWaves * (small_tile + kLanes * sizeof(float));
        const dim3 grid((g.C + kWaves - 1) / kWaves, g.N);
        if (single) {
            KernelTimer timer("encode", stream);
            hipLaunchKernelGGL(encode_small_kernel<kSinglePass>, grid, dim3(kThreads), lds_small, stream, g, act, prod, cps, ctrl,
                               flags, units_stride, map, mtab, mstride, full, fstride);
        } else {
            {
                KernelTimer timer("encode_count", stream);
                hipLaunchKernelGGL(encode_small_kernel<kPublishOnly>, grid, dim3(kThreads), lds_small, stream, g, act, prod, cps,
                                   ctrl, flags, units_stride, map, static_cast<int32_t *>(nullptr), mstride, static_cast<int16_t *>(nullptr), fstride);
            }
            CPOCONV_HIP_TRY(hipGetLastError());
            KernelTimer timer("encode", stream);
            hipLaunchKernelGGL(encode_small_kernel<kPublished>, grid, dim3(kThreads), lds_small, stream, g, act, prod, cps, ctrl,
                               flags, units_stride, map, mtab, mstride, full, fstride);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        return CPOCONV_OK;
    }
    if (g.Ih <= kLanes && g.Iw <= kLanes) {
        // maps of at most 64 x 64 padded cells: the variant whose wavefronts keep their own books
        const size_t lds64 = static_cast<size_t>(g.H) * (g.W | 1) * sizeof(float);
        // Launches with many channel-images run four wavefronts per workgroup: twice the workgroups in
        // flight on a compute unit, half the copies of the per-wavefront bookkeeping (few channel-images:
        // eight wavefronts, the shorter life of a single workgroup counts).
        const bool narrow = static_cast<int64_t>(g.C) * g.N >= kNarrowFrom;
#define CPOCONV_ENCODE64(MODE, NW, ...) \
    hipLaunchKernelGGL((encode_channel64_kernel<MODE, NW>), dim3(g.C, g.N), dim3(NW * kLanes), lds64, stream, g, act, prod, cps, ctrl, \
                       flags, units_stride, map, __VA_ARGS__)
        if (single) {
            KernelTimer timer("encode", stream);
            if (narrow) CPOCONV_ENCODE64(kSinglePass, 4, mtab, mstride, full, fstride, columns, cstride);
            else CPOCONV_ENCODE64(kSinglePass, 8, mtab, mstride, full, fstride, columns, cstride);
        } else {
            {
                KernelTimer timer("encode_count", stream);
                if (narrow)
                    CPOCONV_ENCODE64(kPublishOnly, 4, static_cast<int32_t *>(nullptr), mstride, static_cast<int16_t *>(nullptr), fstride,
                                     static_cast<ColumnEntry *>(nullptr), cstride);
                else
                    CPOCONV_ENCODE64(kPublishOnly, 8, static_cast<int32_t *>(nullptr), mstride, static_cast<int16_t *>(nullptr), fstride,
                                     static_cast<ColumnEntry *>(nullptr), cstride);
            }
            CPOCONV_HIP_TRY(hipGetLastError());
            KernelTimer timer("encode", stream);
            if (narrow) CPOCONV_ENCODE64(kPublished, 4, mtab, mstride, full, fstride, columns, cstride);
            else CPOCONV_ENCODE64(kPublished, 8, mtab, mstride, full, fstride, columns, cstride);
        }
#undef CPOCONV_ENCODE64
        CPOCONV_HIP_TRY(hipGetLastError());
        return CPOCONV_OK;
    }
    if (single) {
        KernelTimer timer("encode", stream);
        hipLaunchKernelGGL(encode_channel_kernel<kSinglePass>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, prod, cps, chunk,
                           ctrl, flags, units_stride, map, mtab, mstride, full, fstride, columns, cstride);
    } else {
        {
            KernelTimer timer("encode_count", stream);
            hipLaunchKernelGGL(encode_channel_kernel<kPublishOnly>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, prod, cps,
                               chunk, ctrl, flags, units_stride, map, static_cast<int32_t *>(nullptr), mstride, static_cast<int16_t *>(nullptr), fstride,
                               static_cast<ColumnEntry *>(nullptr), cstride);
        }
        CPOCONV_HIP_TRY(hipGetLastError());
        KernelTimer timer("encode", stream);
        hipLaunchKernelGGL(encode_channel_kernel<kPublished>, dim3(g.C, g.N), dim3(kThreads), lds, stream, g, act, prod, cps, chunk,
                           ctrl, flags, units_stride, map, mtab, mstride, full, fstride, columns, cstride);
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
