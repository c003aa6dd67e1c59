// ptr -> absolute DA offsets, inside the convolution kernels.
//
// Algorithm 2 reads an entry of -1 in ptr as the entry before it: the NZEs of partition p of an
// overlap type are DA[e_{p-1} .. e_p) with e the forward-filled cumulative counts.  Live
// entries never decrease, so the forward fill is a running maximum.  A wavefront resolves the
// segments of one channel here and writes, per (channel, type), only the table slots of the
// partitions that reach its workgroup's output columns.  NPC / NPF become empty ranges.
#pragma once

#include "common.hpp"

namespace cpoconv {

// ptr entries of one channel a wavefront can stage (n_types * (1 + Ow) must fit)
constexpr int kStageInts = 256;

// inclusive running maximum over the 64 lanes (data-parallel-primitive moves: shifts inside
// rows of 16 lanes, then the last lane of a row broadcast to the rows after it)
__device__ __forceinline__ int wave_running_max(int v)
{
    constexpr int kLow = static_cast<int>(0x80000000u);   // identity of max
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x111, 0xf, 0xf, false));   // row_shr:1
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x112, 0xf, 0xf, false));   // row_shr:2
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x114, 0xf, 0xf, false));   // row_shr:4
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x118, 0xf, 0xf, false));   // row_shr:8
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x142, 0xa, 0xf, false));   // row_bcast:15 -> rows 1, 3
    v = max(v, __builtin_amdgcn_update_dpp(kLow, v, 0x143, 0xc, 0xf, false));   // row_bcast:31 -> rows 2, 3
    return v;
}

// Can resolve_ptr_rows handle the layer?  One lane per partition, one staged channel per wavefront.
inline bool resolve_in_kernel_ok(const Geometry &g)
{
    return g.Ow <= kLanes && g.n_types * (1 + g.Ow) <= kStageInts;
}

// Fills tab[(cl * n_types + i) * SPANX + e] for the channels cb .. cb+nb-1 (cl = channel - cb),
// present types i and slots e < SPANX: slot e holds the DA offset one past the NZEs of partition
// p_lo(i) - 1 + e (clamped to the last partition), p_lo(i) = max(0, x0 - type_id[i]); slot 0 is
// therefore the first NZE of partition p_lo.  Wavefront `wave` of `nwaves` takes channels
// cl = wave, wave + nwaves, ..; stage_all gives kStageInts ints of LDS per wavefront.
template <int SPANX>
__device__ __forceinline__ void resolve_ptr_rows(const Geometry &g, const int32_t *__restrict__ ptr,
                                                 const int32_t *__restrict__ chan_off, int cb, int nb, int x0,
                                                 int32_t *tab, int32_t *stage_all, int wave, int nwaves, int lane)
{
    static_assert(SPANX <= kLanes, "one lane per table slot");
    constexpr int R = 4;                          // channels whose loads are in flight together
    constexpr int KR = kStageInts / kLanes;       // registers holding one staged channel
    int32_t *stage = stage_all + wave * kStageInts;
    for (int cl0 = wave; cl0 < nb; cl0 += nwaves * R) {
        // the side-band offsets of R channels, then their ptr entries: two load latencies per R
        // channels instead of two per channel
        int seg[R], len[R], base[R], held[R][KR];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int c = min(cb + cl0 + r * nwaves, g.C - 1);
            seg[r] = chan_off[c];
            len[r] = chan_off[c + 1];
            base[r] = chan_off[(g.C + 1) + c];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            seg[r] = __builtin_amdgcn_readfirstlane(seg[r]);
            len[r] = __builtin_amdgcn_readfirstlane(len[r]) - seg[r];
            base[r] = __builtin_amdgcn_readfirstlane(base[r]);
            if (cl0 + r * nwaves >= nb) len[r] = 0;
#pragma unroll
            for (int k = 0; k < KR; ++k)
                held[r][k] = k * kLanes + lane < len[r] ? ptr[seg[r] + k * kLanes + lane] : 0;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int cl = cl0 + r * nwaves;
            if (cl >= nb) break;
#pragma unroll
            for (int k = 0; k < KR; ++k) stage[k * kLanes + lane] = held[r][k];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const bool npc = stage[0] == CPOCONV_NPC;
            int pos = 0, at = base[r];
            for (int i = 0; i < g.n_types; ++i) {
                const int t = g.type_id[i];
                int live = 0;   // 0: no NZE, 1: [pType, e_0 .. e_{Ow-1}], 2: the three-entry NOP segment
                if (!npc) live = (g.nop3 && t == 0) ? 2 : (stage[pos] == CPOCONV_NPF ? 0 : 1);
                int e = -1;
                if (lane < g.Ow) {
                    if (live == 1) e = stage[pos + 1 + lane];
                    else if (live == 2) e = lane < g.Ow - 1 ? stage[pos + 1] : stage[pos + 2];
                }
                const int m = max(wave_running_max(e), 0);              // NZEs of the type in partitions 0 .. lane
                const int total = __builtin_amdgcn_readlane(m, kLanes - 1);
                const int p = min(max(0, x0 - t) - 1 + lane, g.Ow - 1);  // partition of table slot `lane`
                const int upto = __shfl(m, max(p, 0), kLanes);
                if (lane < SPANX) tab[(cl * g.n_types + i) * SPANX + lane] = at + (p < 0 ? 0 : upto);
                at += total;
                pos += npc ? 0 : (live == 2 ? 3 : (live == 1 ? 1 + g.Ow : 1));
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the stage is reused for the wavefront's next channel
        }
    }
}

}  // namespace cpoconv
