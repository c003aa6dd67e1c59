/*
 * CPU oracle for CPO / CPS sparse-activation convolution.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, sequential implementation of what the GPU library computes, written from
 * the paper "High Performance Convolution Using Sparsity and Patterns for Inference in Deep
 * CNNs" (arXiv 2104.08314).  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; it shares no code with the HIP library and the HIP library
 * never calls it.
 *
 * What follows the paper directly
 *   orc_conv_direct      Eq. 1 (Section 3.1), with stride and zero padding made explicit.
 *   orc_geometry         horizontal partitions, overlap types and the in-partition
 *                        row-major index (Sections 3.1 and 3.2).
 *   orc_encode           Algorithm 1 (CPO) and Algorithm 3 (CPS), Sections 3.3 and 3.4.
 *   orc_sparse_conv      Algorithm 2 (CPO) and Algorithm 4 (CPS).
 *   orc_decode           inverse of orc_encode (used for the decode(encode(x)) == x pin).
 *   orc_im2col_lower     im2col lowering as described in Section 3.1.
 *   orc_gemm             plain matrix product of the kernel matrix with the lowered matrix.
 *   orc_select           offline per-layer selection, Section 3.5.
 *
 * Pins (tests/test_oracle_*.py): the worked example of Fig. 1 as told by the text of
 * Sections 3.3 and 3.4; the SI closed forms for |DA|, |IN_cpo|, |IN_cps| and |ptr|;
 * decode(encode(x)) == x; exhaustive 4x4 binary maps and random tiny layers against
 * orc_conv_direct; orc_conv_direct against a library convolution and hand-derived cases.
 *
 * Parity unpinned (the paper fixes nothing to check against):
 *   - the numeric values of the NPF / NPC flags and the 32-bit width of ptr / IN;
 *   - everything at stride > 1 (the paper gives no strided algorithm or example; the
 *     multiplicity-based generalisation below is pinned only by brute force and invariants).
 *
 * Floating point: sums are accumulated in double and rounded once to float.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_NPF (-2) /* "No Ptr Flag": an overlap type of a live channel holds no NZE */
#define ORC_NPC (-3) /* "No Ptr Channel": the whole channel holds no NZE              */

#define ORC_OK 0
#define ORC_BAD_SHAPE (-2)
#define ORC_TOO_SMALL (-3)

typedef struct {
    int32_t C, H, W, K, kh, kw, stride;
    int32_t pad_h, pad_w; /* zero rows above and below, zero columns left and right */
} orc_shape;

/* ------------------------------------------------------------------------------------ */
/* Geometry (Sections 3.1-3.2).                                                          */
/*                                                                                       */
/* The padded map (Ih = H + 2 pad_h rows, Iw = W + 2 pad_w columns; Algorithm 1 takes the */
/* column padding as its own input, Pad_Left) is cut into Ow partitions of width kw, partition */
/* p starting at column p*stride.  A padded column j lies in m(j) partitions; its        */
/* overlap type is pType = m(j)-1 (0 = NOP, 1 = overlap2, ..., kw-1 = overlap-kw).  Only */
/* the first partition that holds the column, p0(j), indexes it; the index of cell       */
/* (h, j) is what(j) + h*kw with what(j) = j - p0(j)*stride the column inside p0.        */
/* ------------------------------------------------------------------------------------ */

static int shape_ok(const orc_shape *s)
{
    if (s->C < 1 || s->H < 1 || s->W < 1 || s->K < 1) return 0;
    if (s->kh < 1 || s->kw < 1 || s->stride < 1 || s->pad_h < 0 || s->pad_w < 0) return 0;
    if (s->H + 2 * s->pad_h < s->kh || s->W + 2 * s->pad_w < s->kw) return 0;
    return 1;
}

/* info[0..5] = Ih, Iw, Oh, Ow, nop3, top.
 * cls/p0/what/real: Iw entries each.  present: kw entries.
 * cls = -1 for a column no partition covers (possible only when stride does not divide
 * Iw-kw).  real = 1 for columns of the unpadded map.  A type is present when it holds a
 * real column: types made of padding only are never emitted (Algorithm 1 starts at
 * pType = Pad_Left).
 * nop3 = 1 when the NOP type uses Algorithm 1's three-entry segment (VALID padding,
 * stride 1).  top = the type CPS packs (overlap-kw at stride 1), or -1. */
int orc_geometry(const orc_shape *s, int32_t *info, int32_t *cls, int32_t *p0, int32_t *what,
                 int32_t *real, int32_t *present)
{
    if (!shape_ok(s)) return ORC_BAD_SHAPE;
    int Ih = s->H + 2 * s->pad_h, Iw = s->W + 2 * s->pad_w;
    int Oh = (Ih - s->kh) / s->stride + 1, Ow = (Iw - s->kw) / s->stride + 1;
    for (int t = 0; t < s->kw; ++t) present[t] = 0;
    for (int j = 0; j < Iw; ++j) {
        int m = 0, first = -1;
        for (int p = 0; p < Ow; ++p) {
            if (p * s->stride <= j && j <= p * s->stride + s->kw - 1) {
                if (first < 0) first = p;
                ++m;
            }
        }
        real[j] = (j >= s->pad_w && j < s->pad_w + s->W);
        if (m == 0) {
            cls[j] = -1; p0[j] = -1; what[j] = -1;
        } else {
            cls[j] = m - 1; p0[j] = first; what[j] = j - first * s->stride;
            if (real[j]) present[m - 1] = 1;
        }
    }
    int top = (s->kw + s->stride - 1) / s->stride - 1;
    if (top < 1 || !present[top]) top = -1;
    info[0] = Ih; info[1] = Iw; info[2] = Oh; info[3] = Ow;
    info[4] = (s->stride == 1 && s->pad_w == 0 && s->kw >= 2 && Ow >= 2);
    info[5] = top;
    return ORC_OK;
}

/* Largest possible |ptr| (no skip flag anywhere). */
int64_t orc_max_ptr(const orc_shape *s)
{
    if (!shape_ok(s)) return ORC_BAD_SHAPE;
    int Ow = (s->W + 2 * s->pad_w - s->kw) / s->stride + 1;
    return (int64_t)s->C * s->kw * (1 + Ow) + 3;
}

/* A cell is a non-zero element when its value differs from zero.  +0 and -0 are zeros,
 * denormals and NaN are not; the test is done on the bit pattern so that no flush-to-zero
 * mode can change it. */
static int is_nze(float v)
{
    uint32_t b;
    memcpy(&b, &v, 4);
    return (b & 0x7fffffffu) != 0;
}

/* Padded-map read. */
static float padded(const float *act, const orc_shape *s, int c, int h, int j)
{
    int hr = h - s->pad_h, jr = j - s->pad_w;
    if (hr < 0 || hr >= s->H || jr < 0 || jr >= s->W) return 0.0f;
    return act[((int64_t)c * s->H + hr) * s->W + jr];
}

/* ------------------------------------------------------------------------------------ */
/* Encoders: Algorithm 1 (algo = 0, CPO) and Algorithm 3 (algo = 1, CPS).                */
/*                                                                                       */
/* Streams, for channels in order, inside a channel for present types ascending, inside  */
/* a type for partitions ascending, inside a partition for columns ascending, inside a   */
/* column for rows ascending:                                                            */
/*   DA   value of every NZE                                                             */
/*   IN   CPO: its index what + h*kw.  CPS: the same except in the top type, where rows  */
/*        are grouped four by four (set4, padded row h, the last set zero-extended):     */
/*        3 or 4 NZEs -> {index of the set's first NZE, pattern}, pattern = sum of       */
/*        2^(h mod 4) over the set's NZEs; 2 NZEs -> the two indices negated; 1 -> the   */
/*        index negated (Section 3.4).                                                   */
/*   ptr  per channel: NPC if the channel has no NZE; else per present type: NPF if the  */
/*        type has no NZE, else [pType, e_0 .. e_{Ow-1}], e_p = number of NZEs of this   */
/*        type in this channel up to and including the columns first seen in partition   */
/*        p, or -1 when no column of this type is first seen in p (Section 3.3: B, C, E  */
/*        are -1 and D repeats 5 in the worked example).  With VALID padding at stride 1 */
/*        the NOP type is the three entries [0, n_first_col, n_first_col + n_last_col]   */
/*        and has no NPF form (Algorithm 1, NOP block; SI, size of ptr: NOP takes 3).    */
/* chan_off: side band, 3*(C+1) entries: ptr / DA / IN offset of every channel and the   */
/* totals (Algorithm 2 is written without per-channel offsets; a reader that does not   */
/* walk the channels in order needs it).  lens = |ptr|, |DA|, |IN|.                      */
/* ------------------------------------------------------------------------------------ */
int orc_encode(const float *act, const orc_shape *s, int algo, int32_t *ptr, int64_t ptr_cap,
               float *da, int32_t *in, int64_t da_cap, int32_t *chan_off, int64_t *lens)
{
    if (!shape_ok(s)) return ORC_BAD_SHAPE;
    int Iw = s->W + 2 * s->pad_w, Ih = s->H + 2 * s->pad_h;
    int32_t info[6];
    int32_t *cls = malloc(sizeof(int32_t) * Iw * 4), *p0 = cls + Iw, *what = p0 + Iw,
            *real = what + Iw;
    int32_t *present = malloc(sizeof(int32_t) * s->kw);
    orc_geometry(s, info, cls, p0, what, real, present);
    int Ow = info[3], nop3 = info[4], top = info[5];
    int kw = s->kw, C = s->C;
    int64_t ptr_sh = 0, nda = 0, nin = 0;
    int rc = ORC_OK;

    for (int c = 0; c < C && rc == ORC_OK; ++c) {
        chan_off[c] = (int32_t)ptr_sh;
        chan_off[(C + 1) + c] = (int32_t)nda;
        chan_off[2 * (C + 1) + c] = (int32_t)nin;
        int64_t ptr_start = ptr_sh;
        int64_t nz_ch = 0;
        if (ptr_sh + (int64_t)kw * (1 + Ow) + 3 > ptr_cap) { rc = ORC_TOO_SMALL; break; }
        if (nda + (int64_t)Ih * Iw > da_cap) { rc = ORC_TOO_SMALL; break; }
        for (int t = 0; t < kw; ++t) {
            if (!present[t]) continue;
            int64_t nz_ptr = 0;
            int64_t seg = ptr_sh;
            int three = (nop3 && t == 0);
            if (three) {
                ptr[ptr_sh++] = 0;
            } else {
                ptr[seg] = t;
                for (int p = 0; p < Ow; ++p) ptr[seg + 1 + p] = -1;
            }
            for (int j = 0; j < Iw; ++j) {
                if (cls[j] != t || !real[j]) continue;
                if (algo == 1 && t == top) {
                    /* Algorithm 3: set4 packing of the indices of this column */
                    for (int q = 0; 4 * q < Ih; ++q) {
                        int pattern = 0, nz_col = 0;
                        int32_t aux[4];
                        for (int b = 0; b < 4; ++b) {
                            int h = 4 * q + b;
                            if (h >= Ih) break;
                            float v = padded(act, s, c, h, j);
                            if (is_nze(v)) {
                                da[nda++] = v;
                                pattern += 1 << b;
                                aux[nz_col++] = what[j] + h * kw;
                                ++nz_ptr;
                            }
                        }
                        if (nz_col >= 3) {
                            in[nin++] = aux[0];
                            in[nin++] = pattern;
                        } else if (nz_col == 2) {
                            in[nin++] = -aux[0];
                            in[nin++] = -aux[1];
                        } else if (nz_col == 1) {
                            in[nin++] = -aux[0];
                        }
                    }
                } else {
                    /* function G of Algorithm 1 */
                    for (int h = 0; h < Ih; ++h) {
                        float v = padded(act, s, c, h, j);
                        if (is_nze(v)) {
                            da[nda++] = v;
                            in[nin++] = what[j] + h * kw;
                            ++nz_ptr;
                        }
                    }
                }
                if (three) ptr[ptr_sh++] = (int32_t)nz_ptr;
                else ptr[seg + 1 + p0[j]] = (int32_t)nz_ptr;
            }
            if (!three) {
                if (nz_ptr > 0) ptr_sh = seg + 1 + Ow;
                else { ptr[seg] = ORC_NPF; ptr_sh = seg + 1; }
            }
            nz_ch += nz_ptr;
        }
        if (nz_ch == 0) { /* skip channel: rewind what this channel wrote */
            ptr_sh = ptr_start;
            ptr[ptr_sh++] = ORC_NPC;
        }
    }
    chan_off[C] = (int32_t)ptr_sh;
    chan_off[(C + 1) + C] = (int32_t)nda;
    chan_off[2 * (C + 1) + C] = (int32_t)nin;
    lens[0] = ptr_sh; lens[1] = nda; lens[2] = nin;
    free(cls); free(present);
    return rc;
}

/* ------------------------------------------------------------------------------------ */
/* Walking an encoded map.                                                               */
/* ------------------------------------------------------------------------------------ */

/* Position of a set bit of a set4 pattern relative to the pattern's first set bit; g
 * counts the pattern's NZEs from 0 (role of nextOffset in Algorithm 4, non-incremental). */
static int pattern_row_offset(int pattern, int g)
{
    int first = -1, seen = 0;
    for (int b = 0; b < 4; ++b) {
        if (pattern & (1 << b)) {
            if (first < 0) first = b;
            if (seen == g) return b - first;
            ++seen;
        }
    }
    return -1;
}

static int pattern_size(int pattern)
{
    int n = 0;
    for (int b = 0; b < 4; ++b) n += (pattern >> b) & 1;
    return n;
}

/* convSpMv of Algorithm 2 for one NZE and one output kernel k.
 * index -> padded row h = index / kw and partition column what = index % kw.  The NZE meets
 * kernel row l at output row y = (h - l) / stride when that division is exact, and kernel
 * column what - i*stride at output column part + i for i = 0..pType.  Wk = weights of kernel
 * k and channel c, kh x kw flattened row by row (Section 3.3). */
static void conv_spmv(double *Ok, const float *Wk, const orc_shape *s, int Oh, int Ow, int pType,
                      float value, int part, int index)
{
    int h = index / s->kw, wh = index % s->kw;
    for (int l = 0; l < s->kh; ++l) {
        int d = h - l;
        if (d < 0 || d % s->stride != 0) continue;
        int y = d / s->stride;
        if (y >= Oh) continue;
        for (int i = 0; i <= pType; ++i)
            Ok[(int64_t)y * Ow + part + i] += (double)value * (double)Wk[l * s->kw + wh - i * s->stride];
    }
}

/* Algorithm 2 (algo = 0) / Algorithm 4 (algo = 1): out[k][y][x], K x Oh x Ow, from the
 * encoded map and weights K x C x kh x kw.  ptr is read only: the "-1 takes the previous
 * entry" rule of Algorithm 2 is applied to a local copy of the range end. */
int orc_sparse_conv(const int32_t *ptr, const float *da, const int32_t *in, const orc_shape *s,
                    int algo, const float *weights, float *out)
{
    if (!shape_ok(s)) return ORC_BAD_SHAPE;
    int Iw = s->W + 2 * s->pad_w;
    int32_t info[6];
    int32_t *cls = malloc(sizeof(int32_t) * Iw * 4), *p0 = cls + Iw, *what = p0 + Iw,
            *real = what + Iw;
    int32_t *present = malloc(sizeof(int32_t) * s->kw);
    orc_geometry(s, info, cls, p0, what, real, present);
    int Oh = info[2], Ow = info[3], nop3 = info[4], top = info[5];
    int64_t plane = (int64_t)Oh * Ow;
    double *Ok = malloc(sizeof(double) * plane);

    for (int k = 0; k < s->K; ++k) {
        memset(Ok, 0, sizeof(double) * plane);
        int64_t ptr_sh = 0, da_sh = 0, in_sh = 0; /* running starts of the current channel */
        for (int c = 0; c < s->C; ++c) {
            const float *Wk = weights + ((int64_t)k * s->C + c) * s->kh * s->kw;
            if (ptr[ptr_sh] == ORC_NPC) { ++ptr_sh; continue; }
            for (int t = 0; t < s->kw; ++t) {
                if (!present[t]) continue;
                if (nop3 && t == 0) {
                    int n_first = ptr[ptr_sh + 1], n_both = ptr[ptr_sh + 2];
                    for (int x = 0; x < n_first; ++x)
                        conv_spmv(Ok, Wk, s, Oh, Ow, 0, da[da_sh + x], 0, in[in_sh + x]);
                    for (int x = n_first; x < n_both; ++x)
                        conv_spmv(Ok, Wk, s, Oh, Ow, 0, da[da_sh + x], Ow - 1, in[in_sh + x]);
                    ptr_sh += 3; da_sh += n_both; in_sh += n_both;
                    continue;
                }
                if (ptr[ptr_sh] == ORC_NPF) { ++ptr_sh; continue; }
                int pType = ptr[ptr_sh];
                int x = 0;        /* DA cursor inside this type */
                int64_t ti = 0;   /* IN cursor inside this type (differs from x for CPS) */
                for (int part = 0; part < Ow; ++part) {
                    int end = ptr[ptr_sh + 1 + part];
                    if (end < 0) end = x; /* no new column in this partition */
                    while (x < end) {
                        if (algo == 1 && t == top) {
                            int entry = in[in_sh + ti];
                            if (entry < 0) { /* singleton */
                                conv_spmv(Ok, Wk, s, Oh, Ow, pType, da[da_sh + x], part, -entry);
                                ++x; ++ti;
                            } else {         /* {first index, pattern} */
                                int pattern = in[in_sh + ti + 1];
                                int n = pattern_size(pattern);
                                for (int g = 0; g < n; ++g) {
                                    int index = entry + s->kw * pattern_row_offset(pattern, g);
                                    conv_spmv(Ok, Wk, s, Oh, Ow, pType, da[da_sh + x], part, index);
                                    ++x;
                                }
                                ti += 2;
                            }
                        } else {
                            conv_spmv(Ok, Wk, s, Oh, Ow, pType, da[da_sh + x], part, in[in_sh + x]);
                            ++x; ++ti;
                        }
                    }
                }
                ptr_sh += 1 + Ow; da_sh += x; in_sh += ti;
            }
        }
        for (int64_t i = 0; i < plane; ++i) out[(int64_t)k * plane + i] = (float)Ok[i];
    }
    free(Ok); free(cls); free(present);
    return ORC_OK;
}

/* Inverse of orc_encode: rebuilds the C x H x W map.  Cells that the encoding does not cover
 * stay zero. */
int orc_decode(const int32_t *ptr, const float *da, const int32_t *in, const orc_shape *s,
               int algo, float *act)
{
    if (!shape_ok(s)) return ORC_BAD_SHAPE;
    int Iw = s->W + 2 * s->pad_w;
    int32_t info[6];
    int32_t *cls = malloc(sizeof(int32_t) * Iw * 4), *p0 = cls + Iw, *what = p0 + Iw,
            *real = what + Iw;
    int32_t *present = malloc(sizeof(int32_t) * s->kw);
    orc_geometry(s, info, cls, p0, what, real, present);
    int Ow = info[3], nop3 = info[4], top = info[5];
    int rc = ORC_OK;
    memset(act, 0, sizeof(float) * (size_t)s->C * s->H * s->W);
    int64_t ip = 0, id = 0, ii = 0;
#define PUT(part, index, value)                                                         \
    do {                                                                                \
        int hh = (index) / s->kw - s->pad_h, jj = (part) * s->stride + (index) % s->kw - s->pad_w; \
        if (hh < 0 || hh >= s->H || jj < 0 || jj >= s->W) rc = ORC_BAD_SHAPE;          \
        else act[((int64_t)c * s->H + hh) * s->W + jj] = (value);                       \
    } while (0)
    for (int c = 0; c < s->C; ++c) {
        if (ptr[ip] == ORC_NPC) { ++ip; continue; }
        for (int t = 0; t < s->kw; ++t) {
            if (!present[t]) continue;
            if (nop3 && t == 0) {
                int n_first = ptr[ip + 1], n_both = ptr[ip + 2];
                for (int x = 0; x < n_both; ++x) PUT(x < n_first ? 0 : Ow - 1, in[ii + x], da[id + x]);
                ip += 3; id += n_both; ii += n_both;
                continue;
            }
            if (ptr[ip] == ORC_NPF) { ++ip; continue; }
            int x = 0; int64_t ti = 0;
            for (int part = 0; part < Ow; ++part) {
                int end = ptr[ip + 1 + part];
                if (end < 0) end = x;
                while (x < end) {
                    int entry = in[ii + ti];
                    if (algo == 1 && t == top && entry >= 0) {
                        int pattern = in[ii + ti + 1];
                        int n = pattern_size(pattern);
                        for (int g = 0; g < n; ++g) {
                            PUT(part, entry + s->kw * pattern_row_offset(pattern, g), da[id + x]);
                            ++x;
                        }
                        ti += 2;
                    } else {
                        PUT(part, entry < 0 ? -entry : entry, da[id + x]);
                        ++x; ++ti;
                    }
                }
            }
            ip += 1 + Ow; id += x; ii += ti;
        }
    }
#undef PUT
    free(cls); free(present);
    return rc;
}

/* ------------------------------------------------------------------------------------ */
/* Dense definitions.                                                                    */
/* ------------------------------------------------------------------------------------ */

/* Eq. 1 with batch 1: O(k,y,x) = sum_c sum_l sum_w Ipad(c, y*stride+l, x*stride+w) W(k,c,l,w),
 * cross-correlation (no kernel flip), pad_h zero rows above and below, pad_w zero columns left
 * and right. */
int orc_conv_direct(const float *act, const orc_shape *s, const float *weights, float *out)
{
    if (!shape_ok(s)) return ORC_BAD_SHAPE;
    int Oh = (s->H + 2 * s->pad_h - s->kh) / s->stride + 1;
    int Ow = (s->W + 2 * s->pad_w - s->kw) / s->stride + 1;
    for (int k = 0; k < s->K; ++k)
        for (int y = 0; y < Oh; ++y)
            for (int x = 0; x < Ow; ++x) {
                double acc = 0.0;
                for (int c = 0; c < s->C; ++c)
                    for (int l = 0; l < s->kh; ++l)
                        for (int w = 0; w < s->kw; ++w)
                            acc += (double)padded(act, s, c, y * s->stride + l, x * s->stride + w) *
                                   (double)weights[(((int64_t)k * s->C + c) * s->kh + l) * s->kw + w];
                out[((int64_t)k * Oh + y) * Ow + x] = (float)acc;
            }
    return ORC_OK;
}

/* im2col: lowered[(c*kh + l)*kw + w][y*Ow + x] = Ipad(c, y*stride + l, x*stride + w); the
 * lowered matrix has C*kh*kw rows and Oh*Ow columns (S_im2col elements, SI). */
int orc_im2col_lower(const float *act, const orc_shape *s, float *lowered)
{
    if (!shape_ok(s)) return ORC_BAD_SHAPE;
    int Oh = (s->H + 2 * s->pad_h - s->kh) / s->stride + 1;
    int Ow = (s->W + 2 * s->pad_w - s->kw) / s->stride + 1;
    int64_t N = (int64_t)Oh * Ow;
    for (int c = 0; c < s->C; ++c)
        for (int l = 0; l < s->kh; ++l)
            for (int w = 0; w < s->kw; ++w) {
                int64_t row = ((int64_t)c * s->kh + l) * s->kw + w;
                for (int y = 0; y < Oh; ++y)
                    for (int x = 0; x < Ow; ++x)
                        lowered[row * N + (int64_t)y * Ow + x] =
                            padded(act, s, c, y * s->stride + l, x * s->stride + w);
            }
    return ORC_OK;
}

/* out[M x N] = a[M x Kd] * b[Kd x N], row-major, double accumulation. */
int orc_gemm(const float *a, const float *b, int64_t M, int64_t N, int64_t Kd, float *out)
{
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t q = 0; q < Kd; ++q) acc += (double)a[i * Kd + q] * (double)b[q * N + j];
            out[i * N + j] = (float)acc;
        }
    return ORC_OK;
}

/* Section 3.5: per layer, total time of each method over the M offline inputs; "favour
 * time" (mode 0) picks the faster of im2col and CPO, "favour space" (mode 1) the faster of
 * im2col and CPS.  Returns 0 = im2col, 1 = CPO, 2 = CPS; im2col, the default method, keeps
 * a tie. */
int orc_select(const double *t_im2col, const double *t_cpo, const double *t_cps, int m, int mode)
{
    double a = 0.0, b = 0.0;
    for (int i = 0; i < m; ++i) {
        a += t_im2col[i];
        b += (mode == 0) ? t_cpo[i] : t_cps[i];
    }
    if (b < a) return mode == 0 ? 1 : 2;
    return 0;
}
