// Addressing of the operands of the phantom layer's matrix products.
//
// Every product of Eq. (ylq), Eq. (backprop) and Eq. (bpL)-(bpD) is a product of
// "concatenated" operands: the local block followed by one segment per peer
// (X | G_1 | ... | G_{p-1}  against  L | D_1 | ... | D_{p-1}), or the transpose
// of such an operand.  A View describes one logical 2-D operand [rows x cols]
// whose element (r, c) lives in one of two memory regions:
//   region 0 (the local block):   p0[r_off0 + c_off0]
//   region 1 (the peer segments): p1[r_off1 + c_off1]
// One of the two indices "decides" the region: below `split` it is region 0,
// above it the index is cut into (segment i, position w) and the segment is
// mapped to a memory slot (slot = i, or i+1 from the skipped slot on, which is
// how rank j passes over its own entry of a gathered [p, B, k] buffer).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace phantom {

struct Axis {
    int32_t decides;     // 1: this index selects the region
    int32_t split;       // decides: indices < split are region 0
    int32_t seg;         // decides: segment length in region 1 (>= 1)
    uint32_t magic;      // ceil(2^32 / seg): idx / seg == __umulhi(idx, magic) while idx * seg < 2^32 (seg >= 2)
    int64_t mult0;       // region 0 offset = idx * mult0
    int64_t mult1;       // region 1 offset = idx * mult1 (not deciding) or slot*seg_stride + w*mult1 (deciding)
    int64_t seg_stride;
};

struct View {
    void *p0;
    void *p1;
    int64_t g0, g1;      // element offsets added per group (rank held on this GPU)
    Axis r, c;
    int32_t skip0;       // skipped slot = skip0 + group * skip_g
    int32_t skip_g;
};

struct Loc {
    int64_t off0, off1;
    int32_t region;      // 0 / 1 if this index decides, else -1
};

__device__ __forceinline__ Loc locate(const Axis &ax, int idx, int skip)
{
    Loc l;
    if (!ax.decides) {
        l.off0 = (int64_t)idx * ax.mult0;
        l.off1 = (int64_t)idx * ax.mult1;
        l.region = -1;
    } else if (idx < ax.split) {
        l.off0 = (int64_t)idx * ax.mult0;
        l.off1 = 0;
        l.region = 0;
    } else {
        int t = idx - ax.split;
        int i = t / ax.seg;
        int w = t - i * ax.seg;
        int slot = i + (i >= skip ? 1 : 0);
        l.off0 = 0;
        l.off1 = (int64_t)slot * ax.seg_stride + (int64_t)w * ax.mult1;
        l.region = 1;
    }
    return l;
}

// element offset and region of (r, c) given the two locators
__device__ __forceinline__ int64_t join(const Loc &lr, const Loc &lc, int &region)
{
    region = lr.region > lc.region ? lr.region : lc.region;
    if (region < 0) region = 0;
    return region ? lr.off1 + lc.off1 : lr.off0 + lc.off0;
}

// ---- host-side constructors -------------------------------------------------
inline Axis axis_plain(int64_t mult0, int64_t mult1)
{
    Axis a{};
    a.decides = 0; a.split = 0; a.seg = 1; a.magic = 0; a.mult0 = mult0; a.mult1 = mult1; a.seg_stride = 0;
    return a;
}
inline Axis axis_seg(int split, int seg, int64_t mult0, int64_t mult1, int64_t seg_stride)
{
    Axis a{};
    a.decides = 1; a.split = split; a.seg = seg < 1 ? 1 : seg; a.mult0 = mult0; a.mult1 = mult1; a.seg_stride = seg_stride;
    a.magic = a.seg > 1 ? (uint32_t)((0x100000000ull + (uint32_t)a.seg - 1) / (uint32_t)a.seg) : 0u;
    return a;
}
constexpr int32_t NO_SKIP = 0x3fffffff;

// plain row-major [rows x cols], leading dimension ld
inline View view_plain(const void *p, int64_t ld, int64_t gstride)
{
    View v{};
    v.p0 = const_cast<void *>(p); v.p1 = nullptr; v.g0 = gstride; v.g1 = 0;
    v.r = axis_plain(ld, 0); v.c = axis_plain(1, 0);
    v.skip0 = NO_SKIP; v.skip_g = 0;
    return v;
}
// transpose of a plain row-major matrix: element (r, c) = p[c*ld + r]
inline View view_plain_t(const void *p, int64_t ld, int64_t gstride)
{
    View v = view_plain(p, ld, gstride);
    v.r = axis_plain(1, 0); v.c = axis_plain(ld, 0);
    return v;
}
// [rows x (head_cols + q*seg)]: head row-major with ld0, then q segments, segment i = row-major [rows x seg]
// at tail + slot(i)*seg_stride
inline View view_rowseg(const void *head, int64_t ld0, int head_cols, int64_t ghead,
                        const void *tail, int seg, int64_t seg_stride, int64_t gtail,
                        int32_t skip0 = NO_SKIP, int32_t skip_g = 0)
{
    View v{};
    v.p0 = const_cast<void *>(head); v.p1 = const_cast<void *>(tail); v.g0 = ghead; v.g1 = gtail;
    v.r = axis_plain(ld0, seg);
    v.c = axis_seg(head_cols, seg, 1, 1, seg_stride);
    v.skip0 = skip0; v.skip_g = skip_g;
    return v;
}
// transpose of view_rowseg: element (r, c) = rowseg(c, r)
inline View view_rowseg_t(const void *head, int64_t ld0, int head_cols, int64_t ghead,
                          const void *tail, int seg, int64_t seg_stride, int64_t gtail,
                          int32_t skip0 = NO_SKIP, int32_t skip_g = 0)
{
    View v = view_rowseg(head, ld0, head_cols, ghead, tail, seg, seg_stride, gtail, skip0, skip_g);
    Axis t = v.r; v.r = v.c; v.c = t;
    return v;
}

}  // namespace phantom

namespace phantom {
// two row-major matrices stacked along the reduction index and read transposed:
// element (r, c) = c < split ? top[c*ld0 + r] : bottom[(c-split)*ld1 + r]
inline View view_colstack(const void *top, int64_t ld0, int split, int64_t gtop,
                          const void *bottom, int64_t ld1, int bottom_rows, int64_t gbottom)
{
    View v{};
    v.p0 = const_cast<void *>(top); v.p1 = const_cast<void *>(bottom); v.g0 = gtop; v.g1 = gbottom;
    v.r = axis_plain(1, 1);
    v.c = axis_seg(split, bottom_rows, ld0, ld1, 0);
    v.skip0 = NO_SKIP; v.skip_g = 0;
    return v;
}
}  // namespace phantom
