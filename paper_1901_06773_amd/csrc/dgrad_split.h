// Host-side arithmetic that cuts the data gradient of a strided convolution into stride-1
// convolutions, one per residue class of the dx position (no device code here).
#pragma once
#include <cstddef>

namespace acc {

// The dx positions (y0 + stride*p, x0 + stride*q), p < P, q < Q, receive only the filter taps
// r = r0 + j*stride, t = t0 + j'*stride; over them dx is a stride-1 convolution of dy with the
// nr x ns sub-filter  wt[ci][r'][t'][co] = w[co][r0 + (nr-1-r')*stride][t0 + (ns-1-t')*stride][ci]
// padded by pad_y / pad_x.  wt_offset: byte offset of the sub-filter in one buffer that holds
// those of all parts (256-byte aligned).
struct DgradPart {
  int y0, x0, p, q;
  int nr, ns, r0, t0;
  int pad_y, pad_x;
  size_t wt_offset;
};
enum { kMaxDgradParts = 16 };

// Lists the residue classes that have at least one tap (at most stride^2 <= kMaxDgradParts) for
// an h x wd input.  Classes without taps get no contribution (*covers_all = false: dx must be
// cleared first unless it is accumulated into).  Returns the number of parts, or -1 if the
// shape is not supported (stride > 4, or a part that would need negative padding).
// elem_size: bytes per filter element.
inline int dgrad_split(int h, int wd, int cin, int cout, int r, int s, int stride, int pad, int elem_size,
                       DgradPart* parts, bool* covers_all, size_t* wt_bytes) {
  if (h <= 0 || wd <= 0 || cin <= 0 || cout <= 0 || r <= 0 || s <= 0 || stride <= 0 || stride > 4 || pad < 0 ||
      elem_size <= 0)
    return -1;
  // one axis: residue a of the dx coordinate -> taps r0, r0+stride, ...; dy coordinate of tap j at
  // dx = a + stride*p is p + d - j with d = (a + pad - r0) / stride
  struct Axis { int count, taps, tap0, padding; };
  auto axis = [&](int size, int taps_total, int a, Axis* ax) {
    ax->count = a < size ? (size - a + stride - 1) / stride : 0;
    ax->tap0 = (a + pad) % stride;
    ax->taps = ax->tap0 < taps_total ? (taps_total - ax->tap0 + stride - 1) / stride : 0;
    const int d = (a + pad - ax->tap0) / stride;
    ax->padding = ax->taps - 1 - d;
  };
  int n = 0;
  size_t off = 0;
  bool all = true;
  for (int a = 0; a < stride; ++a)
    for (int b = 0; b < stride; ++b) {
      Axis ay, ax;
      axis(h, r, a, &ay);
      axis(wd, s, b, &ax);
      if (ay.count == 0 || ax.count == 0) continue;        // no such dx position
      if (ay.taps == 0 || ax.taps == 0) { all = false; continue; }
      if (ay.padding < 0 || ax.padding < 0) return -1;
      DgradPart& pt = parts[n++];
      pt.y0 = a; pt.x0 = b; pt.p = ay.count; pt.q = ax.count;
      pt.nr = ay.taps; pt.ns = ax.taps; pt.r0 = ay.tap0; pt.t0 = ax.tap0;
      pt.pad_y = ay.padding; pt.pad_x = ax.padding;
      pt.wt_offset = off;
      off += ((size_t)cin * cout * pt.nr * pt.ns * (size_t)elem_size + 255) & ~(size_t)255;
    }
  if (covers_all) *covers_all = all;
  if (wt_bytes) *wt_bytes = off;
  return n;
}

}  // namespace acc
