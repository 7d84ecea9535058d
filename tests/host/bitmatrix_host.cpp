// Host build of the library's in-register bit-matrix transposes, for the CPU tests.
#include "../../paper_2502_18554_amd/csrc/zc_bitmatrix.h"

extern "C" {

// cls: 8, 16 or 32.  d: 32 two's complement deltas.  out: sign word, then planes 0..30
// (unused planes are zero).
void bm_planes_from_deltas(const int32_t* din, int cls, uint32_t* out) {
  int32_t d[32];
  for (int j = 0; j < 32; ++j) d[j] = din[j];
  for (int i = 0; i < 32; ++i) out[i] = 0;
  if (cls == 8) {
    uint32_t r[8];
    zc::planes_from_deltas8(d, r);
    out[0] = r[7];
    for (int p = 0; p < 7; ++p) out[1 + p] = r[p];
  } else if (cls == 816) {            // widths up to 7 by way of the paired 16-bit fields
    uint32_t f[16], r[8];
    for (int j = 0; j < 16; ++j) f[j] = zc::field16_pair(d[j], d[j + 16]);
    zc::planes8_from_fields16(f, r);
    out[0] = r[7];
    for (int p = 0; p < 7; ++p) out[1 + p] = r[p];
  } else if (cls == 16) {
    uint32_t r[16];
    zc::planes_from_deltas16(d, r);
    out[0] = r[15];
    for (int p = 0; p < 15; ++p) out[1 + p] = r[p];
  } else {
    uint32_t lo[16], hi[16];
    zc::planes_from_deltas32(d, lo, hi);
    out[0] = hi[15];
    for (int p = 0; p < 16; ++p) out[1 + p] = lo[p];
    for (int p = 0; p < 15; ++p) out[17 + p] = hi[p];
  }
}

void bm_deltas_from_planes(const uint32_t* in, int cls, int32_t* dout) {
  int32_t d[32];
  if (cls == 8) {
    uint32_t r[8];
    r[7] = in[0];
    for (int p = 0; p < 7; ++p) r[p] = in[1 + p];
    zc::deltas_from_planes8(r, d);
  } else if (cls == 16) {
    uint32_t r[16];
    r[15] = in[0];
    for (int p = 0; p < 15; ++p) r[p] = in[1 + p];
    zc::deltas_from_planes16(r, d);
  } else {
    uint32_t lo[16], hi[16];
    hi[15] = in[0];
    for (int p = 0; p < 16; ++p) lo[p] = in[1 + p];
    for (int p = 0; p < 15; ++p) hi[p] = in[17 + p];
    zc::deltas_from_planes32(lo, hi, d);
  }
  for (int j = 0; j < 32; ++j) dout[j] = d[j];
}

}  // extern "C"
