// zcref — reference CPU codec for the fZ-light error-bounded compressor and the
// compressed-Allreduce local reduce step of ZCCL (arXiv 2502.18554).
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single-threaded
// definition of what the GPU library must compute, written from the paper's prose
// (Section 3.3, the paragraph that introduces fZ-light: multi-layer blocks, fused
// quantisation + Lorenzo prediction, a 4-byte first-value outlier, sign bits, a one-byte
// code length "log max", fixed-length bit-shifting encoding, constant blocks; Section 3.1.2
// and the Sum aggregation equation of Section 3.2 for the reduce step and for one round of
// the ring reduce-scatter; the statement in Section 3.2 that a once-compressed point stays
// within the error bound).
// Only tests, the smoke check and the benchmark's CPU-baseline leg may call it.  It shares
// no code, header, table or constant with the HIP library.
//
// Every function here is pinned by tests/test_oracle_*.py against values worked by hand,
// closed forms, numpy/Python library routines and brute force; none is "parity unpinned".
//
// Stream layout (little endian).  The paper stores code lengths inline in a serial stream;
// here the same three kinds of data are laid out as dense tables so that block positions
// can be recomputed with a prefix sum:
//   0   u32  magic 0x314C435A ("ZCL1")
//   4   u16  version = 1
//   6   u8   block_log2 = 5        (32 values per block)
//   7   u8   guard_log2 = 6        (quantisation step shrunk by 2^-6, see quant_step)
//   8   u64  n                     (number of values)
//   16  u32  eb_bits               (binary32 pattern of the absolute error bound)
//   20  u32  nsum                  (how many original buffers are summed in this stream)
//   24  u64  total_bytes
//   32  width table   : nb bytes (code length of each block), zero padded to 16
//   ..  outlier table : nb int32 (first code of each block), zero padded to 16
//   ..  payload       : for every block with width w > 0, in block order:
//                       u32 sign word (bit j set iff delta j < 0), then w plane words,
//                       least significant plane first, bit j of plane p = bit p of |delta j|
//   nb = ceil(n / 32); a block of width 0 has no payload.
//
// Indexed variant (Section 3.5.2 keeps the compressed size of every chunk in an index at the
// front of the buffer, so that chunks can be handled one by one; here a chunk is a segment of
// 64 blocks): version = 2 when no block is wider than 15 bits, else 3, and between the header
// and the width table sits an index of nseg + 1 u32, nseg = ceil(nb / 64): entry i is the
// payload word offset of the first block of segment i, entry nseg the number of payload
// words; zero padded to 16 bytes.  A reader accepts version 3 without a wide block, but not
// version 2 with one.  zcref_set_indexed() chooses which variant is written and accepted.

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

enum Status : int {
  OK = 0, ERR_ARG = 1, ERR_CAPACITY = 2, ERR_FORMAT = 3, ERR_NONFINITE = 4,
  ERR_RANGE = 5, ERR_BOUND = 6, ERR_MISMATCH = 7
};

constexpr uint32_t kMagic = 0x314C435Au;
constexpr size_t kBlock = 32;
constexpr size_t kHeader = 32;
constexpr uint64_t kMaxN = uint64_t(1) << 31;
constexpr int64_t kMaxCode = (int64_t(1) << 30) - 1;
constexpr size_t kSegBlocks = 64;

bool g_indexed = false;       // which stream variant is written and accepted

size_t pad16(size_t v) { return (v + 15) / 16 * 16; }
size_t num_blocks(size_t n) { return (n + kBlock - 1) / kBlock; }
size_t num_segments(size_t nb) { return (nb + kSegBlocks - 1) / kSegBlocks; }
size_t index_bytes(size_t nb) { return g_indexed ? pad16(4 * (num_segments(nb) + 1)) : 0; }
size_t tables_end(size_t nb) { return kHeader + pad16(nb) + pad16(4 * nb) + index_bytes(nb); }

// Error bound accepted by the codec: finite, and at least 2^-96 so that no reconstructed
// value can be a binary32 subnormal.
bool eb_valid(float eb) { return std::isfinite(eb) && eb >= std::ldexp(1.0f, -96); }

// Quantisation step.  A step of exactly 2*eb leaves no room for the final rounding of the
// reconstructed value to binary32, so the step is 2*eb*(1 - 2^-6) = eb*63/32, which is
// exact in binary64 (24-bit significand times a 6-bit integer).
double quant_step(float eb) { return double(eb) * 63.0 / 32.0; }

// Code length of a block: number of bits of the largest delta magnitude (0 for 0).
// The paper writes "log max"; the bit count is the reading that keeps max = 1 distinct
// from a constant block.
unsigned bit_length(uint32_t m) {
  unsigned w = 0;
  while (m) { ++w; m >>= 1; }
  return w;
}

size_t payload_size(unsigned w) { return w == 0 ? 0 : 4 * (1 + size_t(w)); }

void put_u16(uint8_t* p, uint16_t v) { p[0] = uint8_t(v); p[1] = uint8_t(v >> 8); }
void put_u32(uint8_t* p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = uint8_t(v >> (8 * i)); }
void put_u64(uint8_t* p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = uint8_t(v >> (8 * i)); }
uint16_t get_u16(const uint8_t* p) { return uint16_t(p[0] | (p[1] << 8)); }
uint32_t get_u32(const uint8_t* p) { uint32_t v = 0; for (int i = 3; i >= 0; --i) v = (v << 8) | p[i]; return v; }
uint64_t get_u64(const uint8_t* p) { uint64_t v = 0; for (int i = 7; i >= 0; --i) v = (v << 8) | p[i]; return v; }

float bits_to_float(uint32_t b) { float f; std::memcpy(&f, &b, 4); return f; }
uint32_t float_to_bits(float f) { uint32_t b; std::memcpy(&b, &f, 4); return b; }

// ---- quantisation (Section 3.3: "fused quantization", the multiplication it mentions) ----
// One binary64 multiply by the reciprocal of the step, then round half to even.
// Returns OK, ERR_NONFINITE or ERR_RANGE for one value.
int quantize_one(float x, double inv, int32_t* q) {
  if (!std::isfinite(x)) return ERR_NONFINITE;
  double r = double(x) * inv;
  double t = std::nearbyint(r);   // default rounding mode: to nearest, ties to even
  if (std::fabs(t) > double(kMaxCode)) return ERR_RANGE;
  *q = int32_t(t);
  return OK;
}

float dequantize_one(int32_t q, double s) { return float(double(q) * s); }

// ---- encoding of integer codes into a stream (Section 3.3: Lorenzo prediction, sign bits,
// code length, fixed-length encoding, constant block) ----
int encode_codes(const int32_t* q, size_t n, uint32_t eb_bits, uint32_t nsum,
                 uint8_t* out, size_t out_cap, size_t* out_bytes) {
  const size_t nb = num_blocks(n);
  std::vector<uint8_t> width(nb);
  std::vector<int32_t> outlier(nb);
  std::vector<uint32_t> words;            // payload, block after block
  std::vector<uint32_t> seg_start;        // payload word offset of every 64th block
  bool wide = false;
  for (size_t b = 0; b < nb; ++b) {
    if (b % kSegBlocks == 0) seg_start.push_back(uint32_t(words.size()));
    int64_t Q[kBlock];
    for (size_t j = 0; j < kBlock; ++j) {
      size_t i = b * kBlock + j;
      Q[j] = q[i < n ? i : n - 1];        // tail of the last block repeats the last code
    }
    int64_t d[kBlock];
    d[0] = 0;                             // the first value travels as the outlier
    for (size_t j = 1; j < kBlock; ++j) d[j] = Q[j] - Q[j - 1];
    uint32_t maxmag = 0;
    for (size_t j = 0; j < kBlock; ++j) {
      uint32_t mag = uint32_t(d[j] < 0 ? -d[j] : d[j]);
      if (mag > maxmag) maxmag = mag;
    }
    unsigned w = bit_length(maxmag);
    if (w > 15) wide = true;
    width[b] = uint8_t(w);
    outlier[b] = int32_t(Q[0]);
    if (w == 0) continue;
    uint32_t sign = 0;
    for (size_t j = 0; j < kBlock; ++j) if (d[j] < 0) sign |= uint32_t(1) << j;
    words.push_back(sign);
    for (unsigned p = 0; p < w; ++p) {
      uint32_t plane = 0;
      for (size_t j = 0; j < kBlock; ++j) {
        uint32_t mag = uint32_t(d[j] < 0 ? -d[j] : d[j]);
        plane |= ((mag >> p) & 1u) << j;
      }
      words.push_back(plane);
    }
  }
  const size_t total = tables_end(nb) + 4 * words.size();
  if (out_bytes) *out_bytes = total;
  if (total > out_cap) return ERR_CAPACITY;
  std::memset(out, 0, tables_end(nb));
  put_u32(out + 0, kMagic);
  put_u16(out + 4, g_indexed ? (wide ? 3 : 2) : 1);
  out[6] = 5;
  out[7] = 6;
  put_u64(out + 8, n);
  put_u32(out + 16, eb_bits);
  put_u32(out + 20, nsum);
  put_u64(out + 24, total);
  uint8_t* ix = out + kHeader;
  uint8_t* wt = ix + index_bytes(nb);
  uint8_t* ot = wt + pad16(nb);
  uint8_t* pl = ot + pad16(4 * nb);
  if (g_indexed) {
    seg_start.push_back(uint32_t(words.size()));      // the closing entry: all payload words
    for (size_t i = 0; i < seg_start.size(); ++i) put_u32(ix + 4 * i, seg_start[i]);
  }
  for (size_t b = 0; b < nb; ++b) wt[b] = width[b];
  for (size_t b = 0; b < nb; ++b) put_u32(ot + 4 * b, uint32_t(outlier[b]));
  for (size_t i = 0; i < words.size(); ++i) put_u32(pl + 4 * i, words[i]);
  return OK;
}

struct Parsed {
  uint64_t n = 0, total = 0;
  uint32_t eb_bits = 0, nsum = 0;
  size_t nb = 0;
  const uint8_t* widths = nullptr;
  const uint8_t* outliers = nullptr;
  const uint8_t* payload = nullptr;
  std::vector<uint64_t> off;              // byte offset of each block inside the payload
};

// Header and table validation shared by decompress, reduce and inspect.
int parse_stream(const uint8_t* in, size_t in_bytes, Parsed* ps) {
  if (in_bytes < kHeader) return ERR_FORMAT;
  const unsigned version = get_u16(in + 4);
  if (get_u32(in) != kMagic || in[6] != 5 || in[7] != 6) return ERR_FORMAT;
  if (g_indexed ? (version != 2 && version != 3) : version != 1) return ERR_FORMAT;
  ps->n = get_u64(in + 8);
  ps->eb_bits = get_u32(in + 16);
  ps->nsum = get_u32(in + 20);
  ps->total = get_u64(in + 24);
  if (ps->n > kMaxN) return ERR_FORMAT;
  if (!eb_valid(bits_to_float(ps->eb_bits))) return ERR_FORMAT;
  if (ps->nsum < 1) return ERR_FORMAT;
  ps->nb = num_blocks(size_t(ps->n));
  if (ps->total > in_bytes || ps->total < tables_end(ps->nb)) return ERR_FORMAT;
  const uint8_t* index = in + kHeader;
  ps->widths = index + index_bytes(ps->nb);
  ps->outliers = ps->widths + pad16(ps->nb);
  ps->payload = ps->outliers + pad16(4 * ps->nb);
  ps->off.resize(ps->nb);
  uint64_t acc = 0;
  bool wide = false;
  for (size_t b = 0; b < ps->nb; ++b) {
    if (ps->widths[b] > 31) return ERR_FORMAT;
    if (ps->widths[b] > 15) wide = true;
    // the index must say what the width table implies
    if (g_indexed && b % kSegBlocks == 0 && get_u32(index + 4 * (b / kSegBlocks)) != acc / 4) return ERR_FORMAT;
    ps->off[b] = acc;                     // exclusive prefix sum of the block sizes
    acc += payload_size(ps->widths[b]);
  }
  if (g_indexed && get_u32(index + 4 * num_segments(ps->nb)) != acc / 4) return ERR_FORMAT;
  if (g_indexed && version == 2 && wide) return ERR_FORMAT;
  if (tables_end(ps->nb) + acc != ps->total) return ERR_FORMAT;
  return OK;
}

// Integer codes of a parsed stream: undo the fixed-length encoding and the Lorenzo chain.
// Arithmetic is modulo 2^32, so a hostile stream cannot cause undefined behaviour.
void decode_codes(const Parsed& ps, int32_t* q) {
  for (size_t b = 0; b < ps.nb; ++b) {
    unsigned w = ps.widths[b];
    const uint8_t* p = ps.payload + ps.off[b];
    uint32_t cur = get_u32(ps.outliers + 4 * b);
    for (size_t j = 0; j < kBlock; ++j) {
      size_t i = b * kBlock + j;
      if (i >= ps.n) break;
      if (w > 0) {
        uint32_t sign = get_u32(p);
        uint32_t mag = 0;
        for (unsigned pl = 0; pl < w; ++pl) mag |= ((get_u32(p + 4 * (1 + pl)) >> j) & 1u) << pl;
        cur += ((sign >> j) & 1u) ? (0u - mag) : mag;
      }
      q[i] = int32_t(cur);
    }
  }
}

}  // namespace

extern "C" {

// Which stream variant the functions below write and accept: 0 plain, 1 indexed.
void zcref_set_indexed(int on) { g_indexed = on != 0; }

// Worst-case stream size of the chosen variant: every block at width 31 costs 1 + 4 + 128 bytes.
size_t zcref_compress_bound(size_t n) {
  size_t nb = num_blocks(n);
  return tables_end(nb) + 128 * nb;
}

// Integer codes only (Section 3.3, quantisation stage).  q has room for n values.
int zcref_quantize(const float* in, size_t n, float abs_eb, int32_t* q) {
  if (!eb_valid(abs_eb) || n > kMaxN || (n && (!in || !q))) return ERR_ARG;
  const double inv = 1.0 / quant_step(abs_eb);
  int worst = OK;
  for (size_t i = 0; i < n; ++i) {
    int32_t c = 0;
    int st = quantize_one(in[i], inv, &c);
    q[i] = c;
    if (st == ERR_NONFINITE) worst = ERR_NONFINITE;
    else if (st == ERR_RANGE && worst != ERR_NONFINITE) worst = ERR_RANGE;
  }
  return worst;
}

// Encode given integer codes (test helper for widths that no in-domain input reaches).
int zcref_encode_codes(const int32_t* q, size_t n, float abs_eb, uint32_t nsum,
                       void* out, size_t out_cap, size_t* out_bytes) {
  if (!eb_valid(abs_eb) || n > kMaxN || nsum < 1 || (n && !q) || !out) return ERR_ARG;
  return encode_codes(q, n, float_to_bits(abs_eb), nsum, static_cast<uint8_t*>(out), out_cap, out_bytes);
}

// Compress n binary32 values under an absolute error bound (Section 3.3).
// Status precedence: ARG, NONFINITE, RANGE, CAPACITY, BOUND.  On BOUND the stream is
// complete: some reconstructed value misses the bound because the input lies outside the
// domain max|x| <= 2^18 * eb in which the guard makes the bound certain (Section 3.2:
// every point of a once-compressed chunk stays within the bound).
int zcref_compress(const float* in, size_t n, float abs_eb,
                   void* out, size_t out_cap, size_t* out_bytes) {
  if (!eb_valid(abs_eb) || n > kMaxN || (n && !in) || !out) return ERR_ARG;
  const double ebd = double(abs_eb);
  const double s = quant_step(abs_eb);
  std::vector<int32_t> q(n);
  int st = zcref_quantize(in, n, abs_eb, q.data());
  if (st != OK) return st;
  st = encode_codes(q.data(), n, float_to_bits(abs_eb), 1, static_cast<uint8_t*>(out), out_cap, out_bytes);
  if (st != OK) return st;
  for (size_t i = 0; i < n; ++i) {
    double err = std::fabs(double(in[i]) - double(dequantize_one(q[i], s)));
    if (!(err <= ebd)) return ERR_BOUND;
  }
  return OK;
}

// Decompress a stream to binary32 values: x' = float(double(code) * step).
// Status precedence: ARG, FORMAT, CAPACITY.
int zcref_decompress(const void* in, size_t in_bytes, float* out, size_t out_cap_elems, size_t* n_out) {
  if (!in) return ERR_ARG;
  Parsed ps;
  int st = parse_stream(static_cast<const uint8_t*>(in), in_bytes, &ps);
  if (st != OK) return st;
  if (n_out) *n_out = size_t(ps.n);
  if (ps.n > out_cap_elems) return ERR_CAPACITY;
  if (ps.n && !out) return ERR_ARG;
  std::vector<int32_t> q(ps.n);
  decode_codes(ps, q.data());
  const double s = quant_step(bits_to_float(ps.eb_bits));
  for (size_t i = 0; i < ps.n; ++i) out[i] = dequantize_one(q[i], s);
  return OK;
}

// A chunk of a stream on its own (Section 3.5.2 handles a buffer chunk by chunk, so that one
// chunk can be decompressed while the next is still on its way): the values
// [first_value, first_value + count) of the stream, first_value a multiple of 2048 (a segment
// of 64 blocks), cut off at the stream's end.  By definition the same values as a slice of
// the whole decompression.  *n_out = how many values that is.
// Status: ARG (first_value not a multiple of 2048, or beyond n), FORMAT, CAPACITY.
int zcref_decompress_range(const void* in, size_t in_bytes, size_t first_value, size_t count, float* out,
                           size_t out_cap_elems, size_t* n_out) {
  if (!in || first_value % (kSegBlocks * kBlock) != 0) return ERR_ARG;
  Parsed ps;
  int st = parse_stream(static_cast<const uint8_t*>(in), in_bytes, &ps);
  if (st != OK) return st;
  if (first_value > ps.n) return ERR_ARG;
  const size_t m = std::min<uint64_t>(count, ps.n - first_value);
  if (n_out) *n_out = m;
  if (m > out_cap_elems) return ERR_CAPACITY;
  if (m && !out) return ERR_ARG;
  std::vector<int32_t> q(ps.n);
  decode_codes(ps, q.data());
  const double s = quant_step(bits_to_float(ps.eb_bits));
  for (size_t i = 0; i < m; ++i) out[i] = dequantize_one(q[first_value + i], s);
  return OK;
}

// Look inside a stream: integer codes (n), code lengths (nb), payload byte offsets (nb).
// Any of the three outputs may be null.
int zcref_inspect(const void* in, size_t in_bytes, int32_t* q, uint8_t* widths, uint64_t* offsets) {
  if (!in) return ERR_ARG;
  Parsed ps;
  int st = parse_stream(static_cast<const uint8_t*>(in), in_bytes, &ps);
  if (st != OK) return st;
  if (q) decode_codes(ps, q);
  if (widths) std::memcpy(widths, ps.widths, ps.nb);
  if (offsets) for (size_t b = 0; b < ps.nb; ++b) offsets[b] = ps.off[b];
  return OK;
}

// Local step of the compressed Allreduce (Section 3.1.2; aggregation functions of Section 3.2):
// k compressed operands on one common grid -> the compressed aggregate.  Decode every operand
// to its integer codes, combine them value by value, encode the results.
// op 0, Sum: the codes are added.  Because all operands share the step, the sum of grid points
// is a grid point and no new quantisation error appears.
// op 1 / 2, Max / Min: the largest / smallest code.  The quantiser is monotone, so the largest
// code is the code of the largest value: the result is the stream of the elementwise maximum
// (minimum) of the original buffers compressed once, within one error bound of it whatever k is.
// nsum of the result is the sum of the operands' nsum (the number of buffers it stands for).
// Status precedence: ARG, FORMAT, MISMATCH, RANGE, CAPACITY.
int zcref_reduce_op(const void* const* chunks, const size_t* chunk_bytes, int k, int op,
                    void* out, size_t out_cap, size_t* out_bytes) {
  if (k < 1 || !chunks || !chunk_bytes || !out || op < 0 || op > 2) return ERR_ARG;
  for (int i = 0; i < k; ++i) if (!chunks[i]) return ERR_ARG;
  std::vector<Parsed> ps(k);
  for (int i = 0; i < k; ++i) {
    int st = parse_stream(static_cast<const uint8_t*>(chunks[i]), chunk_bytes[i], &ps[i]);
    if (st != OK) return st;
  }
  uint64_t nsum = 0;
  for (int i = 0; i < k; ++i) {
    if (ps[i].n != ps[0].n || ps[i].eb_bits != ps[0].eb_bits) return ERR_MISMATCH;
    nsum += ps[i].nsum;
  }
  if (nsum > 0xFFFFFFFFull) return ERR_RANGE;
  const size_t n = size_t(ps[0].n);
  std::vector<int64_t> total(n, 0);
  std::vector<int32_t> q(n);
  for (int i = 0; i < k; ++i) {
    decode_codes(ps[i], q.data());
    for (size_t j = 0; j < n; ++j) {
      if (op == 0) total[j] += q[j];
      else if (i == 0) total[j] = q[j];
      else if (op == 1) total[j] = std::max<int64_t>(total[j], q[j]);
      else total[j] = std::min<int64_t>(total[j], q[j]);
    }
  }
  for (size_t j = 0; j < n; ++j) {
    if (total[j] > kMaxCode || total[j] < -kMaxCode) return ERR_RANGE;
    q[j] = int32_t(total[j]);
  }
  return encode_codes(q.data(), n, ps[0].eb_bits, uint32_t(nsum), static_cast<uint8_t*>(out), out_cap, out_bytes);
}

int zcref_reduce(const void* const* chunks, const size_t* chunk_bytes, int k,
                 void* out, size_t out_cap, size_t* out_bytes) {
  return zcref_reduce_op(chunks, chunk_bytes, k, 0, out, out_cap, out_bytes);
}

// One round of the ring reduce-scatter (Section 3.1.2: per round a received compressed chunk
// is decompressed, reduced with the local chunk and compressed again; the Sum chain of
// Section 3.2 adds one bounded error per such round).  The received stream is decoded to
// binary32 values, the local uncompressed values are added in binary32, and the sums are
// compressed under the stream's own bound.  nsum grows by one.
// op: 0 Sum, 1 Max, 2 Min (the aggregation functions of Section 3.2; for Max and Min the
// round keeps the larger, or smaller, of the decoded and the local value).
// Status precedence: ARG, FORMAT, MISMATCH (n_local differs from the stream's n), NONFINITE,
// RANGE, CAPACITY, BOUND (measured against the binary32 values that were compressed).
int zcref_reduce_step_op(const void* in, size_t in_bytes, const float* local, size_t n_local, int op,
                         void* out, size_t out_cap, size_t* out_bytes) {
  if (!in || !out || op < 0 || op > 2) return ERR_ARG;
  Parsed ps;
  int st = parse_stream(static_cast<const uint8_t*>(in), in_bytes, &ps);
  if (st != OK) return st;
  if (ps.n != n_local) return ERR_MISMATCH;
  if (ps.n && !local) return ERR_ARG;
  if (uint64_t(ps.nsum) + 1 > 0xFFFFFFFFull) return ERR_RANGE;
  const size_t n = size_t(ps.n);
  const float eb = bits_to_float(ps.eb_bits);
  const double s = quant_step(eb);
  std::vector<int32_t> q(n);
  decode_codes(ps, q.data());
  std::vector<float> y(n);
  for (size_t i = 0; i < n; ++i) {
    const float a = dequantize_one(q[i], s), b = local[i];
    if (op == 0) y[i] = a + b;
    else if (!std::isfinite(b)) y[i] = b;          // a NaN or an infinity is an error whatever the comparison says
    else if (op == 1) y[i] = a > b ? a : b;
    else y[i] = a < b ? a : b;
  }
  st = zcref_quantize(y.data(), n, eb, q.data());
  if (st != OK) return st;
  st = encode_codes(q.data(), n, ps.eb_bits, ps.nsum + 1, static_cast<uint8_t*>(out), out_cap, out_bytes);
  if (st != OK) return st;
  for (size_t i = 0; i < n; ++i) {
    double err = std::fabs(double(y[i]) - double(dequantize_one(q[i], s)));
    if (!(err <= double(eb))) return ERR_BOUND;
  }
  return OK;
}

int zcref_reduce_step(const void* in, size_t in_bytes, const float* local, size_t n_local,
                      void* out, size_t out_cap, size_t* out_bytes) {
  return zcref_reduce_step_op(in, in_bytes, local, n_local, 0, out, out_cap, out_bytes);
}

// The Average aggregation of Section 3.2: a stream that holds the sum of nsum buffers is
// decoded to that sum divided by nsum.  x' = float((double(q) * s) * r) with r = 1.0 / nsum,
// one binary64 division for the whole stream.  Status as zcref_decompress.
int zcref_decompress_average(const void* in, size_t in_bytes, float* out, size_t out_cap_elems, size_t* n_out) {
  if (!in) return ERR_ARG;
  Parsed ps;
  int st = parse_stream(static_cast<const uint8_t*>(in), in_bytes, &ps);
  if (st != OK) return st;
  if (n_out) *n_out = size_t(ps.n);
  if (ps.n > out_cap_elems) return ERR_CAPACITY;
  if (ps.n && !out) return ERR_ARG;
  std::vector<int32_t> q(ps.n);
  decode_codes(ps, q.data());
  const double s = quant_step(bits_to_float(ps.eb_bits));
  const double r = 1.0 / double(ps.nsum);
  for (size_t i = 0; i < ps.n; ++i) out[i] = float((double(q[i]) * s) * r);
  return OK;
}

// Quality of a reconstruction `test` against its original `ref` (the measures of Section 3.3's
// quality table and of Section 4.6): out[0] = max |ref - test|, out[1] = sum of squared
// differences, out[2] = min(ref), out[3] = max(ref), all in binary64 and in index order.
// With range = max - min: RMSE = sqrt(out[1] / n), NRMSE = RMSE / range, PSNR = 20 log10(range / RMSE).
// n = 0 gives {0, 0, +inf, -inf}.  Status: ARG.
int zcref_quality(const float* ref, const float* test, size_t n, double* out) {
  if (!out || (n && (!ref || !test))) return ERR_ARG;
  double worst = 0.0, sse = 0.0, lo = INFINITY, hi = -INFINITY;
  for (size_t i = 0; i < n; ++i) {
    const double d = double(ref[i]) - double(test[i]);
    const double a = std::fabs(d);
    if (a > worst || std::isnan(a)) worst = a;
    sse += d * d;
    if (double(ref[i]) < lo) lo = ref[i];
    if (double(ref[i]) > hi) hi = ref[i];
  }
  out[0] = worst; out[1] = sse; out[2] = lo; out[3] = hi;
  return OK;
}

}  // extern "C"
