/* zc — fZ-light error-bounded lossy compression and the compressed-Allreduce local step,
 * hand-written for AMD MI355X (gfx950).  C ABI; every pointer named d_* is DEVICE memory,
 * everything else is host memory.  The library allocates no device memory and keeps no
 * settings: what varies between calls is said by each call's arguments (`flags`), and the
 * caller owns inputs, outputs and the workspace.  (The only thing that lives between calls is
 * the optional kernel timer of zc_profile_enable, a measurement aid.)
 *
 * Method: ZCCL, arXiv 2502.18554.  fZ-light is described in Section 3.3 (block partition,
 * fused quantisation + 1D Lorenzo prediction, first value kept as a 4-byte outlier, sign
 * bits, one-byte code length "log max", fixed-length bit-shifting encoding, constant
 * blocks).  The reduce step is the per-round "decompress, reduce, recompress" of the
 * collective computation framework (Section 3.1.2) with the Sum aggregation of Section 3.2.
 *
 * Plain stream (little endian), n values, nb = ceil(n / 32) blocks of 32 values:
 *    0  u32 magic 0x314C435A   4  u16 version 1   6  u8 block_log2 5   7  u8 guard_log2 6
 *    8  u64 n                 16  u32 eb_bits (binary32 pattern of abs_eb)
 *   20  u32 nsum (1 after zc_compress, sum of the operands' nsum after a reduce)
 *   24  u64 total_bytes
 *   32  width table   nb bytes, zero padded to a multiple of 16
 *   ..  outlier table nb int32 (first code of each block), zero padded to a multiple of 16
 *   ..  payload: for each block of width w > 0, in block order, (1 + w) u32 words:
 *       sign word (bit j set iff delta j < 0), then planes p = 0..w-1, least significant
 *       first, bit j of plane p = bit p of |delta j|.  A block of width 0 has no payload.
 *  Codes: q = rint(x / s) with s = abs_eb * 63/32 (binary64, round half to even);
 *  deltas: d0 = 0, dj = qj - q(j-1) inside a block; the last block is padded with its last
 *  code; width = bit count of max |dj|; reconstruction x' = (float)((double)q * s).
 *
 * Indexed stream (the default of every call): the same with the chunk size table of Section
 * 3.5.2 in front of the data (the compressed size of every chunk is kept ahead of the data so
 * that a chunk can be taken up without looking at the rest).  Here a chunk is a segment of 64
 * blocks (2048 values), the share of one wave.  Version is 2, or 3 when some block is wider
 * than 15 bits, and between the header and the width table sits an index of nseg + 1 u32,
 * nseg = ceil(nb / 64), zero padded to a multiple of 16 bytes: entry i is the payload word
 * offset of block 64 i, entry nseg the number of payload words.  Everything else is as above.
 * Producers write the index as a by-product of placing their payload; consumers read their
 * segments' positions from it instead of first summing the width table, which makes every
 * call on indexed streams a single kernel launch.  Costs 4 bytes per 2048 values.
 *
 * flags (an OR of the flag bits below; 0 = the defaults):
 *   ZC_STREAM_PLAIN     every stream of this call, read or written, is a plain stream.  A
 *                       stream of the other variant is ZC_ERR_FORMAT.  Consumers of plain
 *                       streams run two small kernels ahead of their main kernel to sum the
 *                       width table.
 *   ZC_TILES_BY_TICKET  (calls that write a stream) tiles of 256 or 512 blocks are claimed by
 *                       workgroups with atomic tickets instead of being taken by workgroup id.
 *                       The single-pass placement of the output (a device-wide exclusive sum of
 *                       block sizes by look-back) needs every tile before a tile in work to be
 *                       in work or finished.  By workgroup id that rests on the GPU starting the
 *                       workgroups of a launch in increasing id order, which is how its
 *                       dispatcher works but not an architectural promise; tickets need no
 *                       such assumption and cost an atomic round trip per workgroup (about 7 % more
 *                       time on the 512^3 benchmark step; every XCD must receive workgroups of
 *                       the launch, i.e. no CU mask that leaves one out).  Either way a wait that does
 *                       not end within 2^20 polls ends the call with ZC_ERR_HIP, never in a hang.
 *   ZC_CHAINS_COHERENT  (calls that write a stream) the look-back reads every tile descriptor
 *                       with device-coherent loads.  By default a tile reads the descriptors of
 *                       the tiles 8, 16, ... before it through the L2 cache of its XCD, which is
 *                       faster and is where they are written when workgroup ids (and tickets) go
 *                       round the 8 XCDs; where they do not, such a read may find nothing new for
 *                       a while, and the tile turns to coherent loads by itself after 16 tries.
 *                       The flag skips the tries.  Results are the same either way.
 * An index that contradicts the width table, a width above 31, or a width above 15 in a
 * version-2 stream is ZC_ERR_FORMAT, which the kernels find as they use each segment: the
 * output of such a call is unspecified.
 *
 * Calls are asynchronous on the given HIP stream unless the last size pointer is non-NULL,
 * in which case the call synchronises the stream and returns the final status and size.
 * In the asynchronous form the status and size are collected later with zc_finish on the
 * same workspace.  One workspace serves one call at a time; its content between calls is
 * irrelevant (nothing in it ever needs clearing).  Calls on different workspaces may run
 * concurrently, on several HIP streams or from several host threads.
 */
#ifndef ZC_H
#define ZC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ZC_OK = 0,
  ZC_ERR_ARG = 1,       /* null pointer, misaligned buffer, abs_eb not finite / < 2^-96, n > 2^31, k out of range, unknown flag or op, workspace too small */
  ZC_ERR_CAPACITY = 2,  /* output buffer too small; nothing is written past its end */
  ZC_ERR_FORMAT = 3,    /* not a valid stream: header fields, truncated, width > 31, sizes do not add up, the other stream variant, an index that contradicts the widths */
  ZC_ERR_NONFINITE = 4, /* NaN or Inf in the input */
  ZC_ERR_RANGE = 5,     /* a code (or a sum of codes) exceeds 2^30 - 1 in magnitude */
  ZC_ERR_BOUND = 6,     /* some |x - x'| > abs_eb: input outside max|x| <= 2^18 abs_eb; the stream is still complete and decodable */
  ZC_ERR_MISMATCH = 7,  /* reduce operands differ in n or abs_eb */
  ZC_ERR_HIP = 8        /* a HIP runtime call failed, or an internal wait ran out */
} zc_status;

#define ZC_MAX_N (1ull << 31)
#define ZC_MAX_K 64

#define ZC_STREAM_PLAIN 1u
#define ZC_TILES_BY_TICKET 2u
#define ZC_CHAINS_COHERENT 4u

/* Worst-case stream size in bytes for n values (every block at width 31: 133 B per 128 B):
 * of the default (indexed) variant, or of the variant that flags name. */
size_t zc_compress_bound(size_t n);
size_t zc_compress_bound_ex(size_t n, unsigned flags);

/* Workspace bytes needed by any call on at most n_max values with at most k_max reduce
 * operands (k_max < 1 is taken as 1).  The workspace is device memory, 16-byte aligned;
 * its content between calls is irrelevant. */
size_t zc_workspace_bytes(size_t n_max, int k_max);

/* fZ-light compression (Section 3.3).  d_in: n binary32 values, 16-byte aligned.
 * d_out: out_cap bytes, 16-byte aligned, receives the stream.  out_bytes (host, may be NULL):
 * receives total_bytes, also when the status is ZC_ERR_CAPACITY or ZC_ERR_BOUND.
 * Errors: ARG, NONFINITE, RANGE, CAPACITY, BOUND (in this order of precedence), HIP.
 * On any error except BOUND the content of d_out is unspecified.
 * zc_compress is zc_compress_ex with flags 0. */
int zc_compress(const float* d_in, size_t n, float abs_eb,
                void* d_out, size_t out_cap, size_t* out_bytes,
                void* d_ws, size_t ws_bytes, void* hip_stream);
int zc_compress_ex(const float* d_in, size_t n, float abs_eb,
                   void* d_out, size_t out_cap, size_t* out_bytes,
                   void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* zc_compress for callers that cannot allocate device memory or bring a workspace along: code
 * whose stream is being captured into a HIP graph, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and errors as zc_compress, without d_ws and ws_bytes: the
 * workspace is an array in the library's own device image (about 2.4 MB on every GPU the library
 * runs on, held until the process ends), sized for n <= ZC_NOALLOC_MAX_N; a larger n is
 * ZC_ERR_ARG.  The call allocates nothing, on the device or through any library.  The GPU of
 * hip_stream must be the current device.  All calls on one GPU share that one array: calls that
 * overlap in time on one GPU (two host threads, two HIP streams) race on it and are not
 * allowed; calls one after the other on one stream are fine, nothing in the array needs clearing.
 * The first call on a GPU looks up the array's address (hipGetSymbolAddress): make it before a
 * capture starts.  The asynchronous form (out_bytes NULL) is completed by zc_finish(NULL, ...). */
#define ZC_NOALLOC_MAX_N (1ull << 27)
int zc_compress_noalloc(const float* d_in, size_t n, float abs_eb,
                        void* d_out, size_t out_cap, size_t* out_bytes, void* hip_stream);

/* zc_compress in parts (Section 3.5.2 produces a buffer chunk by chunk, so that a chunk can be
 * sent while the next one is being compressed): this call compresses the values
 * [first_value, first_value + count) of the n values at d_in into the stream at d_out.  The
 * parts of one stream are given in ascending order, without gaps, to the same d_out and d_ws
 * with the same flags, on one HIP stream (or ordered by events), starting with first_value = 0,
 * which also writes the header; first_value and count are multiples of 16384, except that the
 * last part ends at n.  n and abs_eb are the same in every part; only the values of the
 * part need to be in place at d_in when it is given.  Between the parts the workspace must not
 * be used for anything else.  After a part has run, the stream's tables
 * and payload up to its end are final, and out_bytes (or zc_finish) tells how many bytes of the
 * stream that is; of an indexed stream header and index then describe
 * a stream that can be read up to there (zc_decompress_range) while later parts are produced.
 * After the last part the stream is the one zc_compress writes.  Errors of all parts
 * accumulate in the workspace.  Errors: as zc_compress, and ARG for a part that is not as above. */
int zc_compress_part(const float* d_in, size_t n, float abs_eb, size_t first_value, size_t count,
                     void* d_out, size_t out_cap, size_t* out_bytes,
                     void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* fZ-light decompression (inverse of the stages of Section 3.3).  d_in: stream of in_bytes
 * bytes (trailing bytes beyond total_bytes are ignored), 16-byte aligned.  d_out: room for
 * out_cap_elems binary32 values, 16-byte aligned.  n_out (host, may be NULL): receives n.
 * Errors: ARG, FORMAT, CAPACITY (nothing is written), HIP.
 * zc_decompress is zc_decompress_ex with flags 0 (it reads what zc_compress writes). */
int zc_decompress(const void* d_in, size_t in_bytes,
                  float* d_out, size_t out_cap_elems, size_t* n_out,
                  void* d_ws, size_t ws_bytes, void* hip_stream);
int zc_decompress_ex(const void* d_in, size_t in_bytes,
                     float* d_out, size_t out_cap_elems, size_t* n_out,
                     void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* zc_decompress for the Average aggregation of Section 3.2 (Corollary 1: the error of the
 * average of n buffers has variance sigma^2 / n): the stream holds the sum of nsum buffers, and
 * every value is divided by nsum on the way out, x' = (float)(((double)q * s) * r) with
 * r = 1.0 / nsum (one binary64 division per wave).  Arguments and errors as zc_decompress_ex. */
int zc_decompress_average(const void* d_in, size_t in_bytes, float* d_out, size_t out_cap_elems, size_t* n_out,
                          void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* One chunk of a stream on its own (Section 3.5.2 handles a buffer chunk by chunk, so that a
 * chunk can be decompressed while others are still on their way or being worked on, for
 * instance by calls on several HIP streams, each with a workspace of its own): the values
 * [first_value, first_value + count) of the stream, cut off at its end, go to d_out[0 ...].
 * first_value must be a multiple of 2048 (a segment of 64 blocks).  Only the header, the tables
 * and the payload of those segments are read; of an indexed stream
 * not even the whole width table, only the index entries and width bytes of the segments
 * (of a plain stream the whole width table is summed first, in every call, and the workspace
 * must be large enough for the whole stream, zc_workspace_bytes(n, 1)).
 * n_out (host, may be NULL): receives how many values that is.
 * Errors: ARG (also: first_value not a multiple of 2048, or beyond the stream's n), FORMAT,
 * CAPACITY (out_cap_elems smaller than the part), HIP. */
int zc_decompress_range(const void* d_in, size_t in_bytes, size_t first_value, size_t count,
                        float* d_out, size_t out_cap_elems, size_t* n_out,
                        void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* Decompression of k streams in one call: the tail of the compressed Allgather (Section 3.5.1:
 * a rank decompresses all the chunks it has received at the end), one launch instead of k.
 * d_chunks, chunk_bytes, d_outs, out_cap_elems: HOST arrays of k entries (device pointers 16-byte
 * aligned); stream i is decoded into d_outs[i] exactly as zc_decompress_ex would.  The streams need
 * not agree in n or bound.  n_out (host array of k entries, may be NULL): receives every
 * stream's n.  In the asynchronous form zc_finish reports the sum of the k values of n.
 * Errors: ARG, FORMAT (a malformed header in any stream: nothing is written then), CAPACITY (that
 * stream is not written, the others are), HIP. */
int zc_decompress_many(const void* const* d_chunks, const size_t* chunk_bytes, int k,
                       float* const* d_outs, const size_t* out_cap_elems, size_t* n_out,
                       void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* Local step of the compressed Allreduce (Section 3.1.2, Sum of Section 3.2): k compressed
 * operands of the same n and abs_eb -> the compressed sum, computed on the integer codes, so
 * no new quantisation error appears and decompress(out) is within nsum * abs_eb of the exact
 * sum of the original buffers.  d_chunks: HOST array of k device pointers (16-byte aligned
 * streams); chunk_bytes: HOST array of their sizes; 1 <= k <= ZC_MAX_K.
 * Errors: ARG, FORMAT, MISMATCH, RANGE, CAPACITY, HIP.
 * zc_reduce_compressed is zc_reduce_compressed_ex with flags 0. */
int zc_reduce_compressed(const void* const* d_chunks, const size_t* chunk_bytes, int k,
                         void* d_out, size_t out_cap, size_t* out_bytes,
                         void* d_ws, size_t ws_bytes, void* hip_stream);
int zc_reduce_compressed_ex(const void* const* d_chunks, const size_t* chunk_bytes, int k,
                            void* d_out, size_t out_cap, size_t* out_bytes,
                            void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* One round of the ring reduce-scatter (Section 3.1.2: a received compressed chunk is
 * decompressed, reduced with the local chunk and compressed again; Section 3.2, Sum: each such
 * round adds at most abs_eb to the error).  d_chunk: the received stream (chunk_bytes bytes,
 * 16-byte aligned).  d_local: n_local binary32 values, 16-byte aligned; n_local must equal
 * the stream's n.  d_out receives the stream of dequantised(received) + local, the addition in
 * binary32, under the received stream's own bound; its nsum is the received one + 1.
 * out_bytes (host, may be NULL): receives total_bytes.  Nothing but the two streams and the
 * local values moves through memory.
 * Errors: ARG, FORMAT, MISMATCH, NONFINITE, RANGE, CAPACITY, BOUND (against the binary32
 * sums; the stream is complete then), HIP.
 * zc_reduce_step is zc_reduce_step_op with ZC_OP_SUM and flags 0. */
int zc_reduce_step(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local,
                   void* d_out, size_t out_cap, size_t* out_bytes,
                   void* d_ws, size_t ws_bytes, void* hip_stream);

/* The same round for the other aggregation functions of Section 3.2.  op: ZC_OP_SUM,
 * ZC_OP_MAX or ZC_OP_MIN: d_out receives the stream of the larger (smaller)
 * of dequantised(received) and local.  Because the quantiser is monotone and maps its own
 * grid points to themselves, a ring of such rounds yields exactly the stream of the elementwise
 * maximum (minimum) of all buffers: the error stays within abs_eb however many rounds there are,
 * inside Theorem 2's variance.  A NaN or an infinity among the local values is NONFINITE.
 * Errors as zc_reduce_step, and ARG for an unknown op. */
#define ZC_OP_SUM 0
#define ZC_OP_MAX 1
#define ZC_OP_MIN 2
int zc_reduce_step_op(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local, int op,
                      void* d_out, size_t out_cap, size_t* out_bytes,
                      void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* The local step of the compressed Allreduce for all three aggregation functions of Section 3.2
 * on k compressed operands: op ZC_OP_SUM is zc_reduce_compressed_ex; ZC_OP_MAX / ZC_OP_MIN give the
 * stream of the largest / smallest code of every value.  The operands share the quantisation step
 * and the quantiser is monotone, so that is exactly the stream of the elementwise maximum (minimum)
 * of the original buffers compressed once: within abs_eb of it whatever k is (inside Theorem 2's
 * variance), and equal to what a ring of zc_reduce_step_op rounds over the same buffers ends in.
 * nsum of the result is the sum of the operands' nsum.  Arguments and errors as
 * zc_reduce_compressed_ex, and ARG for an unknown op. */
int zc_reduce_compressed_op(const void* const* d_chunks, const size_t* chunk_bytes, int k, int op,
                            void* d_out, size_t out_cap, size_t* out_bytes,
                            void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* The Sum of zc_reduce_compressed_ex and the round of zc_reduce_step_op done in parts (Section 3.5.2
 * works on a buffer chunk by chunk inside the rounds of the collective, so that the codec runs on
 * the chunks that have arrived while the others are still on their way): this call produces the
 * values [first_value, first_value + count) of the result.  The parts of one result are given in
 * ascending order, without gaps, to the same d_out and d_ws, on one HIP stream (or ordered by
 * events), starting with first_value = 0, which also writes the header; first_value and count are
 * multiples of 8192, except that the last part ends at n.  Indexed streams only (flags without
 * ZC_STREAM_PLAIN).  Of every operand only the header, and the index entries, width bytes, outliers
 * and payload of the part's segments are read, so an operand need not be complete beyond them;
 * chunk_bytes are the operands' full sizes.  n (for the k-way form; n_local for the round) is what
 * the parts are laid out for and must be the streams' n.  Between the parts the workspace must not
 * be used for anything else.  After a part has run, the result's tables and payload up to its end are
 * final, header and index describe a stream that can be read up to there (zc_decompress_range), and
 * out_bytes (or zc_finish) tells how many bytes of the stream that is; after the last part the stream
 * is the one the call in one piece writes.  Errors of all parts accumulate in the workspace.
 * Errors: as the calls in one piece, and ARG for a part that is not as above. */
int zc_reduce_compressed_part(const void* const* d_chunks, const size_t* chunk_bytes, int k, size_t n,
                              size_t first_value, size_t count,
                              void* d_out, size_t out_cap, size_t* out_bytes,
                              void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);
int zc_reduce_step_part(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local, int op,
                        size_t first_value, size_t count,
                        void* d_out, size_t out_cap, size_t* out_bytes,
                        void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* Quality of a reconstruction d_test against its original d_ref (n binary32 values each,
 * 16-byte aligned): the sums behind the paper's quality figures (NRMSE in Section 3.3, PSNR
 * and NRMSE in Section 4.6).  out4 (host, 4 doubles): max |ref - test|, sum of squared
 * differences, min(ref), max(ref), accumulated in binary64 in a fixed order.  With range =
 * max - min and RMSE = sqrt(sum / n): NRMSE = RMSE / range, PSNR = 20 log10(range / RMSE).
 * n = 0 gives {0, 0, +inf, -inf}.  Synchronous.  The workspace must hold at least
 * zc_workspace_bytes(n, 1) bytes.  Errors: ARG, HIP. */
int zc_quality(const float* d_ref, const float* d_test, size_t n, double* out4,
               void* d_ws, size_t ws_bytes, void* hip_stream);

/* Completes an asynchronous call: synchronises hip_stream, returns the status of the last
 * call that used d_ws and stores its size result (total_bytes, or n for zc_decompress) in
 * *result (host, may be NULL).  d_ws NULL: the call was zc_compress_noalloc on the current device. */
int zc_finish(const void* d_ws, size_t* result, void* hip_stream);

/* Reads and validates a stream header (synchronises hip_stream); the variant is told by the
 * header's version word.  Any output may be NULL.  flags: ZC_STREAM_PLAIN for a plain stream,
 * 0 for an indexed one: what the calls that read this stream must be given. */
int zc_peek_header(const void* d_in, size_t in_bytes, size_t* n, float* abs_eb,
                   unsigned* nsum, size_t* total_bytes, unsigned* flags, void* hip_stream);

const char* zc_strerror(int status);

/* Staged checks of the stream's parts (Section 3.3, one stage each). */

/* Quantisation stage only: d_q[i] = rint(d_in[i] / s).  Synchronous.
 * Errors: ARG, NONFINITE, RANGE, BOUND, HIP. */
int zc_debug_quantize(const float* d_in, size_t n, float abs_eb, int32_t* d_q,
                      void* d_ws, size_t ws_bytes, void* hip_stream);

/* Payload offset of every block, in 4-byte words, recomputed from a stream's width table
 * (and, of an indexed stream, its index) into d_off_words[nb].  Synchronous.
 * Errors: ARG, FORMAT, CAPACITY (off_cap < nb), HIP. */
int zc_debug_block_offsets(const void* d_in, size_t in_bytes, uint32_t* d_off_words, size_t off_cap,
                           void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags);

/* Measurement aid (not part of the method).  While enabled, zc_compress, zc_decompress,
 * zc_decompress_average, zc_decompress_many, zc_reduce_compressed, zc_reduce_step and
 * zc_reduce_step_op (and their _ex forms) hand a pair of HIP events to the launch of their
 * main kernel on the call's stream (hipExtLaunchKernelGGL), which stamps them with that
 * kernel's start and end (the compress kernel over the full tiles, the decompress, reduce or
 * step kernel; not the small kernels that run ahead of it for plain streams).
 * zc_profile_collect waits for the recorded pairs, stores up to cap elapsed times in
 * milliseconds in ms[] and the matching ZC_KERNEL_* ids in kernel[] (host arrays, either may
 * be NULL) in call order, forgets them, and returns how many it stored (a negative status on
 * a HIP error).  The events are host objects created on first use and reused.  on: 0 off,
 * 1 every kind of main kernel, or a sum of (1 << ZC_KERNEL_x) to time only those kinds (a
 * timed launch costs a few microseconds).  Leave it disabled while a stream is being
 * captured into a HIP graph.  Enabling or disabling forgets the pairs recorded so far. */
#define ZC_KERNEL_COMPRESS 1
#define ZC_KERNEL_DECOMPRESS 2
#define ZC_KERNEL_REDUCE 3
#define ZC_KERNEL_REDUCE_STEP 4
#define ZC_KERNEL_STREAM 5
int zc_profile_enable(int on);
int zc_profile_collect(float* ms, int* kernel, int cap);

/* Measurement aid (not part of the method): a kernel that only streams, with the access shape
 * of the codec's kernels (workgroups of 512 threads, every lane 16 bytes per access, 8 KiB per
 * workgroup and access, non-temporal), so that a kernel's rate can be put beside what the
 * memory system gives a kernel of the same read : write mix that does nothing else.  Workgroup
 * t of `tiles` reads loads x 8 KiB at d_in + t x loads x 8 KiB and writes stores x 8 KiB at
 * d_out + t x stores x 8 KiB (every store holds the exclusive-or of what the lane read, so no
 * load is dead).  loads and stores in 0..16, not both 0; d_in (device, tiles x loads x 8 KiB,
 * may be NULL when loads is 0) and d_out (device, tiles x stores x 8 KiB, may be NULL when
 * stores is 0) 16-byte aligned.  Asynchronous on hip_stream; its launch is timed as
 * ZC_KERNEL_STREAM while zc_profile_enable asks for that.  Errors: ARG, HIP. */
int zc_debug_stream(const void* d_in, void* d_out, size_t tiles, int loads, int stores, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ZC_H */
