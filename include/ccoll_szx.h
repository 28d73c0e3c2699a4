/* libccoll_szx -- the data-parallel hot path of C-Coll on one AMD MI355X (gfx950).
 *
 * C-Coll (arXiv 2304.03890) speeds up MPI collectives with an error-bounded lossy
 * compressor, a customised SZx.  This library is that compressor and the per-round
 * compute of the compressed ring reduce-scatter, as hand-written HIP kernels:
 *
 *   - ccoll_szx_compress / ccoll_szx_decompress[_range]: block-wise SZx coding of
 *     float32 under an absolute error bound, in the chunked layout of the paper's
 *     Sec. III-E.2 (chunks of 5120 points, one 4-byte compressed size per chunk kept
 *     together at the front of the buffer as an index);
 *   - ccoll_reduce_step: the round of Sec. III-A.2 / Eq. 2 -- decompress the chunk that
 *     arrived, add the local chunk (float32 sum), compress the result -- fused so that
 *     the summed floats never touch device memory.
 *
 * Contract (Sec. III-B): after one compression every finite value satisfies
 * fabs((double)x - (double)x') <= (double)abs_eb; NaN / Inf are kept bit-exactly.
 *
 * Stream "CSX1" (little-endian):
 *   off  0 u32 magic 'C','S','X','1'      off  4 u16 128 (block)   off  6 u16 5120 (chunk)
 *   off  8 u64 n                          off 16 u32 bits(abs_eb)  off 20 u32 nchunks
 *   off 24 u64 total_bytes                off 32 u32 chunk_size[nchunks]
 *   then the chunk payloads, each a multiple of 4 bytes:
 *     u64 bitmap (bit j set = block j not constant), f32 mu[blocks], u16 body_size[k],
 *     u8 reqlen[k] (9..24, or 32 = raw), pad to 4, bodies (2-bit lead codes, then the
 *     bytes that differ from the previous element's, MSB first), pad to 4.
 *
 * All data pointers named d_* are DEVICE pointers (e.g. torch.Tensor.data_ptr()); they stay
 * owned by the caller and the library never allocates or frees inside a compress /
 * decompress / reduce call (the paper measured 23 % overhead from freeing buffers the
 * compressor had allocated, Sec. III-D).  Work is enqueued on the stream given to
 * ccoll_create.  The plain calls wait for the result; the *_async calls only enqueue and
 * leave {bytes, status} in device memory.
 *
 * Every function returns CCOLL_OK (0) or a negative code; nothing throws or aborts, and a
 * corrupt input stream is never read or written out of bounds.
 */
#ifndef CCOLL_SZX_H
#define CCOLL_SZX_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CCOLL_OK        0
#define CCOLL_EINVAL   (-1)  /* null pointer, abs_eb not finite or <= 0, n > 2^31, misaligned pointer, bad range */
#define CCOLL_ENOSPC   (-2)  /* output capacity too small; nothing beyond the capacity was written */
#define CCOLL_ECORRUPT (-3)  /* input stream malformed (header, index or a chunk inconsistent) */
#define CCOLL_EHIP     (-4)  /* HIP runtime error */
#define CCOLL_ETIMEDOUT (-5) /* a workgroup gave up waiting (about a second) for the size of an earlier group of
                                chunks: the device made no progress on this launch; retry */

#define CCOLL_BLOCK_ELEMS 128
#define CCOLL_CHUNK_ELEMS 5120   /* paper, Sec. III-E.2 */

typedef struct ccoll_ctx ccoll_ctx;

/* One context = one device + one stream + a scan workspace (16 bytes per chunk of the largest input reserved
 * for, plus spill slots for chunks that outgrow on-chip staging: 44.5 KB per wavefront of the widest launch,
 * at most 137 MB).  On failure *out is NULL.
 * hip_stream is a hipStream_t (NULL = the default stream).  Not thread-safe: calls on one
 * context must not overlap. */
int  ccoll_create(ccoll_ctx **out, int device, void *hip_stream);
/* Grows the workspace so that inputs of up to max_n elements need no allocation later.
 * Call outside timed regions; the hot calls fail with CCOLL_EINVAL if n exceeds it. */
int  ccoll_reserve(ccoll_ctx *ctx, size_t max_n);
void ccoll_destroy(ccoll_ctx *ctx);
/* How long a workgroup of compress / reduce_step polls for the sizes of earlier chunk groups before it gives
 * up with CCOLL_ETIMEDOUT (every other waiting workgroup of the launch then leaves too, and the output is
 * not valid).  polls = 0 restores the default (about a second).  Meant for tests of that path and for
 * callers that share the device with long-running kernels. */
int  ccoll_set_scan_wait(ccoll_ctx *ctx, unsigned int polls);
/* Measurement aid.  start_event / stop_event: two hipEvent_t created by the caller with timing enabled
 * (either may be null).  The coding or decoding kernel of the next compress / decompress / reduce_step call on
 * this context (not its index scan) is launched so that the events take the start and the end of that kernel
 * itself; hipEventElapsedTime(start, stop), once stop has completed, is the kernel's duration without the gaps
 * that events recorded around the call would include.  One call consumes the pair; a call that launches no
 * such kernel (n == 0, a refused argument) leaves it armed. */
int  ccoll_time_next_kernel(ccoll_ctx *ctx, void *start_event, void *stop_event);

/* Upper bound of the stream size for n elements: 32 + ceil(n/5120) * 22052. */
size_t ccoll_szx_max_compressed_bytes(size_t n);

/* Compression of d_in[0..n) under abs_eb (Sec. III-C fixed-accuracy mode; chunk layout of
 * Sec. III-E.2).  d_in: device, 4-byte aligned (16-byte alignment takes the fast path).
 * d_out: device, 4-byte aligned, out_cap bytes.  out_bytes (host) receives the stream size.
 * CCOLL_ENOSPC if out_cap is too small: then *out_bytes is the size that was needed, or 0 if out_cap does not
 * even hold the header and the front index (32 + 4 * ceil(n / 5120) bytes). */
int ccoll_szx_compress(ccoll_ctx *ctx, const float *d_in, size_t n, float abs_eb,
                       void *d_out, size_t out_cap, size_t *out_bytes);

/* Inverse: d_out[0..n) from the stream d_in[0..in_bytes).  n must equal the header's n. */
int ccoll_szx_decompress(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, float *d_out, size_t n);

/* Elements [first_elem, first_elem+count) only (the paper's chunk-start pointer derived from
 * the front index, Sec. III-E.2).  first_elem must be a multiple of 128; n is the element
 * count of the whole stream.  d_out[0] receives element first_elem. */
int ccoll_szx_decompress_range(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n,
                               size_t first_elem, size_t count, float *d_out);

/* The same when many ranges of one stream are decoded (the paper's C-Scatter / C-Bcast: compressed once at
 * the root, every receiver decodes its part, Sec. III-A.1 and IV-C): ccoll_szx_index checks the header and the
 * front index once and keeps the chunk-start pointers in the context; ccoll_szx_decompress_range_indexed then
 * decodes a range without walking the index again.  The pointers stay valid until the next ccoll_szx_index,
 * ccoll_szx_decompress[_range] or ccoll_reduce_step* call on the context; the indexed call returns
 * CCOLL_EINVAL unless d_in, in_bytes and n are those of the indexed stream.  The stream must not change in
 * between. */
int ccoll_szx_index(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n);
int ccoll_szx_decompress_range_indexed(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n,
                                       size_t first_elem, size_t count, float *d_out);

/* Many ranges of one stream at once (C-Scatter, Sec. III-A.1 and IV-C: the root compresses once, every
 * receiver's part is decoded from the same stream): the header and the front index are checked once and the
 * ranges are decoded by one launch per CCOLL_MAX_RANGES_PER_LAUNCH ranges.  first_elem[r] (multiples of 128),
 * count[r] and d_out[r] (device pointers, 4-byte aligned) are HOST arrays of nranges entries, read before the
 * call returns; d_out[r][0] receives element first_elem[r].  Ranges may overlap or leave gaps. */
#define CCOLL_MAX_RANGES_PER_LAUNCH 64
int ccoll_szx_decompress_ranges(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n, size_t nranges,
                                const size_t *first_elem, const size_t *count, float *const *d_out);

/* One round of the compressed ring reduce-scatter (Sec. III-A.2, Eq. 2):
 * cout = compress(local + decompress(cin), abs_eb), float32 round-to-nearest sum.
 * n = element count of d_local and of the stream in d_cin. */
int ccoll_reduce_step(ccoll_ctx *ctx, const float *d_local, size_t n, const void *d_cin, size_t cin_bytes,
                      float abs_eb, void *d_cout, size_t cout_cap, size_t *cout_bytes);

/* The same round for the other reductions the paper names (Sec. III-B: Sum, Average, Max, Min; an Average is
 * a Sum that the caller divides once at the end).  CCOLL_OP_MAX / CCOLL_OP_MIN take the larger / smaller
 * operand under the total order of the bit patterns (-NaN < -Inf < ... < -0 < +0 < ... < +Inf < +NaN), so the
 * result does not depend on which operand is local.  Any other op: CCOLL_EINVAL. */
#define CCOLL_OP_SUM 0
#define CCOLL_OP_MAX 1
#define CCOLL_OP_MIN 2
int ccoll_reduce_step_op(ccoll_ctx *ctx, int op, const float *d_local, size_t n, const void *d_cin,
                         size_t cin_bytes, float abs_eb, void *d_cout, size_t cout_cap, size_t *cout_bytes);

/* Enqueue-only variants.  d_result: device pointer to two 64-bit words that receive
 * {stream bytes written (compress, reduce) or 0 (decompress), status code as a signed
 * 64-bit value} when the work completes; NULL keeps the result inside the context, to be
 * fetched with ccoll_wait.  Argument errors are still reported by the return value. */
int ccoll_szx_compress_async(ccoll_ctx *ctx, const float *d_in, size_t n, float abs_eb,
                             void *d_out, size_t out_cap, unsigned long long *d_result);
int ccoll_szx_decompress_async(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, float *d_out, size_t n,
                               unsigned long long *d_result);
int ccoll_szx_decompress_range_async(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n,
                                     size_t first_elem, size_t count, float *d_out,
                                     unsigned long long *d_result);
int ccoll_szx_decompress_ranges_async(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n, size_t nranges,
                                      const size_t *first_elem, const size_t *count, float *const *d_out,
                                      unsigned long long *d_result);
int ccoll_szx_index_async(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n, unsigned long long *d_result);
int ccoll_szx_decompress_range_indexed_async(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n,
                                             size_t first_elem, size_t count, float *d_out,
                                             unsigned long long *d_result);
int ccoll_reduce_step_async(ccoll_ctx *ctx, const float *d_local, size_t n, const void *d_cin,
                            size_t cin_bytes, float abs_eb, void *d_cout, size_t cout_cap,
                            unsigned long long *d_result);
int ccoll_reduce_step_op_async(ccoll_ctx *ctx, int op, const float *d_local, size_t n, const void *d_cin,
                               size_t cin_bytes, float abs_eb, void *d_cout, size_t cout_cap,
                               unsigned long long *d_result);

/* For callers that cannot allocate device memory or hold a context: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The same decompression as ccoll_szx_decompress_async, with
 * no context: what the context would hold for the call (its result and error words and the chunk-start
 * offsets derived from the front index, 8 bytes per chunk) lives in a static device array inside the library,
 * about 210 KB, which every device that runs the library keeps until the process ends.  The call allocates
 * and frees nothing and only enqueues kernels (no memset, no copy) on hip_stream (a hipStream_t, NULL = the
 * default stream) of `device`.
 *   n <= CCOLL_STATIC_MAX_ELEMS, else CCOLL_EINVAL (use a context for larger streams).
 *   d_result: device, 8-byte aligned, two 64-bit words, required: receives {0, status as a signed 64-bit value}
 *   when the work completes (CCOLL_OK, or CCOLL_ECORRUPT for a malformed or truncated stream).
 * All calls on one device share that device's array: calls that overlap in time on one device (two streams,
 * two threads) race and give undefined results; calls that follow each other on one stream are fine.  The
 * first call on a device resolves the array's address (hipGetSymbolAddress): make it outside a capture. */
#define CCOLL_STATIC_MAX_ELEMS 134217728   /* 2^27 */
int ccoll_szx_decompress_static(int device, void *hip_stream, const void *d_in, size_t in_bytes,
                                float *d_out, size_t n, unsigned long long *d_result);

/* PIPE-SZx (Sec. III-E.2): the paper compresses a message in chunks so that the transfer of what is coded
 * can go on while the rest is still being coded, and decompresses what has arrived while the rest is still on
 * its way.  Here one stream (one header, one front index: the same bytes as ccoll_szx_compress gives) is
 * written by several launches, each coding a piece of consecutive chunks:
 *   ccoll_szx_compress_begin       starts a stream of n elements in d_out (writes the header with a total of 0);
 *   ccoll_szx_compress_chunks_async  codes chunks [chunk_first, chunk_end) of d_in (the address of element 0 of the
 *     whole input).  Pieces follow each other without gaps from chunk 0 on; every piece but the last ends at a
 *     multiple of CCOLL_PIECE_CHUNKS chunks.  When the launch has completed, the front index entries and payloads
 *     of all chunks below chunk_end are final, and d_progress (device, 8-byte aligned, two 64-bit words, may be
 *     NULL) holds {chunk_end, stream bytes that are final}; the last piece also writes the header's total.
 *     d_result as for the other *_async calls ({stream bytes so far, status}).
 *   No other compress or reduce call may use the context between begin and the last piece (the pieces share the
 *   context's scan state); such a call ends the open stream, and further pieces return CCOLL_EINVAL.
 *   ccoll_szx_decompress_chunks_async  decodes chunks [chunk_first, chunk_end) of a stream of n elements of which
 *     only the header, the front index entries and the payloads of the chunks below chunk_end need to have arrived
 *     (in_bytes: the bytes that are there; the header's total is not looked at).  d_out[0] receives element
 *     5120 * chunk_first.
 *   ccoll_szx_forward_async  stands in for the transport on one device: copies what has become final between two
 *     progress words (d_from = NULL: the start of the stream) from d_src to the same offsets of d_dst, on any
 *     stream of `device`; with the last piece the final header goes along.  Enqueue it behind the piece (an event). */
#define CCOLL_PIECE_CHUNKS 12
int ccoll_szx_compress_begin(ccoll_ctx *ctx, size_t n, float abs_eb, void *d_out, size_t out_cap);
int ccoll_szx_compress_chunks_async(ccoll_ctx *ctx, const float *d_in, size_t chunk_first, size_t chunk_end,
                                    unsigned long long *d_progress, unsigned long long *d_result);
int ccoll_szx_decompress_chunks_async(ccoll_ctx *ctx, const void *d_in, size_t in_bytes, size_t n,
                                      size_t chunk_first, size_t chunk_end, float *d_out,
                                      unsigned long long *d_result);
int ccoll_szx_forward_async(int device, void *hip_stream, void *d_dst, const void *d_src, size_t n,
                            const unsigned long long *d_from, const unsigned long long *d_upto);

/* Waits for the context's stream.  Returns the status of the *_async calls that kept their result in the
 * context (d_result = NULL) and were enqueued since the previous ccoll_wait: CCOLL_OK if all of them went
 * well, else the code of the latest one that failed.  *bytes (may be NULL) receives the byte count of the
 * last such call. */
int ccoll_wait(ccoll_ctx *ctx, size_t *bytes);

const char *ccoll_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CCOLL_SZX_H */
