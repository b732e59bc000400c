/*
 * neuzip.h -- C ABI of the MI355X (gfx950) NeuZip codec library.
 *
 * What the library does (NeuZip, arXiv 2410.20650): a bf16 weight tensor is
 * split into its exponent bytes and a packed sign|mantissa stream (Alg. 1
 * "split"; App. D), the low-entropy exponents are entropy-coded with an
 * asymmetric numeral system (Sec. 2.2 "Compression algorithm"), and the
 * tensor is rebuilt bit-exactly into caller-provided temporary space right
 * before a layer uses it (Sec. 2.2 Eq. (3); Alg. 1 "decompression"/"merge").
 * The lossy inference variant keeps only the k leading mantissa bits
 * (Sec. 2.3), k in {3, 1, 0}.
 *
 * Conventions for every entry point
 *   - d_* arguments are DEVICE pointers owned by the caller, h_* arguments are
 *     HOST pointers owned by the caller.  Nothing is retained after the call's
 *     stream work has completed.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     All kernels and copies of a call are enqueued on it.
 *   - Tensors are flat, contiguous arrays of n_elems 16-bit words (32-bit
 *     words for NEUZIP_F32); the shape of the matrix is irrelevant to the
 *     codec.  d_src / d_dst must be aligned to 16 bytes.  n_elems must be
 *     below 2^32.
 *   - Errors are reported through the return code only (no exceptions, no
 *     aborts, nothing is printed).  On error no output argument is modified
 *     unless stated otherwise.
 *   - If a call that compresses into an existing blob fails after its kernels
 *     have started (out of memory while growing the stream, a HIP error), that
 *     blob holds no tensor any more: decompress, linear, update, recompress and
 *     export return NEUZIP_EINVAL for it until a compress call has succeeded.
 *   - A blob belongs to the device that was current when it was created; every
 *     call that launches work on it must be made with that device current
 *     (NEUZIP_EINVAL otherwise).  neuzip_free may be called from any device.
 *   - Calls that touch different blobs may run concurrently from different
 *     host threads; compress calls are serialised inside the library because
 *     they share one per-device workspace.
 */
#ifndef NEUZIP_H
#define NEUZIP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Opaque handle of one compressed tensor.  The library owns the device memory
 * behind it until neuzip_free. */
typedef struct neuzip_blob neuzip_blob;

/* Element types.  The paper works on BFloat16 only (Sec. 2.1, footnote); the other two go beyond it.
 * NEUZIP_F32: the upper half of an IEEE binary32 word is a bf16 word (sign, the same 8 exponent
 * bits, 7 mantissa bits) and is compressed exactly as one; the lower half, 16 mantissa bits without
 * structure, is kept as a raw plane after the sign|mantissa stream.
 * NEUZIP_F16: IEEE binary16 (sign, 5 exponent bits, 10 mantissa bits); the upper byte of a word
 * (sign, exponent, two mantissa bits) is the entropy-coded symbol in place of the bf16 exponent
 * byte, the lower byte is stored in place of the sign|mantissa byte.
 * Both are lossless only: mantissa_bits must be 7 and there is no block-wise normalisation
 * (EUNSUPPORTED / EINVAL otherwise).  Header word 56 of the container holds the element type.
 * neuzip_compress, _batch, _guarded, neuzip_recompress, the three decompress calls, export and
 * import take such tensors; neuzip_linear and neuzip_update do not (EUNSUPPORTED). */
enum { NEUZIP_BF16 = 0, NEUZIP_F32 = 1, NEUZIP_F16 = 2 };

enum {
    NEUZIP_OK = 0,
    NEUZIP_EINVAL = -1,       /* bad argument (null pointer, misaligned, wrong n/dtype/mantissa_bits) */
    NEUZIP_ENOMEM = -2,       /* device or host allocation failed, or h_buf too small */
    NEUZIP_EHIP = -3,         /* a HIP runtime call failed; see neuzip_last_hip_error() */
    NEUZIP_ECORRUPT = -4,     /* a container or a decoded stream is not well formed */
    NEUZIP_EUNSUPPORTED = -5  /* a size, or a combination of element type and option, that is not supported */
};

/* Format constants of the stream (mirrored in every container header). */
enum {
    NEUZIP_PROB_BITS = 12,        /* frequencies sum to 2^12 */
    NEUZIP_CHUNK = 4096,          /* exponent symbols per independently decodable chunk */
    NEUZIP_STATES_PER_CHUNK = 16, /* rANS states per chunk, each with a private word run */
    NEUZIP_RUN = 8                /* consecutive symbols one state codes per turn */
};

/*
 * neuzip_compress -- Alg. 1 initialisation loop and the re-compression after a
 * weight update ("split", "compression", "store"); Sec. 2.3 for k < 7.
 *
 *   d_src          n_elems bf16 words on the device (read only).
 *   dtype          NEUZIP_BF16, or NEUZIP_F32 / NEUZIP_F16 (n_elems words of that type; see the element types).
 *   mantissa_bits  7 = lossless; 3, 1 or 0 = keep that many leading mantissa
 *                  bits, truncating toward zero.
 *   blob           in/out.  *blob == NULL: a new blob is created.  Otherwise
 *                  *blob must be a blob of this library with the same n_elems
 *                  and mantissa_bits; its device memory is reused (and grown
 *                  if the new stream is longer), its old content is lost, and it
 *                  keeps the guard band it was made with (neuzip_compress_guarded).
 *
 * Builds the exponent histogram, the 12-bit frequency table, encodes every
 * 4096-symbol chunk with 16 rANS states, and stores exponent stream and
 * sign|mantissa stream in device memory sized for this tensor (the word
 * section with 1/64 of headroom, 0.3 % of the container, so that a blob which
 * is compressed into again after an update seldom has to be re-allocated).
 * Synchronises hip_stream once (the stream length is data dependent).
 * n_elems == 0 yields a valid empty blob.
 */
int neuzip_compress(const void *d_src, uint64_t n_elems, int dtype, int mantissa_bits,
                    void *hip_stream, neuzip_blob **blob);

/*
 * neuzip_compress_blockwise -- the lossy variant with block-wise normalisation (Sec. 2.3, last
 * paragraph; block sizes as in the block-size study of Sec. 3).
 *
 *   block_size     0 (same as neuzip_compress) or 32, 64, 128, 256, 512 consecutive weights.
 *   mantissa_bits  3, 1 or 0 when block_size != 0 (7 -> EINVAL: normalisation is lossy).
 *
 * Reading of the paper taken here: the coefficient of a block is the 7-bit mantissa of its
 * largest-magnitude weight (first one on ties), stored in one byte per block; with
 * c = 1 + coef/128 every weight is stored as bf16(w / c) before truncation and is returned as
 * bf16(stored * c), both rounded to nearest even in IEEE binary32.  The largest weight of each
 * block is reproduced exactly.  Everything else is as for neuzip_compress; neuzip_decompress
 * and the other entry points recognise such blobs by themselves.
 */
int neuzip_compress_blockwise(const void *d_src, uint64_t n_elems, int dtype, int mantissa_bits,
                              uint32_t block_size, void *hip_stream, neuzip_blob **blob);

/*
 * neuzip_compress_batch -- the same compression (Alg. 1 backward loop: "split", "compression",
 * "store" for every weight of a layer after its update) for several tensors at once: each
 * kernel of the pipeline runs once per group of up to 8 tensors and the host waits once per
 * group, so small tensors overlap with the others.
 *
 *   d_srcs, n_elems  host arrays of count entries: device pointer (16-byte aligned) and element
 *                    count of each tensor.
 *   mantissa_bits, block_size   shared by all tensors; meaning as above.
 *   blobs            host array of count handles, in/out with the rules of neuzip_compress
 *                    (NULL entries are created; other entries must match and be distinct).
 * A group whose encoder slots would exceed the workspace limit (neuzip_set_workspace_limit) is
 * taken in parts, with one wait per part; the results are the same.
 * On error, blobs created for the failing group are released and its entries of blobs are
 * not changed; groups completed before keep their results.
 */
int neuzip_compress_batch(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int dtype,
                          int mantissa_bits, uint32_t block_size, void *hip_stream, neuzip_blob **blobs);

/*
 * neuzip_compress_guarded / neuzip_recompress -- Alg. 1 backward loop: every weight is compressed
 * again right after its update ("compression", "store"), i.e. once per tensor per training step.
 * The exponent statistics hardly move from one step to the next, so the table of the step before
 * can code the updated tensor, and the pass that counts exponents (one of the two reads of the
 * tensor) can be left out.  Not described in the paper; the reading taken here:
 *
 *   neuzip_compress_guarded   as neuzip_compress_batch without normalisation, but the table gives
 *       f = 1 to every exponent up to `guard` (0..255) below the smallest and above the largest
 *       one that occurs, and to exponent 0 (an update w - lr * g cancels exactly to +-0 now and
 *       then), so that values an update newly produces still have a code.  guard = 0 is the
 *       plain table.  The guard is kept in the blob and in header word 52 of the container.  For
 *       NEUZIP_F16 the band is taken on the coded symbol, the word's upper byte (sign, exponent, two
 *       mantissa bits): byte values up to `guard` below the smallest and above the largest one that
 *       occurs, and byte 0.
 *   neuzip_recompress         blobs[i] (which must hold a compressed tensor) receives d_srcs[i],
 *       a tensor of neuzip_elems(blobs[i]) words, coded with the table the blob already holds:
 *       one pass over the source that splits, packs and encodes.  If a tensor holds an exponent
 *       its table has no room for, that tensor is compressed afresh (statistics, new table with
 *       the blob's guard) and rebuilt[i] is set to 1, else 0 (rebuilt may be NULL).  Block-wise
 *       normalised blobs always take the second route.  After a table has been reused
 *       neuzip_histogram reports EINVAL for the blob (no counts were taken).
 *   Both work on host arrays of count entries like neuzip_compress_batch and synchronise the
 *   stream once per group of up to 8 tensors.  A caller that wants a fresh table every N steps
 *   calls neuzip_compress_guarded then.
 */
int neuzip_compress_guarded(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int dtype,
                            int mantissa_bits, uint32_t guard, void *hip_stream, neuzip_blob **blobs);
int neuzip_recompress(const void *const *d_srcs, uint32_t count, void *hip_stream, neuzip_blob *const *blobs,
                      uint32_t *rebuilt);

/*
 * neuzip_update -- the backward loop of Alg. 1 for the weights of a layer: each weight is
 * decompressed into temporary space, the optimiser step is applied, and the weight is compressed
 * again ("decompression", "merge", the update, "split", "compression", "store"); Sec. 2.2 applies
 * vanilla SGD layer by layer during the backward pass, so that neither the full set of gradients
 * nor an uncompressed model ever exists:
 *     W_hat <- decompress(c);   W_hat <- W_hat - lr * grad;   c <- compress(W_hat)
 *
 *   blobs       host array of count blobs holding lossless bf16 weights (mantissa_bits 7, no
 *               normalisation; anything else -> EUNSUPPORTED), distinct; they receive the new weights.
 *   d_grads     host array of count device pointers: the gradient of each weight, bf16 words,
 *               neuzip_elems(blobs[i]) of them, 16-byte aligned (read only).
 *   d_weights   host array of count device pointers, 16-byte aligned: temporary space of
 *               neuzip_elems(blobs[i]) bf16 words each, overlapping neither one another nor the
 *               gradients; on return it holds the new weights uncompressed (the caller may use
 *               or discard them; but see weights_ready = 2).
 *   lr          learning rate.
 *   weights_ready  NEUZIP_UPDATE_FROM_BLOB (0): the library decompresses blobs[i] itself.
 *               NEUZIP_UPDATE_WEIGHTS_READY (1): d_weights[i] already holds exactly
 *               decompress(blobs[i]) -- the backward pass has just decompressed the weight for the
 *               input gradient -- and that pass is skipped.  NEUZIP_UPDATE_WEIGHTS_READY_DISCARD (2):
 *               the same, and the caller has no use for the new weights uncompressed: they are
 *               not written back (a third less memory traffic), and d_weights[i] afterwards holds
 *               the old weight, or the new one for a tensor whose table was rebuilt.
 *               NEUZIP_UPDATE_FROM_BLOB_DISCARD (3): as 0, but d_weights is mere scratch space
 *               whose content afterwards is as for 2 (the library decompresses into it and then
 *               proceeds as for 2, which moves fewer bytes than 0).
 *   rebuilt     as for neuzip_recompress; may be NULL.
 * Reading taken for the arithmetic, which the paper leaves open: per element, in IEEE binary32,
 * the product lr * g and then the difference w - (lr * g) are each rounded to nearest (no fused
 * multiply-add), and the result is rounded to the nearest bf16, ties to even; a NaN result is
 * stored as 0x7FC0.  With weights_ready = 0 the decoder applies the step on its way out (the old
 * weight is never written) and the new weight is then coded as by neuzip_recompress; otherwise the
 * one-pass encoder of neuzip_recompress reads weight and gradient, forms the new weight, writes it
 * back to d_weights and codes it.  Either way the table the blob holds is used, with the fallback
 * to fresh statistics.  Synchronises the stream once per group of up to 8 weights.
 */
enum {
    NEUZIP_UPDATE_FROM_BLOB = 0,
    NEUZIP_UPDATE_WEIGHTS_READY = 1,
    NEUZIP_UPDATE_WEIGHTS_READY_DISCARD = 2,
    NEUZIP_UPDATE_FROM_BLOB_DISCARD = 3
};
int neuzip_update(neuzip_blob *const *blobs, const void *const *d_grads, void *const *d_weights, uint32_t count,
                  float lr, int weights_ready, void *hip_stream, uint32_t *rebuilt);

/*
 * neuzip_decompress -- Sec. 2.2 Eq. (3), Alg. 1 "decompression" + "merge":
 * decodes the exponents and reassembles bf16 words into the caller's
 * temporary space in one fused kernel.
 *
 *   d_dst    room for n_elems words of the blob's element type on the device, 16-byte aligned.
 *   n_elems, dtype must equal what the blob was made from (else EINVAL).
 *
 * Never allocates, never synchronises.  For mantissa_bits < 7 the dropped
 * mantissa bits come back as zeros.  A malformed stream is detected on the
 * device and reported by the next neuzip_check on this blob.
 */
int neuzip_decompress(const neuzip_blob *blob, void *d_dst, uint64_t n_elems, int dtype,
                      void *hip_stream);

/*
 * neuzip_decompress_sequence -- the per-layer schedule of Sec. 2.2 / Alg. 1
 * forward loop: every blob, in the given order, is decompressed into the same
 * temporary space on hip_stream, so that the whole model is never held
 * uncompressed.
 *
 *   blobs          host array of count blob handles.
 *   d_scratch      device buffer of scratch_elems bf16 words (2 * scratch_elems bytes), 16-byte
 *                  aligned; must hold the largest tensor, a binary32 blob counting two words
 *                  per element (else EINVAL, nothing is run).
 *   h_offsets      NULL, or a host array of count entries that receives where each tensor goes:
 *                  its first 16-bit word's index in the space.
 * Neighbouring blobs of one kind (element type, mantissa_bits, normalisation) that fit the space
 * together -- the projections of a layer, say -- are placed one behind the other, each at a
 * 256-byte boundary, and share one launch (at most 8 per launch), so that tensors too small to
 * fill the GPU on their own overlap; the next group starts at the front of the space again and
 * overwrites it.  When the call's work has run, the tensors of the last group are what the space
 * holds.  A caller that consumes the weights between the groups issues one call per layer.
 * Never allocates, never synchronises.
 */
int neuzip_decompress_sequence(const neuzip_blob *const *blobs, uint32_t count, void *d_scratch,
                               uint64_t scratch_elems, uint64_t *h_offsets, void *hip_stream);

/*
 * neuzip_decompress_batch -- Sec. 2.2 Eq. (3) / Alg. 1 "decompression" + "merge" for the
 * weights that a layer uses together (e.g. q, k, v, o, gate, up, down): blob i is
 * decompressed to d_dsts[i], all in as few launches as possible, so that tensors too small
 * to fill the GPU on their own overlap with the others.
 *
 *   blobs, d_dsts  host arrays of count entries; d_dsts[i] is a device buffer of
 *                  neuzip_elems(blobs[i]) words of the blob's element type, 16-byte aligned, not overlapping any
 *                  other destination.
 * Tensors are grouped by mantissa_bits (one launch per group of up to 8).  Never allocates,
 * never synchronises.  On EINVAL nothing has been launched.
 */
int neuzip_decompress_batch(const neuzip_blob *const *blobs, void *const *d_dsts, uint32_t count,
                            void *hip_stream);

/*
 * neuzip_linear -- the compressed forward pass of a linear layer, Sec. 2.2:
 *     W_hat <- decompress(c_l);   x_l <- W_hat x_{l-1} + b_l
 * as one fused kernel: the decoded weights go from the decoder's registers straight into the
 * matrix cores and W_hat is never written to memory.
 *
 *   weight        blob of a row-major out_features x in_features bf16 matrix (any mantissa_bits,
 *                 with or without block-wise normalisation; other element types ->
 *                 EUNSUPPORTED).  in_features must be a multiple of 128 and out_features *
 *                 in_features must equal neuzip_elems(weight).
 *   d_x           tokens x in_features bf16 activations, row-major, 16-byte aligned.
 *   tokens        at least 1.  The kernel holds the partial sums of up to 64 tokens; a larger
 *                 batch goes through in tiles of 64, each of which decodes the weight again (for
 *                 more than a few tiles, decompressing once and a dense GEMM is the faster way).
 *   d_bias        out_features floats on the device, or NULL.
 *   d_y           tokens x out_features floats, row-major; overwritten.
 * Products are exact, sums are accumulated in float32 by the matrix cores and, across the pieces
 * of a row, by float atomics, so the last bits can differ from run to run.  Never allocates,
 * never synchronises; a malformed stream is reported by neuzip_check as for neuzip_decompress.
 */
int neuzip_linear(const neuzip_blob *weight, uint64_t out_features, uint64_t in_features, const void *d_x,
                  uint32_t tokens, const float *d_bias, float *d_y, void *hip_stream);

/*
 * neuzip_linear_batch -- the same compressed forward pass (Sec. 2.2) for several weights that are
 * applied to the same activations, such as the q, k and v projections of an attention block or the
 * gate and up projections of an MLP: y_i <- W_hat_i x + b_i for i < count in one launch, so that
 * weights too small to fill the GPU on their own overlap with the others.
 *
 *   weights, out_features, d_y   host arrays of count entries (count at most 4, else EINVAL); weight i is
 *                 out_features[i] x in_features, d_y[i] receives tokens x out_features[i] floats.
 *                 All weights have the same mantissa_bits and are either all block-wise normalised
 *                 or none is (else EINVAL).
 *   d_bias        NULL (no biases), or a host array of count device pointers, each NULL or
 *                 out_features[i] floats.
 *   in_features, d_x, tokens     as for neuzip_linear; the activations are shared.
 * Otherwise as neuzip_linear (which is this call with count = 1).  On EINVAL nothing has been launched.
 */
int neuzip_linear_batch(const neuzip_blob *const *weights, const uint64_t *out_features, uint32_t count,
                        uint64_t in_features, const void *d_x, uint32_t tokens, const float *const *d_bias,
                        float *const *d_y, void *hip_stream);

/* Releases the blob and its device memory.  NULL is a no-op. */
void neuzip_free(neuzip_blob *blob);

/* Size in bytes of the blob's container (header, table, offsets, states, run
 * lengths, words, sign|mantissa stream, padding): what neuzip_export writes.
 * This is the figure bits/weight is computed from (Sec. 2.1: compression
 * ratio).  0 for NULL. */
uint64_t neuzip_compressed_bytes(const neuzip_blob *blob);

/* Bytes of device memory the blob actually holds (container sections plus
 * alignment padding and the derived cumulative and slot tables). */
uint64_t neuzip_device_bytes(const neuzip_blob *blob);

/* Element count, mantissa bits, normalisation block size (0 = none), guard band of the table
 * (0 = none) and element type the blob was made with (-1 for something that is not a blob). */
uint64_t neuzip_elems(const neuzip_blob *blob);
uint32_t neuzip_block_size(const neuzip_blob *blob);
uint32_t neuzip_guard(const neuzip_blob *blob);
int neuzip_mantissa_bits(const neuzip_blob *blob);
int neuzip_dtype(const neuzip_blob *blob);

/*
 * neuzip_export / neuzip_import -- the container as one flat host byte buffer
 * (App. D storage layout: compressed exponents next to the signed mantissas).
 * Export synchronises hip_stream.  With h_buf == NULL only *written is set.
 * Import validates every section on the host before anything is uploaded
 * (ECORRUPT otherwise) and creates a new blob.
 */
int neuzip_export(const neuzip_blob *blob, void *h_buf, uint64_t cap, uint64_t *written,
                  void *hip_stream);
int neuzip_import(const void *h_buf, uint64_t len, void *hip_stream, neuzip_blob **blob);

/* Exponent statistics of the tensor the blob was compressed from (Sec. 2.2):
 * h_counts receives the 256-bin histogram (EINVAL for imported blobs, which
 * carry no counts), h_freq the quantised frequencies that sum to 4096. */
int neuzip_histogram(const neuzip_blob *blob, uint32_t h_counts[256]);
int neuzip_frequencies(const neuzip_blob *blob, uint16_t h_freq[256]);

/*
 * neuzip_stream_probe -- measurement aid for the throughput experiment of Sec. 3 (the throughput
 * figure compares against plain data movement): one kernel that only moves bytes the way the fused
 * decoder does, in the decoder's launch shape -- workgroups of 512 lanes that own 32 chunks of 8 KB
 * of output and hold the decoder's LDS, a 128-bit copy of their share of the input into LDS at the
 * start, then per lane and turn a field load of 8, 4, 2 or 1 bytes and a 16-byte store 256 bytes
 * apart, four turns at a time, non-temporal stores from 128 MB of output up -- reading (nearly all
 * of) in_bytes from d_in and writing out_bytes to d_out.  Its rate is the ceiling for a decoder with
 * that access pattern and byte mix on the machine at hand.
 *   d_in, d_out   device buffers, 16-byte aligned; in_bytes and out_bytes multiples of 16; out_bytes
 *                 at least 8208; in_bytes between 1/16 of out_bytes (plus one workgroup's worth) and
 *                 about 1.2 times out_bytes; d_out is overwritten with a pattern.  EINVAL otherwise.
 * Never allocates, never synchronises.
 */
int neuzip_stream_probe(const void *d_in, uint64_t in_bytes, void *d_out, uint64_t out_bytes, void *hip_stream);

/* Synchronises hip_stream and returns ECORRUPT if any decompression of this
 * blob so far found a state that did not return to its initial value or a
 * word run that was not consumed exactly; clears the flag. */
int neuzip_check(const neuzip_blob *blob, void *hip_stream);

/*
 * neuzip_compress_noalloc -- neuzip_compress for callers that cannot allocate device or pinned
 * memory at the time of the call: code that runs where hipMalloc is forbidden (a region under
 * stream capture, a tight serving or training loop, a harness that intercepts allocation).
 *
 *   d_src, n_elems, dtype, mantissa_bits, hip_stream   as for neuzip_compress.
 *   blob    an existing blob of this library made from a tensor of the same n_elems, dtype and
 *           mantissa_bits without block-wise normalisation (else EINVAL / EUNSUPPORTED).  It
 *           receives the new tensor; its old content is lost; its guard band is kept.
 *
 * The result is the same as neuzip_compress into that blob: same table, same stream, same container.
 * What differs: the pipeline's workspace (histogram bins, encoder constants, run slots, word
 * counts, the record of the stream length) is a fixed array of about 6.6 MB inside the library's
 * device code, present once on every GPU the library runs on until the process ends, and the
 * stream length comes back by a copy from it.  The call makes no hipMalloc, hipHostMalloc or
 * hipFree.  Limits and error behaviour:
 *   - n_elems <= NEUZIP_NOALLOC_MAX_ELEMS, else EUNSUPPORTED (nothing is run).
 *   - the blob's word section is not grown: if the new stream needs more room than the blob
 *     holds, the call returns ENOMEM and the blob holds no tensor until a compress call succeeds
 *     (its fixed sections have been overwritten by then).  A blob last filled by a tensor of the
 *     same or a higher exponent entropy has room.
 *   - all calls on one GPU share that GPU's array: calls that overlap in time on one GPU (from
 *     several host threads or streams) race and must be serialised by the caller.  The array
 *     keeps the last call's contents; the call clears what has to start at zero.
 * Synchronises hip_stream once, like neuzip_compress.
 */
#define NEUZIP_NOALLOC_MAX_ELEMS (1ull << 22)
int neuzip_compress_noalloc(const void *d_src, uint64_t n_elems, int dtype, int mantissa_bits,
                            void *hip_stream, neuzip_blob *blob);

/* Device bytes of the workspace that compress calls share and keep between calls: the encoder's
 * run slots -- 16 x 200 words per 4096-element chunk, 1.56 bytes per element of the largest batch
 * compressed so far, but never more than the workspace limit below -- plus word counts and histogram
 * bins.  It is not part of any blob; Sec. 2.2's peak-memory accounting has to count it while weights
 * are being compressed (training), and neuzip_release_workspace returns it (inference, once the
 * model is compressed).  0 if none is held. */
uint64_t neuzip_workspace_bytes(void);

/* Limit on the encoder's run slots, in bytes (default 384 MiB, i.e. 251 M elements; 0 restores the
 * default; at least one group of 16 chunks, 102400 bytes, is always allowed).  A batch that would need
 * more is compressed tensor by tensor, and a single tensor that would need more goes through the
 * encoder in tiles of whole chunks, with one wait for the host per tile; the containers are the
 * same.  A workspace already larger than the new limit is freed.  Applies to all compress, recompress
 * and update calls except neuzip_compress_noalloc.  Not to be called while such a call runs. */
int neuzip_set_workspace_limit(uint64_t slot_bytes);

/* Frees the per-device workspace compress keeps between calls. */
int neuzip_release_workspace(void);

const char *neuzip_strerror(int code);
/* hipError_t of the last failing HIP call on this host thread (0 if none). */
int neuzip_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif
