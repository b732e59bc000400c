/*
 * NeuZip CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-purpose C implementation of what the NeuZip hot path
 * computes: bf16 weights are split into sign / exponent / mantissa (Alg. 1,
 * "split"; App. D), the exponent bytes are entropy-coded with a range-variant
 * asymmetric numeral system (Sec. 2.2, "Compression algorithm"), the sign and
 * the (optionally truncated, Sec. 2.3) mantissa are stored together as a
 * packed signed field, and decoding merges the three parts back (Alg. 1,
 * "merge").  Everything is written element by element in the order the text
 * gives, with no blocking, fusion or SIMD, so that it can be read against the
 * paper by eye.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this.  It shares no source, header, table generator or helper with the HIP
 * library and neither includes the other.
 *
 * Parity status: decoded values (lossless identity, lossy truncation), the
 * split/pack bit layout, the histogram, the frequency table and the rANS step
 * arithmetic are pinned by tests against definitions outside this file.  The
 * byte layout of the compressed stream is not given by the paper at all
 * (it names only "ANS"): for that layout the status is "parity unpinned" --
 * it is fixed by the format description below and cross-checked by a second,
 * independent pure-Python codec.
 *
 * ---------------------------------------------------------------------------
 * Stream format (all integers little-endian)
 *
 *   PROB_BITS = 12 (M = 4096), CHUNK = 4096 exponent symbols, K = 16 rANS
 *   states per chunk, G = 8 consecutive symbols per state turn, 32-bit states
 *   with lower bound L = 2^16, renormalisation in 16-bit words.
 *
 *   Within a chunk, local symbol i belongs to state j = (i mod (K*G)) / G.
 *   Every state codes its own symbols in ascending i when decoding and owns a
 *   private run of 16-bit words, stored in the order the decoder consumes
 *   them.
 *
 *   container := header(64 B) | freq[256] u16 | offsets[n_chunks+1] u32
 *              | states[n_chunks*K] u32 | lens[n_chunks*K] u8
 *              | words[total_words] u16 | signmant[ceil(n*(k+1)/8)] u8
 *              | low[n] u16               (only when header word 56, element type, is 1 = binary32)
 *              | coef[ceil(n/block)] u8   (only when header word 48, block, is not 0)
 *   header: magic u32 @0, version u32 @4, n u64 @8, k @16, PROB_BITS @20, CHUNK @24, K @28,
 *   G @32, n_chunks @36, total_words u64 @40, block @48, guard @52, element type @56 (u32 unless
 *   noted), rest 0.
 *   every section is zero-padded to a multiple of 16 bytes.
 *   offsets[c] = number of words that belong to chunks before c.
 *   Inside chunk c the K private runs follow each other, state 0 first;
 *   lens[c*K+j] is the run length of state j in words (at most 193).
 */
#ifndef NEUZIP_ORACLE_H
#define NEUZIP_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    NZO_PROB_BITS = 12,
    NZO_M = 1 << NZO_PROB_BITS,
    NZO_CHUNK = 4096,
    NZO_K = 16,
    NZO_G = 8,
    NZO_HEADER_BYTES = 64
};
#define NZO_L 65536u
#define NZO_MAGIC 0x315A554Eu /* "NUZ1" */

enum { NZO_OK = 0, NZO_EINVAL = -1, NZO_ENOSPACE = -2, NZO_ECORRUPT = -4, NZO_ESTALE = -6 };

/* Alg. 1 "split": bf16 word -> sign bit, 8-bit exponent, 7-bit mantissa. */
void nzo_split(const uint16_t *w, uint64_t n, uint8_t *sign, uint8_t *expo, uint8_t *mant);
/* Alg. 1 "merge": inverse of nzo_split. */
void nzo_merge(const uint8_t *sign, const uint8_t *expo, const uint8_t *mant, uint64_t n, uint16_t *w);
/* Sec. 2.3: keep the k most significant mantissa bits, clear the rest. */
void nzo_truncate(const uint16_t *w, uint64_t n, int k, uint16_t *out);
/* Sec. 2.3 / App. D: signed (k+1)-bit field = sign on top of the k kept
 * mantissa bits, 8/(k+1) fields per byte, first element in the low bits. */
uint64_t nzo_signmant_bytes(uint64_t n, int k);
int nzo_pack_signmant(const uint16_t *w, uint64_t n, int k, uint8_t *out);

/* Sec. 2.3, block-wise normalisation (reading stated in the .c file): one
 * coefficient byte per block of 32..512 consecutive weights = mantissa of the
 * largest-magnitude weight; stored weight = bf16(w / c), decoded weight =
 * bf16(stored * c) with c = 1 + coef/128. */
uint64_t nzo_block_count(uint64_t n, uint32_t block);
int nzo_block_coefficients(const uint16_t *w, uint64_t n, uint32_t block, uint8_t *coef);
void nzo_normalise(const uint16_t *w, uint64_t n, uint32_t block, const uint8_t *coef, uint16_t *out);
void nzo_denormalise(const uint16_t *w, uint64_t n, uint32_t block, const uint8_t *coef, uint16_t *out);

/* Sec. 2.2: symbol statistics over the 256 exponent values. */
void nzo_histogram(const uint16_t *w, uint64_t n, uint64_t cnt[256]);
/* Eq. (1) on the empirical distribution, bits per symbol. */
double nzo_entropy(const uint64_t cnt[256]);
/* Expected code length per symbol under the quantised table, bits. */
double nzo_cross_entropy(const uint64_t cnt[256], const uint16_t freq[256]);
/* Integer quantisation of the counts to frequencies that sum to M. */
int nzo_quantise(const uint64_t cnt[256], uint16_t freq[256]);
/* The same, but every exponent within `guard` of the occupied range counts as occurring (f >= 1),
 * so that the table can still code the tensor after a small update.  guard = 0: plain rule. */
int nzo_quantise_guarded(const uint64_t cnt[256], uint32_t guard, uint16_t freq[256]);

/* One coding step for a symbol with frequency f and cumulative start c.
 * Encoding moves the low 16 bits of x out first when needed (*emitted = 1,
 * *word holds them); decoding takes next_word in when x falls below L. */
uint32_t nzo_rans_encode_step(uint32_t x, uint32_t f, uint32_t c, uint16_t *word, int *emitted);
uint32_t nzo_rans_decode_step(uint32_t x, uint32_t f, uint32_t c, uint16_t next_word, int *consumed);

/* rANS over one chunk of m symbols with K states and turn length G.
 * words_cap is per state; state j writes words[j*words_cap ...]. */
int nzo_encode_chunk(const uint8_t *sym, uint32_t m, const uint16_t freq[256], int K, int G,
                     uint32_t *states, uint16_t *lens, uint16_t *words, uint32_t words_cap);
int nzo_decode_chunk(uint8_t *sym, uint32_t m, const uint16_t freq[256], int K, int G,
                     const uint32_t *states, const uint16_t *lens, const uint16_t *words,
                     uint32_t words_cap);

/* Whole-tensor container. */
uint64_t nzo_compress_bound(uint64_t n, int k);
int nzo_compress(const uint16_t *w, uint64_t n, int k, uint8_t *blob, uint64_t cap,
                 uint64_t *written, int threads);
/* Table with a guard band; header word 52 holds the guard. */
int nzo_compress_guarded(const uint16_t *w, uint64_t n, int k, uint32_t guard, uint8_t *blob,
                         uint64_t cap, uint64_t *written, int threads);
/* Compression with an earlier table instead of fresh statistics (Alg. 1 recompresses after every
 * update); NZO_ESTALE when an exponent of w has frequency 0 in that table. */
int nzo_compress_with_table(const uint16_t *w, uint64_t n, int k, const uint16_t freq[256],
                            uint32_t guard, uint8_t *blob, uint64_t cap, uint64_t *written,
                            int threads);
/* Lossy container with block-wise normalisation (k in {3,1,0}); header word 48 holds the
 * block size and a section coef[ceil(n/block)] u8 follows the sign|mantissa stream. */
int nzo_compress_blockwise(const uint16_t *w, uint64_t n, int k, uint32_t block, uint8_t *blob,
                           uint64_t cap, uint64_t *written, int threads);
int nzo_decompress(const uint8_t *blob, uint64_t len, uint16_t *out, uint64_t n, int threads);
/* binary32 tensors (not in the paper, which uses BFloat16 only): the upper halves go through the
 * lossless path as bf16 words, the lower halves are stored raw in a plane after the
 * sign|mantissa stream; header word 56 is 1. */
/* element types recorded in header word 56 */
#define NZO_ELEM_BF16 0u
#define NZO_ELEM_F32 1u
#define NZO_ELEM_F16 2u

int nzo_compress_f32(const uint32_t *w, uint64_t n, uint8_t *blob, uint64_t cap, uint64_t *written, int threads);
int nzo_compress_f32_with_table(const uint32_t *w, uint64_t n, const uint16_t *freq, uint32_t guard, uint8_t *blob,
                                uint64_t cap, uint64_t *written, int threads);
int nzo_decompress_f32(const uint8_t *blob, uint64_t len, uint32_t *out, uint64_t n, int threads);

/* binary16 words: upper byte entropy-coded in place of the exponent, lower byte raw; freq / guard as
 * for nzo_compress_with_table (freq may be NULL for fresh statistics). */
int nzo_compress_f16(const uint16_t *w, uint64_t n, const uint16_t *freq, uint32_t guard, uint8_t *blob, uint64_t cap,
                     uint64_t *written, int threads);
int nzo_decompress_f16(const uint8_t *blob, uint64_t len, uint16_t *out, uint64_t n, int threads);
/* Reads n, k and the stored frequencies out of a container. */
int nzo_blob_info(const uint8_t *blob, uint64_t len, uint64_t *n, int *k, uint64_t *total_words,
                  uint16_t freq[256]);

#ifdef __cplusplus
}
#endif
#endif
