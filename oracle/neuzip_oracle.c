/*
 * NeuZip CPU oracle -- TEST INFRASTRUCTURE ONLY.  See neuzip_oracle.h for the
 * scope, the parity status and the stream format.
 */
#include "neuzip_oracle.h"

#include <math.h>
#include <pthread.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Alg. 1 "split" / "merge", App. D: a bf16 word is                    */
/*   bit 15 sign | bits 14..7 exponent | bits 6..0 mantissa            */
/* ------------------------------------------------------------------ */
void nzo_split(const uint16_t *w, uint64_t n, uint8_t *sign, uint8_t *expo, uint8_t *mant)
{
    for (uint64_t i = 0; i < n; i++) {
        uint16_t u = w[i];
        sign[i] = (uint8_t)(u >> 15);
        expo[i] = (uint8_t)((u >> 7) & 0xFF);
        mant[i] = (uint8_t)(u & 0x7F);
    }
}

void nzo_merge(const uint8_t *sign, const uint8_t *expo, const uint8_t *mant, uint64_t n, uint16_t *w)
{
    for (uint64_t i = 0; i < n; i++)
        w[i] = (uint16_t)(((uint16_t)sign[i] << 15) | ((uint16_t)expo[i] << 7) | mant[i]);
}

static int valid_k(int k) { return k == 7 || k == 3 || k == 1 || k == 0; }

/* Sec. 2.3: only the k leading mantissa bits survive; sign and exponent are
 * untouched, the dropped bits read as zero (truncation toward zero). */
void nzo_truncate(const uint16_t *w, uint64_t n, int k, uint16_t *out)
{
    uint16_t dropped = (uint16_t)((1u << (7 - k)) - 1u);
    for (uint64_t i = 0; i < n; i++)
        out[i] = (uint16_t)(w[i] & (uint16_t)~dropped);
}

uint64_t nzo_signmant_bytes(uint64_t n, int k)
{
    uint64_t bits = n * (uint64_t)(k + 1);
    return (bits + 7) / 8;
}

/* Sec. 2.3 / App. D: sign and kept mantissa bits form one signed field of
 * k+1 bits (sign on top); 8/(k+1) fields share a byte, element i in bits
 * [(i mod P)*(k+1), ...) of byte i/P. */
int nzo_pack_signmant(const uint16_t *w, uint64_t n, int k, uint8_t *out)
{
    if (!valid_k(k))
        return NZO_EINVAL;
    int width = k + 1;
    int per_byte = 8 / width;
    memset(out, 0, nzo_signmant_bytes(n, k));
    for (uint64_t i = 0; i < n; i++) {
        uint16_t u = w[i];
        unsigned sign = u >> 15;
        unsigned mant = u & 0x7F;
        unsigned field = (sign << k) | (mant >> (7 - k));
        out[i / per_byte] |= (uint8_t)(field << ((i % per_byte) * width));
    }
    return NZO_OK;
}

/* ------------------------------------------------------------------ */
/* Block-wise normalisation of the lossy variant (Sec. 2.3, last        */
/* paragraph; block sizes 32..512 in the block-size study of Sec. 3).   */
/*                                                                      */
/* Reading taken here: a block is `block` consecutive weights.  Its     */
/* coefficient is the mantissa of the weight of largest magnitude (the  */
/* exponent is ignored; first such weight on ties), one byte per block. */
/* With c = 1 + coef/128 every weight is stored as bf16(w / c), so the  */
/* largest weight becomes a power of two and passes through mantissa    */
/* truncation unchanged; decoding returns bf16(stored * c).  Both       */
/* roundings are to nearest even; the arithmetic is IEEE binary32.      */
/* ------------------------------------------------------------------ */
static float bf16_value(uint16_t u)
{
    uint32_t bits = (uint32_t)u << 16;
    float v;
    memcpy(&v, &bits, 4);
    return v;
}

static uint16_t bf16_round(float v)
{
    uint32_t bits;
    memcpy(&bits, &v, 4);
    if ((bits & 0x7FFFFFFFu) > 0x7F800000u) /* NaN stays NaN */
        return (uint16_t)((bits >> 16) | 0x40u);
    /* round to nearest, ties to the even bf16 */
    return (uint16_t)((bits + 0x7FFFu + ((bits >> 16) & 1u)) >> 16);
}

static int valid_block(uint32_t block)
{
    return block == 32 || block == 64 || block == 128 || block == 256 || block == 512;
}

uint64_t nzo_block_count(uint64_t n, uint32_t block) { return block ? (n + block - 1) / block : 0; }

int nzo_block_coefficients(const uint16_t *w, uint64_t n, uint32_t block, uint8_t *coef)
{
    if (!valid_block(block))
        return NZO_EINVAL;
    for (uint64_t b = 0; b * block < n; b++) {
        uint64_t end = (b + 1) * block < n ? (b + 1) * block : n;
        uint64_t best = b * block;
        for (uint64_t i = b * block + 1; i < end; i++)
            if ((w[i] & 0x7FFFu) > (w[best] & 0x7FFFu)) /* magnitude order of bf16 words */
                best = i;
        coef[b] = (uint8_t)(w[best] & 0x7Fu);
    }
    return NZO_OK;
}

void nzo_normalise(const uint16_t *w, uint64_t n, uint32_t block, const uint8_t *coef, uint16_t *out)
{
    for (uint64_t i = 0; i < n; i++) {
        float c = 1.0f + (float)coef[i / block] / 128.0f;
        out[i] = bf16_round(bf16_value(w[i]) / c);
    }
}

void nzo_denormalise(const uint16_t *w, uint64_t n, uint32_t block, const uint8_t *coef, uint16_t *out)
{
    for (uint64_t i = 0; i < n; i++) {
        float c = 1.0f + (float)coef[i / block] / 128.0f;
        out[i] = bf16_round(bf16_value(w[i]) * c);
    }
}

/* ------------------------------------------------------------------ */
/* Symbol statistics (Sec. 2.2) and Eq. (1)                            */
/* ------------------------------------------------------------------ */
void nzo_histogram(const uint16_t *w, uint64_t n, uint64_t cnt[256])
{
    memset(cnt, 0, 256 * sizeof(uint64_t));
    for (uint64_t i = 0; i < n; i++)
        cnt[(w[i] >> 7) & 0xFF]++;
}

double nzo_entropy(const uint64_t cnt[256])
{
    uint64_t total = 0;
    for (int s = 0; s < 256; s++)
        total += cnt[s];
    if (total == 0)
        return 0.0;
    double h = 0.0;
    for (int s = 0; s < 256; s++) {
        if (cnt[s] == 0)
            continue;
        double p = (double)cnt[s] / (double)total;
        h -= p * log2(p);
    }
    return h;
}

double nzo_cross_entropy(const uint64_t cnt[256], const uint16_t freq[256])
{
    uint64_t total = 0;
    for (int s = 0; s < 256; s++)
        total += cnt[s];
    if (total == 0)
        return 0.0;
    double h = 0.0;
    for (int s = 0; s < 256; s++) {
        if (cnt[s] == 0)
            continue;
        double p = (double)cnt[s] / (double)total;
        h -= p * log2((double)freq[s] / (double)NZO_M);
    }
    return h;
}

/* Frequencies proportional to the counts, integer only:
 *   f = max(1, floor(cnt * M / N)) for every symbol that occurs, else 0;
 *   a shortfall goes to the most frequent symbol (lowest value on a tie);
 *   an excess is taken, one at a time, from the symbol whose f is largest
 *   at that moment (lowest value on a tie). */
int nzo_quantise(const uint64_t cnt[256], uint16_t freq[256])
{
    return nzo_quantise_guarded(cnt, 0, freq);
}

/* The same with a guard band for tables that outlive the tensor they were counted on (Alg. 1
 * compresses every weight again after each update; a table kept from the step before must be
 * able to code exponents the update newly produces).  With guard > 0 the symbols "that occur"
 * are taken to be every exponent from (smallest occurring - guard) to (largest occurring +
 * guard), clipped to 0..255, and symbol 0 as well (the exponent of +-0: an update w - lr * g
 * cancels exactly now and then, far below every other exponent that occurs): the ones with
 * count 0 get f = 1 by the same max(1, .) rule.  guard = 0 is the plain rule.  Not in the paper. */
int nzo_quantise_guarded(const uint64_t cnt[256], uint32_t guard, uint16_t freq[256])
{
    uint64_t total = 0;
    int lo = 256, hi = -1;
    for (int s = 0; s < 256; s++) {
        total += cnt[s];
        if (cnt[s] > 0) {
            if (lo == 256)
                lo = s;
            hi = s;
        }
    }
    uint32_t f[256];
    int64_t sum = 0;
    for (int s = 0; s < 256; s++) {
        int member = cnt[s] > 0;
        if (guard > 0 && total > 0 &&
            (s == 0 || ((int64_t)s >= (int64_t)lo - (int64_t)guard && (int64_t)s <= (int64_t)hi + (int64_t)guard)))
            member = 1;
        if (!member || total == 0) {
            f[s] = 0;
            continue;
        }
        /* cnt < 2^52 is required for the product to stay inside 64 bits */
        uint64_t scaled = cnt[s] * (uint64_t)NZO_M / total;
        f[s] = scaled < 1 ? 1u : (uint32_t)scaled;
        sum += f[s];
    }
    if (total == 0) {
        for (int s = 0; s < 256; s++)
            freq[s] = 0;
        return NZO_OK;
    }
    int64_t rest = (int64_t)NZO_M - sum;
    if (rest > 0) {
        int best = 0;
        for (int s = 1; s < 256; s++)
            if (cnt[s] > cnt[best])
                best = s;
        f[best] += (uint32_t)rest;
    }
    while (rest < 0) {
        int best = 0;
        for (int s = 1; s < 256; s++)
            if (f[s] > f[best])
                best = s;
        f[best]--;
        rest++;
    }
    for (int s = 0; s < 256; s++)
        freq[s] = (uint16_t)f[s];
    return NZO_OK;
}

/* ------------------------------------------------------------------ */
/* rANS (Sec. 2.2 "Compression algorithm", range variant of ANS)       */
/*                                                                      */
/* State x lives in [L, L * 2^16).  Coding symbol s with frequency f    */
/* and cumulative start c:                                              */
/*     encode:  x <- floor(x / f) * M + c + (x mod f)                   */
/*     decode:  slot = x mod M;  s = symbol whose [c, c+f) holds slot;  */
/*              x <- f * floor(x / M) + slot - c                        */
/* The encoder first moves the low 16 bits of x out whenever the step   */
/* would leave the interval; the decoder pulls them back when x drops   */
/* below L.  Encoding runs over the symbols backwards so that decoding  */
/* runs forwards.                                                       */
/* ------------------------------------------------------------------ */
uint32_t nzo_rans_encode_step(uint32_t x, uint32_t f, uint32_t c, uint16_t *word, int *emitted)
{
    /* smallest x for which the step would reach L * 2^16 */
    uint64_t limit = ((uint64_t)(NZO_L >> NZO_PROB_BITS) << 16) * f;
    *emitted = 0;
    *word = 0;
    if ((uint64_t)x >= limit) {
        *word = (uint16_t)(x & 0xFFFF);
        *emitted = 1;
        x >>= 16;
    }
    return ((x / f) << NZO_PROB_BITS) + (x % f) + c;
}

uint32_t nzo_rans_decode_step(uint32_t x, uint32_t f, uint32_t c, uint16_t next_word, int *consumed)
{
    uint32_t slot = x & (NZO_M - 1);
    uint32_t xn = f * (x >> NZO_PROB_BITS) + slot - c;
    *consumed = 0;
    if (xn < NZO_L) {
        xn = (xn << 16) | next_word;
        *consumed = 1;
    }
    return xn;
}

static void cumulative(const uint16_t freq[256], uint32_t cum[257])
{
    cum[0] = 0;
    for (int s = 0; s < 256; s++)
        cum[s + 1] = cum[s] + freq[s];
}

static int state_of(uint32_t i, int K, int G) { return (int)((i % (uint32_t)(K * G)) / (uint32_t)G); }

int nzo_encode_chunk(const uint8_t *sym, uint32_t m, const uint16_t freq[256], int K, int G,
                     uint32_t *states, uint16_t *lens, uint16_t *words, uint32_t words_cap)
{
    uint32_t cum[257];
    cumulative(freq, cum);
    if (m > 0 && cum[256] != NZO_M)
        return NZO_EINVAL;
    uint32_t *wpos = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)K);
    if (!wpos)
        return NZO_ENOSPACE;
    for (int j = 0; j < K; j++) {
        states[j] = NZO_L;
        wpos[j] = words_cap; /* runs are filled from the back */
    }
    for (uint32_t r = 0; r < m; r++) {
        uint32_t i = m - 1 - r;
        int j = state_of(i, K, G);
        uint32_t s = sym[i];
        uint32_t f = freq[s];
        if (f == 0) {
            free(wpos);
            return NZO_EINVAL;
        }
        uint16_t word;
        int emitted;
        states[j] = nzo_rans_encode_step(states[j], f, cum[s], &word, &emitted);
        if (emitted) {
            if (wpos[j] == 0) {
                free(wpos);
                return NZO_ENOSPACE;
            }
            wpos[j]--;
            words[(size_t)j * words_cap + wpos[j]] = word;
        }
    }
    for (int j = 0; j < K; j++) {
        uint32_t len = words_cap - wpos[j];
        lens[j] = (uint16_t)len;
        memmove(&words[(size_t)j * words_cap], &words[(size_t)j * words_cap + wpos[j]],
                (size_t)len * sizeof(uint16_t));
    }
    free(wpos);
    return NZO_OK;
}

int nzo_decode_chunk(uint8_t *sym, uint32_t m, const uint16_t freq[256], int K, int G,
                     const uint32_t *states, const uint16_t *lens, const uint16_t *words,
                     uint32_t words_cap)
{
    uint32_t cum[257];
    cumulative(freq, cum);
    if (m > 0 && cum[256] != NZO_M)
        return NZO_ECORRUPT;
    /* slot -> symbol, written out from the definition of the intervals */
    uint8_t slot_symbol[NZO_M];
    for (int s = 0; s < 256; s++)
        for (uint32_t t = cum[s]; t < cum[s + 1]; t++)
            slot_symbol[t] = (uint8_t)s;

    uint32_t *x = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)K);
    uint32_t *pos = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)K);
    if (!x || !pos) {
        free(x);
        free(pos);
        return NZO_ENOSPACE;
    }
    for (int j = 0; j < K; j++) {
        x[j] = states[j];
        pos[j] = 0;
    }
    int rc = NZO_OK;
    for (uint32_t i = 0; i < m && rc == NZO_OK; i++) {
        int j = state_of(i, K, G);
        uint32_t s = slot_symbol[x[j] & (NZO_M - 1)];
        sym[i] = (uint8_t)s;
        uint16_t next = pos[j] < lens[j] ? words[(size_t)j * words_cap + pos[j]] : 0;
        int consumed;
        x[j] = nzo_rans_decode_step(x[j], freq[s], cum[s], next, &consumed);
        if (consumed) {
            if (pos[j] >= lens[j]) {
                rc = NZO_ECORRUPT;
                break;
            }
            pos[j]++;
        }
    }
    /* a well-formed chunk leaves every state where the encoder started and
     * every run fully consumed */
    for (int j = 0; j < K && rc == NZO_OK; j++)
        if (x[j] != NZO_L || pos[j] != lens[j])
            rc = NZO_ECORRUPT;
    free(x);
    free(pos);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Container                                                            */
/* ------------------------------------------------------------------ */
static uint64_t pad16(uint64_t v) { return (v + 15) & ~(uint64_t)15; }

static void put32(uint8_t *p, uint32_t v)
{
    p[0] = (uint8_t)v;
    p[1] = (uint8_t)(v >> 8);
    p[2] = (uint8_t)(v >> 16);
    p[3] = (uint8_t)(v >> 24);
}
static void put64(uint8_t *p, uint64_t v)
{
    put32(p, (uint32_t)v);
    put32(p + 4, (uint32_t)(v >> 32));
}
static uint32_t get32(const uint8_t *p)
{
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
static uint64_t get64(const uint8_t *p) { return (uint64_t)get32(p) | ((uint64_t)get32(p + 4) << 32); }
static void put16(uint8_t *p, uint16_t v)
{
    p[0] = (uint8_t)v;
    p[1] = (uint8_t)(v >> 8);
}
static uint16_t get16(const uint8_t *p) { return (uint16_t)(p[0] | (p[1] << 8)); }

/* Room for one state's words.  A step grows log2(x + 1) by at most 12 bits, an emitted word
 * shrinks it by at least 16 - log2(17/16) bits, so 256 symbols give at most 193 words. */
#define NZO_RUN_CAP 200u
#define NZO_RUN_MAX 193u

static uint64_t chunks_of(uint64_t n) { return (n + NZO_CHUNK - 1) / NZO_CHUNK; }

uint64_t nzo_compress_bound(uint64_t n, int k)
{
    uint64_t nc = chunks_of(n);
    return NZO_HEADER_BYTES + 512 + pad16((nc + 1) * 4) + nc * NZO_K * 4 + nc * NZO_K +
           pad16(nc * NZO_K * NZO_RUN_CAP * 2) + pad16(nzo_signmant_bytes(n, k)) + pad16(nzo_block_count(n, 32)) + pad16(n * 2);
}

typedef struct {
    const uint16_t *w;
    uint64_t n;
    const uint16_t *freq;
    uint64_t c_begin, c_end;
    uint32_t *states; /* [nc*K] */
    uint16_t *lens;   /* [nc*K] */
    uint16_t *words;  /* [nc*K*RUN_CAP] */
    int rc;
} enc_job;

static void *enc_worker(void *arg)
{
    enc_job *job = (enc_job *)arg;
    uint8_t expo[NZO_CHUNK];
    for (uint64_t c = job->c_begin; c < job->c_end; c++) {
        uint64_t base = c * NZO_CHUNK;
        uint32_t m = (uint32_t)((job->n - base) < NZO_CHUNK ? (job->n - base) : NZO_CHUNK);
        for (uint32_t i = 0; i < m; i++)
            expo[i] = (uint8_t)((job->w[base + i] >> 7) & 0xFF);
        int rc = nzo_encode_chunk(expo, m, job->freq, NZO_K, NZO_G, job->states + c * NZO_K,
                                  job->lens + c * NZO_K,
                                  job->words + c * NZO_K * NZO_RUN_CAP, NZO_RUN_CAP);
        if (rc != NZO_OK) {
            job->rc = rc;
            return NULL;
        }
        /* the bound derived above the capacity: no state of a 4096-symbol chunk emits more */
        for (int j = 0; j < NZO_K; j++) {
            if (job->lens[c * NZO_K + j] > NZO_RUN_MAX) {
                job->rc = NZO_ENOSPACE;
                return NULL;
            }
        }
    }
    return NULL;
}

static int compress_impl(const uint16_t *w, uint64_t n, int k, uint32_t block, const uint8_t *coef,
                         const uint16_t *given_freq, uint32_t guard, const uint16_t *low, uint32_t elem, uint8_t *blob, uint64_t cap,
                         uint64_t *written, int threads);

int nzo_compress(const uint16_t *w, uint64_t n, int k, uint8_t *blob, uint64_t cap,
                 uint64_t *written, int threads)
{
    return compress_impl(w, n, k, 0, NULL, NULL, 0, NULL, NZO_ELEM_BF16, blob, cap, written, threads);
}

/* The table keeps a guard band (nzo_quantise_guarded); header word 52 records the guard. */
int nzo_compress_guarded(const uint16_t *w, uint64_t n, int k, uint32_t guard, uint8_t *blob,
                         uint64_t cap, uint64_t *written, int threads)
{
    if (guard > 255)
        return NZO_EINVAL;
    return compress_impl(w, n, k, 0, NULL, NULL, guard, NULL, NZO_ELEM_BF16, blob, cap, written, threads);
}

/* Compression with a table that was made earlier (from the weights before an update): no
 * statistics are taken from w.  NZO_ESTALE if w holds an exponent the table gives no room. */
/* A kept table must sum to M (all zero for an empty tensor) and give every exponent that
 * occurs a non-zero frequency. */
static int kept_table_serves(const uint16_t *w, uint64_t n, const uint16_t freq[256], uint32_t guard)
{
    if (!freq || guard > 255)
        return NZO_EINVAL;
    uint32_t sum = 0;
    for (int s = 0; s < 256; s++)
        sum += freq[s];
    if (sum != NZO_M && !(n == 0 && sum == 0))
        return NZO_EINVAL;
    uint64_t cnt[256];
    nzo_histogram(w, n, cnt);
    for (int s = 0; s < 256; s++)
        if (cnt[s] > 0 && freq[s] == 0)
            return NZO_ESTALE;
    return NZO_OK;
}

int nzo_compress_with_table(const uint16_t *w, uint64_t n, int k, const uint16_t freq[256],
                            uint32_t guard, uint8_t *blob, uint64_t cap, uint64_t *written,
                            int threads)
{
    int rc = kept_table_serves(w, n, freq, guard);
    if (rc != NZO_OK)
        return rc;
    return compress_impl(w, n, k, 0, NULL, freq, guard, NULL, NZO_ELEM_BF16, blob, cap, written, threads);
}

/* Lossy variant with block-wise normalisation: the coefficients are taken from the original
 * weights, the weights are normalised, and the normalised tensor goes through the same path. */
int nzo_compress_blockwise(const uint16_t *w, uint64_t n, int k, uint32_t block, uint8_t *blob,
                           uint64_t cap, uint64_t *written, int threads)
{
    if (!valid_block(block) || k == 7 || !valid_k(k))
        return NZO_EINVAL;
    uint64_t nb = nzo_block_count(n, block);
    uint8_t *coef = (uint8_t *)malloc((size_t)nb + 1);
    uint16_t *normal = (uint16_t *)malloc((size_t)(n + 1) * sizeof(uint16_t));
    if (!coef || !normal) {
        free(coef);
        free(normal);
        return NZO_ENOSPACE;
    }
    nzo_block_coefficients(w, n, block, coef);
    nzo_normalise(w, n, block, coef, normal);
    int rc = compress_impl(normal, n, k, block, coef, NULL, 0, NULL, NZO_ELEM_BF16, blob, cap, written, threads);
    free(coef);
    free(normal);
    return rc;
}

static int compress_impl(const uint16_t *w, uint64_t n, int k, uint32_t block, const uint8_t *coef,
                         const uint16_t *given_freq, uint32_t guard, const uint16_t *low, uint32_t elem, uint8_t *blob, uint64_t cap,
                         uint64_t *written, int threads)
{
    if (!valid_k(k) || n >= ((uint64_t)1 << 32))
        return NZO_EINVAL;
    if (threads < 1)
        threads = 1;
    uint64_t nc = chunks_of(n);

    uint64_t cnt[256];
    uint16_t freq[256];
    if (given_freq) {
        memcpy(freq, given_freq, sizeof(freq));
    } else {
        nzo_histogram(w, n, cnt);
        nzo_quantise_guarded(cnt, guard, freq);
    }

    uint32_t *states = (uint32_t *)malloc((size_t)(nc * NZO_K + 1) * sizeof(uint32_t));
    uint16_t *lens = (uint16_t *)malloc((size_t)(nc * NZO_K + 1) * sizeof(uint16_t));
    uint16_t *words = (uint16_t *)malloc((size_t)(nc * NZO_K * NZO_RUN_CAP + 1) * sizeof(uint16_t));
    if (!states || !lens || !words) {
        free(states);
        free(lens);
        free(words);
        return NZO_ENOSPACE;
    }

    if ((uint64_t)threads > nc)
        threads = nc ? (int)nc : 1;
    enc_job *jobs = (enc_job *)calloc((size_t)threads, sizeof(enc_job));
    pthread_t *tid = (pthread_t *)calloc((size_t)threads, sizeof(pthread_t));
    for (int t = 0; t < threads; t++) {
        jobs[t].w = w;
        jobs[t].n = n;
        jobs[t].freq = freq;
        jobs[t].c_begin = nc * (uint64_t)t / (uint64_t)threads;
        jobs[t].c_end = nc * (uint64_t)(t + 1) / (uint64_t)threads;
        jobs[t].states = states;
        jobs[t].lens = lens;
        jobs[t].words = words;
        jobs[t].rc = NZO_OK;
    }
    if (threads == 1) {
        enc_worker(&jobs[0]);
    } else {
        for (int t = 0; t < threads; t++)
            pthread_create(&tid[t], NULL, enc_worker, &jobs[t]);
        for (int t = 0; t < threads; t++)
            pthread_join(tid[t], NULL);
    }
    int rc = NZO_OK;
    for (int t = 0; t < threads; t++)
        if (jobs[t].rc != NZO_OK)
            rc = jobs[t].rc;
    free(jobs);
    free(tid);

    uint64_t total_words = 0;
    for (uint64_t i = 0; i < nc * NZO_K; i++)
        total_words += lens[i];

    uint64_t sm_bytes = nzo_signmant_bytes(n, k);
    uint64_t off_freq = NZO_HEADER_BYTES;
    uint64_t off_offsets = off_freq + 512;
    uint64_t off_states = off_offsets + pad16((nc + 1) * 4);
    uint64_t off_lens = off_states + nc * NZO_K * 4;
    uint64_t off_words = off_lens + nc * NZO_K;
    uint64_t off_sm = off_words + pad16(total_words * 2);
    uint64_t off_low = off_sm + pad16(sm_bytes);
    uint64_t off_coef = off_low + (low ? pad16(n * 2) : 0);
    uint64_t size = off_coef + pad16(nzo_block_count(n, block));
    if (written)
        *written = size;
    if (rc == NZO_OK && (size > cap || total_words >= ((uint64_t)1 << 32)))
        rc = NZO_ENOSPACE;
    if (rc != NZO_OK) {
        free(states);
        free(lens);
        free(words);
        return rc;
    }

    memset(blob, 0, size);
    put32(blob + 0, NZO_MAGIC);
    put32(blob + 4, 1);
    put64(blob + 8, n);
    put32(blob + 16, (uint32_t)k);
    put32(blob + 20, NZO_PROB_BITS);
    put32(blob + 24, NZO_CHUNK);
    put32(blob + 28, NZO_K);
    put32(blob + 32, NZO_G);
    put32(blob + 36, (uint32_t)nc);
    put64(blob + 40, total_words);
    put32(blob + 48, block); /* 0: no block-wise normalisation, no coefficient section */
    put32(blob + 52, guard); /* guard band the table was made with (0: none) */
    for (int s = 0; s < 256; s++)
        put16(blob + off_freq + 2 * s, freq[s]);

    uint64_t run = 0; /* words written so far */
    for (uint64_t c = 0; c < nc; c++) {
        put32(blob + off_offsets + 4 * c, (uint32_t)run);
        for (int j = 0; j < NZO_K; j++) {
            uint64_t idx = c * NZO_K + j;
            put32(blob + off_states + 4 * idx, states[idx]);
            blob[off_lens + idx] = (uint8_t)lens[idx];
            for (uint32_t t = 0; t < lens[idx]; t++)
                put16(blob + off_words + 2 * (run + t), words[idx * NZO_RUN_CAP + t]);
            run += lens[idx];
        }
    }
    put32(blob + off_offsets + 4 * nc, (uint32_t)run);
    put32(blob + 56, elem); /* element type: 0 bf16, 1 binary32 (with a plane of low halves), 2 binary16 */
    nzo_pack_signmant(w, n, k, blob + off_sm);
    if (low)
        for (uint64_t i = 0; i < n; i++)
            put16(blob + off_low + 2 * i, low[i]);
    if (block)
        memcpy(blob + off_coef, coef, nzo_block_count(n, block));

    free(states);
    free(lens);
    free(words);
    return NZO_OK;
}

typedef struct {
    uint64_t n, nc, total_words;
    int k;
    uint32_t block;
    uint32_t elem; /* element type; binary32: a plane of low halves follows the sign|mantissa stream */
    const uint8_t *low;
    const uint8_t *freq, *offsets, *states, *lens, *words, *sm, *coef;
} blob_view;

static int open_blob(const uint8_t *blob, uint64_t len, blob_view *v)
{
    if (len < NZO_HEADER_BYTES + 512)
        return NZO_ECORRUPT;
    if (get32(blob) != NZO_MAGIC || get32(blob + 4) != 1)
        return NZO_ECORRUPT;
    v->n = get64(blob + 8);
    v->k = (int)get32(blob + 16);
    if (!valid_k(v->k) || get32(blob + 20) != NZO_PROB_BITS || get32(blob + 24) != NZO_CHUNK ||
        get32(blob + 28) != NZO_K || get32(blob + 32) != NZO_G)
        return NZO_ECORRUPT;
    v->nc = get32(blob + 36);
    v->total_words = get64(blob + 40);
    v->block = get32(blob + 48);
    if (v->nc != chunks_of(v->n))
        return NZO_ECORRUPT;
    if (v->block != 0 && (!valid_block(v->block) || v->k == 7))
        return NZO_ECORRUPT;
    uint64_t off_freq = NZO_HEADER_BYTES;
    uint64_t off_offsets = off_freq + 512;
    uint64_t off_states = off_offsets + pad16((v->nc + 1) * 4);
    uint64_t off_lens = off_states + v->nc * NZO_K * 4;
    uint64_t off_words = off_lens + v->nc * NZO_K;
    uint64_t off_sm = off_words + pad16(v->total_words * 2);
    v->elem = get32(blob + 56);
    if (v->elem > NZO_ELEM_F16 || (v->elem != NZO_ELEM_BF16 && (v->k != 7 || v->block != 0)))
        return NZO_ECORRUPT;
    uint64_t off_low = off_sm + pad16(nzo_signmant_bytes(v->n, v->k));
    uint64_t off_coef = off_low + (v->elem == NZO_ELEM_F32 ? pad16(v->n * 2) : 0);
    uint64_t size = off_coef + pad16(nzo_block_count(v->n, v->block));
    if (size != len)
        return NZO_ECORRUPT;
    v->freq = blob + off_freq;
    v->offsets = blob + off_offsets;
    v->states = blob + off_states;
    v->lens = blob + off_lens;
    v->words = blob + off_words;
    v->sm = blob + off_sm;
    v->low = blob + off_low;
    v->coef = blob + off_coef;
    return NZO_OK;
}

int nzo_blob_info(const uint8_t *blob, uint64_t len, uint64_t *n, int *k, uint64_t *total_words,
                  uint16_t freq[256])
{
    blob_view v;
    int rc = open_blob(blob, len, &v);
    if (rc != NZO_OK)
        return rc;
    if (n)
        *n = v.n;
    if (k)
        *k = v.k;
    if (total_words)
        *total_words = v.total_words;
    if (freq)
        for (int s = 0; s < 256; s++)
            freq[s] = get16(v.freq + 2 * s);
    return NZO_OK;
}

typedef struct {
    const blob_view *v;
    const uint16_t *freq;
    uint64_t c_begin, c_end;
    uint16_t *out;
    int rc;
} dec_job;

static void *dec_worker(void *arg)
{
    dec_job *job = (dec_job *)arg;
    const blob_view *v = job->v;
    int k = v->k;
    int width = k + 1;
    int per_byte = 8 / width;
    uint8_t expo[NZO_CHUNK];
    uint32_t states[NZO_K];
    uint16_t lens[NZO_K];
    uint16_t *words = (uint16_t *)malloc(sizeof(uint16_t) * NZO_K * NZO_RUN_CAP);
    if (!words) {
        job->rc = NZO_ENOSPACE;
        return NULL;
    }
    for (uint64_t c = job->c_begin; c < job->c_end; c++) {
        uint64_t base = c * NZO_CHUNK;
        uint32_t m = (uint32_t)((v->n - base) < NZO_CHUNK ? (v->n - base) : NZO_CHUNK);
        uint64_t run = get32(v->offsets + 4 * c);
        uint64_t next = get32(v->offsets + 4 * (c + 1));
        uint64_t have = 0;
        int bad = 0;
        for (int j = 0; j < NZO_K; j++) {
            uint64_t idx = c * NZO_K + j;
            states[j] = get32(v->states + 4 * idx);
            lens[j] = v->lens[idx];
            if (lens[j] > NZO_RUN_CAP || run + have + lens[j] > v->total_words) {
                bad = 1;
                break;
            }
            for (uint32_t t = 0; t < lens[j]; t++)
                words[(size_t)j * NZO_RUN_CAP + t] = get16(v->words + 2 * (run + have + t));
            have += lens[j];
        }
        if (bad || run + have != next) {
            job->rc = NZO_ECORRUPT;
            break;
        }
        int rc = nzo_decode_chunk(expo, m, job->freq, NZO_K, NZO_G, states, lens, words, NZO_RUN_CAP);
        if (rc != NZO_OK) {
            job->rc = rc;
            break;
        }
        /* Alg. 1 "merge": sign | decoded exponent | kept mantissa bits, zeros below */
        for (uint32_t i = 0; i < m; i++) {
            uint64_t g = base + i;
            unsigned field = (v->sm[g / per_byte] >> ((g % per_byte) * width)) & ((1u << width) - 1u);
            unsigned sign = field >> k;
            unsigned mant = (field & ((1u << k) - 1u)) << (7 - k);
            job->out[g] = (uint16_t)((sign << 15) | ((unsigned)expo[i] << 7) | mant);
        }
    }
    free(words);
    return NULL;
}

static int decompress_halves(const uint8_t *blob, uint64_t len, uint16_t *out, uint64_t n, int threads, uint32_t want_elem)
{
    blob_view v;
    int rc = open_blob(blob, len, &v);
    if (rc != NZO_OK)
        return rc;
    if (v.n != n || v.elem != want_elem)
        return NZO_EINVAL;
    if (get32(v.offsets) != 0 || get32(v.offsets + 4 * v.nc) != v.total_words)
        return NZO_ECORRUPT;
    uint16_t freq[256];
    for (int s = 0; s < 256; s++)
        freq[s] = get16(v.freq + 2 * s);
    if (threads < 1)
        threads = 1;
    if ((uint64_t)threads > v.nc)
        threads = v.nc ? (int)v.nc : 1;
    dec_job *jobs = (dec_job *)calloc((size_t)threads, sizeof(dec_job));
    pthread_t *tid = (pthread_t *)calloc((size_t)threads, sizeof(pthread_t));
    for (int t = 0; t < threads; t++) {
        jobs[t].v = &v;
        jobs[t].freq = freq;
        jobs[t].c_begin = v.nc * (uint64_t)t / (uint64_t)threads;
        jobs[t].c_end = v.nc * (uint64_t)(t + 1) / (uint64_t)threads;
        jobs[t].out = out;
        jobs[t].rc = NZO_OK;
    }
    if (threads == 1) {
        dec_worker(&jobs[0]);
    } else {
        for (int t = 0; t < threads; t++)
            pthread_create(&tid[t], NULL, dec_worker, &jobs[t]);
        for (int t = 0; t < threads; t++)
            pthread_join(tid[t], NULL);
    }
    for (int t = 0; t < threads; t++)
        if (jobs[t].rc != NZO_OK)
            rc = jobs[t].rc;
    free(jobs);
    free(tid);
    if (rc == NZO_OK && v.block)
        nzo_denormalise(out, n, v.block, v.coef, out);
    return rc;
}

int nzo_decompress(const uint8_t *blob, uint64_t len, uint16_t *out, uint64_t n, int threads)
{
    return decompress_halves(blob, len, out, n, threads, NZO_ELEM_BF16);
}

/* ------------------------------------------------------------------ */
/* binary32 tensors (the paper works on BFloat16 only, Sec. 2.1).       */
/* The upper half of a binary32 word is a bf16 word: sign, the same 8   */
/* exponent bits, the 7 leading mantissa bits.  It goes through the     */
/* path above unchanged (lossless only); the lower halves, 16 further   */
/* mantissa bits that do not compress, are stored as they are in a      */
/* plane of their own after the sign|mantissa stream.                   */
/* ------------------------------------------------------------------ */
int nzo_compress_f32(const uint32_t *w, uint64_t n, uint8_t *blob, uint64_t cap, uint64_t *written, int threads)
{
    return nzo_compress_f32_with_table(w, n, NULL, 0, blob, cap, written, threads);
}

/* The same with a guard band, and with a table kept from an earlier compression when freq is
 * not NULL (the rules of nzo_compress_with_table, applied to the upper halves). */
int nzo_compress_f32_with_table(const uint32_t *w, uint64_t n, const uint16_t *freq, uint32_t guard, uint8_t *blob,
                                uint64_t cap, uint64_t *written, int threads)
{
    uint16_t *high = (uint16_t *)malloc((size_t)(n + 1) * sizeof(uint16_t));
    uint16_t *low = (uint16_t *)malloc((size_t)(n + 1) * sizeof(uint16_t));
    if (!high || !low) {
        free(high);
        free(low);
        return NZO_ENOSPACE;
    }
    for (uint64_t i = 0; i < n; i++) {
        high[i] = (uint16_t)(w[i] >> 16);
        low[i] = (uint16_t)(w[i] & 0xFFFF);
    }
    int rc = guard > 255 ? NZO_EINVAL : (freq ? kept_table_serves(high, n, freq, guard) : NZO_OK);
    if (rc == NZO_OK)
        rc = compress_impl(high, n, 7, 0, NULL, freq, guard, low, NZO_ELEM_F32, blob, cap, written, threads);
    free(high);
    free(low);
    return rc;
}

int nzo_decompress_f32(const uint8_t *blob, uint64_t len, uint32_t *out, uint64_t n, int threads)
{
    uint16_t *high = (uint16_t *)malloc((size_t)(n + 1) * sizeof(uint16_t));
    if (!high)
        return NZO_ENOSPACE;
    int rc = decompress_halves(blob, len, high, n, threads, NZO_ELEM_F32);
    if (rc == NZO_OK) {
        blob_view v;
        open_blob(blob, len, &v);
        for (uint64_t i = 0; i < n; i++)
            out[i] = ((uint32_t)high[i] << 16) | get16(v.low + 2 * i);
    }
    free(high);
    return rc;
}

/* ------------------------------------------------------------------ */
/* binary16 tensors (beyond the paper, which works on BFloat16).        */
/* sign 1 | exponent 5 | mantissa 10.  The upper byte of a word (sign,  */
/* exponent, two mantissa bits) takes the place of the bf16 exponent    */
/* byte as the entropy-coded symbol and the lower byte (eight mantissa  */
/* bits) the place of the sign|mantissa byte.  That is the lossless     */
/* bf16 path applied to the word with its bits rearranged:              */
/*   bits 15..8 -> 14..7,  bit 7 -> 15,  bits 6..0 stay,                */
/* so the container is the bf16 container of the rearranged words with  */
/* element type 2 in its header.                                        */
/* ------------------------------------------------------------------ */
static uint16_t f16_to_fields(uint16_t u) { return (uint16_t)(((u & 0x80u) << 8) | ((u >> 8) << 7) | (u & 0x7Fu)); }
static uint16_t f16_from_fields(uint16_t v) { return (uint16_t)((((v >> 7) & 0xFFu) << 8) | ((v >> 8) & 0x80u) | (v & 0x7Fu)); }

int nzo_compress_f16(const uint16_t *w, uint64_t n, const uint16_t *freq, uint32_t guard, uint8_t *blob, uint64_t cap,
                     uint64_t *written, int threads)
{
    uint16_t *fields = (uint16_t *)malloc((size_t)(n + 1) * sizeof(uint16_t));
    if (!fields)
        return NZO_ENOSPACE;
    for (uint64_t i = 0; i < n; i++)
        fields[i] = f16_to_fields(w[i]);
    int rc = guard > 255 ? NZO_EINVAL : (freq ? kept_table_serves(fields, n, freq, guard) : NZO_OK);
    if (rc == NZO_OK)
        rc = compress_impl(fields, n, 7, 0, NULL, freq, guard, NULL, NZO_ELEM_F16, blob, cap, written, threads);
    free(fields);
    return rc;
}

int nzo_decompress_f16(const uint8_t *blob, uint64_t len, uint16_t *out, uint64_t n, int threads)
{
    int rc = decompress_halves(blob, len, out, n, threads, NZO_ELEM_F16);
    if (rc == NZO_OK)
        for (uint64_t i = 0; i < n; i++)
            out[i] = f16_from_fields(out[i]);
    return rc;
}
