// NeuZip codec for MI355X (gfx950): HIP kernels and the C ABI declared in
// include/neuzip.h.
//
// Stream format (little-endian):
//   container := header(64 B) | freq[256] u16 | offsets[nc+1] u32 | states[nc*16] u32
//              | lens[nc*16] u8 | words[total] u16 | signmant[ceil(n*(k+1)/8)] u8
//   every section zero-padded to 16 bytes.  A chunk is 4096 exponent symbols; local symbol i
//   belongs to rANS state j = (i mod 128) / 8, so a state codes runs of 8 neighbouring symbols.
//   Each state owns a private run of 16-bit words (lens[] words long, at most 193) stored in
//   the order the decoder consumes them; the 16 runs of a chunk follow each other and
//   offsets[c] counts the words before chunk c.
//
// Why this shape on CDNA4: one lane walks one state.  Because every state has its own word
// run, a refill is a lane-private pointer bump and a 16-bit LDS read, with no cross-lane
// ballot/prefix on the per-symbol dependency chain.  Runs of 8 symbols make each lane own 8
// neighbouring bf16 words, so the merged output leaves as one 128-bit store and the
// sign|mantissa bytes arrive as one 64-bit load; 16 lanes cover 256 contiguous output bytes.

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>

#include "neuzip.h"

namespace {

constexpr uint32_t kProbBits = NEUZIP_PROB_BITS;
constexpr uint32_t kM = 1u << kProbBits;
constexpr uint32_t kChunk = NEUZIP_CHUNK;
constexpr uint32_t kStates = NEUZIP_STATES_PER_CHUNK;
constexpr uint32_t kRun = NEUZIP_RUN;
constexpr uint32_t kTurn = kStates * kRun;          // symbols per turn of all states (128)
constexpr uint32_t kTurns = kChunk / kTurn;         // turns per full chunk (32)
constexpr uint32_t kRansL = 1u << 16;
// Words one state can emit for its 256 symbols.  Every step grows log2(x + 1) by at most 12 bits and
// every emitted word shrinks it by at least 16 - log2(17/16) bits, which bounds a run by 193 words.
constexpr uint32_t kRunCap = 200;
constexpr uint32_t kMagic = 0x315A554Eu;            // "NUZ1"
constexpr uint32_t kHeaderBytes = 64;

// Decoder launch shape: at most 512 threads = 8 waves, each wave walks 4 chunks (4 x 16 states).
constexpr uint32_t kDecThreads = 512;
constexpr uint32_t kDecChunksPerWg = kDecThreads / kStates;   // 32
// LDS: 16 KB slot table + staged word runs.  Two workgroups share a CU's 160 KB.
constexpr uint32_t kStageBytes = 62 * 1024;
// Turns (of 8 symbols per state) whose loads and stores are issued together.
#ifndef NEUZIP_TURN_GROUP
#define NEUZIP_TURN_GROUP 2
#endif
constexpr uint32_t kTurnGroup = NEUZIP_TURN_GROUP;
static_assert(kTurns % kTurnGroup == 0, "a chunk is a whole number of turn groups");

thread_local int g_last_hip_error = 0;

inline bool hip_ok(hipError_t e)
{
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return false;
    }
    return true;
}
#define NZ_HIP(call)                 \
    do {                             \
        if (!hip_ok(call))           \
            return NEUZIP_EHIP;      \
    } while (0)

inline uint64_t pad_to(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
inline bool valid_k(int k) { return k == 7 || k == 3 || k == 1 || k == 0; }
inline uint64_t signmant_bytes(uint64_t n, int k) { return (n * static_cast<uint64_t>(k + 1) + 7) / 8; }
inline uint32_t chunks_of(uint64_t n) { return static_cast<uint32_t>((n + kChunk - 1) / kChunk); }

// ------------------------------------------------------------------------------------------
// Device-side table block that sits at the start of every blob's fixed allocation.
// ------------------------------------------------------------------------------------------
struct TableBlock {
    uint16_t freq[256];    // quantised frequencies (stored in the container)
    uint16_t cum[264];     // exclusive cumulative frequencies, cum[256] = 4096 (derived)
    uint32_t counts[256];  // exponent histogram of the source tensor
    uint32_t status[4];    // [0] != 0: a decode found a malformed stream
    uint32_t lone;         // the only exponent value of the tensor (its f is 4096), else 256
    uint32_t pad[55];
    // decoder slot table (derived): lut[slot] = symbol | f << 8 | (slot - cum[symbol]) << 20
    uint32_t lut[4096];
};
static_assert(sizeof(TableBlock) % 256 == 0, "table block keeps later sections aligned");

// Per-symbol encoder constants (16 bytes, one ds_read_b128).
//   The step is x <- (x / f) * M + (x mod f) + cum = q * (M - f) + x + cum with q = floor(x / f).
//   limit: the state is renormalised before the step when x >= limit = f << 20, so q < 2^20.
//   rcp: a float slightly below 1/f, (1/f)(1 - 2^-21).  float(x) * rcp, truncated, is q or q - 1
//   (three roundings of 2^-24 cannot overcome the 2^-21 bias, and q * 1.5 * 2^-21 < 1); one
//   compare of the remainder against f settles it.  All of this runs at full VALU rate, unlike a
//   32-bit multiply-high.
struct EncSym {
    float rcp;
    uint32_t limit;
    uint32_t cmpl_cum;  // (M - f) | cum << 16
    uint32_t f;
};

// ------------------------------------------------------------------------------------------
// Compression works on a batch of up to 8 tensors that share mantissa_bits and block size (the
// weights of a layer): every kernel of the pipeline is launched once for the whole batch, so
// tensors too small to fill the chip overlap with the others.  A single tensor is a batch of one.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kBatchMax = 8;

struct CompressItem {
    const uint16_t *src;
    uint64_t n;
    TableBlock *tb;
    uint32_t *offsets;
    uint32_t *states;
    uint8_t *lens;
    uint8_t *sm;
    uint8_t *coef;
    uint16_t *words;       // known only after the stream length has been read back
    uint32_t n_chunks;
    uint32_t block;        // 0: no block-wise normalisation
    uint32_t group_base;   // first encoder group (16 chunks) of this tensor in the workspace arrays
    uint32_t hist_end;     // first workgroup after this tensor's in the histogram launch
    uint32_t enc_end;      // ... in the encode launch
    uint32_t compact_end;  // ... in the compaction launch
};

struct CompressBatch {
    CompressItem it[kBatchMax];
    uint32_t count;
    uint32_t seq;  // stamp of this call
};

// Host-visible results of one compress call (pinned host memory the kernels write directly).
struct HostRecord {
    uint32_t seq;  // stamp of the compress call whose results are complete (written last)
    uint32_t pad;
    struct Item {
        uint32_t total_words[2];
        uint32_t counts[256];
        uint16_t freq[256];
    } item[kBatchMax];
};

// ------------------------------------------------------------------------------------------
// Small helpers
// ------------------------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t *p, uint32_t value, uint32_t count)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count)
        p[i] = value;
}

__device__ inline uint32_t exponent_of(uint32_t u) { return (u >> 7) & 0xFFu; }

template <int KB>
__device__ inline uint32_t signmant_field(uint32_t u)
{
    // sign on top of the KB leading mantissa bits (Sec. 2.3 / App. D: one signed field)
    return ((u >> 15) << KB) | ((u & 0x7Fu) >> (7 - KB));
}

template <int KB>
__device__ inline void store_fields(uint8_t *sm, uint64_t vec, uint64_t packed)
{
    if constexpr (KB == 7)
        reinterpret_cast<uint2 *>(sm)[vec] = make_uint2(static_cast<uint32_t>(packed), static_cast<uint32_t>(packed >> 32));
    else if constexpr (KB == 3)
        reinterpret_cast<uint32_t *>(sm)[vec] = static_cast<uint32_t>(packed);
    else if constexpr (KB == 1)
        reinterpret_cast<uint16_t *>(sm)[vec] = static_cast<uint16_t>(packed);
    else
        sm[vec] = static_cast<uint8_t>(packed);
}

// ------------------------------------------------------------------------------------------
// Block-wise normalisation of the lossy variant (Sec. 2.3): a block of 32..512 consecutive
// weights shares one coefficient byte, the mantissa of its largest-magnitude weight; with
// c = 1 + coef/128 a weight is stored as bf16(w / c) and comes back as bf16(stored * c), so the
// largest weight is a power of two while stored and is not touched by the mantissa truncation.
// IEEE binary32 arithmetic, results rounded to the nearest-even bf16; NaNs are passed through
// with the quiet bit set, without going through the FP unit.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t bf16_round_bits(uint32_t bits32)
{
    return (bits32 + 0x7FFFu + ((bits32 >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ bool bf16_is_nan(uint32_t u) { return (u & 0x7FFFu) > 0x7F80u; }

__device__ __forceinline__ uint32_t normalise_word(uint32_t u, float c)
{
    if (bf16_is_nan(u))
        return u | 0x40u;
    return bf16_round_bits(__float_as_uint(__uint_as_float(u << 16) / c)) & 0xFFFFu;
}

__device__ __forceinline__ uint32_t denormalise_word(uint32_t u, float c)
{
    if (bf16_is_nan(u))
        return u | 0x40u;
    return bf16_round_bits(__float_as_uint(__fmul_rn(__uint_as_float(u << 16), c))) & 0xFFFFu;
}

__device__ __forceinline__ float coefficient(uint32_t coef) { return 1.0f + static_cast<float>(coef) * 0.0078125f; }

// ------------------------------------------------------------------------------------------
// Kernel 1: exponent histogram fused with the sign|mantissa split (Alg. 1 "split").
// One pass over the bf16 words: 2 B/elem read, (k+1)/8 B/elem written.  Counts go to 32
// bank-private copies of the 256 bins in LDS (copy = lane mod 32, so the 64 lanes of a wave
// hit 32 different banks whatever the symbol skew is), then one global atomic per bin.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kHistThreads = 256;
constexpr uint32_t kHistCopies = 32;

// Which tensor of the batch a workgroup of one of the wide launches works on.
struct ItemSlot {
    uint32_t item;   // index into the batch
    uint32_t wg;     // workgroup index inside the tensor's share of the launch
    uint32_t wgs;    // workgroups of that share
};

template <uint32_t CompressItem::*END>
__device__ __forceinline__ ItemSlot item_of_workgroup(const CompressBatch &b)
{
    uint32_t i = 0, first = 0;
    while (i + 1 < b.count && blockIdx.x >= b.it[i].*END) {
        first = b.it[i].*END;
        ++i;
    }
    return {i, blockIdx.x - first, b.it[i].*END - first};
}

template <int KB>
__global__ __launch_bounds__(kHistThreads) void hist_split_kernel(const CompressBatch b,
                                                                 uint32_t *__restrict__ counts_ws)
{
    const ItemSlot slot = item_of_workgroup<&CompressItem::hist_end>(b);
    const uint16_t *__restrict__ src = b.it[slot.item].src;
    const uint64_t n = b.it[slot.item].n;
    uint8_t *__restrict__ sm = b.it[slot.item].sm;
    uint32_t *__restrict__ counts = counts_ws + 256 * slot.item;
    __shared__ uint32_t bins[256 * kHistCopies];
    for (uint32_t i = threadIdx.x; i < 256 * kHistCopies; i += kHistThreads)
        bins[i] = 0;
    __syncthreads();

    const uint32_t copy = threadIdx.x & (kHistCopies - 1);
    const uint64_t n_vec = n / 8;
    const uint64_t stride = static_cast<uint64_t>(slot.wgs) * kHistThreads;
    const uint4 *src4 = reinterpret_cast<const uint4 *>(src);
    // four 128-bit loads are in flight per lane before any of them is used
    constexpr uint32_t kDepth = 4;
    for (uint64_t v0 = static_cast<uint64_t>(slot.wg) * kHistThreads + threadIdx.x; v0 < n_vec;
         v0 += stride * kDepth) {
        uint4 d[kDepth];
#pragma unroll
        for (uint32_t r = 0; r < kDepth; ++r) {
            const uint64_t v = v0 + r * stride;
            d[r] = v < n_vec ? src4[v] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (uint32_t r = 0; r < kDepth; ++r) {
            const uint64_t v = v0 + r * stride;
            if (v >= n_vec)
                break;
            const uint32_t w[4] = {d[r].x, d[r].y, d[r].z, d[r].w};
            uint64_t packed = 0;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t lo = w[p] & 0xFFFFu, hi = w[p] >> 16;
                atomicAdd(&bins[exponent_of(lo) * kHistCopies + copy], 1u);
                atomicAdd(&bins[exponent_of(hi) * kHistCopies + copy], 1u);
                packed |= static_cast<uint64_t>(signmant_field<KB>(lo)) << ((2 * p) * (KB + 1));
                packed |= static_cast<uint64_t>(signmant_field<KB>(hi)) << ((2 * p + 1) * (KB + 1));
            }
            store_fields<KB>(sm, v, packed);
        }
    }
    // ragged tail (n mod 8 elements): one thread, element by element
    if (slot.wg == 0 && threadIdx.x == 0) {
        constexpr uint32_t per_byte = 8 / (KB + 1);
        uint32_t acc = 0, filled = 0;
        for (uint64_t i = n_vec * 8; i < n; ++i) {
            const uint32_t u = src[i];
            atomicAdd(&bins[exponent_of(u) * kHistCopies + copy], 1u);
            acc |= signmant_field<KB>(u) << (filled * (KB + 1));
            if (++filled == per_byte) {
                sm[i / per_byte] = static_cast<uint8_t>(acc);
                acc = 0;
                filled = 0;
            }
        }
        if (filled)
            sm[(n - 1) / per_byte] = static_cast<uint8_t>(acc);
    }
    __syncthreads();
    // thread b sums the 32 copies of bin b, starting at a rotated copy to spread the banks
    {
        const uint32_t b = threadIdx.x;
        uint32_t sum = 0;
#pragma unroll 8
        for (uint32_t i = 0; i < kHistCopies; ++i)
            sum += bins[b * kHistCopies + ((i + b) & (kHistCopies - 1))];
        if (sum)
            atomicAdd(&counts[b], sum);
    }
}

// ------------------------------------------------------------------------------------------
// Kernel 1b: the same pass for block-wise normalised lossy compression.  A block of B weights
// is B/8 neighbouring lanes (each lane holds 8 weights), so the largest magnitude of a block is
// a shuffle reduction over 4..64 lanes; its mantissa is the block's coefficient.  The lane then
// normalises its weights and proceeds as kernel 1 on the normalised words.
// ------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(kHistThreads) void hist_split_norm_kernel(const CompressBatch b,
                                                                      uint32_t *__restrict__ counts_ws)
{
    const ItemSlot slot = item_of_workgroup<&CompressItem::hist_end>(b);
    const uint16_t *__restrict__ src = b.it[slot.item].src;
    const uint64_t n = b.it[slot.item].n;
    const uint32_t block = b.it[slot.item].block;
    uint8_t *__restrict__ coef_out = b.it[slot.item].coef;
    uint8_t *__restrict__ sm = b.it[slot.item].sm;
    uint32_t *__restrict__ counts = counts_ws + 256 * slot.item;
    __shared__ uint32_t bins[256 * kHistCopies];
    for (uint32_t i = threadIdx.x; i < 256 * kHistCopies; i += kHistThreads)
        bins[i] = 0;
    __syncthreads();

    const uint32_t copy = threadIdx.x & (kHistCopies - 1);
    const uint32_t lanes_per_block = block / 8;                 // 4 .. 64, a power of two
    const uint64_t n_vec = (n + 7) / 8;                         // the last vector may be partial
    const uint64_t stride = static_cast<uint64_t>(slot.wgs) * kHistThreads;
    constexpr uint32_t per_byte = 8 / (KB + 1);
    // the trip count is the same for all lanes of a wave, so every lane takes part in the shuffles
    const uint64_t wave_first = static_cast<uint64_t>(slot.wg) * kHistThreads + (threadIdx.x & ~63u);
    for (uint64_t base = wave_first; base < n_vec; base += stride) {
        const uint64_t v = base + (threadIdx.x & 63u);
        const uint64_t first = v * 8;
        const uint32_t valid = first >= n ? 0u : (n - first < 8 ? static_cast<uint32_t>(n - first) : 8u);
        uint32_t w[8];
        if (valid == 8) {
            const uint4 d = reinterpret_cast<const uint4 *>(src)[v];
            const uint32_t q[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                w[2 * p] = q[p] & 0xFFFFu;
                w[2 * p + 1] = q[p] >> 16;
            }
        } else {
#pragma unroll
            for (uint32_t t = 0; t < 8; ++t)
                w[t] = t < valid ? src[first + t] : 0u;
        }
        // key = magnitude | earliest position wins ties | mantissa of that weight
        uint32_t key = 0;
        const uint32_t pos0 = static_cast<uint32_t>(first % block);
#pragma unroll
        for (uint32_t t = 0; t < 8; ++t) {
            const uint32_t cand = ((w[t] & 0x7FFFu) << 16) | ((511u - (pos0 + t)) << 7) | (w[t] & 0x7Fu);
            key = (t < valid && cand > key) ? cand : key;
        }
        for (uint32_t d = 1; d < lanes_per_block; d <<= 1) {
            const uint32_t o = __shfl_xor(key, d, 64);
            key = o > key ? o : key;
        }
        const uint32_t coef = key & 0x7Fu;
        if (valid && pos0 == 0)
            coef_out[first / block] = static_cast<uint8_t>(coef);
        const float c = coefficient(coef);
        uint64_t packed = 0;
#pragma unroll
        for (uint32_t t = 0; t < 8; ++t) {
            if (t < valid) {
                const uint32_t u = normalise_word(w[t], c);
                atomicAdd(&bins[exponent_of(u) * kHistCopies + copy], 1u);
                packed |= static_cast<uint64_t>(signmant_field<KB>(u)) << (t * (KB + 1));
            }
        }
        if (valid == 8) {
            store_fields<KB>(sm, v, packed);
        } else {
            for (uint32_t t = 0; t < valid; t += per_byte)  // whole bytes; a last partial byte has zero high bits
                sm[(first + t) / per_byte] = static_cast<uint8_t>(packed >> (t * (KB + 1)));
        }
    }
    __syncthreads();
    {
        const uint32_t b = threadIdx.x;
        uint32_t sum = 0;
#pragma unroll 8
        for (uint32_t i = 0; i < kHistCopies; ++i)
            sum += bins[b * kHistCopies + ((i + b) & (kHistCopies - 1))];
        if (sum)
            atomicAdd(&counts[b], sum);
    }
}

// ------------------------------------------------------------------------------------------
// Kernel 2: counts -> frequencies that sum to 4096, cumulative table, encoder constants.
// One workgroup of 256 threads, thread s owns symbol s.  Integer only:
//   f = max(1, floor(cnt * 4096 / N)) for symbols that occur, else 0; a shortfall goes to the
//   most frequent symbol (lowest value on a tie); an excess is taken one unit at a time from
//   the symbol whose f is largest at that moment (lowest value on a tie).
// ------------------------------------------------------------------------------------------
__device__ inline uint64_t block_max_u64(uint64_t v, uint64_t *scratch)
{
    // 256 threads = 4 waves
    for (int off = 32; off > 0; off >>= 1) {
        const uint64_t o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    uint64_t r = scratch[0];
    for (int i = 1; i < 4; ++i)
        r = scratch[i] > r ? scratch[i] : r;
    return r;
}

__device__ inline uint64_t block_sum_u64(uint64_t v, uint64_t *scratch)
{
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

__global__ __launch_bounds__(256) void table_kernel(const CompressBatch b, uint32_t *__restrict__ counts_all,
                                                    EncSym *__restrict__ enc_all)
{
    // one workgroup per tensor of the batch
    uint32_t *__restrict__ counts_ws = counts_all + 256 * blockIdx.x;
    TableBlock *__restrict__ tb = b.it[blockIdx.x].tb;
    EncSym *__restrict__ enc = enc_all + 256 * blockIdx.x;
    __shared__ uint64_t scratch[4];
    __shared__ uint32_t scan[256];
    const uint32_t s = threadIdx.x;
    // the histogram was accumulated in the workspace; keep a copy in the blob and leave the
    // workspace bins at zero for the next tensor
    const uint64_t cnt = counts_ws[s];
    counts_ws[s] = 0;
    tb->counts[s] = static_cast<uint32_t>(cnt);
    if (s < 4)
        tb->status[s] = 0;
    const uint64_t total = block_sum_u64(cnt, scratch);
    uint32_t f = 0;
    if (total > 0) {
        if (cnt > 0) {
            const uint64_t scaled = cnt * kM / total;
            f = scaled < 1 ? 1u : static_cast<uint32_t>(scaled);
        }
        const int32_t sum = static_cast<int32_t>(block_sum_u64(f, scratch));
        int32_t rest = static_cast<int32_t>(kM) - sum;
        if (rest > 0) {
            const uint64_t key = (cnt << 8) | (255u - s);
            const uint64_t best = block_max_u64(key, scratch);
            if (key == best)
                f += static_cast<uint32_t>(rest);
        }
        if (rest < 0) {
            // Usual case: the most frequent symbol stays the largest through all -rest decrements
            // (its key after -rest - 1 of them still beats the runner-up's), so it takes them all.
            const uint64_t key = (static_cast<uint64_t>(f) << 8) | (255u - s);
            const uint64_t best = block_max_u64(key, scratch);
            const uint64_t second = block_max_u64(key == best ? 0 : key, scratch);
            const uint64_t best_late = best - (static_cast<uint64_t>(-rest - 1) << 8);
            if ((best >> 8) >= static_cast<uint64_t>(-rest) && best_late > second) {
                if (key == best)
                    f -= static_cast<uint32_t>(-rest);
                rest = 0;
            }
        }
        while (rest < 0) {  // general case, one unit at a time; uniform across the workgroup
            const uint64_t key = (static_cast<uint64_t>(f) << 8) | (255u - s);
            const uint64_t best = block_max_u64(key, scratch);
            if (key == best)
                --f;
            ++rest;
        }
    }
    // inclusive cumulative sum over the 256 symbols: wave scan, then the sums of the waves before
    {
        uint32_t incl = f;
#pragma unroll
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d, 64);
            if ((s & 63u) >= d)
                incl += o;
        }
        __syncthreads();
        if ((s & 63u) == 63u)
            scratch[s >> 6] = incl;
        __syncthreads();
        for (uint32_t wv = 0; wv < (s >> 6); ++wv)
            incl += static_cast<uint32_t>(scratch[wv]);
        scan[s] = incl;
    }
    __syncthreads();
    const uint32_t cum = scan[s] - f;
    tb->freq[s] = static_cast<uint16_t>(f);
    tb->cum[s] = static_cast<uint16_t>(cum);
    if (s == 255)
        tb->cum[256] = static_cast<uint16_t>(scan[255]);
    if (s == 0)
        tb->lone = 256;
    __syncthreads();
    if (f == kM)
        tb->lone = s;

    // encoder constants first: the encode kernel waits for them, the decoder table is not urgent
    EncSym e = {0.0f, 0xFFFFFFFFu, 0u, 1u};
    if (f > 0) {
        e.rcp = __fmul_rn(__fdiv_rn(1.0f, static_cast<float>(f)), 1.0f - 0x1p-21f);
        e.limit = f >= kM ? 0xFFFFFFFFu : (f << 20);  // f = 4096 only for a one-symbol tensor: never renormalises
        e.cmpl_cum = (kM - f) | (cum << 16);
        e.f = f;
    }
    enc[s] = e;

    // decoder slot table: thread s fills slots s, s + 256, ...; scan[t] = cum[t + 1].  The 16
    // binary searches of a thread are independent, so their LDS reads overlap.
    if (total > 0) {
        constexpr uint32_t kPer = kM / 256;
        uint32_t lo[kPer], hi[kPer];
#pragma unroll
        for (uint32_t r = 0; r < kPer; ++r) {
            lo[r] = 0;
            hi[r] = 255;
        }
#pragma unroll
        for (uint32_t step = 0; step < 8; ++step) {
#pragma unroll
            for (uint32_t r = 0; r < kPer; ++r) {  // smallest t with cum[t + 1] > slot
                const uint32_t mid = (lo[r] + hi[r]) >> 1;
                const bool above = scan[mid] > s + 256 * r;
                hi[r] = above ? mid : hi[r];
                lo[r] = above ? lo[r] : (mid < hi[r] ? mid + 1 : hi[r]);
            }
        }
#pragma unroll
        for (uint32_t r = 0; r < kPer; ++r) {
            const uint32_t slot = s + 256 * r, t = lo[r];
            const uint32_t begin = t ? scan[t - 1] : 0u;
            tb->lut[slot] = t | (((scan[t] - begin) & 0xFFFu) << 8) | ((slot - begin) << 20);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Kernel 3: chunked rANS encoder (Sec. 2.2 "Compression algorithm").  One lane per state.
// A state visits its symbols back to front; the words it pushes out are collected, back to
// front, in a 16-word LDS ring and leave for the state's own 200-word slot of the workspace in
// 16-byte pieces, so that the tail of the slot read forwards is the decoder's order.  Final
// states and run lengths go straight to their place in the blob; the chunk's word count goes to
// the workspace for the offsets scan.  The next turn's 8 bf16 words are requested before the
// current turn is coded.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kEncThreads = 256;
constexpr uint32_t kChunksPerGroup = kEncThreads / kStates;  // 16 chunks per encoder workgroup
constexpr uint32_t kRingWords = 16;  // per state; two halves of 8 words = 16 bytes

struct EncState {
    uint32_t x;
    uint32_t wp;          // next free position in the slot is wp - 1 (words, counts down from kRunCap)
};

__device__ __forceinline__ void rans_put(EncState &st, const EncSym e, uint16_t *__restrict__ ring)
{
    if (st.x >= e.limit) {
        --st.wp;
        ring[st.wp & (kRingWords - 1)] = static_cast<uint16_t>(st.x);
        st.x >>= 16;
    }
    uint32_t q = static_cast<uint32_t>(__fmul_rn(__uint2float_rn(st.x), e.rcp));  // q or q - 1
    const uint32_t r = st.x - __umul24(q, e.f);
    q += r >= e.f ? 1u : 0u;
    st.x = __umul24(q, e.cmpl_cum & 0xFFFFu) + st.x + (e.cmpl_cum >> 16);
}

// Moves the 8-word group completed during the last turn (at most one: a turn pushes at most 8
// words) from the ring to the slot.  Positions run down from wp_before to wp_after; group g
// (positions 8g .. 8g+7) is complete once position 8g has been written.
__device__ __forceinline__ void ring_flush(uint32_t wp_before, uint32_t wp_after, const uint16_t *__restrict__ ring,
                                           uint16_t *__restrict__ slot)
{
    const uint32_t g = (wp_after + 7) >> 3;  // lowest group whose first position is >= wp_after
    if (g * 8 < wp_before) {
        const uint4 v = *reinterpret_cast<const uint4 *>(ring + ((g * 8) & (kRingWords - 1)));
        *reinterpret_cast<uint4 *>(slot + g * 8) = v;
    }
}

template <bool NORM>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(const CompressBatch b,
                                                            const EncSym *__restrict__ enc_all,
                                                            uint32_t *__restrict__ chunk_words_all,
                                                            uint32_t *__restrict__ group_words_all,
                                                            uint16_t *__restrict__ slots_all,
                                                            HostRecord *__restrict__ record)
{
    const ItemSlot slot_id = item_of_workgroup<&CompressItem::enc_end>(b);
    const CompressItem &it = b.it[slot_id.item];
    const uint16_t *__restrict__ src = it.src;
    const uint64_t n = it.n;
    const uint8_t *__restrict__ coef = it.coef;
    const uint32_t block = NORM ? it.block : 1u;
    const uint32_t n_chunks = it.n_chunks;
    const TableBlock *__restrict__ tb = it.tb;
    uint32_t *__restrict__ states = it.states;
    uint8_t *__restrict__ lens = it.lens;
    // this tensor's part of the workspace arrays
    const uint32_t group = it.group_base + slot_id.wg;
    uint32_t *__restrict__ chunk_words = chunk_words_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup;
    uint16_t *__restrict__ slots = slots_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup * kStates * kRunCap;
    const EncSym *__restrict__ enc_g = enc_all + 256 * slot_id.item;

    __shared__ uint4 enc_raw[256];
    __shared__ __align__(16) uint16_t rings[kEncThreads * kRingWords];
    __shared__ uint32_t group_chunk[kEncThreads / kStates];
    enc_raw[threadIdx.x] = reinterpret_cast<const uint4 *>(enc_g)[threadIdx.x];
    if (slot_id.wg == 0) {
        // statistics for the host: posted early, they land long before this kernel ends
        record->item[slot_id.item].counts[threadIdx.x] = tb->counts[threadIdx.x];
        record->item[slot_id.item].freq[threadIdx.x] = tb->freq[threadIdx.x];
    }
    __syncthreads();
    const EncSym *enc = reinterpret_cast<const EncSym *>(enc_raw);

    const uint32_t lane_id = slot_id.wg * kEncThreads + threadIdx.x;  // = chunk * 16 + state
    const uint32_t c = lane_id / kStates, j = lane_id % kStates;
    const bool live = c < n_chunks;
    const uint64_t base = static_cast<uint64_t>(c) * kChunk;
    const uint32_t m = !live ? 0u : ((n - base) < kChunk ? static_cast<uint32_t>(n - base) : kChunk);
    uint16_t *slot = slots + static_cast<uint64_t>(lane_id) * kRunCap;
    uint16_t *ring = rings + threadIdx.x * kRingWords;
    EncState st = {kRansL, kRunCap};

    if (m == kChunk) {
        const uint4 *src4 = reinterpret_cast<const uint4 *>(src + base) + j;
        uint4 d = src4[(kTurns - 1) * kStates];
        for (int q = static_cast<int>(kTurns) - 1; q >= 0; --q) {
            const uint4 d_next = src4[(q > 0 ? q - 1 : 0) * kStates];
            const uint32_t w[4] = {d.x, d.y, d.z, d.w};
            const uint32_t wp_before = st.wp;
            // with block-wise normalisation the exponents coded are those of bf16(w / c)
            float c = 1.0f;
            if constexpr (NORM)
                c = coefficient(coef[(base + static_cast<uint32_t>(q) * kTurn + j * kRun) / block]);
#pragma unroll
            for (int p = 3; p >= 0; --p) {
                const uint32_t hi = NORM ? normalise_word(w[p] >> 16, c) : (w[p] >> 16);
                const uint32_t lo = NORM ? normalise_word(w[p] & 0xFFFFu, c) : (w[p] & 0xFFFFu);
                rans_put(st, enc[exponent_of(hi)], ring);
                rans_put(st, enc[exponent_of(lo)], ring);
            }
            ring_flush(wp_before, st.wp, ring, slot);
            d = d_next;
        }
    } else if (m > 0) {
        for (int q = static_cast<int>(kTurns) - 1; q >= 0; --q) {
            const uint32_t wp_before = st.wp;
            for (int t = static_cast<int>(kRun) - 1; t >= 0; --t) {
                const uint32_t i = static_cast<uint32_t>(q) * kTurn + j * kRun + static_cast<uint32_t>(t);
                if (i < m) {
                    uint32_t u = src[base + i];
                    if constexpr (NORM)
                        u = normalise_word(u, coefficient(coef[(base + i) / block]));
                    rans_put(st, enc[exponent_of(u)], ring);
                }
            }
            ring_flush(wp_before, st.wp, ring, slot);
        }
    }
    const uint32_t len = kRunCap - st.wp;
    if (live) {
        // the incomplete group at the low end: word by word
        for (uint32_t p = st.wp; p < ((st.wp + 7) & ~7u) && p < kRunCap; ++p)
            slot[p] = ring[p & (kRingWords - 1)];
        states[lane_id] = st.x;
        lens[lane_id] = static_cast<uint8_t>(len);
    }
    // words of the whole chunk (16 neighbouring lanes), then of the workgroup's 16 chunks
    uint32_t sum = len;
#pragma unroll
    for (uint32_t dlt = 1; dlt < kStates; dlt <<= 1)
        sum += __shfl_xor(sum, dlt, kStates);
    if (j == 0) {
        group_chunk[threadIdx.x / kStates] = sum;
        if (live)
            chunk_words[c] = sum;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
        for (uint32_t i = 0; i < kEncThreads / kStates; ++i)
            total += group_chunk[i];
        group_words_all[group] = total;
    }
}

// ------------------------------------------------------------------------------------------
// Kernel 4: exclusive prefix sum of the words per encoder workgroup (16 chunks each).  One
// workgroup walks the groups in tiles of 4096; the per-chunk offsets follow from these in the
// compaction kernel.  The total goes to the blob's last offset and to the host.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void offsets_kernel(const CompressBatch b,
                                                              const uint32_t *__restrict__ group_words_all,
                                                              uint64_t *__restrict__ group_prefix_all,
                                                              uint32_t *__restrict__ done,
                                                              HostRecord *__restrict__ record)
{
    // one workgroup per tensor of the batch
    const CompressItem &it = b.it[blockIdx.x];
    const uint32_t n_groups = (it.n_chunks + kChunksPerGroup - 1) / kChunksPerGroup;
    const uint32_t *__restrict__ group_words = group_words_all + it.group_base;
    uint64_t *__restrict__ group_prefix = group_prefix_all + it.group_base;
    uint32_t *__restrict__ last_offset = it.offsets + it.n_chunks;
    __shared__ uint64_t wave_sum[kScanThreads / 64];
    __shared__ uint64_t carry_s;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t carry = 0;
    for (uint32_t tile = 0; tile < n_groups; tile += kScanThreads * 4) {
        const uint32_t i0 = tile + tid * 4;
        uint32_t v[4];
#pragma unroll
        for (uint32_t r = 0; r < 4; ++r)
            v[r] = i0 + r < n_groups ? group_words[i0 + r] : 0u;
        const uint64_t mine = static_cast<uint64_t>(v[0]) + v[1] + v[2] + v[3];
        uint64_t incl = mine;  // inclusive scan over the wave
#pragma unroll
        for (uint32_t d = 1; d < 64; d <<= 1) {
            const uint64_t o = __shfl_up(incl, d, 64);
            if (lane >= d)
                incl += o;
        }
        if (lane == 63)
            wave_sum[wave] = incl;
        __syncthreads();
        uint64_t before = carry;
        for (uint32_t wv = 0; wv < wave; ++wv)
            before += wave_sum[wv];
        uint64_t run = before + incl - mine;
#pragma unroll
        for (uint32_t r = 0; r < 4; ++r) {
            if (i0 + r < n_groups)
                group_prefix[i0 + r] = run;
            run += v[r];
        }
        if (tid == kScanThreads - 1)
            carry_s = run;
        __syncthreads();
        carry = carry_s;
    }
    if (tid == 0) {
        last_offset[0] = static_cast<uint32_t>(carry);
        last_offset[1] = 0;
        record->item[blockIdx.x].total_words[0] = static_cast<uint32_t>(carry);
        record->item[blockIdx.x].total_words[1] = static_cast<uint32_t>(carry >> 32);  // non-zero: too long for 32-bit offsets
        // the workgroup that finishes last publishes the stamp and rearms the counter
        __threadfence_system();
        if (atomicAdd(done, 1u) == b.count - 1) {
            *done = 0;
            __threadfence_system();
            __hip_atomic_store(&record->seq, b.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Kernel 5: gather the runs from the workspace slots into the blob's word section and write the
// chunk offsets.  One wave per chunk; the 16 runs are read with all loads in flight, then written.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kCompactThreads = 256;

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(const CompressBatch b,
                                                                 const uint16_t *__restrict__ slots_all,
                                                                 const uint32_t *__restrict__ chunk_words_all,
                                                                 const uint64_t *__restrict__ group_prefix_all)
{
    const ItemSlot slot_id = item_of_workgroup<&CompressItem::compact_end>(b);
    const CompressItem &it = b.it[slot_id.item];
    const uint32_t n_chunks = it.n_chunks;
    const uint8_t *__restrict__ lens = it.lens;
    uint32_t *__restrict__ offsets = it.offsets;
    uint16_t *__restrict__ words = it.words;
    const uint16_t *__restrict__ slots = slots_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup * kStates * kRunCap;
    const uint32_t *__restrict__ chunk_words = chunk_words_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup;
    const uint64_t *__restrict__ group_prefix = group_prefix_all + it.group_base;

    const uint32_t c = slot_id.wg * (kCompactThreads / 64) + threadIdx.x / 64;
    const uint32_t lane = threadIdx.x & 63;
    if (c >= n_chunks)
        return;
    // run length of state (lane mod 16) and its start inside the chunk (16-lane exclusive prefix)
    const uint32_t my_len = lens[c * kStates + (lane & 15)];
    uint32_t start = my_len;
#pragma unroll
    for (uint32_t d = 1; d < kStates; d <<= 1) {
        const uint32_t o = __shfl_up(start, d, kStates);
        if ((lane & 15) >= d)
            start += o;
    }
    start -= my_len;
    uint16_t v[kStates];
    uint32_t len_j[kStates], start_j[kStates];
#pragma unroll
    for (uint32_t j = 0; j < kStates; ++j) {
        len_j[j] = __shfl(my_len, j, 64);
        start_j[j] = __shfl(start, j, 64);
        const uint16_t *from = slots + static_cast<uint64_t>(c * kStates + j) * kRunCap + (kRunCap - len_j[j]);
        v[j] = lane < len_j[j] ? from[lane] : static_cast<uint16_t>(0);
    }
    // words before this chunk: those before its encoder group plus the earlier chunks of the group
    const uint32_t g = c / kChunksPerGroup, in_group = c % kChunksPerGroup;
    uint32_t earlier = lane < in_group ? chunk_words[g * kChunksPerGroup + lane] : 0u;
#pragma unroll
    for (uint32_t d = 1; d < kChunksPerGroup; d <<= 1)
        earlier += __shfl_xor(earlier, d, kChunksPerGroup);
    const uint64_t at0 = group_prefix[g] + __shfl(earlier, 0, 64);
    if (lane == 0)
        offsets[c] = static_cast<uint32_t>(at0);
#pragma unroll
    for (uint32_t j = 0; j < kStates; ++j)
        if (lane < len_j[j])
            words[at0 + start_j[j] + lane] = v[j];
    // runs longer than a wave (more than 4 bits per symbol): the rest, run by run
    for (uint32_t j = 0; j < kStates; ++j) {
        const uint16_t *from = slots + static_cast<uint64_t>(c * kStates + j) * kRunCap + (kRunCap - len_j[j]);
        for (uint32_t i = lane + 64; i < len_j[j]; i += 64)
            words[at0 + start_j[j] + i] = from[i];
    }
}

// ------------------------------------------------------------------------------------------
// Kernel 6: fused decoder (Alg. 1 "decompression" + "merge"; Sec. 2.2 Eq. (3)).
//
// A workgroup owns blockDim.x / 16 neighbouring chunks (at most 32).  It copies the 4096-entry
// slot table (symbol | f << 8 | (slot - cum) << 20, prepared once per tensor) and the chunks'
// word runs -- one contiguous piece of the blob -- into LDS with 128-bit loads behind a single
// barrier, and then every lane walks one
// state: 32 turns of 8 symbols; per symbol one table read, one multiply-add, one compare, and
// a lane-private refill that touches LDS only when a word is consumed.  The 8 decoded
// exponents are merged with the 8 sign|mantissa fields and leave as one 128-bit store; the
// fields of the next turn are requested before the current turn is decoded.
// ------------------------------------------------------------------------------------------
template <int KB>
__device__ __forceinline__ uint64_t load_fields(const uint8_t *__restrict__ sm, uint64_t first_elem)
{
    // the (KB+1)*8 field bits of 8 neighbouring elements
    if constexpr (KB == 7) {
        const uint2 v = *reinterpret_cast<const uint2 *>(sm + first_elem);
        return static_cast<uint64_t>(v.x) | (static_cast<uint64_t>(v.y) << 32);
    } else if constexpr (KB == 3) {
        return *reinterpret_cast<const uint32_t *>(sm + first_elem / 2);
    } else if constexpr (KB == 1) {
        return *reinterpret_cast<const uint16_t *>(sm + first_elem / 4);
    } else {
        return sm[first_elem / 8];
    }
}

// Two bf16 words (sign << 15 | exponent << 7 | kept mantissa bits << (7 - KB)) from the field
// bits of a pair of neighbouring elements and the two slot-table entries that decoded them
// (exponent in the low byte of an entry).
template <int KB>
__device__ __forceinline__ uint32_t merge_pair(uint64_t fields, int pair, uint32_t entry_lo, uint32_t entry_hi)
{
    // [0, exponent_hi, 0, exponent_lo]
    const uint32_t expo = __builtin_amdgcn_perm(entry_hi, entry_lo, 0x0c040c00u);
    if constexpr (KB == 7) {
        // lossless: a field is the byte sign << 7 | mantissa.  Spread the two bytes over the two
        // halfwords ([b1, b1, b0, b0]) and keep bit 15 and bits 6..0 of each.
        const uint32_t half = static_cast<uint32_t>(fields >> (32 * (pair >> 1)));
        const uint32_t twice = __builtin_amdgcn_perm(half, half, (pair & 1) ? 0x03030202u : 0x01010000u);
        return (expo << 7) | (twice & 0x807F807Fu);
    } else if constexpr (KB == 3) {
        // byte `pair` of the 32 field bits holds two nibbles s m2 m1 m0 (low nibble = first element).
        // Nibbles into halfwords, then one multiply by 2^4 + 2^12 puts m at bits 6..4 and s at bit 15.
        const uint32_t v = static_cast<uint32_t>(fields);
        const uint32_t even = v & 0x0F0F0F0Fu, odd = (v >> 4) & 0x0F0F0F0Fu;
        const uint32_t nib = __builtin_amdgcn_perm(odd, even, 0x0c000c00u | ((4u + pair) << 16) | pair);
        return (expo << 7) | (__umul24(nib, 0x1010u) & 0x80708070u);
    } else if constexpr (KB == 1) {
        // nibble `pair` of the 16 field bits is s1 m1 s0 m0: m0 -> bit 6, s0 -> 15, m1 -> 22, s1 -> 31
        const uint32_t f2 = (static_cast<uint32_t>(fields) >> (4 * pair)) & 0xFu;
        const uint32_t spread = __umul24(f2 << 16, 0x1010u) + __umul24(f2, 0x4040u);
        return (expo << 7) | (spread & 0x80408040u);
    } else {
        // bits 2*pair and 2*pair + 1 of the 8 field bits are the two signs
        const uint32_t v = static_cast<uint32_t>(fields);
        return (expo << 7) | ((v << (15 - 2 * pair)) & 0x8000u) | ((v << (30 - 2 * pair)) & 0x80000000u);
    }
}

struct LdsWords {
    const uint8_t *base;  // LDS copy of the workgroup's runs
    __device__ __forceinline__ uint32_t peek(uint32_t at) const { return *reinterpret_cast<const uint16_t *>(base + at); }
};
struct GlobalWords {
    const uint8_t *base;  // the lane's run inside the blob
    __device__ __forceinline__ uint32_t peek(uint32_t at) const { return *reinterpret_cast<const uint16_t *>(base + at); }
};
struct NoWords {
    __device__ __forceinline__ uint32_t peek(uint32_t) const { return 0; }
};

// One rANS decoding step of a lane's state; returns the slot-table entry (symbol in its low
// byte).  `next` always holds the word at byte position wp of the lane's word source, so a
// refill is a shift-or; the following word is fetched only then.
template <class WordSrc>
__device__ __forceinline__ uint32_t rans_get(const uint32_t *__restrict__ lut, uint32_t &x, uint32_t &wp,
                                             uint32_t &next, const WordSrc &src)
{
    const uint32_t e = lut[x & (kM - 1)];
    x = __umul24((e >> 8) & 0xFFFu, x >> kProbBits) + (e >> 20);
    if (x < kRansL) {
        x = (x << 16) | next;
        wp += 2;
        next = src.peek(wp);
    }
    return e;
}

// Walks one state over its part of chunk [base, base + m) and writes the merged bf16 words.
// LONE: the tensor has a single exponent value (f = 4096): the state never moves and there are
// no words.  Returns through x / wp what the well-formedness check needs.
// Field bits of 8 neighbouring elements; with block-wise normalisation (KB < 7, so the fields
// take at most 32 bits) the block's coefficient byte rides in bits 32..39.
template <int KB, bool NORM>
__device__ __forceinline__ uint64_t load_turn(const uint8_t *__restrict__ sm, const uint8_t *__restrict__ coef,
                                              uint32_t block, uint64_t first_elem)
{
    uint64_t f = load_fields<KB>(sm, first_elem);
    if constexpr (NORM)
        f |= static_cast<uint64_t>(coef[first_elem / block]) << 32;
    return f;
}

// bf16(stored * c) on the two halves of a merged dword
__device__ __forceinline__ uint32_t denormalise_pair(uint32_t d, float c)
{
    return denormalise_word(d & 0xFFFFu, c) | (denormalise_word(d >> 16, c) << 16);
}

template <int KB, bool LONE, bool NORM, class WordSrc>
__device__ __forceinline__ void walk_state(const uint32_t *__restrict__ lut, const WordSrc &src, uint32_t lone,
                                           uint32_t &x, uint32_t &wp, const uint8_t *__restrict__ sm,
                                           const uint8_t *__restrict__ coef, uint32_t block,
                                           uint64_t (&fields)[kTurnGroup], uint16_t *__restrict__ out,
                                           uint64_t base, uint32_t m, uint32_t j)
{
    // `fields` arrives holding the field bits of the state's first kTurnGroup turns (full chunks only)
    uint32_t next = LONE ? 0u : src.peek(wp);
    if (m == kChunk) {
        uint4 *out4 = reinterpret_cast<uint4 *>(out + base) + j;
        const uint64_t first = base + j * kRun;
        // Turns are taken in groups: the field loads of the next group are issued together before
        // the current group is decoded, and the group's 128-bit stores leave back to back, so
        // each state keeps several memory requests in flight and a chunk is written in bursts of
        // kTurnGroup * 256 contiguous bytes.
        for (uint32_t q0 = 0; q0 < kTurns; q0 += kTurnGroup) {
            uint64_t fields_next[kTurnGroup];
            // the last group re-reads its own fields (stays in bounds)
            const uint32_t qn = q0 + kTurnGroup < kTurns ? q0 + kTurnGroup : q0;
#pragma unroll
            for (uint32_t r = 0; r < kTurnGroup; ++r)
                fields_next[r] = load_turn<KB, NORM>(sm, coef, block, first + (qn + r) * kTurn);
            uint4 o[kTurnGroup];
#pragma unroll
            for (uint32_t r = 0; r < kTurnGroup; ++r) {
                uint32_t e[8];
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    e[t] = LONE ? lone : rans_get(lut, x, wp, next, src);
                o[r].x = merge_pair<KB>(fields[r], 0, e[0], e[1]);
                o[r].y = merge_pair<KB>(fields[r], 1, e[2], e[3]);
                o[r].z = merge_pair<KB>(fields[r], 2, e[4], e[5]);
                o[r].w = merge_pair<KB>(fields[r], 3, e[6], e[7]);
                if constexpr (NORM) {
                    const float c = coefficient(static_cast<uint32_t>(fields[r] >> 32) & 0x7Fu);
                    o[r].x = denormalise_pair(o[r].x, c);
                    o[r].y = denormalise_pair(o[r].y, c);
                    o[r].z = denormalise_pair(o[r].z, c);
                    o[r].w = denormalise_pair(o[r].w, c);
                }
            }
#pragma unroll
            for (uint32_t r = 0; r < kTurnGroup; ++r) {
                // streamed out once: non-temporal, so the words do not displace the tables in cache
                uint4 *dst = &out4[(q0 + r) * kStates];
                __builtin_nontemporal_store(o[r].x, &dst->x);
                __builtin_nontemporal_store(o[r].y, &dst->y);
                __builtin_nontemporal_store(o[r].z, &dst->z);
                __builtin_nontemporal_store(o[r].w, &dst->w);
                fields[r] = fields_next[r];
            }
        }
    } else {
        // ragged last chunk: element by element
        constexpr uint32_t width = KB + 1, per_byte = 8 / width;
        for (uint32_t q = 0; q < kTurns; ++q) {
            for (uint32_t t = 0; t < kRun; ++t) {
                const uint32_t i = q * kTurn + j * kRun + t;
                if (i >= m)
                    continue;
                const uint32_t sym = (LONE ? lone : rans_get(lut, x, wp, next, src)) & 0xFFu;
                const uint64_t g = base + i;
                const uint32_t field = (sm[g / per_byte] >> ((g % per_byte) * width)) & ((1u << width) - 1u);
                uint32_t u = ((field >> KB) << 15) | (sym << 7) | ((field & ((1u << KB) - 1u)) << (7 - KB));
                if constexpr (NORM)
                    u = denormalise_word(u, coefficient(coef[g / block]));
                out[g] = static_cast<uint16_t>(u);
            }
        }
    }
}

// What the decoder needs to know about one tensor (all device pointers).
struct DecodeArgs {
    const TableBlock *tb;
    const uint32_t *offsets;
    const uint32_t *states;
    const uint8_t *lens;
    const uint16_t *words;
    const uint8_t *sm;
    const uint8_t *coef;  // block coefficients (block-wise normalised blobs only)
    uint16_t *out;
    uint32_t *status;
    uint64_t n;
    uint32_t n_chunks;
    uint32_t block;       // 0: no block-wise normalisation
    uint32_t wg_end;      // batches: first workgroup index after this tensor's
};

// Decodes the chunks of workgroup `wg` of one tensor.
template <int KB, bool NORM>
__device__ __forceinline__ void decode_workgroup(const TableBlock *__restrict__ tb,
                                                 const uint32_t *__restrict__ offsets,
                                                 const uint32_t *__restrict__ states,
                                                 const uint8_t *__restrict__ lens,
                                                 const uint16_t *__restrict__ words,
                                                 const uint8_t *__restrict__ sm,
                                                 const uint8_t *__restrict__ coef, uint32_t block,
                                                 uint16_t *__restrict__ out,
                                                 uint64_t n, uint32_t n_chunks, uint32_t *__restrict__ status,
                                                 uint32_t wg, uint32_t *__restrict__ lut, uint8_t *__restrict__ stage)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t threads = blockDim.x;            // a multiple of 64, at most kDecThreads
    const uint32_t chunks_per_wg = threads / kStates;
    const uint32_t c0 = wg * chunks_per_wg;
    const uint32_t c1 = c0 + chunks_per_wg < n_chunks ? c0 + chunks_per_wg : n_chunks;
    const uint32_t c = c0 + tid / kStates;
    const uint32_t j = tid % kStates;
    const bool live = c < n_chunks;
    const uint32_t id = c * kStates + j;
    const uint64_t base = static_cast<uint64_t>(c) * kChunk;
    const uint32_t m = !live ? 0u : ((n - base) < kChunk ? static_cast<uint32_t>(n - base) : kChunk);

    // ---- every load that depends on nothing is issued first, so their latencies overlap
    const uint32_t off0 = offsets[c0];
    const uint32_t off1 = offsets[c1];
    const uint32_t off_c = live ? offsets[c] : 0u;
    uint32_t x = live ? states[id] : kRansL;
    const uint32_t len = live ? lens[id] : 0u;
    const uint32_t lone = tb->lone;
    uint64_t fields0[kTurnGroup];
#pragma unroll
    for (uint32_t r = 0; r < kTurnGroup; ++r)
        fields0[r] = m == kChunk ? load_turn<KB, NORM>(sm, coef, block, base + r * kTurn + j * kRun) : 0;
    const uint4 *lut_g = reinterpret_cast<const uint4 *>(tb->lut);
    uint4 lut_piece[2];  // 16 KB table / 16 B = 1024 pieces; 2 per thread at 512 threads
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r) {
        const uint32_t i = tid + r * threads;
        lut_piece[r] = i < kM / 4 ? lut_g[i] : make_uint4(0, 0, 0, 0);
    }

    // ---- stage the word runs of chunks [c0, c1): one contiguous piece of the blob
    const uint64_t byte0 = static_cast<uint64_t>(off0) * 2;
    const uint64_t byte1 = static_cast<uint64_t>(off1) * 2;
    const uint64_t aligned0 = byte0 & ~static_cast<uint64_t>(15);
    const uint64_t stage_len = byte1 - aligned0;
    const bool staged = stage_len + 16 <= kStageBytes;  // room for the one-word look-ahead
    if (staged) {
        const uint4 *from = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(words) + aligned0);
        uint4 *to = reinterpret_cast<uint4 *>(stage);
        for (uint32_t i = tid; i * 16 < stage_len; i += threads)
            to[i] = from[i];
    }
    // ---- slot table into LDS (small workgroups loop over the remaining pieces)
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r) {
        const uint32_t i = tid + r * threads;
        if (i < kM / 4)
            reinterpret_cast<uint4 *>(lut)[i] = lut_piece[r];
    }
    for (uint32_t i = tid + 2 * threads; i < kM / 4; i += threads)
        reinterpret_cast<uint4 *>(lut)[i] = lut_g[i];
    __syncthreads();

    // ---- one lane, one state
    if (!live)
        return;
    // start of this state's run: chunk offset + lengths of the states before it (16-lane prefix)
    uint32_t before = len;
#pragma unroll
    for (uint32_t d = 1; d < kStates; d <<= 1) {
        const uint32_t o = __shfl_up(before, d, kStates);
        if (j >= d)
            before += o;
    }
    before -= len;
    const uint64_t run_byte = (static_cast<uint64_t>(off_c) + before) * 2;

    uint32_t wp = 0, wp_begin = 0;
    if (lone < 256) {
        walk_state<KB, true, NORM>(lut, NoWords{}, lone, x, wp, sm, coef, block, fields0, out, base, m, j);
    } else if (staged) {
        wp = wp_begin = static_cast<uint32_t>(run_byte - aligned0);
        walk_state<KB, false, NORM>(lut, LdsWords{stage}, 0u, x, wp, sm, coef, block, fields0, out, base, m, j);
    } else {
        // the runs of this workgroup's chunks did not fit the LDS window (more than ~4 bits per
        // symbol): read the words straight from the blob
        walk_state<KB, false, NORM>(lut, GlobalWords{reinterpret_cast<const uint8_t *>(words) + run_byte}, 0u, x, wp,
                                    sm, coef, block, fields0, out, base, m, j);
    }
    // a well-formed run is consumed exactly and leaves the state where the encoder started
    if (x != kRansL || wp - wp_begin != 2 * len)
        atomicOr(status, 1u);
}

template <int KB, bool NORM>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(const DecodeArgs a)
{
    __shared__ __align__(16) uint32_t lut[kM];
    __shared__ __align__(16) uint8_t stage[kStageBytes];
    decode_workgroup<KB, NORM>(a.tb, a.offsets, a.states, a.lens, a.words, a.sm, a.coef, a.block, a.out, a.n,
                               a.n_chunks, a.status, blockIdx.x, lut, stage);
}

// Several tensors in one launch (a layer's weights): workgroups [t[i-1].wg_end, t[i].wg_end)
// belong to tensor i.  Small tensors, which alone cannot fill the chip, overlap with the others.
struct BatchArgs {
    DecodeArgs t[kBatchMax];
    uint32_t count;
};

template <int KB, bool NORM>
__global__ __launch_bounds__(kDecThreads) void decode_batch_kernel(const BatchArgs b)
{
    __shared__ __align__(16) uint32_t lut[kM];
    __shared__ __align__(16) uint8_t stage[kStageBytes];
    uint32_t i = 0, first = 0;
    while (i + 1 < b.count && blockIdx.x >= b.t[i].wg_end) {
        first = b.t[i].wg_end;
        ++i;
    }
    const DecodeArgs &a = b.t[i];
    decode_workgroup<KB, NORM>(a.tb, a.offsets, a.states, a.lens, a.words, a.sm, a.coef, a.block, a.out, a.n,
                               a.n_chunks, a.status, blockIdx.x - first, lut, stage);
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
inline bool valid_block(uint32_t b) { return b == 32 || b == 64 || b == 128 || b == 256 || b == 512; }
inline uint64_t block_count(uint64_t n, uint32_t block) { return block ? (n + block - 1) / block : 0; }

struct Layout {
    uint64_t offsets, states, lens, sm, coef, total;  // byte positions inside the fixed allocation
};

Layout fixed_layout(uint64_t n, int k, uint32_t block)
{
    const uint64_t nc = chunks_of(n);
    Layout l;
    l.offsets = sizeof(TableBlock);
    l.states = l.offsets + pad_to((nc + 2) * 4, 256);
    l.lens = l.states + pad_to(nc * kStates * 4, 256);
    l.sm = l.lens + pad_to(nc * kStates, 256);
    l.coef = l.sm + pad_to(signmant_bytes(n, k), 256) + 256;
    l.total = l.coef + pad_to(block_count(n, block), 256);
    return l;
}

struct Container {
    uint64_t freq, offsets, states, lens, words, sm, coef, total;  // byte positions in the flat container
};

Container container_layout(uint64_t n, int k, uint64_t total_words, uint32_t block)
{
    const uint64_t nc = chunks_of(n);
    Container c;
    c.freq = kHeaderBytes;
    c.offsets = c.freq + 512;
    c.states = c.offsets + pad_to((nc + 1) * 4, 16);
    c.lens = c.states + nc * kStates * 4;
    c.words = c.lens + nc * kStates;
    c.sm = c.words + pad_to(total_words * 2, 16);
    c.coef = c.sm + pad_to(signmant_bytes(n, k), 16);
    c.total = c.coef + pad_to(block_count(n, block), 16);
    return c;
}

}  // namespace

struct neuzip_blob {
    uint32_t magic;
    int device;
    uint64_t n;
    int k;
    uint32_t block;  // block size of the block-wise normalisation, 0 = none
    uint32_t n_chunks;
    uint64_t total_words;
    uint8_t *fixed;
    uint64_t fixed_bytes;
    uint8_t *words;
    uint64_t words_bytes;  // capacity of the word allocation
    Layout at;
    bool have_counts;
    uint32_t h_counts[256];
    uint16_t h_freq[256];
};

namespace {

constexpr uint32_t kBlobMagic = 0x424C5A4Eu;

inline TableBlock *table_of(const neuzip_blob *b) { return reinterpret_cast<TableBlock *>(b->fixed); }
inline uint32_t *offsets_of(const neuzip_blob *b) { return reinterpret_cast<uint32_t *>(b->fixed + b->at.offsets); }
inline uint32_t *states_of(const neuzip_blob *b) { return reinterpret_cast<uint32_t *>(b->fixed + b->at.states); }
inline uint8_t *lens_of(const neuzip_blob *b) { return b->fixed + b->at.lens; }
inline uint8_t *sm_of(const neuzip_blob *b) { return b->fixed + b->at.sm; }
inline uint8_t *coef_of(const neuzip_blob *b) { return b->fixed + b->at.coef; }
inline bool is_blob(const neuzip_blob *b) { return b && b->magic == kBlobMagic; }

// Per-process compress workspace: histogram bins and encoder constants for the tensors of a batch,
// per-chunk / per-group word counts, run slots, and pinned host memory for the results.
struct Workspace {
    int device = -1;
    EncSym *enc = nullptr;            // kBatchMax x 256
    uint32_t *counts = nullptr;       // kBatchMax x 256 histogram bins, zero between compress calls
    uint32_t *done = nullptr;         // offsets-kernel workgroups that have finished (rearmed by the last)
    uint32_t *chunk_words = nullptr;  // words per chunk
    uint32_t *group_words = nullptr;  // words per encoder workgroup (16 chunks), input of the scan
    uint64_t *group_prefix = nullptr; // its exclusive prefix sum, per tensor
    uint64_t group_cap = 0;           // encoder groups the arrays and the slots are sized for
    uint16_t *slots = nullptr;
    HostRecord *pinned = nullptr;     // pinned host memory, written by the encode and offsets kernels
    uint32_t seq = 0;                 // stamp of the last compress call
    hipEvent_t idle = nullptr;        // recorded after the last kernel that uses the workspace
};
std::mutex g_ws_mutex;
Workspace g_ws;

int release_workspace_locked()
{
    int rc = NEUZIP_OK;
    if (g_ws.device >= 0) {
        int cur = 0;
        if (!hip_ok(hipGetDevice(&cur)))
            return NEUZIP_EHIP;
        if (!hip_ok(hipSetDevice(g_ws.device)))
            return NEUZIP_EHIP;
        if (g_ws.idle) {
            if (!hip_ok(hipEventSynchronize(g_ws.idle)))
                rc = NEUZIP_EHIP;
            (void)hipEventDestroy(g_ws.idle);
        }
        void *device_arrays[] = {g_ws.enc, g_ws.counts, g_ws.chunk_words, g_ws.group_words, g_ws.group_prefix,
                                 g_ws.slots};  // `done` lives inside the counts allocation
        for (void *ptr : device_arrays)
            if (ptr)
                (void)hipFree(ptr);
        if (g_ws.pinned)
            (void)hipHostFree(g_ws.pinned);
        (void)hipSetDevice(cur);
    }
    g_ws = Workspace();
    return rc;
}

// Waits until the offsets kernel of call `seq` has published its record.  The stamp arrives a
// few microseconds after the kernel's last store, well before a blocking stream synchronise would
// wake up; after a bounded spin the stream is synchronised anyway, which also surfaces errors.
bool wait_for_record(uint32_t seq, hipStream_t stream)
{
    const volatile uint32_t *stamp = &g_ws.pinned->seq;
    const auto start = std::chrono::steady_clock::now();
    for (uint32_t spins = 0;; ++spins) {
        if (__atomic_load_n(stamp, __ATOMIC_ACQUIRE) == seq)
            return true;
        if ((spins & 1023u) == 1023u &&
            std::chrono::steady_clock::now() - start > std::chrono::milliseconds(20))
            break;
    }
    if (!hip_ok(hipStreamSynchronize(stream)))
        return false;
    return __atomic_load_n(stamp, __ATOMIC_ACQUIRE) == seq;
}

int ensure_workspace(int device, uint64_t n_groups, hipStream_t stream)
{
    if (g_ws.device != device) {
        const int rc = release_workspace_locked();
        if (rc != NEUZIP_OK)
            return rc;
        g_ws.device = device;
        NZ_HIP(hipMalloc(reinterpret_cast<void **>(&g_ws.enc), kBatchMax * 256 * sizeof(EncSym)));
        NZ_HIP(hipMalloc(reinterpret_cast<void **>(&g_ws.counts), (kBatchMax * 256 + 64) * sizeof(uint32_t)));
        g_ws.done = g_ws.counts + kBatchMax * 256;  // shares the allocation; cleared with the bins below
        NZ_HIP(hipHostMalloc(reinterpret_cast<void **>(&g_ws.pinned), sizeof(HostRecord), hipHostMallocDefault));
        std::memset(g_ws.pinned, 0, sizeof(HostRecord));
        g_ws.seq = 0;
        NZ_HIP(hipEventCreateWithFlags(&g_ws.idle, hipEventDisableTiming));
        hipLaunchKernelGGL(fill_u32_kernel, dim3(kBatchMax + 1), dim3(256), 0, stream, g_ws.counts, 0u,
                           kBatchMax * 256 + 64);
        NZ_HIP(hipGetLastError());
        NZ_HIP(hipEventRecord(g_ws.idle, stream));
    }
    // the previous user of the workspace may still be running on another stream
    NZ_HIP(hipStreamWaitEvent(stream, g_ws.idle, 0));
    if (g_ws.group_cap < n_groups) {
        NZ_HIP(hipEventSynchronize(g_ws.idle));
        void *old_arrays[] = {g_ws.chunk_words, g_ws.group_words, g_ws.group_prefix, g_ws.slots};
        for (void *ptr : old_arrays)
            if (ptr)
                NZ_HIP(hipFree(ptr));
        g_ws.chunk_words = g_ws.group_words = nullptr;
        g_ws.group_prefix = nullptr;
        g_ws.slots = nullptr;
        g_ws.group_cap = 0;
        const uint64_t chunks = n_groups * kChunksPerGroup;
        if (hipMalloc(reinterpret_cast<void **>(&g_ws.chunk_words), (chunks + 4) * 4) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&g_ws.group_words), (n_groups + 4) * 4) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&g_ws.group_prefix), (n_groups + 4) * 8) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&g_ws.slots), chunks * kStates * kRunCap * 2) != hipSuccess) {
            (void)hipGetLastError();
            return NEUZIP_ENOMEM;
        }
        g_ws.group_cap = n_groups;
    }
    return NEUZIP_OK;
}

int alloc_blob(uint64_t n, int k, uint32_t block, neuzip_blob **out)
{
    neuzip_blob *b = new (std::nothrow) neuzip_blob();
    if (!b)
        return NEUZIP_ENOMEM;
    std::memset(b, 0, sizeof(*b));
    b->magic = kBlobMagic;
    b->n = n;
    b->k = k;
    b->block = block;
    b->n_chunks = chunks_of(n);
    b->at = fixed_layout(n, k, block);
    if (!hip_ok(hipGetDevice(&b->device))) {
        delete b;
        return NEUZIP_EHIP;
    }
    if (hipMalloc(reinterpret_cast<void **>(&b->fixed), b->at.total) != hipSuccess) {
        (void)hipGetLastError();
        delete b;
        return NEUZIP_ENOMEM;
    }
    b->fixed_bytes = b->at.total;
    *out = b;
    return NEUZIP_OK;
}

int reserve_words(neuzip_blob *b, uint64_t total_words)
{
    // slack behind the last word: the decoder copies whole 16-byte pieces, looks one word ahead,
    // and a state fed a damaged stream may walk up to 256 words past the start of its run
    const uint64_t need = pad_to(total_words * 2, 256) + 1024;
    if (b->words_bytes < need) {
        if (b->words) {
            NZ_HIP(hipFree(b->words));
            b->words = nullptr;
            b->words_bytes = 0;
        }
        if (hipMalloc(reinterpret_cast<void **>(&b->words), need) != hipSuccess) {
            (void)hipGetLastError();
            return NEUZIP_ENOMEM;
        }
        b->words_bytes = need;
    }
    return NEUZIP_OK;
}

// Chunks per decoder workgroup.  32 (8 waves) measured best at every size: two such workgroups
// fill a CU's LDS with 16 waves, and smaller workgroups lower that occupancy.
// NEUZIP_DECODE_CHUNKS_PER_WG (4..32, multiple of 4) overrides the choice for tuning runs.
uint32_t decode_chunks_per_wg()
{
    static int forced = -1;
    if (forced < 0) {
        const char *env = std::getenv("NEUZIP_DECODE_CHUNKS_PER_WG");
        const int v = env ? std::atoi(env) : 0;
        forced = (v >= 4 && v <= static_cast<int>(kDecChunksPerWg) && v % 4 == 0) ? v : 0;
    }
    return forced > 0 ? static_cast<uint32_t>(forced) : kDecChunksPerWg;
}

DecodeArgs decode_args(const neuzip_blob *b, void *d_dst)
{
    DecodeArgs a;
    a.tb = table_of(b);
    a.offsets = offsets_of(b);
    a.states = states_of(b);
    a.lens = lens_of(b);
    a.words = reinterpret_cast<const uint16_t *>(b->words);
    a.sm = sm_of(b);
    a.coef = coef_of(b);
    a.block = b->block;
    a.out = static_cast<uint16_t *>(d_dst);
    a.status = table_of(b)->status;
    a.n = b->n;
    a.n_chunks = b->n_chunks;
    a.wg_end = 0;
    return a;
}

template <int KB, bool NORM>
int launch_decode(const neuzip_blob *b, void *d_dst, hipStream_t stream)
{
    const uint32_t per = decode_chunks_per_wg();
    const uint32_t groups = (b->n_chunks + per - 1) / per;
    hipLaunchKernelGGL((decode_kernel<KB, NORM>), dim3(groups), dim3(per * kStates), 0, stream,
                       decode_args(b, d_dst));
    return hip_ok(hipGetLastError()) ? NEUZIP_OK : NEUZIP_EHIP;
}

int decode_dispatch(const neuzip_blob *b, void *d_dst, hipStream_t stream)
{
    if (b->n == 0)
        return NEUZIP_OK;
    if (b->block) {
        switch (b->k) {
        case 3: return launch_decode<3, true>(b, d_dst, stream);
        case 1: return launch_decode<1, true>(b, d_dst, stream);
        default: return launch_decode<0, true>(b, d_dst, stream);
        }
    }
    switch (b->k) {
    case 7: return launch_decode<7, false>(b, d_dst, stream);
    case 3: return launch_decode<3, false>(b, d_dst, stream);
    case 1: return launch_decode<1, false>(b, d_dst, stream);
    default: return launch_decode<0, false>(b, d_dst, stream);
    }
}

// variant = mantissa_bits, + 8 for block-wise normalised blobs
inline int decode_variant(const neuzip_blob *b) { return b->k + (b->block ? 8 : 0); }

int launch_batch(const BatchArgs &args, int variant, uint32_t groups, hipStream_t stream)
{
    const dim3 grid(groups), block(kDecThreads);
    switch (variant) {
    case 7: hipLaunchKernelGGL((decode_batch_kernel<7, false>), grid, block, 0, stream, args); break;
    case 3: hipLaunchKernelGGL((decode_batch_kernel<3, false>), grid, block, 0, stream, args); break;
    case 1: hipLaunchKernelGGL((decode_batch_kernel<1, false>), grid, block, 0, stream, args); break;
    case 0: hipLaunchKernelGGL((decode_batch_kernel<0, false>), grid, block, 0, stream, args); break;
    case 11: hipLaunchKernelGGL((decode_batch_kernel<3, true>), grid, block, 0, stream, args); break;
    case 9: hipLaunchKernelGGL((decode_batch_kernel<1, true>), grid, block, 0, stream, args); break;
    default: hipLaunchKernelGGL((decode_batch_kernel<0, true>), grid, block, 0, stream, args); break;
    }
    return hip_ok(hipGetLastError()) ? NEUZIP_OK : NEUZIP_EHIP;
}

// An empty tensor: a zeroed table block (a fill kernel, not a memset node, so the call stays safe
// to record into a graph) and a single zero offset.
int compress_empty(neuzip_blob *b, hipStream_t stream)
{
    hipLaunchKernelGGL(fill_u32_kernel, dim3((sizeof(TableBlock) / 4 + 255) / 256), dim3(256), 0, stream,
                       reinterpret_cast<uint32_t *>(b->fixed), 0u, static_cast<uint32_t>(sizeof(TableBlock) / 4));
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, stream, offsets_of(b), 0u, 2u);
    if (!hip_ok(hipGetLastError()) || !hip_ok(hipStreamSynchronize(stream)))
        return NEUZIP_EHIP;
    std::memset(b->h_counts, 0, sizeof(b->h_counts));
    std::memset(b->h_freq, 0, sizeof(b->h_freq));
    b->have_counts = true;
    b->total_words = 0;
    return NEUZIP_OK;
}

template <int KB>
void launch_hist(const CompressBatch &batch, bool norm, uint32_t groups, hipStream_t stream)
{
    if (norm)
        hipLaunchKernelGGL(hist_split_norm_kernel<KB>, dim3(groups), dim3(kHistThreads), 0, stream, batch,
                           g_ws.counts);
    else
        hipLaunchKernelGGL(hist_split_kernel<KB>, dim3(groups), dim3(kHistThreads), 0, stream, batch, g_ws.counts);
}

// Compresses up to kBatchMax tensors (arguments already validated) with one pass of the pipeline.
int compress_some(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int k, uint32_t block,
                  hipStream_t stream, neuzip_blob **blobs)
{
    neuzip_blob *work[kBatchMax];
    bool fresh[kBatchMax];
    for (uint32_t i = 0; i < count; ++i) {
        work[i] = blobs[i];
        fresh[i] = false;
    }
    bool bins_dirty = false;  // the histogram kernel ran but the table kernel did not clear the bins
    auto fail = [&](int rc) {
        if (bins_dirty && g_ws.counts)
            hipLaunchKernelGGL(fill_u32_kernel, dim3(kBatchMax), dim3(256), 0, stream, g_ws.counts, 0u,
                               kBatchMax * 256);
        for (uint32_t i = 0; i < count; ++i)
            if (fresh[i])
                neuzip_free(work[i]);
        return rc;
    };
    for (uint32_t i = 0; i < count; ++i) {
        if (!work[i]) {
            const int rc = alloc_blob(n_elems[i], k, block, &work[i]);
            if (rc != NEUZIP_OK)
                return fail(rc);
            fresh[i] = true;
        }
        work[i]->have_counts = false;
        work[i]->total_words = 0;
    }

    // the batch proper: tensors that have elements
    CompressBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    uint32_t owner[kBatchMax];
    uint32_t hist_groups = 0, enc_groups = 0, compact_groups = 0;
    for (uint32_t i = 0; i < count; ++i) {
        neuzip_blob *b = work[i];
        if (b->n == 0) {
            const int rc = compress_empty(b, stream);
            if (rc != NEUZIP_OK)
                return fail(rc);
            continue;
        }
        CompressItem &it = batch.it[batch.count];
        owner[batch.count++] = i;
        it.src = static_cast<const uint16_t *>(d_srcs[i]);
        it.n = b->n;
        it.tb = table_of(b);
        it.offsets = offsets_of(b);
        it.states = states_of(b);
        it.lens = lens_of(b);
        it.sm = sm_of(b);
        it.coef = coef_of(b);
        it.words = nullptr;
        it.n_chunks = b->n_chunks;
        it.block = block;
        it.group_base = enc_groups;
        // every workgroup of the histogram pass pays for clearing and merging its 32 KB of bins: give
        // it at least 8 vectors (64 elements) per thread, and no tensor more workgroups than fit the chip
        uint64_t hg = ((b->n + 7) / 8 + kHistThreads * 8 - 1) / (kHistThreads * 8);
        hg = hg < 1 ? 1 : (hg > 1280 ? 1280 : hg);
        hist_groups += static_cast<uint32_t>(hg);
        enc_groups += (b->n_chunks + kChunksPerGroup - 1) / kChunksPerGroup;
        compact_groups += (b->n_chunks + kCompactThreads / 64 - 1) / (kCompactThreads / 64);
        it.hist_end = hist_groups;
        it.enc_end = enc_groups;
        it.compact_end = compact_groups;
    }
    if (batch.count > 0) {
        std::lock_guard<std::mutex> guard(g_ws_mutex);
        int rc = ensure_workspace(work[owner[0]]->device, enc_groups, stream);
        if (rc != NEUZIP_OK)
            return fail(rc);
        batch.seq = ++g_ws.seq;

        switch (k) {
        case 7: launch_hist<7>(batch, block != 0, hist_groups, stream); break;
        case 3: launch_hist<3>(batch, block != 0, hist_groups, stream); break;
        case 1: launch_hist<1>(batch, block != 0, hist_groups, stream); break;
        default: launch_hist<0>(batch, block != 0, hist_groups, stream); break;
        }
        if (!hip_ok(hipGetLastError()))
            return fail(NEUZIP_EHIP);
        bins_dirty = true;
        // the table kernel also returns the workspace histogram bins to zero
        hipLaunchKernelGGL(table_kernel, dim3(batch.count), dim3(256), 0, stream, batch, g_ws.counts, g_ws.enc);
        if (hip_ok(hipGetLastError()))
            bins_dirty = false;
        if (block)
            hipLaunchKernelGGL(encode_kernel<true>, dim3(enc_groups), dim3(kEncThreads), 0, stream, batch, g_ws.enc,
                               g_ws.chunk_words, g_ws.group_words, g_ws.slots, g_ws.pinned);
        else
            hipLaunchKernelGGL(encode_kernel<false>, dim3(enc_groups), dim3(kEncThreads), 0, stream, batch, g_ws.enc,
                               g_ws.chunk_words, g_ws.group_words, g_ws.slots, g_ws.pinned);
        hipLaunchKernelGGL(offsets_kernel, dim3(batch.count), dim3(kScanThreads), 0, stream, batch, g_ws.group_words,
                           g_ws.group_prefix, g_ws.done, g_ws.pinned);
        if (!hip_ok(hipGetLastError()))
            return fail(NEUZIP_EHIP);

        // the stream lengths are data dependent: wait for them (and the statistics), which the
        // kernels write straight into pinned host memory, the stamp last
        if (!wait_for_record(batch.seq, stream))
            return fail(NEUZIP_EHIP);
        for (uint32_t j = 0; j < batch.count; ++j) {
            const HostRecord::Item &r = g_ws.pinned->item[j];
            neuzip_blob *b = work[owner[j]];
            if (r.total_words[1] != 0)
                return fail(NEUZIP_EUNSUPPORTED);  // more than 2^32 words
            rc = reserve_words(b, r.total_words[0]);
            if (rc != NEUZIP_OK)
                return fail(rc);
            b->total_words = r.total_words[0];
            std::memcpy(b->h_counts, r.counts, 1024);
            std::memcpy(b->h_freq, r.freq, 512);
            b->have_counts = true;
            batch.it[j].words = reinterpret_cast<uint16_t *>(b->words);
        }
        hipLaunchKernelGGL(compact_kernel, dim3(compact_groups), dim3(kCompactThreads), 0, stream, batch, g_ws.slots,
                           g_ws.chunk_words, g_ws.group_prefix);
        if (!hip_ok(hipGetLastError()) || !hip_ok(hipEventRecord(g_ws.idle, stream)))
            return fail(NEUZIP_EHIP);
    }
    for (uint32_t i = 0; i < count; ++i)
        blobs[i] = work[i];
    return NEUZIP_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------
extern "C" {

int neuzip_compress(const void *d_src, uint64_t n_elems, int dtype, int mantissa_bits, void *hip_stream,
                    neuzip_blob **blob)
{
    return neuzip_compress_batch(&d_src, &n_elems, 1, dtype, mantissa_bits, 0, hip_stream, blob);
}

int neuzip_compress_blockwise(const void *d_src, uint64_t n_elems, int dtype, int mantissa_bits,
                              uint32_t block_size, void *hip_stream, neuzip_blob **blob)
{
    return neuzip_compress_batch(&d_src, &n_elems, 1, dtype, mantissa_bits, block_size, hip_stream, blob);
}

int neuzip_compress_batch(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int dtype,
                          int mantissa_bits, uint32_t block_size, void *hip_stream, neuzip_blob **blobs)
{
    if (count == 0)
        return NEUZIP_OK;
    if (!d_srcs || !n_elems || !blobs || dtype != NEUZIP_BF16 || !valid_k(mantissa_bits))
        return NEUZIP_EINVAL;
    if (block_size != 0 && (!valid_block(block_size) || mantissa_bits == 7))
        return NEUZIP_EINVAL;
    for (uint32_t i = 0; i < count; ++i) {
        if (n_elems[i] > 0 && (!d_srcs[i] || (reinterpret_cast<uintptr_t>(d_srcs[i]) & 15u)))
            return NEUZIP_EINVAL;
        if (n_elems[i] >= (1ull << 32))
            return NEUZIP_EUNSUPPORTED;
        const neuzip_blob *b = blobs[i];
        if (b && (!is_blob(b) || b->n != n_elems[i] || b->k != mantissa_bits || b->block != block_size))
            return NEUZIP_EINVAL;
        for (uint32_t j = 0; j < i; ++j)
            if (b && blobs[j] == b)
                return NEUZIP_EINVAL;  // one blob cannot receive two tensors
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (uint32_t first = 0; first < count; first += kBatchMax) {
        const uint32_t m = count - first < kBatchMax ? count - first : kBatchMax;
        const int rc = compress_some(d_srcs + first, n_elems + first, m, mantissa_bits, block_size, stream,
                                     blobs + first);
        if (rc != NEUZIP_OK)
            return rc;
    }
    return NEUZIP_OK;
}

int neuzip_decompress(const neuzip_blob *blob, void *d_dst, uint64_t n_elems, int dtype, void *hip_stream)
{
    if (!is_blob(blob) || dtype != NEUZIP_BF16 || blob->n != n_elems)
        return NEUZIP_EINVAL;
    if (n_elems > 0 && (!d_dst || (reinterpret_cast<uintptr_t>(d_dst) & 15u)))
        return NEUZIP_EINVAL;
    return decode_dispatch(blob, d_dst, static_cast<hipStream_t>(hip_stream));
}

int neuzip_decompress_sequence(const neuzip_blob *const *blobs, uint32_t count, void *d_scratch,
                               uint64_t scratch_elems, void *hip_stream)
{
    if (count > 0 && !blobs)
        return NEUZIP_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_scratch) & 15u)
        return NEUZIP_EINVAL;
    for (uint32_t i = 0; i < count; ++i) {
        if (!is_blob(blobs[i]) || blobs[i]->n > scratch_elems || (blobs[i]->n > 0 && !d_scratch))
            return NEUZIP_EINVAL;
    }
    for (uint32_t i = 0; i < count; ++i) {
        const int rc = decode_dispatch(blobs[i], d_scratch, static_cast<hipStream_t>(hip_stream));
        if (rc != NEUZIP_OK)
            return rc;
    }
    return NEUZIP_OK;
}

int neuzip_decompress_batch(const neuzip_blob *const *blobs, void *const *d_dsts, uint32_t count, void *hip_stream)
{
    if (count > 0 && (!blobs || !d_dsts))
        return NEUZIP_EINVAL;
    for (uint32_t i = 0; i < count; ++i) {
        if (!is_blob(blobs[i]))
            return NEUZIP_EINVAL;
        if (blobs[i]->n > 0 && (!d_dsts[i] || (reinterpret_cast<uintptr_t>(d_dsts[i]) & 15u)))
            return NEUZIP_EINVAL;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // tensors of the same kind (mantissa_bits, normalised or not) share launches of up to
    // kBatchMax tensors, in the given order
    static const int kinds[7] = {7, 3, 1, 0, 11, 9, 8};
    for (int k : kinds) {
        BatchArgs args;
        args.count = 0;
        uint32_t groups = 0;
        for (uint32_t i = 0; i <= count; ++i) {
            const bool flush = (i == count) || (args.count == kBatchMax);
            if (flush && args.count > 0) {
                const int rc = launch_batch(args, k, groups, stream);
                if (rc != NEUZIP_OK)
                    return rc;
                args.count = 0;
                groups = 0;
            }
            if (i == count)
                break;
            const neuzip_blob *b = blobs[i];
            if (decode_variant(b) != k || b->n == 0)
                continue;
            DecodeArgs a = decode_args(b, d_dsts[i]);
            groups += (b->n_chunks + kDecChunksPerWg - 1) / kDecChunksPerWg;
            a.wg_end = groups;
            args.t[args.count++] = a;
        }
    }
    return NEUZIP_OK;
}

void neuzip_free(neuzip_blob *blob)
{
    if (!is_blob(blob))
        return;
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    if (have_cur && cur != blob->device)
        hipSetDevice(blob->device);
    if (blob->fixed)
        hipFree(blob->fixed);
    if (blob->words)
        hipFree(blob->words);
    if (have_cur && cur != blob->device)
        hipSetDevice(cur);
    blob->magic = 0;
    delete blob;
}

uint64_t neuzip_compressed_bytes(const neuzip_blob *blob)
{
    if (!is_blob(blob))
        return 0;
    return container_layout(blob->n, blob->k, blob->total_words, blob->block).total;
}

uint64_t neuzip_device_bytes(const neuzip_blob *blob)
{
    if (!is_blob(blob))
        return 0;
    return blob->fixed_bytes + blob->words_bytes;
}

uint64_t neuzip_elems(const neuzip_blob *blob) { return is_blob(blob) ? blob->n : 0; }
uint32_t neuzip_block_size(const neuzip_blob *blob) { return is_blob(blob) ? blob->block : 0; }
int neuzip_mantissa_bits(const neuzip_blob *blob) { return is_blob(blob) ? blob->k : -1; }

int neuzip_export(const neuzip_blob *blob, void *h_buf, uint64_t cap, uint64_t *written, void *hip_stream)
{
    if (!is_blob(blob))
        return NEUZIP_EINVAL;
    const Container lay = container_layout(blob->n, blob->k, blob->total_words, blob->block);
    if (written)
        *written = lay.total;
    if (!h_buf)
        return written ? NEUZIP_OK : NEUZIP_EINVAL;
    if (cap < lay.total)
        return NEUZIP_ENOMEM;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint8_t *p = static_cast<uint8_t *>(h_buf);
    std::memset(p, 0, lay.total);
    auto put32 = [&](uint64_t at, uint32_t v) { std::memcpy(p + at, &v, 4); };
    auto put64 = [&](uint64_t at, uint64_t v) { std::memcpy(p + at, &v, 8); };
    put32(0, kMagic);
    put32(4, 1);
    put64(8, blob->n);
    put32(16, static_cast<uint32_t>(blob->k));
    put32(20, kProbBits);
    put32(24, kChunk);
    put32(28, kStates);
    put32(32, kRun);
    put32(36, blob->n_chunks);
    put64(40, blob->total_words);
    put32(48, blob->block);
    const uint64_t nc = blob->n_chunks;
    NZ_HIP(hipMemcpyAsync(p + lay.freq, table_of(blob)->freq, 512, hipMemcpyDeviceToHost, stream));
    NZ_HIP(hipMemcpyAsync(p + lay.offsets, offsets_of(blob), (nc + 1) * 4, hipMemcpyDeviceToHost, stream));
    if (nc) {
        NZ_HIP(hipMemcpyAsync(p + lay.states, states_of(blob), nc * kStates * 4, hipMemcpyDeviceToHost, stream));
        NZ_HIP(hipMemcpyAsync(p + lay.lens, lens_of(blob), nc * kStates, hipMemcpyDeviceToHost, stream));
    }
    if (blob->total_words)
        NZ_HIP(hipMemcpyAsync(p + lay.words, blob->words, blob->total_words * 2, hipMemcpyDeviceToHost, stream));
    if (blob->n)
        NZ_HIP(hipMemcpyAsync(p + lay.sm, sm_of(blob), signmant_bytes(blob->n, blob->k), hipMemcpyDeviceToHost,
                              stream));
    if (blob->n && blob->block)
        NZ_HIP(hipMemcpyAsync(p + lay.coef, coef_of(blob), block_count(blob->n, blob->block), hipMemcpyDeviceToHost,
                              stream));
    NZ_HIP(hipStreamSynchronize(stream));
    return NEUZIP_OK;
}

int neuzip_import(const void *h_buf, uint64_t len, void *hip_stream, neuzip_blob **blob)
{
    if (!h_buf || !blob)
        return NEUZIP_EINVAL;
    if (len < kHeaderBytes + 512)
        return NEUZIP_ECORRUPT;
    const uint8_t *p = static_cast<const uint8_t *>(h_buf);
    auto get32 = [&](uint64_t at) { uint32_t v; std::memcpy(&v, p + at, 4); return v; };
    auto get64 = [&](uint64_t at) { uint64_t v; std::memcpy(&v, p + at, 8); return v; };
    if (get32(0) != kMagic || get32(4) != 1 || get32(20) != kProbBits || get32(24) != kChunk ||
        get32(28) != kStates || get32(32) != kRun)
        return NEUZIP_ECORRUPT;
    const uint64_t n = get64(8);
    const int k = static_cast<int>(get32(16));
    const uint64_t total_words = get64(40);
    const uint32_t block = get32(48);
    if (!valid_k(k) || n >= (1ull << 32) || total_words >= (1ull << 32))
        return NEUZIP_ECORRUPT;
    if (block != 0 && (!valid_block(block) || k == 7))
        return NEUZIP_ECORRUPT;
    const uint32_t nc = chunks_of(n);
    if (get32(36) != nc)
        return NEUZIP_ECORRUPT;
    const Container lay = container_layout(n, k, total_words, block);
    if (lay.total != len)
        return NEUZIP_ECORRUPT;

    // every section is checked here, on the host, so that the decoder's indexing holds
    uint16_t freq[256];
    uint16_t cum[264] = {0};
    std::memcpy(freq, p + lay.freq, 512);
    uint32_t sum = 0;
    for (int s = 0; s < 256; ++s) {
        cum[s] = static_cast<uint16_t>(sum);
        sum += freq[s];
        if (sum > kM)
            return NEUZIP_ECORRUPT;
    }
    cum[256] = static_cast<uint16_t>(sum);
    if (sum != (n ? kM : 0u))
        return NEUZIP_ECORRUPT;
    uint64_t run = 0;
    for (uint32_t c = 0; c < nc; ++c) {
        if (get32(lay.offsets + 4ull * c) != run)
            return NEUZIP_ECORRUPT;
        for (uint32_t j = 0; j < kStates; ++j) {
            const uint32_t l = p[lay.lens + static_cast<uint64_t>(c) * kStates + j];
            if (l > kRunCap)
                return NEUZIP_ECORRUPT;
            run += l;
        }
    }
    if (get32(lay.offsets + 4ull * nc) != run || run != total_words)
        return NEUZIP_ECORRUPT;

    neuzip_blob *b = nullptr;
    int rc = alloc_blob(n, k, block, &b);
    if (rc != NEUZIP_OK)
        return rc;
    auto fail = [&](int code) {
        neuzip_free(b);
        return code;
    };
    rc = reserve_words(b, total_words);
    if (rc != NEUZIP_OK)
        return fail(rc);
    b->total_words = total_words;
    std::memcpy(b->h_freq, freq, 512);
    b->have_counts = false;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    static thread_local TableBlock tb;  // 18 KB: off the stack
    std::memset(&tb, 0, sizeof(tb));
    std::memcpy(tb.freq, freq, 512);
    std::memcpy(tb.cum, cum, sizeof(tb.cum));
    tb.lone = 256;
    for (uint32_t sym = 0; sym < 256; ++sym) {
        if (freq[sym] == kM)
            tb.lone = sym;
        for (uint32_t slot = cum[sym]; slot < static_cast<uint32_t>(cum[sym]) + freq[sym]; ++slot)
            tb.lut[slot] = sym | ((freq[sym] & 0xFFFu) << 8) | ((slot - cum[sym]) << 20);
    }
    const uint32_t zeros[2] = {0, 0};
    if (!hip_ok(hipMemcpyAsync(b->fixed, &tb, sizeof(tb), hipMemcpyHostToDevice, stream)) ||
        !hip_ok(hipMemcpyAsync(offsets_of(b), p + lay.offsets, (nc + 1ull) * 4, hipMemcpyHostToDevice, stream)) ||
        !hip_ok(hipMemcpyAsync(offsets_of(b) + nc + 1, zeros, 4, hipMemcpyHostToDevice, stream)))
        return fail(NEUZIP_EHIP);
    if (nc && (!hip_ok(hipMemcpyAsync(states_of(b), p + lay.states, nc * kStates * 4ull, hipMemcpyHostToDevice, stream)) ||
               !hip_ok(hipMemcpyAsync(lens_of(b), p + lay.lens, nc * static_cast<uint64_t>(kStates), hipMemcpyHostToDevice, stream))))
        return fail(NEUZIP_EHIP);
    if (total_words && !hip_ok(hipMemcpyAsync(b->words, p + lay.words, total_words * 2, hipMemcpyHostToDevice, stream)))
        return fail(NEUZIP_EHIP);
    if (n && !hip_ok(hipMemcpyAsync(sm_of(b), p + lay.sm, signmant_bytes(n, k), hipMemcpyHostToDevice, stream)))
        return fail(NEUZIP_EHIP);
    if (n && block) {
        for (uint64_t i = 0; i < block_count(n, block); ++i)
            if (p[lay.coef + i] > 127)
                return fail(NEUZIP_ECORRUPT);
        if (!hip_ok(hipMemcpyAsync(coef_of(b), p + lay.coef, block_count(n, block), hipMemcpyHostToDevice, stream)))
            return fail(NEUZIP_EHIP);
    }
    if (!hip_ok(hipStreamSynchronize(stream)))  // tb and zeros must outlive the copies
        return fail(NEUZIP_EHIP);
    *blob = b;
    return NEUZIP_OK;
}

int neuzip_histogram(const neuzip_blob *blob, uint32_t h_counts[256])
{
    if (!is_blob(blob) || !h_counts || !blob->have_counts)
        return NEUZIP_EINVAL;
    std::memcpy(h_counts, blob->h_counts, sizeof(blob->h_counts));
    return NEUZIP_OK;
}

int neuzip_frequencies(const neuzip_blob *blob, uint16_t h_freq[256])
{
    if (!is_blob(blob) || !h_freq)
        return NEUZIP_EINVAL;
    std::memcpy(h_freq, blob->h_freq, sizeof(blob->h_freq));
    return NEUZIP_OK;
}

int neuzip_check(const neuzip_blob *blob, void *hip_stream)
{
    if (!is_blob(blob))
        return NEUZIP_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint32_t flag = 0;
    NZ_HIP(hipMemcpyAsync(&flag, table_of(blob)->status, 4, hipMemcpyDeviceToHost, stream));
    NZ_HIP(hipStreamSynchronize(stream));
    if (flag) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, stream, table_of(blob)->status, 0u, 1u);
        NZ_HIP(hipGetLastError());
        NZ_HIP(hipStreamSynchronize(stream));
        return NEUZIP_ECORRUPT;
    }
    return NEUZIP_OK;
}

int neuzip_release_workspace(void)
{
    std::lock_guard<std::mutex> guard(g_ws_mutex);
    return release_workspace_locked();
}

const char *neuzip_strerror(int code)
{
    switch (code) {
    case NEUZIP_OK: return "ok";
    case NEUZIP_EINVAL: return "invalid argument";
    case NEUZIP_ENOMEM: return "out of memory or buffer too small";
    case NEUZIP_EHIP: return "HIP runtime error";
    case NEUZIP_ECORRUPT: return "malformed container or stream";
    case NEUZIP_EUNSUPPORTED: return "size not supported";
    default: return "unknown error";
    }
}

int neuzip_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
