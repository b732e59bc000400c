// Compression kernels of the NeuZip codec for gfx950, three launches per call: histogram +
// sign|mantissa split (with and without block-wise normalisation), whose last workgroup per tensor
// builds the frequency table; the chunked rANS encoder, whose last workgroup per tensor turns the
// word counts into offsets; the compaction.  Every kernel works on a batch of up to 8 tensors
// described by a CompressBatch.
#pragma once

#include "neuzip_format.h"

namespace nz {

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

// The fields of 8 neighbouring bf16 words (four dwords), packed low element first.  For the
// lossless width a field is the word's low byte with its top bit replaced by the sign: two byte
// permutes gather the low and the high bytes of four words, one bit-select joins them.
template <int KB>
__device__ __forceinline__ uint64_t pack_fields(const uint32_t (&w)[4])
{
    if constexpr (KB == 7) {
        uint32_t out[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t low = __builtin_amdgcn_perm(w[2 * h + 1], w[2 * h], 0x06040200u);
            const uint32_t high = __builtin_amdgcn_perm(w[2 * h + 1], w[2 * h], 0x07050301u);
            out[h] = (low & 0x7F7F7F7Fu) | (high & 0x80808080u);
        }
        return static_cast<uint64_t>(out[0]) | (static_cast<uint64_t>(out[1]) << 32);
    } else {
        uint64_t packed = 0;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            packed |= static_cast<uint64_t>(signmant_field<KB>(w[p] & 0xFFFFu)) << ((2 * p) * (KB + 1));
            packed |= static_cast<uint64_t>(signmant_field<KB>(w[p] >> 16)) << ((2 * p + 1) * (KB + 1));
        }
        return packed;
    }
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

// binary16 words (HALF; beyond the paper's BFloat16): the coded symbol is a word's upper byte
// (sign, 5 exponent bits, 2 mantissa bits), the stored field its lower byte (8 mantissa bits).
template <bool HALF>
__device__ __forceinline__ uint32_t symbol_of(uint32_t u)
{
    return HALF ? (u >> 8) & 0xFFu : exponent_of(u);
}

template <int KB, bool HALF>
__device__ __forceinline__ uint32_t field_of(uint32_t u)
{
    if constexpr (HALF)
        return u & 0xFFu;
    else
        return signmant_field<KB>(u);
}

template <int KB, bool HALF>
__device__ __forceinline__ uint64_t fields_of(const uint32_t (&w)[4])
{
    if constexpr (HALF) {
        // the lower bytes of 8 neighbouring words, first element lowest
        static_assert(KB == 7, "binary16 tensors are lossless only");
        return static_cast<uint64_t>(__builtin_amdgcn_perm(w[1], w[0], 0x06040200u)) |
               (static_cast<uint64_t>(__builtin_amdgcn_perm(w[3], w[2], 0x06040200u)) << 32);
    } else {
        return pack_fields<KB>(w);
    }
}

// ------------------------------------------------------------------------------------------
// Block-wise normalisation of the lossy variant (Sec. 2.3): a block of 32..512 consecutive
// weights shares one coefficient byte, the mantissa of its largest-magnitude weight; with
// c = 1 + coef/128 a weight is stored as bf16(w / c) and comes back as bf16(stored * c), so the
// largest weight is a power of two while stored and is not touched by the mantissa truncation.
// IEEE binary32 arithmetic, results rounded to the nearest-even bf16; NaNs are passed through
// with the quiet bit set, without going through the FP unit.
// ------------------------------------------------------------------------------------------
// binary32 -> bf16, round to nearest even: the conversion instruction of gfx950
__device__ __forceinline__ uint32_t bf16_of(float v)
{
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(v));
}

__device__ __forceinline__ bool bf16_is_nan(uint32_t u) { return (u & 0x7FFFu) > 0x7F80u; }

__device__ __forceinline__ uint32_t normalise_word(uint32_t u, float c)
{
    if (bf16_is_nan(u))
        return u | 0x40u;
    return bf16_of(__uint_as_float(u << 16) / c);
}

__device__ __forceinline__ uint32_t denormalise_word(uint32_t u, float c)
{
    if (bf16_is_nan(u))
        return u | 0x40u;
    return bf16_of(__fmul_rn(__uint_as_float(u << 16), c));
}

__device__ __forceinline__ float coefficient(uint32_t coef) { return 1.0f + static_cast<float>(coef) * 0.0078125f; }

// ------------------------------------------------------------------------------------------
// Element types.  The method is stated for BFloat16 (Sec. 2.1).  A binary32 word carries the same
// sign and exponent bits in its upper half, which is a bf16 word; that half goes through the
// lossless path unchanged and the lower half, 16 mantissa bits without structure, is kept as a
// raw plane.  SourceVec holds 8 neighbouring elements of either type as the kernels read them:
// one 128-bit load (bf16) or two (binary32, WIDE), and hands out the four dwords of bf16 words.
// ------------------------------------------------------------------------------------------
template <bool WIDE>
struct SourceVec {
    uint4 a, b;  // b: elements 4..7 of a binary32 vector
    // p: the tensor as 128-bit pieces; v: index of the 8-element vector
    __device__ __forceinline__ void load(const uint4 *__restrict__ p, uint64_t v)
    {
        if constexpr (WIDE) {
            a = p[2 * v];
            b = p[2 * v + 1];
        } else {
            a = p[v];
        }
    }
    __device__ __forceinline__ void clear() { a = b = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void words(uint32_t (&w)[4]) const
    {
        if constexpr (WIDE) {
            // upper halves of two neighbours into one dword, first element low
            w[0] = __builtin_amdgcn_perm(a.y, a.x, 0x07060302u);
            w[1] = __builtin_amdgcn_perm(a.w, a.z, 0x07060302u);
            w[2] = __builtin_amdgcn_perm(b.y, b.x, 0x07060302u);
            w[3] = __builtin_amdgcn_perm(b.w, b.z, 0x07060302u);
        } else {
            w[0] = a.x;
            w[1] = a.y;
            w[2] = a.z;
            w[3] = a.w;
        }
    }
    // the lower halves of a binary32 vector, in element order
    __device__ __forceinline__ uint4 lows() const
    {
        return make_uint4(__builtin_amdgcn_perm(a.y, a.x, 0x05040100u), __builtin_amdgcn_perm(a.w, a.z, 0x05040100u),
                          __builtin_amdgcn_perm(b.y, b.x, 0x05040100u), __builtin_amdgcn_perm(b.w, b.z, 0x05040100u));
    }
};

// Element i of a tensor of either type as a bf16 word; for binary32 the lower half goes to the plane.
template <bool WIDE, bool KEEP_LOW>
__device__ __forceinline__ uint32_t source_word(const void *__restrict__ src, uint16_t *__restrict__ low, uint64_t i)
{
    if constexpr (WIDE) {
        const uint32_t u = static_cast<const uint32_t *>(src)[i];
        if constexpr (KEEP_LOW)
            low[i] = static_cast<uint16_t>(u);
        return u >> 16;
    } else {
        return static_cast<const uint16_t *>(src)[i];
    }
}

// Stores and atomics issued so far by this wave have been performed (their acknowledgements are in)
// before anything that follows.
__device__ __forceinline__ void wait_for_memory_acks() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ------------------------------------------------------------------------------------------
// Counts -> frequencies that sum to 4096, cumulative table: by ONE wave, lane l owning symbols
// 4l .. 4l + 3, with lane shuffles only (no barrier), so that every encoder workgroup can derive
// the table of its tensor from the 256 counts by itself and no launch is spent on it.
// Integer only:
//   f = max(1, floor(cnt * 4096 / N)) for symbols that occur, else 0; a shortfall goes to the
//   most frequent symbol (lowest value on a tie); an excess is taken one unit at a time from
//   the symbol whose f is largest at that moment (lowest value on a tie).
// ------------------------------------------------------------------------------------------
// Inclusive scan of v over the 64 lanes of the wave with data-parallel-primitive moves (vector ALU
// rate: no trip through the LDS crossbar as with a lane shuffle): inside each row of 16 lanes by
// shifts of 1, 2, 4, 8 (a lane without a source keeps the identity), then the last lane of rows 0
// and 2 is added into rows 1 and 3, then lane 31 into rows 2 and 3.  All 64 lanes must be active.
template <class Op>
__device__ __forceinline__ uint32_t wave_scan_u32(uint32_t v, uint32_t identity, Op op)
{
#define NZ_DPP(ctrl, rows) \
    static_cast<uint32_t>(__builtin_amdgcn_update_dpp(static_cast<int>(identity), static_cast<int>(v), ctrl, rows, 0xf, false))
    v = op(v, NZ_DPP(0x111, 0xf));  // row_shr:1
    v = op(v, NZ_DPP(0x112, 0xf));  // row_shr:2
    v = op(v, NZ_DPP(0x114, 0xf));  // row_shr:4
    v = op(v, NZ_DPP(0x118, 0xf));  // row_shr:8
    v = op(v, NZ_DPP(0x142, 0xa));  // row_bcast:15 into rows 1 and 3
    v = op(v, NZ_DPP(0x143, 0xc));  // row_bcast:31 into rows 2 and 3
#undef NZ_DPP
    return v;
}

struct OpAdd {
    __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a + b; }
};
struct OpMax {
    __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; }
};

// Sum / maximum over the wave, the same value in every lane (lane 63 of the scan, read out as a scalar).
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(wave_scan_u32(v, 0u, OpAdd{})), 63));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(wave_scan_u32(v, 0u, OpMax{})), 63));
}

// The frequencies (f) and exclusive cumulative frequencies (cum) of symbols 4 * lane .. 4 * lane + 3
// from their counts, which add up to `total`; returns the tensor's only exponent value if it has
// just one, else 256.  Must be called by all 64 lanes of a wave.
__device__ inline uint32_t build_table_wave(const uint32_t (&cnt)[4], uint64_t total, uint32_t guard, uint32_t (&f)[4],
                                            uint32_t (&cum)[4])
{
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        f[i] = 0;
    if (total > 0) {
        const float total_f = static_cast<float>(total);
        // With a guard band every exponent from (lowest occurring - guard) to (highest occurring +
        // guard), and exponent 0 (an update cancels exactly to +-0 now and then), is treated as
        // occurring: it gets f = 1 and can be coded after a weight update without a new table.
        uint32_t hi = 0, lo = 0;
        if (guard > 0) {
            uint32_t top = 0, bottom = 0;  // highest occupied symbol + 1; 256 - lowest occupied symbol
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t s = 4 * lane + i;
                if (cnt[i] > 0) {
                    top = s + 1 > top ? s + 1 : top;
                    bottom = 256 - s > bottom ? 256 - s : bottom;
                }
            }
            hi = wave_max_u32(top) - 1;
            lo = 256 - wave_max_u32(bottom);
        }
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t s = 4 * lane + i;
            const bool member = cnt[i] > 0 || (guard > 0 && (s == 0 || (s + guard >= lo && s <= hi + guard)));
            if (member) {
                // floor(cnt * 4096 / total) without a 64-bit division: the float quotient is within one
                // of it (its relative error is below 2^-22 and the quotient at most 4096), and the exact
                // remainder tells which way
                const uint64_t num = static_cast<uint64_t>(cnt[i]) * kM;
                uint32_t q = static_cast<uint32_t>(__fdiv_rn(static_cast<float>(num), total_f));
                q = q > kM ? kM : q;
                const int64_t r = static_cast<int64_t>(num - static_cast<uint64_t>(q) * total);
                if (r < 0)
                    q -= 1;
                else if (r >= static_cast<int64_t>(total))
                    q += 1;
                f[i] = q < 1 ? 1u : q;
            }
            sum += f[i];
        }
        int32_t rest = static_cast<int32_t>(kM) - static_cast<int32_t>(wave_sum_u32(sum));
        if (rest > 0) {
            // the most frequent symbol, the lowest one on a tie
            uint32_t most = cnt[0];
#pragma unroll
            for (int i = 1; i < 4; ++i)
                most = cnt[i] > most ? cnt[i] : most;
            most = wave_max_u32(most);
            uint32_t who = 0;  // 256 - symbol of this lane's lowest symbol with that count
#pragma unroll
            for (int i = 3; i >= 0; --i)
                who = cnt[i] == most ? 256 - (4 * lane + i) : who;
            who = 256 - wave_max_u32(who);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (4 * lane + i == who)
                    f[i] += static_cast<uint32_t>(rest);
        }
        while (rest < 0) {  // uniform across the wave
            uint32_t key = 0, runner = 0;  // the two largest (f, lowest symbol first) of this lane
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t k = (f[i] << 8) | (255u - (4 * lane + i));
                runner = k > key ? key : (k > runner ? k : runner);
                key = k > key ? k : key;
            }
            const uint32_t best = wave_max_u32(key);
            const uint32_t second = wave_max_u32(key == best ? runner : key);
            // Usual case: the largest symbol stays the largest through all -rest decrements (its key
            // after -rest - 1 of them still beats the runner-up's), so it takes them all at once.
            const uint32_t want = static_cast<uint32_t>(-rest);
            const bool all_at_once = (best >> 8) >= want && best - ((want - 1) << 8) > second;
            const uint32_t take = all_at_once ? want : 1u;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (((f[i] << 8) | (255u - (4 * lane + i))) == best)
                    f[i] -= take;
            rest += static_cast<int32_t>(take);
        }
    }
    // exclusive cumulative sums: over the lanes before, then inside the lane
    const uint32_t mine = f[0] + f[1] + f[2] + f[3];
    cum[0] = wave_scan_u32(mine, 0u, OpAdd{}) - mine;
    cum[1] = cum[0] + f[0];
    cum[2] = cum[1] + f[1];
    cum[3] = cum[2] + f[2];
    uint32_t lone = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        lone = f[i] == kM ? 4 * lane + i + 1 : lone;
    lone = wave_max_u32(lone);
    return lone ? lone - 1 : 256u;
}

// Encoder constants of a symbol.  A symbol without room in the table (f = 0) gets constants that
// leave the state as it is and a zero reciprocal, by which the encoder recognises it.
__device__ inline EncSym encoder_constants(uint32_t f, uint32_t cum)
{
    EncSym e = {0.0f, 0xFFFF0000u, 1u, 0};
    if (f > 0) {
        e.rcp = __fmul_rn(__fdiv_rn(1.0f, static_cast<float>(f)), 1.0f - 0x1p-21f);
        // f = 4096 only for a one-symbol tensor: the state stays at 2^16 and never renormalises
        e.limit_cum = (f >= kM ? 0xFFFF0000u : (f << 20)) | cum;
        e.f = f;
        e.neg_cmpl = static_cast<int32_t>(f) - static_cast<int32_t>(kM);
    }
    return e;
}

// Decoder slot table of a tensor: lut[slot] = symbol | f << 8 | (slot - cum[symbol]) << 20.
// 256 threads; scan[t] = cum[t + 1] (in LDS, complete); thread s fills slots s, s + 256, ...
__device__ inline void build_slot_table(TableBlock *__restrict__ tb, const uint32_t *__restrict__ scan)
{
    const uint32_t s = threadIdx.x;
    if (scan[255] != kM)
        return;  // an empty table: nothing decodes through it
    // (four searches at a time: this runs beside the encoders in their kernel and must not raise its
    // register count)
    constexpr uint32_t kPer = kM / 256, kAtOnce = 4;
#pragma unroll 1
    for (uint32_t r0 = 0; r0 < kPer; r0 += kAtOnce) {
        uint32_t lo[kAtOnce], hi[kAtOnce];
#pragma unroll
        for (uint32_t r = 0; r < kAtOnce; ++r) {
            lo[r] = 0;
            hi[r] = 255;
        }
#pragma unroll
        for (uint32_t step = 0; step < 8; ++step) {
#pragma unroll
            for (uint32_t r = 0; r < kAtOnce; ++r) {  // smallest t with cum[t + 1] > slot
                const uint32_t mid = (lo[r] + hi[r]) >> 1;
                const bool above = scan[mid] > s + 256 * (r0 + r);
                hi[r] = above ? mid : hi[r];
                lo[r] = above ? lo[r] : (mid < hi[r] ? mid + 1 : hi[r]);
            }
        }
#pragma unroll
        for (uint32_t r = 0; r < kAtOnce; ++r) {
            const uint32_t slot = s + 256 * (r0 + r), t = lo[r];
            const uint32_t begin = t ? scan[t - 1] : 0u;
            tb->lut[slot] = t | (((scan[t] - begin) & 0xFFFu) << 8) | ((slot - begin) << 20);
        }
    }
}

constexpr uint32_t kHistCopies = 32;

// End of a histogram workgroup: thread b sums the 32 copies of bin b (starting at a rotated copy to
// spread the banks) and adds the sum to the workspace bin.
__device__ __forceinline__ void merge_bins(const uint32_t *__restrict__ bins, uint32_t *__restrict__ counts)
{
    __syncthreads();
    const uint32_t s = threadIdx.x;
    if (s >= 256)
        return;
    uint32_t sum = 0;
#pragma unroll 8
    for (uint32_t i = 0; i < kHistCopies; ++i)
        sum += bins[s * kHistCopies + ((i + s) & (kHistCopies - 1))];
    if (sum)
        atomicAdd(&counts[s], sum);
}

// ------------------------------------------------------------------------------------------
// Kernel 1: exponent histogram fused with the sign|mantissa split (Alg. 1 "split").
// One pass over the bf16 words: 2 B/elem read, (k+1)/8 B/elem written.  Counts go to 32
// bank-private copies of the 256 bins in LDS (copy = lane mod 32, so the 64 lanes of a wave
// hit 32 different banks whatever the symbol skew is), then one global atomic per bin.
// ------------------------------------------------------------------------------------------
// Workgroups of 256 threads for tensors that stream through HBM, of 1024 threads (and fewer of them)
// for a batch that fits the last-level cache: there the pass is short, and the merges of the
// workgroups' bins into the global ones, which all arrive at its end, are what is left to shorten.
constexpr uint32_t kHistThreadsMax = 1024;

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

template <int KB, bool WIDE = false, bool HALF = false>
__global__ __launch_bounds__(kHistThreadsMax) void hist_split_kernel(const CompressBatch b,
                                                                 uint32_t *__restrict__ counts_ws)
{
    const ItemSlot slot = item_of_workgroup<&CompressItem::hist_end>(b);
    const void *__restrict__ src = b.it[slot.item].src;
    const uint64_t n = b.it[slot.item].n;
    uint8_t *__restrict__ sm = b.it[slot.item].sm;
    uint16_t *__restrict__ low = b.it[slot.item].low;
    uint32_t *__restrict__ counts = counts_ws + 256 * slot.item;
    __shared__ uint32_t bins[256 * kHistCopies];
    for (uint32_t i = threadIdx.x; i < 256 * kHistCopies; i += blockDim.x)
        bins[i] = 0;
    __syncthreads();

    const uint32_t copy = threadIdx.x & (kHistCopies - 1);
    const uint64_t n_vec = n / 8;
    const uint64_t stride = static_cast<uint64_t>(slot.wgs) * blockDim.x;
    const uint4 *src4 = static_cast<const uint4 *>(src);
    // eight 128-bit loads are in flight per lane before any of them is used (four vectors of
    // binary32, which take two loads each); measured 5 % faster than four on a cache-resident tensor
    constexpr uint32_t kDepth = WIDE ? 4 : 8;
    for (uint64_t v0 = static_cast<uint64_t>(slot.wg) * blockDim.x + threadIdx.x; v0 < n_vec;
         v0 += stride * kDepth) {
        SourceVec<WIDE> d[kDepth];
#pragma unroll
        for (uint32_t r = 0; r < kDepth; ++r) {
            const uint64_t v = v0 + r * stride;
            if (v < n_vec)
                d[r].load(src4, v);
            else
                d[r].clear();
        }
#pragma unroll
        for (uint32_t r = 0; r < kDepth; ++r) {
            const uint64_t v = v0 + r * stride;
            if (v >= n_vec)
                break;
            uint32_t w[4];
            d[r].words(w);
            if constexpr (WIDE)
                reinterpret_cast<uint4 *>(low)[v] = d[r].lows();
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t lo = w[p] & 0xFFFFu, hi = w[p] >> 16;
                atomicAdd(&bins[symbol_of<HALF>(lo) * kHistCopies + copy], 1u);
                atomicAdd(&bins[symbol_of<HALF>(hi) * kHistCopies + copy], 1u);
            }
            store_fields<KB>(sm, v, fields_of<KB, HALF>(w));
        }
    }
    // ragged tail (n mod 8 elements): one thread, element by element
    if (slot.wg == 0 && threadIdx.x == 0) {
        constexpr uint32_t per_byte = 8 / (KB + 1);
        uint32_t acc = 0, filled = 0;
        for (uint64_t i = n_vec * 8; i < n; ++i) {
            const uint32_t u = source_word<WIDE, true>(src, low, i);
            atomicAdd(&bins[symbol_of<HALF>(u) * kHistCopies + copy], 1u);
            acc |= field_of<KB, HALF>(u) << (filled * (KB + 1));
            if (++filled == per_byte) {
                sm[i / per_byte] = static_cast<uint8_t>(acc);
                acc = 0;
                filled = 0;
            }
        }
        if (filled)
            sm[(n - 1) / per_byte] = static_cast<uint8_t>(acc);
    }
    merge_bins(bins, counts);
}

// ------------------------------------------------------------------------------------------
// Kernel 1b: the same pass for block-wise normalised lossy compression.  A block of B weights
// is B/8 neighbouring lanes (each lane holds 8 weights), so the largest magnitude of a block is
// a shuffle reduction over 4..64 lanes; its mantissa is the block's coefficient.  The lane then
// normalises its weights and proceeds as kernel 1 on the normalised words.
// ------------------------------------------------------------------------------------------
template <int KB>
__global__ __launch_bounds__(kHistThreadsMax) void hist_split_norm_kernel(const CompressBatch b,
                                                                      uint32_t *__restrict__ counts_ws)
{
    const ItemSlot slot = item_of_workgroup<&CompressItem::hist_end>(b);
    const uint16_t *__restrict__ src = static_cast<const uint16_t *>(b.it[slot.item].src);
    const uint64_t n = b.it[slot.item].n;
    const uint32_t block = b.it[slot.item].block;
    uint8_t *__restrict__ coef_out = b.it[slot.item].coef;
    uint8_t *__restrict__ sm = b.it[slot.item].sm;
    uint32_t *__restrict__ counts = counts_ws + 256 * slot.item;
    __shared__ uint32_t bins[256 * kHistCopies];
    for (uint32_t i = threadIdx.x; i < 256 * kHistCopies; i += blockDim.x)
        bins[i] = 0;
    __syncthreads();

    const uint32_t copy = threadIdx.x & (kHistCopies - 1);
    const uint32_t lanes_per_block = block / 8;                 // 4 .. 64, a power of two
    const uint32_t block_shift = 31u - static_cast<uint32_t>(__clz(static_cast<int>(block)));
    const uint64_t n_vec = (n + 7) / 8;                         // the last vector may be partial
    const uint64_t stride = static_cast<uint64_t>(slot.wgs) * blockDim.x;
    constexpr uint32_t per_byte = 8 / (KB + 1);
    // the trip count is the same for all lanes of a wave, so every lane takes part in the shuffles
    const uint64_t wave_first = static_cast<uint64_t>(slot.wg) * blockDim.x + (threadIdx.x & ~63u);
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
        const uint32_t pos0 = static_cast<uint32_t>(first & (block - 1));  // block sizes are powers of two
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
            coef_out[first >> block_shift] = static_cast<uint8_t>(coef);
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
    merge_bins(bins, counts);
}

// The weight update of the backward loop (Alg. 1: W_hat <- W_hat - lr * grad) on the two halves of
// a merged dword: product and difference each rounded to binary32 (no fused multiply-add), the
// result rounded to the nearest-even bf16, a NaN result stored as 0x7FC0.
__device__ __forceinline__ float sgd_step(float w, float g, float lr)
{
#pragma clang fp contract(off)
    const float step = lr * g;
    return w - step;
}

__device__ __forceinline__ uint32_t update_pair(uint32_t w, uint32_t g, float lr)
{
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
    const f32x2_t v = {sgd_step(__uint_as_float(w << 16), __uint_as_float(g << 16), lr),
                       sgd_step(__uint_as_float(w & 0xFFFF0000u), __uint_as_float(g & 0xFFFF0000u), lr)};
    uint32_t r = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
    if (__builtin_expect(__builtin_isunordered(v[0], v[1]), 0)) {  // one compare finds a NaN in either half
        if (v[0] != v[0])
            r = (r & 0xFFFF0000u) | 0x7FC0u;
        if (v[1] != v[1])
            r = (r & 0x0000FFFFu) | 0x7FC00000u;
    }
    return r;
}

__device__ __forceinline__ uint32_t update_word(uint32_t w, uint32_t g, float lr)
{
    const float v = sgd_step(__uint_as_float(w << 16), __uint_as_float(g << 16), lr);
    return v != v ? 0x7FC0u : bf16_of(v);
}

// The weight step alone, in place: w <- w - lr * g over n bf16 words (for the rare tensor whose
// kept table did not serve after a fused step that was asked not to write the new weight back).
__global__ __launch_bounds__(256) void sgd_update_kernel(uint16_t *__restrict__ w, const uint16_t *__restrict__ g,
                                                         uint64_t n, float lr)
{
    const uint64_t n_vec = n / 8;
    uint4 *w4 = reinterpret_cast<uint4 *>(w);
    const uint4 *g4 = reinterpret_cast<const uint4 *>(g);
    for (uint64_t v = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; v < n_vec;
         v += static_cast<uint64_t>(gridDim.x) * blockDim.x) {
        const uint4 a = w4[v], c = g4[v];
        w4[v] = make_uint4(update_pair(a.x, c.x, lr), update_pair(a.y, c.y, lr), update_pair(a.z, c.z, lr),
                           update_pair(a.w, c.w, lr));
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (uint64_t i = n_vec * 8; i < n; ++i)
            w[i] = static_cast<uint16_t>(update_word(w[i], g[i], lr));
}

// ------------------------------------------------------------------------------------------
// Kernel 3: chunked rANS encoder (Sec. 2.2 "Compression algorithm").  One lane per state.
// A state visits its symbols back to front; the words it pushes out are collected, back to
// front, in a 16-word LDS ring and leave for the state's 200-word slot of the workspace in
// 16-byte pieces (interleaved with the other states' of the chunk, see slot_word), so that the
// tail of the slot read forwards is the decoder's order.  Final
// states and run lengths go straight to their place in the blob; the chunk's word count goes to
// the workspace for the offsets scan.  A turn's 8 bf16 words are requested two turns ahead.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kEncThreads = 256;
constexpr uint32_t kChunksPerGroup = kEncThreads / kStates;  // 16 chunks per encoder workgroup
constexpr uint32_t kRingWords = 16;  // per state; two halves of 8 words = 16 bytes

struct EncState {
    uint32_t x;
    uint32_t wp;          // next free position in the slot is wp - 1 (words, counts down from kRunCap);
                          // brought up to date once per turn (ring_advance)
    uint32_t cur;         // byte position of the last word written in the workgroup's ring array:
                          // lane * 32 + 2 * (wp mod 16)
};

// rings: the workgroup's ring array as bytes; lane_ring: this lane's 32-byte ring in it (threadIdx.x * 32)
__device__ __forceinline__ void rans_put(EncState &st, const EncSym e, uint8_t *__restrict__ rings, uint32_t lane_ring)
{
    if ((st.x >> 16) >= (e.limit_cum >> 16)) {
        // one position down, wrapping inside the lane's 16 words: two instructions for the address
        st.cur = lane_ring | ((st.cur - 2u) & (2u * kRingWords - 2u));
        *reinterpret_cast<uint16_t *>(rings + st.cur) = static_cast<uint16_t>(st.x);
        // (the shift as written keeps the compiler from sharing it with the test above, which reads the
        // state's upper half through an operand select and needs no shift of its own)
        asm volatile("v_lshrrev_b32 %0, 16, %0" : "+v"(st.x));
    }
    // -q or -(q - 1): the conversion truncates toward zero, as it does for the positive product
    int32_t qn = static_cast<int32_t>(-__fmul_rn(__uint2float_rn(st.x), e.rcp));
    const uint32_t r = static_cast<uint32_t>(__mul24(qn, static_cast<int32_t>(e.f))) + st.x;
    qn -= r >= e.f ? 1 : 0;
    const uint32_t grown = static_cast<uint32_t>(__mul24(qn, e.neg_cmpl)) + st.x;
    // + cum, the lower half of limit_cum, taken by the add's operand select
    asm("v_add_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
        : "=v"(st.x)
        : "v"(grown), "v"(e.limit_cum));
}

// Layout of a chunk's 16 slots in the workspace (16 x 200 words): word position p of state j sits
// at ((p / 8) * 16 + j) * 8 + p % 8, i.e. the 16-byte pieces of the 16 states are interleaved.
// The states of a chunk fill their pieces at about the same pace, from the top down, so the
// pieces that leave within a few turns of each other are neighbours in memory and merge into
// whole cache lines before they are written back; slot-by-slot they would be 400 bytes apart and
// reach memory as partial lines (measured: 1.5x the encode time on tensors beyond the cache).
__device__ __forceinline__ uint32_t slot_word(uint32_t j, uint32_t p)
{
    return (((p >> 3) * kStates + j) << 3) | (p & 7u);
}

// The words pushed since `cur_before` (at most 8 per turn, so the ring position tells) come off wp.
__device__ __forceinline__ void ring_advance(EncState &st, uint32_t cur_before)
{
    st.wp -= ((cur_before - st.cur) & (2u * kRingWords - 2u)) >> 1;
}

// Moves the 8-word group completed during the last turn (at most one: a turn pushes at most 8
// words) from the ring to the slot.  Positions run down from wp_before to wp_after; group g
// (positions 8g .. 8g+7) is complete once position 8g has been written.
__device__ __forceinline__ void ring_flush(uint32_t wp_before, uint32_t wp_after, const uint16_t *__restrict__ ring,
                                           uint16_t *__restrict__ chunk_slots, uint32_t j)
{
    const uint32_t g = (wp_after + 7) >> 3;  // lowest group whose first position is >= wp_after
    if (g * 8 < wp_before) {
        const uint4 v = *reinterpret_cast<const uint4 *>(ring + ((g * 8) & (kRingWords - 1)));
        *reinterpret_cast<uint4 *>(chunk_slots + slot_word(j, g * 8)) = v;
    }
}

// SPLIT >= 0: the one-pass variant used for recompression with an existing table.  There is no
// histogram pass to produce the sign|mantissa stream, so this kernel packs and stores the fields
// (SPLIT = mantissa bits) of the words it codes, and it reports, through stale[item], any exponent
// that the table has no room for (such symbols leave the state unchanged; the host then falls
// back to a compression with fresh statistics).
// UPD (with SPLIT = 7): the backward loop's weight step fused in.  The source holds the decompressed
// weight, `grad` its gradient; the kernel forms W - lr * grad, writes it back over the source and
// codes it, so the new weight is read once and never re-read from memory.
template <bool NORM, int SPLIT, bool WIDE = false, bool HALF = false, bool UPD = false>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(const CompressBatch b,
                                                            const uint32_t *__restrict__ counts_ws,
                                                            uint32_t *__restrict__ chunk_words_all,
                                                            uint32_t *__restrict__ group_words_all,
                                                            uint32_t *__restrict__ super_words_all,
                                                            uint16_t *__restrict__ slots_all,
                                                            HostRecord *__restrict__ record,
                                                            CallState *__restrict__ state)
{
    static_assert(!(NORM && SPLIT >= 0), "the one-pass variant has no block maxima to normalise with");
    static_assert(!(WIDE || HALF) || (!NORM && (SPLIT < 0 || SPLIT == 7)), "binary32 and binary16 tensors are lossless only");
    static_assert(!(WIDE && HALF), "one element type");
    static_assert(!UPD || (SPLIT == 7 && !NORM && !WIDE && !HALF), "only lossless bf16 weights are trained");
    constexpr int KB = SPLIT >= 0 ? SPLIT : 7;
    __shared__ uint4 enc_raw[256];
    __shared__ __align__(32) uint16_t rings[kEncThreads * kRingWords];
    __shared__ uint32_t group_chunk[kEncThreads / kStates];
    const uint32_t all_groups = b.it[b.count - 1].enc_end;
    const bool table_wg = blockIdx.x >= all_groups;  // behind the encoders' (fresh tables only): one per tensor
    ItemSlot slot_id;
    if (table_wg)
        slot_id = {blockIdx.x - all_groups, 0u, 0u};
    else
        slot_id = item_of_workgroup<&CompressItem::enc_end>(b);
    const CompressItem &it = b.it[slot_id.item];
    const void *__restrict__ src = it.src;
    uint16_t *__restrict__ low = it.low;
    const uint16_t *__restrict__ grad = it.grad;
    const float lr = b.lr;
    const uint64_t n = it.n;
    const uint8_t *__restrict__ coef = it.coef;
    const uint32_t block_shift = NORM ? 31u - static_cast<uint32_t>(__clz(static_cast<int>(it.block | 1u))) : 0u;
    const uint32_t n_chunks = it.n_chunks;
    TableBlock *__restrict__ tb = it.tb;
    uint32_t *__restrict__ states = it.states;
    uint8_t *__restrict__ lens = it.lens;
    // this tensor's part of the workspace arrays
    const uint32_t group = it.group_base + slot_id.wg;
    uint32_t *__restrict__ chunk_words = chunk_words_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup;
    uint16_t *__restrict__ slots = slots_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup * kStates * kRunCap;

    const uint32_t lane_id = slot_id.wg * kEncThreads + threadIdx.x;  // = chunk * 16 + state
    const uint32_t c = lane_id / kStates, j = lane_id % kStates;
    const bool live = !table_wg && c < n_chunks;
    const uint64_t base = static_cast<uint64_t>(c) * kChunk;
    const uint32_t m = !live ? 0u : ((n - base) < kChunk ? static_cast<uint32_t>(n - base) : kChunk);
    // The source words of a full chunk are requested two turns ahead, in three buffers used in
    // rotation; the first two requests go out here, so that they travel while the table is made.
    // This state's first 8-element vector of the chunk; a turn later is kStates vectors on.
    const uint4 *src4 = static_cast<const uint4 *>(src) + (base / 8 + j) * (WIDE ? 2 : 1);
    // the gradients travel with the weights, one 128-bit piece per turn
    const uint4 *grad4 = UPD ? reinterpret_cast<const uint4 *>(grad) + (base / 8 + j) : nullptr;
    SourceVec<WIDE> d0, d1, d2;
    uint4 g0 = make_uint4(0, 0, 0, 0), g1 = g0, g2 = g0;
    if (m == kChunk) {
        d0.load(src4, (kTurns - 1) * kStates);
        d1.load(src4, (kTurns - 2) * kStates);
        if constexpr (UPD) {
            g0 = grad4[(kTurns - 1) * kStates];
            g1 = grad4[(kTurns - 2) * kStates];
        }
    }

    // ---- encoder constants of the 256 symbols
    if constexpr (SPLIT < 0) {
        // Fresh statistics: the histogram pass has left the 256 counts in the workspace; the first wave
        // of every workgroup turns them into the table by itself (the same arithmetic everywhere, so
        // the same table).  The tensor's first workgroup also puts the table into the blob and posts
        // the statistics to the host.
        if (threadIdx.x < 64) {
            const uint32_t lane = threadIdx.x;
            const uint4 c4 = reinterpret_cast<const uint4 *>(counts_ws + 256 * slot_id.item)[lane];
            const uint32_t cnt[4] = {c4.x, c4.y, c4.z, c4.w};
            uint32_t f[4], cum[4];
            const uint32_t lone = build_table_wave(cnt, it.table_n, it.guard, f, cum);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const EncSym e = encoder_constants(f[i], cum[i]);
                enc_raw[4 * lane + i] = make_uint4(__float_as_uint(e.rcp), e.limit_cum, e.f, static_cast<uint32_t>(e.neg_cmpl));
            }
            if (table_wg) {
                uint32_t *scan = reinterpret_cast<uint32_t *>(rings);  // scan[t] = cum[t + 1]
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    scan[4 * lane + i] = cum[i] + f[i];
            } else if (slot_id.wg == 0) {
                reinterpret_cast<uint4 *>(tb->counts)[lane] = c4;
                reinterpret_cast<uint2 *>(tb->freq)[lane] = make_uint2(f[0] | (f[1] << 16), f[2] | (f[3] << 16));
                reinterpret_cast<uint2 *>(tb->cum)[lane] = make_uint2(cum[0] | (cum[1] << 16), cum[2] | (cum[3] << 16));
                if (lane == 63)
                    tb->cum[256] = static_cast<uint16_t>(cum[3] + f[3]);
                if (lane < 4)
                    tb->status[lane] = 0;
                if (lane == 0)
                    tb->lone = lone;
                // The statistics for the host, as whole-wave stores (1 KB and 512 B).  They are complete when
                // this kernel ends; the stamp that tells the host to look is written by the kernel after it.
                HostRecord::Item *mine = &record->item[slot_id.item];
                reinterpret_cast<uint4 *>(mine->counts)[lane] = c4;
                reinterpret_cast<uint2 *>(mine->freq)[lane] = make_uint2(f[0] | (f[1] << 16), f[2] | (f[3] << 16));
            }
        }
    } else {
        // the table the blob holds
        const EncSym e = encoder_constants(tb->freq[threadIdx.x], tb->cum[threadIdx.x]);
        enc_raw[threadIdx.x] = make_uint4(__float_as_uint(e.rcp), e.limit_cum, e.f, static_cast<uint32_t>(e.neg_cmpl));
    }
    __syncthreads();
    if (table_wg) {
        // fills in the decoder's slot table while the others encode
        build_slot_table(tb, reinterpret_cast<const uint32_t *>(rings));
        return;
    }
    const EncSym *enc = reinterpret_cast<const EncSym *>(enc_raw);

    uint16_t *chunk_slots = slots + static_cast<uint64_t>(c) * kStates * kRunCap;
    uint16_t *ring = rings + threadIdx.x * kRingWords;
    uint8_t *ring_bytes = reinterpret_cast<uint8_t *>(rings);
    const uint32_t lane_ring = threadIdx.x * (2u * kRingWords);
    EncState st = {kRansL, kRunCap, lane_ring + 2u * (kRunCap % kRingWords)};
    float least_rcp = 1.0f;  // 0 once a symbol without room in the table has been met
    uint8_t *__restrict__ sm = it.sm;

    if (m == kChunk) {
        // One turn: the vector of turn q - 2 is requested into the buffer that is free (the wait for a
        // turn's words then leaves the stores of the turn before -- ring flush, fields -- in flight
        // instead of waiting for them), then turn q is coded from its buffer.
        auto turn = [&](const SourceVec<WIDE> &d, const uint4 &g, SourceVec<WIDE> &d_after, uint4 &g_after, int q) {
            d_after.load(src4, (q > 1 ? q - 2 : 0) * kStates);
            if constexpr (UPD)
                g_after = grad4[(q > 1 ? q - 2 : 0) * kStates];
            uint32_t w[4];
            d.words(w);
            if constexpr (UPD) {
                w[0] = update_pair(w[0], g.x, lr);
                w[1] = update_pair(w[1], g.y, lr);
                w[2] = update_pair(w[2], g.z, lr);
                w[3] = update_pair(w[3], g.w, lr);
                // if the caller wants it, the new weight replaces the old one in its buffer (same lane,
                // same place)
                if (b.keep_new)
                    reinterpret_cast<uint4 *>(const_cast<void *>(src))[base / 8 + static_cast<uint32_t>(q) * kStates + j] =
                        make_uint4(w[0], w[1], w[2], w[3]);
            }
            const uint32_t wp_before = st.wp, cur_before = st.cur;
            if constexpr (SPLIT >= 0) {
                store_fields<KB>(sm, base / 8 + static_cast<uint32_t>(q) * kStates + j, fields_of<KB, HALF>(w));
                if constexpr (WIDE)
                    reinterpret_cast<uint4 *>(low)[base / 8 + static_cast<uint32_t>(q) * kStates + j] = d.lows();
            }
            // with block-wise normalisation the exponents coded are those of bf16(w / c)
            float c = 1.0f;
            if constexpr (NORM)
                c = coefficient(coef[(base + static_cast<uint32_t>(q) * kTurn + j * kRun) >> block_shift]);
#pragma unroll
            for (int p = 3; p >= 0; --p) {
                const uint32_t hi = NORM ? normalise_word(w[p] >> 16, c) : (w[p] >> 16);
                const uint32_t lo = NORM ? normalise_word(w[p] & 0xFFFFu, c) : (w[p] & 0xFFFFu);
                const EncSym e_hi = enc[symbol_of<HALF>(hi)], e_lo = enc[symbol_of<HALF>(lo)];
                if constexpr (SPLIT >= 0) {
                    least_rcp = fminf(least_rcp, fminf(e_hi.rcp, e_lo.rcp));
                    // (taken here and now: left to the scheduler, the minimum is put off to the end of the
                    // loop body and every symbol's four registers stay occupied until then)
                    asm volatile("" : "+v"(least_rcp));
                }
                rans_put(st, e_hi, ring_bytes, lane_ring);
                rans_put(st, e_lo, ring_bytes, lane_ring);
            }
            ring_advance(st, cur_before);
            ring_flush(wp_before, st.wp, ring, chunk_slots, j);
        };
        // turns in groups of three (so that no buffer has to be copied into another); what is left over
        // when the number of turns is no multiple of three comes last, with the rotation continued
        int q = static_cast<int>(kTurns) - 1;
        for (; q >= 2; q -= 3) {
            turn(d0, g0, d2, g2, q);
            turn(d1, g1, d0, g0, q - 1);
            turn(d2, g2, d1, g1, q - 2);
        }
        if constexpr (kTurns % 3 >= 1)
            turn(d0, g0, d2, g2, q);
        if constexpr (kTurns % 3 == 2)
            turn(d1, g1, d0, g0, q - 1);
    } else if (m > 0) {
        for (int q = static_cast<int>(kTurns) - 1; q >= 0; --q) {
            const uint32_t wp_before = st.wp, cur_before = st.cur;
            uint64_t packed = 0;
            for (int t = static_cast<int>(kRun) - 1; t >= 0; --t) {
                const uint32_t i = static_cast<uint32_t>(q) * kTurn + j * kRun + static_cast<uint32_t>(t);
                if (i < m) {
                    uint32_t u = source_word<WIDE, (SPLIT >= 0)>(src, low, base + i);
                    if constexpr (UPD) {
                        u = update_word(u, grad[base + i], lr);
                        if (b.keep_new)
                            static_cast<uint16_t *>(const_cast<void *>(src))[base + i] = static_cast<uint16_t>(u);
                    }
                    if constexpr (NORM)
                        u = normalise_word(u, coefficient(coef[(base + i) >> block_shift]));
                    const EncSym e = enc[symbol_of<HALF>(u)];
                    if constexpr (SPLIT >= 0) {
                        least_rcp = fminf(least_rcp, e.rcp);
                        packed |= static_cast<uint64_t>(field_of<KB, HALF>(u)) << (static_cast<uint32_t>(t) * (KB + 1));
                    }
                    rans_put(st, e, ring_bytes, lane_ring);
                }
            }
            if constexpr (SPLIT >= 0) {
                // the fields of this lane's run: whole bytes; a last partial byte has zero high bits
                constexpr uint32_t per_byte = 8 / (KB + 1);
                const uint32_t first = static_cast<uint32_t>(q) * kTurn + j * kRun;
                const uint32_t valid = first >= m ? 0u : (m - first < kRun ? m - first : kRun);
                for (uint32_t t = 0; t < valid; t += per_byte)
                    sm[(base + first + t) / per_byte] = static_cast<uint8_t>(packed >> (t * (KB + 1)));
            }
            ring_advance(st, cur_before);
            ring_flush(wp_before, st.wp, ring, chunk_slots, j);
        }
    }
    if constexpr (SPLIT >= 0) {
        if (least_rcp == 0.0f)
            atomicOr(&state->stale[slot_id.item], 1u);
    }
    const uint32_t len = kRunCap - st.wp;
    if (live) {
        // the incomplete group at the low end: word by word
        for (uint32_t p = st.wp; p < ((st.wp + 7) & ~7u) && p < kRunCap; ++p)
            chunk_slots[slot_word(j, p)] = ring[p & (kRingWords - 1)];
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
        // words of this workgroup: for the compaction's offsets (by group, and added up per 64 groups
        // and per tensor, so that a chunk's offset is a short sum) and for the host (the total)
        uint32_t total = 0;
        for (uint32_t i = 0; i < kEncThreads / kStates; ++i)
            total += group_chunk[i];
        group_words_all[group] = total;
        atomicAdd(&super_words_all[it.super_base + slot_id.wg / kSuperGroups], total);
        atomicAdd(&state->total[slot_id.item], static_cast<unsigned long long>(total));
    }
}

// ------------------------------------------------------------------------------------------
// Kernel 4: gather the runs from the workspace slots into the blob's word section and write the
// chunk offsets.  One wave per chunk.  The chunk's slot pieces are read with 128-bit loads and
// laid out in LDS as the 16 runs one after the other, shifted so that LDS and destination agree
// modulo 16 bytes; the chunk then leaves with 128-bit stores (2-byte stores only for the few
// words before the first and after the last 16-byte boundary, which neighbouring chunks share).
// A chunk's offset is the sum of the words of the groups before its own -- whole blocks of 64
// groups from the encoder's per-block sums, the rest group by group -- and of the chunks before it
// in its group.
// The launch usually follows the encoder's at once, before the host knows the stream's length, into
// the room the blob has: a tensor whose words do not fit that room, or whose kept table turned out
// stale, is left alone, and the host launches again once it has made room.  In that first launch
// (b.report) the first wave of each tensor also tells the host the length, and returns to zero what
// the next call needs at zero: the histogram bins and the other copy of the call state.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kCompactThreads = 256;

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(const CompressBatch b,
                                                                 const uint16_t *__restrict__ slots_all,
                                                                 const uint32_t *__restrict__ chunk_words_all,
                                                                 const uint32_t *__restrict__ group_words_all,
                                                                 const uint32_t *__restrict__ super_words_all,
                                                                 const CallState *__restrict__ state,
                                                                 uint32_t *__restrict__ counts_ws,
                                                                 CallState *__restrict__ state_next,
                                                                 uint32_t *__restrict__ super_next, uint32_t super_cap,
                                                                 uint32_t *__restrict__ all_done,
                                                                 HostRecord *__restrict__ record)
{
    const ItemSlot slot_id = item_of_workgroup<&CompressItem::compact_end>(b);
    const CompressItem &it = b.it[slot_id.item];
    const uint32_t n_chunks = it.n_chunks;
    const unsigned long long own_words = state->total[slot_id.item];
    const unsigned long long all_words = it.words_before + own_words;  // up to the end of this tile
    const uint32_t was_stale = state->stale[slot_id.item];
    if (b.report && slot_id.wg == 0 && threadIdx.x < 64) {
        const uint32_t lane = threadIdx.x;
        // every workgroup of the encoder launch has read the counts: the bins go back to zero
        if (!b.keep_counts)
            reinterpret_cast<uint4 *>(counts_ws + 256 * slot_id.item)[lane] = make_uint4(0, 0, 0, 0);
        // the other copy of the call state, for the call after this one (nobody is using it now)
        if (slot_id.item == 0) {
            for (uint32_t i = lane; i < sizeof(CallState) / 4; i += 64)
                reinterpret_cast<uint32_t *>(state_next)[i] = 0;
            for (uint32_t i = lane; i < super_cap; i += 64)
                super_next[i] = 0;
        }
        if (lane == 0) {
            if (n_chunks > 0) {
                it.offsets[n_chunks] = static_cast<uint32_t>(all_words);
                it.offsets[n_chunks + 1] = 0;
            }
            // The record is host memory the host polls.  Its words are written past the caches; once
            // they are acknowledged this tensor counts as reported, and the tensor reported last
            // writes the stamp, which therefore cannot overtake any of them.
            HostRecord::Item *mine = &record->item[slot_id.item];
            // (the words of this item alone: the host adds up the tiles of a tensor)
            __hip_atomic_store(&mine->total_words[0], static_cast<uint32_t>(own_words), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(&mine->total_words[1], static_cast<uint32_t>(own_words >> 32), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_SYSTEM);  // non-zero: too long for 32-bit offsets
            __hip_atomic_store(&mine->stale, was_stale, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            wait_for_memory_acks();
            if (atomicAdd(all_done, 1u) == b.count - 1) {
                *all_done = 0;
                __hip_atomic_store(&record->seq, b.seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
    }
    // (the same decision in all workgroups of the tensor)
    if (n_chunks == 0 || was_stale != 0 || all_words > it.words_cap || (all_words >> 32) != 0)
        return;
    const uint8_t *__restrict__ lens = it.lens;
    uint32_t *__restrict__ offsets = it.offsets;
    uint16_t *__restrict__ words = it.words;
    const uint16_t *__restrict__ slots = slots_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup * kStates * kRunCap;
    const uint32_t *__restrict__ chunk_words = chunk_words_all + static_cast<uint64_t>(it.group_base) * kChunksPerGroup;
    const uint32_t *__restrict__ group_words = group_words_all + it.group_base;
    const uint32_t *__restrict__ super_words = super_words_all + it.super_base;

    __shared__ __align__(16) uint16_t gathered[kCompactThreads / 64][kStates * kRunCap + 8];
    const uint32_t wave = threadIdx.x / 64, lane = threadIdx.x & 63;
    const uint32_t c = slot_id.wg * (kCompactThreads / 64) + wave;
    const bool live = c < n_chunks;   // (no early return: the workgroup meets at a barrier)
    constexpr uint32_t kRowsPerPass = 64 / kStates;  // slot rows (one piece per state) the wave reads at a time
    const uint32_t j = lane % kStates;  // the lane's state: lanes 64 apart in the piece loop keep it
    uint16_t *__restrict__ mine = gathered[wave];
    uint32_t total = 0, shift = 0;
    uint64_t at0 = 0;
    if (live) {
        const uint16_t *__restrict__ chunk_slots = slots + static_cast<uint64_t>(c) * kStates * kRunCap;
        // Slot pieces (8 words of one state) are taken row by row from the top of the slots down:
        // this lane reads, for its state j, rows lane / 16, lane / 16 + 4, ...  The top 8 rows (64
        // words per state: all of a run at up to 4 bits per symbol) are requested at once, before
        // the run lengths that say how much of them is needed have arrived.
        constexpr uint32_t kRows = kRunCap / 8, kAhead = 2;
        const uint32_t row0 = lane / kStates;
        uint4 ahead[kAhead];
#pragma unroll
        for (uint32_t k = 0; k < kAhead; ++k)
            ahead[k] = *reinterpret_cast<const uint4 *>(chunk_slots + slot_word(j, (kRows - 1 - (row0 + kRowsPerPass * k)) * 8));
        // run length of state j and its start inside the chunk (16-lane exclusive prefix)
        const uint32_t my_len = lens[c * kStates + j];
        uint32_t start = my_len;
#pragma unroll
        for (uint32_t d = 1; d < kStates; d <<= 1) {
            const uint32_t o = __shfl_up(start, d, kStates);
            if (j >= d)
                start += o;
        }
        total = __shfl(start, kStates - 1, kStates);
        start -= my_len;
        // words before this chunk: the whole blocks of 64 encoder groups before its group, the groups
        // before it in its block, the chunks before it in its group
        const uint32_t g = c / kChunksPerGroup, in_group = c % kChunksPerGroup;
        const uint32_t blocks = g / kSuperGroups, in_block = g % kSuperGroups;
        // (32-bit sums: the tensor's words, which fit the destination, are fewer than 2^32)
        uint32_t before = lane < in_block ? group_words[blocks * kSuperGroups + lane] : 0u;
        before += lane < in_group ? chunk_words[g * kChunksPerGroup + lane] : 0u;
        for (uint32_t i = lane; i < blocks; i += 64)
            before += super_words[i];
        at0 = it.words_before + wave_sum_u32(before);
        if (lane == 0)
            offsets[c] = static_cast<uint32_t>(at0);
        shift = static_cast<uint32_t>(at0 & 7u);

        const uint32_t first_pos = kRunCap - my_len;   // position of the run's first word in its slot
        const uint32_t first_piece = first_pos >> 3;   // rows below it hold nothing of this state
        for (uint32_t k = 0;; ++k) {
            const uint32_t row = row0 + kRowsPerPass * k;
            if (row >= kRows || kRows - 1 - row < first_piece)
                break;
            const uint32_t piece = kRows - 1 - row;
            uint4 v;
            if (k < kAhead)
                v = k == 0 ? ahead[0] : ahead[1];
            else
                v = *reinterpret_cast<const uint4 *>(chunk_slots + slot_word(j, piece * 8));
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (uint32_t t = 0; t < 8; ++t) {
                const uint32_t pos = piece * 8 + t;
                if (pos >= first_pos)
                    mine[shift + start + (pos - first_pos)] = static_cast<uint16_t>(w[t >> 1] >> (16 * (t & 1)));
            }
        }
    }
    __syncthreads();
    if (!live)
        return;
    uint16_t *__restrict__ out = words + at0;
    const uint32_t head = total < ((8 - shift) & 7u) ? total : ((8 - shift) & 7u);  // words up to the 16-byte boundary
    if (lane < head)
        out[lane] = mine[shift + lane];
    const uint32_t n_body = (total - head) / 8;
    for (uint32_t p = lane; p < n_body; p += 64)
        *reinterpret_cast<uint4 *>(out + head + 8 * p) = *reinterpret_cast<const uint4 *>(mine + shift + head + 8 * p);
    const uint32_t tail = total - head - 8 * n_body;
    if (lane < tail)
        out[head + 8 * n_body + lane] = mine[shift + head + 8 * n_body + lane];
}

}  // namespace nz
