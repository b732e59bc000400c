// Fused rANS decode + merge kernels of the NeuZip codec for gfx950 (single tensor and batch).
#pragma once

#include <type_traits>

#include "neuzip_format.h"
#include "neuzip_compress_kernels.h"

namespace nz {

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

// binary16 words: the decoded symbol is the word's upper byte, the field its lower byte.
__device__ __forceinline__ uint32_t merge_pair_half(uint64_t fields, int pair, uint32_t entry_lo, uint32_t entry_hi)
{
    const uint32_t sym = __builtin_amdgcn_perm(entry_hi, entry_lo, 0x0c040c00u);  // [0, symbol_hi, 0, symbol_lo]
    const uint32_t half = static_cast<uint32_t>(fields >> (32 * (pair >> 1)));
    // [symbol_hi, field_hi, symbol_lo, field_lo]
    return __builtin_amdgcn_perm(sym, half, (pair & 1) ? 0x06030402u : 0x06010400u);
}

// Lossy tensors with one or no mantissa bit: spreading a few field bits over two bf16 words costs more
// vector instructions than the decoding itself, so it is looked up instead.  A small LDS table, filled
// by the workgroup, maps
//   k = 1: a byte of field bits (four elements, s m per element) to the sign and mantissa bits of two
//          dwords of output (256 entries of 8 bytes);
//   k = 0: a nibble of sign bits (four elements) to the sign bits of two dwords (16 entries).
// A turn's 8 elements take two reads; few distinct addresses are in flight at a time for k = 0.
template <int KB>
constexpr uint32_t kSpreadEntries = KB == 1 ? 256u : (KB == 0 ? 16u : 1u);
template <int KB>
constexpr uint32_t kStageBytesOf = kStageBytes - (KB == 1 ? 2048u : (KB == 0 ? 128u : 0u));  // same LDS in all

template <int KB>
__device__ __forceinline__ uint2 spread_entry(uint32_t i)
{
    if constexpr (KB == 1) {
        // nibble s1 m1 s0 m0: m0 -> bit 6, s0 -> 15, m1 -> 22, s1 -> 31
        auto one = [](uint32_t f) { return ((f & 1u) << 6) | ((f & 2u) << 14) | ((f & 4u) << 20) | ((f & 8u) << 28); };
        return make_uint2(one(i & 0xFu), one(i >> 4));
    } else {
        // signs s3 s2 s1 s0: even elements -> bit 15, odd ones -> bit 31
        return make_uint2(((i & 1u) << 15) | ((i & 2u) << 30), ((i & 4u) << 13) | ((i & 8u) << 28));
    }
}

// The four output dwords of a turn (k = 1 or 0) from its field bits, the eight slot-table entries
// that decoded its exponents, and the table above.
template <int KB>
__device__ __forceinline__ uint4 merge_turn_small(uint64_t fields, const uint32_t (&e)[8], const uint2 *__restrict__ spread)
{
    static_assert(KB == 1 || KB == 0, "wider fields are merged arithmetically");
    const uint32_t v = static_cast<uint32_t>(fields);
    const uint2 a = spread[KB == 1 ? (v & 0xFFu) : (v & 0xFu)];
    const uint2 b = spread[KB == 1 ? ((v >> 8) & 0xFFu) : ((v >> 4) & 0xFu)];
    uint4 o;
    o.x = (__builtin_amdgcn_perm(e[1], e[0], 0x0c040c00u) << 7) | a.x;
    o.y = (__builtin_amdgcn_perm(e[3], e[2], 0x0c040c00u) << 7) | a.y;
    o.z = (__builtin_amdgcn_perm(e[5], e[4], 0x0c040c00u) << 7) | b.x;
    o.w = (__builtin_amdgcn_perm(e[7], e[6], 0x0c040c00u) << 7) | b.y;
    return o;
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
                                              uint32_t block, uint64_t first_elem)  // block: log2 of the block size
{
    uint64_t f = load_fields<KB>(sm, first_elem);
    if constexpr (NORM)
        f |= static_cast<uint64_t>(coef[first_elem >> block]) << 32;  // `block` is log2 of the block size here
    return f;
}

// bf16(stored * c) on the two halves of a merged dword: two multiplies, one packed conversion;
// a NaN keeps its bits and gets the quiet bit, as in denormalise_word
__device__ __forceinline__ uint32_t denormalise_pair(uint32_t d, float c)
{
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
    const f32x2_t prod = {__fmul_rn(__uint_as_float(d << 16), c), __fmul_rn(__uint_as_float(d & 0xFFFF0000u), c)};
    uint32_t r = __builtin_bit_cast(uint32_t, __builtin_convertvector(prod, bf16x2_t));
    // c lies in [1, 2): a product is a NaN only if the stored word is one; one compare finds either
    if (__builtin_expect(__builtin_isunordered(prod[0], prod[1]), 0)) {
        if (bf16_is_nan(d & 0xFFFFu))
            r = (r & 0xFFFF0000u) | (d & 0xFFFFu) | 0x40u;
        if (bf16_is_nan(d >> 16))
            r = (r & 0x0000FFFFu) | (d & 0xFFFF0000u) | 0x400000u;
    }
    return r;
}

// UPD: the words written are the decoded weights after the update with the gradient `grad` (bf16
// words, same indexing as the output) and the rate lr.  HALF: the tensor is binary16.
template <int KB, bool LONE, bool NORM, bool STREAM, bool UPD, bool HALF, class WordSrc>
__device__ __forceinline__ void walk_state(const uint32_t *__restrict__ lut, const uint2 *__restrict__ spread,
                                           const WordSrc &src, uint32_t lone,
                                           uint32_t &x, uint32_t &wp, const uint8_t *__restrict__ sm,
                                           const uint8_t *__restrict__ coef, uint32_t block,
                                           uint64_t (&fields)[KB == 7 ? kTurnGroupStream : kTurnGroup],
                                           uint16_t *__restrict__ out,
                                           uint64_t base, uint32_t m, uint32_t j,
                                           const uint16_t *__restrict__ grad = nullptr, float lr = 0.0f)
{
    static_assert(!(UPD || HALF) || (KB == 7 && !NORM), "trained weights and binary16 tensors are lossless only");
    static_assert(!(UPD && HALF), "only bf16 weights are trained");
    // `fields` arrives holding the field bits of the state's first turns (full chunks only)
    constexpr uint32_t kGroup = (STREAM && KB == 7 && !UPD) ? kTurnGroupStream : kTurnGroup;
    uint32_t next = LONE ? 0u : src.peek(wp);
    if (m == kChunk) {
        uint4 *out4 = reinterpret_cast<uint4 *>(out + base) + j;
        const uint64_t first = base + j * kRun;
        // the gradients of a turn: the 128 bits the lane's output words come from
        const uint4 *grad4 = UPD ? reinterpret_cast<const uint4 *>(grad + base) + j : nullptr;
        uint4 grads[kGroup];
        if constexpr (UPD) {
#pragma unroll
            for (uint32_t r = 0; r < kGroup; ++r)
                grads[r] = grad4[r * kStates];
        }
        // Turns are taken in groups: the field loads of the next group are issued together before
        // the current group is decoded, and the group's 128-bit stores leave back to back, so
        // each state keeps several memory requests in flight and a chunk is written in bursts of
        // kGroup * 256 contiguous bytes.
        for (uint32_t q0 = 0; q0 < kTurns; q0 += kGroup) {
            uint64_t fields_next[kGroup];
            // the last group re-reads its own fields (stays in bounds)
            const uint32_t qn = q0 + kGroup < kTurns ? q0 + kGroup : q0;
#pragma unroll
            for (uint32_t r = 0; r < kGroup; ++r)
                fields_next[r] = load_turn<KB, NORM>(sm, coef, block, first + (qn + r) * kTurn);
            uint4 grads_next[kGroup];
            if constexpr (UPD) {
#pragma unroll
                for (uint32_t r = 0; r < kGroup; ++r)
                    grads_next[r] = grad4[(qn + r) * kStates];
            }
            uint4 o[kGroup];
#pragma unroll
            for (uint32_t r = 0; r < kGroup; ++r) {
                uint32_t e[8];
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    e[t] = LONE ? lone : rans_get(lut, x, wp, next, src);
                if constexpr (HALF) {
                    o[r].x = merge_pair_half(fields[r], 0, e[0], e[1]);
                    o[r].y = merge_pair_half(fields[r], 1, e[2], e[3]);
                    o[r].z = merge_pair_half(fields[r], 2, e[4], e[5]);
                    o[r].w = merge_pair_half(fields[r], 3, e[6], e[7]);
                } else if constexpr (KB <= 1) {
                    o[r] = merge_turn_small<KB>(fields[r], e, spread);
                } else {
                    o[r].x = merge_pair<KB>(fields[r], 0, e[0], e[1]);
                    o[r].y = merge_pair<KB>(fields[r], 1, e[2], e[3]);
                    o[r].z = merge_pair<KB>(fields[r], 2, e[4], e[5]);
                    o[r].w = merge_pair<KB>(fields[r], 3, e[6], e[7]);
                }
                if constexpr (NORM) {
                    const float c = coefficient(static_cast<uint32_t>(fields[r] >> 32) & 0x7Fu);
                    o[r].x = denormalise_pair(o[r].x, c);
                    o[r].y = denormalise_pair(o[r].y, c);
                    o[r].z = denormalise_pair(o[r].z, c);
                    o[r].w = denormalise_pair(o[r].w, c);
                }
                if constexpr (UPD) {
                    o[r].x = update_pair(o[r].x, grads[r].x, lr);
                    o[r].y = update_pair(o[r].y, grads[r].y, lr);
                    o[r].z = update_pair(o[r].z, grads[r].z, lr);
                    o[r].w = update_pair(o[r].w, grads[r].w, lr);
                }
            }
#pragma unroll
            for (uint32_t r = 0; r < kGroup; ++r) {
                uint4 *dst = &out4[(q0 + r) * kStates];
                if constexpr (STREAM) {
                    // a tensor larger than the last-level cache: non-temporal stores
                    __builtin_nontemporal_store(o[r].x, &dst->x);
                    __builtin_nontemporal_store(o[r].y, &dst->y);
                    __builtin_nontemporal_store(o[r].z, &dst->z);
                    __builtin_nontemporal_store(o[r].w, &dst->w);
                } else {
                    *dst = o[r];
                }
                fields[r] = fields_next[r];
                if constexpr (UPD)
                    grads[r] = grads_next[r];
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
                uint32_t u = HALF ? (sym << 8) | field
                                  : ((field >> KB) << 15) | (sym << 7) | ((field & ((1u << KB) - 1u)) << (7 - KB));
                if constexpr (NORM)
                    u = denormalise_word(u, coefficient(coef[g >> block]));
                if constexpr (UPD)
                    u = update_word(u, grad[g], lr);
                out[g] = static_cast<uint16_t>(u);
            }
        }
    }
}

// The same walk for a binary32 tensor (lossless only): the decoded bf16 word is the upper half
// of the element and the lower half comes from the raw plane, so a turn reads 16 B of lower
// halves next to its 8 B of fields and writes two 128-bit pieces.
template <bool LONE, bool STREAM, class WordSrc>
__device__ __forceinline__ void walk_state_wide(const uint32_t *__restrict__ lut, const WordSrc &src, uint32_t lone,
                                                uint32_t &x, uint32_t &wp, const uint8_t *__restrict__ sm,
                                                const uint16_t *__restrict__ low, uint32_t *__restrict__ out,
                                                uint64_t base, uint32_t m, uint32_t j)
{
    constexpr uint32_t kGroup = kTurnGroup;
    uint32_t next = LONE ? 0u : src.peek(wp);
    if (m == kChunk) {
        // where this lane stores: its own pieces 2j and 2j + 1 of a turn's 32, or, after the exchange
        // described below, pieces (j / 8) * 16 + j % 8 and 8 further
        uint4 *out4 = reinterpret_cast<uint4 *>(out + base) + (STREAM ? (j >> 3) * 16 + (j & 7) : 2 * j);
        const uint32_t lane = threadIdx.x & 63u;
        const uint32_t pull[2] = {((lane & ~7u) + ((lane & 7u) >> 1)) * 4u, ((lane & ~7u) + 4u + ((lane & 7u) >> 1)) * 4u};
        const bool odd = lane & 1u;
        const uint4 *low4 = reinterpret_cast<const uint4 *>(low + base) + j;
        const uint64_t first = base + j * kRun;
        uint64_t fields[kGroup];
        uint4 lows[kGroup];
#pragma unroll
        for (uint32_t r = 0; r < kGroup; ++r) {
            fields[r] = load_fields<7>(sm, first + r * kTurn);
            lows[r] = low4[r * kStates];
        }
        for (uint32_t q0 = 0; q0 < kTurns; q0 += kGroup) {
            uint64_t fields_next[kGroup];
            uint4 lows_next[kGroup];
            const uint32_t qn = q0 + kGroup < kTurns ? q0 + kGroup : q0;  // the last group re-reads its own
#pragma unroll
            for (uint32_t r = 0; r < kGroup; ++r) {
                fields_next[r] = load_fields<7>(sm, first + (qn + r) * kTurn);
                lows_next[r] = low4[(qn + r) * kStates];
            }
            uint4 o[2 * kGroup];
#pragma unroll
            for (uint32_t r = 0; r < kGroup; ++r) {
                uint32_t e[8];
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    e[t] = LONE ? lone : rans_get(lut, x, wp, next, src);
                const uint32_t h[4] = {merge_pair<7>(fields[r], 0, e[0], e[1]), merge_pair<7>(fields[r], 1, e[2], e[3]),
                                       merge_pair<7>(fields[r], 2, e[4], e[5]), merge_pair<7>(fields[r], 3, e[6], e[7])};
                const uint32_t l[4] = {lows[r].x, lows[r].y, lows[r].z, lows[r].w};
                // element = upper half << 16 | lower half: this lane's 8 elements as 16-byte pieces 2j, 2j + 1
                // of the turn's 32
                uint32_t mine[2][4];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    mine[d >> 1][2 * (d & 1)] = __builtin_amdgcn_perm(h[d], l[d], 0x05040100u);
                    mine[d >> 1][2 * (d & 1) + 1] = __builtin_amdgcn_perm(h[d], l[d], 0x07060302u);
                }
                // A 128-bit store of piece 2j by every lane leaves every other 16 bytes of a cache line
                // to a second instruction.  In the cache that is harmless, but once the tensor streams
                // to HBM such half-written lines cost a third of the store rate.  There the 8 lanes of
                // an octet trade pieces: store `half` of lane t writes piece 8 * half + t of the
                // octet's 16, which lane 4 * half + t / 2 holds (its first piece for even t), and each
                // store instruction covers whole 128-byte lines.  (The 16 lane exchanges per turn cost
                // 20 % of the rate of a cache-resident tensor, which therefore keeps the plain stores.)
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    uint32_t got[4];
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        if constexpr (STREAM) {
                            const uint32_t first = __builtin_amdgcn_ds_bpermute(static_cast<int>(pull[half]),
                                                                                static_cast<int>(mine[0][d]));
                            const uint32_t second = __builtin_amdgcn_ds_bpermute(static_cast<int>(pull[half]),
                                                                                 static_cast<int>(mine[1][d]));
                            got[d] = odd ? second : first;
                        } else {
                            got[d] = mine[half][d];
                        }
                    }
                    o[2 * r + half] = make_uint4(got[0], got[1], got[2], got[3]);
                }
            }
#pragma unroll
            for (uint32_t r = 0; r < kGroup; ++r) {
#pragma unroll
                for (uint32_t half = 0; half < 2; ++half) {
                    uint4 *dst = &out4[(q0 + r) * kStates * 2 + half * (STREAM ? 8 : 1)];
                    const uint4 v = o[2 * r + half];
                    if constexpr (STREAM) {
                        __builtin_nontemporal_store(v.x, &dst->x);
                        __builtin_nontemporal_store(v.y, &dst->y);
                        __builtin_nontemporal_store(v.z, &dst->z);
                        __builtin_nontemporal_store(v.w, &dst->w);
                    } else {
                        *dst = v;
                    }
                }
                fields[r] = fields_next[r];
                lows[r] = lows_next[r];
            }
        }
    } else {
        // ragged last chunk: element by element
        for (uint32_t q = 0; q < kTurns; ++q) {
            for (uint32_t t = 0; t < kRun; ++t) {
                const uint32_t i = q * kTurn + j * kRun + t;
                if (i >= m)
                    continue;
                const uint32_t sym = (LONE ? lone : rans_get(lut, x, wp, next, src)) & 0xFFu;
                const uint64_t g = base + i;
                const uint32_t field = sm[g];
                out[g] = ((field >> 7) << 31) | (sym << 23) | ((field & 0x7Fu) << 16) | low[g];
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
    const uint16_t *low;  // lower halves (binary32 blobs only)
    const uint16_t *grad; // gradient of the weight, bf16 words (update variant only)
    float lr;             // learning rate (update variant only)
    void *out;            // bf16 words, or binary32 words for a binary32 blob
    uint32_t *status;
    uint64_t n;
    uint32_t n_chunks;
    uint32_t block;       // 0: no block-wise normalisation
    uint32_t stream_out;  // non-zero: the output does not fit the last-level cache, store non-temporally
    uint32_t wg_end;      // batches: first workgroup index after this tensor's
};

// Decodes the chunks of workgroup `wg` of one tensor.
// MODE: what is written -- the decoded bf16 words (kPlain), binary32 words joined with their
// lower halves (kWide), the decoded weights after the update of the backward loop (kUpdate), or
// binary16 words (kHalf).
enum DecodeMode { kPlain = 0, kWide = 1, kUpdate = 2, kHalf = 3 };

template <int KB, bool NORM, int MODE>
__device__ __forceinline__ void decode_workgroup(const TableBlock *__restrict__ tb,
                                                 const uint32_t *__restrict__ offsets,
                                                 const uint32_t *__restrict__ states,
                                                 const uint8_t *__restrict__ lens,
                                                 const uint16_t *__restrict__ words,
                                                 const uint8_t *__restrict__ sm,
                                                 const uint8_t *__restrict__ coef, uint32_t block,
                                                 const uint16_t *__restrict__ low, void *__restrict__ out_any,
                                                 const uint16_t *__restrict__ grad, float lr, bool stream_out,
                                                 uint64_t n, uint32_t n_chunks, uint32_t *__restrict__ status,
                                                 uint32_t wg, uint32_t *__restrict__ lut, uint8_t *__restrict__ stage,
                                                 uint2 *__restrict__ spread)
{
    constexpr bool WIDE = MODE == kWide, UPD = MODE == kUpdate, HALF = MODE == kHalf;
    static_assert(MODE == kPlain || (KB == 7 && !NORM), "binary32 blobs and trained weights are lossless only");
    block = 31u - static_cast<uint32_t>(__clz(static_cast<int>(block | 1u)));  // a power of two: from here on its log2
    uint16_t *__restrict__ out = static_cast<uint16_t *>(out_any);
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
    constexpr uint32_t kPreload = KB == 7 ? kTurnGroupStream : kTurnGroup;  // the largest group a variant uses
    uint64_t fields0[kPreload];
#pragma unroll
    for (uint32_t r = 0; r < kPreload; ++r)
        fields0[r] = !WIDE && m == kChunk ? load_turn<KB, NORM>(sm, coef, block, base + r * kTurn + j * kRun) : 0;
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
    const bool staged = stage_len + 16 <= kStageBytesOf<KB>;  // room for the one-word look-ahead
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
    if constexpr (KB <= 1) {
        for (uint32_t i = tid; i < kSpreadEntries<KB>; i += threads)
            spread[i] = spread_entry<KB>(i);
    }
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

    // (the streaming and the cached store variants are separate instantiations: merged into one
    // loop the compiler drops the non-temporal hint)
    uint32_t wp = 0, wp_begin = 0;
    if constexpr (WIDE) {
        uint32_t *out32 = static_cast<uint32_t *>(out_any);
        if (lone < 256) {
            if (stream_out)
                walk_state_wide<true, true>(lut, NoWords{}, lone, x, wp, sm, low, out32, base, m, j);
            else
                walk_state_wide<true, false>(lut, NoWords{}, lone, x, wp, sm, low, out32, base, m, j);
        } else if (staged) {
            wp = wp_begin = static_cast<uint32_t>(run_byte - aligned0);
            if (stream_out)
                walk_state_wide<false, true>(lut, LdsWords{stage}, 0u, x, wp, sm, low, out32, base, m, j);
            else
                walk_state_wide<false, false>(lut, LdsWords{stage}, 0u, x, wp, sm, low, out32, base, m, j);
        } else {
            const GlobalWords direct{reinterpret_cast<const uint8_t *>(words) + run_byte};
            if (stream_out)
                walk_state_wide<false, true>(lut, direct, 0u, x, wp, sm, low, out32, base, m, j);
            else
                walk_state_wide<false, false>(lut, direct, 0u, x, wp, sm, low, out32, base, m, j);
        }
    } else if (lone < 256) {
        if (stream_out)
            walk_state<KB, true, NORM, true, UPD, HALF>(lut, spread, NoWords{}, lone, x, wp, sm, coef, block, fields0, out, base, m, j, grad, lr);
        else
            walk_state<KB, true, NORM, false, UPD, HALF>(lut, spread, NoWords{}, lone, x, wp, sm, coef, block, fields0, out, base, m, j, grad, lr);
    } else if (staged) {
        wp = wp_begin = static_cast<uint32_t>(run_byte - aligned0);
        if (stream_out)
            walk_state<KB, false, NORM, true, UPD, HALF>(lut, spread, LdsWords{stage}, 0u, x, wp, sm, coef, block, fields0, out, base, m,
                                              j, grad, lr);
        else
            walk_state<KB, false, NORM, false, UPD, HALF>(lut, spread, LdsWords{stage}, 0u, x, wp, sm, coef, block, fields0, out, base, m,
                                               j, grad, lr);
    } else {
        // the runs of this workgroup's chunks did not fit the LDS window (more than ~4 bits per
        // symbol): read the words straight from the blob
        const GlobalWords direct{reinterpret_cast<const uint8_t *>(words) + run_byte};
        if (stream_out)
            walk_state<KB, false, NORM, true, UPD, HALF>(lut, spread, direct, 0u, x, wp, sm, coef, block, fields0, out, base, m, j, grad, lr);
        else
            walk_state<KB, false, NORM, false, UPD, HALF>(lut, spread, direct, 0u, x, wp, sm, coef, block, fields0, out, base, m, j, grad, lr);
    }
    // a well-formed run is consumed exactly and leaves the state where the encoder started
    if (x != kRansL || wp - wp_begin != 2 * len)
        atomicOr(status, 1u);
}

template <int KB, bool NORM, int MODE = kPlain>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(const DecodeArgs a)
{
    __shared__ __align__(16) uint32_t lut[kM];
    __shared__ __align__(16) uint8_t stage[kStageBytesOf<KB>];
    __shared__ uint2 spread[kSpreadEntries<KB>];
    decode_workgroup<KB, NORM, MODE>(a.tb, a.offsets, a.states, a.lens, a.words, a.sm, a.coef, a.block, a.low, a.out,
                                     a.grad, a.lr, a.stream_out != 0, a.n, a.n_chunks, a.status, blockIdx.x, lut, stage,
                                     spread);
}

// Several tensors in one launch (a layer's weights): workgroups [t[i-1].wg_end, t[i].wg_end)
// belong to tensor i.  Small tensors, which alone cannot fill the chip, overlap with the others.
struct BatchArgs {
    DecodeArgs t[kBatchMax];
    uint32_t count;
};

template <int KB, bool NORM, int MODE = kPlain>
__global__ __launch_bounds__(kDecThreads) void decode_batch_kernel(const BatchArgs b)
{
    __shared__ __align__(16) uint32_t lut[kM];
    __shared__ __align__(16) uint8_t stage[kStageBytesOf<KB>];
    __shared__ uint2 spread[kSpreadEntries<KB>];
    uint32_t i = 0, first = 0;
    while (i + 1 < b.count && blockIdx.x >= b.t[i].wg_end) {
        first = b.t[i].wg_end;
        ++i;
    }
    const DecodeArgs &a = b.t[i];
    decode_workgroup<KB, NORM, MODE>(a.tb, a.offsets, a.states, a.lens, a.words, a.sm, a.coef, a.block, a.low, a.out,
                                     a.grad, a.lr, a.stream_out != 0, a.n, a.n_chunks, a.status, blockIdx.x - first, lut,
                                     stage, spread);
}

// ------------------------------------------------------------------------------------------
// Measurement aid: the decoder's memory traffic without its arithmetic, in the decoder's own launch
// shape.  A workgroup of 512 lanes owns 32 chunks of 8 KB of output and holds the decoder's LDS (so the
// same 16 waves per CU are resident); it first copies its share of the "word" input into LDS with
// 128-bit loads behind one barrier; then lane (chunk, state) reads FW bytes of "field" input and writes
// 16 bytes per turn, 256 bytes apart, turns taken four at a time with the next four field loads in
// flight, non-temporal stores for outputs beyond the last-level cache -- the decoder's instructions
// with nothing between them.  What it reaches is the ceiling for a decoder with this access pattern on
// this machine; the decoder's own rate is reported against it.
// ------------------------------------------------------------------------------------------
template <int FW, bool STREAM>
__global__ __launch_bounds__(kDecThreads) void stream_probe_kernel(const uint8_t *__restrict__ fields,
                                                                   const uint4 *__restrict__ words, uint32_t word_vecs_per_wg,
                                                                   uint4 *__restrict__ out, uint32_t n_chunks,
                                                                   uint32_t *__restrict__ sink)
{
    __shared__ __align__(16) uint32_t lut[kM];
    __shared__ __align__(16) uint8_t stage[kStageBytes];
    const uint32_t tid = threadIdx.x, c = blockIdx.x * kDecChunksPerWg + tid / kStates, j = tid % kStates;
    const uint4 *from = words + static_cast<uint64_t>(blockIdx.x) * word_vecs_per_wg;
    for (uint32_t i = tid; i < word_vecs_per_wg; i += kDecThreads)
        reinterpret_cast<uint4 *>(stage)[i % (kStageBytes / 16)] = from[i];
    lut[tid] = tid;
    __syncthreads();
    uint32_t acc = lut[(tid * 7u) % kM] ^ reinterpret_cast<const uint32_t *>(stage)[tid];
    if (c >= n_chunks)
        return;
    typedef typename std::conditional<FW == 8, uint2, typename std::conditional<FW == 4, uint32_t,
            typename std::conditional<FW == 2, uint16_t, uint8_t>::type>::type>::type field_t;
    const field_t *f = reinterpret_cast<const field_t *>(fields + static_cast<uint64_t>(c) * (kTurns * kStates * FW)) + j;
    uint4 *o = out + static_cast<uint64_t>(c) * (kChunk / 8) + j;
    constexpr uint32_t kBurst = kTurnGroupStream;
    field_t now[kBurst];
#pragma unroll
    for (uint32_t r = 0; r < kBurst; ++r)
        now[r] = f[r * kStates];
    for (uint32_t q = 0; q < kTurns; q += kBurst) {
        field_t next[kBurst];
        const uint32_t qn = q + kBurst < kTurns ? q + kBurst : q;
#pragma unroll
        for (uint32_t r = 0; r < kBurst; ++r)
            next[r] = f[(qn + r) * kStates];
#pragma unroll
        for (uint32_t r = 0; r < kBurst; ++r) {
            uint32_t lo, hi;
            if constexpr (FW == 8) {
                lo = now[r].x;
                hi = now[r].y;
            } else {
                lo = now[r];
                hi = q;
            }
            const uint4 w = make_uint4(lo, hi, acc, q + r);
            uint4 *dst = &o[(q + r) * kStates];
            if constexpr (STREAM) {
                __builtin_nontemporal_store(w.x, &dst->x);
                __builtin_nontemporal_store(w.y, &dst->y);
                __builtin_nontemporal_store(w.z, &dst->z);
                __builtin_nontemporal_store(w.w, &dst->w);
            } else {
                *dst = w;
            }
            now[r] = next[r];
        }
    }
    if (acc == 0x9E3779B9u)  // keeps the LDS reads alive; practically never taken
        atomicOr(sink, 1u);
}

}  // namespace nz
