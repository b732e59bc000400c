// Format constants and the device-side structures shared by the compression and decompression
// kernels of the NeuZip codec (see neuzip.hip for the stream format).
#pragma once

#include <hip/hip_runtime.h>
#include <cstddef>
#include <cstdint>
#include "neuzip.h"

namespace nz {

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
// Turns (of 8 symbols per state) whose loads and stores are issued together: 2 for tensors that
// live in the last-level cache and for the lossy widths, 4 for lossless tensors that stream
// through HBM (more bytes in flight; measured +2-3 % there, -6 % on cache-resident sizes and
// -7 % on the lossy widths).
constexpr uint32_t kTurnGroup = 2;
constexpr uint32_t kTurnGroupStream = 4;
static_assert(kTurns % kTurnGroup == 0 && kTurns % kTurnGroupStream == 0, "a chunk is a whole number of turn groups");


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

// Per-symbol encoder constants (16 bytes, one ds_read_b128), derived by every encoder workgroup from
// the frequencies and cumulative frequencies of the tensor's table.
//   The step is x <- (x / f) * M + (x mod f) + cum = q * (M - f) + x + cum with q = floor(x / f).
//   limit_cum: the state is renormalised before the step when x >= f << 20, so q < 2^20.  f << 20
//   has no bits in its lower half, so the test compares the upper halves only (x >> 16 against
//   f << 4) and the lower half of the same dword carries cum (both halves are read through the
//   sub-dword operand selects of the compare and the add, without an instruction to extract them).
//   rcp: a float slightly below 1/f, (1/f)(1 - 2^-21).  float(x) * rcp, truncated, is q or q - 1
//   (three roundings of 2^-24 cannot overcome the 2^-21 bias, and q * 1.5 * 2^-21 < 1); one
//   compare of the remainder against f settles it.  All of this runs at full VALU rate, unlike a
//   32-bit multiply-high.  The quotient is formed negated (the sign rides on the float multiply),
//   so that the remainder x - q f and the new state are one 24-bit multiply-add each:
//   r = (-q) f + x, x' = (-q)(f - M) + x (+ cum).
struct EncSym {
    float rcp;
    uint32_t limit_cum;  // f << 20 | cum (upper half 0xFFFF: never renormalises)
    uint32_t f;
    int32_t neg_cmpl;    // f - M
};

// ------------------------------------------------------------------------------------------
// Compression works on a batch of up to 8 tensors that share mantissa_bits and block size (the
// weights of a layer): every kernel of the pipeline is launched once for the whole batch, so
// tensors too small to fill the chip overlap with the others.  A single tensor is a batch of one.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kBatchMax = 8;

struct CompressItem {
    const void *src;       // bf16 words, or binary32 words when the batch is of that type
    uint64_t n;
    // A tensor whose encoder slots would exceed the workspace limit goes through the encoder and the
    // compaction in tiles of whole chunks.  A tile is an item of its own whose pointers (source, states,
    // lens, offsets, fields, ...) start at the tile's first chunk and whose n is the tile's elements;
    // table_n is the element count of the whole tensor (the table is the tensor's), words_before the
    // words of the tiles before it (its chunk offsets and its place in the word section start there).
    uint64_t table_n;
    uint64_t words_before;
    TableBlock *tb;
    uint32_t *offsets;
    uint32_t *states;
    uint8_t *lens;
    uint8_t *sm;
    uint8_t *coef;
    uint16_t *low;         // binary32 tensors: the plane of lower halves
    const uint16_t *grad;  // weight step fused into the encoder: the gradient (src is then written too)
    uint16_t *words;       // the blob's word section (the compaction's destination) ...
    uint64_t words_cap;    // ... and the words it has room for
    uint32_t n_chunks;
    uint32_t block;        // 0: no block-wise normalisation
    uint32_t guard;        // exponents this far outside the occupied range keep f = 1 in the table
    uint32_t group_base;   // first encoder group (16 chunks) of this tensor in the workspace arrays
    uint32_t super_base;   // first entry of this tensor in the array of words per 64 encoder groups
    uint32_t hist_end;     // first workgroup after this tensor's in the histogram launch
    uint32_t enc_end;      // ... in the encode launch
    uint32_t compact_end;  // ... in the compaction launch
};

struct CompressBatch {
    CompressItem it[kBatchMax];
    uint32_t count;
    uint32_t seq;  // stamp of this call
    float lr;      // learning rate of the fused weight step
    uint32_t keep_new;  // fused weight step: write the new weight back over the source
    uint32_t report;    // compaction launch: also report the stream lengths to the host and tidy the workspace
    uint32_t keep_counts;  // ... but leave the histogram bins: further tiles of the tensor need them
};

// What the encoder workgroups of a call add up for the compaction and for the host, in the workspace.
// There are two copies, used by alternate calls: while one call's compaction reads its copy, it
// returns the other one (and the histogram bins) to zero for the call that follows.
struct CallState {
    unsigned long long total[kBatchMax];  // words of tensor i
    uint32_t stale[kBatchMax];            // recompression met an exponent without room in tensor i's table
    uint32_t pad[8];
};
constexpr uint32_t kSuperGroups = 64;  // encoder groups whose words are also added up in one entry

// Host-visible results of one compress call (pinned host memory the kernels write directly).
struct HostRecord {
    uint32_t seq;  // stamp of the compress call whose results are complete (written last)
    uint32_t pad[3];  // (the items, and the arrays in them, are 16-byte aligned)
    struct Item {
        uint32_t total_words[2];
        uint32_t stale;    // recompression only: an exponent had no room in the blob's table
        uint32_t pad;
        uint32_t counts[256];
        uint16_t freq[256];
    } item[kBatchMax];
};
static_assert(sizeof(HostRecord::Item) % 16 == 0 && offsetof(HostRecord, item) % 16 == 0, "whole-wave 128-bit stores");

}  // namespace nz
