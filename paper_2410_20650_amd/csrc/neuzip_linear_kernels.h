// Linear layer on a compressed weight for gfx950: the rANS decoder feeding the matrix cores.
//
// Sec. 2.2, compressed forward pass:  W_hat <- decompress(c_l);  x_l <- W_hat x_{l-1} + b_l.
// Here the two steps are one kernel: the decoded and merged bf16 words of a state's turn (8
// neighbouring weights of one row) are, as they stand in the lane's registers, one lane's share
// of the B operand of v_mfma_f32_16x16x32_bf16, so W_hat is never written to memory.
//
// Operand shapes of that instruction (wave64):  A is 16 x 32 (lane l holds row l % 16,
// k = 8 * (l / 16) .. + 7),  B is 32 x 16 (lane l holds column l % 16, same k),  D is 16 x 16
// float (lane l holds column l % 16, rows 4 * (l / 16) .. + 3).  A = 16 tokens of the
// activations, B = 16 rows of the weight, both over the same 32 input features.
//
// Lane assignment.  A workgroup of 512 threads walks 32 chunks as two groups of 16.  In a group,
// wave sq (0..3) and lane l own state j = 4 * sq + l / 16 of chunk number l % 16 of the group.
// At turn t that state holds the weights at flat index chunk * 4096 + t * 128 + j * 8 .. + 7, so
// a wave holds, for 16 chunks, the 32 neighbouring input features t * 128 + sq * 32 .. + 31:
// exactly a B operand, provided the 16 chunks sit at the same input-feature offset.  Chunks that
// are `stride` = in_features / gcd(in_features, 4096) apart do (stride * 4096 is a whole number of
// rows), so a group is chunks first + stride * (0..15); its columns are rows `rstep` apart.
// Every wave accumulates its own share of the input features of a row piece and adds the
// partial sums to y with float atomics when the row ends (y starts as the bias, or zero).
//
// Two forms, template parameter COLS.  COLS = 16 is the above.  COLS = 32 uses
// v_mfma_f32_32x32x16_bf16 (A 32 x 16, B 16 x 32, lane l: row / column l % 32, k = 8 * (l / 32)
// .. + 7; D: lane l holds column l % 32 and rows (r / 4) * 8 + (l / 32) * 4 + r % 4, r = 0..15):
// the workgroup's 32 chunks form one group, wave w and lane l own state 2 w + l / 32 of chunk
// l % 32.  The weights held per wave and turn are the same 512, but one 128-bit activation load
// per lane now serves 32 tokens instead of 16, which is what limits larger batches.
#pragma once

#include "neuzip_format.h"
#include "neuzip_decode_kernels.h"

namespace nz {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

// Accumulator tile and matrix instruction of the two forms
template <int COLS>
struct LinearTile;
template <>
struct LinearTile<16> {
    typedef f32x4_t acc_t;
    static constexpr int kRegs = 4;
    static __device__ __forceinline__ acc_t mma(bf16x8_t a, bf16x8_t b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    // token (row of D) held in register r of lane `lane`
    static __device__ __forceinline__ uint32_t row(uint32_t lane, int r) { return (lane >> 4) * 4 + r; }
};
template <>
struct LinearTile<32> {
    typedef f32x16_t acc_t;
    static constexpr int kRegs = 16;
    static __device__ __forceinline__ acc_t mma(bf16x8_t a, bf16x8_t b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t row(uint32_t lane, int r)
    {
        return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
    }
};

constexpr uint32_t kLinThreads = 512;
constexpr uint32_t kLinMaxTokens = 64;

struct LinearArgs {
    const TableBlock *tb;
    const uint32_t *offsets;
    const uint32_t *states;
    const uint8_t *lens;
    const uint16_t *words;
    const uint8_t *sm;
    const uint8_t *coef;   // block coefficients (block-wise normalised blobs only)
    uint32_t block_shift;  // log2 of the block size of the normalisation
    const uint16_t *x;     // [tokens][in_features] bf16
    float *y;              // [tokens][out_features], holds the bias (or zero) on entry
    uint32_t *status;
    uint64_t n;
    uint32_t n_chunks;
    uint32_t in_features;
    uint32_t out_features;
    uint32_t tokens;
    uint32_t stride;       // chunks between neighbouring columns of a group
    uint32_t rstep;        // rows between neighbouring columns of a group
    uint32_t n_groups;
};

// Several weights applied to the same kind of input in one launch (the q, k and v projections of an
// attention block, say): workgroups [wg_end[i-1], wg_end[i]) belong to weight i.  Weights too small to
// fill the chip on their own overlap with the others.
constexpr uint32_t kLinBatchMax = 4;
struct LinearBatchArgs {
    LinearArgs t[kLinBatchMax];
    uint32_t wg_end[kLinBatchMax];
    uint32_t count;
};
struct LinearInitBatchArgs {
    float *y[kLinBatchMax];
    const float *bias[kLinBatchMax];
    uint32_t out_features[kLinBatchMax];
    uint32_t wg_end[kLinBatchMax];
    uint32_t tokens, count;
};

// y[t][o] = bias[o] (or 0): the accumulation target of the kernel below
__global__ void linear_init_kernel(float *__restrict__ y, const float *__restrict__ bias, uint32_t tokens,
                                   uint32_t out_features)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < static_cast<uint64_t>(tokens) * out_features)
        y[i] = bias ? bias[i % out_features] : 0.0f;
}

__global__ void linear_init_batch_kernel(const LinearInitBatchArgs b)
{
    uint32_t i = 0, first = 0;
    while (i + 1 < b.count && blockIdx.x >= b.wg_end[i]) {
        first = b.wg_end[i];
        ++i;
    }
    const uint64_t at = static_cast<uint64_t>(blockIdx.x - first) * blockDim.x + threadIdx.x;
    if (at < static_cast<uint64_t>(b.tokens) * b.out_features[i])
        b.y[i][at] = b.bias[i] ? b.bias[i][at % b.out_features[i]] : 0.0f;
}

__device__ __forceinline__ void atomic_add_f32(float *p, float v)
{
    // the hardware float add of the memory system (no compare-and-swap loop); y is ordinary
    // device memory, which is what that instruction requires
    unsafeAtomicAdd(p, v);
}

// NORM: the blob is block-wise normalised (Sec. 2.3): the merged words are multiplied by their block's
// coefficient, as in the decoder, before they enter the matrix instruction.
template <int KB, int COLS, int MT, bool LONE, bool NORM, class WordSrc>
__device__ __forceinline__ void linear_walk(const uint32_t *__restrict__ lut, const WordSrc &src, uint32_t lone,
                                            uint32_t &x, uint32_t &wp, const uint8_t *__restrict__ sm,
                                            const LinearArgs &a, uint64_t base, uint32_t kk, uint32_t turns,
                                            uint32_t j, uint32_t lane)
{
    const uint32_t in = a.in_features;
    typedef LinearTile<COLS> Tile;
    constexpr uint32_t kPerWave = 64 / COLS;         // states of a chunk held by one wave (4 or 2)
    const uint32_t col = lane & (COLS - 1);          // column of B and of D: this lane's chunk
    const uint32_t kq = (j % kPerWave) * 8u;         // this lane's 8 input features inside the wave's 32 or 16
    const uint32_t ksq = (j / kPerWave) * kPerWave * 8u;  // the wave's features inside the turn's 128
    // Position in the matrix: the row is the lane's own (its chunk's); the input-feature offset kk
    // is that of the group's first chunk, which all 16 chunks share -- lanes without a chunk use
    // it too, because every lane supplies activations to A.
    uint32_t row = static_cast<uint32_t>(base / in);
    // rows of the activations this lane supplies to A (clamped: rows past `tokens` are never stored)
    const uint16_t *xrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        uint32_t t = mt * COLS + col;
        t = t < a.tokens ? t : a.tokens - 1;
        xrow[mt] = a.x + static_cast<uint64_t>(t) * in + ksq + kq;
    }
    typename Tile::acc_t acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < Tile::kRegs; ++r)
            acc[mt][r] = 0.0f;

    uint32_t next = LONE ? 0u : src.peek(wp);
    const uint64_t first = base + j * kRun;
    uint64_t fields = turns > 0 ? load_turn<KB, NORM>(sm, a.coef, a.block_shift, first) : 0;
    uint4 xa[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        xa[mt] = *reinterpret_cast<const uint4 *>(xrow[mt] + kk);

    // the trip count is the same for every lane of the wave (the matrix instruction needs them
    // all); a lane whose chunk is shorter or absent supplies zeros
    for (uint32_t q = 0; q < kTurns; ++q) {
        const bool mine = q < turns;
        // requests for the next turn go out before this turn is decoded
        const uint32_t kk_next = kk + kTurn == in ? 0u : kk + kTurn;
        uint64_t fields_next = 0;
        if (q + 1 < turns)
            fields_next = load_turn<KB, NORM>(sm, a.coef, a.block_shift, first + (q + 1) * kTurn);
        uint4 xa_next[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            xa_next[mt] = *reinterpret_cast<const uint4 *>(xrow[mt] + kk_next);

        union {
            uint32_t u[4];
            bf16x8_t v;
        } b;
        b.u[0] = b.u[1] = b.u[2] = b.u[3] = 0;
        if (mine) {
            uint32_t e[8];
#pragma unroll
            for (int t = 0; t < 8; ++t)
                e[t] = LONE ? lone : rans_get(lut, x, wp, next, src);
            b.u[0] = merge_pair<KB>(fields, 0, e[0], e[1]);
            b.u[1] = merge_pair<KB>(fields, 1, e[2], e[3]);
            b.u[2] = merge_pair<KB>(fields, 2, e[4], e[5]);
            b.u[3] = merge_pair<KB>(fields, 3, e[6], e[7]);
            if constexpr (NORM) {
                const float c = coefficient(static_cast<uint32_t>(fields >> 32) & 0x7Fu);
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    b.u[d] = denormalise_pair(b.u[d], c);
            }
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            union {
                uint4 q4;
                bf16x8_t v;
            } av;
            av.q4 = xa[mt];
            acc[mt] = Tile::mma(av.v, b.v, acc[mt]);
        }
        // end of a row of the weight (or of the chunk): this wave's partial sums leave for y.
        // (Summing the waves of a group in LDS first was tried: the barriers and the extra
        // registers cost more than the atomics they save.)
        if (kk_next == 0 || q + 1 == kTurns) {
            const bool col_live = mine && row < a.out_features;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int r = 0; r < Tile::kRegs; ++r) {
                    const uint32_t t = mt * COLS + Tile::row(lane, r);
                    if (col_live && t < a.tokens)
                        atomic_add_f32(a.y + static_cast<uint64_t>(t) * a.out_features + row, acc[mt][r]);
                    acc[mt][r] = 0.0f;
                }
            }
            row += kk_next == 0 ? 1u : 0u;
        }
        kk = kk_next;
        fields = fields_next;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            xa[mt] = xa_next[mt];
    }
}

template <int KB, int COLS, int MT, bool NORM>
__device__ __forceinline__ void linear_workgroup(const LinearArgs &a, uint32_t wg, uint32_t *__restrict__ lut,
                                                 uint8_t *__restrict__ stage)
{
    constexpr uint32_t kLinGroupChunks = COLS;                       // columns of the B operand
    constexpr uint32_t kGroupsPerWg = kDecChunksPerWg / COLS;        // 2 or 1
    constexpr uint32_t kWavesPerGroup = kLinThreads / 64 / kGroupsPerWg;  // 4 or 8
    constexpr uint32_t kPerWave = 64 / COLS;                         // states of a chunk per wave: 4 or 2
    constexpr uint32_t kLinGroupBytes = kStageBytes / kGroupsPerWg;  // LDS window of one group's word runs
    constexpr uint32_t kColsPerWave = COLS / kWavesPerGroup;         // columns a wave copies: 4
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = tid >> 6, lane = tid & 63u;
    const uint32_t g = wave / kWavesPerGroup, sq = wave % kWavesPerGroup;
    const uint32_t col = lane & (COLS - 1);
    const uint32_t j = sq * kPerWave + lane / COLS;
    const uint32_t group = wg * kGroupsPerWg + g;
    const bool group_live = group < a.n_groups;
    // group -> its COLS chunks: `stride` groups interleave inside a block of COLS * stride chunks
    const uint32_t block_id = group / a.stride, first_in_block = group % a.stride;
    const uint64_t c64 = static_cast<uint64_t>(block_id) * kLinGroupChunks * a.stride + first_in_block +
                         static_cast<uint64_t>(a.stride) * col;
    const bool live = group_live && c64 < a.n_chunks;
    const uint32_t kk0 = static_cast<uint32_t>(
        (static_cast<uint64_t>(block_id) * kLinGroupChunks * a.stride + first_in_block) * kChunk % a.in_features);
    const uint32_t c = live ? static_cast<uint32_t>(c64) : 0u;
    const uint64_t base = static_cast<uint64_t>(c) * kChunk;
    const uint32_t m = !live ? 0u : ((a.n - base) < kChunk ? static_cast<uint32_t>(a.n - base) : kChunk);
    const uint32_t turns = m / kTurn;   // in_features is a multiple of 128, so chunks hold whole turns

    // ---- loads that depend on nothing
    const uint32_t off_c = live ? a.offsets[c] : 0u;
    const uint32_t off_c1 = live ? a.offsets[c + 1] : 0u;
    uint32_t x = live ? a.states[c * kStates + j] : kRansL;
    uint4 lens16 = make_uint4(0, 0, 0, 0);
    if (live)
        lens16 = *reinterpret_cast<const uint4 *>(a.lens + static_cast<uint64_t>(c) * kStates);
    const uint32_t lone = a.tb->lone;
    const uint4 *lut_g = reinterpret_cast<const uint4 *>(a.tb->lut);
    uint4 lut_piece[2];
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r)
        lut_piece[r] = lut_g[tid + r * kLinThreads];

    // ---- stage the word runs of the group's chunks: each chunk's piece of the blob, from the
    // 16-byte boundary below its first word, one after the other in the group's window
    const uint64_t byte0 = static_cast<uint64_t>(off_c) * 2, byte1 = static_cast<uint64_t>(off_c1) * 2;
    const uint64_t aligned0 = byte0 & ~static_cast<uint64_t>(15);
    const uint32_t piece = live ? static_cast<uint32_t>((byte1 - aligned0 + 15) & ~static_cast<uint64_t>(15)) : 0u;
    uint32_t place = piece;  // exclusive prefix over the columns (lanes with equal lane / COLS agree)
#pragma unroll
    for (uint32_t d = 1; d < COLS; d <<= 1) {
        const uint32_t o = __shfl_up(place, d, COLS);
        if (col >= d)
            place += o;
    }
    const uint32_t group_bytes = __shfl(place, COLS - 1, COLS);
    place -= piece;
    const bool staged = group_bytes + 16 <= kLinGroupBytes;
    uint8_t *window = stage + g * kLinGroupBytes;
    if (staged && group_live) {
#pragma unroll
        for (uint32_t r = 0; r < kColsPerWave; ++r) {
            const uint32_t from_col = sq * kColsPerWave + r;  // wave sq copies 4 columns
            const uint32_t lo = __shfl(static_cast<uint32_t>(aligned0), from_col, 64);
            const uint32_t hi = __shfl(static_cast<uint32_t>(aligned0 >> 32), from_col, 64);
            const uint32_t len = __shfl(piece, from_col, 64);
            const uint32_t at = __shfl(place, from_col, 64);
            const uint4 *from = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(a.words) +
                                                                ((static_cast<uint64_t>(hi) << 32) | lo));
            uint4 *to = reinterpret_cast<uint4 *>(window + at);
            for (uint32_t i = lane; i * 16 < len; i += 64)
                to[i] = from[i];
        }
    }
#pragma unroll
    for (uint32_t r = 0; r < 2; ++r)
        reinterpret_cast<uint4 *>(lut)[tid + r * kLinThreads] = lut_piece[r];
    __syncthreads();
    if (!group_live)
        return;  // the whole wave leaves together

    // ---- start of this state's run: the chunk's offset plus the lengths of the states before it
    const uint32_t lw[4] = {lens16.x, lens16.y, lens16.z, lens16.w};
    uint32_t before = 0, len = 0;
#pragma unroll
    for (uint32_t s = 0; s < kStates; ++s) {
        const uint32_t l8 = (lw[s >> 2] >> (8 * (s & 3u))) & 0xFFu;
        before += s < j ? l8 : 0u;
        len = s == j ? l8 : len;
    }
    const uint64_t run_byte = (static_cast<uint64_t>(off_c) + before) * 2;

    uint32_t wp = 0, wp_begin = 0;
    if (lone < 256) {
        linear_walk<KB, COLS, MT, true, NORM>(lut, NoWords{}, lone, x, wp, a.sm, a, base, kk0, turns, j, lane);
    } else if (staged) {
        wp = wp_begin = g * kLinGroupBytes + place + static_cast<uint32_t>(run_byte - aligned0);
        linear_walk<KB, COLS, MT, false, NORM>(lut, LdsWords{stage}, 0u, x, wp, a.sm, a, base, kk0, turns, j, lane);
    } else {
        const GlobalWords direct{reinterpret_cast<const uint8_t *>(a.words) + run_byte};
        linear_walk<KB, COLS, MT, false, NORM>(lut, direct, 0u, x, wp, a.sm, a, base, kk0, turns, j, lane);
    }
    if (live && (x != kRansL || wp - wp_begin != 2 * len))
        atomicOr(a.status, 1u);
}

template <int KB, int COLS, int MT, bool NORM = false>
__global__ __launch_bounds__(kLinThreads) void linear_kernel(const LinearArgs a)
{
    __shared__ __align__(16) uint32_t lut[kM];
    __shared__ __align__(16) uint8_t stage[kStageBytes];
    linear_workgroup<KB, COLS, MT, NORM>(a, blockIdx.x, lut, stage);
}

template <int KB, int COLS, int MT, bool NORM = false>
__global__ __launch_bounds__(kLinThreads) void linear_batch_kernel(const LinearBatchArgs b)
{
    __shared__ __align__(16) uint32_t lut[kM];
    __shared__ __align__(16) uint8_t stage[kStageBytes];
    uint32_t i = 0, first = 0;
    while (i + 1 < b.count && blockIdx.x >= b.wg_end[i]) {
        first = b.wg_end[i];
        ++i;
    }
    linear_workgroup<KB, COLS, MT, NORM>(b.t[i], blockIdx.x - first, lut, stage);
}

}  // namespace nz
