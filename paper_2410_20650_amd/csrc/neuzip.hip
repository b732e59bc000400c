// NeuZip codec for MI355X (gfx950): host side of the C ABI declared in include/neuzip.h.  The
// kernels live in neuzip_compress_kernels.h, neuzip_decode_kernels.h and neuzip_linear_kernels.h, the shared constants and
// device structures in neuzip_format.h; all of it is compiled as this one translation unit.
//
// Stream format (little-endian):
//   container := header(64 B) | freq[256] u16 | offsets[nc+1] u32 | states[nc*16] u32
//              | lens[nc*16] u8 | words[total] u16 | signmant[ceil(n*(k+1)/8)] u8
//              | low[n] u16 (binary32 blobs only: the lower halves of the elements)
//              | coef[ceil(n/block)] u8 (block-wise normalised blobs only)
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

#include "neuzip_format.h"
#include "neuzip_compress_kernels.h"
#include "neuzip_decode_kernels.h"
#include "neuzip_linear_kernels.h"

using namespace nz;

namespace {

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

constexpr uint64_t pad_to(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
inline bool valid_k(int k) { return k == 7 || k == 3 || k == 1 || k == 0; }
inline uint64_t signmant_bytes(uint64_t n, int k) { return (n * static_cast<uint64_t>(k + 1) + 7) / 8; }
inline uint32_t chunks_of(uint64_t n) { return static_cast<uint32_t>((n + kChunk - 1) / kChunk); }

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
inline bool valid_block(uint32_t b) { return b == 32 || b == 64 || b == 128 || b == 256 || b == 512; }
inline uint64_t block_count(uint64_t n, uint32_t block) { return block ? (n + block - 1) / block : 0; }

struct Layout {
    uint64_t offsets, states, lens, sm, low, coef, total;  // byte positions inside the fixed allocation
};

// f32: the tensor's elements are binary32; the plane of their lower halves follows the sign|mantissa stream
Layout fixed_layout(uint64_t n, int k, uint32_t block, bool f32)
{
    const uint64_t nc = chunks_of(n);
    Layout l;
    l.offsets = sizeof(TableBlock);
    l.states = l.offsets + pad_to((nc + 2) * 4, 256);
    l.lens = l.states + pad_to(nc * kStates * 4, 256);
    l.sm = l.lens + pad_to(nc * kStates, 256);
    l.low = l.sm + pad_to(signmant_bytes(n, k), 256) + 256;
    l.coef = l.low + (f32 ? pad_to(n * 2, 256) + 256 : 0);
    l.total = l.coef + pad_to(block_count(n, block), 256);
    return l;
}

struct Container {
    uint64_t freq, offsets, states, lens, words, sm, low, coef, total;  // byte positions in the flat container
};

Container container_layout(uint64_t n, int k, uint64_t total_words, uint32_t block, bool f32)
{
    const uint64_t nc = chunks_of(n);
    Container c;
    c.freq = kHeaderBytes;
    c.offsets = c.freq + 512;
    c.states = c.offsets + pad_to((nc + 1) * 4, 16);
    c.lens = c.states + nc * kStates * 4;
    c.words = c.lens + nc * kStates;
    c.sm = c.words + pad_to(total_words * 2, 16);
    c.low = c.sm + pad_to(signmant_bytes(n, k), 16);
    c.coef = c.low + (f32 ? pad_to(n * 2, 16) : 0);
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
    uint32_t guard;  // guard band of the frequency table, 0 = none
    int elem;        // NEUZIP_BF16; NEUZIP_F32 (lossless only: a plane of lower halves rides along); NEUZIP_F16 (lossless only)
    bool has_table;  // holds a compressed tensor (and so a table that recompression can reuse)
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
inline uint16_t *low_of(const neuzip_blob *b) { return reinterpret_cast<uint16_t *>(b->fixed + b->at.low); }
inline bool is_blob(const neuzip_blob *b) { return b && b->magic == kBlobMagic; }

// A blob lives on the device that was current when it was made; kernels are launched on the
// current device, so the two must agree.
inline bool on_current_device(const neuzip_blob *b)
{
    int cur = -1;
    return hipGetDevice(&cur) == hipSuccess && cur == b->device;
}

// Per-process compress workspace: histogram bins and encoder constants for the tensors of a batch,
// per-chunk / per-group word counts, run slots, and pinned host memory for the results.
struct Workspace {
    int device = -1;
    uint32_t *counts = nullptr;       // kBatchMax x 256 histogram bins, zero between compress calls; behind them, in
                                      // the same allocation, the two copies of the call state and a counter
    CallState *state = nullptr;       // [2], used by alternate calls (stamp & 1)
    uint32_t *all_done = nullptr;     // tensors of the batch that have been reported to the host
    uint32_t *super_words = nullptr;  // [2][super_cap] words per 64 encoder groups, used by alternate calls
    uint32_t super_cap = 0;
    uint32_t *chunk_words = nullptr;  // words per chunk
    uint32_t *group_words = nullptr;  // words per encoder workgroup (16 chunks), input of the scan
    uint64_t group_cap = 0;           // encoder groups the arrays and the slots are sized for
    uint16_t *slots = nullptr;
    HostRecord *pinned = nullptr;     // pinned host memory, written by the encode kernel
    uint32_t seq = 0;                 // stamp of the last compress call
    hipEvent_t idle = nullptr;        // recorded after the last kernel that uses the workspace
    hipStream_t last_stream = nullptr; // ... on this stream
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
        void *device_arrays[] = {g_ws.counts, g_ws.chunk_words, g_ws.group_words, g_ws.super_words, g_ws.slots};
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

// Waits until the encode kernel of call `seq` has published its record.  The stamp arrives a
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

// Words of the small allocation: the histogram bins of a batch, two call states, a counter (padded).
constexpr uint32_t kSmallWords = kBatchMax * 256 + 2 * sizeof(CallState) / 4 + 16;
// Entries of one copy of the per-64-groups array for a batch of n_groups encoder groups in all: every
// tensor of the batch may end with a partial block.
inline uint32_t super_entries(uint64_t n_groups) { return static_cast<uint32_t>(n_groups / kSuperGroups + kBatchMax + 1); }

// Returns everything a failed call may have left behind in the workspace to zero.
void reset_workspace(const Workspace &ws, hipStream_t stream)
{
    if (ws.counts)
        hipLaunchKernelGGL(fill_u32_kernel, dim3((kSmallWords + 255) / 256), dim3(256), 0, stream, ws.counts, 0u,
                           kSmallWords);
    if (ws.super_words)
        hipLaunchKernelGGL(fill_u32_kernel, dim3((2 * ws.super_cap + 255) / 256), dim3(256), 0, stream, ws.super_words, 0u,
                           2 * ws.super_cap);
    (void)hipGetLastError();
}

// First use on a device: the arrays whose size does not depend on the tensors.
int create_workspace(int device, hipStream_t stream)
{
    g_ws.device = device;
    NZ_HIP(hipMalloc(reinterpret_cast<void **>(&g_ws.counts), kSmallWords * sizeof(uint32_t)));
    g_ws.state = reinterpret_cast<CallState *>(g_ws.counts + kBatchMax * 256);
    g_ws.all_done = g_ws.counts + kBatchMax * 256 + 2 * sizeof(CallState) / 4;
    NZ_HIP(hipHostMalloc(reinterpret_cast<void **>(&g_ws.pinned), sizeof(HostRecord), hipHostMallocDefault));
    std::memset(g_ws.pinned, 0, sizeof(HostRecord));
    g_ws.seq = 0;
    NZ_HIP(hipEventCreateWithFlags(&g_ws.idle, hipEventDisableTiming));
    hipLaunchKernelGGL(fill_u32_kernel, dim3((kSmallWords + 255) / 256), dim3(256), 0, stream, g_ws.counts, 0u,
                       kSmallWords);
    NZ_HIP(hipGetLastError());
    NZ_HIP(hipEventRecord(g_ws.idle, stream));
    g_ws.last_stream = stream;
    return NEUZIP_OK;
}

int ensure_workspace(int device, uint64_t n_groups, hipStream_t stream)
{
    if (g_ws.device != device) {
        int rc = release_workspace_locked();
        if (rc != NEUZIP_OK)
            return rc;
        rc = create_workspace(device, stream);
        if (rc != NEUZIP_OK) {
            // a half-built workspace must not be taken for a complete one by the next call
            (void)hipGetLastError();
            (void)release_workspace_locked();
            return rc;
        }
    }
    // the previous user of the workspace may still be running on another stream (on the same one, the
    // stream's own order does)
    if (stream != g_ws.last_stream)
        NZ_HIP(hipStreamWaitEvent(stream, g_ws.idle, 0));
    g_ws.last_stream = stream;
    if (g_ws.group_cap < n_groups) {
        NZ_HIP(hipEventSynchronize(g_ws.idle));
        void *old_arrays[] = {g_ws.chunk_words, g_ws.group_words, g_ws.super_words, g_ws.slots};
        for (void *ptr : old_arrays)
            if (ptr)
                NZ_HIP(hipFree(ptr));
        g_ws.chunk_words = g_ws.group_words = g_ws.super_words = nullptr;
        g_ws.slots = nullptr;
        g_ws.group_cap = 0;
        g_ws.super_cap = 0;
        const uint64_t chunks = n_groups * kChunksPerGroup;
        const uint32_t super_cap = super_entries(n_groups);
        if (hipMalloc(reinterpret_cast<void **>(&g_ws.chunk_words), (chunks + 4) * 4) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&g_ws.group_words), (n_groups + 4) * 4) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&g_ws.super_words), 2ull * super_cap * 4) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&g_ws.slots), chunks * kStates * kRunCap * 2) != hipSuccess) {
            (void)hipGetLastError();
            return NEUZIP_ENOMEM;
        }
        g_ws.group_cap = n_groups;
        g_ws.super_cap = super_cap;
        // both copies start at zero (the call state behind the bins is zero between calls anyway)
        hipLaunchKernelGGL(fill_u32_kernel, dim3((2 * super_cap + 255) / 256), dim3(256), 0, stream, g_ws.super_words, 0u,
                           2 * super_cap);
        NZ_HIP(hipGetLastError());
    }
    return NEUZIP_OK;
}

int alloc_blob(uint64_t n, int k, uint32_t block, int elem, neuzip_blob **out)
{
    neuzip_blob *b = new (std::nothrow) neuzip_blob();
    if (!b)
        return NEUZIP_ENOMEM;
    std::memset(b, 0, sizeof(*b));
    b->magic = kBlobMagic;
    b->n = n;
    b->k = k;
    b->block = block;
    b->elem = elem;
    b->n_chunks = chunks_of(n);
    b->at = fixed_layout(n, k, block, elem == NEUZIP_F32);
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
        // A blob that receives a new version of its tensor after every update grows and shrinks
        // by a little each time: an allocation gets 1/64 of headroom (0.3 % of the container), so
        // that this does not mean a new allocation per call.
        if (b->words) {
            NZ_HIP(hipFree(b->words));
            b->words = nullptr;
            b->words_bytes = 0;
        }
        const uint64_t roomy = pad_to(need + need / 64, 256);
        if (hipMalloc(reinterpret_cast<void **>(&b->words), roomy) != hipSuccess) {
            (void)hipGetLastError();
            return NEUZIP_ENOMEM;
        }
        b->words_bytes = roomy;
    }
    return NEUZIP_OK;
}

// Words a blob's word section has room for: reserve_words() would be content with it as it is.
inline uint64_t words_room(const neuzip_blob *b)
{
    return b->words_bytes >= 1024 ? (b->words_bytes - 1024) / 256 * 256 / 2 : 0;
}

// Chunks per decoder workgroup.  32 (8 waves) measured best from ~16 M elements up: two such
// workgroups fill a CU's LDS with 16 waves, and smaller workgroups lower that occupancy.  A small
// tensor cannot fill the chip either way and is a chain of 256 dependent steps per lane; there
// workgroups of 16 chunks spread the waves over twice as many CUs (4-7 % faster up to 16 M elements).
// NEUZIP_DECODE_CHUNKS_PER_WG (4..32, multiple of 4) overrides the choice for tuning runs.
// binary16 symbols carry 5-6 bits each (sign and two mantissa bits ride in the symbol), so only
// 16 chunks' words fit the LDS window: such blobs always take workgroups of 16 chunks.
uint32_t decode_chunks_per_wg(uint32_t n_chunks, bool f16 = false)
{
    if (f16)
        return 16u;
    static int forced = -1;
    if (forced < 0) {
        const char *env = std::getenv("NEUZIP_DECODE_CHUNKS_PER_WG");
        const int v = env ? std::atoi(env) : 0;
        forced = (v >= 4 && v <= static_cast<int>(kDecChunksPerWg) && v % 4 == 0) ? v : 0;
    }
    if (forced > 0)
        return static_cast<uint32_t>(forced);
    return n_chunks <= 4096 ? 16u : kDecChunksPerWg;
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
    a.low = low_of(b);
    a.grad = nullptr;
    a.lr = 0.0f;
    a.block = b->block;
    // 2 bytes out + ~1.3 in per element against 256 MB of Infinity Cache: beyond ~64 M elements
    // (half as many of binary32) the tensor streams through HBM and non-temporal stores measured
    // 5 % faster; below they cost 3 %
    a.stream_out = ((b->elem == NEUZIP_F32) ? 2 * b->n : b->n) >= (64ull << 20) ? 1u : 0u;
    a.out = d_dst;
    a.status = table_of(b)->status;
    a.n = b->n;
    a.n_chunks = b->n_chunks;
    a.wg_end = 0;
    return a;
}

template <int KB, bool NORM, int MODE = kPlain>
int launch_decode(const neuzip_blob *b, void *d_dst, hipStream_t stream)
{
    const uint32_t per = decode_chunks_per_wg(b->n_chunks, b->elem == NEUZIP_F16);
    const uint32_t groups = (b->n_chunks + per - 1) / per;
    hipLaunchKernelGGL((decode_kernel<KB, NORM, MODE>), dim3(groups), dim3(per * kStates), 0, stream,
                       decode_args(b, d_dst));
    return hip_ok(hipGetLastError()) ? NEUZIP_OK : NEUZIP_EHIP;
}

int decode_dispatch(const neuzip_blob *b, void *d_dst, hipStream_t stream)
{
    if (b->n == 0)
        return NEUZIP_OK;
    if (b->elem == NEUZIP_F32)
        return launch_decode<7, false, kWide>(b, d_dst, stream);
    if (b->elem == NEUZIP_F16)
        return launch_decode<7, false, kHalf>(b, d_dst, stream);
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

// variant = mantissa_bits, + 8 for block-wise normalised blobs, + 16 for binary32, + 32 for binary16
// blobs; kUpdateVariant is the lossless bf16 decoder that applies the weight step
constexpr int kUpdateVariant = 100;
inline int decode_variant(const neuzip_blob *b)
{
    return b->k + (b->block ? 8 : 0) + (b->elem == NEUZIP_F32 ? 16 : 0) + (b->elem == NEUZIP_F16 ? 32 : 0);
}

// chunks per workgroup of a batch launch of the given variant
inline uint32_t batch_chunks_per_wg(int variant) { return variant == 39 ? 16u : kDecChunksPerWg; }

int launch_batch(const BatchArgs &args, int variant, uint32_t groups, hipStream_t stream)
{
    const dim3 grid(groups), block(batch_chunks_per_wg(variant) * kStates);
    switch (variant) {
    case 7: hipLaunchKernelGGL((decode_batch_kernel<7, false>), grid, block, 0, stream, args); break;
    case 3: hipLaunchKernelGGL((decode_batch_kernel<3, false>), grid, block, 0, stream, args); break;
    case 1: hipLaunchKernelGGL((decode_batch_kernel<1, false>), grid, block, 0, stream, args); break;
    case 0: hipLaunchKernelGGL((decode_batch_kernel<0, false>), grid, block, 0, stream, args); break;
    case 11: hipLaunchKernelGGL((decode_batch_kernel<3, true>), grid, block, 0, stream, args); break;
    case 9: hipLaunchKernelGGL((decode_batch_kernel<1, true>), grid, block, 0, stream, args); break;
    case 23: hipLaunchKernelGGL((decode_batch_kernel<7, false, kWide>), grid, block, 0, stream, args); break;
    case 39: hipLaunchKernelGGL((decode_batch_kernel<7, false, kHalf>), grid, block, 0, stream, args); break;
    case kUpdateVariant: hipLaunchKernelGGL((decode_batch_kernel<7, false, kUpdate>), grid, block, 0, stream, args); break;
    default: hipLaunchKernelGGL((decode_batch_kernel<0, true>), grid, block, 0, stream, args); break;
    }
    return hip_ok(hipGetLastError()) ? NEUZIP_OK : NEUZIP_EHIP;
}

// Which form of the kernel: 16 columns (tiles of 16 tokens) or 32 columns (tiles of 32 tokens).
// The wide form halves the activation traffic per token but doubles the waves that add partial
// sums to one output, so it pays for more than 16 tokens on shapes whose chunks never straddle
// rows of the weight (stride 1: no row ends inside a chunk); measured on 14336 x 4096 and
// 4096 x 14336.
inline uint32_t linear_columns(uint32_t tokens, uint32_t stride) { return tokens > 16 && stride == 1 ? 32u : 16u; }

// One weight: the plain kernel (its arguments are the first entry); several: the batch kernel.
template <int KB, bool NORM>
void launch_linear(const LinearBatchArgs &batch, uint32_t cols, uint32_t wgs, hipStream_t stream)
{
    const dim3 grid(wgs), block(kLinThreads);
    const uint32_t tokens = batch.t[0].tokens;
#define NZ_LINEAR(COLS, MT)                                                                                       \
    do {                                                                                                          \
        if (batch.count == 1)                                                                                     \
            hipLaunchKernelGGL((linear_kernel<KB, COLS, MT, NORM>), grid, block, 0, stream, batch.t[0]);          \
        else                                                                                                      \
            hipLaunchKernelGGL((linear_batch_kernel<KB, COLS, MT, NORM>), grid, block, 0, stream, batch);         \
    } while (0)
    if (cols == 32) {
        if (tokens <= 32)
            NZ_LINEAR(32, 1);
        else
            NZ_LINEAR(32, 2);
        return;
    }
    switch ((tokens + 15) / 16) {
    case 1: NZ_LINEAR(16, 1); break;
    case 2: NZ_LINEAR(16, 2); break;
    case 3: NZ_LINEAR(16, 3); break;
    default: NZ_LINEAR(16, 4); break;
    }
#undef NZ_LINEAR
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
    b->has_table = true;
    return NEUZIP_OK;
}

template <int KB>
void launch_hist(const Workspace &ws, const CompressBatch &batch, bool norm, uint32_t groups, uint32_t threads,
                 hipStream_t stream)
{
    if (norm)
        hipLaunchKernelGGL(hist_split_norm_kernel<KB>, dim3(groups), dim3(threads), 0, stream, batch, ws.counts);
    else
        hipLaunchKernelGGL(hist_split_kernel<KB>, dim3(groups), dim3(threads), 0, stream, batch, ws.counts);
}

// Bytes of encoder slots one group of 16 chunks takes, and the limit on the slot array: a batch that
// needs more is compressed tensor by tensor, and a tensor that alone needs more in tiles of whole groups.
constexpr uint64_t kSlotBytesPerGroup = static_cast<uint64_t>(kChunksPerGroup) * kStates * kRunCap * 2;
// (384 MiB: the seven weights of a Llama-3-8B layer, 218 M elements, still go through as one batch --
// measured 8 % faster than in two parts -- and the 525 M-element embedding takes three tiles, 3 % slower
// than in one piece with 0.82 GB of slots)
constexpr uint64_t kDefaultSlotLimit = 384ull << 20;
uint64_t g_slot_limit = kDefaultSlotLimit;
inline uint64_t slot_limit_groups()
{
    const uint64_t g = g_slot_limit / kSlotBytesPerGroup;
    return g < 1 ? 1 : g;
}

// Makes room for `want` words in a blob's word section while keeping the first `keep` words it holds
// (the tiles compacted so far).
int grow_words_keeping(neuzip_blob *b, uint64_t want, uint64_t keep, hipStream_t stream)
{
    const uint64_t need = pad_to(want * 2, 256) + 1024;
    if (b->words_bytes >= need)
        return NEUZIP_OK;
    const uint64_t roomy = pad_to(need + need / 64, 256);
    uint8_t *fresh = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&fresh), roomy) != hipSuccess) {
        (void)hipGetLastError();
        return NEUZIP_ENOMEM;
    }
    if (b->words) {
        if (keep > 0) {
            const uint64_t bytes = pad_to(keep * 2, 16) < b->words_bytes ? pad_to(keep * 2, 16) : b->words_bytes;
            if (!hip_ok(hipMemcpyAsync(fresh, b->words, bytes, hipMemcpyDeviceToDevice, stream)) ||
                !hip_ok(hipStreamSynchronize(stream))) {
                (void)hipFree(fresh);
                return NEUZIP_EHIP;
            }
        }
        if (!hip_ok(hipFree(b->words))) {
            (void)hipFree(fresh);
            return NEUZIP_EHIP;
        }
    }
    b->words = fresh;
    b->words_bytes = roomy;
    return NEUZIP_OK;
}

// The encoder launch of a compress pass.  variant: kUpdateVariant, 39 (binary16), 23 (binary32) or the
// mantissa width; reuse: the one-pass encoders that code with the table the blob holds.
bool launch_encode(const Workspace &ws, const CompressBatch &batch, uint32_t workgroups, int variant, bool reuse, int elem,
                   uint32_t block, uint32_t *super_words, CallState *state, hipStream_t stream)
{
    const dim3 grid(workgroups), threads(kEncThreads);
#define NZ_ENCODE(...)                                                                                          \
    hipLaunchKernelGGL((encode_kernel<__VA_ARGS__>), grid, threads, 0, stream, batch, ws.counts, ws.chunk_words, \
                       ws.group_words, super_words, ws.slots, ws.pinned, state)
    if (reuse) {
        switch (variant) {
        case kUpdateVariant: NZ_ENCODE(false, 7, false, false, true); break;
        case 39: NZ_ENCODE(false, 7, false, true); break;
        case 23: NZ_ENCODE(false, 7, true); break;
        case 7: NZ_ENCODE(false, 7); break;
        case 3: NZ_ENCODE(false, 3); break;
        case 1: NZ_ENCODE(false, 1); break;
        default: NZ_ENCODE(false, 0); break;
        }
    } else if (elem == NEUZIP_F16) {
        NZ_ENCODE(false, -1, false, true);
    } else if (elem == NEUZIP_F32) {
        NZ_ENCODE(false, -1, true);
    } else if (block) {
        NZ_ENCODE(true, -1);
    } else {
        NZ_ENCODE(false, -1);
    }
#undef NZ_ENCODE
    return hip_ok(hipGetLastError());
}

bool launch_compaction(const Workspace &ws, const CompressBatch &batch, uint32_t workgroups, uint32_t *super_words,
                       CallState *state, CallState *state_next, uint32_t *super_next, hipStream_t stream)
{
    hipLaunchKernelGGL(compact_kernel, dim3(workgroups), dim3(kCompactThreads), 0, stream, batch, ws.slots, ws.chunk_words,
                       ws.group_words, super_words, state, ws.counts, state_next, super_next, ws.super_cap, ws.all_done,
                       ws.pinned);
    return hip_ok(hipGetLastError());
}

void launch_histogram(const Workspace &ws, const CompressBatch &batch, int variant, bool norm, uint32_t groups,
                      uint32_t threads, hipStream_t stream)
{
    const dim3 grid(groups), block(threads);
    switch (variant) {
    case 39: hipLaunchKernelGGL((hist_split_kernel<7, false, true>), grid, block, 0, stream, batch, ws.counts); break;
    case 23: hipLaunchKernelGGL((hist_split_kernel<7, true>), grid, block, 0, stream, batch, ws.counts); break;
    case 7: launch_hist<7>(ws, batch, norm, groups, threads, stream); break;
    case 3: launch_hist<3>(ws, batch, norm, groups, threads, stream); break;
    case 1: launch_hist<1>(ws, batch, norm, groups, threads, stream); break;
    default: launch_hist<0>(ws, batch, norm, groups, threads, stream); break;
    }
}

constexpr uint32_t kKeepGuard = 0xFFFFFFFFu;  // compress_some: every blob keeps the guard band it has

// Compresses up to kBatchMax tensors (arguments already validated) with one pass of the pipeline.
// reuse = false: statistics are taken from the tensors and new tables are built (with the given
// guard band).  reuse = true: every blob holds a table already and the tensors are coded with
// those, in one pass over the source; rebuilt[i] is set for the tensors whose table turned out
// not to cover them, which are then compressed the first way.  d_grads (with reuse, lossless bf16
// only): the sources are weights that first take the step W - lr * grad in that same pass; the new
// weights replace them if keep_new is set (else only those of rebuilt tensors do).
// fixed_ws: a workspace of fixed size that lives in the library's static device array, for the entry
// point that allocates nothing (reuse = false, every blob exists already); nullptr: the shared
// workspace that grows on demand.
// One tensor whose encoder slots would not fit the workspace limit: the histogram pass runs over the
// whole tensor once, then encoder and compaction take the tensor in tiles of whole encoder groups.  A
// tile is an item of its own (pointers at the tile's first chunk, table_n and words_before tell the
// kernels about the rest), and the host waits for each tile's length before the next tile reuses the
// slots; the word section grows, keeping what it holds, when a tile does not fit.  *stale: a kept
// table turned out not to cover the tensor (reuse only); nothing of the pass is kept then.
int compress_tiled(neuzip_blob *b, const void *d_src, const void *d_grad, int k, uint32_t block, int elem, bool reuse,
                   float lr, bool keep_new, hipStream_t stream, bool *stale)
{
    *stale = false;
    Workspace &ws = g_ws;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    const uint32_t groups_total = (b->n_chunks + kChunksPerGroup - 1) / kChunksPerGroup;
    const uint32_t tile_groups = static_cast<uint32_t>(slot_limit_groups() < groups_total ? slot_limit_groups() : groups_total);
    int rc = ensure_workspace(b->device, tile_groups, stream);
    if (rc != NEUZIP_OK)
        return rc;
    const int variant = d_grad ? kUpdateVariant : (elem == NEUZIP_F32 ? 23 : (elem == NEUZIP_F16 ? 39 : k));
    const uint32_t src_bytes = elem == NEUZIP_F32 ? 4u : 2u;
    bool bins_dirty = false;
    auto fail = [&](int code) {
        if (bins_dirty)
            reset_workspace(ws, stream);
        b->has_table = false;
        return code;
    };
    CompressBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    batch.count = 1;
    batch.lr = lr;
    batch.keep_new = keep_new ? 1u : 0u;
    CompressItem &it = batch.it[0];
    it.tb = table_of(b);
    it.table_n = b->n;
    it.block = block;
    it.guard = b->guard;
    if (!reuse) {
        // statistics of the whole tensor (and its fields, coefficients and lower halves)
        it.src = d_src;
        it.n = b->n;
        it.sm = sm_of(b);
        it.coef = coef_of(b);
        it.low = low_of(b);
        it.n_chunks = b->n_chunks;
        const uint64_t bytes = b->n * src_bytes;
        const uint32_t threads = bytes <= (128ull << 20) ? kHistThreadsMax : 256u;
        const uint32_t cap = threads == 256u ? 1280u : 512u;
        uint64_t hg = ((b->n + 7) / 8 + threads * 8 - 1) / (threads * 8);
        hg = hg < 1 ? 1 : (hg > cap ? cap : hg);
        it.hist_end = static_cast<uint32_t>(hg);
        launch_histogram(ws, batch, variant, block != 0, it.hist_end, threads, stream);
        if (!hip_ok(hipGetLastError()))
            return fail(NEUZIP_EHIP);
        bins_dirty = true;
    }
    uint64_t words_before = 0;
    for (uint32_t g0 = 0; g0 < groups_total; g0 += tile_groups) {
        const uint32_t g1 = g0 + tile_groups < groups_total ? g0 + tile_groups : groups_total;
        const uint32_t c0 = g0 * kChunksPerGroup;
        const uint32_t c1 = g1 * kChunksPerGroup < b->n_chunks ? g1 * kChunksPerGroup : b->n_chunks;
        const uint64_t e0 = static_cast<uint64_t>(c0) * kChunk;
        const uint64_t e1 = static_cast<uint64_t>(c1) * kChunk < b->n ? static_cast<uint64_t>(c1) * kChunk : b->n;
        const bool last = g1 == groups_total;
        it.src = static_cast<const uint8_t *>(d_src) + e0 * src_bytes;
        it.grad = d_grad ? static_cast<const uint16_t *>(d_grad) + e0 : nullptr;
        it.n = e1 - e0;
        it.offsets = offsets_of(b) + c0;
        it.states = states_of(b) + static_cast<uint64_t>(c0) * kStates;
        it.lens = lens_of(b) + static_cast<uint64_t>(c0) * kStates;
        it.sm = sm_of(b) + e0 * static_cast<uint64_t>(k + 1) / 8;
        it.coef = block ? coef_of(b) + e0 / block : coef_of(b);
        it.low = low_of(b) ? low_of(b) + e0 : nullptr;
        it.n_chunks = c1 - c0;
        it.group_base = 0;
        it.super_base = 0;
        it.enc_end = g1 - g0;
        it.compact_end = (it.n_chunks + kCompactThreads / 64 - 1) / (kCompactThreads / 64);
        it.words = reinterpret_cast<uint16_t *>(b->words);
        it.words_cap = words_room(b);
        it.words_before = words_before;
        batch.seq = ++ws.seq;
        batch.keep_counts = last ? 0u : 1u;
        const uint32_t copy = batch.seq & 1u;
        CallState *state = ws.state + copy, *state_next = ws.state + (copy ^ 1u);
        uint32_t *super_words = ws.super_words + copy * ws.super_cap;
        uint32_t *super_next = ws.super_words + (copy ^ 1u) * ws.super_cap;
        // (the workgroup that fills in the decoder's slot table rides with the first tile)
        if (!launch_encode(ws, batch, it.enc_end + ((!reuse && g0 == 0) ? 1u : 0u), variant, reuse, elem, block, super_words,
                           state, stream))
            return fail(NEUZIP_EHIP);
        bins_dirty = true;  // (sums of this tile; the compaction's report clears them)
        batch.report = 1;
        if (!launch_compaction(ws, batch, it.compact_end, super_words, state, state_next, super_next, stream))
            return fail(NEUZIP_EHIP);
        if (!wait_for_record(batch.seq, stream))
            return fail(NEUZIP_EHIP);
        bins_dirty = !reuse && !last;  // the histogram bins stay until the last tile has been encoded
        const HostRecord::Item &r = ws.pinned->item[0];
        if (reuse && r.stale) {
            // The table does not cover this tile: the tensor will be compressed afresh.  A weight step
            // that writes the new weights back still has to reach the remaining tiles.
            *stale = true;
            b->has_table = false;
            if (!(d_grad && keep_new)) {
                (void)hipEventRecord(ws.idle, stream);
                return NEUZIP_OK;
            }
        }
        if (r.total_words[1] != 0)
            return fail(NEUZIP_EUNSUPPORTED);
        const uint64_t upto = words_before + r.total_words[0];
        if (upto >= (1ull << 32))
            return fail(NEUZIP_EUNSUPPORTED);  // more than 2^32 words
        if (!*stale && upto > it.words_cap) {
            // no room (or no word section yet): size it for the whole tensor at the rate seen so far
            const uint64_t guess = last ? upto : upto / c1 * b->n_chunks + upto % c1 * b->n_chunks / c1;
            rc = grow_words_keeping(b, last ? upto : guess + guess / 32, words_before, stream);
            if (rc != NEUZIP_OK)
                return fail(rc);
            it.words = reinterpret_cast<uint16_t *>(b->words);
            it.words_cap = words_room(b);
            batch.report = 0;
            if (!launch_compaction(ws, batch, it.compact_end, super_words, state, state_next, super_next, stream))
                return fail(NEUZIP_EHIP);
        }
        words_before = upto;
        if (!reuse && g0 == 0) {
            std::memcpy(b->h_counts, r.counts, 1024);
            std::memcpy(b->h_freq, r.freq, 512);
            b->have_counts = true;
        }
    }
    if (!*stale) {
        b->total_words = words_before;
        b->has_table = true;
    }
    if (!hip_ok(hipEventRecord(ws.idle, stream)))
        return NEUZIP_EHIP;
    return NEUZIP_OK;
}

int compress_some(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int k, uint32_t block, int elem,
                  uint32_t guard, bool reuse, uint32_t *rebuilt, hipStream_t stream, neuzip_blob **blobs,
                  const void *const *d_grads = nullptr, float lr = 0.0f, bool keep_new = true,
                  Workspace *fixed_ws = nullptr)
{
    Workspace &ws = fixed_ws ? *fixed_ws : g_ws;
    auto groups_of = [](uint64_t n) { return (static_cast<uint64_t>(chunks_of(n)) + kChunksPerGroup - 1) / kChunksPerGroup; };
    if (!fixed_ws && count > 1) {
        // a batch whose encoder slots would exceed the workspace limit goes through in parts: runs of
        // neighbouring tensors that fit together (a tensor that alone does not fit is a part of its own)
        uint64_t groups = 0;
        for (uint32_t i = 0; i < count; ++i)
            groups += groups_of(n_elems[i]);
        if (groups > slot_limit_groups()) {
            bool was_null[kBatchMax];
            for (uint32_t i = 0; i < count; ++i)
                was_null[i] = blobs[i] == nullptr;
            for (uint32_t first = 0; first < count;) {
                uint32_t m = 1;
                uint64_t part = groups_of(n_elems[first]);
                while (first + m < count && part + groups_of(n_elems[first + m]) <= slot_limit_groups()) {
                    part += groups_of(n_elems[first + m]);
                    ++m;
                }
                const int rc = compress_some(d_srcs + first, n_elems + first, m, k, block, elem, guard, reuse,
                                             rebuilt ? rebuilt + first : nullptr, stream, blobs + first,
                                             d_grads ? d_grads + first : nullptr, lr, keep_new, nullptr);
                if (rc != NEUZIP_OK) {
                    for (uint32_t j = 0; j < first; ++j) {
                        if (was_null[j]) {
                            neuzip_free(blobs[j]);
                            blobs[j] = nullptr;
                        }
                    }
                    return rc;
                }
                first += m;
            }
            return NEUZIP_OK;
        }
    }
    neuzip_blob *work[kBatchMax];
    bool fresh[kBatchMax];
    for (uint32_t i = 0; i < count; ++i) {
        work[i] = blobs[i];
        fresh[i] = false;
    }
    bool touched = false;     // kernels that write into the blobs have been launched
    bool ws_dirty = false;    // kernels have run whose sums in the workspace no later kernel has cleared
    auto fail = [&](int rc) {
        if (ws_dirty)
            reset_workspace(ws, stream);
        for (uint32_t i = 0; i < count; ++i) {
            if (fresh[i])
                neuzip_free(work[i]);
            else if (touched)
                work[i]->has_table = false;  // partly overwritten: holds no tensor until compressed again
        }
        return rc;
    };
    for (uint32_t i = 0; i < count; ++i) {
        if (!work[i]) {
            const int rc = alloc_blob(n_elems[i], k, block, elem, &work[i]);
            if (rc != NEUZIP_OK)
                return fail(rc);
            fresh[i] = true;
        }
        work[i]->have_counts = false;
        if (!reuse) {
            work[i]->total_words = 0;
            work[i]->has_table = false;
            if (guard != kKeepGuard)
                work[i]->guard = guard;
        }
    }

    // the batch proper: tensors that have elements
    CompressBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    uint32_t owner[kBatchMax];
    const void *stale_src[kBatchMax];
    const void *stale_grad[kBatchMax];
    uint64_t stale_n[kBatchMax];
    neuzip_blob *stale_blob[kBatchMax];
    uint32_t stale_owner[kBatchMax];
    uint32_t stale_count = 0;
    uint32_t hist_groups = 0, enc_groups = 0, compact_groups = 0, super_used = 0;
    // Shape of the histogram launch.  A batch that fits the last-level cache (measured on 58.7 M
    // elements: 33.7 -> 28.9 us) gets few workgroups of 1024 threads; one that streams through HBM
    // (measured on 525 M elements: 305 against 315-323 us) many of 256.
    uint64_t batch_bytes = 0;
    for (uint32_t i = 0; i < count; ++i)
        batch_bytes += work[i]->n * (elem == NEUZIP_F32 ? 4u : 2u);
    const uint32_t hist_threads = batch_bytes <= (128ull << 20) ? kHistThreadsMax : 256u;
    const uint32_t hist_cap = hist_threads == 256u ? 1280u : 512u;
    // a single tensor beyond the workspace limit: in tiles
    const bool tiled = !fixed_ws && count == 1 && groups_of(work[0]->n) > slot_limit_groups();
    if (tiled) {
        bool stale = false;
        touched = true;
        const int rc = compress_tiled(work[0], d_srcs[0], d_grads ? d_grads[0] : nullptr, k, block, elem, reuse, lr, keep_new,
                                      stream, &stale);
        if (rc != NEUZIP_OK)
            return fail(rc);
        if (stale) {
            stale_src[0] = d_srcs[0];
            stale_grad[0] = d_grads ? d_grads[0] : nullptr;
            stale_n[0] = n_elems[0];
            stale_blob[0] = work[0];
            stale_owner[0] = 0;
            stale_count = 1;
        }
    }
    for (uint32_t i = 0; i < count && !tiled; ++i) {
        neuzip_blob *b = work[i];
        if (b->n == 0) {
            const int rc = reuse ? NEUZIP_OK : compress_empty(b, stream);
            if (rc != NEUZIP_OK)
                return fail(rc);
            b->have_counts = true;
            continue;
        }
        CompressItem &it = batch.it[batch.count];
        owner[batch.count++] = i;
        it.src = d_srcs[i];
        it.n = b->n;
        it.table_n = b->n;
        it.tb = table_of(b);
        it.offsets = offsets_of(b);
        it.states = states_of(b);
        it.lens = lens_of(b);
        it.sm = sm_of(b);
        it.coef = coef_of(b);
        it.low = low_of(b);
        it.grad = d_grads ? static_cast<const uint16_t *>(d_grads[i]) : nullptr;
        it.words = nullptr;
        it.n_chunks = b->n_chunks;
        it.block = block;
        it.guard = b->guard;
        it.group_base = enc_groups;
        it.super_base = super_used;
        super_used += ((b->n_chunks + kChunksPerGroup - 1) / kChunksPerGroup + kSuperGroups - 1) / kSuperGroups;
        // every workgroup of the histogram pass pays for clearing and merging its 32 KB of bins: give
        // it at least 8 vectors (64 elements) per thread, and no tensor more workgroups than fit the chip
        uint64_t hg = ((b->n + 7) / 8 + hist_threads * 8 - 1) / (hist_threads * 8);
        hg = hg < 1 ? 1 : (hg > hist_cap ? hist_cap : hg);
        hist_groups += static_cast<uint32_t>(hg);
        enc_groups += (b->n_chunks + kChunksPerGroup - 1) / kChunksPerGroup;
        compact_groups += (b->n_chunks + kCompactThreads / 64 - 1) / (kCompactThreads / 64);
        it.hist_end = hist_groups;
        it.enc_end = enc_groups;
        it.compact_end = compact_groups;
    }
    if (batch.count > 0) {
        std::lock_guard<std::mutex> lock(g_ws_mutex);
        int rc = NEUZIP_OK;
        if (fixed_ws) {
            if (enc_groups > ws.group_cap)
                return fail(NEUZIP_EUNSUPPORTED);
            // the static array keeps what the last call left: bins, call states and sums start at zero
            reset_workspace(ws, stream);
        } else {
            rc = ensure_workspace(work[owner[0]]->device, enc_groups, stream);
            if (rc != NEUZIP_OK)
                return fail(rc);
        }
        batch.seq = ++ws.seq;
        batch.lr = lr;
        batch.keep_new = keep_new ? 1u : 0u;
        touched = true;
        // the call state and the sums per 64 groups exist twice; calls alternate between the copies
        const uint32_t copy = batch.seq & 1u;
        CallState *state = ws.state + copy, *state_next = ws.state + (copy ^ 1u);
        uint32_t *super_words = ws.super_words + copy * ws.super_cap;
        uint32_t *super_next = ws.super_words + (copy ^ 1u) * ws.super_cap;

        // Three launches.  The histogram pass (fresh statistics only).  The encoder, every workgroup of
        // which derives the table from the counts by itself; with fresh tables its launch carries one
        // more workgroup per tensor, which fills in the decoder's slot table meanwhile.  The compaction,
        // which also works out the chunk offsets, tells the host the stream lengths and returns the
        // workspace's sums to zero.
        const int variant = d_grads ? kUpdateVariant : (elem == NEUZIP_F32 ? 23 : (elem == NEUZIP_F16 ? 39 : k));
        if (!reuse) {
            launch_histogram(ws, batch, variant, block != 0, hist_groups, hist_threads, stream);
            if (!hip_ok(hipGetLastError()))
                return fail(NEUZIP_EHIP);
            ws_dirty = true;
        }
        if (!launch_encode(ws, batch, enc_groups + (reuse ? 0u : batch.count), variant, reuse, elem, block, super_words, state,
                           stream))
            return fail(NEUZIP_EHIP);
        ws_dirty = true;

        // The stream lengths are data dependent.  The compaction is launched right away all the same:
        // a blob that already has a word section (one that is compressed into again, as in a training
        // loop) has its words moved into the room it has, and the kernel itself leaves a tensor alone
        // whose words turn out not to fit, or whose kept table turned out stale.  It also writes the
        // lengths into pinned host memory, the stamp last, which is what the host then waits for.
        for (uint32_t j = 0; j < batch.count; ++j) {
            const neuzip_blob *b = work[owner[j]];
            batch.it[j].words = reinterpret_cast<uint16_t *>(b->words);
            batch.it[j].words_cap = words_room(b);
        }
        auto launch_compact = [&](bool report) {
            batch.report = report ? 1u : 0u;
            return launch_compaction(ws, batch, compact_groups, super_words, state, state_next, super_next, stream);
        };
        if (!launch_compact(true))
            return fail(NEUZIP_EHIP);
        ws_dirty = false;
        HostRecord::Item fetched[kBatchMax];  // fixed workspace: the record lies in device memory and is copied out
        if (fixed_ws) {
            if (!hip_ok(hipMemcpyAsync(fetched, &ws.pinned->item[0], sizeof(HostRecord::Item) * batch.count,
                                       hipMemcpyDeviceToHost, stream)) ||
                !hip_ok(hipStreamSynchronize(stream)))
                return fail(NEUZIP_EHIP);
        } else if (!wait_for_record(batch.seq, stream)) {
            return fail(NEUZIP_EHIP);
        }
        uint32_t n_stale = 0;
        bool late = false;
        for (uint32_t j = 0; j < batch.count; ++j) {
            const HostRecord::Item &r = fixed_ws ? fetched[j] : ws.pinned->item[j];
            neuzip_blob *b = work[owner[j]];
            if (reuse && r.stale) {
                // its table does not cover the new values: nothing of this pass is kept (the
                // compaction has left such a tensor alone); it is compressed afresh below
                stale_src[n_stale] = d_srcs[owner[j]];
                stale_grad[n_stale] = d_grads ? d_grads[owner[j]] : nullptr;
                stale_n[n_stale] = n_elems[owner[j]];
                stale_blob[n_stale] = b;
                stale_owner[n_stale++] = owner[j];
                b->has_table = false;
                batch.it[j].n_chunks = 0;
                continue;
            }
            if (r.total_words[1] != 0)
                return fail(NEUZIP_EUNSUPPORTED);  // more than 2^32 words
            if (r.total_words[0] <= batch.it[j].words_cap) {
                batch.it[j].n_chunks = 0;  // in place already: the kernel took the same decision
            } else {
                if (fixed_ws)  // no allocation: the stream must fit the room the blob has
                    return fail(NEUZIP_ENOMEM);
                rc = reserve_words(b, r.total_words[0]);
                if (rc != NEUZIP_OK)
                    return fail(rc);
                batch.it[j].words = reinterpret_cast<uint16_t *>(b->words);
                batch.it[j].words_cap = words_room(b);
                late = true;
            }
            b->total_words = r.total_words[0];
            if (!reuse) {
                std::memcpy(b->h_counts, r.counts, 1024);
                std::memcpy(b->h_freq, r.freq, 512);
                b->have_counts = true;
            }
            b->has_table = true;
        }
        // the tensors that had no room (or no word section yet), now that it is allocated
        if (late && !launch_compact(false))
            return fail(NEUZIP_EHIP);
        if (!fixed_ws && !hip_ok(hipEventRecord(ws.idle, stream)))
            return fail(NEUZIP_EHIP);
        stale_count = n_stale;
    }
    if (stale_count > 0) {
        // a fused weight step that did not write the new weights back: form them now, in place
        if (d_grads && !keep_new) {
            for (uint32_t j = 0; j < stale_count; ++j) {
                const uint64_t vecs = (stale_n[j] + 7) / 8;
                const uint32_t wgs = static_cast<uint32_t>(vecs / 256 + 1 < 4096 ? vecs / 256 + 1 : 4096);
                hipLaunchKernelGGL(sgd_update_kernel, dim3(wgs), dim3(256), 0, stream,
                                   static_cast<uint16_t *>(const_cast<void *>(stale_src[j])),
                                   static_cast<const uint16_t *>(stale_grad[j]), stale_n[j], lr);
            }
            if (!hip_ok(hipGetLastError()))
                return NEUZIP_EHIP;
        }
        // same stream, so the pass above has finished with the workspace before this one starts
        const int rc = compress_some(stale_src, stale_n, stale_count, k, block, elem, kKeepGuard, false, nullptr, stream,
                                     stale_blob);
        if (rc != NEUZIP_OK)
            return rc;
        for (uint32_t j = 0; j < stale_count; ++j)
            if (rebuilt)
                rebuilt[stale_owner[j]] = 1;
    }
    for (uint32_t i = 0; i < count; ++i)
        blobs[i] = work[i];
    return NEUZIP_OK;
}

int compress_batch(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int dtype, int mantissa_bits,
                   uint32_t block_size, uint32_t guard, void *hip_stream, neuzip_blob **blobs);

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

int neuzip_set_workspace_limit(uint64_t slot_bytes)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    g_slot_limit = slot_bytes == 0 ? kDefaultSlotLimit : slot_bytes;
    // a workspace that was grown beyond the new limit is given back
    if (g_ws.device >= 0 && g_ws.group_cap > slot_limit_groups())
        return release_workspace_locked();
    return NEUZIP_OK;
}

int neuzip_compress_blockwise(const void *d_src, uint64_t n_elems, int dtype, int mantissa_bits,
                              uint32_t block_size, void *hip_stream, neuzip_blob **blob)
{
    return neuzip_compress_batch(&d_src, &n_elems, 1, dtype, mantissa_bits, block_size, hip_stream, blob);
}

int neuzip_compress_batch(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int dtype,
                          int mantissa_bits, uint32_t block_size, void *hip_stream, neuzip_blob **blobs)
{
    // (a blob that is compressed into again keeps the guard band it was made with)
    return compress_batch(d_srcs, n_elems, count, dtype, mantissa_bits, block_size, kKeepGuard, hip_stream, blobs);
}

int neuzip_compress_guarded(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int dtype,
                            int mantissa_bits, uint32_t guard, void *hip_stream, neuzip_blob **blobs)
{
    if (guard > 255)
        return NEUZIP_EINVAL;
    return compress_batch(d_srcs, n_elems, count, dtype, mantissa_bits, 0, guard, hip_stream, blobs);
}

int neuzip_recompress(const void *const *d_srcs, uint32_t count, void *hip_stream, neuzip_blob *const *blobs,
                      uint32_t *rebuilt)
{
    if (count == 0)
        return NEUZIP_OK;
    if (!d_srcs || !blobs)
        return NEUZIP_EINVAL;
    for (uint32_t i = 0; i < count; ++i) {
        const neuzip_blob *b = blobs[i];
        if (!is_blob(b) || !b->has_table || !on_current_device(b))
            return NEUZIP_EINVAL;
        if (b->n > 0 && (!d_srcs[i] || (reinterpret_cast<uintptr_t>(d_srcs[i]) & 15u)))
            return NEUZIP_EINVAL;
        for (uint32_t j = 0; j < i; ++j)
            if (blobs[j] == b)
                return NEUZIP_EINVAL;
    }
    if (rebuilt)
        for (uint32_t i = 0; i < count; ++i)
            rebuilt[i] = 0;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // neighbouring tensors of the same kind share a pass, up to kBatchMax at a time; block-wise
    // normalised blobs need the block maxima first and always take the two-pass route
    uint32_t first = 0;
    while (first < count) {
        const neuzip_blob *lead = blobs[first];
        uint32_t m = 1;
        while (first + m < count && m < kBatchMax && blobs[first + m]->k == lead->k &&
               blobs[first + m]->block == lead->block && blobs[first + m]->elem == lead->elem)
            ++m;
        uint64_t n_elems[kBatchMax];
        neuzip_blob *group[kBatchMax];
        for (uint32_t j = 0; j < m; ++j) {
            n_elems[j] = blobs[first + j]->n;
            group[j] = blobs[first + j];
        }
        const bool reuse = lead->block == 0;
        const int rc = compress_some(d_srcs + first, n_elems, m, lead->k, lead->block, lead->elem, kKeepGuard, reuse,
                                     rebuilt ? rebuilt + first : nullptr, stream, group);
        if (rc != NEUZIP_OK)
            return rc;
        if (!reuse && rebuilt)
            for (uint32_t j = 0; j < m; ++j)
                rebuilt[first + j] = 1;
        first += m;
    }
    return NEUZIP_OK;
}

int neuzip_update(neuzip_blob *const *blobs, const void *const *d_grads, void *const *d_weights, uint32_t count, float lr,
                  int weights_ready, void *hip_stream, uint32_t *rebuilt)
{
    if (count == 0)
        return NEUZIP_OK;
    if (!blobs || !d_grads || !d_weights || weights_ready < 0 || weights_ready > 3)
        return NEUZIP_EINVAL;
    for (uint32_t i = 0; i < count; ++i) {
        const neuzip_blob *b = blobs[i];
        if (!is_blob(b) || !b->has_table || !on_current_device(b))
            return NEUZIP_EINVAL;
        if (b->k != 7 || b->block != 0 || b->elem != NEUZIP_BF16)
            return NEUZIP_EUNSUPPORTED;  // training keeps bf16 weights without loss
        if (b->n > 0 && (!d_grads[i] || !d_weights[i] || d_grads[i] == d_weights[i] ||
                         (reinterpret_cast<uintptr_t>(d_grads[i]) & 15u) ||
                         (reinterpret_cast<uintptr_t>(d_weights[i]) & 15u)))
            return NEUZIP_EINVAL;
        for (uint32_t j = 0; j < i; ++j)
            if (blobs[j] == b)
                return NEUZIP_EINVAL;
    }
    if (rebuilt)
        for (uint32_t i = 0; i < count; ++i)
            rebuilt[i] = 0;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // Two routes, chosen by what the caller holds (measured on a 4096 x 14336 weight: 148 and 122 us;
    // either route in the other's place costs 10-20 % more, because of the bytes it moves).
    // a) Only the blob: the decoder applies the step on its way out, so that d_weights receives the
    //    new weight at once (the old one is never written), and the plain kept-table encoder follows.
    // b) The decompressed weight is at hand: one pass of the encoder over weight and gradient forms
    //    the new weight, writes it back (unless the caller has no use for it) and codes it.
    // c) Only the blob, and no use for the new weight uncompressed: a plain decompression into
    //    d_weights, then (b) without the write-back (135 us; the fewest bytes of all).
    if (weights_ready == NEUZIP_UPDATE_FROM_BLOB_DISCARD) {
        const int rc = neuzip_decompress_batch(blobs, d_weights, count, hip_stream);
        if (rc != NEUZIP_OK)
            return rc;
    }
    if (weights_ready == NEUZIP_UPDATE_FROM_BLOB) {
        uint64_t batch_elems = 0;
        for (uint32_t i = 0; i < count; ++i)
            batch_elems += blobs[i]->n;
        const bool stream_out = batch_elems >= (64ull << 20);
        BatchArgs args;
        args.count = 0;
        uint32_t groups = 0;
        for (uint32_t i = 0; i <= count; ++i) {
            const bool flush = (i == count) || (args.count == kBatchMax);
            if (flush && args.count > 0) {
                const int rc = launch_batch(args, kUpdateVariant, groups, stream);
                if (rc != NEUZIP_OK)
                    return rc;
                args.count = 0;
                groups = 0;
            }
            if (i == count)
                break;
            const neuzip_blob *b = blobs[i];
            if (b->n == 0)
                continue;
            DecodeArgs a = decode_args(b, d_weights[i]);
            a.grad = static_cast<const uint16_t *>(d_grads[i]);
            a.lr = lr;
            a.stream_out = stream_out ? 1u : 0u;
            groups += (b->n_chunks + kDecChunksPerWg - 1) / kDecChunksPerWg;
            a.wg_end = groups;
            args.t[args.count++] = a;
        }
    }
    // the new weights are coded with the tables the blobs hold (fresh tables where those do not serve)
    for (uint32_t first = 0; first < count; first += kBatchMax) {
        const uint32_t m = count - first < kBatchMax ? count - first : kBatchMax;
        uint64_t n_elems[kBatchMax];
        neuzip_blob *group[kBatchMax];
        for (uint32_t j = 0; j < m; ++j) {
            n_elems[j] = blobs[first + j]->n;
            group[j] = blobs[first + j];
        }
        const int rc = compress_some(d_weights + first, n_elems, m, 7, 0, NEUZIP_BF16, kKeepGuard, true,
                                     rebuilt ? rebuilt + first : nullptr, stream, group,
                                     weights_ready != NEUZIP_UPDATE_FROM_BLOB ? d_grads + first : nullptr, lr,
                                     weights_ready == NEUZIP_UPDATE_WEIGHTS_READY);
        if (rc != NEUZIP_OK)
            return rc;
    }
    return NEUZIP_OK;
}

uint32_t neuzip_guard(const neuzip_blob *blob) { return is_blob(blob) ? blob->guard : 0; }

int neuzip_linear(const neuzip_blob *weight, uint64_t out_features, uint64_t in_features, const void *d_x,
                  uint32_t tokens, const float *d_bias, float *d_y, void *hip_stream)
{
    return neuzip_linear_batch(&weight, &out_features, 1, in_features, d_x, tokens, &d_bias, &d_y, hip_stream);
}

int neuzip_linear_batch(const neuzip_blob *const *weights, const uint64_t *out_features, uint32_t count,
                        uint64_t in_features, const void *d_x, uint32_t tokens, const float *const *d_bias,
                        float *const *d_y, void *hip_stream)
{
    if (count == 0)
        return NEUZIP_OK;
    if (!weights || !out_features || !d_y || !d_x || tokens == 0 || count > kLinBatchMax)
        return NEUZIP_EINVAL;
    if (in_features == 0 || in_features % kTurn != 0 || in_features >= (1ull << 31) ||
        (reinterpret_cast<uintptr_t>(d_x) & 15u))
        return NEUZIP_EINVAL;
    for (uint32_t i = 0; i < count; ++i) {
        const neuzip_blob *w = weights[i];
        if (!is_blob(w) || !w->has_table || !on_current_device(w) || !d_y[i])
            return NEUZIP_EINVAL;
        if (out_features[i] == 0 || out_features[i] >= (1ull << 31) || out_features[i] * in_features != w->n)
            return NEUZIP_EINVAL;
        if ((reinterpret_cast<uintptr_t>(d_y[i]) & 3u) || (d_bias && (reinterpret_cast<uintptr_t>(d_bias[i]) & 3u)))
            return NEUZIP_EINVAL;
        if (w->elem != NEUZIP_BF16)
            return NEUZIP_EUNSUPPORTED;
        // one launch serves one kind of weight
        if (w->k != weights[0]->k || (w->block != 0) != (weights[0]->block != 0))
            return NEUZIP_EINVAL;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint64_t gcd = in_features, r = kChunk;
    while (r) {
        const uint64_t t = gcd % r;
        gcd = r;
        r = t;
    }
    LinearBatchArgs batch;
    LinearInitBatchArgs init;
    std::memset(&batch, 0, sizeof(batch));
    std::memset(&init, 0, sizeof(init));
    batch.count = init.count = count;
    init.tokens = tokens;
    uint32_t init_wgs = 0;
    for (uint32_t i = 0; i < count; ++i) {
        const neuzip_blob *w = weights[i];
        LinearArgs &a = batch.t[i];
        a.tb = table_of(w);
        a.offsets = offsets_of(w);
        a.states = states_of(w);
        a.lens = lens_of(w);
        a.words = reinterpret_cast<const uint16_t *>(w->words);
        a.sm = sm_of(w);
        a.status = table_of(w)->status;
        a.n = w->n;
        a.n_chunks = w->n_chunks;
        a.in_features = static_cast<uint32_t>(in_features);
        a.out_features = static_cast<uint32_t>(out_features[i]);
        a.coef = coef_of(w);
        a.block_shift = 0;
        while (w->block && (1u << a.block_shift) < w->block)
            ++a.block_shift;
        a.stride = static_cast<uint32_t>(in_features / gcd);
        a.rstep = static_cast<uint32_t>(kChunk / gcd);
        const uint64_t cells = static_cast<uint64_t>(tokens) * out_features[i];
        init.y[i] = d_y[i];
        init.bias[i] = d_bias ? d_bias[i] : nullptr;
        init.out_features[i] = a.out_features;
        init_wgs += static_cast<uint32_t>((cells + 255) / 256);
        init.wg_end[i] = init_wgs;
    }
    if (count == 1)
        hipLaunchKernelGGL(linear_init_kernel, dim3(init_wgs), dim3(256), 0, stream, init.y[0], init.bias[0], tokens,
                           init.out_features[0]);
    else
        hipLaunchKernelGGL(linear_init_batch_kernel, dim3(init_wgs), dim3(256), 0, stream, init);
    // the kernel holds the partial sums of at most 64 tokens: larger batches go through in tiles of 64
    // (each tile decodes the weights again: beyond a few tiles decompressing once and a dense product win)
    const neuzip_blob *first = weights[0];
    for (uint32_t t0 = 0; t0 < tokens; t0 += kLinMaxTokens) {
        const uint32_t tile = tokens - t0 < kLinMaxTokens ? tokens - t0 : kLinMaxTokens;
        const uint32_t cols = linear_columns(tile, batch.t[0].stride);  // chunks per group = columns of the matrix instruction
        const uint32_t groups_per_wg = kDecChunksPerWg / cols;
        uint32_t wgs = 0;
        for (uint32_t i = 0; i < count; ++i) {
            LinearArgs &a = batch.t[i];
            a.tokens = tile;
            a.x = static_cast<const uint16_t *>(d_x) + static_cast<uint64_t>(t0) * in_features;
            a.y = d_y[i] + static_cast<uint64_t>(t0) * out_features[i];
            const uint64_t per_block = static_cast<uint64_t>(cols) * a.stride;
            a.n_groups = static_cast<uint32_t>((weights[i]->n_chunks + per_block - 1) / per_block * a.stride);
            wgs += (a.n_groups + groups_per_wg - 1) / groups_per_wg;
            batch.wg_end[i] = wgs;
        }
        if (first->block) {
            switch (first->k) {
            case 3: launch_linear<3, true>(batch, cols, wgs, stream); break;
            case 1: launch_linear<1, true>(batch, cols, wgs, stream); break;
            default: launch_linear<0, true>(batch, cols, wgs, stream); break;
            }
        } else {
            switch (first->k) {
            case 7: launch_linear<7, false>(batch, cols, wgs, stream); break;
            case 3: launch_linear<3, false>(batch, cols, wgs, stream); break;
            case 1: launch_linear<1, false>(batch, cols, wgs, stream); break;
            default: launch_linear<0, false>(batch, cols, wgs, stream); break;
            }
        }
        if (!hip_ok(hipGetLastError()))
            return NEUZIP_EHIP;
    }
    return hip_ok(hipGetLastError()) ? NEUZIP_OK : NEUZIP_EHIP;
}

}  // extern "C"

namespace {

int compress_batch(const void *const *d_srcs, const uint64_t *n_elems, uint32_t count, int dtype, int mantissa_bits,
                   uint32_t block_size, uint32_t guard, void *hip_stream, neuzip_blob **blobs)
{
    if (count == 0)
        return NEUZIP_OK;
    if (!d_srcs || !n_elems || !blobs || (dtype != NEUZIP_BF16 && dtype != NEUZIP_F32 && dtype != NEUZIP_F16) ||
        !valid_k(mantissa_bits))
        return NEUZIP_EINVAL;
    if (block_size != 0 && (!valid_block(block_size) || mantissa_bits == 7))
        return NEUZIP_EINVAL;
    if (dtype != NEUZIP_BF16 && mantissa_bits != 7)
        return NEUZIP_EUNSUPPORTED;  // binary32 and binary16 tensors are compressed without loss only
    for (uint32_t i = 0; i < count; ++i) {
        if (n_elems[i] > 0 && (!d_srcs[i] || (reinterpret_cast<uintptr_t>(d_srcs[i]) & 15u)))
            return NEUZIP_EINVAL;
        if (n_elems[i] >= (1ull << 32))
            return NEUZIP_EUNSUPPORTED;
        const neuzip_blob *b = blobs[i];
        if (b && (!is_blob(b) || b->n != n_elems[i] || b->k != mantissa_bits || b->block != block_size ||
                  b->elem != dtype || !on_current_device(b)))
            return NEUZIP_EINVAL;
        for (uint32_t j = 0; j < i; ++j)
            if (b && blobs[j] == b)
                return NEUZIP_EINVAL;  // one blob cannot receive two tensors
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (uint32_t first = 0; first < count; first += kBatchMax) {
        const uint32_t m = count - first < kBatchMax ? count - first : kBatchMax;
        const int rc = compress_some(d_srcs + first, n_elems + first, m, mantissa_bits, block_size, dtype, guard, false,
                                     nullptr, stream, blobs + first);
        if (rc != NEUZIP_OK)
            return rc;
    }
    return NEUZIP_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Compression for callers that cannot allocate: the compress workspace of one tensor of at most
// NEUZIP_NOALLOC_MAX_ELEMS elements, carved out of a device array that is part of the library's
// code object.  Each GPU holds its own copy of the array at its own address; the address is asked
// for once per device (with that device current) and only that pointer is ever handed to kernels
// or copies -- the array's name is not a device address in host code.
// ------------------------------------------------------------------------------------------
namespace {

constexpr uint32_t kFixedChunks = static_cast<uint32_t>(NEUZIP_NOALLOC_MAX_ELEMS / kChunk);
constexpr uint32_t kFixedGroups = kFixedChunks / kChunksPerGroup;
static_assert(NEUZIP_NOALLOC_MAX_ELEMS % (kChunk * kChunksPerGroup) == 0, "whole encoder groups");
constexpr uint64_t kFixedCountsAt = 0;                                                     // bins, call states, counter
constexpr uint64_t kFixedRecordAt = kFixedCountsAt + pad_to(kSmallWords * 4, 256);
constexpr uint64_t kFixedChunkWordsAt = kFixedRecordAt + pad_to(sizeof(HostRecord), 256);
constexpr uint64_t kFixedGroupWordsAt = kFixedChunkWordsAt + pad_to((kFixedChunks + 4) * 4, 256);
constexpr uint32_t kFixedSuperCap = kFixedGroups / kSuperGroups + kBatchMax + 1;
constexpr uint64_t kFixedSuperAt = kFixedGroupWordsAt + pad_to((kFixedGroups + 4) * 4, 256);
constexpr uint64_t kFixedSlotsAt = kFixedSuperAt + pad_to(2 * kFixedSuperCap * 4, 256);
constexpr uint64_t kFixedBytes = kFixedSlotsAt + static_cast<uint64_t>(kFixedChunks) * kStates * kRunCap * 2;

static __device__ __align__(256) unsigned char scratch[kFixedBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint8_t *g_scratch_ptr[kMaxDevices];   // per device: where that device holds the array
uint32_t g_scratch_seq[kMaxDevices];   // per device: stamp of the last call

// The array of the current device, asked for on the first call there.
int scratch_of_current_device(int *device, uint8_t **ptr)
{
    NZ_HIP(hipGetDevice(device));
    if (*device < 0 || *device >= kMaxDevices)
        return NEUZIP_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[*device]) {
        void *at = nullptr;
        NZ_HIP(hipGetSymbolAddress(&at, HIP_SYMBOL(scratch)));
        if (!at)
            return NEUZIP_EHIP;
        g_scratch_ptr[*device] = static_cast<uint8_t *>(at);
    }
    *ptr = g_scratch_ptr[*device];
    return NEUZIP_OK;
}

}  // namespace

extern "C" {

int neuzip_compress_noalloc(const void *d_src, uint64_t n_elems, int dtype, int mantissa_bits, void *hip_stream,
                            neuzip_blob *blob)
{
    if ((dtype != NEUZIP_BF16 && dtype != NEUZIP_F32 && dtype != NEUZIP_F16) || !valid_k(mantissa_bits))
        return NEUZIP_EINVAL;
    if (dtype != NEUZIP_BF16 && mantissa_bits != 7)
        return NEUZIP_EUNSUPPORTED;
    if (!is_blob(blob) || blob->n != n_elems || blob->k != mantissa_bits || blob->elem != dtype ||
        !on_current_device(blob))
        return NEUZIP_EINVAL;
    if (blob->block != 0)
        return NEUZIP_EUNSUPPORTED;
    if (n_elems > NEUZIP_NOALLOC_MAX_ELEMS)
        return NEUZIP_EUNSUPPORTED;
    if (n_elems > 0 && (!d_src || (reinterpret_cast<uintptr_t>(d_src) & 15u)))
        return NEUZIP_EINVAL;
    int device = -1;
    uint8_t *base = nullptr;
    const int rc = scratch_of_current_device(&device, &base);
    if (rc != NEUZIP_OK)
        return rc;
    Workspace ws;
    ws.device = device;
    ws.counts = reinterpret_cast<uint32_t *>(base + kFixedCountsAt);
    ws.state = reinterpret_cast<CallState *>(ws.counts + kBatchMax * 256);
    ws.all_done = ws.counts + kBatchMax * 256 + 2 * sizeof(CallState) / 4;
    ws.super_words = reinterpret_cast<uint32_t *>(base + kFixedSuperAt);
    ws.super_cap = kFixedSuperCap;
    ws.pinned = reinterpret_cast<HostRecord *>(base + kFixedRecordAt);  // device memory here: copied out, not read in place
    ws.chunk_words = reinterpret_cast<uint32_t *>(base + kFixedChunkWordsAt);
    ws.group_words = reinterpret_cast<uint32_t *>(base + kFixedGroupWordsAt);
    ws.slots = reinterpret_cast<uint16_t *>(base + kFixedSlotsAt);
    ws.group_cap = kFixedGroups;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        ws.seq = g_scratch_seq[device]++;
    }
    return compress_some(&d_src, &n_elems, 1, mantissa_bits, 0, dtype, kKeepGuard, false, nullptr,
                         static_cast<hipStream_t>(hip_stream), &blob, nullptr, 0.0f, true, &ws);
}

int neuzip_decompress(const neuzip_blob *blob, void *d_dst, uint64_t n_elems, int dtype, void *hip_stream)
{
    if (!is_blob(blob) || !blob->has_table || dtype != blob->elem ||
        blob->n != n_elems || !on_current_device(blob))
        return NEUZIP_EINVAL;
    if (n_elems > 0 && (!d_dst || (reinterpret_cast<uintptr_t>(d_dst) & 15u)))
        return NEUZIP_EINVAL;
    return decode_dispatch(blob, d_dst, static_cast<hipStream_t>(hip_stream));
}

int neuzip_decompress_sequence(const neuzip_blob *const *blobs, uint32_t count, void *d_scratch,
                               uint64_t scratch_elems, uint64_t *h_offsets, void *hip_stream)
{
    if (count > 0 && !blobs)
        return NEUZIP_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_scratch) & 15u)
        return NEUZIP_EINVAL;
    auto words_of = [](const neuzip_blob *b) { return b->elem == NEUZIP_F32 ? 2 * b->n : b->n; };
    for (uint32_t i = 0; i < count; ++i) {
        if (!is_blob(blobs[i]) || !blobs[i]->has_table || words_of(blobs[i]) > scratch_elems ||
            (blobs[i]->n > 0 && !d_scratch) || !on_current_device(blobs[i]))
            return NEUZIP_EINVAL;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // Neighbouring blobs of one kind that fit the space together are placed one behind the other, each
    // at a 256-byte boundary, and share a launch (up to kBatchMax of them): tensors too small to fill
    // the chip on their own then overlap.  The next group starts at the front of the space again.
    uint32_t first = 0;
    while (first < count) {
        BatchArgs args;
        args.count = 0;
        uint32_t groups = 0;
        uint64_t at = 0;  // 16-bit words from the start of the space
        const int kind = decode_variant(blobs[first]);
        uint32_t i = first, live = first;  // live: the last blob of the group that has elements
        for (; i < count && args.count < kBatchMax; ++i) {
            const neuzip_blob *b = blobs[i];
            if (decode_variant(b) != kind || at + words_of(b) > scratch_elems)
                break;
            if (h_offsets)
                h_offsets[i] = at;
            if (b->n > 0) {
                DecodeArgs a = decode_args(b, static_cast<uint16_t *>(d_scratch) + at);
                groups += (b->n_chunks + batch_chunks_per_wg(kind) - 1) / batch_chunks_per_wg(kind);
                a.wg_end = groups;
                args.t[args.count++] = a;
                live = i;
            }
            at = pad_to(at + words_of(b), 128);
        }
        if (args.count == 1) {
            // a tensor on its own takes the single-tensor launch (its workgroup size follows the tensor's size)
            const int rc = decode_dispatch(blobs[live], args.t[0].out, stream);
            if (rc != NEUZIP_OK)
                return rc;
        } else if (args.count > 1) {
            const bool stream_out = at >= (64ull << 20);  // the group as a whole exceeds the cache
            for (uint32_t t = 0; t < args.count; ++t)
                args.t[t].stream_out = stream_out ? 1u : 0u;
            const int rc = launch_batch(args, kind, groups, stream);
            if (rc != NEUZIP_OK)
                return rc;
        }
        first = i;
    }
    return NEUZIP_OK;
}

int neuzip_decompress_batch(const neuzip_blob *const *blobs, void *const *d_dsts, uint32_t count, void *hip_stream)
{
    if (count > 0 && (!blobs || !d_dsts))
        return NEUZIP_EINVAL;
    for (uint32_t i = 0; i < count; ++i) {
        if (!is_blob(blobs[i]) || !blobs[i]->has_table || !on_current_device(blobs[i]))
            return NEUZIP_EINVAL;
        if (blobs[i]->n > 0 && (!d_dsts[i] || (reinterpret_cast<uintptr_t>(d_dsts[i]) & 15u)))
            return NEUZIP_EINVAL;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint64_t batch_elems = 0;
    for (uint32_t i = 0; i < count; ++i)
        batch_elems += (blobs[i]->elem == NEUZIP_F32) ? 2 * blobs[i]->n : blobs[i]->n;
    const bool stream_out = batch_elems >= (64ull << 20);  // the batch as a whole exceeds the cache
    // tensors of the same kind (mantissa_bits, normalised or not) share launches of up to
    // kBatchMax tensors, in the given order
    static const int kinds[9] = {7, 3, 1, 0, 11, 9, 8, 23, 39};
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
            a.stream_out = stream_out ? 1u : 0u;
            groups += (b->n_chunks + batch_chunks_per_wg(k) - 1) / batch_chunks_per_wg(k);
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
        (void)hipSetDevice(blob->device);
    if (blob->fixed)
        (void)hipFree(blob->fixed);
    if (blob->words)
        (void)hipFree(blob->words);
    if (have_cur && cur != blob->device)
        (void)hipSetDevice(cur);
    blob->magic = 0;
    delete blob;
}

uint64_t neuzip_compressed_bytes(const neuzip_blob *blob)
{
    if (!is_blob(blob))
        return 0;
    return container_layout(blob->n, blob->k, blob->total_words, blob->block, (blob->elem == NEUZIP_F32)).total;
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

int neuzip_dtype(const neuzip_blob *blob) { return is_blob(blob) ? blob->elem : -1; }

int neuzip_export(const neuzip_blob *blob, void *h_buf, uint64_t cap, uint64_t *written, void *hip_stream)
{
    if (!is_blob(blob) || !blob->has_table || (h_buf && !on_current_device(blob)))
        return NEUZIP_EINVAL;
    const Container lay = container_layout(blob->n, blob->k, blob->total_words, blob->block, (blob->elem == NEUZIP_F32));
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
    put32(52, blob->guard);
    put32(56, static_cast<uint32_t>(blob->elem));  // element type
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
    if (blob->n && (blob->elem == NEUZIP_F32))
        NZ_HIP(hipMemcpyAsync(p + lay.low, low_of(blob), blob->n * 2, hipMemcpyDeviceToHost, stream));
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
    const uint32_t guard = get32(52);
    if (guard > 255 || (guard != 0 && block != 0))
        return NEUZIP_ECORRUPT;
    const uint32_t elem = get32(56);
    if (elem > NEUZIP_F16 || (elem != NEUZIP_BF16 && (k != 7 || block != 0)))
        return NEUZIP_ECORRUPT;
    const bool f32 = elem == NEUZIP_F32;
    const uint32_t nc = chunks_of(n);
    if (get32(36) != nc)
        return NEUZIP_ECORRUPT;
    const Container lay = container_layout(n, k, total_words, block, f32);
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
    int rc = alloc_blob(n, k, block, static_cast<int>(elem), &b);
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
    b->guard = guard;
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
    if (n && f32 && !hip_ok(hipMemcpyAsync(low_of(b), p + lay.low, n * 2, hipMemcpyHostToDevice, stream)))
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
    b->has_table = true;
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

int neuzip_stream_probe(const void *d_in, uint64_t in_bytes, void *d_out, uint64_t out_bytes, void *hip_stream)
{
    if ((reinterpret_cast<uintptr_t>(d_in) & 15u) || (reinterpret_cast<uintptr_t>(d_out) & 15u) || (in_bytes & 15u) ||
        (out_bytes & 15u) || !d_out || !d_in)
        return NEUZIP_EINVAL;
    // whole chunks of 8 KB of output; the last 16 bytes of the output are the kernel's sink word
    const uint64_t chunks64 = (out_bytes - 16) / (2 * kChunk);
    if (out_bytes < 2 * kChunk + 16 || chunks64 >= (1ull << 31))
        return NEUZIP_EINVAL;
    const uint32_t n_chunks = static_cast<uint32_t>(chunks64);
    const uint32_t wgs = (n_chunks + kDecChunksPerWg - 1) / kDecChunksPerWg;
    // the input is split the way a container's is: per lane and turn the widest field (8, 4, 2 or 1
    // bytes) the input affords, the rest as "words", an equal share per workgroup
    const uint64_t per_chunk = in_bytes / n_chunks;
    const uint32_t fw = per_chunk >= 8 * kTurns * kStates ? 8u : (per_chunk >= 4 * kTurns * kStates ? 4u
                        : (per_chunk >= 2 * kTurns * kStates ? 2u : (per_chunk >= kTurns * kStates ? 1u : 0u)));
    if (fw == 0)
        return NEUZIP_EINVAL;  // less input than one byte per eight outputs: not a decoder's mix
    const uint64_t field_bytes = static_cast<uint64_t>(wgs) * kDecChunksPerWg * kTurns * kStates * fw;
    if (field_bytes > in_bytes)
        return NEUZIP_EINVAL;
    const uint64_t vecs = (in_bytes - field_bytes) / 16 / wgs;
    const uint32_t word_vecs = static_cast<uint32_t>(vecs < kStageBytes / 16 ? vecs : kStageBytes / 16);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint8_t *fields = static_cast<const uint8_t *>(d_in);
    const uint4 *words = reinterpret_cast<const uint4 *>(fields + field_bytes);
    uint4 *out = static_cast<uint4 *>(d_out);
    uint32_t *sink = reinterpret_cast<uint32_t *>(static_cast<uint8_t *>(d_out) + out_bytes - 16);
    const bool stream_out = out_bytes >= (128ull << 20);
#define NZ_PROBE(FW)                                                                                                 \
    do {                                                                                                             \
        if (stream_out)                                                                                              \
            hipLaunchKernelGGL((stream_probe_kernel<FW, true>), dim3(wgs), dim3(kDecThreads), 0, stream, fields, words, \
                               word_vecs, out, n_chunks, sink);                                                      \
        else                                                                                                         \
            hipLaunchKernelGGL((stream_probe_kernel<FW, false>), dim3(wgs), dim3(kDecThreads), 0, stream, fields, words, \
                               word_vecs, out, n_chunks, sink);                                                      \
    } while (0)
    switch (fw) {
    case 8: NZ_PROBE(8); break;
    case 4: NZ_PROBE(4); break;
    case 2: NZ_PROBE(2); break;
    default: NZ_PROBE(1); break;
    }
#undef NZ_PROBE
    return hip_ok(hipGetLastError()) ? NEUZIP_OK : NEUZIP_EHIP;
}

int neuzip_check(const neuzip_blob *blob, void *hip_stream)
{
    if (!is_blob(blob) || !on_current_device(blob))
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

uint64_t neuzip_workspace_bytes(void)
{
    std::lock_guard<std::mutex> guard(g_ws_mutex);
    if (g_ws.device < 0)
        return 0;
    const uint64_t chunks = g_ws.group_cap * kChunksPerGroup;
    uint64_t bytes = kSmallWords * 4;
    if (g_ws.group_cap)
        bytes += (chunks + 4) * 4 + (g_ws.group_cap + 4) * 4 + 2ull * g_ws.super_cap * 4 + chunks * kStates * kRunCap * 2;
    return bytes;
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
