// Prefetch of a batch's candidate documents from a host-resident table into an HBM staging slot:
// the one-GPU analogue of fetching the re-ranking embeddings from a slower tier into GPU memory
// ahead of scoring (Sec. 4.1, Sec. 4.2: fetch overlapped with other work, so that only what is
// left over shows on the critical path).  Everything runs on the GPU, on a side stream:
//
//   clear   zero the slot's document bitmap and its counters
//   mark    one thread per (query, candidate): set the document's bit; the thread that sets it
//           first reserves the document's rows in the slot (wave-aggregated atomic add), appends
//           the id to the slot's list of distinct documents and notes where the rows come from:
//           ANOTHER slot if an earlier batch's prefetch left the document there (a popular
//           document is fetched from the slow tier once and then handed from slot to slot), else
//           the host table.  A document listed by many queries is copied once.
//   gather  one wave per distinct document: copy its rows into the slot, from another slot
//           (HBM to HBM) or from pinned host memory (read across PCIe by the kernel itself,
//           16 bytes per lane, lane-linear).
//
// The order of documents inside a slot depends on the order in which atomics land; nothing that is
// computed from the slot depends on it.
//
// The other engine (espn_prefetch_packed) finds the distinct documents and packs their rows on the
// host and sends them with plain copies; of the kernels here it uses clear and `publish`, which
// writes the host's findings (distinct ids and the slot row each document starts at) into the
// slot's bitmap and row map.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "maxsim_kernels.h"

namespace espn {

// What a prefetch may take from the table's other slots: the documents their last prefetches placed
// there.  Listed most recently filled first (the likeliest holder of a popular document).
constexpr int MAX_SLOTS = 8;
struct OtherSlots {
    int n;
    const unsigned *bits[MAX_SLOTS - 1];
    const int64_t *row_map[MAX_SLOTS - 1];
    const uint4 *rows[MAX_SLOTS - 1];
};
// "row r of other slot x" as one word; -1 stands for the host table
constexpr int OTHER_SHIFT = 48;

// counters: [0] distinct documents, [1] rows reserved, [2] rows taken from other slots,
//           [3] documents handed out to the copy kernel's waves
__global__ void staging_clear_kernel(unsigned *__restrict__ bits, int64_t n_words,
                                     unsigned long long *__restrict__ counters)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += stride) bits[i] = 0u;
    if (blockIdx.x == 0 && threadIdx.x < 4) counters[threadIdx.x] = 0ull;
}

__global__ __launch_bounds__(256) void staging_mark_kernel(
    const int64_t *__restrict__ cand, int64_t n_pairs, const int64_t *__restrict__ off, int64_t n_docs,
    unsigned *__restrict__ bits, int64_t *__restrict__ row_map, int64_t *__restrict__ uniq,
    int64_t *__restrict__ other_row, const OtherSlots others,
    unsigned long long *__restrict__ counters, int64_t capacity_rows, int64_t capacity_docs,
    unsigned *__restrict__ err)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool first = false;
    int64_t id = 0;
    long long len = 0;
    if (i < n_pairs) {
        id = cand[i];
        if (id >= 0 && id < n_docs) {
            const unsigned m = 1u << (id & 31);
            first = (atomicOr(&bits[id >> 5], m) & m) == 0u;
            if (first) len = off[id + 1] - off[id];
        } else {
            atomicOr(err, ERR_ID_RANGE);
        }
    }
    const uint64_t firsts = __ballot(first);
    if (firsts == 0) return;                                   // wave-uniform
    // inclusive prefix sum of len over the wave
    long long incl = len;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const long long up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    const long long total = __shfl(incl, 63);
    const int n_first = __builtin_popcountll(firsts);
    unsigned long long row_base = 0, doc_base = 0;
    const int leader = __builtin_ctzll(firsts);
    if (lane == leader) {
        row_base = atomicAdd(&counters[1], (unsigned long long)total);
        doc_base = atomicAdd(&counters[0], (unsigned long long)n_first);
    }
    row_base = __shfl(row_base, leader);
    doc_base = __shfl(doc_base, leader);
    if (first) {
        const long long r0 = (long long)row_base + (incl - len);
        const int rank = __builtin_popcountll(firsts & ((1ull << lane) - 1ull));
        const long long slot_pos = (long long)doc_base + rank;
        // every list position below the capacity is written (the copy kernel reads them all);
        // a document that does not fit is listed with no rows
        const bool fits = r0 + len <= capacity_rows && slot_pos < capacity_docs;
        // where another slot holds the document, or -1: read it from the host table
        int64_t from = -1;
        for (int x = 0; x < others.n && from < 0; ++x)
            if ((others.bits[x][id >> 5] >> (id & 31)) & 1u) {
                const int64_t r = others.row_map[x][id];
                if (r >= 0) from = ((int64_t)x << OTHER_SHIFT) | r;
            }
        if (slot_pos < capacity_docs) {
            uniq[slot_pos] = id;
            other_row[slot_pos] = from;
        }
        row_map[id] = fits ? r0 : -1;
        if (!fits) atomicOr(err, ERR_STAGING_FULL);
        else if (from >= 0 && len > 0) atomicAdd(&counters[2], (unsigned long long)len);
    }
}

// The packing engine's share of the slot-to-slot hand-over.  The host knows which documents of the batch an
// earlier packed prefetch left in another slot: documents uniq[first .. n) are copied from there (from[u] = slot
// x << OTHER_SHIFT | first row in x), one wave per document, to row row0[u] of this slot.
struct SlotRows {
    const uint4 *rows[MAX_SLOTS];
};
__global__ __launch_bounds__(256) void staging_handover_kernel(
    const SlotRows all, const int64_t *__restrict__ off, const int64_t *__restrict__ uniq,
    const int64_t *__restrict__ row0, const int64_t *__restrict__ from, int64_t first, int64_t n,
    uint4 *__restrict__ slot, int chunks_per_row)
{
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    for (int64_t u = first + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); u < n; u += n_waves) {
        const int64_t id = uniq[u], f = from[u];
        const int64_t n_chunks = (off[id + 1] - off[id]) * chunks_per_row;
        const uint4 *src = all.rows[f >> OTHER_SHIFT] + (size_t)(f & (((int64_t)1 << OTHER_SHIFT) - 1)) * chunks_per_row;
        uint4 *dst = slot + (size_t)row0[u] * chunks_per_row;
        int64_t x = lane;
        for (; x + 7 * 64 < n_chunks; x += 8 * 64) {
            uint4 v[8];
#pragma unroll
            for (int y = 0; y < 8; ++y) v[y] = src[x + 64 * y];
#pragma unroll
            for (int y = 0; y < 8; ++y) dst[x + 64 * y] = v[y];
        }
        for (; x < n_chunks; x += 64) dst[x] = src[x];
    }
}

// uniq[i] is a distinct document of the batch and row0[i] the slot row its rows were copied to; `handed` of the
// `rows` rows came from other slots
__global__ void staging_publish_kernel(const int64_t *__restrict__ uniq, const int64_t *__restrict__ row0, int64_t n,
                                       unsigned long long rows, unsigned long long handed, unsigned *__restrict__ bits,
                                       int64_t *__restrict__ row_map, unsigned long long *__restrict__ counters)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const int64_t id = uniq[i];
        atomicOr(&bits[id >> 5], 1u << (id & 31));
        row_map[id] = row0[i];
    }
    if (i == 0) {
        counters[0] = (unsigned long long)n;
        counters[1] = rows;
        counters[2] = handed;
        counters[3] = (unsigned long long)n;
    }
}

// chunks_per_row = bytes of a row / 16.  host_emb is device-visible pinned host memory (or HBM);
// documents whose other_row entry is >= 0 are read from the slot it names instead.
__global__ __launch_bounds__(256) void staging_gather_kernel(
    const uint4 *__restrict__ host_emb, const OtherSlots others, const int64_t *__restrict__ off,
    const int64_t *__restrict__ uniq, const int64_t *__restrict__ other_row, const int64_t *__restrict__ row_map,
    unsigned long long *__restrict__ counters, int64_t capacity_docs, uint4 *__restrict__ slot,
    int chunks_per_row)
{
    const int lane = threadIdx.x & 63;
    const int64_t n = min((int64_t)counters[0], capacity_docs);
    // Waves draw documents from a shared counter (counters[3], zeroed by the clear kernel): a wave
    // that draws documents held by another slot is through with them in no time and draws again, so
    // the documents that have to cross PCIe are always spread over all waves and the link stays busy.
    while (true) {
        unsigned long long next = 0;
        if (lane == 0) next = atomicAdd(&counters[3], 1ull);
        const int64_t u = (int64_t)(((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(next >> 32)) << 32) |
                                    (unsigned)__builtin_amdgcn_readfirstlane((int)next));
        if (u >= n) break;
        const int64_t id = uniq[u];
        const int64_t r0 = row_map[id];
        if (r0 < 0) continue;
        const int64_t first = off[id];
        const int64_t n_chunks = (off[id + 1] - first) * chunks_per_row;
        const int64_t from = other_row[u];
        const uint4 *src = host_emb + (size_t)first * chunks_per_row;
        if (from >= 0)
            src = others.rows[from >> OTHER_SHIFT] + (size_t)(from & (((int64_t)1 << OTHER_SHIFT) - 1)) * chunks_per_row;
        uint4 *dst = slot + (size_t)r0 * chunks_per_row;
        int64_t x = lane;
        for (; x + 7 * 64 < n_chunks; x += 8 * 64) {           // 8 KiB in flight per wave
            uint4 v[8];
#pragma unroll
            for (int y = 0; y < 8; ++y) v[y] = src[x + 64 * y];
#pragma unroll
            for (int y = 0; y < 8; ++y) dst[x + 64 * y] = v[y];
        }
        for (; x < n_chunks; x += 64) dst[x] = src[x];
    }
}

// How much the candidate lists of a batch overlap, from a sample: up to 4096 of the batch's (query,
// candidate) pairs, evenly spaced, go into a hash set in LDS (32-bit fingerprints of the ids, open
// addressing, half full at most); the result is the fraction of them whose document was already there.
// Uniformly drawn lists over a large table give about 0, lists that share popular documents far more.
// One workgroup; `out` may be device-visible host memory.
__global__ __launch_bounds__(1024) void sharing_probe_kernel(const int64_t *__restrict__ cand, int64_t n_pairs, int K,
                                                             int ldc, float *__restrict__ out)
{
    constexpr unsigned SLOTS = 8192, SAMPLE = 4096, EMPTY = 0xffffffffu;
    __shared__ unsigned s_set[SLOTS];
    __shared__ unsigned s_repeats;
    for (unsigned i = threadIdx.x; i < SLOTS; i += 1024) s_set[i] = EMPTY;
    if (threadIdx.x == 0) s_repeats = 0u;
    __syncthreads();
    const unsigned n = (unsigned)(n_pairs < (int64_t)SAMPLE ? n_pairs : (int64_t)SAMPLE);
    unsigned mine = 0;
    for (unsigned i = threadIdx.x; i < n; i += 1024) {
        const int64_t pair = (int64_t)i * n_pairs / n;
        const uint64_t id = (uint64_t)cand[(pair / K) * ldc + pair % K];
        unsigned key = (unsigned)id ^ ((unsigned)(id >> 32) * 0x85ebca6bu);
        if (key == EMPTY) key = 0u;
        unsigned slot = (key * 2654435761u) >> 19;                   // 13 bits
        for (unsigned tries = 0; tries < SLOTS; ++tries) {             // the set is never more than half full
            const unsigned seen = atomicCAS(&s_set[slot], EMPTY, key);
            if (seen == EMPTY) break;
            if (seen == key) { ++mine; break; }
            slot = (slot + 1) & (SLOTS - 1);
        }
    }
    if (mine) atomicAdd(&s_repeats, mine);
    __syncthreads();
    if (threadIdx.x == 0) *out = n ? (float)s_repeats / (float)n : 0.f;
}

}  // namespace espn
