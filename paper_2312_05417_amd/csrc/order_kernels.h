// Batches whose candidate lists share documents (Sec. 4.2: the lists of a workload keep coming back to the same
// documents; here: Zipf-distributed lists) are scored in an order that lets the caches serve the repeats:
//
//   listings   counts, over a sample batch, how many lists name each document
//   popular    turns the counts into one bit per document: listed by enough of the sample's queries.  The scoring
//              kernel fetches those through the caches and streams the rest past them.
//   order      per batch: a copy of every query's list sorted by document id, each entry carrying the position it
//              came from (the scores still go there).  The scoring kernel then walks all lists in id order at once.
//
// None of this changes a score: only the order in which pairs are scored and how their rows are fetched.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "maxsim_kernels.h"

namespace espn {

// counts[id] += 1 for every (query, candidate) pair of the sample whose id is in range
__global__ __launch_bounds__(256) void listings_kernel(const int64_t *__restrict__ cand, int64_t n_pairs, int K, int ldc,
                                                       int64_t n_docs, unsigned *__restrict__ counts)
{
    const int64_t pair = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (pair >= n_pairs) return;
    const int64_t id = cand[(pair / K) * ldc + pair % K];
    if (id >= 0 && id < n_docs) atomicAdd(&counts[id], 1u);
}

// bit id of `bits` = counts[id] >= at_least; one thread per word of 32 documents
__global__ __launch_bounds__(256) void popular_kernel(const unsigned *__restrict__ counts, int64_t n_docs, unsigned at_least,
                                                      unsigned *__restrict__ bits)
{
    const int64_t word = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (word * 32 >= n_docs) return;
    unsigned w = 0u;
    for (int x = 0; x < 32; ++x) {
        const int64_t id = word * 32 + x;
        if (id < n_docs && counts[id] >= at_least) w |= 1u << x;
    }
    bits[word] = w;
}

// The lists of the batches one launch orders (the batches one scoring launch takes together)
struct OrderSet {
    int n, B;
    const int64_t *cand[MAX_FUSED];     // each [B, ldc]
    int64_t *ordered[MAX_FUSED];        // each [B, K], written
};

// One workgroup per query (query g of the launch is query g % B of batch g / B): the K <= N entries of its list as
// id << SLOT_BITS | position (an id outside the table as -1: it is scored as such, raises the same flag, and can
// alias nothing), sorted ascending in LDS (bitonic, N a power of two, padded with entries that sort last), written
// to ordered[b * K ..].
template <int N, int T>
__global__ __launch_bounds__(T) void order_lists_kernel(const OrderSet set, int ldc, int K, int64_t n_docs)
{
    static_assert((N & (N - 1)) == 0 && N >= 2 * T && N <= (1 << SLOT_BITS), "one thread per pair of entries, or several");
    __shared__ uint64_t s_key[N];
    const int which = set.n > 1 ? (int)blockIdx.x / set.B : 0;
    const int b = (int)blockIdx.x - which * set.B;
    const int64_t *__restrict__ cand = set.cand[which];
    int64_t *__restrict__ ordered = set.ordered[which];
    for (int i = threadIdx.x; i < N; i += T) {
        uint64_t key = ~(uint64_t)0;
        if (i < K) {
            int64_t id = cand[(size_t)b * ldc + i];
            if (id < 0 || id >= n_docs) id = -1;
            key = ((uint64_t)id << SLOT_BITS) | (uint64_t)i;
        }
        s_key[i] = key;
    }
    __syncthreads();
    for (int size = 2; size <= N; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = threadIdx.x; t < N / 2; t += T) {
                const int i = ((t & ~(stride - 1)) << 1) | (t & (stride - 1)), j = i | stride;
                const uint64_t a = s_key[i], c = s_key[j];
                if ((a > c) == ((i & size) == 0)) {
                    s_key[i] = c;
                    s_key[j] = a;
                }
            }
            __syncthreads();
        }
    }
    for (int i = threadIdx.x; i < K; i += T) ordered[(size_t)b * K + i] = (int64_t)s_key[i];
}

}  // namespace espn
