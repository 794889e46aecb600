// Ranked top-k per query (Sec. 2.1: the re-ranking stage sorts candidates by score).
// Order: score descending, then document id ascending, then candidate slot ascending (the slot
// only separates entries that are identical in the output).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace espn {

struct Ranked {
    float score;
    int64_t id;
    int slot;       // -1: nothing
};

// a ranks strictly before b
__device__ __forceinline__ bool ranks_before(const Ranked &a, const Ranked &b)
{
    if (a.slot < 0) return false;
    if (b.slot < 0) return true;
    if (a.score != b.score) return a.score > b.score;
    if (a.id != b.id) return a.id < b.id;
    return a.slot < b.slot;
}

__device__ __forceinline__ Ranked shfl_xor_ranked(const Ranked &a, int mask)
{
    Ranked o;
    o.score = __shfl_xor(a.score, mask);
    unsigned lo = __shfl_xor((unsigned)(uint64_t)a.id, mask);
    unsigned hi = __shfl_xor((unsigned)((uint64_t)a.id >> 32), mask);
    o.id = (int64_t)(((uint64_t)hi << 32) | lo);
    o.slot = __shfl_xor(a.slot, mask);
    return o;
}

// Selection in k rounds, one workgroup per query, any K and k <= K.  Round j picks the best
// entry that ranks strictly after round j-1's winner; the order is total, so nothing has to be
// marked as taken and the inputs are never modified.  PER entries per thread are cached in
// registers (K <= 256*PER takes no global re-reads); longer lists re-read the tail from L2.
// An entry whose score is NaN is never picked; rounds that find nothing write id -1, score NaN.
template <int PER>
__global__ __launch_bounds__(256) void topk_rounds_kernel(
    const float *__restrict__ scores, const int64_t *__restrict__ cand, int K, int k,
    int64_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    __shared__ Ranked wave_best[4];
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *sc = scores + (size_t)b * K;
    const int64_t *ids = cand + (size_t)b * K;

    Ranked mine[PER];
#pragma unroll
    for (int x = 0; x < PER; ++x) {
        const int slot = tid + 256 * x;
        mine[x].slot = -1;
        mine[x].score = 0.f;
        mine[x].id = 0;
        if (slot < K) {
            const float s = sc[slot];
            if (s == s) { mine[x].score = s; mine[x].id = ids[slot]; mine[x].slot = slot; }
        }
    }

    Ranked prev;
    prev.slot = -1;
    for (int round = 0; round < k; ++round) {
        Ranked best;
        best.slot = -1; best.score = 0.f; best.id = 0;
#pragma unroll
        for (int x = 0; x < PER; ++x) {
            const bool after_prev = (round == 0) || ranks_before(prev, mine[x]);
            if (mine[x].slot >= 0 && after_prev && ranks_before(mine[x], best)) best = mine[x];
        }
        for (int slot = tid + 256 * PER; slot < K; slot += 256) {
            Ranked e;
            e.score = sc[slot];
            if (!(e.score == e.score)) continue;
            e.id = ids[slot];
            e.slot = slot;
            const bool after_prev = (round == 0) || ranks_before(prev, e);
            if (after_prev && ranks_before(e, best)) best = e;
        }
#pragma unroll
        for (int mask = 32; mask >= 1; mask >>= 1) {
            const Ranked o = shfl_xor_ranked(best, mask);
            if (ranks_before(o, best)) best = o;
        }
        if (lane == 0) wave_best[wave] = best;
        __syncthreads();
        best = wave_best[0];
#pragma unroll
        for (int w = 1; w < 4; ++w)
            if (ranks_before(wave_best[w], best)) best = wave_best[w];
        __syncthreads();
        if (tid == 0) {
            out_ids[(size_t)b * k + round] = best.slot >= 0 ? best.id : (int64_t)-1;
            out_scores[(size_t)b * k + round] = best.slot >= 0 ? best.score : __builtin_nanf("");
        }
        prev = best;
        if (best.slot < 0) {
            // nothing left that can be ranked: fill the rest and stop
            if (tid == 0)
                for (int rest = round + 1; rest < k; ++rest) {
                    out_ids[(size_t)b * k + rest] = -1;
                    out_scores[(size_t)b * k + rest] = __builtin_nanf("");
                }
            break;
        }
    }
}

}  // namespace espn
