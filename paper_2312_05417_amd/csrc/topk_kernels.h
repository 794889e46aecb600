// Ranked top-k per query (Sec. 2.1: the re-ranking stage sorts candidates by score).
// Order: score descending, then document id ascending, then candidate slot ascending (the slot
// only separates entries that are identical in the output).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace espn {

// Batches of one shape that a single launch may take together (the pointers travel as kernel arguments).
constexpr int MAX_FUSED = 16;

// NaN test on the bit pattern (device code is built with -fno-honor-nans, which lets the compiler
// fold x != x to false)
__device__ __forceinline__ bool is_nan_bits(float x)
{
    return (__builtin_bit_cast(unsigned, x) & 0x7fffffffu) > 0x7f800000u;
}

// the "no score" marker, built from its bits for the same reason
__device__ __forceinline__ float quiet_nan() { return __builtin_bit_cast(float, 0x7fc00000u); }

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

// Shapes common to the ranking kernels: scores [B, K] dense; cand rows have leading dimension ldc >= K
// and output rows leading dimension ldo >= k (partial re-ranking ranks a prefix of each list into the
// front of a longer output row).
//
// Selection in k rounds, one workgroup per query, any K and k <= K.  Round j picks the best
// entry that ranks strictly after round j-1's winner; the order is total, so nothing has to be
// marked as taken and the inputs are never modified.  PER entries per thread are cached in
// registers (K <= 256*PER takes no global re-reads); longer lists re-read the tail from L2.
// An entry whose score is NaN is never picked; rounds that find nothing write id -1, score NaN.
template <int PER>
__global__ __launch_bounds__(256) void topk_rounds_kernel(
    const float *__restrict__ scores, const int64_t *__restrict__ cand, int ldc, int K, int k, int ldo,
    int64_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    __shared__ Ranked wave_best[4];
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *sc = scores + (size_t)b * K;
    const int64_t *ids = cand + (size_t)b * ldc;

    Ranked mine[PER];
#pragma unroll
    for (int x = 0; x < PER; ++x) {
        const int slot = tid + 256 * x;
        mine[x].slot = -1;
        mine[x].score = 0.f;
        mine[x].id = 0;
        if (slot < K) {
            const float s = sc[slot];
            if (!is_nan_bits(s)) { mine[x].score = s; mine[x].id = ids[slot]; mine[x].slot = slot; }
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
            if (is_nan_bits(e.score)) continue;
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
            out_ids[(size_t)b * ldo + round] = best.slot >= 0 ? best.id : (int64_t)-1;
            out_scores[(size_t)b * ldo + round] = best.slot >= 0 ? best.score : quiet_nan();
        }
        prev = best;
        if (best.slot < 0) {
            // nothing left that can be ranked: fill the rest and stop
            if (tid == 0)
                for (int rest = round + 1; rest < k; ++rest) {
                    out_ids[(size_t)b * ldo + rest] = -1;
                    out_scores[(size_t)b * ldo + rest] = quiet_nan();
                }
            break;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Fast path: one wave per query, K <= 64*PER, k <= 64.
//
// Scores are mapped to unsigned keys that order like the floats (NaN and unused slots -> 0, never
// picked).  Each lane holds PER keys in registers.  The k-th largest of the 64 per-lane maxima is a
// lower bound theta for the k-th best key overall (at least k elements reach it), so every entry
// that can appear in the ranked top-k, including all ties with the k-th, has key >= theta.  Those
// few entries are compacted into LDS together with their ids and slots, and each one counts how many
// others rank before it; entries whose count is below k write themselves to that position.  Only if more than 64 entries survive (massive exact ties) the survivors are ranked by
// the k-round selection, from LDS.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned order_key(float s)
{
    const unsigned raw = __builtin_bit_cast(unsigned, s);
    if (is_nan_bits(s)) return 0u;
    const unsigned u = (raw << 1) == 0u ? 0u : raw;              // -0 and +0 are the same score
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_to_score(unsigned key)
{
    const unsigned u = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    return __builtin_bit_cast(float, u);
}

// LDS one wave needs for topk_wave_body<PER>
template <int PER>
struct TopkWaveLds {
    __attribute__((aligned(16))) unsigned key[64 * PER + 4];    // survivors, then zeros
    int slot[64 * PER];
    int64_t id[64 * PER];
    __attribute__((aligned(16))) unsigned lane_max[64];
    unsigned theta;
    unsigned total;
};

// LDS written by some lanes of a wave and read by others of the same wave: LDS keeps a wave's accesses
// in order, the fence keeps the compiler from moving them
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Executed by ONE wave (lane = 0..63) for one query: sc/ids point at the query's K scores and ids,
// out_ids/out_scores at its k outputs.  Uses no workgroup barrier, so a single wave of a larger
// workgroup may call it.  Counting is done in vector registers against values every lane reads from
// the same LDS address; a version that counted with cross-lane votes (wave maximum k times for the
// threshold, ballots for the compaction, readlane for the ranks) took 7.2 us instead of 5.7 us for
// k = 20 and 10.0 instead of 8.2 us for k = 32 (64 lists of 1000).
template <int PER>
__device__ __forceinline__ void topk_wave_body(
    const float *sc, const int64_t *ids, int K, int k, int64_t *out_ids, float *out_scores, int lane,
    TopkWaveLds<PER> &lds)
{
    unsigned *s_key = lds.key;
    int *s_slot = lds.slot;
    int64_t *s_id = lds.id;

    // scores and ids are fetched together (one round trip to memory instead of two dependent ones)
    unsigned key[PER];
    int64_t idr[PER];
    {
        float v[PER];
#pragma unroll
        for (int x = 0; x < PER; ++x) {      // all loads first: one round trip, not PER of them
            const int slot = min(x * 64 + lane, K - 1);
            v[x] = sc[slot];
            idr[x] = ids[slot];
        }
#pragma unroll
        for (int x = 0; x < PER; ++x) key[x] = (x * 64 + lane < K) ? order_key(v[x]) : 0u;
    }
    unsigned local_max = 0;
#pragma unroll
    for (int x = 0; x < PER; ++x) local_max = max(local_max, key[x]);

    // theta = k-th largest of the 64 per-lane maxima (with multiplicity; 1 if it is 0): a lane holds
    // it if fewer than k maxima are larger and at least k are as large
    lds.lane_max[lane] = local_max;
    if (lane == 0) lds.total = 0u;
    wave_lds_sync();
    {
        int larger = 0, as_large = 0;
#pragma unroll
        for (int j = 0; j < 64; j += 4) {
            const uint4 m = *reinterpret_cast<const uint4 *>(&lds.lane_max[j]);
            larger += (m.x > local_max) + (m.y > local_max) + (m.z > local_max) + (m.w > local_max);
            as_large += (m.x >= local_max) + (m.y >= local_max) + (m.z >= local_max) + (m.w >= local_max);
        }
        if (larger < k && k <= as_large) lds.theta = local_max;     // the same value from every such lane
    }
    wave_lds_sync();
    const unsigned theta = max(lds.theta, 1u);

    // the survivors, in no particular order: a lane reserves room for all of its own with one atomic
    int mine = 0;
#pragma unroll
    for (int x = 0; x < PER; ++x) mine += key[x] >= theta;
    if (mine > 0) {
        int pos = (int)atomicAdd(&lds.total, (unsigned)mine);
#pragma unroll
        for (int x = 0; x < PER; ++x)
            if (key[x] >= theta) {
                s_key[pos] = key[x];
                s_slot[pos] = x * 64 + lane;
                s_id[pos] = idr[x];
                ++pos;
            }
    }
    wave_lds_sync();
    const int total = __builtin_amdgcn_readfirstlane((int)lds.total);

    if (total <= 64) {
        // one survivor per lane: rank = number of survivors that come before it
        if (lane < 4) s_key[total + lane] = 0u;              // keys are read four at a time
        wave_lds_sync();
        const bool have = lane < total;
        const unsigned my_key = have ? s_key[lane] : 0u;
        int rank = 0, same = 0;
        for (int i = 0; i < total; i += 4) {
            const uint4 o = *reinterpret_cast<const uint4 *>(&s_key[i]);
            rank += (o.x > my_key) + (o.y > my_key) + (o.z > my_key) + (o.w > my_key);
            same += (o.x == my_key) + (o.y == my_key) + (o.z == my_key) + (o.w == my_key);
        }
        if (have) {
            const int64_t my_id = s_id[lane];
            if (same > 1) {                                  // the ids only matter among equal scores
                const int my_slot = s_slot[lane];
                for (int i = 0; i < total; ++i) {
                    if (s_key[i] != my_key) continue;
                    const int64_t other = s_id[i];
                    rank += other < my_id || (other == my_id && s_slot[i] < my_slot);
                }
            }
            if (rank < k) {
                out_ids[rank] = my_id;
                out_scores[rank] = key_to_score(my_key);
            }
        }
        // fewer rankable entries than k (NaN scores): mark the rest
        for (int rest = total + lane; rest < k; rest += 64) {
            out_ids[rest] = -1;
            out_scores[rest] = quiet_nan();
        }
        return;
    }

    // many exact ties: k rounds of selection over the survivors held in LDS
    Ranked prev;
    prev.slot = -1;
    for (int round = 0; round < k; ++round) {
        Ranked best;
        best.slot = -1; best.score = 0.f; best.id = 0;
        for (int i = lane; i < total; i += 64) {
            Ranked e;
            e.score = key_to_score(s_key[i]);
            e.slot = s_slot[i];
            e.id = s_id[i];
            const bool after_prev = (round == 0) || ranks_before(prev, e);
            if (after_prev && ranks_before(e, best)) best = e;
        }
#pragma unroll
        for (int mask = 32; mask >= 1; mask >>= 1) {
            const Ranked o = shfl_xor_ranked(best, mask);
            if (ranks_before(o, best)) best = o;
        }
        if (lane == 0) {
            out_ids[round] = best.slot >= 0 ? best.id : (int64_t)-1;
            out_scores[round] = best.slot >= 0 ? best.score : quiet_nan();
        }
        prev = best;
        if (best.slot < 0) {
            for (int rest = round + 1 + lane; rest < k; rest += 64) {
                out_ids[rest] = -1;
                out_scores[rest] = quiet_nan();
            }
            break;
        }
    }
}

template <int PER>
__global__ __launch_bounds__(64) void topk_wave_kernel(
    const float *__restrict__ scores, const int64_t *__restrict__ cand, int ldc, int K, int k, int ldo,
    int64_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    __shared__ TopkWaveLds<PER> lds;
    const int b = blockIdx.x;
    topk_wave_body<PER>(scores + (size_t)b * K, cand + (size_t)b * ldc, K, k, out_ids + (size_t)b * ldo,
                        out_scores + (size_t)b * ldo, (int)threadIdx.x, lds);
}

// The same for the queries of up to MAX_FUSED batches of one shape in one launch: workgroup x ranks query
// x % B of batch x / B (a queue of small batches then costs one ranking launch, not one per batch).
struct TopkSet {
    int n, B;
    const float *scores[MAX_FUSED];     // each [B, K]
    const int64_t *cand[MAX_FUSED];     // each [B, ldc]
    int64_t *out_ids[MAX_FUSED];        // each [B, ldo]
    float *out_scores[MAX_FUSED];
};

template <int PER>
__global__ __launch_bounds__(64) void topk_wave_set_kernel(const TopkSet set, int ldc, int K, int k, int ldo)
{
    __shared__ TopkWaveLds<PER> lds;
    const int which = (int)blockIdx.x / set.B, b = (int)blockIdx.x - which * set.B;
    topk_wave_body<PER>(set.scores[which] + (size_t)b * K, set.cand[which] + (size_t)b * ldc, K, k,
                        set.out_ids[which] + (size_t)b * ldo, set.out_scores[which] + (size_t)b * ldo, (int)threadIdx.x, lds);
}

// ---------------------------------------------------------------------------------------------
// Whole-list sort: one workgroup per query, K <= N entries, any k <= K, at a cost that does not depend on
// k (the selection kernels above take time proportional to k).  Every entry becomes one 64-bit
// word, order key in the upper half and 2^32 - 1 - slot in the lower, so that "larger word first"
// is "score descending, slot ascending"; a bitonic network sorts the N words in LDS, two strides
// per pass (a thread holds four words and applies strides 2h and h to them in registers).
// Passes whose words all belong to the wave that handles them need no workgroup barrier.  The required order among equal scores is by id, which the words do not carry: entries
// of a run of equal keys count, at the end, how many entries of their run go before them (ids are
// read through the slots; such runs are short unless many documents are identical or empty).
// ---------------------------------------------------------------------------------------------
// the larger word goes to a
__device__ __forceinline__ void order_pair(uint64_t &a, uint64_t &b)
{
    const bool swap = a < b;
    const uint64_t t = swap ? b : a;
    b = swap ? a : b;
    a = t;
}

// What the sort kernel ranks: one scored list per query ...
struct OneList {
    const float *scores;        // [B, K]
    const int64_t *cand;        // rows of leading dimension ldc
    int ldc, K;
    __device__ int size() const { return K; }
    __device__ float score(int b, int i) const { return scores[(size_t)b * K + i]; }
    __device__ int64_t id(int b, int i) const { return cand[(size_t)b * ldc + i]; }
};
// ... or two of them, taken as list a followed by list b (Sec. 4.3)
struct TwoLists {
    const int64_t *ids_a;
    const float *sc_a;
    int ka;
    const int64_t *ids_b;
    const float *sc_b;
    int kb;
    __device__ int size() const { return ka + kb; }
    __device__ float score(int b, int i) const
    {
        return i < ka ? sc_a[(size_t)b * ka + i] : sc_b[(size_t)b * kb + (i - ka)];
    }
    __device__ int64_t id(int b, int i) const
    {
        return i < ka ? ids_a[(size_t)b * ka + i] : ids_b[(size_t)b * kb + (i - ka)];
    }
};

template <int N, int T, typename Lists>
__global__ __launch_bounds__(T) void topk_sort_kernel(
    const Lists lists, int k, int ldo, int64_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    static_assert(N >= 256 && (N & (N - 1)) == 0 && T % 64 == 0 && N / 4 >= T, "four words per thread at least");
    __shared__ uint64_t s[N];
    constexpr int W = T / 64, OWN = N / W;              // waves; words of the range a wave handles
    constexpr int QW = N / 4 / W, PW = N / 2 / W;       // groups of four / pairs per wave
    const int b = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int K = lists.size();
    for (int i = tid; i < N; i += T) {
        const unsigned key = i < K ? order_key(lists.score(b, i)) : 0u;      // slots past the list sort last
        s[i] = ((uint64_t)key << 32) | (uint64_t)(0xffffffffu - (unsigned)i);
    }
    bool prev_local = false;
    auto sync = [&](bool local) {
        // local: every word this pass touches was last written by the same wave
        if (local && prev_local) {
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
        } else __syncthreads();
        prev_local = local;
    };
    // Merging two sorted halves of `size` words starts by comparing word o of the block with word
    // size-1-o (the mirror image), after which both halves only need strides size/4 .. 1, all in the
    // same direction: no comparison depends on where in the list it happens.
    for (int size = 2; size <= N; size <<= 1) {
        int stride = size >> 1;
        bool mirrored = true;                   // the first stride of a merge
        while (stride >= 2) {
            const int h = stride >> 1;          // this pass applies strides 2h and h
            sync(4 * h <= OWN);
#pragma unroll
            for (int x = 0; x < QW / 64; ++x) {
                const int g = wave * QW + x * 64 + lane;
                const int o = g & (h - 1);
                const int block = (g & ~(h - 1)) << 2;
                const int i0 = block + o, i1 = i0 + h;
                const int i2 = mirrored ? block + 3 * h - 1 - o : i0 + 2 * h;
                const int i3 = mirrored ? block + 4 * h - 1 - o : i0 + 3 * h;
                uint64_t e0 = s[i0], e1 = s[i1], e2 = s[i2], e3 = s[i3];
                if (mirrored) {                 // o with 4h-1-o, o+h with 3h-1-o
                    order_pair(e0, e3);
                    order_pair(e1, e2);
                } else {                        // stride 2h
                    order_pair(e0, e2);
                    order_pair(e1, e3);
                }
                order_pair(e0, e1);             // stride h
                order_pair(e2, e3);
                s[i0] = e0; s[i1] = e1; s[i2] = e2; s[i3] = e3;
            }
            mirrored = false;
            stride >>= 2;
        }
        if (stride == 1) {                      // size 2: its own mirror image
            sync(true);
#pragma unroll
            for (int x = 0; x < PW / 64; ++x) {
                const int i = 2 * (wave * PW + x * 64 + lane);
                uint64_t e0 = s[i], e1 = s[i + 1];
                order_pair(e0, e1);
                s[i] = e0; s[i + 1] = e1;
            }
        }
    }
    __syncthreads();
    // s[r] is the r-th best (key, slot)
    for (int r = tid; r < K; r += T) {
        const uint64_t e = s[r];
        const unsigned key = (unsigned)(e >> 32);
        const int slot = (int)(0xffffffffu - (unsigned)e);
        const bool tie_left = r > 0 && (unsigned)(s[r - 1] >> 32) == key;
        const bool tie_right = r + 1 < K && (unsigned)(s[r + 1] >> 32) == key;
        if (r >= k && !tie_left) continue;               // nothing can bring it to the front
        if (key == 0u) {                                  // NaN: never ranked
            if (r < k) {
                out_ids[(size_t)b * ldo + r] = -1;
                out_scores[(size_t)b * ldo + r] = quiet_nan();
            }
            continue;
        }
        const int64_t id = lists.id(b, slot);
        int pos = r;
        if (tie_left || tie_right) {
            int first = r;
            while (first > 0 && (unsigned)(s[first - 1] >> 32) == key) --first;
            if (first >= k) continue;
            pos = first;
            for (int j = first; j < K; ++j) {
                const uint64_t o = s[j];
                if ((unsigned)(o >> 32) != key) break;
                const int oslot = (int)(0xffffffffu - (unsigned)o);
                const int64_t oid = lists.id(b, oslot);
                pos += oid < id || (oid == id && oslot < slot);
            }
        }
        if (pos < k) {
            out_ids[(size_t)b * ldo + pos] = id;
            out_scores[(size_t)b * ldo + pos] = key_to_score(key);
        }
    }
}

// Partial re-ranking (Sec. 4.4): ranks R .. k-1 of every query are the candidates that were not
// re-ranked, in the order the first stage listed them; they carry no MaxSim score (NaN).
__global__ void append_unranked_kernel(const int64_t *__restrict__ cand, int ldc, int R, int k,
                                       int64_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    const int b = blockIdx.x;                                   // grid = (B, chunks of 256 ranks)
    const int j = R + blockIdx.y * blockDim.x + threadIdx.x;
    if (j < k) {
        out_ids[(size_t)b * k + j] = cand[(size_t)b * ldc + j];
        out_scores[(size_t)b * k + j] = quiet_nan();
    }
}

// Merge of two scored lists per query (Sec. 4.3: early re-ranked and later re-ranked documents are
// combined by sorting on the score): the first k of their union in ranking order.  One wave per
// query, k stateless selection rounds over the ka + kb entries (slot = position in a followed by b).
__global__ __launch_bounds__(64) void merge_topk_kernel(
    const int64_t *__restrict__ ids_a, const float *__restrict__ sc_a, int ka,
    const int64_t *__restrict__ ids_b, const float *__restrict__ sc_b, int kb, int k,
    int64_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    const int b = blockIdx.x, lane = threadIdx.x, n = ka + kb;
    Ranked prev;
    prev.slot = -1;
    for (int round = 0; round < k; ++round) {
        Ranked best;
        best.slot = -1; best.score = 0.f; best.id = 0;
        for (int i = lane; i < n; i += 64) {
            Ranked e;
            e.slot = i;
            e.score = i < ka ? sc_a[(size_t)b * ka + i] : sc_b[(size_t)b * kb + (i - ka)];
            if (is_nan_bits(e.score)) continue;
            e.id = i < ka ? ids_a[(size_t)b * ka + i] : ids_b[(size_t)b * kb + (i - ka)];
            const bool after_prev = (round == 0) || ranks_before(prev, e);
            if (after_prev && ranks_before(e, best)) best = e;
        }
#pragma unroll
        for (int mask = 32; mask >= 1; mask >>= 1) {
            const Ranked o = shfl_xor_ranked(best, mask);
            if (ranks_before(o, best)) best = o;
        }
        if (lane == 0) {
            out_ids[(size_t)b * k + round] = best.slot >= 0 ? best.id : (int64_t)-1;
            out_scores[(size_t)b * k + round] = best.slot >= 0 ? best.score : quiet_nan();
        }
        prev = best;
        if (best.slot < 0) {
            for (int rest = round + 1 + lane; rest < k; rest += 64) {
                out_ids[(size_t)b * k + rest] = -1;
                out_scores[(size_t)b * k + rest] = quiet_nan();
            }
            break;
        }
    }
}

}  // namespace espn
