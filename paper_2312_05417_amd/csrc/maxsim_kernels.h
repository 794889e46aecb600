// MaxSim scoring kernels for gfx950 (CDNA4): fused candidate gather + Eq. 1 (Sec. 2.1).
//
//   score[b,j] = sum_{i<Q} max_{r in doc(cand[b,j])} <q[b,i,:], emb[r,:]>
//
// Two kernels:
//   maxsim_slice_kernel<D>  D = 32, 64, .. 256: the Q x D x t contraction of each document runs on the
//                           matrix cores (v_mfma_f32_16x16x32_f16); document rows stream from HBM
//                           through a register pipeline into the MFMA A operand, the query sits
//                           in VGPRs.  Rows are binary16, or E4M3 codes widened exactly to binary16
//                           on the way into the MFMA.  Optionally ranks each query's top-k as well.
//   maxsim_generic_kernel   any D multiple of 8, any Q: plain FMA, one wave per document.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "topk_kernels.h"

namespace espn {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr unsigned ERR_ID_RANGE = 1u;        // a candidate id outside [0, n_docs)
constexpr unsigned ERR_STAGING_FULL = 2u;    // a prefetch needed more staging rows than the slot holds
constexpr unsigned ERR_NOT_STAGED = 4u;      // a staged re-rank met a document its slot does not hold

// Where a document's rows are.  Table in HBM: rows off[id] .. off[id+1]-1 of `emb`.  Staged (table in
// host memory, a prefetch copied this batch's documents into an HBM slot): `emb` is the slot, the
// document's first row there is row_map[id], valid only if bit id of staged_bits is set.
//
// Rows are binary16 (2 bytes per component), or E4M3 codes (1 byte per component, OCP 8-bit floating
// point) with one positive scale per document: a stored component stands for doc_scale[id] * decode(code).
struct DocSource {
    const void *emb;
    const int64_t *off;
    const int64_t *row_map;        // nullptr: table in HBM
    const unsigned *staged_bits;
    int64_t n_docs;
    const float *doc_scale;        // nullptr: binary16 rows
    const unsigned *popular;       // one bit per document or nullptr: see is_popular()
};

// Documents that many queries of a batch list (Sec. 4.2 observes that candidate lists of nearby queries repeat
// documents; a sample of the workload's lists names them) are fetched through the caches, where a later query of
// the launch finds them; the others are streamed past the caches (each of their lines is wanted once) and so leave
// the popular ones there.  No map: every document goes through the caches.
__device__ __forceinline__ bool is_popular(const DocSource &src, int64_t id)
{
    if (src.popular == nullptr || id < 0 || id >= src.n_docs) return true;
    return ((src.popular[id >> 5] >> (id & 31)) & 1u) != 0u;
}

// One batch of queries and their candidate lists.
//   cand  [B, ldc] ids, of which the first K of every row are scored (ldc >= K: partial re-ranking
//         scores a prefix of each list)
//   prior [B, ldc] first-stage scores or nullptr; score = MaxSim + alpha * prior (Sec. 3.1)
//   order ORDER_BY_ID: `cand` is not the caller's list but order_lists_kernel's copy of it, each list sorted by
//         document id, an entry = id << SLOT_BITS | position in the caller's list (ldc = K, no prior); scores go
//         to the caller's positions.  The workgroups then run slice by slice (the first slice of every query,
//         then the second ...), not query by query: the workgroups resident at one time walk the same range of
//         ids in the same direction, so a document that several of them list is asked for by all of them within
//         a short time, and only the first request leaves the L2.
struct Batch {
    const uint16_t *q;      // [B, Q, D]
    const int64_t *cand;
    const float *prior;
    float alpha;
    int ldc;
    int Q;
    int K;
    int order;              // 0 or ORDER_BY_ID
};
constexpr int ORDER_BY_ID = 1;
constexpr int SLOT_BITS = 20;                               // lists of up to 2^20 entries, ids below 2^43
constexpr int64_t SLOT_MASK = ((int64_t)1 << SLOT_BITS) - 1;

__device__ __forceinline__ float with_prior(const Batch &bt, int b, int j, float maxsim)
{
    return bt.prior ? fmaf(bt.alpha, bt.prior[(size_t)b * bt.ldc + j], maxsim) : maxsim;
}

// The batches one launch of the matrix-core kernel scores: n batches of B queries each, all of the shape
// that `Batch` describes (its own pointers are not used then).  Query g of the launch is query g % B of batch
// g / B.  A queue of small batches scored by one launch streams like one large batch: no launch gaps, and
// the look-ups of one batch's documents overlap with the row streaming of the batches before it.
struct BatchSet {
    int n, B;
    const uint16_t *q[MAX_FUSED];       // each [B, Q, D]
    const int64_t *cand[MAX_FUSED];     // each [B, ldc]
    const float *prior[MAX_FUSED];      // each [B, ldc] or nullptr
    float *scores[MAX_FUSED];           // each [B, K], written
    int64_t *out_ids[MAX_FUSED];        // RANK: each [B, ldo], written
    float *out_scores[MAX_FUSED];
};

// (first row, row count) of document `id`; count 0 and an error flag (if err is given) if it cannot
// be read.
__device__ __forceinline__ void locate_document(const DocSource &src, int64_t id, unsigned *err,
                                                int64_t &row0, int &ntok)
{
    row0 = 0;
    ntok = 0;
    if (id < 0 || id >= src.n_docs) {
        if (err) atomicOr(err, ERR_ID_RANGE);
        return;
    }
    const int64_t first = src.off[id];
    const int n = (int)(src.off[id + 1] - first);
    if (src.row_map == nullptr) {
        row0 = first;
        ntok = n;
        return;
    }
    const int64_t staged = src.row_map[id];
    if (((src.staged_bits[id >> 5] >> (id & 31)) & 1u) == 0u || staged < 0) {
        if (err) atomicOr(err, ERR_NOT_STAGED);
        return;
    }
    row0 = staged;
    ntok = n;
}

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

__device__ __forceinline__ int64_t readlane64(int64_t v, int lane)
{
    unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), lane);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// max(a, b, c); becomes one v_max3_f32.  (Device code is built with -fno-honor-nans: without it the
// compiler first quiets a possible signalling NaN in every operand, a v_max_f32 x, x, x each, which
// triples the VALU work of the per-tile maximum.  The operands are MFMA results of finite inputs.)
__device__ __forceinline__ float max3(float a, float b, float c)
{
    return fmaxf(fmaxf(a, b), c);
}

// running maximum m updated with the four values of an accumulator
__device__ __forceinline__ float max_into(float m, const floatx4 &a)
{
    return max3(max3(m, a[0], a[1]), a[2], a[3]);
}

// value of `v` in lane (lane ^ mask), through a precomputed byte address (4 * (lane ^ mask))
__device__ __forceinline__ float from_lane(int addr, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(addr, __builtin_bit_cast(int, v)));
}

// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
__device__ __forceinline__ float row16_sum(float v)
{
    // quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
    return v;
}

// ---------------------------------------------------------------------------------------------
// Matrix-core kernel.
//
// v_mfma_f32_16x16x32_f16 computes a 16x16 tile C[m][n] += sum_k A[m][k] B[k][n], k = 0..31; lane l
// supplies A[l%16][8*(l/16)..+7] and B[8*(l/16)..+7][l%16] and receives C[4*(l/16)+v][l%16],
// v = 0..3.  Here m indexes 16 document rows (a "tile"), n indexes 16 query rows, so after the MFMA
// a lane holds the dot products of ONE query row with FOUR document rows: the max over document
// rows is mostly an in-lane v_max over accumulator registers carried across the tiles of a
// document, finished by two cross-lane steps per document; the sum over query rows is one 16-lane
// DPP reduction per document.
//
// The dot product does not care in which order the D components are visited as long as both
// operands agree.  The k slots are assigned so that what a lane feeds to successive MFMA steps are
// ADJACENT bytes of one table row (lane (r = l%16, c = l/16) owns bytes [c*D/2, (c+1)*D/2) of tile
// row r); the query fragments are gathered once per wave with the same assignment.
//
// How the rows reach that layout differs with the row length:
//   D = 32   a 16-row tile is 1 KiB; lane l loads bytes [16 l, 16 l + 16) of it (one fully
//            coalesced, non-temporal instruction), then four ds_bpermute_b32 move chunk c of row r
//            from lane 4r + c to lane r + 16c.  Loading in the MFMA layout directly (16 B per lane at
//            a 64 B stride) was measured ~30 % slower on the same gather.  Tiles of binary16 rows start
//            on 128-byte lines: a document that starts in the middle of a line takes the row before it
//            into its first tile and never uses it (the bpermute source is clamped from below as well).
//   D >= 64  two ways (template argument LINEAR), chosen per launch by the host:
//            LINEAR  the tile, 16 * D * EB contiguous bytes, is loaded lane-linearly, 1 KiB per
//            instruction, so that every cache line is asked for exactly once and by one
//            instruction: such loads can be non-temporal, which this machine streams 13 % faster
//            (256-byte rows: 761 -> 673 us per 4.5 GB launch).  The wave then writes the tile to an
//            LDS scratch of its own (rows padded by 16 bytes against bank conflicts) and reads it
//            back in the MFMA layout: 2 x NW/4 LDS instructions per tile, 7 us of the launch.
//            otherwise  a lane loads its D/2 contiguous bytes directly (D = 128: 4 x
//            global_load_dwordx4): no transpose, but the four instructions come back to every
//            line, so the loads have to be ordinary ones (non-temporal: 1.8 times slower).  They
//            leave the rows in the caches, which is what a batch wants whose queries share
//            documents (2048 queries with Zipf-distributed lists: 0.98 of the HBM peak this way,
//            0.85 with non-temporal loads).  This instantiation holds both ways and chooses per
//            document (DocCursor::cached, wave-uniform): with a map of the popular documents
//            (DocSource::popular) only those go through the caches and the others are streamed
//            past them the LINEAR way, which keeps the popular ones there (the same lists: 4.66 ->
//            4.4 ms per batch; 3.8 ms with the lists taken in id order, Batch::order).
//
// Work split.  A workgroup of WAVES waves owns a SLICE of one query's candidate list (up to
// MAX_SLICE consecutive candidates).  All its threads first look the slice's documents up
// (candidate id -> offset pair) and leave the descriptors in LDS, so the two dependent memory
// round trips are paid once per workgroup and not once per wave.  (Wave w also looks the w-th
// document up itself and requests its first tile before the barrier that ends the table fill, so
// that rows are on their way while the slowest look-up of the workgroup is still outstanding.)
// The waves then take the other documents of the slice one at a time through an LDS counter, which
// keeps every wave busy until the slice is exhausted however uneven the documents are.  The tiles of the documents a wave takes form one
// sequence that is software-pipelined P deep through registers: the load for tile u+P is issued
// right after tile u is consumed, across document boundaries.  Loads are unconditional (an
// exhausted cursor re-reads a row of its last tile) so that the number of loads in flight is static
// and the waits the compiler inserts are exact.
//
// A partial last tile: rows beyond the document's end are replaced by its last row (D >= 64: the
// load address is clamped; D = 32: the bpermute source is clamped).  A duplicated row cannot change
// a maximum, so no masking is needed.  Rows of the query beyond Q are zero vectors: they add
// max(0,..,0) = 0 to the sum.
//
// Ranking (RANK = true; launches with one slice of at most RANK_MAX candidates per query, such as the
// re-ranked prefix of partial re-ranking).  The workgroup also keeps the order keys of its scores
// and the ids in LDS and ranks them when the slice is done: the threads split the (entry,
// competitor) pairs among themselves and count, per entry, how many entries come before it (keys
// are read from LDS at addresses a whole wave shares and compared in vector registers; counting
// with one cross-lane vote per 64 competitors was measured slower, each vote stalling the wave
// on a vector-to-scalar hand-over); an entry whose count is below k writes itself
// to that rank.  No second launch.  Longer lists are ranked by the stand-alone kernel: it spreads
// the ranking of all queries over the whole device at once, which beats ranking at the tail of
// each workgroup, and slices of one query cannot meet cheaply (an agent-scope release / acquire
// pair per slice writes back and invalidates a whole L2 each: measured +25 % on the kernel).
// ---------------------------------------------------------------------------------------------
constexpr int MAX_SLICE = 1024;      // candidates per workgroup at most (LDS descriptor table)
constexpr int RANK_MAX = 256;        // candidates per query at most for ranking inside the scoring kernel

// Position of a wave in the sequence of tiles it streams (wave-uniform).
struct DocCursor {
    int64_t row0;       // first table row of the current document (ALIGN: of the cache line it starts in)
    int t;              // its row count (ALIGN: counted from row0, i.e. with the `lead` rows before it)
    int lead;           // ALIGN: rows of the first tile that precede the document (they share its first cache line)
    int tile;           // first row of the current tile (a multiple of the rows per tile)
    int idx;            // index of the current document in the slice
    bool done;          // moved past the last tile (position stays on the last tile)
    bool cached;        // the document is fetched through the caches (rows of 128 bytes and more: in the MFMA layout)
    __device__ __forceinline__ bool last_tile(int rows_per_tile) const { return tile + rows_per_tile >= t; }
};

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));

// Registers one lane holds of one tile: EB = bytes per component (2: binary16, 1: E4M3).  A tile is 16
// rows, one MFMA's worth; 32-byte rows (32 E4M3 codes) come 64 to a tile, two 16-byte loads per lane: a document
// of forty such rows is then one tile and not two (against tiles of 32 rows: 282-284 instead of 293 us per
// launch of 16 batches of 64 queries, 23.4-23.9 instead of 25.0 us per single batch).
template <int D, int EB>
struct TileBuf {
    static constexpr int ROWS = (D == 32 && EB == 1) ? 64 : 16;
    static constexpr int NW = ROWS * D * EB / 256;  // dwords
    unsigned w[NW];
};

template <int D, int EB, bool LINEAR>
__device__ __forceinline__ void issue_tile_load(TileBuf<D, EB> &buf, const uint8_t *__restrict__ emb,
                                                const DocCursor &cur, int lane)
{
    constexpr int ROW = D * EB;                    // bytes per row
    // A cursor that has run out of documents keeps loading, so that the number of loads in flight stays static:
    // one row of its last tile, not the whole tile again (P times per wave at the end of every slice; 2048 queries
    // with Zipf lists 3.80 -> 3.71 ms, 256 queries with uniform lists 1344 -> 1335 us per two batches, 64-byte rows
    // no difference; 32-byte rows lose 3 % by it and keep re-reading the tile).
    const int t = (cur.done && !(D == 32 && EB == 1)) ? cur.tile + 1 : cur.t;
    if (D > 32 && (LINEAR || !cur.cached)) {
        // lane-linear: the tile is 16 * ROW contiguous bytes; instruction x takes its x-th KiB, lane l the
        // l-th 16-byte piece of that.  Every byte is asked for exactly once, whole cache lines by one
        // instruction each: non-temporal loads.  Past the document's end: the last valid piece.
        const int npiece = min(16, t - cur.tile) * (ROW / 16);
        const uint4v *p = reinterpret_cast<const uint4v *>(emb + ((size_t)cur.row0 + cur.tile) * ROW);
#pragma unroll
        for (int x = 0; x < TileBuf<D, EB>::NW / 4; ++x) {
            const uint4v v = __builtin_nontemporal_load(p + min(64 * x + lane, npiece - 1));
            buf.w[4 * x] = v.x; buf.w[4 * x + 1] = v.y; buf.w[4 * x + 2] = v.z; buf.w[4 * x + 3] = v.w;
        }
    } else if constexpr (D == 32) {
        // lane-linear: the tile is 1 KiB (16 rows of 64 bytes) or 2 KiB (64 rows of 32 bytes), lane l loads its
        // l-th 16 bytes of every KiB; past the document's end: the last valid piece.  Every byte of the tile is
        // asked for exactly once, whole lines by one instruction each.  LINEAR: a non-temporal load (no claim on cache space the
        // look-ups could use: 1.5 % faster on a 32 us launch of binary16 rows, 1.9 % with 1024 queries a third
        // of whose documents repeat); otherwise an ordinary load, which leaves the rows in the caches for the
        // other queries of the batch that list the document (Zipf lists: 25 instead of 34 us).
        const int npiece = min(TileBuf<D, EB>::ROWS, t - cur.tile) * (ROW / 16);
        const uint4v *p = reinterpret_cast<const uint4v *>(emb + ((size_t)cur.row0 + cur.tile) * ROW);
#pragma unroll
        for (int x = 0; x < TileBuf<D, EB>::NW / 4; ++x) {
            uint4v v;
            if (LINEAR || !cur.cached) v = __builtin_nontemporal_load(p + min(64 * x + lane, npiece - 1));
            else v = p[min(64 * x + lane, npiece - 1)];
            buf.w[4 * x] = v.x; buf.w[4 * x + 1] = v.y; buf.w[4 * x + 2] = v.z; buf.w[4 * x + 3] = v.w;
        }
    } else {
        // lane (r, c) loads the c-th quarter of tile row r: D/2 contiguous bytes (binary16) or D/4 (E4M3)
        const int r = lane & 15, c = lane >> 4;
        const int row = min(cur.tile + r, t - 1);
        const uint4 *p = reinterpret_cast<const uint4 *>(emb + ((size_t)cur.row0 + row) * ROW + c * (ROW / 4));
#pragma unroll
        for (int x = 0; x < TileBuf<D, EB>::NW / 4; ++x) {
            const uint4 v = p[x];
            buf.w[4 * x] = v.x; buf.w[4 * x + 1] = v.y; buf.w[4 * x + 2] = v.z; buf.w[4 * x + 3] = v.w;
        }
    }
}

// Eight consecutive components as binary16: two dwords of E4M3 codes are widened exactly
// (v_cvt_scalef32_pk_f16_fp8 with scale 1), four dwords of binary16 are taken as they are.
template <int EB>
__device__ __forceinline__ half8 fragment_of(const unsigned *w)
{
    if constexpr (EB == 2) {
        const uint4 v = {w[0], w[1], w[2], w[3]};
        return __builtin_bit_cast(half8, v);
    } else {
        const half2v h01 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[0], 1.0f, false);
        const half2v h23 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[0], 1.0f, true);
        const half2v h45 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[1], 1.0f, false);
        const half2v h67 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[1], 1.0f, true);
        const half8 a = {h01[0], h01[1], h23[0], h23[1], h45[0], h45[1], h67[0], h67[1]};
        return a;
    }
}

// Shape of what a ranking kernel leaves (k = 0: no ranking); the rows themselves are BatchSet's out_ids / out_scores.
struct RankOut {
    int k;                  // entries per query
    int ldo;                // leading dimension of the output rows (>= k)
};

// LDS a workgroup keeps for ranking its slice (nothing when it only scores)
template <bool RANK>
struct RankLds {
    __attribute__((aligned(16))) unsigned key[RANK_MAX + 4];    // order_key of the scores, then zeros
    unsigned count[RANK_MAX];       // entries ahead (low half) and entries of equal score, itself included (high half)
    int64_t id[RANK_MAX];
};
template <>
struct RankLds<false> {};

// grid = B * slices workgroups of WAVES * 64 threads: a workgroup takes one slice of one query's list
template <int D, int WAVES, int P, int EB, bool RANK, int QG = 2, bool LINEAR = false>
__global__ __launch_bounds__(WAVES * 64) void maxsim_slice_kernel(
    const DocSource src, const Batch bt, const BatchSet set, unsigned *__restrict__ err, int slice, const RankOut ro)
{
    static_assert(D % 32 == 0 && D >= 32 && D <= 256 && (EB == 2 || D == 32 || D == 128) && WAVES >= 1 && WAVES <= 16 &&
                      P >= 1 && (QG == 2 || (QG == 4 && D <= 128)), "unsupported shape");
    __shared__ int64_t s_row0[MAX_SLICE];
    __shared__ int s_ntok[MAX_SLICE];
    __shared__ float s_scale[EB == 1 ? MAX_SLICE : 1];
    __shared__ int s_slot[MAX_SLICE];       // position in the query's list, | CACHED_BIT: fetched through the caches
    __shared__ int s_next;
    __shared__ RankLds<RANK> s_rank;
    // LINEAR: where a wave turns a tile from the order it was loaded in into the order the MFMA wants;
    // rows are one piece apart from a multiple of the bank period, so that the 16 rows a read touches
    // fall on different banks
    constexpr int ROW_PIECES = D * EB / 16;
    __shared__ uint4 s_tile[D > 32 ? WAVES * 16 * (ROW_PIECES + 1) : (D == 32 && EB == 1) ? WAVES * 2 * TileBuf<D, EB>::ROWS : 1];

    const uint8_t *__restrict__ emb = static_cast<const uint8_t *>(src.emb);
    const int Q = bt.Q, K = bt.K;
    // 64-byte binary16 rows: tiles start on 128-byte lines (a document that starts in the middle of a line takes
    // the row before it into its first tile and ignores it), so that no line is part of two tiles: a tile's load
    // is non-temporal, and a line that two tiles share was fetched twice (2.6 % of the bytes; a queue of 400
    // batches of 64 queries: 25.7 instead of 26.0 us per batch, measured twice each on one machine).  32-byte
    // rows (E4M3) lose 1-3 % by it (measured again in long launches), although a quarter of what they fetch is
    // such waste: that path is not bound by fetched bytes.
    constexpr bool ALIGN = D == 32 && EB == 2;
    constexpr int LINE_ROWS = 128 / (D * EB) > 0 ? 128 / (D * EB) : 1;      // rows per 128-byte line
    constexpr int KS = D / 32;              // MFMA steps per 16-row tile
    constexpr int CACHED_BIT = 1 << 30;
    constexpr int TR = TileBuf<D, EB>::ROWS;   // rows per load tile
    const int lane = threadIdx.x & 63;
    const int r = lane & 15, c = lane >> 4;
    const int xor16 = (lane ^ 16) * 4, xor32 = (lane ^ 32) * 4;     // ds_bpermute addresses
    // A one-dimensional grid of B * slices workgroups (slices = workgroups per query).  Workgroups are
    // handed to the eight XCDs (each with an L2 of its own) in turn, by linear index.  With a multiple of
    // eight queries, the slices of a query are given linear indices that are equal modulo 8, so that they
    // run on one XCD and share its copy of the query matrix.  An XCD takes its queries one after the other, all
    // slices of each; with lists in id order it takes the slices one after the other, each for all its queries.
    const unsigned slices = (unsigned)((K + slice - 1) / slice);
    const unsigned n_queries = gridDim.x / slices;
    int g = (int)(blockIdx.x / slices), slice_index = (int)(blockIdx.x % slices);      // g: query of the launch
    const bool by_id = bt.order == ORDER_BY_ID;
    if (by_id) {                                                // slice by slice
        g = (int)(blockIdx.x % n_queries);
        slice_index = (int)(blockIdx.x / n_queries);
    }
    if ((n_queries & 7u) == 0u) {
        const unsigned within = blockIdx.x >> 3;                // position among the XCD's workgroups
        const unsigned per_xcd = n_queries >> 3;                // queries of an XCD
        g = (int)((blockIdx.x & 7u) + 8u * (by_id ? within % per_xcd : within / slices));
        slice_index = (int)(by_id ? within / per_xcd : within % slices);
    }
    // which batch of the launch the query belongs to (wave-uniform: the pointers stay in scalar registers)
    const int which = set.n > 1 ? g / set.B : 0;
    const int b = g - which * set.B;
    const uint16_t *__restrict__ q = set.q[which];
    const int64_t *__restrict__ cand = set.cand[which];
    const float *__restrict__ prior = set.prior[which];
    float *__restrict__ scores = set.scores[which];
    auto total_of = [&](int j, float maxsim) {                  // Sec. 3.1: MaxSim + alpha * first-stage score
        return prior ? fmaf(bt.alpha, prior[(size_t)b * bt.ldc + j], maxsim) : maxsim;
    };
    const int j_begin = slice_index * slice;
    const int n = min(slice, K - j_begin);  // >= 1 by construction of the grid

    // Wave w starts on the w-th document of the slice without waiting for anybody: it looks that
    // document up itself and requests its first tile, so rows are on their way while the slice's
    // descriptor table is still being filled (which ends with a barrier, i.e. with the slowest
    // look-up of the workgroup).
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));     // in a scalar register
    const size_t cand0 = (size_t)b * bt.ldc + j_begin;
    int64_t id_own = -1, id_fill = -1;
    if (wave < n) id_own = cand[cand0 + wave];
    if ((int)threadIdx.x < n) id_fill = cand[cand0 + threadIdx.x];
    if (by_id) id_own >>= SLOT_BITS;                            // (arithmetic: an id out of range is stored as -1)
    DocCursor ld, cs;
    ld.done = true;
    ld.idx = wave;
    ld.tile = 0;
    {
        int64_t row0 = 0;
        int ntok = 0;
        if (wave < n) locate_document(src, id_own, nullptr, row0, ntok);   // flags are raised by the table fill
        ld.t = __builtin_amdgcn_readfirstlane(ntok);
        ld.row0 = readlane64(row0, 0);
        ld.lead = 0;
        ld.cached = __builtin_amdgcn_readfirstlane((int)is_popular(src, id_own)) != 0;
        if constexpr (ALIGN) {
            ld.lead = ld.t > 0 ? (int)(ld.row0 & (LINE_ROWS - 1)) : 0;
            ld.row0 -= ld.lead;
            ld.t += ld.lead;
        }
    }
    const bool own_first = ld.t > 0;
    TileBuf<D, EB> buf[P];
    if (own_first) {
        ld.done = false;
        issue_tile_load<D, EB, LINEAR>(buf[0], emb, ld, lane);
    }

    // descriptors of the slice's documents; a document with nothing to read has its score here
    for (int i = threadIdx.x; i < n; i += WAVES * 64) {
        int64_t id = i == (int)threadIdx.x ? id_fill : cand[cand0 + i];
        int slot = j_begin + i;
        if (by_id) {
            slot = (int)(id & SLOT_MASK);
            id >>= SLOT_BITS;
        }
        int64_t row0;
        int ntok;
        locate_document(src, id, err, row0, ntok);
        s_row0[i] = row0;
        s_ntok[i] = ntok;
        s_slot[i] = slot | (is_popular(src, id) ? CACHED_BIT : 0);
        if constexpr (EB == 1) s_scale[i] = ntok > 0 ? src.doc_scale[id] : 1.f;
        if constexpr (RANK) s_rank.id[i] = id;
        if (ntok == 0) {
            const float none = total_of(slot, neg_inf());
            scores[(size_t)b * K + slot] = none;
            if constexpr (RANK) s_rank.key[i] = order_key(none);
        }
    }
    if (threadIdx.x == 0) s_next = min(WAVES, n);      // the first WAVES documents are spoken for
    if constexpr (RANK) {
        if (threadIdx.x < 4) s_rank.key[n + threadIdx.x] = 0u;
        if (threadIdx.x < RANK_MAX) s_rank.count[threadIdx.x] = 0u;
    }

    // query fragments: qf[h][s] = components 8*(KS*c+s) .. +7 of query row r + 16h (QG groups of 16 rows)
    half8 qf[QG][KS];
#pragma unroll
    for (int h = 0; h < QG; ++h) {
        const int nq = r + 16 * h;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (nq < Q) v = *reinterpret_cast<const half8 *>(q + ((size_t)b * Q + nq) * D + 8 * (KS * c + s));
            qf[h][s] = v;
        }
    }
    __syncthreads();

    // the next document of the slice that has rows, or -1 (wave-uniform)
    auto grab = [&]() -> int {
        while (true) {
            int i = 0;
            if (lane == 0) i = atomicAdd(&s_next, 1);
            i = __builtin_amdgcn_readfirstlane(i);
            if (i >= n) return -1;
            if (__builtin_amdgcn_readfirstlane(s_ntok[i]) > 0) return i;
        }
    };
    auto enter = [&](DocCursor &cur, int i) {
        cur.idx = i;
        cur.t = __builtin_amdgcn_readfirstlane(s_ntok[i]);
        cur.row0 = readlane64(s_row0[i], 0);
        cur.tile = 0;
        cur.lead = 0;
        cur.cached = (__builtin_amdgcn_readfirstlane(s_slot[i]) & CACHED_BIT) != 0;
        if constexpr (ALIGN) {          // (only documents with rows are entered)
            cur.lead = (int)(cur.row0 & (LINE_ROWS - 1));
            cur.row0 -= cur.lead;
            cur.t += cur.lead;
        }
    };

    // The load cursor runs P tiles ahead of the compute cursor; lane (s & 63) of `ring` remembers
    // which document was the s-th one the wave took, for the compute cursor to follow.
    int ring = wave, ld_seq = 1, cs_seq = 1;
    if (!own_first) {
        // nothing of its own (an empty document, or fewer documents than waves): take one from the rest
        const int i = grab();
        if (i >= 0) {
            enter(ld, i);
            ld.done = false;
            ring = i;
            issue_tile_load<D, EB, LINEAR>(buf[0], emb, ld, lane);
        }
    }
    if (!ld.done) {
        cs = ld;

        auto ld_advance = [&]() {
            if (ld.done) return;
            if (!ld.last_tile(TR)) { ld.tile += TR; return; }
            const int i = grab();
            if (i < 0) { ld.done = true; return; }
            enter(ld, i);
            if (lane == (ld_seq & 63)) ring = i;
            ++ld_seq;
        };
        auto cs_advance = [&]() {
            if (!cs.last_tile(TR)) { cs.tile += TR; return; }
            // the load cursor has left this document already: no further one means the end
            if (cs_seq == ld_seq) { cs.done = true; return; }
            enter(cs, __builtin_amdgcn_readlane(ring, cs_seq & 63));
            ++cs_seq;
        };

        ld_advance();
#pragma unroll
        for (int p = 1; p < P; ++p) {
            issue_tile_load<D, EB, LINEAR>(buf[p], emb, ld, lane);
            ld_advance();
        }

        float m[QG];
#pragma unroll
        for (int h = 0; h < QG; ++h) m[h] = neg_inf();
        while (!cs.done) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (!cs.done) {
                    // 16 rows, as MFMA operand fragments, against the query: maxima into m
                    auto contract = [&](const half8 (&a)[KS]) {
                        floatx4 acc[QG];
#pragma unroll
                        for (int h = 0; h < QG; ++h) acc[h] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int s = 0; s < KS; ++s) {
#pragma unroll
                            for (int h = 0; h < QG; ++h)
                                acc[h] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[s], qf[h][s], acc[h], 0, 0, 0);
                        }
#pragma unroll
                        for (int h = 0; h < QG; ++h) m[h] = max_into(m[h], acc[h]);
                    };
                    half8 a[KS];
                    if constexpr (D == 32 && EB == 1) {
                        // 64 rows of 32 bytes as loaded: lane l holds bytes [16 l, 16 l + 16) of each KiB of the tile.
                        // Through the wave's own 2 KiB of LDS, lane (r, c) takes bytes [8 c, 8 c + 8) of row
                        // min(16 x + r, rows-1) of each quarter x of the tile (a quarter is contracted only if the
                        // document reaches into it)
                        uint4 *scr = s_tile + wave * 2 * TR;
#pragma unroll
                        for (int x = 0; x < TR / 32; ++x)
                            scr[64 * x + lane] = uint4{buf[p].w[4 * x], buf[p].w[4 * x + 1], buf[p].w[4 * x + 2], buf[p].w[4 * x + 3]};
                        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        const int rows = min(TR, cs.t - cs.tile);
                        const int first = cs.tile == 0 ? cs.lead : 0;          // ALIGN: rows before the document are not its own
                        const uint2 *pieces = reinterpret_cast<const uint2 *>(scr);
                        uint2 part[TR / 16];
                        part[0] = pieces[4 * max(min(r, rows - 1), first) + c];
#pragma unroll
                        for (int x = 1; x < TR / 16; ++x) part[x] = pieces[4 * min(16 * x + r, rows - 1) + c];
                        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                        __builtin_amdgcn_wave_barrier();
#pragma unroll
                        for (int x = 0; x < TR / 16; ++x) {
                            if (x == 0 || rows > 16 * x) {       // wave-uniform
                                const unsigned w_x[2] = {part[x].x, part[x].y};
                                a[0] = fragment_of<EB>(w_x);
                                contract(a);
                            }
                        }
                    } else {
                        if constexpr (D == 32) {
                            // lane (r, c) takes piece c of tile row min(r, rows-1) from lane 4*row + c
                            const int rows = min(16, cs.t - cs.tile);
                            const int first = cs.tile == 0 ? cs.lead : 0;      // ALIGN: the row before the document is not its own
                            const int from = (4 * max(min(r, rows - 1), first) + c) * 4;
                            unsigned w[TileBuf<D, EB>::NW];
#pragma unroll
                            for (int x = 0; x < TileBuf<D, EB>::NW; ++x)
                                w[x] = (unsigned)__builtin_amdgcn_ds_bpermute(from, (int)buf[p].w[x]);
                            a[0] = fragment_of<EB>(w);
                        } else if (LINEAR || !cs.cached) {      // D > 32, loaded lane-linearly
                            // piece q of the tile (row q / ROW_PIECES, position q % ROW_PIECES) is in register
                            // group q / 64 of lane q % 64; lane (r, c) wants pieces c * NW/4 .. of row min(r, rows-1)
                            constexpr int NX = TileBuf<D, EB>::NW / 4;
                            uint4 *scr = s_tile + wave * 16 * (ROW_PIECES + 1);
#pragma unroll
                            for (int x = 0; x < NX; ++x) {
                                const int q = 64 * x + lane;
                                scr[(q / ROW_PIECES) * (ROW_PIECES + 1) + q % ROW_PIECES] =
                                    uint4{buf[p].w[4 * x], buf[p].w[4 * x + 1], buf[p].w[4 * x + 2], buf[p].w[4 * x + 3]};
                            }
                            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                            __builtin_amdgcn_wave_barrier();
                            const int rows = min(16, cs.t - cs.tile);
                            const uint4 *mine = scr + min(r, rows - 1) * (ROW_PIECES + 1) + c * NX;
                            unsigned w[TileBuf<D, EB>::NW];
#pragma unroll
                            for (int x = 0; x < NX; ++x) {
                                const uint4 v = mine[x];
                                w[4 * x] = v.x; w[4 * x + 1] = v.y; w[4 * x + 2] = v.z; w[4 * x + 3] = v.w;
                            }
                            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                            __builtin_amdgcn_wave_barrier();
#pragma unroll
                            for (int s = 0; s < KS; ++s) a[s] = fragment_of<EB>(&w[2 * EB * s]);
                        } else {
#pragma unroll
                            for (int s = 0; s < KS; ++s) a[s] = fragment_of<EB>(&buf[p].w[2 * EB * s]);
                        }
                        contract(a);
                    }
                    if (cs.last_tile(TR)) {
                        // max over the four row groups (lanes l, l^16, l^32, l^48 hold the same query row)
#pragma unroll
                        for (int h = 0; h < QG; ++h) {
                            m[h] = max3(m[h], from_lane(xor16, m[h]), m[h]);
                            m[h] = max3(m[h], from_lane(xor32, m[h]), m[h]);
                        }
                        // sum over the query rows: rows r, r+16, ... in-lane, then across the 16 lanes
                        float in_lane = m[0];
#pragma unroll
                        for (int h = 1; h < QG; ++h) in_lane += m[h];
                        float sum = row16_sum(in_lane);
#pragma unroll
                        for (int h = 0; h < QG; ++h) m[h] = neg_inf();
                        // one positive scale per document: max and sum commute with it
                        if constexpr (EB == 1) sum *= s_scale[cs.idx];
                        if (lane == 0) {
                            const int slot = s_slot[cs.idx] & ~CACHED_BIT;
                            const float total = total_of(slot, sum);
                            scores[(size_t)b * K + slot] = total;
                            if constexpr (RANK) s_rank.key[cs.idx] = order_key(total);
                        }
                    }
                    cs_advance();
                }
                issue_tile_load<D, EB, LINEAR>(buf[p], emb, ld, lane);
                ld_advance();
            }
        }
    }

    if constexpr (RANK) {
        // one slice per query and n <= RANK_MAX <= blockDim.x: the slice is the query's whole list.
        // Order: score descending, id ascending, position ascending; NaN scores (key 0) are never
        // ranked.  An entry's rank is the number of entries ahead of it.  The threads form a
        // (entries x parts) grid: thread (e, part) compares entry e with the part-th share of the
        // list (keys read from LDS at addresses the whole wave shares, counts kept in vector
        // registers, no cross-lane votes) and adds what it found to the entry's counter.
        constexpr int T = WAVES * 64;
        constexpr int LG_T = T == 1024 ? 10 : T == 512 ? 9 : T == 256 ? 8 : -1;
        static_assert(LG_T > 0 && RANK_MAX == 256 && RANK_MAX <= T, "one thread per entry at least");
        __syncthreads();                                      // every key is in LDS
        const int lg = n <= 64 ? 6 : n <= 128 ? 7 : 8;        // entries rounded up to 64, 128 or 256 columns
        const int e = threadIdx.x & ((1 << lg) - 1);
        const int part = threadIdx.x >> lg;                   // wave-uniform
        const int groups = (n + 3) >> 2;                      // keys are read four at a time; keys n .. n+3 are zero
        const int per = (groups + (T >> lg) - 1) >> (LG_T - lg);
        const int j_end = min(groups, (part + 1) * per) * 4;
        const unsigned mine = e < n ? s_rank.key[e] : 0u;
        int ahead = 0, same = 0;
        for (int j = part * per * 4; j < j_end; j += 4) {
            const uint4 kk = *reinterpret_cast<const uint4 *>(&s_rank.key[j]);
            ahead += (kk.x > mine) + (kk.y > mine) + (kk.z > mine) + (kk.w > mine);
            same += (kk.x == mine) + (kk.y == mine) + (kk.z == mine) + (kk.w == mine);
        }
        if (mine != 0u && (ahead | same) != 0) atomicAdd(&s_rank.count[e], (unsigned)ahead | ((unsigned)same << 16));
        __syncthreads();
        int64_t *oi = set.out_ids[which] + (size_t)b * ro.ldo;
        float *os = set.out_scores[which] + (size_t)b * ro.ldo;
        if (part == 0 && mine != 0u) {
            const unsigned found = s_rank.count[e];
            int rank = (int)(found & 0xffffu);
            const int64_t id = s_rank.id[e];
            if ((found >> 16) > 1u) {                         // the ids only matter among equal scores
                for (int j = 0; j < n; ++j) {
                    if (s_rank.key[j] != mine) continue;
                    const int64_t other = s_rank.id[j];
                    rank += other < id || (other == id && j < e);
                }
            }
            if (rank < ro.k) {
                oi[rank] = id;
                os[rank] = key_to_score(mine);
            }
        }
        // ranks nothing can fill
        if (wave == 0) {
            int rankable = 0;
            for (int j = 0; j < n; j += 64)
                rankable += __builtin_popcountll(__ballot(j + lane < n && s_rank.key[min(j + lane, n - 1)] != 0u));
            for (int rest = rankable + lane; rest < ro.k; rest += 64) {
                oi[rest] = -1;
                os[rest] = quiet_nan();
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Generic kernel: any D multiple of 8, any Q whose matrix fits the dynamic LDS given at launch.
// One wave per candidate; lanes stride over the document's rows; the query matrix is in LDS and
// is read as wave-wide broadcasts.  Query rows are taken 16 at a time.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void unpack8(const uint4 &u, float (&f)[8])
{
    const _Float16 *hp = reinterpret_cast<const _Float16 *>(&u);
#pragma unroll
    for (int x = 0; x < 8; ++x) f[x] = (float)hp[x];
}

__global__ __launch_bounds__(256) void maxsim_generic_kernel(
    const DocSource src, int D, const Batch bt, float *__restrict__ scores, unsigned *__restrict__ err)
{
    const uint16_t *__restrict__ q = bt.q;
    const int Q = bt.Q, K = bt.K;
    extern __shared__ uint4 q_lds[];         // [Q][D/8] chunks of 8 binary16
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const unsigned per_query = (unsigned)((K + 3) / 4);     // one-dimensional grid: B * ceil(K / 4) workgroups
    const int b = (int)(blockIdx.x / per_query);
    const int chunks = D / 8;
    const uint4 *qsrc = reinterpret_cast<const uint4 *>(q + (size_t)b * Q * D);
    for (int x = threadIdx.x; x < Q * chunks; x += blockDim.x) q_lds[x] = qsrc[x];
    __syncthreads();

    const int j = (int)(blockIdx.x % per_query) * 4 + wave;
    if (j >= K) return;
    int64_t s0;
    int t;
    {
        // lane 0 looks the document up (and raises the flag once), the wave shares the result
        int64_t s0_lane = 0;
        int t_lane = 0;
        if (lane == 0) locate_document(src, bt.cand[(size_t)b * bt.ldc + j], err, s0_lane, t_lane);
        s0 = readlane64(s0_lane, 0);
        t = __builtin_amdgcn_readlane(t_lane, 0);
    }
    const uint4 *rows = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(src.emb) + (size_t)s0 * D);

    float total = 0.f;
    for (int i0 = 0; i0 < Q; i0 += 16) {
        const int nq = min(16, Q - i0);
        float best[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) best[i] = neg_inf();
        for (int row = lane; row < t; row += 64) {
            float dot[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) dot[i] = 0.f;
            for (int ch = 0; ch < chunks; ++ch) {
                float x[8], y[8];
                unpack8(rows[(size_t)row * chunks + ch], x);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (i < nq) {
                        unpack8(q_lds[(i0 + i) * chunks + ch], y);
#pragma unroll
                        for (int e = 0; e < 8; ++e) dot[i] = fmaf(x[e], y[e], dot[i]);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) best[i] = fmaxf(best[i], dot[i]);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float m = best[i];
#pragma unroll
            for (int sh = 32; sh >= 1; sh >>= 1) m = fmaxf(m, __shfl_xor(m, sh));
            if (i < nq) total += m;
        }
    }
    if (lane == 0) scores[(size_t)b * K + j] = with_prior(bt, b, j, total);
}

}  // namespace espn
