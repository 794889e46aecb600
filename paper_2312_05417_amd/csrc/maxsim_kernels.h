// MaxSim scoring kernels for gfx950 (CDNA4): fused candidate gather + Eq. 1 (Sec. 2.1).
//
//   score[b,j] = sum_{i<Q} max_{r in doc(cand[b,j])} <q[b,i,:], emb[r,:]>
//
// Two kernels:
//   maxsim_mfma_kernel<D>   D in {32,128}: the Q x D x t contraction of each document runs on the
//                           matrix cores (v_mfma_f32_16x16x32_f16); document rows stream from HBM
//                           through a register pipeline into the MFMA A operand, the query sits
//                           in VGPRs.  Rows are binary16, or E4M3 codes widened exactly to binary16
//                           on the way into the MFMA.
//   maxsim_generic_kernel   any D multiple of 8, any Q: plain FMA, one wave per document.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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
};

// One batch of queries and their candidate lists.
//   cand  [B, ldc] ids, of which the first K of every row are scored (ldc >= K: partial re-ranking
//         scores a prefix of each list)
//   prior [B, ldc] first-stage scores or nullptr; score = MaxSim + alpha * prior (Sec. 3.1)
struct Batch {
    const uint16_t *q;      // [B, Q, D]
    const int64_t *cand;
    const float *prior;
    float alpha;
    int ldc;
    int Q;
    int K;
};

__device__ __forceinline__ float with_prior(const Batch &bt, int b, int j, float maxsim)
{
    return bt.prior ? fmaf(bt.alpha, bt.prior[(size_t)b * bt.ldc + j], maxsim) : maxsim;
}

// (first row, row count) of document `id`; count 0 and an error flag if it cannot be read.
__device__ __forceinline__ void locate_document(const DocSource &src, int64_t id, unsigned *err,
                                                int64_t &row0, int &ntok)
{
    row0 = 0;
    ntok = 0;
    if (id < 0 || id >= src.n_docs) {
        atomicOr(err, ERR_ID_RANGE);
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
        atomicOr(err, ERR_NOT_STAGED);
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
// One wave scores DOCS consecutive candidates of one query.  v_mfma_f32_16x16x32_f16 computes a
// 16x16 tile C[m][n] += sum_k A[m][k] B[k][n], k = 0..31; lane l supplies A[l%16][8*(l/16)..+7]
// and B[8*(l/16)..+7][l%16] and receives C[4*(l/16)+v][l%16], v = 0..3.  Here m indexes 16
// document rows (a "tile"), n indexes 16 query rows, so after the MFMA a lane holds the dot
// products of ONE query row with FOUR document rows: the max over document rows is mostly an
// in-lane v_max over accumulator registers carried across the tiles of a document, finished by two
// cross-lane steps per document; the sum over query rows is one 16-lane DPP reduction per document.
//
// The dot product does not care in which order the D components are visited as long as both
// operands agree.  The k slots are assigned so that what a lane feeds to successive MFMA steps are
// ADJACENT bytes of one table row (lane (r = l%16, c = l/16) owns bytes [c*D/2, (c+1)*D/2) of tile
// row r); the query fragments are gathered once per wave with the same assignment.
//
// How the rows reach that layout differs with the row length:
//   D = 128  a lane loads its 64 contiguous bytes directly (4 x global_load_dwordx4); measured, this
//            access pattern streams ragged documents at the same rate as lane-linear loads.
//   D = 32   a 16-row tile is 1 KiB; lane l loads bytes [16 l, 16 l + 16) of it (one fully
//            coalesced instruction), then four ds_bpermute_b32 move chunk c of row r from lane
//            4r + c to lane r + 16c.  Loading in the MFMA layout directly (16 B per lane at a 64 B
//            stride) was measured ~30 % slower on the same gather.
//
// All tiles of the wave's documents form one sequence that is software-pipelined P deep through
// registers: the load for tile u+P is issued right after tile u is consumed, across document
// boundaries.  Loads are unconditional (an exhausted cursor re-reads its last tile) so that the
// number of loads in flight is static and the waits the compiler inserts are exact.
//
// A partial last tile: rows beyond the document's end are replaced by its last row (D = 128: the
// load address is clamped; D = 32: the bpermute source is clamped).  A duplicated row cannot change
// a maximum, so no masking is needed.  Rows of the query beyond Q are zero vectors: they add
// max(0,..,0) = 0 to the sum.
// ---------------------------------------------------------------------------------------------

// Wave-uniform cursor over the tiles of the wave's non-empty documents.
struct TileCursor {
    uint64_t pending;   // documents not yet entered (bit i: candidate j0+i has rows)
    int doc;            // lane index of the current document
    int t;              // its row count
    int tile;           // first row of the current tile (multiple of 16)
    int64_t row0;       // its first table row
    bool done;          // moved past the last tile (position stays on the last tile)

    __device__ __forceinline__ void enter_next(int ntok, int64_t row0_lane)
    {
        doc = __builtin_ctzll(pending);
        pending &= pending - 1;
        t = __builtin_amdgcn_readlane(ntok, doc);
        row0 = readlane64(row0_lane, doc);
        tile = 0;
    }
    __device__ __forceinline__ bool last_tile() const { return tile + 16 >= t; }
    __device__ __forceinline__ void advance(int ntok, int64_t row0_lane)
    {
        if (!last_tile()) tile += 16;
        else if (pending) enter_next(ntok, row0_lane);
        else done = true;
    }
};

typedef _Float16 half2v __attribute__((ext_vector_type(2)));

// Registers one lane holds of one 16-row tile: EB = bytes per component (2: binary16, 1: E4M3).
template <int D, int EB>
struct TileBuf {
    static constexpr int NW = D / 32 * 2 * EB;     // dwords
    unsigned w[NW];
};

template <int D, int EB>
__device__ __forceinline__ void issue_tile_load(TileBuf<D, EB> &buf, const uint8_t *__restrict__ emb,
                                                const TileCursor &cur, int lane)
{
    constexpr int ROW = D * EB;                    // bytes per row
    if constexpr (D == 32) {
        // lane-linear: piece `lane` of the 64 pieces of the 16-row tile (16 B each for binary16 rows,
        // 8 B for E4M3 rows); past the document's end: the last valid piece
        const int npiece = min(16, cur.t - cur.tile) * 4;
        const uint8_t *p = emb + ((size_t)cur.row0 + cur.tile) * ROW;
        const int piece = min(lane, npiece - 1);
        if constexpr (EB == 2) {
            const uint4 v = reinterpret_cast<const uint4 *>(p)[piece];
            buf.w[0] = v.x; buf.w[1] = v.y; buf.w[2] = v.z; buf.w[3] = v.w;
        } else {
            const uint2 v = reinterpret_cast<const uint2 *>(p)[piece];
            buf.w[0] = v.x; buf.w[1] = v.y;
        }
    } else {
        // lane (r, c) loads the c-th quarter of tile row r: 64 contiguous bytes (binary16) or 32 (E4M3)
        const int r = lane & 15, c = lane >> 4;
        const int row = min(cur.tile + r, cur.t - 1);
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

// Scores candidates j0 .. j0+DOCS-1 (j0 < K) of query b with the calling wave and stores them.
template <int D, int DOCS, int P, int EB>
__device__ __forceinline__ void maxsim_mfma_wave(
    const DocSource &src, const Batch &bt, int b, int j0, float *__restrict__ scores, unsigned *__restrict__ err)
{
    const uint8_t *__restrict__ emb = static_cast<const uint8_t *>(src.emb);
    const uint16_t *__restrict__ q = bt.q;
    const int Q = bt.Q, K = bt.K;
    static_assert((D == 32 || D == 128) && DOCS >= 1 && DOCS <= 64 && P >= 1, "unsupported shape");
    constexpr int KS = D / 32;              // MFMA steps per 16-row tile
    const int lane = threadIdx.x & 63;
    const int r = lane & 15, c = lane >> 4;
    const int xor16 = (lane ^ 16) * 4, xor32 = (lane ^ 32) * 4;     // ds_bpermute addresses
    const int ndoc = min(DOCS, K - j0);

    // per-lane document descriptors: lane i describes candidate j0 + i
    int64_t row0 = 0;
    int ntok = 0;
    float doc_scale = 1.f;
    if (lane < ndoc) {
        const int64_t id = bt.cand[(size_t)b * bt.ldc + j0 + lane];
        locate_document(src, id, err, row0, ntok);
        if (EB == 1 && ntok > 0) doc_scale = src.doc_scale[id];
    }

    // query fragments: qf[h][s] = components 8*(KS*c+s) .. +7 of query row r + 16h
    half8 qf[2][KS];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int n = r + 16 * h;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (n < Q)
                v = *reinterpret_cast<const half8 *>(q + ((size_t)b * Q + n) * D + 8 * (KS * c + s));
            qf[h][s] = v;
        }
    }

    float result = neg_inf();                // lane i keeps the score of candidate j0 + i
    const uint64_t nonempty = __ballot(ntok > 0);
    if (nonempty) {
        TileCursor ld;
        ld.pending = nonempty;
        ld.done = false;
        ld.enter_next(ntok, row0);
        TileCursor cs = ld;

        TileBuf<D, EB> buf[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            issue_tile_load<D, EB>(buf[p], emb, ld, lane);
            ld.advance(ntok, row0);
        }

        float m0 = neg_inf(), m1 = neg_inf();
        while (!cs.done) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (!cs.done) {
                    half8 a[KS];
                    if constexpr (D == 32) {
                        // lane (r, c) takes piece c of tile row min(r, rows-1) from lane 4*row + c
                        const int rows = min(16, cs.t - cs.tile);
                        const int from = (4 * min(r, rows - 1) + c) * 4;
                        unsigned w[TileBuf<D, EB>::NW];
#pragma unroll
                        for (int x = 0; x < TileBuf<D, EB>::NW; ++x)
                            w[x] = (unsigned)__builtin_amdgcn_ds_bpermute(from, (int)buf[p].w[x]);
                        a[0] = fragment_of<EB>(w);
                    } else {
#pragma unroll
                        for (int s = 0; s < KS; ++s) a[s] = fragment_of<EB>(&buf[p].w[2 * EB * s]);
                    }
                    floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < KS; ++s) {
                        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[s], qf[0][s], acc0, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[s], qf[1][s], acc1, 0, 0, 0);
                    }
                    m0 = max_into(m0, acc0);
                    m1 = max_into(m1, acc1);
                    if (cs.last_tile()) {
                        // max over the four row groups (lanes l, l^16, l^32, l^48 hold the same query row)
                        m0 = max3(m0, from_lane(xor16, m0), m0);
                        m1 = max3(m1, from_lane(xor16, m1), m1);
                        m0 = max3(m0, from_lane(xor32, m0), m0);
                        m1 = max3(m1, from_lane(xor32, m1), m1);
                        // sum over the 32 query rows: rows r and r+16 in-lane, then across the 16 lanes
                        const float sum = row16_sum(m0 + m1);
                        if (lane == cs.doc) result = sum;
                        m0 = neg_inf();
                        m1 = neg_inf();
                    }
                    cs.advance(ntok, row0);
                }
                issue_tile_load<D, EB>(buf[p], emb, ld, lane);
                ld.advance(ntok, row0);
            }
        }
    }
    if (EB == 1) result *= doc_scale;        // one positive scale per document: max and sum commute with it
    if (lane < ndoc) scores[(size_t)b * K + j0 + lane] = with_prior(bt, b, j0 + lane, result);
}

// grid = (ceil(ceil(K / DOCS) / 4), B), 256 threads: wave w of workgroup x takes candidates
// (4x + w) * DOCS .. of query blockIdx.y
template <int D, int DOCS, int P, int EB>
__global__ __launch_bounds__(256) void maxsim_mfma_kernel(
    const DocSource src, const Batch bt, float *__restrict__ scores, unsigned *__restrict__ err)
{
    const int j0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * DOCS;
    if (j0 >= bt.K) return;
    maxsim_mfma_wave<D, DOCS, P, EB>(src, bt, blockIdx.y, j0, scores, err);
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
    const int b = blockIdx.y;
    const int chunks = D / 8;
    const uint4 *qsrc = reinterpret_cast<const uint4 *>(q + (size_t)b * Q * D);
    for (int x = threadIdx.x; x < Q * chunks; x += blockDim.x) q_lds[x] = qsrc[x];
    __syncthreads();

    const int j = blockIdx.x * 4 + wave;
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
