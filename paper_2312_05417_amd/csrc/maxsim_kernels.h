// MaxSim scoring kernels for gfx950 (CDNA4): fused candidate gather + Eq. 1 (Sec. 2.1).
//
//   score[b,j] = sum_{i<Q} max_{r in doc(cand[b,j])} <q[b,i,:], emb[r,:]>
//
// Two kernels:
//   maxsim_mfma_kernel<D>   D in {32,128}: the Q x D x t contraction of each document runs on the
//                           matrix cores (v_mfma_f32_16x16x32_f16); document rows stream from HBM
//                           straight into the MFMA A operand, the query sits in VGPRs.
//   maxsim_generic_kernel   any D multiple of 8, any Q: plain FMA, one wave per document.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace espn {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr unsigned ERR_ID_RANGE = 1u;

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

__device__ __forceinline__ int64_t readlane64(int64_t v, int lane)
{
    unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), lane);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// ---------------------------------------------------------------------------------------------
// Matrix-core kernel.
//
// One wave scores DOCS consecutive candidates of one query.  v_mfma_f32_16x16x32_f16 computes a
// 16x16 tile C[m][n] += sum_k A[m][k] B[k][n] with k = 0..31; lane l supplies A[l%16][8*(l/16)..+7]
// and B[8*(l/16)..+7][l%16] and receives C[4*(l/16)+v][l%16], v = 0..3.  Here m indexes 16
// document rows (tokens), n indexes 16 query rows, so after the MFMA a lane holds the dot products
// of ONE query row with FOUR document rows: the max over document rows is mostly an in-lane
// v_max over accumulator registers, finished by two cross-lane steps per document, and the sum over
// query rows is a 16-lane reduction per document.
//
// The dot product does not care in which order the D components are visited as long as both
// operands agree, so the k slots are assigned such that a lane's A fragments for successive MFMA
// steps are ADJACENT bytes of one table row: lane (r = l%16, c = l/16) reads bytes
// [c*D/2, (c+1)*D/2) of row r of the tile (16 B for D=32, 64 B for D=128).  The query fragments
// are gathered once per wave with the same assignment.
//
// A partial last tile re-reads the document's last row for the missing rows: a duplicated row
// cannot change a maximum, so no masking is needed.  Rows of the query beyond Q are zero vectors:
// they add max(0,..,0) = 0 to the sum.
// ---------------------------------------------------------------------------------------------
template <int D, int DOCS>
__global__ __launch_bounds__(256) void maxsim_mfma_kernel(
    const uint16_t *__restrict__ emb, const int64_t *__restrict__ off, int64_t n_docs,
    const uint16_t *__restrict__ q, const int64_t *__restrict__ cand,
    int B, int Q, int K, float *__restrict__ scores, unsigned *__restrict__ err)
{
    static_assert(D % 32 == 0 && DOCS >= 1 && DOCS <= 64, "unsupported tile shape");
    constexpr int KS = D / 32;              // MFMA steps per 16-row tile
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int b = blockIdx.y;
    const int j0 = (blockIdx.x * 4 + wave) * DOCS;   // first candidate slot of this wave
    if (j0 >= K) return;
    const int ndoc = min(DOCS, K - j0);

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

    // per-lane document descriptors: lane i describes candidate j0 + i
    int64_t row0 = 0;
    int ntok = -1;                           // -1: invalid id
    if (lane < ndoc) {
        const int64_t id = cand[(size_t)b * K + j0 + lane];
        if (id >= 0 && id < n_docs) {
            row0 = off[id];
            ntok = (int)(off[id + 1] - row0);
        } else {
            atomicOr(err, ERR_ID_RANGE);
        }
    }

    float result = neg_inf();                // lane i keeps the score of candidate j0 + i
    for (int i = 0; i < ndoc; ++i) {
        const int t = __builtin_amdgcn_readlane(ntok, i);
        if (t <= 0) continue;                // empty or invalid: -inf
        const int64_t s0 = readlane64(row0, i);
        const uint16_t *base = emb + (size_t)s0 * D + 8 * KS * c;
        float m0 = neg_inf(), m1 = neg_inf();
        for (int tile = 0; tile < t; tile += 16) {
            const int row = min(tile + r, t - 1);
            const half8 *p = reinterpret_cast<const half8 *>(base + (size_t)row * D);
            half8 a[KS];
#pragma unroll
            for (int s = 0; s < KS; ++s) a[s] = p[s];
            floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[s], qf[0][s], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[s], qf[1][s], acc1, 0, 0, 0);
            }
            m0 = fmaxf(m0, fmaxf(fmaxf(acc0[0], acc0[1]), fmaxf(acc0[2], acc0[3])));
            m1 = fmaxf(m1, fmaxf(fmaxf(acc1[0], acc1[1]), fmaxf(acc1[2], acc1[3])));
        }
        // max over the four row groups (lanes l, l^16, l^32, l^48 hold the same query row)
        m0 = fmaxf(m0, __shfl_xor(m0, 16));
        m1 = fmaxf(m1, __shfl_xor(m1, 16));
        m0 = fmaxf(m0, __shfl_xor(m0, 32));
        m1 = fmaxf(m1, __shfl_xor(m1, 32));
        // sum over the 32 query rows: rows r and r+16 in-lane, then over the 16 lanes of a group
        float sum = m0 + m1;
        sum += __shfl_xor(sum, 1);
        sum += __shfl_xor(sum, 2);
        sum += __shfl_xor(sum, 4);
        sum += __shfl_xor(sum, 8);
        if (lane == i) result = sum;
    }
    if (lane < ndoc) scores[(size_t)b * K + j0 + lane] = result;
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
    const uint16_t *__restrict__ emb, const int64_t *__restrict__ off, int64_t n_docs, int D,
    const uint16_t *__restrict__ q, const int64_t *__restrict__ cand,
    int B, int Q, int K, float *__restrict__ scores, unsigned *__restrict__ err)
{
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
    const int64_t id = cand[(size_t)b * K + j];
    if (id < 0 || id >= n_docs) {
        if (lane == 0) {
            atomicOr(err, ERR_ID_RANGE);
            scores[(size_t)b * K + j] = neg_inf();
        }
        return;
    }
    const int64_t s0 = off[id];
    const int t = (int)(off[id + 1] - s0);
    const uint4 *rows = reinterpret_cast<const uint4 *>(emb + (size_t)s0 * D);

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
    if (lane == 0) scores[(size_t)b * K + j] = total;
}

}  // namespace espn
