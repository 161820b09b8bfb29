// Pieces of the layer product H = Z W (Section 3, Eq. 1) on the fp64 matrix cores that more than one kernel uses:
// tile loads with clamped addresses and their way into LDS.
#pragma once
#include "common.hpp"

namespace csgs {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BK = 32;
constexpr int LDS_STRIDE = BK + 4;

template <int V>
__device__ inline float4 load4(const float *__restrict__ p)
{
    if (V == 4) return *reinterpret_cast<const float4 *>(p);
    if (V == 2) {
        const float2 a = *reinterpret_cast<const float2 *>(p);
        const float2 b = *reinterpret_cast<const float2 *>(p + 2);
        return make_float4(a.x, a.y, b.x, b.y);
    }
    return make_float4(p[0], p[1], p[2], p[3]);
}

// The same kernel serves the layer's forward product and its two gradient products; they differ in
// how the operands lie in memory and in where the result goes:
//   FWD  H  = Z W        A(m,k) = Z[m][k]           B(k,n) = W[k][n]      C float [M x N]
//   DZ   dZ = G W^T      A(m,k) = G[m][k]           B(k,n) = W[n][k]      C float [M x N]
//   DW   dW = Z^T G      A(m,k) = Z[k][m]           B(k,n) = G[k][n]      partial sums in double,
//        the reduction dimension (the rows of the sampled layer) split over blockIdx.y; a second
//        kernel adds the parts in a fixed order.
enum { MODE_FWD = 0, MODE_DZ = 1, MODE_DW = 2 };

// Loads of a tile never sit in divergent control flow (a wavefront would then wait for each load
// before it issues the next): a group that is out of range reads a clamped, valid address instead, and
// a bit of `ok` per loaded piece says whether the value counts; stash_tile() turns the others into
// zeros on the way to LDS, after the MFMAs of the current chunk.
//
// Tile [ROWS][BK] of a matrix whose element (r, k) sits at P[r * ld + k] (k contiguous): ROWS * 8
// groups of 4 consecutive k; thread t takes groups t + 256 i, each as 4 / V pieces of V floats
// (the host picks V so that K is a multiple of it: a piece is inside the row or outside).  Bit
// 4 i + j of `ok` belongs to float j of group i.
template <int ROWS, int V, bool FULL>
__device__ inline void fetch_kmajor(const float *__restrict__ P, int64_t ld, int R, int K, int64_t r0, int k0, int tid,
                                    float4 (&reg)[ROWS / 32], uint32_t &ok)
{
    ok = 0;
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int idx = tid + i * 256;
        const int r = idx >> 3, kq = (idx & 7) * 4;
        const int64_t gr = r0 + r;
        const int gk = k0 + kq;
        if (FULL) {
            reg[i] = load4<V>(P + gr * ld + gk);
        } else {
            const bool row_ok = gr < R;
            const float *row = P + (row_ok ? gr : (int64_t)R - 1) * ld;
            float t[4];
#pragma unroll
            for (int j = 0; j < 4; j += V) {
                const bool k_ok = gk + j + V <= K;
                const bool in = row_ok && k_ok;
                const float *q = row + (k_ok ? gk + j : K - V);   // the last whole piece of a real row stands in
                if (V == 4) {
                    const float4 v = *reinterpret_cast<const float4 *>(q);
                    t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
                } else if (V == 2) {
                    const float2 v = *reinterpret_cast<const float2 *>(q);
                    t[j] = v.x; t[j + 1] = v.y;
                } else {
                    t[j] = *q;
                }
                if (in) ok |= ((1u << V) - 1u) << (4 * i + j);
            }
            reg[i] = make_float4(t[0], t[1], t[2], t[3]);
        }
    }
}

// Tile [ROWS][BK] of a matrix whose element (r, k) sits at P[k * ld + r] (r contiguous).  Lane <-> r
// (coalesced across lanes), each thread takes runs of 4 consecutive k of one r, which become one
// 128-bit store into the LDS tile.
template <int ROWS, bool FULL>
__device__ inline void fetch_rmajor(const float *__restrict__ P, int64_t ld, int R, int K, int64_t r0, int k0, int tid,
                                    float4 (&reg)[ROWS / 32], uint32_t &ok)
{
    ok = 0;
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int idx = tid + i * 256;          // ROWS * 8 groups
        const int r = idx % ROWS, kg = (idx / ROWS) * 4;
        const int64_t gr = r0 + r;
        const int gk = k0 + kg;
        float t[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool r_ok = FULL || gr < R, k_ok = FULL || gk + j < K;
            t[j] = P[(int64_t)(k_ok ? gk + j : K - 1) * ld + (r_ok ? gr : (int64_t)R - 1)];   // the nearest real element stands in
            if (r_ok && k_ok) ok |= 1u << (4 * i + j);
        }
        reg[i] = make_float4(t[0], t[1], t[2], t[3]);
    }
}

// Registers -> LDS tile [ROWS][LDS_STRIDE], with the (r, k) of each group as the fetch above had it;
// values whose bit in `ok` is clear become zeros.
// SWZ: rows of 32 words without padding; the 16-byte column c of row r sits at column c ^ ((r >> 1) & 7), which
// spreads 16 consecutive rows' reads of one column over all banks as the padding does, in 8/9 of the space.
template <int ROWS, bool KMAJOR, bool FULL, bool SWZ = false>
__device__ inline void stash_tile(float *S, int tid, const float4 (&reg)[ROWS / 32], uint32_t ok, bool whole)
{
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int idx = tid + i * 256;
        const int r = KMAJOR ? (idx >> 3) : (idx % ROWS);
        const int k = KMAJOR ? (idx & 7) * 4 : (idx / ROWS) * 4;
        float4 v = reg[i];
        if (!FULL && !whole) {   // `whole` is the same for the whole block: every bit of `ok` is set
            v.x = (ok >> (4 * i + 0)) & 1u ? v.x : 0.f;
            v.y = (ok >> (4 * i + 1)) & 1u ? v.y : 0.f;
            v.z = (ok >> (4 * i + 2)) & 1u ? v.z : 0.f;
            v.w = (ok >> (4 * i + 3)) & 1u ? v.w : 0.f;
        }
        if (SWZ) *reinterpret_cast<float4 *>(&S[r * BK + (((k >> 2) ^ ((r >> 1) & 7)) << 2)]) = v;
        else *reinterpret_cast<float4 *>(&S[r * LDS_STRIDE + k]) = v;
    }
}

}  // namespace csgs
