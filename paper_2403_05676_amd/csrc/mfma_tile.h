// fp32 MFMA tile product for gfx950: acc += A_tile x B_tile^T over the whole depth d, where A is a block of
// rows of one matrix and B a block of rows of another (both row-major, depth contiguous), i.e. the
// dot products <a_i, b_j>.  Used by the coarse quantiser (queries x centres) and by the encoder's list
// assignment (vectors x centres); the squared distance is then |a|^2 + |b|^2 - 2 <a, b>.
//
// Shape: one workgroup = 4 waves arranged WM x WN; a wave owns a patch of PM x PN blocks of
// v_mfma_f32_32x32x2f32 (32 x 32 each), so the workgroup tile is (32*PM*WM) rows of A by (32*PN*WN) rows of B.  The depth is walked
// in steps of TK: each thread fetches 16-byte pieces of the A and B rows from global memory (two steps ahead:
// one step is in registers on its way while another sits in the second LDS buffer), stores them depth-major
// in LDS (so that the 32 lanes of a half-wave read 32 consecutive floats), and the waves feed the matrix
// cores from there.  The instruction consumes two depth slots at a time, one from lanes 0-31 and one from
// lanes 32-63; A and B use the same pairing (k, k + TK/2), which is all that matters for a sum over the depth.
//
// Accumulator layout of one 32 x 32 block (checked on hardware): lane l, register r holds row
// (r % 4) + 4 * (l / 32) + 8 * (r / 4), column l % 32.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace piperag {

typedef float mfma_acc_t __attribute__((ext_vector_type(16)));

template <int WM, int WN, int PM, int PN, int TK = 16>
struct MfmaTile {
    static constexpr int kTileK = TK;          // depth per step (multiple of 16)
    static_assert(TK % 16 == 0, "depth step");
    static_assert(WM * WN == 4, "four waves per workgroup");
    static constexpr int kRowsA = 32 * PM * WM, kRowsB = 32 * PN * WN;
    static_assert(kRowsA % 64 == 0 && kRowsB % 64 == 0, "a depth step of a tile side is a whole number of 16-byte pieces per thread");
    static constexpr int kLdA = kRowsA + 1, kLdB = kRowsB + 1;
    static constexpr int kQ = kTileK / 4;                                                             // 16-byte pieces per row per step
    static constexpr int kPiecesA = kRowsA * kQ / 256, kPiecesB = kRowsB * kQ / 256;                  // pieces per thread
    static constexpr size_t kLdsFloats = 2 * (size_t)kTileK * (kLdA + kLdB);                          // double-buffered

    // Rows a_row0 .. of A (na rows in total, stride lda) against rows b_row0 .. of B (nb rows, stride ldb).
    // Rows beyond na / nb and depth beyond d read as zero.  d % 4 == 0, rows 16-byte aligned.
    // acc[bi][bj] is the block (rows 32*bi.., columns 32*bj..) of this wave's patch.
    __device__ static void run(const float *__restrict__ A, int64_t na, int64_t lda, int64_t a_row0,
                               const float *__restrict__ B, int64_t nb, int64_t ldb, int64_t b_row0, int d,
                               float *s_mem, mfma_acc_t (&acc)[PM][PN]) {
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
        const int wr = wave / WN, wc = wave % WN;
        float *sA[2] = {s_mem, s_mem + kTileK * kLdA};
        float *sB[2] = {s_mem + 2 * kTileK * kLdA, s_mem + 2 * kTileK * kLdA + kTileK * kLdB};
#pragma unroll
        for (int bi = 0; bi < PM; ++bi)
#pragma unroll
            for (int bj = 0; bj < PN; ++bj)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.f;

        struct Regs { float4 a[kPiecesA], b[kPiecesB]; };
        auto fetch = [&](Regs &rg, int k0) {
#pragma unroll
            for (int p = 0; p < kPiecesA; ++p) {
                const int e = tid + p * 256;             // piece index: row = e / kQ, depth piece = e % kQ
                const int64_t row = a_row0 + e / kQ;
                const int k = k0 + (e % kQ) * 4;
                rg.a[p] = (row < na && k < d) ? *reinterpret_cast<const float4 *>(A + row * lda + k) : float4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int p = 0; p < kPiecesB; ++p) {
                const int e = tid + p * 256;
                const int64_t row = b_row0 + e / kQ;
                const int k = k0 + (e % kQ) * 4;
                rg.b[p] = (row < nb && k < d) ? *reinterpret_cast<const float4 *>(B + row * ldb + k) : float4{0.f, 0.f, 0.f, 0.f};
            }
        };
        auto stash = [&](const Regs &rg, int buf) {
#pragma unroll
            for (int p = 0; p < kPiecesA; ++p) {
                const int e = tid + p * 256, row = e / kQ, kq = (e % kQ) * 4;
                sA[buf][(kq + 0) * kLdA + row] = rg.a[p].x; sA[buf][(kq + 1) * kLdA + row] = rg.a[p].y;
                sA[buf][(kq + 2) * kLdA + row] = rg.a[p].z; sA[buf][(kq + 3) * kLdA + row] = rg.a[p].w;
            }
#pragma unroll
            for (int p = 0; p < kPiecesB; ++p) {
                const int e = tid + p * 256, row = e / kQ, kq = (e % kQ) * 4;
                sB[buf][(kq + 0) * kLdB + row] = rg.b[p].x; sB[buf][(kq + 1) * kLdB + row] = rg.b[p].y;
                sB[buf][(kq + 2) * kLdB + row] = rg.b[p].z; sB[buf][(kq + 3) * kLdB + row] = rg.b[p].w;
            }
        };
        const int half = lane >> 5, l32 = lane & 31;
        auto multiply = [&](int buf) {
            const float *a_base = sA[buf] + wr * (32 * PM) + l32;
            const float *b_base = sB[buf] + wc * (32 * PN) + l32;
#pragma unroll
            for (int p = 0; p < kTileK / 2; ++p) {
                const int k = p + half * (kTileK / 2);          // lanes 0-31: depth p, lanes 32-63: depth p + TK/2
                float av[PM], bv[PN];
#pragma unroll
                for (int bi = 0; bi < PM; ++bi) av[bi] = a_base[k * kLdA + 32 * bi];
#pragma unroll
                for (int bj = 0; bj < PN; ++bj) bv[bj] = b_base[k * kLdB + 32 * bj];
#pragma unroll
                for (int bi = 0; bi < PM; ++bi)
#pragma unroll
                    for (int bj = 0; bj < PN; ++bj)
                        acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[bi], bv[bj], acc[bi][bj], 0, 0, 0);
            }
        };

        // Steps beyond the depth fetch zeros, so the pipeline needs no tail cases: step s is multiplied from LDS
        // buffer s % 2 while step s + 1 is stored into the other buffer and step s + 2 is being fetched.
        const int nsteps = (d + kTileK - 1) / kTileK;
        Regs r0, r1;
        fetch(r0, 0);
        fetch(r1, kTileK);
        __syncthreads();                 // the previous user of the LDS buffers is done
        stash(r0, 0);
        __syncthreads();
        for (int s = 0; s < nsteps; s += 2) {
            fetch(r0, (s + 2) * kTileK);
            multiply(0);
            stash(r1, 1);
            __syncthreads();
            if (s + 1 < nsteps) {
                fetch(r1, (s + 3) * kTileK);
                multiply(1);
                stash(r0, 0);
                __syncthreads();
            }
        }
    }

    // Row (within the workgroup tile) and column of accumulator register r of block (bi, bj) for this lane.
    __device__ static __forceinline__ int acc_row(int bi, int r) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        return (wave / WN) * (32 * PM) + bi * 32 + (r % 4) + 4 * (lane >> 5) + 8 * (r / 4);
    }
    __device__ static __forceinline__ int acc_col(int bj) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        return (wave % WN) * (32 * PN) + bj * 32 + (lane & 31);
    }
};

}  // namespace piperag
