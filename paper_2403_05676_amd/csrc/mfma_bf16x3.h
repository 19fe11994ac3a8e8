// Split-bf16 MFMA tile product for gfx950: dot products <a_i, b_j> of fp32 rows at close to fp32 accuracy on
// the bf16 matrix cores.  Every fp32 value v is written as hi + lo with hi = bf16(v) and lo = bf16(v - hi)
// (16 significant bits together); <a, b> ~ <a_hi, b_hi> + <a_hi, b_lo> + <a_lo, b_hi>, accumulated in fp32
// by three v_mfma_f32_32x32x16_bf16 per 32 x 32 block and 16 depth values.  The dropped lo*lo term and the
// rounding of lo are 2^-16 relative per product.  Used by the encoder's list assignment, where the centres'
// split is precomputed once and the vectors are split on the fly.
//
// Shape: workgroup = 4 waves as 2 x 2; a wave owns 128 rows of A x 64 rows of B = 4 x 2 blocks; the
// workgroup tile is 256 rows of A (fp32 in memory) by 128 rows of B (pre-split bf16 in memory).  Depth step
// 16.  LDS holds, per operand part, [depth half][row][8 bf16] so that the 32 lanes of a half-wave read 32
// consecutive 16-byte groups; lanes 0-31 take depth values 0-7 of the step and lanes 32-63 values 8-15, for
// A and B alike, which is all a sum over the depth needs.  Two steps are in flight: one in registers, one in
// the second LDS buffer.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace piperag {

typedef float acc16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

struct Bf16x3Tile {
    static constexpr int kRowsA = 256, kRowsB = 128, kTileK = 16;
    static constexpr int kPartA = 2 * kRowsA * 16, kPartB = 2 * kRowsB * 16;          // bytes of one hi or lo part per step
    static constexpr size_t kLdsBytes = 2 * (2 * (size_t)kPartA + 2 * (size_t)kPartB);  // double-buffered

    // Splits 8 floats into their bf16 hi and lo parts.
    __device__ static __forceinline__ void split8(const float4 &u, const float4 &v, bf16x8_t &hi, bf16x8_t &lo) {
        const float f[8] = {u.x, u.y, u.z, u.w, v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const __bf16 h = (__bf16)f[i];
            hi[i] = h;
            lo[i] = (__bf16)(f[i] - (float)h);
        }
    }

    // Rows a_row0.. of A (fp32, na rows, stride lda) against rows b_row0.. of B given as split bf16 matrices
    // b_hi / b_lo (nb rows, stride ldb elements).  Rows beyond na / nb and depth beyond d count as zero.
    // d % 8 == 0; A rows 16-byte aligned, B rows 16-byte aligned.  acc[bi][bj]: block rows 32*bi.., columns 32*bj..
    // of this wave's 128 x 64 patch; same register layout as the fp32 tile product.
    __device__ static void run(const float *__restrict__ A, int64_t na, int64_t lda, int64_t a_row0,
                               const uint16_t *__restrict__ b_hi, const uint16_t *__restrict__ b_lo, int64_t nb, int64_t ldb,
                               int64_t b_row0, int d, unsigned char *s_mem, acc16_t (&acc)[4][2]) {
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
        const int wr = wave >> 1, wc = wave & 1;
        unsigned char *sAh[2] = {s_mem, s_mem + kPartA * 2 + kPartB * 2};
        unsigned char *sAl[2] = {sAh[0] + kPartA, sAh[1] + kPartA};
        unsigned char *sBh[2] = {sAh[0] + 2 * kPartA, sAh[1] + 2 * kPartA};
        unsigned char *sBl[2] = {sBh[0] + kPartB, sBh[1] + kPartB};
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int bj = 0; bj < 2; ++bj)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[bi][bj][r] = 0.f;

        // per step: A has 256 rows x 2 depth halves = 512 items of 8 floats (2 per thread); B has 128 x 2 = 256
        // items of 8 bf16 per part (1 per thread)
        struct Regs { float4 a[2][2]; uint4 bh, bl; };
        const uint4 zero4 = {0u, 0u, 0u, 0u};
        auto fetch = [&](Regs &rg, int k0) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int item = tid + p * 256, row = item >> 1, half = item & 1;
                const int64_t gr = a_row0 + row;
                const int k = k0 + half * 8;
                const bool ok = gr < na && k < d;
                rg.a[p][0] = ok ? *reinterpret_cast<const float4 *>(A + gr * lda + k) : float4{0.f, 0.f, 0.f, 0.f};
                rg.a[p][1] = ok ? *reinterpret_cast<const float4 *>(A + gr * lda + k + 4) : float4{0.f, 0.f, 0.f, 0.f};
            }
            {
                const int row = tid >> 1, half = tid & 1;
                const int64_t gr = b_row0 + row;
                const int k = k0 + half * 8;
                const bool ok = gr < nb && k < d;
                rg.bh = ok ? *reinterpret_cast<const uint4 *>(b_hi + gr * ldb + k) : zero4;
                rg.bl = ok ? *reinterpret_cast<const uint4 *>(b_lo + gr * ldb + k) : zero4;
            }
        };
        auto stash = [&](const Regs &rg, int buf) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int item = tid + p * 256, row = item >> 1, half = item & 1;
                bf16x8_t hi, lo;
                split8(rg.a[p][0], rg.a[p][1], hi, lo);
                const int off = (half * kRowsA + row) * 16;
                *reinterpret_cast<bf16x8_t *>(sAh[buf] + off) = hi;
                *reinterpret_cast<bf16x8_t *>(sAl[buf] + off) = lo;
            }
            {
                const int row = tid >> 1, half = tid & 1;
                const int off = (half * kRowsB + row) * 16;
                *reinterpret_cast<uint4 *>(sBh[buf] + off) = rg.bh;
                *reinterpret_cast<uint4 *>(sBl[buf] + off) = rg.bl;
            }
        };
        const int half = lane >> 5, l32 = lane & 31;
        auto multiply = [&](int buf) {
            const int a_off = (half * kRowsA + wr * 128 + l32) * 16, b_off = (half * kRowsB + wc * 64 + l32) * 16;
            bf16x8_t ah[4], al[4], bh[2], bl[2];
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                ah[bi] = *reinterpret_cast<const bf16x8_t *>(sAh[buf] + a_off + bi * 32 * 16);
                al[bi] = *reinterpret_cast<const bf16x8_t *>(sAl[buf] + a_off + bi * 32 * 16);
            }
#pragma unroll
            for (int bj = 0; bj < 2; ++bj) {
                bh[bj] = *reinterpret_cast<const bf16x8_t *>(sBh[buf] + b_off + bj * 32 * 16);
                bl[bj] = *reinterpret_cast<const bf16x8_t *>(sBl[buf] + b_off + bj * 32 * 16);
            }
#pragma unroll
            for (int bi = 0; bi < 4; ++bi)
#pragma unroll
                for (int bj = 0; bj < 2; ++bj) {
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[bi], bh[bj], acc[bi][bj], 0, 0, 0);
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[bi], bl[bj], acc[bi][bj], 0, 0, 0);
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[bi], bh[bj], acc[bi][bj], 0, 0, 0);
                }
        };

        // Steps beyond the depth fetch zeros, so the pipeline needs no tail cases.
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
        return (wave >> 1) * 128 + bi * 32 + (r % 4) + 4 * (lane >> 5) + 8 * (r / 4);
    }
    __device__ static __forceinline__ int acc_col(int bj) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        return (wave & 1) * 64 + bj * 32 + (lane & 31);
    }
};

}  // namespace piperag
