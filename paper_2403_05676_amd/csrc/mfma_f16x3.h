// Split-fp16 MFMA tile product for gfx950: dot products <a_i, b_j> of fp32 rows at fp32 accuracy on the fp16
// matrix cores.  A matrix is scaled by a power of two s so that its largest magnitude lies in [2^14, 2^15), and
// every scaled value v is written as hi + lo with hi = fp16(v) and lo = fp16(v - hi): 22 significant bits
// together (|v - hi - lo| <= 2^-24 |v|, or 2^-25 in absolute terms where lo is subnormal, i.e. 2^-39 of the
// matrix's largest magnitude).  <a, b> ~ <a_hi, b_hi> + <a_hi, b_lo> + <a_lo, b_hi>, accumulated in fp32 by three
// v_mfma_f32_32x32x16_f16 per 32 x 32 block and 16 depth values; the dropped lo*lo term is 2^-24 relative per
// product, so each product is as accurate as an fp32 multiplication (3 * 2^-24 |a||b|), and the caller undoes the
// two scales exactly.  Used by the encoder's list assignment.
//
// Operands are split beforehand into the "chunk-major" layout below, so that what a workgroup needs for one
// depth step is a few contiguous kilobytes (every cache line fetched is used whole; with row-major operands a
// 16-value step touches a quarter of each line and the tile product is bound by L2 traffic, not by the matrix
// cores):
//   element (row, k) of a part (hi or lo) sits at ((k / 8) * rows_pad + row) * 8 + k % 8,
// rows_pad = rows rounded up to kRowPad, the number of 8-value chunks rounded up to even; padding holds zeros,
// so the tile product needs no bounds checks.
//
// Shape: workgroup = 8 waves as 2 x 4; the tile is 256 rows of A by 256 rows of B; a wave owns 128 x 64 = 4 x 2
// blocks.  (The product is bound by the traffic of its operands from beyond the 4 MiB L2 of an XCD, which is
// proportional to 1 / rows of A + 1 / rows of B per multiply-add: measured with a 256 x 128 tile, 52 % to 60 % of
// the L2 requests missed, 4.4 TB/s from the fabric, whatever the order of the tiles.)  The accumulator of a block
// keeps 16 rows of one column per lane, so A should be the operand over which the caller reduces (the centres,
// for an arg-min): the reduction then runs over a lane's own registers.
// Depth step 16 = two chunks; lanes 0-31 take the first chunk of the step and lanes 32-63 the second, for A and
// B alike, which is all a sum over the depth needs.  LDS holds [chunk of the step][row][8 fp16] per part, the
// same order as in memory.  Two steps are in flight: one in registers, one in the second LDS buffer.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace piperag {

typedef float acc16_t __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

struct F16x3Tile {
    static constexpr int kRowsA = 256, kRowsB = 256, kTileK = 16, kRowPad = 256, kThreads = 512;
    static constexpr int kPartA = 2 * kRowsA * 16, kPartB = 2 * kRowsB * 16;          // bytes of one hi or lo part per step
    static constexpr size_t kLdsBytes = 2 * (2 * (size_t)kPartA + 2 * (size_t)kPartB);  // double-buffered

    __host__ __device__ static int64_t rows_pad(int64_t rows) { return (rows + kRowPad - 1) / kRowPad * kRowPad; }
    __host__ __device__ static int chunks_pad(int d) { return ((d + 7) / 8 + 1) / 2 * 2; }
    // elements (uint16) of one part of a split matrix
    __host__ __device__ static size_t part_elems(int64_t rows, int d) { return (size_t)chunks_pad(d) * (size_t)rows_pad(rows) * 8; }

    // Rows a_row0 .. +255 of A against rows b_row0 .. +255 of B over the whole depth; both row ranges lie within
    // the padded matrices.  a_rp / b_rp: padded row counts; nchunks: chunks_pad(d).
    // acc[bi][bj]: block rows 32*bi.., columns 32*bj.. of this wave's 128 x 64 patch.
    __device__ static void run(const uint16_t *__restrict__ a_hi, const uint16_t *__restrict__ a_lo, int64_t a_rp, int64_t a_row0,
                               const uint16_t *__restrict__ b_hi, const uint16_t *__restrict__ b_lo, int64_t b_rp, int64_t b_row0,
                               int nchunks, unsigned char *s_mem, acc16_t (&acc)[4][2]) {
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
        const int wr = wave >> 2, wc = wave & 3;
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

        // per step and part: A is 2 chunks x 256 rows = 512 pieces of 16 bytes, B likewise: one piece of each per
        // thread (chunk tid / 256, row tid % 256); LDS offset = piece * 16
        struct Regs { uint4 ah, al, bh, bl; };
        const uint4 zero4 = {0u, 0u, 0u, 0u};
        const int pc = tid >> 8, pr = tid & 255;
        const uint4 *pa_hi = reinterpret_cast<const uint4 *>(a_hi) + (int64_t)pc * a_rp + a_row0 + pr;
        const uint4 *pa_lo = reinterpret_cast<const uint4 *>(a_lo) + (int64_t)pc * a_rp + a_row0 + pr;
        const uint4 *pb_hi = reinterpret_cast<const uint4 *>(b_hi) + (int64_t)pc * b_rp + b_row0 + pr;
        const uint4 *pb_lo = reinterpret_cast<const uint4 *>(b_lo) + (int64_t)pc * b_rp + b_row0 + pr;
        auto fetch = [&](Regs &rg, int c0) {            // c0: first chunk of the step
            if (c0 < nchunks) {                         // uniform
                rg.ah = pa_hi[(int64_t)c0 * a_rp];
                rg.al = pa_lo[(int64_t)c0 * a_rp];
                rg.bh = pb_hi[(int64_t)c0 * b_rp];
                rg.bl = pb_lo[(int64_t)c0 * b_rp];
            } else {
                rg.ah = rg.al = rg.bh = rg.bl = zero4;
            }
        };
        auto stash = [&](const Regs &rg, int buf) {
            *reinterpret_cast<uint4 *>(sAh[buf] + tid * 16) = rg.ah;
            *reinterpret_cast<uint4 *>(sAl[buf] + tid * 16) = rg.al;
            *reinterpret_cast<uint4 *>(sBh[buf] + tid * 16) = rg.bh;
            *reinterpret_cast<uint4 *>(sBl[buf] + tid * 16) = rg.bl;
        };
        const int half = lane >> 5, l32 = lane & 31;
        auto multiply = [&](int buf) {
            const int a_off = (half * kRowsA + wr * 128 + l32) * 16, b_off = (half * kRowsB + wc * 64 + l32) * 16;
            f16x8_t ah[4], al[4], bh[2], bl[2];
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                ah[bi] = *reinterpret_cast<const f16x8_t *>(sAh[buf] + a_off + bi * 32 * 16);
                al[bi] = *reinterpret_cast<const f16x8_t *>(sAl[buf] + a_off + bi * 32 * 16);
            }
#pragma unroll
            for (int bj = 0; bj < 2; ++bj) {
                bh[bj] = *reinterpret_cast<const f16x8_t *>(sBh[buf] + b_off + bj * 32 * 16);
                bl[bj] = *reinterpret_cast<const f16x8_t *>(sBl[buf] + b_off + bj * 32 * 16);
            }
#pragma unroll
            for (int bi = 0; bi < 4; ++bi)
#pragma unroll
                for (int bj = 0; bj < 2; ++bj) {
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al[bi], bh[bj], acc[bi][bj], 0, 0, 0);
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[bi], bl[bj], acc[bi][bj], 0, 0, 0);
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[bi], bh[bj], acc[bi][bj], 0, 0, 0);
                }
        };

        // Steps beyond the depth fetch zeros, so the pipeline needs no tail cases.
        const int nsteps = nchunks / 2;
        Regs r0, r1;
        fetch(r0, 0);
        fetch(r1, 2);
        __syncthreads();                 // the previous user of the LDS buffers is done
        stash(r0, 0);
        __syncthreads();
        for (int s = 0; s < nsteps; s += 2) {
            fetch(r0, 2 * (s + 2));
            multiply(0);
            stash(r1, 1);
            __syncthreads();
            if (s + 1 < nsteps) {
                fetch(r1, 2 * (s + 3));
                multiply(1);
                stash(r0, 0);
                __syncthreads();
            }
        }
    }

    // Row of A and row of B (both within the workgroup tile) of accumulator register r of block (bi, bj) for this lane.
    __device__ static __forceinline__ int acc_row(int bi, int r) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        return (wave >> 2) * 128 + bi * 32 + (r % 4) + 4 * (lane >> 5) + 8 * (r / 4);
    }
    __device__ static __forceinline__ int acc_col(int bj) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        return (wave & 3) * 64 + bj * 32 + (lane & 31);
    }
};

}  // namespace piperag
