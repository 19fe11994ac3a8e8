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
// rows_pad = rows rounded up to kRowPad, the number of 8-value chunks rounded up to a multiple of 4; padding holds zeros,
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
// same order as in memory, so a step travels from memory to LDS as it is: by loads that write LDS directly
// (global_load_lds_dwordx4: a wave's 64 x 16 bytes land side by side at the LDS address in M0), without passing
// through registers - the 16 registers per thread that a staged copy needs are not there beside 128 accumulators,
// and a copy staged over one turn only left the loads too little time (a sixth of the kernel's cycles went to
// waiting for them).
// The steps of all the A tiles a workgroup walks form one stream with four LDS buffers: in turn t the matrix
// instructions of step t run on fragments already in registers, the fragments of step t + 1 are read from LDS,
// step t + 2 has been asked for a turn ago and must have landed by the end of the turn, and step t + 3 is asked
// for.  Nothing drains between two tiles.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace piperag {

typedef float acc16_t __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

struct F16x3Tile {
    static constexpr int kRowsA = 256, kRowsB = 256, kTileK = 16, kRowPad = 256, kThreads = 512;
    static constexpr int kPartA = 2 * kRowsA * 16, kPartB = 2 * kRowsB * 16;          // bytes of one hi or lo part per step
    static constexpr int kStepBytes = 2 * kPartA + 2 * kPartB;                       // one step of both operands, hi and lo
    static constexpr int kBuffers = 4;
    static constexpr size_t kLdsBytes = kBuffers * (size_t)kStepBytes;

    __host__ __device__ static int64_t rows_pad(int64_t rows) { return (rows + kRowPad - 1) / kRowPad * kRowPad; }
    __host__ __device__ static int chunks_pad(int d) { return ((d + 7) / 8 + 3) / 4 * 4; }
    // elements (uint16) of one part of a split matrix
    __host__ __device__ static size_t part_elems(int64_t rows, int d) { return (size_t)chunks_pad(d) * (size_t)rows_pad(rows) * 8; }

    // One wave's share of a part of a step, from memory straight into LDS: lane l's 16 bytes at gbase + voff go to LDS
    // byte address lds_addr + 16 l (lds_addr the same in all lanes).  The compiler does not see these loads: whoever
    // reads the LDS they write waits for them with wait_direct_loads() and a barrier.  (M0 is set and left: it is a
    // reserved register that compiled code for this target touches only for operations these kernels do not use -
    // the compiler's own direct loads, relative register moves, messages - and cannot be named as clobbered.)
    __device__ static __forceinline__ void load_to_lds(const void *gbase, uint32_t voff, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
    }
    // the same for one float per lane (lane l's value goes to lds_addr + 4 l)
    __device__ static __forceinline__ void load_to_lds_f32(const void *gbase, uint32_t voff, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                     :: "s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
    }
    // waits until at most `newest` of this wave's memory operations (in issue order) are outstanding
    template <int NEWEST>
    __device__ static __forceinline__ void wait_direct_loads() {
        static_assert(NEWEST >= 0 && NEWEST < 16, "the count must fit the instruction's field");
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NEWEST) : "memory");
    }
    __device__ static __forceinline__ uint32_t lds_address(const void *p) {
        return (uint32_t)reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) unsigned char *)p);
    }

    // `ntiles` tiles of A (rows a_row0 + 256 t .. +255) against rows b_row0 .. +255 of B, each over the whole depth;
    // all row ranges lie within the padded matrices.  a_rp / b_rp: padded row counts; nchunks: chunks_pad(d).
    // hook(t, s) is called by every thread before step s of tile t is multiplied, before the turn's direct loads are
    // issued (for work the caller wants spread over the stream; a direct load of its own issued there has landed
    // after the barrier that ends the turn); tile_done(t, acc) when tile t is complete, with acc[bi][bj] = block rows
    // 32*bi.., columns 32*bj.. of this wave's 128 x 64 patch.  Between two calls of either there is at least one
    // workgroup barrier.  s_mem: kLdsBytes, free for other use after a barrier behind the call.
    template <class Hook, class TileDone>
    __device__ static void run_tiles(const uint16_t *__restrict__ a_hi, const uint16_t *__restrict__ a_lo, int64_t a_rp,
                                     int64_t a_row0, int ntiles, const uint16_t *__restrict__ b_hi,
                                     const uint16_t *__restrict__ b_lo, int64_t b_rp, int64_t b_row0, int nchunks,
                                     unsigned char *s_mem, Hook hook, TileDone tile_done) {
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
        const int wr = wave >> 2, wc = wave & 3;
        const int nsteps = nchunks / 2;                          // even (chunks_pad), since the fragment registers alternate
        // per step and part: A is 2 chunks x 256 rows = 512 pieces of 16 bytes, B likewise: one piece of each per
        // thread (chunk tid / 256, row tid % 256), a wave's 64 pieces side by side; LDS offset within the part =
        // piece * 16.  Addresses: a base common to the workgroup (scalar registers) plus a 32-bit byte offset per thread.
        const int pc = tid >> 8, pr = tid & 255;
        const uint32_t lane_a = (uint32_t)((pc * a_rp + pr) * 16), lane_b = (uint32_t)((pc * b_rp + pr) * 16);
        const unsigned char *ga_hi = reinterpret_cast<const unsigned char *>(a_hi) + a_row0 * 16;
        const unsigned char *ga_lo = reinterpret_cast<const unsigned char *>(a_lo) + a_row0 * 16;
        const unsigned char *gb_hi = reinterpret_cast<const unsigned char *>(b_hi) + b_row0 * 16;
        const unsigned char *gb_lo = reinterpret_cast<const unsigned char *>(b_lo) + b_row0 * 16;
        const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_address(s_mem) + (uint32_t)wave * 1024u);
        // Every fetch is four loads (beyond the last tile it repeats that tile's steps, which nobody multiplies).
        int ft = 0, fs = 0;                                      // (tile, step) of the next fetch
        auto fetch = [&](int buf) __attribute__((always_inline)) {
            const int64_t ao = ((int64_t)(2 * fs) * a_rp + (int64_t)ft * kRowsA) * 16, bo = (int64_t)(2 * fs) * b_rp * 16;
            const uint32_t dst = lds_wave + (uint32_t)(buf * kStepBytes);
            load_to_lds(ga_hi + ao, lane_a, dst);
            load_to_lds(ga_lo + ao, lane_a, dst + kPartA);
            load_to_lds(gb_hi + bo, lane_b, dst + 2 * kPartA);
            load_to_lds(gb_lo + bo, lane_b, dst + 2 * kPartA + kPartB);
            if (++fs == nsteps) { fs = 0; ft = min(ft + 1, ntiles - 1); }
        };
        const int half = lane >> 5, l32 = lane & 31;
        const int a_off = (half * kRowsA + wr * 128 + l32) * 16, b_off = 2 * kPartA + (half * kRowsB + wc * 64 + l32) * 16;
        // Operands of a step in registers: the wave's four A blocks (hi, lo) once, its two B blocks twice over (this
        // step's and the next one's).  A turn first asks LDS for the next step's B blocks, then multiplies block row
        // after block row, refilling each A block from the next step's buffer as soon as its matrix instructions are
        // issued, so that the LDS reads are spread over the turn and served beside the matrix instructions (all at
        // the end of the turn, as the compiler orders them when left alone, the eight waves' 96 KiB are served while
        // the matrix cores wait).
        f16x8_t ah[4], al[4];
        struct BFrags { f16x8_t bh[2], bl[2]; };
        auto read_a = [&](int bi, int buf) __attribute__((always_inline)) {
            const unsigned char *base = s_mem + buf * kStepBytes + a_off + bi * 32 * 16;
            ah[bi] = *reinterpret_cast<const f16x8_t *>(base);
            al[bi] = *reinterpret_cast<const f16x8_t *>(base + kPartA);
        };
        auto read_b = [&](BFrags &f, int buf) __attribute__((always_inline)) {
            const unsigned char *base = s_mem + buf * kStepBytes;
#pragma unroll
            for (int bj = 0; bj < 2; ++bj) {
                f.bh[bj] = *reinterpret_cast<const f16x8_t *>(base + b_off + bj * 32 * 16);
                f.bl[bj] = *reinterpret_cast<const f16x8_t *>(base + kPartB + b_off + bj * 32 * 16);
            }
        };
        acc16_t acc[4][2];
        // multiplies the step held in (ah, al, cur) and reads the step in LDS buffer `nbuf` into (ah, al, nxt);
        // first: the tile's first step starts from zero
        auto turn = [&](const BFrags &cur, BFrags &nxt, int nbuf, bool first) __attribute__((always_inline)) {
            read_b(nxt, nbuf);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                const f16x8_t xh = ah[bi], xl = al[bi];
#pragma unroll
                for (int bj = 0; bj < 2; ++bj) {
                    acc16_t c = acc[bi][bj];
                    if (first) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) c[r] = 0.f;
                    }
                    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(xl, cur.bh[bj], c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(xh, cur.bl[bj], c, 0, 0, 0);
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xh, cur.bh[bj], c, 0, 0, 0);
                }
                read_a(bi, nbuf);
                __builtin_amdgcn_sched_barrier(0);
            }
        };

        // At the top of turn t (t = the stream's step number): the fragments of step t are in registers, LDS buffer
        // (t + 1) % 4 holds step t + 1, step t + 2 is on its way to buffer (t + 2) % 4, and buffer (t + 3) % 4, which
        // held step t - 1, is free: its last readers (turn t - 2) are two barriers back.
        BFrags f0, f1;
        __syncthreads();                 // the previous user of the LDS buffers is done
        fetch(0);
        fetch(1);
        fetch(2);
        wait_direct_loads<4>();          // steps 0 and 1 have landed
        __syncthreads();
        read_b(f0, 0);
#pragma unroll
        for (int bi = 0; bi < 4; ++bi) read_a(bi, 0);
        int nb = 1;                      // buffer of step t + 1
        for (int t = 0; t < ntiles; ++t) {
            for (int s = 0; s < nsteps; s += 2) {
                hook(t, s);
                fetch((nb + 2) & 3);
                if (s == 0) turn(f0, f1, nb, true); else turn(f0, f1, nb, false);
                wait_direct_loads<4>();  // all but this turn's four: step t + 2 has landed
                __syncthreads();
                nb = (nb + 1) & 3;
                hook(t, s + 1);
                fetch((nb + 2) & 3);
                turn(f1, f0, nb, false);
                wait_direct_loads<4>();
                __syncthreads();
                nb = (nb + 1) & 3;
            }
            tile_done(t, acc);
        }
        wait_direct_loads<0>();          // the last fetches (repeats nobody reads) must not land in LDS that is reused
        __syncthreads();
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
