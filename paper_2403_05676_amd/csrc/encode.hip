// Database construction on the GPU (Section 2, "Database construction"; Appendix "Detailed Evaluation
// Setup", Software: every vector is assigned to one of nlist inverted lists and quantised into M code
// bytes).  list(x) = argmin_j ||x - centre_j||^2, code[m] = argmin_j ||x_m - pq[m][j]||^2, both in the
// direct (difference) form in fp32, lowest index on equal values.
#include <stdlib.h>

#include "common.h"
#include "mfma_bf16x3.h"
#include "mfma_tile.h"

using namespace piperag;

namespace piperag {
int check_can_add(piperag_index *ix, int64_t n);
int append_ids(piperag_index *ix, int64_t n, const int64_t *ids_dev, hipStream_t st);
void rownorm(const float *a, int64_t n, int d, int64_t lda, float *out, hipStream_t st);
}  // namespace piperag

namespace {

constexpr int TM = 64, TN = 64, TK = 16, LDT = 68;   // tile of rows x centres x coordinates; padded LDS stride

// Nearest-centre assignment.  One workgroup = 64 rows of x against all centres, 64 at a time; each thread
// accumulates a 4x4 patch of squared differences from coordinate-major LDS tiles.
__global__ __launch_bounds__(256) void assign_kernel(const float *__restrict__ x, int64_t n, int d, int64_t ldx,
                                                     const float *__restrict__ cent, int nlist,
                                                     int32_t *__restrict__ out_idx, float *__restrict__ out_dist,
                                                     int vec4) {
    __shared__ __align__(16) float xs[TK * LDT];
    __shared__ __align__(16) float cs[TK * LDT];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * TM;
    const int lr = tid >> 2, lk = (tid & 3) * 4;          // this thread loads 4 coordinates of row lr of each tile

    float best_d[4];
    int best_j[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { best_d[i] = __builtin_inff(); best_j[i] = 0; }

    for (int j0 = 0; j0 < nlist; j0 += TN) {
        float acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) acc[i][jj] = 0.f;

        for (int k0 = 0; k0 < d; k0 += TK) {
            float xv[4] = {0.f, 0.f, 0.f, 0.f}, cv[4] = {0.f, 0.f, 0.f, 0.f};
            const int64_t xr = row0 + lr;
            const int cr = j0 + lr;
            const int kk = k0 + lk;
            if (vec4) {
                if (xr < n && kk < d) {
                    const float4 v = *reinterpret_cast<const float4 *>(x + xr * ldx + kk);
                    xv[0] = v.x; xv[1] = v.y; xv[2] = v.z; xv[3] = v.w;
                }
                if (cr < nlist && kk < d) {
                    const float4 v = *reinterpret_cast<const float4 *>(cent + (size_t)cr * d + kk);
                    cv[0] = v.x; cv[1] = v.y; cv[2] = v.z; cv[3] = v.w;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (xr < n && kk + i < d) xv[i] = x[xr * ldx + kk + i];
                    if (cr < nlist && kk + i < d) cv[i] = cent[(size_t)cr * d + kk + i];
                }
            }
            __syncthreads();                      // previous tile fully consumed
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xs[(lk + i) * LDT + lr] = xv[i];
                cs[(lk + i) * LDT + lr] = cv[i];
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < TK; ++k) {
                const float4 a = *reinterpret_cast<const float4 *>(&xs[k * LDT + ty * 4]);
                const float4 b = *reinterpret_cast<const float4 *>(&cs[k * LDT + tx * 4]);
                const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const float diff = av[i] - bv[jj];
                        acc[i][jj] += diff * diff;
                    }
            }
        }
        // argmin over this tile's 64 centres for each of the thread's 4 rows, then over the 16 threads of the row
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float bd = __builtin_inff();
            int bj = 0x7FFFFFFF;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int j = j0 + tx * 4 + jj;
                if (j < nlist && acc[i][jj] < bd) { bd = acc[i][jj]; bj = j; }
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                const float od = __shfl_xor(bd, off, 64);
                const int oj = __shfl_xor(bj, off, 64);
                if (od < bd || (od == bd && oj < bj)) { bd = od; bj = oj; }
            }
            if (bd < best_d[i]) { best_d[i] = bd; best_j[i] = bj; }
        }
    }
    if (tx == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t r = row0 + ty * 4 + i;
            if (r < n) {
                out_idx[r] = best_j[i];
                if (out_dist) out_dist[r] = best_d[i];
            }
        }
    }
}

// PQ encoding.  One workgroup = 256 rows; for each sub-quantiser the 256 centres and the rows' slices are
// staged in LDS and every thread scans the centres for its row.  Codes are collected in LDS and written
// out as one contiguous run.
__global__ __launch_bounds__(256) void pq_encode_kernel(const float *__restrict__ x, int64_t n, int d,
                                                        const float *__restrict__ pq, int M, int dsub,
                                                        const int32_t *__restrict__ lists, const float *__restrict__ cent,
                                                        uint8_t *__restrict__ out_codes) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *cs = reinterpret_cast<float *>(smem);              // [256][dsub]
    float *xs = cs + kKsub * dsub;                             // [dsub][256]
    uint8_t *code_s = reinterpret_cast<uint8_t *>(xs + dsub * 256);   // [256][M]
    const int tid = threadIdx.x;
    const int64_t row0 = (int64_t)blockIdx.x * 256;
    const int rows = (int)min<int64_t>(256, n - row0);
    for (int m = 0; m < M; ++m) {
        __syncthreads();
        for (int i = tid; i < kKsub * dsub; i += 256) cs[i] = pq[(size_t)m * kKsub * dsub + i];
        for (int e = tid; e < 256 * dsub; e += 256) {
            const int r = e / dsub, t = e - r * dsub;
            float v = r < rows ? x[(row0 + r) * d + m * dsub + t] : 0.f;
            if (lists && r < rows) v -= cent[(size_t)lists[row0 + r] * d + m * dsub + t];   // residual to the list's centre
            xs[t * 256 + r] = v;
        }
        __syncthreads();
        float best = __builtin_inff();
        int bj = 0;
        for (int j = 0; j < kKsub; ++j) {
            float acc = 0.f;
            for (int t = 0; t < dsub; ++t) {
                const float diff = xs[t * 256 + tid] - cs[j * dsub + t];
                acc += diff * diff;
            }
            if (acc < best) { best = acc; bj = j; }
        }
        code_s[tid * M + m] = (uint8_t)bj;
    }
    __syncthreads();
    uint8_t *dst = out_codes + (size_t)row0 * M;
    for (int i = tid; i < rows * M; i += 256) dst[i] = code_s[i];
}

// PQ encoding on the matrix cores: code[x][m] = argmin_j |x_m - P[m][j]|^2 = argmin_j (|P[m][j]|^2 - 2 <x_m, P[m][j]>).
// One workgroup = 128 vectors, a wave = 32 of them; for each sub-quantiser the 256 centres are the row operand of
// v_mfma_f32_32x32x2f32 and the wave's 32 vectors the column operand: 8 blocks of 32 centres x 32 vectors.  The
// centres come from the depth-major copy pqE[m][t][j], whose row t = dsub holds the squared norms: with the
// vectors entered as (-2 x_m, 1) the product is the quantity to minimise itself.  A lane then holds 128 centres
// of one vector in its own registers and keeps the running best in ascending centre order (strict "<": lower
// index on equal values); the two lanes that share a vector are combined with one shuffle.  Codes are
// collected in LDS and written out as one contiguous run.  T = pqe_rows(dsub) depth rows (even), dsub <= 32.
__global__ __launch_bounds__(256) void pq_encode_mfma_kernel(const float *__restrict__ x, int64_t n, int d,
                                                             const float *__restrict__ pqE, int M, int dsub, int T,
                                                             const int32_t *__restrict__ lists, const float *__restrict__ cent,
                                                             uint8_t *__restrict__ out_codes) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *sA = reinterpret_cast<float *>(smem);                  // [T][256]
    uint8_t *code_s = reinterpret_cast<uint8_t *>(sA + T * kKsub);   // [128][M]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int64_t row0 = (int64_t)blockIdx.x * 128;
    const int rows = (int)min<int64_t>(128, n - row0);
    const int64_t myrow = row0 + wave * 32 + l32;
    const float *xr = x + myrow * d;
    const bool live = myrow < n;
    // residual indexes quantise x - c_l (one fp32 subtraction), l the vector's list
    const float *cr = lists && live ? cent + (size_t)lists[myrow] * d : nullptr;
    for (int m = 0; m < M; ++m) {
        __syncthreads();                                          // the previous sub-quantiser's centres are no longer read
        const float4 *src = reinterpret_cast<const float4 *>(pqE + (size_t)m * T * kKsub);
        for (int e = tid; e < T * kKsub / 4; e += 256) reinterpret_cast<float4 *>(sA)[e] = src[e];
        __syncthreads();
        mfma_acc_t acc[8];
#pragma unroll
        for (int bi = 0; bi < 8; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[bi][r] = 0.f;
        for (int p = 0; p < T / 2; ++p) {
            const int t = 2 * p + half;                           // lanes 0-31: depth 2p, lanes 32-63: depth 2p + 1
            float bv = t == dsub ? 1.f : 0.f;                     // the row of norms; padding rows are zero on both sides
            if (t < dsub) {
                float v = live ? xr[m * dsub + t] : 0.f;
                if (cr) v -= cr[m * dsub + t];
                bv = -2.f * v;
            }
            const float *a = sA + t * kKsub + l32;
#pragma unroll
            for (int bi = 0; bi < 8; ++bi) acc[bi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bi * 32], bv, acc[bi], 0, 0, 0);
        }
        float best = __builtin_inff();
        int bj = 0;
#pragma unroll
        for (int bi = 0; bi < 8; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float v = acc[bi][r];
                if (v < best) { best = v; bj = bi * 32 + (r % 4) + 4 * half + 8 * (r / 4); }   // ascending in bi, r
            }
        const float ov = __shfl_xor(best, 32, 64);
        const int oj = __shfl_xor(bj, 32, 64);
        if (ov < best || (ov == best && oj < bj)) bj = oj;
        if (half == 0) code_s[(wave * 32 + l32) * M + m] = (uint8_t)bj;
    }
    __syncthreads();
    uint8_t *dst = out_codes + (size_t)row0 * M;
    for (int i = tid; i < rows * M; i += 256) dst[i] = code_s[i];
}

// Squared norms of the rows of a matrix: one wavefront per row.
__global__ __launch_bounds__(256) void rownorm_kernel(const float *__restrict__ a, int64_t n, int d, int64_t lda,
                                                      float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    float acc = 0.f;
    for (int t = lane; t < d; t += 64) { const float v = a[row * lda + t]; acc += v * v; }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) out[row] = acc;
}

// Nearest-centre assignment on the matrix cores: |x - c|^2 = |x|^2 + |c|^2 - 2 <x, c>, and |x|^2 does not
// change the argmin, so a workgroup takes 128 rows of x, walks over the centres 128 at a time with the fp32
// MFMA tile product and keeps, per row, the smallest |c|^2 - 2 <x, c> and its centre (lower index on equal
// values).  Requires d % 4 == 0 and 16-byte aligned rows.
using AssignTile = MfmaTile<2, 2, 2, 2>;

__global__ __launch_bounds__(256) void assign_mfma_kernel(const float *__restrict__ x, int64_t n, int d, int64_t ldx,
                                                          const float *__restrict__ cent, const float *__restrict__ cnorm,
                                                          int K, int32_t *__restrict__ out_idx, float *__restrict__ out_dist) {
    __shared__ __align__(16) float s_mem[AssignTile::kLdsFloats];
    const int tid = threadIdx.x, lane = tid & 63, wc = (tid >> 6) % 2;
    const int64_t row0 = (int64_t)blockIdx.x * AssignTile::kRowsA;
    float best_v[2][16];
    int best_j[2][16];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int r = 0; r < 16; ++r) { best_v[bi][r] = __builtin_inff(); best_j[bi][r] = 0; }

    for (int j0 = 0; j0 < K; j0 += AssignTile::kRowsB) {
        mfma_acc_t acc[2][2];
        AssignTile::run(x, n, ldx, row0, cent, K, d, j0, d, s_mem, acc);
        const int c0 = j0 + AssignTile::acc_col(0), c1 = j0 + AssignTile::acc_col(1);
        const float n0 = c0 < K ? cnorm[c0] : __builtin_inff(), n1 = c1 < K ? cnorm[c1] : __builtin_inff();
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float v0 = n0 - 2.f * acc[bi][0][r], v1 = n1 - 2.f * acc[bi][1][r];
                float v = v0;
                int c = c0;
                if (v1 < v0) { v = v1; c = c1; }
#pragma unroll
                for (int off = 1; off < 32; off <<= 1) {      // over the 32 lanes (columns) of this half-wave
                    const float ov = __shfl_xor(v, off, 64);
                    const int oc = __shfl_xor(c, off, 64);
                    if (ov < v || (ov == v && oc < c)) { v = ov; c = oc; }
                }
                if (v < best_v[bi][r]) { best_v[bi][r] = v; best_j[bi][r] = c; }
            }
    }
    // the two waves that share these rows (column halves wc = 0, 1) meet in LDS
    __syncthreads();
    float *s_v = s_mem;
    int *s_j = reinterpret_cast<int *>(s_mem + 2 * AssignTile::kRowsA);
    if ((lane & 31) == 0) {
#pragma unroll
        for (int bi = 0; bi < 2; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = AssignTile::acc_row(bi, r);
                s_v[row * 2 + wc] = best_v[bi][r];
                s_j[row * 2 + wc] = best_j[bi][r];
            }
    }
    __syncthreads();
    if (tid < AssignTile::kRowsA && row0 + tid < n) {
        float v = s_v[tid * 2];
        int j = s_j[tid * 2];
        if (s_v[tid * 2 + 1] < v) { v = s_v[tid * 2 + 1]; j = s_j[tid * 2 + 1]; }   // equal values: the lower half holds the lower index
        out_idx[row0 + tid] = j;
        if (out_dist) {
            float xn = 0.f;
            const float *xr = x + (row0 + tid) * ldx;
            for (int t = 0; t < d; ++t) xn += xr[t] * xr[t];
            out_dist[row0 + tid] = fmaxf(0.f, v + xn);
        }
    }
}

// rows of x (stride ldx floats) against K centres; 16-byte loads only when every row start is 16-byte aligned
// bf16 hi / lo parts of an fp32 matrix (n rows of d values, stride ld) in the chunk-major layout of
// mfma_bf16x3.h; one thread per (row, chunk of 8 values), padding rows and chunks are written as zeros.
__global__ void split_bf16_kernel(const float *__restrict__ src, int64_t n, int d, int64_t ld, int64_t rows_pad, int nchunks,
                                  uint16_t *__restrict__ hi, uint16_t *__restrict__ lo) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows_pad * nchunks) return;
    const int64_t row = e / nchunks;
    const int c = (int)(e % nchunks);
    uint16_t h[8], l[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int k = c * 8 + t;
        const float v = (row < n && k < d) ? src[row * ld + k] : 0.f;
        const __bf16 vh = (__bf16)v;
        const __bf16 vl = (__bf16)(v - (float)vh);
        h[t] = __builtin_bit_cast(uint16_t, vh);
        l[t] = __builtin_bit_cast(uint16_t, vl);
    }
    const size_t o = ((size_t)c * rows_pad + row) * 8;
#pragma unroll
    for (int t = 0; t < 8; ++t) { hi[o + t] = h[t]; lo[o + t] = l[t]; }
}

// Nearest-centre assignment with the split-bf16 tile product: 128 vectors per workgroup against the centres 256
// at a time.  The centres are the tile's A operand, so a lane holds, for each of its two vector columns, 64
// centres of the tile in its own registers: the running best (|c|^2 - 2 <x, c>, centre) of a column is kept
// per lane and compared register by register in ascending centre order (a strict "<" keeps the lower index on
// equal values); lanes and waves that share a column are combined once at the end.
__global__ __launch_bounds__(256, 2) void assign_bf16x3_kernel(const float *__restrict__ x, int64_t n, int d, int64_t ldx,
                                                            const uint16_t *__restrict__ xhi, const uint16_t *__restrict__ xlo,
                                                            int64_t x_rp, const uint16_t *__restrict__ chi,
                                                            const uint16_t *__restrict__ clo, int64_t c_rp,
                                                            const float *__restrict__ cnorm, int K,
                                                            int32_t *__restrict__ out_idx, float *__restrict__ out_dist) {
    extern __shared__ __align__(16) unsigned char bsmem[];
    float *s_cn = reinterpret_cast<float *>(bsmem + Bf16x3Tile::kLdsBytes);        // [2][256] centre norms of a tile (+inf: no centre)
    float *s_bv = s_cn + 2 * Bf16x3Tile::kRowsA;                                    // [128 vectors][2 wave rows]
    int *s_bj = reinterpret_cast<int *>(s_bv + 2 * Bf16x3Tile::kRowsB);
    const int tid = threadIdx.x, lane = tid & 63, wr = tid >> 7;
    const int64_t row0 = (int64_t)blockIdx.x * Bf16x3Tile::kRowsB;
    const int nchunks = Bf16x3Tile::chunks_pad(d);
    float bv[2] = {__builtin_inff(), __builtin_inff()};
    int bc[2] = {0, 0};
    int tile = 0;
    for (int j0 = 0; j0 < K; j0 += Bf16x3Tile::kRowsA, ++tile) {
        float *cn = s_cn + (tile & 1) * Bf16x3Tile::kRowsA;    // read after the barriers inside run(); rewritten two tiles later
        cn[tid] = j0 + tid < K ? cnorm[j0 + tid] : __builtin_inff();
        acc16_t acc[4][2];
        Bf16x3Tile::run(chi, clo, c_rp, j0, xhi, xlo, x_rp, row0, nchunks, bsmem, acc);
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int r0 = Bf16x3Tile::acc_row(bi, 4 * g);                     // rows r0 .. r0+3 are registers 4g .. 4g+3
                const float4 nn = *reinterpret_cast<const float4 *>(cn + r0);
                const float nv[4] = {nn.x, nn.y, nn.z, nn.w};
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int bj = 0; bj < 2; ++bj) {
                        const float v = nv[t] - 2.f * acc[bi][bj][4 * g + t];
                        if (v < bv[bj]) { bv[bj] = v; bc[bj] = j0 + r0 + t; }
                    }
            }
    }
    // lanes l and l + 32 hold the same columns (different centres), then the two wave rows
#pragma unroll
    for (int bj = 0; bj < 2; ++bj) {
        const float ov = __shfl_xor(bv[bj], 32, 64);
        const int oc = __shfl_xor(bc[bj], 32, 64);
        if (ov < bv[bj] || (ov == bv[bj] && oc < bc[bj])) { bv[bj] = ov; bc[bj] = oc; }
        if (lane < 32) {
            const int col = Bf16x3Tile::acc_col(bj);
            s_bv[col * 2 + wr] = bv[bj];
            s_bj[col * 2 + wr] = bc[bj];
        }
    }
    __syncthreads();
    if (tid < Bf16x3Tile::kRowsB && row0 + tid < n) {
        float v = s_bv[tid * 2];
        int j = s_bj[tid * 2];
        const float v1 = s_bv[tid * 2 + 1];
        const int j1 = s_bj[tid * 2 + 1];
        if (v1 < v || (v1 == v && j1 < j)) { v = v1; j = j1; }
        out_idx[row0 + tid] = j;
        if (out_dist) {
            float xn = 0.f;
            const float *xr = x + (row0 + tid) * ldx;
            for (int t = 0; t < d; ++t) xn += xr[t] * xr[t];
            out_dist[row0 + tid] = fmaxf(0.f, v + xn);
        }
    }
}

// cnorm: squared norms of the centres (f32 [K]) or NULL.  The matrix-core path is taken when the shape pays for
// it and allows 16-byte loads; otherwise the direct-form VALU kernel runs.
// chi / clo: bf16 split of the centres (u16 [K*d] each) or NULL.  The matrix-core paths are taken when the shape
// pays for them and allows 16-byte loads: split-bf16 first, fp32 MFMA second; otherwise the direct-form VALU
// kernel runs.
void launch_split(const float *src, int64_t n, int d, int64_t ld, uint16_t *hi, uint16_t *lo, hipStream_t st);

int launch_assign(const float *x, int64_t n, int d, int64_t ldx, const float *cent, const float *cnorm, const uint16_t *chi,
                  const uint16_t *clo, int K, int32_t *out_idx, float *out_dist, hipStream_t st) {
    const int vec4 = (d % 4 == 0) && (ldx % 4 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(cent) % 16 == 0);
    const bool mfma = vec4 && cnorm != nullptr && K >= 128 && d >= 64;
    const bool bf16 = cnorm != nullptr && K >= 128 && d >= 64 && chi != nullptr && clo != nullptr;
    constexpr size_t kBfLds = Bf16x3Tile::kLdsBytes + sizeof(float) * (2 * Bf16x3Tile::kRowsA + 4 * Bf16x3Tile::kRowsB);
    if (bf16) {
        static bool configured = false;
        if (!configured) {
            PR_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&assign_bf16x3_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBfLds));
            configured = true;
        }
        // the vectors are split slice by slice into a scratch area that lives in stream order
        const int64_t slice = std::max<int64_t>(Bf16x3Tile::kRowPad, ((int64_t)1 << 28) / ((int64_t)Bf16x3Tile::chunks_pad(d) * 8) /
                                                                         Bf16x3Tile::kRowPad * Bf16x3Tile::kRowPad);
        const int64_t cap_rows = std::min(slice, Bf16x3Tile::rows_pad(n));
        const size_t part = Bf16x3Tile::part_elems(cap_rows, d);
        uint16_t *xs = nullptr;
        PR_CHECK_HIP(hipMallocAsync(reinterpret_cast<void **>(&xs), 2 * part * sizeof(uint16_t), st));
        const int nchunks = Bf16x3Tile::chunks_pad(d);
        const int64_t c_rp = Bf16x3Tile::rows_pad(K);
        for (int64_t a = 0; a < n; a += slice) {
            const int64_t cnt = std::min(slice, n - a), rp = Bf16x3Tile::rows_pad(cnt);
            launch_split(x + a * ldx, cnt, d, ldx, xs, xs + part, st);
            hipLaunchKernelGGL(assign_bf16x3_kernel, dim3((unsigned)((cnt + Bf16x3Tile::kRowsB - 1) / Bf16x3Tile::kRowsB)), dim3(256),
                               kBfLds, st, x + a * ldx, cnt, d, ldx, xs, xs + part, rp, chi, clo, c_rp, cnorm, K, out_idx + a,
                               out_dist ? out_dist + a : nullptr);
            (void)nchunks;
        }
        PR_CHECK_HIP(hipFreeAsync(xs, st));
        return PIPERAG_OK;
    }
    constexpr int64_t kSlice = 1 << 22;              // rows per launch
    for (int64_t a = 0; a < n; a += kSlice) {
        const int64_t cnt = n - a < kSlice ? n - a : kSlice;
        if (mfma)
            hipLaunchKernelGGL(assign_mfma_kernel, dim3((unsigned)((cnt + AssignTile::kRowsA - 1) / AssignTile::kRowsA)), dim3(256), 0,
                               st, x + a * ldx, cnt, d, ldx, cent, cnorm, K, out_idx + a, out_dist ? out_dist + a : nullptr);
        else
            hipLaunchKernelGGL(assign_kernel, dim3((unsigned)((cnt + TM - 1) / TM)), dim3(256), 0, st, x + a * ldx, cnt, d, ldx, cent,
                               K, out_idx + a, out_dist ? out_dist + a : nullptr, vec4);
    }
    return PIPERAG_OK;
}

// Splits n rows of d values (stride ld) into the chunk-major bf16 hi / lo parts; each part holds
// Bf16x3Tile::part_elems(n, d) elements.
void launch_split(const float *src, int64_t n, int d, int64_t ld, uint16_t *hi, uint16_t *lo, hipStream_t st) {
    const int64_t rp = Bf16x3Tile::rows_pad(n);
    const int nchunks = Bf16x3Tile::chunks_pad(d);
    hipLaunchKernelGGL(split_bf16_kernel, dim3((unsigned)((rp * nchunks + 255) / 256)), dim3(256), 0, st, src, n, d, ld, rp, nchunks, hi,
                       lo);
}

void launch_rownorm(const float *a, int64_t n, int d, int64_t lda, float *out, hipStream_t st) {
    hipLaunchKernelGGL(rownorm_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, a, n, d, lda, out);
}

// ---- k-means training ------------------------------------------------------------------------
constexpr float kFixScale = 16777216.f;             // 2^24: coordinate sums are kept in 40.24 fixed point

__global__ void gather_rows_kernel(const float *__restrict__ x, int64_t ldx, int d, const int64_t *__restrict__ rows,
                                   float *__restrict__ out) {
    const int j = blockIdx.x;
    for (int t = threadIdx.x; t < d; t += blockDim.x) out[(size_t)j * d + t] = x[rows[j] * ldx + t];
}

__global__ void kmeans_accum_kernel(const float *__restrict__ x, int64_t ldx, int d, const int32_t *__restrict__ assign,
                                    long long *__restrict__ sum, int *__restrict__ count) {
    const int64_t row = blockIdx.x;
    const int a = assign[row];
    for (int t = threadIdx.x; t < d; t += blockDim.x)
        atomicAdd(reinterpret_cast<unsigned long long *>(&sum[(size_t)a * d + t]),
                  (unsigned long long)__float2ll_rn(x[row * ldx + t] * kFixScale));
    if (threadIdx.x == 0) atomicAdd(&count[a], 1);
}

__global__ void kmeans_update_kernel(const long long *__restrict__ sum, const int *__restrict__ count, int K, int d,
                                     float *__restrict__ cent) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)K * d) return;
    const int c = count[e / d];
    if (c > 0) cent[e] = (float)((double)sum[e] * (1.0 / 16777216.0) / (double)c);
}

__global__ void zero_kernel(unsigned long long *__restrict__ p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

}  // namespace

namespace piperag {
void rownorm(const float *a, int64_t n, int d, int64_t lda, float *out, hipStream_t st) { launch_rownorm(a, n, d, lda, out, st); }
void split_bf16(const float *src, int64_t n, int d, uint16_t *hi, uint16_t *lo, hipStream_t st) { launch_split(src, n, d, d, hi, lo, st); }
size_t split_bf16_elems(int64_t n, int d) { return Bf16x3Tile::part_elems(n, d); }
}  // namespace piperag

namespace {

// lists: buffer of n list numbers; assign = true: they are computed here (lists may be NULL for a raw index
// when only codes are wanted), assign = false: they are given (the codes of a residual index need them).
int encode_impl(const piperag_index *ix, const float *x, int64_t n, int32_t *lists, bool assign, uint8_t *out_codes,
                hipStream_t st) {
    const piperag_params &p = ix->p;
    PR_REQUIRE(ix->dsub <= 32, PIPERAG_ERR_ARG, "d/M = %d: the encoder supports at most 32 coordinates per sub-quantiser", ix->dsub);
    int32_t *tmp_lists = nullptr;
    if (p.residual && out_codes && !lists) {                 // codes of residuals need the lists even if the caller does not
        PR_CHECK_HIP(hipMallocAsync(reinterpret_cast<void **>(&tmp_lists), sizeof(int32_t) * (size_t)n, st));
        lists = tmp_lists;
        assign = true;
    }
    if (assign && lists) {
        const int rc = launch_assign(x, n, p.d, p.d, ix->centroids, ix->cnorm, ix->cent_hi, ix->cent_lo, p.nlist, lists, nullptr, st);
        if (rc != PIPERAG_OK) { if (tmp_lists) (void)hipFreeAsync(tmp_lists, st); return rc; }
    }
    const int32_t *res_lists = p.residual ? lists : nullptr;
    constexpr int64_t kSlice = 1 << 22;              // rows per launch
    for (int64_t a = 0; a < n; a += kSlice) {
        const int64_t cnt = n - a < kSlice ? n - a : kSlice;
        if (out_codes) {
            if (ix->dsub >= 4) {                                 // matrix cores
                const int T = pqe_rows(ix->dsub);
                const size_t lds = sizeof(float) * (size_t)T * kKsub + (size_t)128 * p.M;
                static size_t configured = 0;
                if (lds > configured) {
                    PR_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&pq_encode_mfma_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
                    configured = lds;
                }
                hipLaunchKernelGGL(pq_encode_mfma_kernel, dim3((unsigned)((cnt + 127) / 128)), dim3(256), lds, st, x + a * p.d, cnt,
                                   p.d, ix->pqE, p.M, ix->dsub, T, res_lists ? res_lists + a : nullptr, ix->centroids,
                                   out_codes + (size_t)a * p.M);
            } else {
                const size_t lds = sizeof(float) * 2 * kKsub * ix->dsub + (size_t)256 * p.M;
                static size_t configured = 0;
                if (lds > configured) {
                    PR_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&pq_encode_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
                    configured = lds;
                }
                hipLaunchKernelGGL(pq_encode_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), lds, st, x + a * p.d, cnt, p.d,
                                   ix->pq, p.M, ix->dsub, res_lists ? res_lists + a : nullptr, ix->centroids,
                                   out_codes + (size_t)a * p.M);
            }
        }
    }
    if (tmp_lists) PR_CHECK_HIP(hipFreeAsync(tmp_lists, st));
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

}  // namespace

extern "C" {

int piperag_ivf_encode(const piperag_index *index, const float *x_dev, int64_t n, int32_t *out_lists_dev,
                       uint8_t *out_codes_dev, void *stream) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(n >= 0, PIPERAG_ERR_ARG, "n = %lld is negative", (long long)n);
    if (n == 0) return PIPERAG_OK;
    PR_REQUIRE(x_dev != nullptr, PIPERAG_ERR_ARG, "x_dev is NULL");
    PR_CHECK_HIP(hipSetDevice(index->device));
    return encode_impl(index, x_dev, n, out_lists_dev, true, out_codes_dev, (hipStream_t)stream);
}

int piperag_kmeans(const float *x_dev, int64_t n, int32_t d, int64_t ldx, int32_t K, int32_t iters,
                   const int64_t *init_rows_host, float *centroids_out_dev, double *inertia_out_host, void *stream) {
    PR_REQUIRE(x_dev && init_rows_host && centroids_out_dev, PIPERAG_ERR_ARG, "NULL argument");
    PR_REQUIRE(n >= 1 && n <= (1ll << 31) - 1 && d >= 1 && d <= 8192 && ldx >= d, PIPERAG_ERR_ARG, "n / d / ldx out of range");
    PR_REQUIRE(K >= 1 && K <= n && K <= (1 << 20) && iters >= 0, PIPERAG_ERR_ARG, "K = %d / iters = %d out of range", K, iters);
    for (int j = 0; j < K; ++j)
        PR_REQUIRE(init_rows_host[j] >= 0 && init_rows_host[j] < n, PIPERAG_ERR_ARG, "init row %d out of range", j);
    hipStream_t st = (hipStream_t)stream;
    int64_t *rows = nullptr;
    int32_t *assign = nullptr;
    float *adist = nullptr;
    long long *sum = nullptr;
    int *count = nullptr;
    float *cnorm = nullptr;
    uint16_t *chi = nullptr, *clo = nullptr;
    float *hdist = inertia_out_host ? (float *)malloc(sizeof(float) * (size_t)n) : nullptr;
    auto done = [&](int code) {
        (void)hipFree(rows); (void)hipFree(assign); (void)hipFree(adist); (void)hipFree(sum); (void)hipFree(count); (void)hipFree(cnorm); (void)hipFree(chi); (void)hipFree(clo);
        free(hdist);
        return code;
    };
    if (inertia_out_host && !hdist) { set_error("host allocation failed"); return done(PIPERAG_ERR_OOM); }
    if (hipMalloc((void **)&rows, sizeof(int64_t) * K) != hipSuccess || hipMalloc((void **)&assign, sizeof(int32_t) * n) != hipSuccess ||
        hipMalloc((void **)&adist, sizeof(float) * n) != hipSuccess ||
        hipMalloc((void **)&sum, sizeof(long long) * (size_t)K * d) != hipSuccess ||
        hipMalloc((void **)&count, sizeof(int) * (K + 1)) != hipSuccess || hipMalloc((void **)&cnorm, sizeof(float) * K) != hipSuccess) {
        set_error("out of device memory in piperag_kmeans");
        return done(PIPERAG_ERR_OOM);
    }
    const bool use_split = K >= 128 && d >= 64;
    if (use_split && (hipMalloc((void **)&chi, sizeof(uint16_t) * Bf16x3Tile::part_elems(K, d)) != hipSuccess ||
                      hipMalloc((void **)&clo, sizeof(uint16_t) * Bf16x3Tile::part_elems(K, d)) != hipSuccess)) {
        set_error("out of device memory in piperag_kmeans");
        return done(PIPERAG_ERR_OOM);
    }
    hipError_t e = hipMemcpyAsync(rows, init_rows_host, sizeof(int64_t) * K, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { set_error("upload failed: %s", hipGetErrorString(e)); return done(PIPERAG_ERR_HIP); }
    hipLaunchKernelGGL(gather_rows_kernel, dim3(K), dim3(256), 0, st, x_dev, ldx, d, rows, centroids_out_dev);
    const int64_t nsum = (int64_t)K * d;
    for (int it = 0; it < iters; ++it) {
        launch_rownorm(centroids_out_dev, K, d, d, cnorm, st);
        if (use_split) launch_split(centroids_out_dev, K, d, d, chi, clo, st);
        const int rca = launch_assign(x_dev, n, d, ldx, centroids_out_dev, cnorm, chi, clo, K, assign, adist, st);
        if (rca != PIPERAG_OK) return done(rca);
        hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((nsum + 255) / 256)), dim3(256), 0, st, (unsigned long long *)sum, nsum);
        hipLaunchKernelGGL(zero_kernel, dim3((K / 2 + 256) / 256), dim3(256), 0, st, (unsigned long long *)count, (int64_t)(K + 1) / 2);
        hipLaunchKernelGGL(kmeans_accum_kernel, dim3((unsigned)n), dim3(d >= 256 ? 256 : 64), 0, st, x_dev, ldx, d, assign, sum, count);
        hipLaunchKernelGGL(kmeans_update_kernel, dim3((unsigned)((nsum + 255) / 256)), dim3(256), 0, st, sum, count, K, d,
                           centroids_out_dev);
        if (inertia_out_host) {
            e = hipMemcpyAsync(hdist, adist, sizeof(float) * n, hipMemcpyDeviceToHost, st);
            if (e == hipSuccess) e = hipStreamSynchronize(st);
            if (e != hipSuccess) { set_error("read-back failed: %s", hipGetErrorString(e)); return done(PIPERAG_ERR_HIP); }
            double tot = 0.0;
            for (int64_t i = 0; i < n; ++i) tot += (double)hdist[i];
            inertia_out_host[it] = tot;
        }
    }
    e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { set_error("k-means failed: %s", hipGetErrorString(e)); return done(PIPERAG_ERR_HIP); }
    return done(PIPERAG_OK);
}

int piperag_ivf_add(piperag_index *index, const float *x_dev, int64_t n, const int64_t *ids_dev, void *stream) {
    int rc = check_can_add(index, n);
    if (rc != PIPERAG_OK || n == 0) return rc;
    PR_REQUIRE(x_dev != nullptr, PIPERAG_ERR_ARG, "x_dev is NULL");
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(index->device));
    rc = encode_impl(index, x_dev, n, index->st_list + index->nadded, true, index->st_codes + (size_t)index->nadded * index->p.M, st);
    if (rc != PIPERAG_OK) return rc;
    rc = append_ids(index, n, ids_dev, st);
    if (rc != PIPERAG_OK) return rc;
    index->nadded += n;
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

int piperag_ivf_count(piperag_index *index, const float *x_dev, int64_t n, void *stream) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(n >= 0, PIPERAG_ERR_ARG, "n = %lld is negative", (long long)n);
    PR_REQUIRE(!index->finalized && !index->reserved, PIPERAG_ERR_ARG, "count calls come before reserve");
    PR_REQUIRE(index->nadded + n <= index->cap, PIPERAG_ERR_LIMIT, "counting %lld vectors after %lld exceeds the capacity %lld",
               (long long)n, (long long)index->nadded, (long long)index->cap);
    if (n == 0) return PIPERAG_OK;
    PR_REQUIRE(x_dev != nullptr, PIPERAG_ERR_ARG, "x_dev is NULL");
    int rc = begin_build(index, 2);
    if (rc != PIPERAG_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(index->device));
    const piperag_params &p = index->p;
    int32_t *lists = index->st_list + index->nadded;
    rc = launch_assign(x_dev, n, p.d, p.d, index->centroids, index->cnorm, index->cent_hi, index->cent_lo, p.nlist, lists, nullptr, st);
    if (rc != PIPERAG_OK) return rc;
    count_lists(lists, n, index->bd_counts, st);
    index->nadded += n;
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

int piperag_ivf_place(piperag_index *index, const float *x_dev, int64_t n, const int64_t *ids_dev, void *stream) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(n >= 0, PIPERAG_ERR_ARG, "n = %lld is negative", (long long)n);
    PR_REQUIRE(!index->finalized && index->build_mode == 2 && index->reserved, PIPERAG_ERR_ARG, "place calls come after reserve");
    PR_REQUIRE(index->nplaced + n <= index->nadded, PIPERAG_ERR_LIMIT, "placing %lld vectors after %lld exceeds the %lld counted",
               (long long)n, (long long)index->nplaced, (long long)index->nadded);
    if (n == 0) return PIPERAG_OK;
    PR_REQUIRE(x_dev != nullptr, PIPERAG_ERR_ARG, "x_dev is NULL");
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(index->device));
    const piperag_params &p = index->p;
    uint8_t *codes = nullptr;
    int64_t *ids = nullptr;
    PR_CHECK_HIP(hipMallocAsync(reinterpret_cast<void **>(&codes), (size_t)n * p.M, st));
    if (!ids_dev) {
        const hipError_t e = hipMallocAsync(reinterpret_cast<void **>(&ids), sizeof(int64_t) * (size_t)n, st);
        if (e != hipSuccess) { (void)hipFreeAsync(codes, st); set_error("scratch allocation failed: %s", hipGetErrorString(e)); return PIPERAG_ERR_OOM; }
        fill_iota(ids, n, index->nplaced, st);
    }
    int rc = encode_impl(index, x_dev, n, index->st_list + index->nplaced, false, codes, st);
    if (rc == PIPERAG_OK) rc = place_tile(index, index->st_list + index->nplaced, codes, ids_dev ? ids_dev : ids, n, st);
    (void)hipFreeAsync(codes, st);
    if (ids) (void)hipFreeAsync(ids, st);
    if (rc != PIPERAG_OK) return rc;
    index->nplaced += n;
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

}  // extern "C"
