// Database construction on the GPU (Section 2, "Database construction"; Appendix "Detailed Evaluation
// Setup", Software: every vector is assigned to one of nlist inverted lists and quantised into M code
// bytes).  list(x) = argmin_j ||x - centre_j||^2, code[m] = argmin_j ||x_m - pq[m][j]||^2, lowest index on equal
// values.  What decides the arg-min: for lists, on shapes the matrix cores take (128 centres or more, d >= 64), a
// split-fp16 product |c|^2 - 2 <x, c> shortlists two centres per vector and their direct-form fp32 distances
// sum_t (x_t - c_t)^2 decide between the two; on other shapes the direct form alone.  For codes, with 4 or
// more coordinates per sub-quantiser, the fp32 matrix-core product |p|^2 - 2 <x_m, p>; below that the direct form.
#include <stdlib.h>

#include <algorithm>
#include <mutex>

#include "common.h"
#include "mfma_f16x3.h"
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
// vectors entered as (-2 x_m, 1) the product is the quantity v to minimise itself.  A lane then holds 128 centres
// of one vector in its own registers and walks them in ascending centre order (strict "<": lower index on equal
// values); the two lanes that share a vector are combined with lane exchanges.
// v orders the centres like the distance does up to its rounding errors, which are relative to |x_m||p| and not
// to the distance, so the decision is made exact the way the list assignment's is: a lane keeps its smallest v
// with its centre, and its second smallest v; with v1 and v2 the two smallest of the pair, every centre that
// could be the nearest has v <= v1 + margin (margin = 4 (T + 2) 2^-24 (|x_m|^2 + |p1|^2): twice a bound on the
// error of a v over T + 2 roundings).  v2 beyond the margin: v1's centre is the code.  Otherwise (a few (vector,
// sub-quantiser) pairs in a thousand at the benchmark's mixtures) both lanes compute the direct form
// sum_t (x_t - p_t)^2 for all their centres, lower index on equal values.  Codes are collected in LDS and written
// out as one contiguous run.  T = pqe_rows(dsub) depth rows (even), dsub <= 32.
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
    auto x_at = [&](int m, int t) -> float {                     // coordinate t of the m-th slice of this lane's vector
        float v = live ? xr[m * dsub + t] : 0.f;
        if (cr) v -= cr[m * dsub + t];
        return v;
    };
    auto centre_of = [&](int bi, int r) { return bi * 32 + (r % 4) + 4 * half + 8 * (r / 4); };   // of accumulator register r of block bi
    const float inf = __builtin_inff();
    const float margin_scale = 4.f * (float)(T + 2) * 5.9604645e-8f;
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
        float xq = 0.f;                                           // 4 x the squared norm of this lane's depth rows of x_m
        for (int p = 0; p < T / 2; ++p) {
            const int t = 2 * p + half;                           // lanes 0-31: depth 2p, lanes 32-63: depth 2p + 1
            float bv = t == dsub ? 1.f : 0.f;                     // the row of norms; padding rows are zero on both sides
            if (t < dsub) {
                bv = -2.f * x_at(m, t);
                xq += bv * bv;
            }
            const float *a = sA + t * kKsub + l32;
#pragma unroll
            for (int bi = 0; bi < 8; ++bi) acc[bi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bi * 32], bv, acc[bi], 0, 0, 0);
        }
        float b1v = inf, b2v = inf;                               // smallest v and its centre; second smallest v
        int b1c = 0;
#pragma unroll
        for (int bi = 0; bi < 8; ++bi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {                        // ascending in bi, r = ascending centre; no branches
                const float v = acc[bi][r];
                const bool lt = v < b1v;
                b2v = fminf(b2v, lt ? b1v : v);
                b1c = lt ? centre_of(bi, r) : b1c;
                b1v = lt ? v : b1v;
            }
        // the pair's smallest v, its centre and the margin
        const float o1v = __shfl_xor(b1v, 32, 64), o2v = __shfl_xor(b2v, 32, 64), xn = 0.25f * (xq + __shfl_xor(xq, 32, 64));
        const int o1c = __shfl_xor(b1c, 32, 64);
        const bool mine_first = b1v < o1v || (b1v == o1v && b1c < o1c);
        const float v1 = mine_first ? b1v : o1v;
        int code = mine_first ? b1c : o1c;
        const float limit = v1 + margin_scale * (xn + sA[dsub * kKsub + code]);
        // the pair's second smallest v: the other lane's smallest, or the second smallest of either lane
        const float v2 = fminf(fminf(b2v, o2v), mine_first ? o1v : b1v);
        if (__any(v2 <= limit)) {                                 // seldom: direct-form distances decide
            float best_d = inf;
            int best_c = 256;
            if (v2 <= limit) {                                    // the same for both lanes of the pair: every centre of this lane
#pragma unroll
                for (int bi = 0; bi < 8; ++bi)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[bi][r] = 0.f;
                for (int t = 0; t < dsub; ++t) {
                    const float xv = x_at(m, t);
                    const float *a = sA + t * kKsub + 4 * half;
#pragma unroll
                    for (int bi = 0; bi < 8; ++bi)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float e1 = xv - a[bi * 32 + (r % 4) + 8 * (r / 4)];
                            acc[bi][r] += e1 * e1;
                        }
                }
#pragma unroll
                for (int bi = 0; bi < 8; ++bi)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (acc[bi][r] < best_d) { best_d = acc[bi][r]; best_c = centre_of(bi, r); }
                const float od = __shfl_xor(best_d, 32, 64);
                const int oc = __shfl_xor(best_c, 32, 64);
                code = (od < best_d || (od == best_d && oc < best_c)) ? oc : best_c;
            }
        }
        if (half == 0) code_s[(wave * 32 + l32) * M + m] = (uint8_t)code;
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
// Largest magnitude of a matrix (n rows of d values, stride ld), as the bit pattern of the fp32 value, by atomic
// maximum into *out (which the caller has zeroed; bit patterns of non-negative floats order like the values).
__global__ __launch_bounds__(256) void absmax_kernel(const float *__restrict__ src, int64_t n, int d, int64_t ld,
                                                     uint32_t *__restrict__ out) {
    const int64_t total = n * d;
    uint32_t m = 0;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / d;
        m = max(m, __float_as_uint(src[row * ld + (e - row * d)]) & 0x7FFFFFFFu);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0 && m != 0) atomicMax(out, m);
}
__global__ void zero_u32_kernel(uint32_t *p) { *p = 0u; }
__global__ void zero_words_kernel(uint32_t *p, int n) { if ((int)threadIdx.x < n) p[threadIdx.x] = 0u; }

// Power of two s with amax * s in [2^14, 2^15) (1 for a zero matrix), and the exponent of 1 / s.
__device__ __forceinline__ int split_exponent(uint32_t amax_bits) {        // e with s = 2^e
    if (amax_bits == 0) return 0;
    const int ex = min(127, max(-126, (int)(amax_bits >> 23) - 127));      // amax in [2^ex, 2^(ex+1))
    return 14 - ex;
}
__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((uint32_t)(min(127, max(-126, e)) + 127) << 23); }

// Scaled fp16 hi / lo parts of an fp32 matrix (n rows of d values, stride ld) in the chunk-major layout of
// mfma_f16x3.h; the scale comes from the matrix's largest magnitude (*amax, see absmax_kernel).  One thread per
// (row, chunk of 8 values), padding rows and chunks are written as zeros.
__global__ void split_f16_kernel(const float *__restrict__ src, int64_t n, int d, int64_t ld, int64_t rows_pad, int nchunks,
                                 const uint32_t *__restrict__ amax, uint16_t *__restrict__ hi, uint16_t *__restrict__ lo) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows_pad * nchunks) return;
    const float scale = pow2f(split_exponent(*amax));
    const int64_t row = e / nchunks;
    const int c = (int)(e % nchunks);
    uint16_t h[8], l[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int k = c * 8 + t;
        const float v = (row < n && k < d) ? src[row * ld + k] * scale : 0.f;     // exact: a power of two, no overflow by construction
        const _Float16 vh = (_Float16)v;
        const _Float16 vl = (_Float16)(v - (float)vh);
        h[t] = __builtin_bit_cast(uint16_t, vh);
        l[t] = __builtin_bit_cast(uint16_t, vl);
    }
    const size_t o = ((size_t)c * rows_pad + row) * 8;
#pragma unroll
    for (int t = 0; t < 8; ++t) { hi[o + t] = h[t]; lo[o + t] = l[t]; }
}

// ---- nearest-centre assignment on the matrix cores, with an exact decision -------------------------
// Stage 1 (assign_f16x3_kernel): the split-fp16 tile product gives v = |c|^2 - 2 <x, c> for every (vector,
//   centre); per vector and per *source* (one of a fixed partition of the centres into 4 R parts, see below) the
//   two smallest v and their centres are kept, and the third smallest v as a bound on everything not kept.
// Stage 2 (assign_finish_kernel): v orders the centres like the distance does, up to its rounding errors, which
//   are relative to |x||c| and not to the distance.  With v1 the smallest v of a vector, every centre that could
//   be the nearest has v <= v1 + margin (margin = kAssignMargin (|x|^2 + |c1|^2), a bound on twice the error of a
//   v: a few 2^-24 per accumulation step of the product, the norms and the final subtraction).  The kept centres
//   within the margin are compared by their direct-form fp32 distances sum_t (x_t - c_t)^2, lower index on
//   equal values.  If the third smallest v of some source of a centre range is also within the margin, a
//   candidate of that range may not have been kept: the vector goes to stage 3 for that range.
// Stage 3 (assign_rows_direct_kernel + assign_rows_finish_kernel): the direct form against every centre of the
//   range for the (vector, range) pairs stage 2 could not settle (a hundred or two per 262,144 at the benchmark's mixtures; most of them when
//   many centres lie within the rounding error of the nearest one).
constexpr float kAssignMargin = 4e-5f;
constexpr int kAssignWords = 9;                // per (vector, centre range): 8 keys (value bits << 32 | centre) and the bound

__device__ __forceinline__ uint32_t ordered_bits(float v) {                 // unsigned order == float order
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unordered_bits(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}

// A workgroup (8 waves) takes 256 vectors against the centres of its range, 256 at a time.  The centres are the tile's A
// operand, so a lane holds, for each of its two vector columns, 64 centres of the tile in its own registers and
// walks them in ascending centre order (a strict "<" keeps the lower index on equal values); a column's values
// are spread over four such sources (lanes l and l + 32 of the two wave rows), which meet in LDS at the end.
// The centres are split over R ranges of `per_range` centres (a multiple of 256); range r writes kAssignWords
// words for row i at cand[((size_t)r * n + i) * kAssignWords].  grid = (vector tiles rounded up to a multiple of
// 8) * R workgroups.
__global__ __launch_bounds__(F16x3Tile::kThreads, 1) void assign_f16x3_kernel(int64_t n, int nchunks, const uint16_t *__restrict__ xhi,
                                                              const uint16_t *__restrict__ xlo, int64_t x_rp,
                                                              const uint16_t *__restrict__ chi, const uint16_t *__restrict__ clo,
                                                              int64_t c_rp, const uint32_t *__restrict__ x_amax,
                                                              const uint32_t *__restrict__ c_amax,
                                                              const float *__restrict__ cnorm, int K, int R, int per_range,
                                                              uint64_t *__restrict__ cand) {
    extern __shared__ __align__(16) unsigned char bsmem[];
    float *s_cn = reinterpret_cast<float *>(bsmem + F16x3Tile::kLdsBytes);        // [2][256] centre norms of a tile (+inf: no centre)
    const int tid = threadIdx.x, lane = tid & 63, wr = tid >> 8;
    // Which (vector tile, centre range) this workgroup takes.  Workgroups are dealt to the 8 XCDs in turn by
    // their launch number: the R ranges of one vector tile go to workgroups 8 apart, i.e. to one XCD and next to
    // each other in launch order, so that the tile's vectors are fetched into one L2 and found there by the
    // other ranges, while the workgroups that walk the same range on that XCD share the centres.
    const int i = blockIdx.x, g = i / (8 * R), j = i - g * 8 * R;
    const int tile_v = g * 8 + (j & 7), range = j >> 3;
    const int64_t row0 = (int64_t)tile_v * F16x3Tile::kRowsB;
    if (row0 >= n) return;                                     // padding of the last group of 8 tiles (uniform)
    const int jbeg = range * per_range, jend = min(K, jbeg + per_range);
    // the tile product holds <x, c> times the two scales, both powers of two: undone exactly
    const float m2 = -2.f * pow2f(-split_exponent(*x_amax) - split_exponent(*c_amax));
    const float inf = __builtin_inff();
    float b1v[2] = {inf, inf}, b2v[2] = {inf, inf}, b3v[2] = {inf, inf};
    int b1c[2] = {K, K}, b2c[2] = {K, K};                      // K: no centre
    const int ntiles = (jend - jbeg + F16x3Tile::kRowsA - 1) / F16x3Tile::kRowsA;
    // the squared norms of a tile's centres travel beside the stream: asked for at the tile's first step (straight
    // into LDS, buffer t % 2: read when the tile is complete, rewritten two tiles later), and places beyond the
    // range's last centre set to +inf two steps later
    const uint32_t cn_lds = __builtin_amdgcn_readfirstlane(F16x3Tile::lds_address(s_cn) + (uint32_t)(tid >> 6) * 256u);
    auto hook = [&](int t, int s) {
        if (s != 0 && s != 2) return;                           // uniform
        if (tid < F16x3Tile::kRowsA) {                          // whole waves
            const int c = jbeg + t * F16x3Tile::kRowsA + tid;
            if (s == 0) F16x3Tile::load_to_lds_f32(cnorm, (uint32_t)min(c, K - 1) * 4u, cn_lds + (uint32_t)(t & 1) * 1024u);
            else if (c >= jend) s_cn[(t & 1) * F16x3Tile::kRowsA + tid] = inf;
        }
    };
    auto tile_done = [&](int t, const acc16_t (&acc)[4][2]) {
        const float *cn = s_cn + (t & 1) * F16x3Tile::kRowsA;
        const int j0 = jbeg + t * F16x3Tile::kRowsA;
#pragma unroll
        for (int bi = 0; bi < 4; ++bi)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int r0 = F16x3Tile::acc_row(bi, 4 * gq);                     // rows r0 .. r0+3 are registers 4gq .. 4gq+3
                const float4 nn = *reinterpret_cast<const float4 *>(cn + r0);
                const float nv[4] = {nn.x, nn.y, nn.z, nn.w};
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
                    for (int bj = 0; bj < 2; ++bj) {
                        const float v = nv[t4] + m2 * acc[bi][bj][4 * gq + t4];
                        if (v < b3v[bj]) {                     // seldom true once the running values have settled
                            const int c = j0 + r0 + t4;
                            if (v < b2v[bj]) {
                                b3v[bj] = b2v[bj];
                                if (v < b1v[bj]) { b2v[bj] = b1v[bj]; b2c[bj] = b1c[bj]; b1v[bj] = v; b1c[bj] = c; }
                                else { b2v[bj] = v; b2c[bj] = c; }
                            } else {
                                b3v[bj] = v;
                            }
                        }
                    }
            }
    };
    F16x3Tile::run_tiles(chi, clo, c_rp, jbeg, ntiles, xhi, xlo, x_rp, row0, nchunks, bsmem, hook, tile_done);
    __syncthreads();                                           // the tile buffers are free
    uint64_t *s_key = reinterpret_cast<uint64_t *>(bsmem);     // [256 columns][8 keys + 4 bounds]
#pragma unroll
    for (int bj = 0; bj < 2; ++bj) {
        const int col = F16x3Tile::acc_col(bj), src = wr * 2 + (lane >> 5);
        s_key[col * 12 + src * 2] = ((uint64_t)ordered_bits(b1v[bj]) << 32) | (uint32_t)b1c[bj];
        s_key[col * 12 + src * 2 + 1] = ((uint64_t)ordered_bits(b2v[bj]) << 32) | (uint32_t)b2c[bj];
        s_key[col * 12 + 8 + src] = (uint64_t)ordered_bits(b3v[bj]);
    }
    __syncthreads();
    for (int e = tid; e < F16x3Tile::kRowsB * kAssignWords; e += F16x3Tile::kThreads) {   // rows of this tile are contiguous in cand
        const int col = e / kAssignWords, w = e - col * kAssignWords;
        if (row0 + col >= n) continue;
        uint64_t word = s_key[col * 12 + w];
        if (w == 8) {
#pragma unroll
            for (int u = 1; u < 4; ++u) word = min(word, s_key[col * 12 + 8 + u]);
        }
        cand[((size_t)range * n + row0) * kAssignWords + e] = word;
    }
}

// One wavefront per vector (see the head of this section).  A centre range whose bound lies within the margin
// may hold a nearer centre that was not kept: the vector joins that range's list for stage 3 (flist[range][..],
// nflag[range]), and fkey[row] starts as the best found here, for stage 3's atomic minimum.
__global__ __launch_bounds__(256) void assign_finish_kernel(const float *__restrict__ x, int64_t n, int d, int64_t ldx,
                                                            const float *__restrict__ cent, const float *__restrict__ cnorm, int K,
                                                            const uint64_t *__restrict__ cand, int R,
                                                            int32_t *__restrict__ out_idx, float *__restrict__ out_dist,
                                                            uint32_t *__restrict__ flist, int64_t flist_stride,
                                                            unsigned long long *__restrict__ fkey, uint32_t *__restrict__ nflag) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const float *xr = x + row * ldx;
    float xn = 0.f;
    for (int t = lane; t < d; t += 64) xn += xr[t] * xr[t];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) xn += __shfl_xor(xn, off, 64);
    // this lane's share of the words: entry e = range * kAssignWords + w
    constexpr int kPerLane = 3;                                // 64 * 3 >= kAssignWords * 16 ranges
    uint64_t mine[kPerLane];                                   // a key, or ~0
    uint32_t bound[kPerLane];                                  // a range's bound (ordered bits), or ~0
    uint64_t k1 = ~0ull;
#pragma unroll
    for (int u = 0; u < kPerLane; ++u) {
        const int e = lane + 64 * u;
        mine[u] = ~0ull;
        bound[u] = 0xFFFFFFFFu;
        if (e < R * kAssignWords) {
            const int r = e / kAssignWords, w = e - r * kAssignWords;
            const uint64_t word = cand[((size_t)r * n + row) * kAssignWords + w];
            if (w == 8) bound[u] = (uint32_t)word;
            else if ((uint32_t)word < (uint32_t)K) { mine[u] = word; k1 = min(k1, word); }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) k1 = min(k1, (uint64_t)__shfl_xor((unsigned long long)k1, off, 64));
    const bool any = k1 != ~0ull;                              // false only for values that are not numbers
    const float v1 = unordered_bits((uint32_t)(k1 >> 32));
    const float margin = kAssignMargin * (xn + (any ? cnorm[(uint32_t)k1] : 0.f));
    const float limit = v1 + margin;
    // direct-form distance to every kept centre within the margin, one after the other
    float best_d = __builtin_inff();
    int best_c = any ? (int)(uint32_t)k1 : 0;
#pragma unroll
    for (int u = 0; u < kPerLane; ++u) {
        const bool have = mine[u] != ~0ull && unordered_bits((uint32_t)(mine[u] >> 32)) <= limit;
        uint64_t todo = __ballot(have);
        while (todo) {
            const int src = __ffsll((unsigned long long)todo) - 1;
            todo &= todo - 1;
            const int c = (int)(uint32_t)__shfl((unsigned long long)mine[u], src, 64);
            const float *pc = cent + (size_t)c * d;
            float a = 0.f;
            for (int t = lane; t < d; t += 64) { const float e1 = xr[t] - pc[t]; a += e1 * e1; }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
            if (a < best_d || (a == best_d && c < best_c)) { best_d = a; best_c = c; }
        }
    }
    // ranges that may hold a nearer centre than the kept ones
    bool handed_on = false;
#pragma unroll
    for (int u = 0; u < kPerLane; ++u) {
        const int e = lane + 64 * u;
        if (bound[u] != 0xFFFFFFFFu && (!any || unordered_bits(bound[u]) <= limit)) {
            const int r = e / kAssignWords;
            const uint32_t pos = atomicAdd(&nflag[r], 1u);
            flist[(size_t)r * flist_stride + pos] = (uint32_t)row;
            handed_on = true;
        }
    }
    const bool some = __ballot(handed_on) != 0;
    if (lane == 0) {
        out_idx[row] = best_c;
        if (out_dist) out_dist[row] = best_d;
        if (some) fkey[row] = ((unsigned long long)__float_as_uint(best_d) << 32) | (unsigned)best_c;
    }
}

// Stage 3: direct-form distances of a range's listed rows to the centres of one split of that range, 64 rows per
// workgroup at a time (the tiling of assign_kernel); the nearest of a split meets the others', and the best of
// stage 2, by an atomic minimum on (distance bits << 32 | centre) in fkey[row].  grid = (row groups, splits per
// range, ranges); workgroups beyond a list return at once.
__global__ __launch_bounds__(256) void assign_rows_direct_kernel(const float *__restrict__ x, int d, int64_t ldx,
                                                                 const uint32_t *__restrict__ flist, int64_t flist_stride,
                                                                 const uint32_t *__restrict__ nflag,
                                                                 const float *__restrict__ cent, int K, int per_range, int per_split,
                                                                 unsigned long long *__restrict__ fkey) {
    __shared__ __align__(16) float xs[TK * LDT];
    __shared__ __align__(16) float cs[TK * LDT];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int lr = tid >> 2, lk = (tid & 3) * 4;
    const int range = blockIdx.z;
    const int count = (int)nflag[range];
    const uint32_t *list = flist + (size_t)range * flist_stride;
    const int jbeg = range * per_range + blockIdx.y * per_split, jend = min(min(K, (range + 1) * per_range), jbeg + per_split);
    if (jbeg >= jend) return;                                                  // uniform
    for (int p0 = blockIdx.x * TM; p0 < count; p0 += gridDim.x * TM) {          // uniform
        const int64_t my_row = p0 + lr < count ? (int64_t)list[p0 + lr] : -1;
        float best_d[4];
        int best_j[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { best_d[i] = __builtin_inff(); best_j[i] = 0x7FFFFFFF; }
        for (int j0 = jbeg; j0 < jend; j0 += TN) {
            float acc[4][4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) acc[i][jj] = 0.f;
            for (int k0 = 0; k0 < d; k0 += TK) {
                float xv[4], cv[4];
                const int cr = j0 + lr;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int kk = k0 + lk + i;
                    xv[i] = (my_row >= 0 && kk < d) ? x[my_row * ldx + kk] : 0.f;
                    cv[i] = (cr < jend && kk < d) ? cent[(size_t)cr * d + kk] : 0.f;
                }
                __syncthreads();
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
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int jc = j0 + tx * 4 + jj;
                    if (jc < jend && (acc[i][jj] < best_d[i] || (acc[i][jj] == best_d[i] && jc < best_j[i]))) { best_d[i] = acc[i][jj]; best_j[i] = jc; }
                }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int pos = p0 + ty * 4 + i;
            if (pos < count && best_j[i] != 0x7FFFFFFF)
                atomicMin(&fkey[list[pos]], ((unsigned long long)__float_as_uint(best_d[i]) << 32) | (unsigned)best_j[i]);
        }
    }
}
// ... and what the minimum came to, for every listed row (grid.y = ranges; a row listed by several ranges is
// written several times, with the same value).
__global__ void assign_rows_finish_kernel(const uint32_t *__restrict__ flist, int64_t flist_stride, const uint32_t *__restrict__ nflag,
                                          const unsigned long long *__restrict__ fkey, int32_t *__restrict__ out_idx,
                                          float *__restrict__ out_dist) {
    const uint32_t count = nflag[blockIdx.y];
    const uint32_t *list = flist + (size_t)blockIdx.y * flist_stride;
    for (uint32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < count; p += gridDim.x * blockDim.x) {
        const uint32_t row = list[p];
        const unsigned long long key = fkey[row];
        out_idx[row] = (int32_t)(uint32_t)key;
        if (out_dist) out_dist[row] = __uint_as_float((uint32_t)(key >> 32));
    }
}

// cnorm: squared norms of the centres (f32 [K]) or NULL.  The matrix-core path is taken when the shape pays for
// it and allows 16-byte loads; otherwise the direct-form VALU kernel runs.
// chi / clo / c_amax: scaled fp16 split of the centres (u16 [K*d] each) and the word its scale follows from, or NULL.  The matrix-core paths are taken when the shape
// pays for them and allows 16-byte loads: split-fp16 first, fp32 MFMA second; otherwise the direct-form VALU
// kernel runs.
void launch_split(const float *src, int64_t n, int d, int64_t ld, uint32_t *amax, uint16_t *hi, uint16_t *lo, hipStream_t st);

// Centre ranges per vector tile of the split-fp16 assignment: the ranges of a tile run side by side on one XCD
// (see the kernel), 8 vector tiles x 8 ranges filling its 64 workgroup slots.
#ifndef PIPERAG_ASSIGN_RANGES
#define PIPERAG_ASSIGN_RANGES 8
#endif
int assign_ranges() { return PIPERAG_ASSIGN_RANGES; }

int launch_assign(const float *x, int64_t n, int d, int64_t ldx, const float *cent, const float *cnorm, const uint16_t *chi,
                  const uint16_t *clo, const uint32_t *c_amax, int K, int32_t *out_idx, float *out_dist, hipStream_t st) {
    const int vec4 = (d % 4 == 0) && (ldx % 4 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(cent) % 16 == 0);
    const bool mfma = vec4 && cnorm != nullptr && K >= 128 && d >= 64;
    const bool split16 = cnorm != nullptr && K >= 128 && d >= 64 && chi != nullptr && clo != nullptr && c_amax != nullptr;
    constexpr size_t kBfLds = F16x3Tile::kLdsBytes + sizeof(float) * 2 * F16x3Tile::kRowsA;
    if (split16) {
        // the vectors are split slice by slice into a scratch area that lives in stream order; the shortlist
        // (two keys per vector and centre range) follows it
        const int64_t slice = std::max<int64_t>(F16x3Tile::kRowPad, ((int64_t)1 << 28) / ((int64_t)F16x3Tile::chunks_pad(d) * 8) /
                                                                         F16x3Tile::kRowPad * F16x3Tile::kRowPad);
        const int64_t cap_rows = std::min(slice, F16x3Tile::rows_pad(n));
        const size_t part = F16x3Tile::part_elems(cap_rows, d);
        // centre ranges: multiples of 256 centres, at most kAssignRanges of them
        const int tiles_c = (K + F16x3Tile::kRowsA - 1) / F16x3Tile::kRowsA;
        const int R = std::max(1, std::min(std::min(assign_ranges(), 16), tiles_c));
        const int per_range = (tiles_c + R - 1) / R * F16x3Tile::kRowsA;
        const int Ruse = (K + per_range - 1) / per_range;
        const size_t split_bytes = (2 * part * sizeof(uint16_t) + 255) / 256 * 256;
        const size_t cand_bytes = sizeof(uint64_t) * kAssignWords * (size_t)Ruse * cap_rows;
        const size_t flist_bytes = (sizeof(uint32_t) * (size_t)Ruse * cap_rows + 255) / 256 * 256;
        const size_t fkey_bytes = sizeof(unsigned long long) * (size_t)cap_rows;
        unsigned char *scratch = nullptr;
        PR_CHECK_HIP(hipMallocAsync(reinterpret_cast<void **>(&scratch), split_bytes + cand_bytes + flist_bytes + fkey_bytes + 512, st));
        uint16_t *xs = reinterpret_cast<uint16_t *>(scratch);
        uint64_t *cand = reinterpret_cast<uint64_t *>(scratch + split_bytes);
        uint32_t *flist = reinterpret_cast<uint32_t *>(scratch + split_bytes + cand_bytes);
        unsigned long long *fkey = reinterpret_cast<unsigned long long *>(scratch + split_bytes + cand_bytes + flist_bytes);
        uint32_t *x_amax = reinterpret_cast<uint32_t *>(scratch + split_bytes + cand_bytes + flist_bytes + fkey_bytes);
        uint32_t *nflag = x_amax + 64;                       // one count per centre range (at most 16)
        const int nchunks = F16x3Tile::chunks_pad(d);
        const int64_t c_rp = F16x3Tile::rows_pad(K);
        // stage 3 splits a range's centres finely, one 64-centre tile per workgroup where the range allows it: its
        // workgroups are bound by the latency of their loads (a tile takes about 100 us whatever else runs), so a
        // handful of rows is done soonest by as many of them as there are tiles (3.3 ms per launch with 256 centres
        // each); the rows of a long list are walked by a few row groups in turn
        const int splits_target = std::max(1, 1024 / Ruse);
        const int per_split = std::max(TN, (per_range + splits_target - 1) / splits_target / TN * TN);
        const int splits = (per_range + per_split - 1) / per_split;
        for (int64_t a = 0; a < n; a += slice) {
            const int64_t cnt = std::min(slice, n - a), rp = F16x3Tile::rows_pad(cnt);
            launch_split(x + a * ldx, cnt, d, ldx, x_amax, xs, xs + part, st);
            hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, st, nflag, 16);
            const int64_t tiles_v = (cnt + F16x3Tile::kRowsB - 1) / F16x3Tile::kRowsB;
            const unsigned grid = (unsigned)((tiles_v + 7) / 8 * 8 * Ruse);
            hipLaunchKernelGGL(assign_f16x3_kernel, dim3(grid), dim3(F16x3Tile::kThreads), kBfLds, st, cnt, nchunks, xs, xs + part, rp, chi, clo, c_rp,
                               x_amax, c_amax, cnorm, K, Ruse, per_range, cand);
            hipLaunchKernelGGL(assign_finish_kernel, dim3((unsigned)((cnt + 3) / 4)), dim3(256), 0, st, x + a * ldx, cnt, d, ldx, cent,
                               cnorm, K, cand, Ruse, out_idx + a, out_dist ? out_dist + a : nullptr, flist, cap_rows, fkey, nflag);
            const unsigned row_groups = (unsigned)std::min<int64_t>((cnt + TM - 1) / TM, 16);
            hipLaunchKernelGGL(assign_rows_direct_kernel, dim3(row_groups, splits, Ruse), dim3(256), 0, st, x + a * ldx, d, ldx, flist,
                               cap_rows, nflag, cent, K, per_range, per_split, fkey);
            hipLaunchKernelGGL(assign_rows_finish_kernel, dim3(16, Ruse), dim3(256), 0, st, flist, cap_rows, nflag, fkey, out_idx + a,
                               out_dist ? out_dist + a : nullptr);
        }
        PR_CHECK_HIP(hipFreeAsync(scratch, st));
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

// Splits n rows of d values (stride ld) into the chunk-major scaled fp16 hi / lo parts; each part holds
// F16x3Tile::part_elems(n, d) elements.  amax (device, one word) receives the bits of the matrix's largest magnitude,
// from which the scale follows; whoever multiplies the parts needs it to undo the scale.
void launch_split(const float *src, int64_t n, int d, int64_t ld, uint32_t *amax, uint16_t *hi, uint16_t *lo, hipStream_t st) {
    const int64_t rp = F16x3Tile::rows_pad(n);
    const int nchunks = F16x3Tile::chunks_pad(d);
    hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(1), 0, st, amax);
    const unsigned blocks = (unsigned)std::min<int64_t>(4096, (n * d + 255) / 256);
    if (blocks > 0) hipLaunchKernelGGL(absmax_kernel, dim3(blocks), dim3(256), 0, st, src, n, d, ld, amax);
    hipLaunchKernelGGL(split_f16_kernel, dim3((unsigned)((rp * nchunks + 255) / 256)), dim3(256), 0, st, src, n, d, ld, rp, nchunks, amax,
                       hi, lo);
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
// Per device, once: the encoder's kernels may use the whole 160 KiB of LDS as dynamic shared memory.
int configure_encode_kernels(int device) {
    static std::mutex mutex;
    static bool done[64];
    PR_REQUIRE(device >= 0 && device < 64, PIPERAG_ERR_ARG, "device %d out of range", device);
    std::lock_guard<std::mutex> lock(mutex);
    if (done[device]) return PIPERAG_OK;
    int cur = -1;
    PR_CHECK_HIP(hipGetDevice(&cur));
    if (cur != device) PR_CHECK_HIP(hipSetDevice(device));
    const void *kernels[] = {reinterpret_cast<const void *>(&assign_f16x3_kernel), reinterpret_cast<const void *>(&pq_encode_mfma_kernel),
                             reinterpret_cast<const void *>(&pq_encode_kernel)};
    for (const void *k : kernels) {             // whatever the kernel's static LDS leaves of the 160 KiB
        hipFuncAttributes fa;
        PR_CHECK_HIP(hipFuncGetAttributes(&fa, k));
        PR_CHECK_HIP(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - (int)fa.sharedSizeBytes));
    }
    done[device] = true;
    if (cur != device && cur >= 0) PR_CHECK_HIP(hipSetDevice(cur));
    return PIPERAG_OK;
}
void rownorm(const float *a, int64_t n, int d, int64_t lda, float *out, hipStream_t st) { launch_rownorm(a, n, d, lda, out, st); }
void split_f16(const float *src, int64_t n, int d, uint32_t *amax, uint16_t *hi, uint16_t *lo, hipStream_t st) { launch_split(src, n, d, d, amax, hi, lo, st); }
size_t split_f16_elems(int64_t n, int d) { return F16x3Tile::part_elems(n, d); }
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
        const int rc = launch_assign(x, n, p.d, p.d, ix->centroids, ix->cnorm, ix->cent_hi, ix->cent_lo, ix->cent_amax, p.nlist, lists, nullptr, st);
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
                PR_REQUIRE(lds <= 160 * 1024, PIPERAG_ERR_LIMIT, "the encoder needs %zu bytes of LDS (M too large)", lds);
                hipLaunchKernelGGL(pq_encode_mfma_kernel, dim3((unsigned)((cnt + 127) / 128)), dim3(256), lds, st, x + a * p.d, cnt,
                                   p.d, ix->pqE, p.M, ix->dsub, T, res_lists ? res_lists + a : nullptr, ix->centroids,
                                   out_codes + (size_t)a * p.M);
            } else {
                const size_t lds = sizeof(float) * 2 * kKsub * ix->dsub + (size_t)256 * p.M;
                PR_REQUIRE(lds <= 160 * 1024, PIPERAG_ERR_LIMIT, "the encoder needs %zu bytes of LDS (M too large)", lds);
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
    {
        int device = 0;
        PR_CHECK_HIP(hipGetDevice(&device));
        const int rcc = configure_encode_kernels(device);
        if (rcc != PIPERAG_OK) return rcc;
    }
    int64_t *rows = nullptr;
    int32_t *assign = nullptr;
    float *adist = nullptr;
    long long *sum = nullptr;
    int *count = nullptr;
    float *cnorm = nullptr;
    uint16_t *chi = nullptr, *clo = nullptr;
    uint32_t *camax = nullptr;
    float *hdist = inertia_out_host ? (float *)malloc(sizeof(float) * (size_t)n) : nullptr;
    auto done = [&](int code) {
        (void)hipFree(rows); (void)hipFree(assign); (void)hipFree(adist); (void)hipFree(sum); (void)hipFree(count); (void)hipFree(cnorm); (void)hipFree(chi); (void)hipFree(clo); (void)hipFree(camax);
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
    if (use_split && (hipMalloc((void **)&chi, sizeof(uint16_t) * F16x3Tile::part_elems(K, d)) != hipSuccess ||
                      hipMalloc((void **)&clo, sizeof(uint16_t) * F16x3Tile::part_elems(K, d)) != hipSuccess ||
                      hipMalloc((void **)&camax, 256) != hipSuccess)) {
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
        if (use_split) launch_split(centroids_out_dev, K, d, d, camax, chi, clo, st);
        const int rca = launch_assign(x_dev, n, d, ldx, centroids_out_dev, cnorm, chi, clo, camax, K, assign, adist, st);
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
    rc = launch_assign(x_dev, n, p.d, p.d, index->centroids, index->cnorm, index->cent_hi, index->cent_lo, index->cent_amax, p.nlist, lists, nullptr, st);
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
