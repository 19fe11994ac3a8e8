// Search path of libpiperag: coarse quantiser, top-nprobe selection, scan plan, lookup-table build,
// list scan with k-selection, merge of a query's partial results and id gather.  All kernels are written for
// gfx950 (wave64).
//
// Method: Section 3.2 (S3) of the paper - nprobe of the nlist inverted lists are selected per query and
// the product-quantised vectors inside them are compared with the query; Section 2 - the k closest are
// returned.  The retrieval latency model of S3 splits the time into an index-scan term (stages 0-1 here)
// and a vector-scan term proportional to nprobe (stages 2-3).
#include <stdlib.h>

#include <algorithm>
#include <mutex>
#include <type_traits>
#include <vector>

#include "common.h"
#include "mfma_tile.h"

using namespace piperag;

namespace {

// ------------------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------------------

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Work areas in LDS, for functions that are compiled on their own (not inlined into a kernel): there nothing says
// that a plain pointer argument points to LDS, so every access through it is a flat one - slower than an LDS
// instruction, and its completion is counted together with the global loads in flight.  Such a function converts its
// arguments to these types once.  lds_add / lds_min / lds_max take plain or LDS pointers.
typedef __attribute__((address_space(3))) uint64_t lds_u64;
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) unsigned long long lds_ull;
typedef __attribute__((address_space(3))) int64_t lds_i64;
// The same for arguments in global memory: a flat load counts as an LDS access too, so waiting for an LDS result
// would wait for every such load in flight (the gather of the keys prefetches while it writes to LDS).
typedef __attribute__((address_space(1))) uint64_t glb_u64;
typedef __attribute__((address_space(1))) int64_t glb_i64;
typedef __attribute__((address_space(1))) float glb_f32;
template <class P, class V>
__device__ __forceinline__ V lds_add(P p, V v) { return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
template <class P, class V>
__device__ __forceinline__ V lds_min(P p, V v) { return __hip_atomic_fetch_min(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
template <class P, class V>
__device__ __forceinline__ V lds_max(P p, V v) { return __hip_atomic_fetch_max(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

// Workgroup-wide selection: returns a threshold T such that exactly kth of the given keys are <= T.
// Keys equal to kSentinel are ignored; the others must be distinct and at least kth of them must exist
// (if fewer exist, kSentinel - 1 is returned: "keep all").  blockDim is a multiple of 64, >= 64.
// slack > 0: any T with between kth and kth + slack keys <= T will do (it is found in fewer rounds, mostly one).
// Method: bucket counting over the value range that still contains the kth key - 256 equal-width buckets
// over [lo, hi], starting from the actual minimum and maximum, narrowed to one bucket per round - so the
// histogram is spread over the buckets from the first round on, whatever bits the keys have in common.
// for_each_key(f) calls f(key) for every key this thread is responsible for (the threads of the workgroup
// together cover every key exactly once); it is run once per round, so keys may live in registers, LDS or
// global memory.  s_hist: 256 words, s_state: 8 words of LDS (plain or LDS pointers).
// A caller that has looked at every key already passes what the first pass would find (KeyRange: a range that
// contains all valid keys, and their number; the same values in all threads) and saves that pass.
struct KeyRange { bool known; uint64_t lo, hi; unsigned total; };
template <class ForEach, class HistPtr, class StatePtr>
__device__ uint64_t block_select_kth_each(ForEach for_each_key, int kth, HistPtr s_hist, StatePtr s_state, int slack = 0,
                                         KeyRange range = KeyRange{false, 0, 0, 0}) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    uint64_t lo = range.lo, hi = range.hi;
    unsigned total = range.total;
    for (int i = tid; i < 256; i += nt) s_hist[i] = 0;
    if (!range.known) {                                          // uniform
        // first pass: minimum, maximum and number of valid keys
        lo = kSentinel; hi = 0;
        unsigned cnt = 0;
        for_each_key([&](uint64_t key) {
            if (key != kSentinel) { lo = key < lo ? key : lo; hi = key > hi ? key : hi; ++cnt; }
        });
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const uint64_t ol = __shfl_xor(lo, off, 64), oh = __shfl_xor(hi, off, 64);
            lo = ol < lo ? ol : lo; hi = oh > hi ? oh : hi;
            cnt += __shfl_xor(cnt, off, 64);
        }
        if (tid == 0) { s_state[0] = kSentinel; s_state[1] = 0; s_state[2] = 0; }
        __syncthreads();
        if (lane == 0) {
            lds_min(&s_state[0], (unsigned long long)lo);
            lds_max(&s_state[1], (unsigned long long)hi);
            lds_add(&s_state[2], (unsigned long long)cnt);
        }
        __syncthreads();
        lo = s_state[0]; hi = s_state[1];
        total = (unsigned)s_state[2];
    }
    __syncthreads();
    if (total < (unsigned)kth) return kSentinel - 1;
    unsigned need = (unsigned)kth;          // rank of the wanted key among the keys in [lo, hi]
    for (;;) {
        const uint64_t width = hi - lo;
        const int sh = width < 256 ? 0 : (56 - __clzll((long long)width));     // (width >> sh) <= 255
        for_each_key([&](uint64_t key) {
            if (key != kSentinel && key >= lo && key <= hi) lds_add(&s_hist[(unsigned)((key - lo) >> sh)], 1u);
        });
        __syncthreads();
        if (tid < 64) {                     // wave 0: prefix sums over the 256 buckets, 4 per lane, and reset
            unsigned h[4], sum = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { h[j] = s_hist[4 * lane + j]; s_hist[4 * lane + j] = 0; sum += h[j]; }
            unsigned incl = sum;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned o = __shfl_up(incl, off, 64);
                if (lane >= off) incl += o;
            }
            unsigned before = incl - sum;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (before < need && need <= before + h[j]) {      // exactly one bucket qualifies
                    s_state[0] = (unsigned long long)(4 * lane + j);
                    s_state[1] = before;
                    s_state[2] = h[j];
                }
                before += h[j];
            }
        }
        __syncthreads();
        const unsigned bucket = (unsigned)s_state[0], below = (unsigned)s_state[1], inb = (unsigned)s_state[2];
        __syncthreads();
        need -= below;
        lo = lo + ((uint64_t)bucket << sh);
        const uint64_t bhi = lo + ((sh > 0 ? (1ull << sh) : 1ull) - 1ull);
        hi = bhi < hi ? bhi : hi;
        if (inb - need <= (unsigned)slack) return hi;   // every key of this bucket is wanted, or few enough are not: T = its upper end
        // sh == 0 means one key value per bucket, so inb == 1 == need there: the loop ends at the latest then
    }
}

// f(key) for the keys key_at(i), i = 0..n-1, shared out over the workgroup's threads; a thread reads eight of its keys
// at a time, so that the reads (LDS or global memory) overlap.  (A pass over 8,000 keys in LDS by 256 threads takes
// about 3 us either way: four wavefronts that issue one instruction per four cycles each; it is the reads from
// global memory that gain.)  Places beyond n give kSentinel, which f must ignore.
template <class KeyFn, class F>
__device__ __forceinline__ void for_each_key_of(KeyFn key_at, int n, F f) {
    const int nt = blockDim.x;
    for (int i = threadIdx.x; i < n; i += 8 * nt) {
        uint64_t key[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) key[u] = i + u * nt < n ? key_at(i + u * nt) : kSentinel;
#pragma unroll
        for (int u = 0; u < 8; ++u) f(key[u]);
    }
}

// The same for keys addressed by index: key_at(i), i = 0..n-1.
template <class KeyFn, class HistPtr, class StatePtr>
__device__ uint64_t block_select_kth(KeyFn key_at, int n, int kth, HistPtr s_hist, StatePtr s_state, int slack = 0,
                                    KeyRange range = KeyRange{false, 0, 0, 0}) {
    auto each = [&](auto f) { for_each_key_of(key_at, n, f); };
    return block_select_kth_each(each, kth, s_hist, s_state, slack, range);
}

// In-place ascending sort of n <= 64 keys in LDS by one wavefront (all 64 lanes call it): one key per lane, bitonic
// network over lane exchanges, unused lanes hold the sentinel.
__device__ void wave_sort_u64(uint64_t *keys, int n) {
    const int lane = threadIdx.x & 63;
    uint64_t key = lane < n ? keys[lane] : kSentinel;
#pragma unroll
    for (int size = 2; size <= kWave; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const uint64_t other = (uint64_t)__shfl_xor((unsigned long long)key, stride, 64);
            const bool up = (lane & size) == 0 || size == kWave, lower = (lane & stride) == 0;
            const uint64_t lo = key < other ? key : other, hi = key < other ? other : key;
            key = lower == up ? lo : hi;
        }
    }
    if (lane < n) keys[lane] = key;
}

// ------------------------------------------------------------------------------------------------
// Stage 0: coarse distances  D[q][j] = || query_q - centre_j ||^2  (direct form, fp32)
// One wavefront per JT centres at a time; the lanes split the coordinates (VEC floats per lane per 64*VEC
// chunk, so a centre row is read with contiguous wavefront loads, JT of them in flight per lane); QT queries
// of the batch are kept in LDS and share each centre read.  HBM-bound on the centre matrix.
// grid = (centre groups, ceil(nq / QT)).
// ------------------------------------------------------------------------------------------------
template <int QT, int VEC, int JT>
__global__ __launch_bounds__(256) void coarse_rowwise_kernel(const float *__restrict__ q, const float *__restrict__ cent,
                                                             float *__restrict__ D, int nq, int nlist, int d) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *s_q = reinterpret_cast<float *>(smem);  // [QT][d]
    const int q0 = blockIdx.y * QT;
    const int nqt = min(QT, nq - q0);
    for (int i = threadIdx.x; i < QT * d; i += blockDim.x) {
        const int qi = i / d;
        s_q[i] = qi < nqt ? q[(size_t)(q0 + qi) * d + (i - qi * d)] : 0.f;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwaves = gridDim.x * (blockDim.x >> 6);
    for (int j = blockIdx.x * (blockDim.x >> 6) + wave; j < nlist; j += JT * nwaves) {
        const float *row[JT];
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)            // centres past the end re-read centre j (loads stay unconditional)
            row[jt] = cent + (size_t)(j + jt * nwaves < nlist ? j + jt * nwaves : j) * d;
        float acc[JT][QT];
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int qi = 0; qi < QT; ++qi) acc[jt][qi] = 0.f;
        for (int t0 = lane * VEC; t0 < d; t0 += 64 * VEC) {
            float c[JT][VEC];
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                if (VEC == 4) {
                    const float4 v = *reinterpret_cast<const float4 *>(row[jt] + t0);
                    c[jt][0] = v.x; c[jt][1 % VEC] = v.y; c[jt][2 % VEC] = v.z; c[jt][3 % VEC] = v.w;
                } else {
                    c[jt][0] = row[jt][t0];
                }
            }
#pragma unroll
            for (int qi = 0; qi < QT; ++qi) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const float qv = s_q[qi * d + t0 + v];
#pragma unroll
                    for (int jt = 0; jt < JT; ++jt) {
                        const float diff = qv - c[jt][v];
                        acc[jt][qi] += diff * diff;
                    }
                }
            }
        }
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int qi = 0; qi < QT; ++qi) {
                const float s = wave_sum(acc[jt][qi]);
                if (lane == 0 && qi < nqt && j + jt * nwaves < nlist) D[(size_t)(q0 + qi) * nlist + j + jt * nwaves] = s;
            }
    }
}

// Coarse quantiser on the matrix cores for batches: the inner products <q, c_j>, a 64-query x 64-centre tile per
// workgroup with the fp32 MFMA tile product.  When that gives too few workgroups to fill the chip, the depth is
// split over blockIdx.z and every part writes its own partial products P[z][q][j] (summed in a fixed order by
// the selection kernel, which also adds the norms: D = |q|^2 + |c_j|^2 - 2 <q, c_j>, clamped at 0).  The
// lanes of a half-wave hold 32 consecutive centres of one query, so rows are written in contiguous runs.
// Requires d % 4 == 0, dper % 32 == 0 and 16-byte aligned rows.
// grid = (ceil(nlist / 64), ceil(nq / 64), parts).
using CoarseTile = MfmaTile<2, 2, 1, 1, 32>;

__global__ __launch_bounds__(256) void coarse_mfma_kernel(const float *__restrict__ q, int nq, const float *__restrict__ cent,
                                                          int nlist, int d, int dper, float *__restrict__ P) {
    __shared__ __align__(16) float s_mem[CoarseTile::kLdsFloats];
    const int64_t c0 = (int64_t)blockIdx.x * CoarseTile::kRowsB, q0 = (int64_t)blockIdx.y * CoarseTile::kRowsA;
    const int dbeg = blockIdx.z * dper, dlen = min(dper, d - dbeg);
    mfma_acc_t acc[1][1];
    CoarseTile::run(q + dbeg, nq, d, q0, cent + dbeg, nlist, d, c0, dlen, s_mem, acc);
    const int64_t col = c0 + CoarseTile::acc_col(0);
    float *out = P + (size_t)blockIdx.z * nq * nlist;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t row = q0 + CoarseTile::acc_row(0, r);
        if (row < nq && col < nlist) out[row * nlist + col] = acc[0][0][r];
    }
}

// ------------------------------------------------------------------------------------------------
// Stage 1: top-nprobe selection and scan plan.
// ------------------------------------------------------------------------------------------------
// Per-query part of the plan, run by the first wavefront of a workgroup: pfx[i] = number of 64-vector blocks
// in the first i probed lists (i = 0..nprobe), pblk[i] / plen[i] = first block and length of the i-th probed
// list (0 for a skipped entry), *scanned = vectors in the probed lists, *thr = "no bound yet" for the scan's
// shared threshold, *qdone = 0 for the scan's count of finished workgroups.  probe_at(i) gives the i-th probed list or -1.
struct PlanOut {
    int32_t *pfx, *pblk, *plen;
    int64_t *scanned;
    uint32_t *thr;
    float *pcst;                 // residual indexes: |c_l|^2 - 2 <q, c_l> per probe (NULL otherwise)
    uint32_t *qdone;             // scan workgroups (or groups of them) of the query that have finished
};
__device__ __forceinline__ PlanOut plan_of_query(const PlanOut &all, int qi, int probe_stride) {
    return PlanOut{all.pfx + (size_t)qi * (probe_stride + 1), all.pblk + (size_t)qi * probe_stride,
                   all.plen + (size_t)qi * probe_stride, all.scanned + qi, all.thr + qi,
                   all.pcst ? all.pcst + (size_t)qi * probe_stride : nullptr, all.qdone + qi};
}
template <class ProbeFn>
__device__ void plan_query(ProbeFn probe_at, int nprobe, const int32_t *__restrict__ list_blk,
                           const int32_t *__restrict__ list_len, const PlanOut o) {
    int32_t *pfx = o.pfx;
    if (threadIdx.x >= 64) return;
    const int lane = threadIdx.x;
    int32_t running = 0;
    int64_t vecs = 0;
    for (int base = 0; base < nprobe; base += 64) {
        const int i = base + lane;
        const int32_t l = i < nprobe ? probe_at(i) : -1;
        const int32_t nb = l >= 0 ? list_blk[l + 1] - list_blk[l] : 0;
        int64_t len = l >= 0 ? list_len[l] : 0;
        int32_t incl = nb;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int32_t o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        if (i < nprobe) {
            pfx[i] = running + incl - nb;
            o.pblk[i] = l >= 0 ? list_blk[l] : 0;
            o.plen[i] = (int32_t)len;
        }
        running += __shfl(incl, 63, 64);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) len += __shfl_xor(len, off, 64);
        vecs += len;
    }
    if (lane == 0) { pfx[nprobe] = running; *o.scanned = vecs; *o.thr = 0xFFFFFFFFu; *o.qdone = 0; }
}

// Residual indexes, probe lists given by the caller: pcst[q][i] = |c_l|^2 - 2 <q, c_l> for l = the i-th probe
// (0 for a skipped entry).  One wavefront per (probe, query).
__global__ __launch_bounds__(64) void probe_const_kernel(const float *__restrict__ q, const float *__restrict__ cent,
                                                         const float *__restrict__ cn, int d,
                                                         const int32_t *__restrict__ probe, int probe_stride,
                                                         float *__restrict__ pcst) {
    const int qi = blockIdx.y, i = blockIdx.x, lane = threadIdx.x;
    const int32_t l = probe[(size_t)qi * probe_stride + i];
    float acc = 0.f;
    if (l >= 0)
        for (int t = lane; t < d; t += 64) acc += q[(size_t)qi * d + t] * cent[(size_t)l * d + t];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) pcst[(size_t)qi * probe_stride + i] = l >= 0 ? cn[l] - 2.f * acc : 0.f;
}

// Shares the scan workgroups out over the queries (one workgroup): query q gets
// S_q = clamp(ceil(TB_q / per), 1, kMaxSegments) segments, TB_q = its number of blocks and
// per = the smallest number of blocks for which these fit the budget of workgroups (found by bisection; about
// sum of TB / target), so that every workgroup scans about the same number of blocks whatever
// the lengths of the lists a query probes.  seg0[q] = first workgroup of query q (seg0[nq] = workgroups in
// use, at most max(target, nq)); desc[w] = (query, number of the workgroup among the query's, their count,
// chunk counters in use) of workgroup w; desc of spare workgroups has query -1.  A workgroup gets at least
// kMinBlocksPerWG blocks on average (unless its query has fewer), so that small searches are not spread over
// needlessly many workgroups.
constexpr int kShareLdsQueries = 1024;
constexpr int kChunkBlocks = 4;                       // blocks a scan wave works through per turn of its loop; a chunk is 1, 2, 4 or 8 turns
struct ShareOut {
    int32_t *seg0;
    int4 *desc;
    uint32_t *ctr;
    uint32_t *gdone;            // [workgroups] finished workgroups per group of workgroups (zeroed here)
    int fan;                    // workgroups whose keys one selection can merge (more per query: a second level, ~9 us)
};
constexpr int kSoftBlocksPerWG = 64;   // a query that would get a few more workgroups than `fan` gets `fan`, up to this many blocks each

// The sharing itself, by the first 256 threads of the calling workgroup (all of its threads must call it: it
// has barriers).  blocks_of(q) = number of blocks of query q.
template <class BlocksOf>
__device__ void share_plan(BlocksOf blocks_of, int nq, int target, int max_wg, ShareOut o) {
    __shared__ long long s_total;
    __shared__ int32_t s_scan[256];
    __shared__ int32_t s_carry;
    __shared__ int32_t s_seg0[kShareLdsQueries + 1];      // copy of seg0 for the search below (batches up to this size)
    const bool seg_in_lds = nq <= kShareLdsQueries;
    const int tid = threadIdx.x;
    const bool act = tid < 256;
    if (tid == 0) { s_total = 0; s_carry = 0; }
    __syncthreads();
    const long long first_tb = act && tid < nq ? blocks_of(tid) : 0;   // kept for the second use below
    long long mine = first_tb;
    if (act)
        for (int q = tid + 256; q < nq; q += 256) mine += blocks_of(q);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
    if (act && (tid & 63) == 0) atomicAdd(reinterpret_cast<unsigned long long *>(&s_total), (unsigned long long)mine);
    __syncthreads();
    // Workgroups of a query with tb blocks when a workgroup is to take `per` blocks.
    auto segments = [&](long long tb, long long per) -> int32_t {
        int32_t sq = (int32_t)min((long long)kMaxSegments, max(1ll, (tb + per - 1) / per));
        // a small scan spread over a few more workgroups than one selection merges would pay a second merge
        // level for nothing
        if (sq > o.fan && tb <= (long long)o.fan * kSoftBlocksPerWG) sq = o.fan;
        return sq;
    };
    // sum of ceil(TB_q / per) <= total / per + nq, so dividing by (target - nq) keeps the sum within target
    const long long denom = max(1, target - nq);
    long long per = max((long long)kMinBlocksPerWG, (s_total + denom - 1) / denom);
    // That bound leaves up to nq workgroups unused and the queries' shares uneven (a query just above a multiple of
    // `per` has workgroups with little to do; the launch lasts as long as the fullest workgroup: at 64 queries on 480 of
    // 512 workgroups the fullest had 14 % more than an even share).  The smallest `per` whose segments still fit the
    // budget is found by bisection between the even share and that bound, to 1/64 (at most a dozen counts).
    if (seg_in_lds) {
        const long long budget = max(target, nq);
        if (act)
            for (int q = tid; q < nq; q += 256) s_seg0[q] = (int32_t)min(0x7FFFFFFFll, q < 256 ? first_tb : blocks_of(q));
        long long lo = max((long long)kMinBlocksPerWG, (s_total + budget - 1) / budget), hi = per;
        while (hi - lo > (hi >> 6)) {                          // uniform; hi always fits the budget
            const long long mid = (lo + hi) >> 1;
            __syncthreads();                                   // s_seg0 written; the last count read
            if (tid == 0) s_carry = 0;
            __syncthreads();
            int32_t c = 0;
            if (act)
                for (int q = tid; q < nq; q += 256) c += segments(s_seg0[q], mid);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
            if (act && (tid & 63) == 0) atomicAdd(&s_carry, c);
            __syncthreads();
            if (s_carry <= budget) hi = mid; else lo = mid + 1;
        }
        per = hi;
        __syncthreads();
        if (tid == 0) s_carry = 0;
        __syncthreads();
    }
    for (int q0 = 0; q0 < nq; q0 += 256) {
        const int q = q0 + tid;
        int32_t sq = 0;
        if (act && q < nq) {
            const long long tb = q0 == 0 ? first_tb : blocks_of(q);
            sq = segments(tb, per);
        }
        int32_t incl = sq;                                 // inclusive scan: within the wave, then over the four waves
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int32_t up = __shfl_up(incl, off, 64);
            if ((tid & 63) >= off) incl += up;
        }
        if (act && (tid & 63) == 63) s_scan[tid >> 6] = incl;
        __syncthreads();
        const int32_t base = s_carry;
        int32_t before = 0;
        for (int w = 0; w < (tid >> 6) && w < 4; ++w) before += s_scan[w];
        if (act && q < nq) {
            o.seg0[q] = base + before + incl - sq;
            if (seg_in_lds) s_seg0[q] = base + before + incl - sq;
        }
        __syncthreads();
        if (tid == 255) s_carry = base + before + incl;
        __syncthreads();
    }
    if (tid == 0) { o.seg0[nq] = s_carry; if (seg_in_lds) s_seg0[nq] = s_carry; }
    __syncthreads();
    // (typed pointers: a choice between two plain pointers would be made first and the load through it be a flat one)
    typedef __attribute__((address_space(3))) const int32_t lds_ci32;
    typedef __attribute__((address_space(1))) const int32_t glb_ci32;
    lds_ci32 *const seg_lds = (lds_ci32 *)s_seg0;
    glb_ci32 *const seg_glb = (glb_ci32 *)o.seg0;
    auto seg_at = [&](int i) { return seg_in_lds ? seg_lds[i] : seg_glb[i]; };
    const int total_wg = s_carry;
    if (!act) return;
    for (int w = tid; w < max_wg; w += 256) o.gdone[w] = 0;
    for (int w = tid; w < max_wg; w += 256) {
        if (w >= total_wg) { o.desc[w] = int4{-1, 0, 0, 0}; continue; }
        int lo = 0, hi = nq;                               // query of workgroup w: last q with seg0[q] <= w
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (seg_at(mid) <= w) lo = mid; else hi = mid;
        }
        const int seg = w - seg_at(lo), S = seg_at(lo + 1) - seg_at(lo);
        // The query's chunks are dealt to P counters (chunk c belongs to counter c mod P) and its waves likewise
        // (wave g of the query draws from counter g mod P), so that the additions of a query with many
        // workgroups do not all queue up at one address.  Every wave starts on the chunk of its own number;
        // counter p then hands out P * v + p for v = the number of starting chunks it covers, and up.
        const int W = S * kScanWaves, P = min(kCtrPerQuery, max(1, S / 4));
        // Length of the query's chunks, 4 << lg blocks: a chunk must outlast the round trip of the counter addition
        // that fetches the next one (8 blocks do, 4 do not: 16 queries at 4,096 lists scanned 30 % faster with 8), and
        // longer chunks read longer runs of memory (32 blocks, 128 KiB with 64-byte codes: +6 % at 64 queries on
        // 16 GiB of codes) - as long as every wave still gets several of them, or the last chunks decide when the
        // query ends (one query over 512 workgroups: 8 blocks best, 32 blocks 13 % slower), and none when a wave has
        // fewer than 8 blocks to scan in all.
        const long long tbq = blocks_of(lo), per_wave = tbq / W;
        const int lg = per_wave < 8 ? 0 : (per_wave < 64 ? 1 : (per_wave < 128 ? 2 : 3));
        // The query's last W chunks' worth of blocks are handed out in chunks of kChunkBlocks instead: the query is over
        // when the wave that took the last chunk is through with it, and with whole chunks to the end the other waves
        // waited for it about a chunk's time (8 blocks: 10 to 14 us of a 64-query scan that takes 100; afterwards 3 to
        // 5).  full = number of chunks of full length, counted from the front.  Only where a wave gets four full chunks
        // at least: 16 queries at 4,096 lists, 15 blocks per wave, took 79 instead of 63 us with half of their blocks
        // in short chunks.
        const long long len = (long long)kChunkBlocks << lg;
        const int full = per_wave < 32 ? 0x3FFFFFFF : (int)min(0x3FFFFFFFll, max(0ll, tbq / len - W));
        o.desc[w] = int4{lo, seg | (S << 16), full, P | (lg << 8)};
        if (seg == 0)
            for (int c = 0; c < P; ++c) o.ctr[((size_t)lo * kCtrPerQuery + c) * kCtrStride] = (uint32_t)((W - c + P - 1) / P);
    }
}

// As a kernel of its own (one workgroup of 256 threads), for plans made by copy_probes_kernel.
__global__ __launch_bounds__(256) void share_kernel(const int32_t *__restrict__ pfx, int probe_stride, int nprobe, int nq,
                                                    int target, int max_wg, ShareOut o) {
    auto blocks_of = [&](int q) { return (long long)pfx[(size_t)q * (probe_stride + 1) + nprobe]; };
    share_plan(blocks_of, nq, target, max_wg, o);
}

// Keys that one workgroup writes and another reads within the same launch go through device-scope atomic
// stores and loads (they bypass the per-XCD caching that is not coherent across the chip), ordered by
// publish_keys(): wait until this thread's stores are acknowledged, then meet the workgroup; a counter
// increment after that tells the others.  No cache-wide write-back or invalidation is involved (a full fence
// by every finishing workgroup costs far more than the merge itself).
// (plain pointers, or pointers that name the global address space: see glb_u64)
template <class P>
__device__ __forceinline__ void store_key(P p, uint64_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <class P>
__device__ __forceinline__ uint64_t load_key(P p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void publish_keys() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): loads and stores of this thread are complete
    __syncthreads();
}

// Per query, the nprobe smallest D[q][.] ordered by (distance, list), then the query's plan.  G workgroups of NT
// threads per query (512 for slices of up to 8,192 distances, 1024 for longer ones), each with a slice of the
// row: it finishes the slice's distances (partial products summed in a fixed order, norms added), stages them in
// LDS, and selects the slice's min(nprobe, length) smallest keys (distance bits << 32 | list; distances are >= 0,
// so their bit patterns order like the values).  G = 1: those are the probes.  G > 1 (small batches, so that the
// selection is spread over the chip, and rows longer than the LDS staging): the slice's keys go to the query's
// candidate list, and the query's last workgroup to finish (a ticket per query) selects among the G * nprobe
// candidates.  The probes are then sorted, written out, and turned into the query's plan; the workgroup that
// finishes the last query shares the scan workgroups out over the queries (saves a launch).
constexpr int kSelThreads = 512;            // slices of up to kSelSmallRow distances
constexpr int kSelThreadsLong = 1024;       // longer slices (measured on whole rows: 1024 threads are 8 us faster at 16,384 distances, 4 us slower at 4,096)
constexpr int kSelSmallRow = 8192;
constexpr int kSelMaxLdsRow = 32768;        // distances that fit the LDS staging (128 KiB); also the keys of a second-level selection (8 bytes each, half as many)
// Measured (selection kernel, us, nprobe 32; one query / 64 queries): whole rows of 4,096 distances 12.8 / 20.4, of
// 16,384 21.9 / 23.4, of 65,536 (two slices at least) 33.5 / 40.6; slices of 2,048: 16.6 / 21.6, 18.3 / 21.5, 18.6 / 30.2.
// Every selection costs a dozen barrier-separated steps whatever its size, so slicing pays only for long rows.
constexpr int kSelMinSlice = 4096;          // a slice is at least this long
constexpr int kSelTargetWGs = 2048;         // batches get up to this many selection workgroups in all
constexpr int kSelSecondLevel = 4096;       // ... as long as the second level has no more candidates than this (its cost is theirs)

// Workgroups per query for a batch (host and workspace sizing use the same rule).
inline int select_groups(int nlist, int nq, int nprobe, int ncu) {
    const int need = (nlist + kSelMaxLdsRow - 1) / kSelMaxLdsRow;                  // so that a slice fits the staging
    const int np2 = nprobe <= 2 ? 2 : 1 << (32 - __builtin_clz((unsigned)(nprobe - 1)));
    const int cap = std::max(1, std::min(std::min(kSelSecondLevel / np2, nlist / kSelMinSlice), 64));   // second level stays small; slices not too short
    return std::max(need, std::min(cap, std::min(kSelTargetWGs, 8 * ncu) / std::max(1, nq)));
}

template <int NT>
__global__ __launch_bounds__(NT) void select_probes_kernel(const float *__restrict__ D, int nparts, int nq, int G, int slice_len,
                                                           int cand_in_lds, const float *__restrict__ q, int d,
                                                           const float *__restrict__ cn, int nlist, int nprobe,
                                                           int32_t *__restrict__ probe, float *__restrict__ probe_d,
                                                           int probe_stride, const int32_t *__restrict__ list_blk,
                                                           const int32_t *__restrict__ list_len, PlanOut plan,
                                                           uint64_t *__restrict__ selcand, uint32_t *__restrict__ qticket,
                                                           uint32_t *__restrict__ tb, uint32_t *__restrict__ arrived,
                                                           int target, int max_wg, ShareOut share) {
    extern __shared__ __align__(16) unsigned char sel_smem[];
    __shared__ unsigned s_ticket;
    __shared__ unsigned s_hist[256];
    __shared__ unsigned long long s_state[8];
    __shared__ uint64_t s_keys[kMaxNprobe];
    __shared__ unsigned s_count;
    __shared__ float s_qpart[NT / kWave];
    const int qi = blockIdx.x / G, g = blockIdx.x - qi * G, tid = threadIdx.x;
    const int i_beg = g * slice_len, i_end = min(nlist, i_beg + slice_len), len = max(0, i_end - i_beg);
    const float *grow = D + (size_t)qi * nlist;              // the query's row of distances (of part 0, with parts)
    const int np2 = max(2, 1 << (32 - __clz(nprobe - 1)));   // next power of two >= nprobe (>= 2)
    for (int i = tid; i < np2; i += NT) s_keys[i] = kSentinel;
    if (tid == 0) s_count = 0;
    // Inner product with centre i from the parts, summed in order.  With several parts all kCoarseMaxParts loads
    // are made whatever their number (a missing part re-reads the last one and counts as +0), so that the loads
    // of several centres can be in flight together.
    const size_t part_stride = (size_t)nq * nlist;
    auto dot_of = [&](int i) -> float {
        float dot = grow[i];
        if (nparts > 1) {                                    // uniform
#pragma unroll
            for (int p = 1; p < kCoarseMaxParts; ++p) {
                const float v = grow[(size_t)min(p, nparts - 1) * part_stride + i];
                dot += p < nparts ? v : 0.f;
            }
        }
        return dot;
    };
    // the first sweep's products and centre norms are requested before the query's norm is reduced (one memory
    // round trip instead of two)
    constexpr int US = 8;
    float pd[US], pc[US];
    if (nparts > 0) {
#pragma unroll
        for (int u = 0; u < US; ++u) {
            const int i = i_beg + tid + u * NT;
            pd[u] = i < i_end ? dot_of(i) : 0.f;
            pc[u] = i < i_end ? cn[i] : 0.f;
        }
    }
    float qn = 0.f;
    if (nparts > 0 || plan.pcst) {                           // D holds partial inner products, or a residual index: the query's norm
        float part = 0.f;
        for (int t = tid; t < d; t += NT) { const float v = q[(size_t)qi * d + t]; part += v * v; }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
        if ((tid & 63) == 0) s_qpart[tid >> 6] = part;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NT / kWave; ++w) qn += s_qpart[w];    // the same order in every thread
    }
    auto finish = [&](float dot, float cnorm) -> float { return fmaxf(0.f, qn + cnorm - 2.f * dot); };
    uint32_t *s_row = reinterpret_cast<uint32_t *>(sel_smem);    // the slice's distance bits
    const uint32_t *drow = reinterpret_cast<const uint32_t *>(grow);
    for (int i0 = tid; i0 < len; i0 += US * NT) {
        uint32_t v[US];
        if (nparts > 0 && i0 != tid) {                       // later sweeps (uniform)
#pragma unroll
            for (int u = 0; u < US; ++u) {
                const int i = i_beg + i0 + u * NT;
                pd[u] = i < i_end ? dot_of(i) : 0.f;
                pc[u] = i < i_end ? cn[i] : 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < US; ++u) {
            const int i = i_beg + i0 + u * NT;
            v[u] = nparts > 0 ? __float_as_uint(finish(pd[u], pc[u])) : (i < i_end ? drow[i] : 0u);
        }
#pragma unroll
        for (int u = 0; u < US; ++u)
            if (i0 + u * NT < len) s_row[i0 + u * NT] = v[u];
    }
    __syncthreads();
    if (len > 0) {   // first level: the slice's min(nprobe, len) smallest keys (uniform)
        auto key_at = [&](int i) { return ((uint64_t)s_row[i] << 32) | (uint32_t)(i_beg + i); };
        const uint64_t T = block_select_kth(key_at, len, min(nprobe, len), s_hist, s_state);
        for (int i = tid; i < len; i += NT) {
            const uint64_t key = key_at(i);
            if (key <= T) {                                  // exactly min(nprobe, len) keys qualify (keys are distinct)
                const unsigned slot = atomicAdd(&s_count, 1u);
                if (slot < (unsigned)np2) s_keys[slot] = key;
            }
        }
        __syncthreads();
    }
    if (G > 1) {                                             // uniform
        // the slice's keys (padded with the sentinel) join the query's candidates; the last slice to arrive goes on
        uint64_t *mine = selcand + ((size_t)qi * G + g) * nprobe;
        for (int i = tid; i < nprobe; i += NT) store_key(mine + i, s_keys[i]);
        publish_keys();
        if (tid == 0) s_ticket = atomicAdd(&qticket[qi], 1u);
        __syncthreads();
        if (s_ticket != (unsigned)(G - 1)) return;          // uniform
        if (tid == 0) { __hip_atomic_store(&qticket[qi], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); s_count = 0; }
        // G * nprobe candidates: in LDS when they fit there (the slice is no longer needed), else where they are
        uint64_t *s_cand = reinterpret_cast<uint64_t *>(sel_smem);
        const uint64_t *all = selcand + (size_t)qi * G * nprobe;
        const int ncand = G * nprobe;
        const bool in_lds = cand_in_lds != 0;                // uniform
        if (in_lds) {
            for (int i0 = tid; i0 < ncand; i0 += 8 * NT) {   // 8 loads in flight per thread
                uint64_t key[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) key[u] = i0 + u * NT < ncand ? load_key(all + i0 + u * NT) : kSentinel;
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (i0 + u * NT < ncand) s_cand[i0 + u * NT] = key[u];
            }
        }
        for (int i = tid; i < np2; i += NT) s_keys[i] = kSentinel;
        __syncthreads();
        auto cand_at = [&](int i) { return in_lds ? s_cand[i] : load_key(all + i); };
        const uint64_t T = block_select_kth(cand_at, ncand, nprobe, s_hist, s_state);
        for (int i = tid; i < ncand; i += NT) {
            const uint64_t key = cand_at(i);
            if (key <= T && key != kSentinel) {              // exactly nprobe keys qualify (nprobe <= nlist)
                const unsigned slot = atomicAdd(&s_count, 1u);
                if (slot < (unsigned)np2) s_keys[slot] = key;
            }
        }
        __syncthreads();
    }
    if (np2 <= kWave) {                                      // uniform: up to 64 probes are sorted in the registers of one wave
        if (tid < kWave) wave_sort_u64(s_keys, np2);
        __syncthreads();
    } else {
        // More: every key's place is the number of keys below it (the keys are all different), counted with reads
        // that all lanes make at the same LDS address - one pass instead of the 36 to 55 barrier-separated steps of
        // a bitonic network.  The sorted keys pass through the dynamic LDS (free by now, at least 8 * np2 bytes).
        uint64_t *s_sorted = reinterpret_cast<uint64_t *>(sel_smem);
        __syncthreads();
        for (int i = tid; i < nprobe; i += NT) {
            const uint64_t key = s_keys[i];
            int below = 0;
            for (int j0 = 0; j0 < nprobe; j0 += 8) {
                uint64_t other[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) other[u] = s_keys[min(j0 + u, nprobe - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u) below += (j0 + u < nprobe && other[u] < key) ? 1 : 0;
            }
            s_sorted[below] = key;
        }
        __syncthreads();
        for (int i = tid; i < nprobe; i += NT) s_keys[i] = s_sorted[i];
        __syncthreads();
    }
    for (int i = tid; i < nprobe; i += NT) {
        probe[(size_t)qi * probe_stride + i] = (int32_t)(s_keys[i] & 0xFFFFFFFFu);
        probe_d[(size_t)qi * probe_stride + i] = __uint_as_float((uint32_t)(s_keys[i] >> 32));
    }
    auto probe_at = [&](int i) { return (int32_t)(s_keys[i] & 0xFFFFFFFFu); };
    const PlanOut mine = plan_of_query(plan, qi, probe_stride);
    if (mine.pcst)                                           // |q - c|^2 - |q|^2 = |c|^2 - 2 <q, c>
        for (int i = tid; i < nprobe; i += NT) mine.pcst[i] = __uint_as_float((uint32_t)(s_keys[i] >> 32)) - qn;
    plan_query(probe_at, nprobe, list_blk, list_len, mine);
    // The workgroup that finishes the last query shares the scan workgroups out over the queries (saves a launch):
    // every query's workgroup publishes its number of blocks with a device-scope store, waits for it to complete
    // and adds itself to a counter; the last one reads all the numbers and resets the counter for the next search.
    // A single query has nobody to wait for (two round trips to memory less).
    __syncthreads();
    if (nq == 1) {                                           // uniform
        if (tid == 0) s_ticket = (unsigned)mine.pfx[nprobe];
        __syncthreads();
        const long long my_blocks = s_ticket;
        auto blocks_of = [&](int) { return my_blocks; };
        share_plan(blocks_of, 1, target, max_wg, share);
        return;
    }
    if (tid == 0) {
        __hip_atomic_store(&tb[qi], (uint32_t)mine.pfx[nprobe], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
        s_ticket = atomicAdd(arrived, 1u);
    }
    __syncthreads();
    if (s_ticket != (unsigned)(nq - 1)) return;             // uniform
    auto blocks_of = [&](int qq) { return (long long)__hip_atomic_load(&tb[qq], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    share_plan(blocks_of, nq, target, max_wg, share);
    if (tid == 0) __hip_atomic_store(arrived, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Probe lists given by the caller: entries outside 0..nlist-1 and repeats of an earlier entry become -1
// (skipped), so that no list is scanned twice.  Then the query's plan.
__global__ __launch_bounds__(64) void copy_probes_kernel(const int32_t *__restrict__ src, int nprobe, int nlist,
                                                         int32_t *__restrict__ dst, int probe_stride,
                                                         const int32_t *__restrict__ list_blk,
                                                         const int32_t *__restrict__ list_len, PlanOut plan) {
    const int qi = blockIdx.x;
    const int32_t *row = src + (size_t)qi * nprobe;
    int32_t *out = dst + (size_t)qi * probe_stride;
    for (int i = threadIdx.x; i < nprobe; i += blockDim.x) {
        int32_t l = row[i];
        if (l < 0 || l >= nlist) l = -1;
        for (int e = 0; e < i && l >= 0; ++e)
            if (row[e] == l) l = -1;
        out[i] = l;
    }
    __syncthreads();
    auto probe_at = [&](int i) { return out[i]; };
    plan_query(probe_at, nprobe, list_blk, list_len, plan_of_query(plan, qi, probe_stride));
}

// ------------------------------------------------------------------------------------------------
// Stage 2 and 3 share the scan machinery below.
// ------------------------------------------------------------------------------------------------
struct ScanArgs {
    const uint8_t *codes;
    const float *lut;          // [nq][256][Mp]
    const int32_t *pfx;        // [nq][probe_stride+1] block prefix sums of the probed lists
    const int32_t *pblk;       // [nq][probe_stride] first block of each probed list
    const int32_t *plen;       // [nq][probe_stride] length of each probed list
    const float *pcst;         // residual indexes: [nq][probe_stride] constant of each probed list
    const float *tx;           // residual indexes: [slots] term of each stored vector
    uint64_t *part;            // [workgroups][KW] result lists of the queries
    uint32_t *thr;             // [nq] bound on the k-th best distance (bits)
    const int4 *desc;          // [workgroups] (query, number among the query's workgroups, their count, counters in use); query -1: spare
    uint32_t *ctr;             // [nq * kCtrPerQuery * kCtrStride] chunk counters of each query
    int nprobe, probe_stride, k, KW;
    int cap;                   // slots of the workgroup's candidate buffer
    // Result of a query: its workgroups write the keys they still hold at the end to one list (KW slots per
    // workgroup, in `part` from the query's first workgroup on), and the last of them to finish selects the k best
    uint32_t *qdone;           // [nq] workgroups, or groups, of the query that have finished (zeroed by the plan)
    int room;                  // keys that fit the LDS of a selection
    // a query with more than `fan` workgroups collects its keys per group of fan consecutive workgroups first
    int fan;
    uint32_t *gdone;           // [workgroups] finished workgroups of a group, at the group's first workgroup (zeroed by the plan)
    uint64_t *part2;           // [workgroups][KW] the queries' lists when there are groups (the groups' lists are in part)
    const int64_t *ids;
    float *out_d;
    int64_t *out_i;
};

typedef const __attribute__((address_space(3))) float *lds_cfptr;

constexpr int kKeepSlack = 64;                        // pruning keeps between k and k + kKeepSlack candidates
constexpr int kCandRoom = 1472;                       // candidate slots beyond k + kKeepSlack, at most
constexpr int kCandRoomMin = 512;                     // and at least (the scan needs more than kScanThreads)
constexpr int kCandPerThread = (kMaxK + kKeepSlack + kCandRoom + kScanThreads - 1) / kScanThreads;

// LDS carve-up of the scan kernel (all dynamic, so that the table starts at address 0)
struct ScanLds {
    float *lut;                  // [256*Mp]
    uint64_t *cand;              // [cap]
    unsigned long long *state;   // [8]
    unsigned *hist;              // [256]
    unsigned *misc;              // [8]: 0 count, 1 min distance bits, 2 max distance bits, 3 waves done
    int32_t *pfx, *blk, *len;    // probe tables [nprobe+1], [nprobe], [nprobe]
    float *cst;                  // [nprobe] residual indexes: constant of each probed list
};
__device__ __forceinline__ ScanLds carve_lds(unsigned char *smem, int Mp, int cap, int nprobe) {
    ScanLds s;
    s.lut = reinterpret_cast<float *>(smem);
    s.cand = reinterpret_cast<uint64_t *>(smem + (size_t)1024 * Mp);
    s.state = reinterpret_cast<unsigned long long *>(s.cand + cap);
    s.hist = reinterpret_cast<unsigned *>(s.state + 8);
    s.misc = s.hist + 256;
    s.pfx = reinterpret_cast<int32_t *>(s.misc + 8);
    s.blk = s.pfx + (nprobe + 1);
    s.len = s.blk + nprobe;
    s.cst = reinterpret_cast<float *>(s.len + nprobe);
    return s;
}
size_t scan_lds_bytes(int Mp, int cap, int nprobe) {
    return (size_t)1024 * Mp + sizeof(uint64_t) * ((size_t)cap + 8) + sizeof(unsigned) * (256 + 8) +
           sizeof(int32_t) * (4 * (size_t)nprobe + 1);
}

// Distance of this lane's vector of one block, any Mp: table index = byte * Mp + (lane + t) mod Mp.
template <int C>
__device__ __forceinline__ float block_dist_generic(const uint4 (&w)[C], const float *s_lut, int lane_m) {
    constexpr int MP = 16 * C;
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const uint32_t ww[4] = {w[c].x, w[c].y, w[c].z, w[c].w};
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            int m = lane_m + c * 16 + u;
            if (m >= MP) m -= MP;
            const uint32_t byte = (ww[u >> 2] >> (8 * (u & 3))) & 0xFFu;
            const float v = s_lut[byte * MP + m];
            if ((u & 3) == 0) acc0 += v; else if ((u & 3) == 1) acc1 += v; else if ((u & 3) == 2) acc2 += v; else acc3 += v;
        }
    }
    return (acc0 + acc1) + (acc2 + acc3);
}

// Mp = 64 with the table at LDS address 0.  The LDS byte address of lookup t is (code byte << 8) | off(t) with
// off(t) = ((lane + t) mod 64) * 4 < 256, so four consecutive off values fit one register (off4[t / 4], byte
// t % 4) and a single byte permute assembles the address from the code word and that register.
__device__ __forceinline__ float block_dist_m64(const uint4 (&w)[4], const uint32_t (&off4)[16]) {
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t ww[4] = {w[c].x, w[c].y, w[c].z, w[c].w};
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            // result bytes: [0] = byte (u & 3) of off4, [1] = byte (u & 3) of the code word, [2] = [3] = 0
            const uint32_t n = (uint32_t)(u & 3);
            const uint32_t addr = __builtin_amdgcn_perm(ww[u >> 2], off4[c * 4 + (u >> 2)], 0x0c0c0400u + (n << 8) + n);
            const float v = *reinterpret_cast<lds_cfptr>(static_cast<uintptr_t>(addr));
            if (n == 0) acc0 += v; else if (n == 1) acc1 += v; else if (n == 2) acc2 += v; else acc3 += v;
        }
    }
    return (acc0 + acc1) + (acc2 + acc3);
}

__device__ __forceinline__ void make_off4(uint32_t (&off4)[16], int lane) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        off4[i] = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) off4[i] |= ((uint32_t)((lane + 4 * i + j) & 63) << 2) << (8 * j);
    }
}

// Appends the passing lanes' candidates of one block to the workgroup's buffer.
__device__ __forceinline__ void append_candidates(bool pass, uint32_t dbits, uint32_t slot_id, uint64_t *s_cand,
                                                  unsigned *s_count, int cap, int lane) {
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return;
    unsigned base = 0;
    if (lane == 0) base = atomicAdd(s_count, (unsigned)__popcll(mask));
    base = __builtin_amdgcn_readfirstlane(base);
    if (pass) {
        const unsigned slot = base + (unsigned)__popcll(mask & ((1ull << lane) - 1ull));
        if (slot < (unsigned)cap)      // always true (see the callers' capacity argument); guards against logic errors
            s_cand[slot] = ((uint64_t)dbits << 32) | (uint64_t)slot_id;
    }
}

// Prunes the candidate buffer s_cand[0..n), n > k: keeps every key <= T, where the key T is chosen so that
// between k and k + kKeepSlack keys remain, and returns T.  Keys are (distance bits << 32 | slot) and all
// different, so nothing that could be among the k best by (distance, slot) is dropped; no sorting is done.  T
// is found by bucket counting over [min key, max key], narrowed to one of 256 buckets per round: the first
// rounds split by distance, and only if more than the slack allows share one distance do later rounds split
// by slot (8 rounds reach single keys).  Whole workgroup (at least kScanThreads threads), called with all
// threads at the same point; *s.misc (the count) becomes the number kept.
__device__ uint64_t wg_prune(const ScanLds s, int n, int k) {
    const int tid = threadIdx.x, lane = tid & 63, nt = blockDim.x;
    uint64_t mine[kCandPerThread];
    // range of the keys: from the smallest and the largest distance (32-bit lane exchanges instead of 64-bit ones)
    uint32_t dmin = 0xFFFFFFFFu, dmax = 0;
#pragma unroll
    for (int e = 0; e < kCandPerThread; ++e) {
        const int i = tid + e * nt;
        mine[e] = kSentinel;
        if (e * nt < n) {                   // uniform: rounds of the buffer beyond its fill are skipped
            if (i < n) {
                mine[e] = s.cand[i];
                const uint32_t dd = (uint32_t)(mine[e] >> 32);
                dmin = min(dmin, dd); dmax = max(dmax, dd);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        dmin = min(dmin, (uint32_t)__shfl_xor(dmin, off, 64));
        dmax = max(dmax, (uint32_t)__shfl_xor(dmax, off, 64));
    }
    if (tid == 0) { s.state[3] = ~0ull; s.state[4] = 0; }
    for (int i = tid; i < 256; i += nt) s.hist[i] = 0;
    __syncthreads();
    if (lane == 0) {
        atomicMin(&s.state[3], (unsigned long long)dmin << 32);
        atomicMax(&s.state[4], ((unsigned long long)dmax << 32) | 0xFFFFFFFFull);
    }
    __syncthreads();
    uint64_t lo = s.state[3], hi = s.state[4];
    unsigned need = (unsigned)k, kept_below = 0;
    uint64_t T = hi;
    for (int round = 0; round < 8; ++round) {
        const uint64_t width = hi - lo;
        const int sh = width < 256 ? 0 : (56 - __clzll((long long)width));   // (width >> sh) <= 255
#pragma unroll
        for (int e = 0; e < kCandPerThread; ++e)
            if (e * nt < n && mine[e] != kSentinel && mine[e] >= lo && mine[e] <= hi)
                atomicAdd(&s.hist[(unsigned)((mine[e] - lo) >> sh)], 1u);
        __syncthreads();
        if (tid < 64) {                     // wave 0: prefix sums over the 256 buckets, 4 per lane, and reset
            unsigned h[4], sum = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { h[j] = s.hist[4 * lane + j]; s.hist[4 * lane + j] = 0; sum += h[j]; }
            unsigned incl = sum;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned o = __shfl_up(incl, off, 64);
                if (lane >= off) incl += o;
            }
            unsigned before = incl - sum;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (before < need && need <= before + h[j]) {      // the bucket that holds the need-th key
                    s.state[0] = (unsigned long long)(4 * lane + j);
                    s.state[1] = before;
                    s.state[2] = h[j];
                }
                before += h[j];
            }
        }
        __syncthreads();
        const unsigned bucket = (unsigned)s.state[0], before = (unsigned)s.state[1], inb = (unsigned)s.state[2];
        __syncthreads();
        const uint64_t blo = lo + ((uint64_t)bucket << sh);
        const uint64_t edge = min(hi, blo + (((uint64_t)1 << sh) - 1u));
        T = edge;
        // keeping the whole bucket is within the slack (always so once a bucket is a single key)
        if (kept_below + before + inb <= (unsigned)(k + kKeepSlack) || sh == 0) break;
        kept_below += before; need -= before; lo = blo; hi = edge;       // look inside the bucket
    }
    if (tid == 0) s.misc[0] = 0;
    __syncthreads();
    // the kept keys go back to the front of the buffer: one counter update per wave and round
#pragma unroll
    for (int e = 0; e < kCandPerThread; ++e) {
        if (e * nt < n) {                   // uniform
            const bool keep = mine[e] <= T && mine[e] != kSentinel;
            const uint64_t mask = __ballot(keep);
            unsigned base = 0;
            if (lane == 0 && mask != 0) base = atomicAdd(&s.misc[0], (unsigned)__popcll(mask));
            base = __builtin_amdgcn_readfirstlane(base);
            if (keep) s.cand[base + (unsigned)__popcll(mask & ((1ull << lane) - 1ull))] = mine[e];
        }
    }
    __syncthreads();
    return T;
}

// Fresh read of a workgroup counter in LDS.  The pointer is cast to the LDS address space first: a volatile
// read through a generic pointer would be a flat load, which has to wait for every global load in flight
// (the prefetched code blocks) before its value can be used.
__device__ __forceinline__ unsigned lds_peek(const unsigned *p) {
    return *(const volatile __attribute__((address_space(3))) unsigned *)p;
}

// Copy of one query's table (256 x MP floats, contiguous) from global memory into LDS, in two halves so that
// it overlaps other loads: lut_copy_begin() issues the loads, lut_copy_end() completes them; a barrier then
// makes the table visible to the workgroup.  Tables that end below 64 KiB of LDS go straight from global
// memory to LDS (each wave-wide load moves 64 x 16 bytes to consecutive LDS addresses, without passing
// through registers; its LDS base is a 16-bit wave-uniform offset); larger ones are copied through registers
// at the end.
template <int NTHREADS, int MP>
__device__ __forceinline__ void lut_copy_begin(const float *__restrict__ src, float *dst) {
    if constexpr (kKsub * MP * 4 <= 65536) {
        typedef __attribute__((address_space(3))) unsigned char lds_byte;
        typedef __attribute__((address_space(1))) const unsigned char global_byte;
        constexpr int kPieces = kKsub * MP / 4 / NTHREADS;       // 16-byte pieces per thread
        const int tid = threadIdx.x;
        lds_byte *base = (lds_byte *)dst + (tid & ~63) * 16;     // wave-uniform; the hardware adds 16 bytes per lane
        global_byte *g = (global_byte *)src + (size_t)tid * 16;
#pragma unroll
        for (int i = 0; i < kPieces; ++i)
            __builtin_amdgcn_global_load_lds(g + (size_t)i * NTHREADS * 16, base + i * NTHREADS * 16, 16, 0, 0);
    }
}
template <int NTHREADS, int MP>
__device__ __forceinline__ void lut_copy_end(const float *__restrict__ src, float *dst) {
    if constexpr (kKsub * MP * 4 <= 65536) {
        __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0): this thread's direct loads have landed
    } else {
        constexpr int kPieces = kKsub * MP / 4 / NTHREADS;
        const float4 *s4 = reinterpret_cast<const float4 *>(src);
        float4 *d4 = reinterpret_cast<float4 *>(dst);
        constexpr int kChunk = kPieces % 4 == 0 ? 4 : 2;        // pieces in flight per thread
        static_assert(kPieces % kChunk == 0, "whole chunks");
        for (int i0 = 0; i0 < kPieces; i0 += kChunk) {
            float4 v[kChunk];
#pragma unroll
            for (int i = 0; i < kChunk; ++i) v[i] = s4[threadIdx.x + (i0 + i) * NTHREADS];
#pragma unroll
            for (int i = 0; i < kChunk; ++i) d4[threadIdx.x + (i0 + i) * NTHREADS] = v[i];
        }
    }
}

// The query's probe tables (block prefix sums, first block and length of each probed list) go to LDS in two
// halves, loads into registers and stores to LDS, so that other loads can be issued in between.
template <int NTHREADS>
struct ProbeTableRegs {
    static constexpr int kIter = kMaxNprobe / NTHREADS;
    int32_t pf[kIter], pb[kIter], pl[kIter], pf_last;
    float pc[kIter];
};
template <int NTHREADS>
__device__ __forceinline__ void load_probe_tables(const ScanArgs &a, int qi, ProbeTableRegs<NTHREADS> &r) {
    const int tid = threadIdx.x;
    const int32_t *pf = a.pfx + (size_t)qi * (a.probe_stride + 1);
    const int32_t *pb = a.pblk + (size_t)qi * a.probe_stride, *pl = a.plen + (size_t)qi * a.probe_stride;
#pragma unroll
    for (int j = 0; j < ProbeTableRegs<NTHREADS>::kIter; ++j) {
        const int i = tid + j * NTHREADS;
        const bool ok = i < a.nprobe;
        r.pf[j] = ok ? pf[i] : 0; r.pb[j] = ok ? pb[i] : 0; r.pl[j] = ok ? pl[i] : 0;
        r.pc[j] = ok && a.pcst ? a.pcst[(size_t)qi * a.probe_stride + i] : 0.f;
    }
    r.pf_last = pf[a.nprobe];
}
template <int NTHREADS>
__device__ __forceinline__ void store_probe_tables(const ScanArgs &a, const ScanLds &s, const ProbeTableRegs<NTHREADS> &r) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < ProbeTableRegs<NTHREADS>::kIter; ++j) {
        const int i = tid + j * NTHREADS;
        if (i < a.nprobe) { s.pfx[i] = r.pf[j]; s.blk[i] = r.pb[j]; s.len[i] = r.pl[j]; s.cst[i] = r.pc[j]; }
    }
    if (tid == 0) { s.pfx[a.nprobe] = r.pf_last; s.misc[0] = 0; s.misc[3] = 0; }
}

// ------------------------------------------------------------------------------------------------
// Stage 2: lookup tables.  entry(q, m, j) = sum_t (query_q[m*dsub+t] - pq[m][j][t])^2,
// stored in the scan layout lut[q][j][Mp] (rows of padding sub-quantisers m >= M are zero), built from the
// centre-major copy of the codebook pqT[j][m][t] by four workgroups per query (the codebook read, 768 KiB at
// d = 768, is what the build costs, so it is spread over several compute units).
// ------------------------------------------------------------------------------------------------

// One table entry: squared distance between dsub query coordinates and dsub centre coordinates.  DSUB > 0
// fixes dsub at compile time (all loads of several entries can then be in flight together; the query's
// coordinates are in registers).
template <int DSUB>
__device__ __forceinline__ float lut_entry(const float *qs, const float *__restrict__ c, int dsub) {
    float acc = 0.f;
    if (DSUB > 0) {
        float cv[DSUB > 0 ? DSUB : 1];
        if (DSUB % 4 == 0) {
#pragma unroll
            for (int t = 0; t < DSUB; t += 4) {
                const float4 v = *reinterpret_cast<const float4 *>(c + t);
                cv[t] = v.x; cv[(t + 1) % (DSUB > 0 ? DSUB : 1)] = v.y; cv[(t + 2) % (DSUB > 0 ? DSUB : 1)] = v.z;
                cv[(t + 3) % (DSUB > 0 ? DSUB : 1)] = v.w;
            }
        } else {
#pragma unroll
            for (int t = 0; t < DSUB; ++t) cv[t] = c[t];
        }
#pragma unroll
        for (int t = 0; t < DSUB; ++t) {
            const float diff = qs[t] - cv[t];
            acc += diff * diff;
        }
    } else {
        for (int t = 0; t < dsub; ++t) {
            const float diff = qs[t] - c[t];
            acc += diff * diff;
        }
    }
    return acc;
}

// Table build: workgroup (x, q) computes kKsub / gridDim.x rows j of query q's table, a wave a quarter of them, 8
// at a time so that their loads overlap; lane <-> sub-quantiser, so the reads of pqT[j][m][.] and the writes of
// lut[q][j][m] are contiguous.  A lane's slice of the query stays in registers for all its rows when dsub is
// known at compile time (read from LDS per entry, lanes dsub words apart collide on the banks: measured 75 % of
// the LDS cycles at dsub = 12); otherwise it is read from global memory, where it sits in the first-level cache.
// grid = (4, 8 or 16 workgroups per query, nq), 256 threads.
template <int DSUB>
__global__ __launch_bounds__(256) void lut_build_kernel(const float *__restrict__ q, const float *__restrict__ pqT, int d, int M,
                                                        int dsub, int Mp, float *__restrict__ lut_out) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = blockIdx.y;
    const int rows_per_wave = kKsub / (int)gridDim.x / 4;      // 16, 8 or 4
    float *out = lut_out + (size_t)qi * kKsub * Mp;
    for (int m = lane; m < Mp; m += kWave) {
        const float *qg = q + (size_t)qi * d + (size_t)min(m, M - 1) * dsub;
        float qr[DSUB > 0 ? DSUB : 1];
        if (DSUB > 0) {
#pragma unroll
            for (int t = 0; t < DSUB; ++t) qr[t] = qg[t];
        }
        const float *qs = DSUB > 0 ? qr : qg;
        for (int j0 = blockIdx.x * 4 * rows_per_wave + wave * rows_per_wave, it = 0; it < rows_per_wave; it += 8, j0 += 8) {
            float e[8];
            const int nj = min(8, rows_per_wave - it);         // 8, or 4 with 16 workgroups per query (uniform)
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
                e[jj] = (m < M && jj < nj) ? lut_entry<DSUB>(qs, pqT + ((size_t)(j0 + jj) * M + m) * dsub, dsub) : 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
                if (jj < nj) out[(size_t)(j0 + jj) * Mp + m] = e[jj];
        }
    }
}

// Selection from a key list by one workgroup: the k smallest of the keys in list[0..n) (global memory, written by
// this and other workgroups, all different).  Up to `room` keys are gathered into s_keys first (those within
// `bound`, which at least k keys are if k exist) and selected there; a longer list is selected in place, one
// sweep over global memory per round.
// FINAL = true: ids are looked up and the results written to out_d / out_i, sorted by (distance, id) and padded
// with (+inf, -1); s_d / s_id: power-of-two >= k slots.
// FINAL = false: the k smallest keys and up to KW - k more are written to dst[0..KW), unsorted and padded with
// kSentinel (whoever reads them selects again).
// Slots of `list` that hold kSentinel are skipped.
constexpr int kRankMaxK = 256;        // results up to this many are placed by counting (see below)
constexpr int kRankSlack = 128;       // ... among at most this many candidates more than k (more slack ends the counting
                                      // earlier but leaves more candidates to rank: 384 cost batches a quarter more, 64 made
                                      // no difference; the same scheme in the probe selection gained nothing at 32 probes
                                      // and lost 4 us at 256, where ranking 384 candidates costs more than the rounds saved)

template <bool FINAL>
__device__ void select_from_list(const uint64_t *list_in_global, int n, int room, int k, uint32_t bound, uint64_t *keys_in_lds,
                                 unsigned *hist_in_lds, unsigned long long *state_in_lds, unsigned *count_in_lds,
                                 const int64_t *ids_in_global, uint32_t *d_in_lds, int64_t *id_in_lds, float *out_d_in_global,
                                 int64_t *out_i_in_global, uint64_t *dst_in_global, int KW) {
    const glb_u64 *const list = (const glb_u64 *)list_in_global;
    const glb_i64 *const ids = (const glb_i64 *)ids_in_global;
    glb_f32 *const out_d = (glb_f32 *)out_d_in_global;
    glb_i64 *const out_i = (glb_i64 *)out_i_in_global;
    glb_u64 *const dst = (glb_u64 *)dst_in_global;
    lds_u64 *const s_keys = (lds_u64 *)keys_in_lds;              // see the comment at lds_u64
    lds_u32 *const s_hist = (lds_u32 *)hist_in_lds, *const s_count = (lds_u32 *)count_in_lds, *const s_d = (lds_u32 *)d_in_lds;
    lds_ull *const s_state = (lds_ull *)state_in_lds;
    lds_i64 *const s_id = (lds_i64 *)id_in_lds;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int k2 = max(2, 1 << (32 - __clz(k - 1)));
    if (FINAL)
        for (int i = tid; i < k2; i += nt) { s_d[i] = 0xFFFFFFFFu; s_id[i] = 0x7FFFFFFFFFFFFFFFll; }
    if (tid == 0) { *s_count = 0; s_state[5] = 0xFFFFFFFFull; s_state[6] = 0; }
    __syncthreads();
    const bool in_lds = n <= room;                               // uniform
    int found = n;
    KeyRange range{false, 0, 0, 0};
    if (in_lds) {
        // 16 keys per thread at a time; the loads of the next 16 are issued before these are looked at, and a wave
        // adds its passing keys of all 16 to the counter at once (one LDS round trip per wave and turn, not 16)
        constexpr int kPer = 16;
        uint64_t key[kPer], nxt[kPer];
        auto fetch = [&](uint64_t (&dst)[kPer], int i0) {
#pragma unroll
            for (int j = 0; j < kPer; ++j) dst[j] = i0 + j * nt < n ? load_key(list + i0 + j * nt) : kSentinel;
        };
        // (the smallest and the largest distance among the keys gathered are noted on the way: the selection below
        // then starts from their range without a pass of its own over the keys)
        uint32_t dmin = 0xFFFFFFFFu, dmax = 0;
        fetch(key, tid);
        for (int i0 = tid; i0 < n + tid; i0 += kPer * nt) {      // i0 - tid < n: the same number of turns for every thread
            const bool more = i0 - tid + kPer * nt < n;          // uniform
            if (more) fetch(nxt, i0 + kPer * nt);
            uint64_t mask[kPer];
            unsigned total = 0;
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                const uint32_t dj = (uint32_t)(key[j] >> 32);
                const bool ok = key[j] != kSentinel && dj <= bound;
                mask[j] = __ballot(ok);
                total += (unsigned)__popcll(mask[j]);
                dmin = ok ? min(dmin, dj) : dmin;
                dmax = ok ? max(dmax, dj) : dmax;
            }
            unsigned at = 0;
            if ((tid & 63) == 0 && total != 0) at = lds_add(s_count, total);
            at = __builtin_amdgcn_readfirstlane(at);
            const uint64_t below = (1ull << (tid & 63)) - 1ull;
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                if ((mask[j] >> (tid & 63)) & 1ull) s_keys[at + (unsigned)__popcll(mask[j] & below)] = key[j];
                at += (unsigned)__popcll(mask[j]);
            }
            if (more) {
#pragma unroll
                for (int j = 0; j < kPer; ++j) key[j] = nxt[j];
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            dmin = min(dmin, (uint32_t)__shfl_xor(dmin, off, 64));
            dmax = max(dmax, (uint32_t)__shfl_xor(dmax, off, 64));
        }
        if ((tid & 63) == 0) { lds_min(&s_state[5], (unsigned long long)dmin); lds_max(&s_state[6], (unsigned long long)dmax); }
        __syncthreads();
        found = (int)*s_count;
        range = KeyRange{true, (uint64_t)s_state[5] << 32, ((uint64_t)s_state[6] << 32) | 0xFFFFFFFFull, (unsigned)found};
        __syncthreads();
    }
    auto key_at = [&](int i) { return in_lds ? s_keys[i] : load_key(list + i); };
    // Results by counting.  An exact k-th key takes the bucket counting up to eight rounds of four barriers (1 to 7
    // were seen, 3 us each on a few thousand keys), and the results then still have to be ordered.  Instead: a bound
    // T with between k and k + kRankSlack keys below it (one round, seldom two), those candidates side by side in
    // LDS, and for each the number of candidates with a smaller key: that is its rank by (distance, slot) - ranks
    // below k are the results, and the rank is the place in the output unless results share a distance (then the ids
    // of that run decide, as the order is by (distance, id)).
    const int ncand_max = k + kRankSlack;
    if (FINAL && k <= kRankMaxK && nt >= kRankMaxK && (in_lds ? found + ncand_max <= room || found <= ncand_max : ncand_max <= room)) {   // uniform
        const lds_u64 *c_keys = s_keys;                          // the candidates
        int m = found;
        if (found > ncand_max || !in_lds) {
            uint64_t T = kSentinel - 1;
            if (found > ncand_max) T = block_select_kth(key_at, found, k, s_hist, s_state, kRankSlack, range);
            lds_u64 *c_out = in_lds ? s_keys + found : s_keys;
            if (tid == 0) *s_count = 0;
            __syncthreads();
            for_each_key_of(key_at, found, [&](uint64_t key) {
                if (key <= T) c_out[lds_add(s_count, 1u)] = key;     // kSentinel > T
            });
            __syncthreads();
            m = (int)*s_count;
            c_keys = c_out;
        }
        const int cnt = min(m, k);
        for (int j = tid; j < m; j += nt) {
            const uint64_t mine = c_keys[j];
            const int64_t id = ids[(uint32_t)mine];              // asked for before the rank is known: the counting covers the wait
            int rank = 0;
            int i = 0;
            for (; i + 8 <= m; i += 8) {                         // reads that all lanes make at the same address
                uint64_t o[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) o[u] = c_keys[i + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) rank += o[u] < mine ? 1 : 0;
            }
            for (; i < m; ++i) rank += c_keys[i] < mine ? 1 : 0;
            if (rank < k) { s_d[rank] = (uint32_t)(mine >> 32); s_id[rank] = id; }
        }
        __syncthreads();
        for (int r = tid; r < cnt; r += nt) {
            const uint32_t d = s_d[r];
            const int64_t id = s_id[r];
            int place = r;
            if ((r > 0 && s_d[r - 1] == d) || (r + 1 < cnt && s_d[r + 1] == d)) {   // a run of equal distances: by id
                // the run's ends by bisection (s_d is ascending), then the ids of the run, eight reads at a time
                int b = 0, bh = r;                               // first place of the run: first i in [0, r] with s_d[i] >= d
                while (b < bh) { const int mid = (b + bh) >> 1; if (s_d[mid] < d) b = mid + 1; else bh = mid; }
                int e = r + 1, eh = cnt;                         // its end: first i in (r, cnt] with s_d[i] > d (cnt if none)
                while (e < eh) { const int mid = (e + eh) >> 1; if (s_d[mid] > d) eh = mid; else e = mid + 1; }
                place = b;
                int i = b;
                for (; i + 8 <= e; i += 8) {
                    int64_t o[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) o[u] = s_id[i + u];
#pragma unroll
                    for (int u = 0; u < 8; ++u) place += (o[u] < id || (o[u] == id && i + u < r)) ? 1 : 0;
                }
                for (; i < e; ++i) place += (s_id[i] < id || (s_id[i] == id && i < r)) ? 1 : 0;
            }
            out_d[place] = __uint_as_float(d);
            out_i[place] = id;
        }
        for (int i = cnt + tid; i < k; i += nt) { out_d[i] = __builtin_inff(); out_i[i] = -1; }
        return;
    }
    uint64_t T = kSentinel - 1;                                  // no more than k candidates: keep them all
    if (found > k) T = block_select_kth(key_at, found, k, s_hist, s_state, FINAL ? 0 : KW - k, range);
    if (tid == 0) *s_count = 0;
    __syncthreads();
    for_each_key_of(key_at, found, [&](uint64_t key) {
        if (key <= T) {                                          // at most k (FINAL) or KW keys qualify (keys are distinct; kSentinel > T)
            const unsigned slot = lds_add(s_count, 1u);
            if (FINAL) { s_d[slot] = (uint32_t)(key >> 32); s_id[slot] = ids[(uint32_t)key]; }
            else store_key(dst + slot, key);
        }
    });
    __syncthreads();
    const int cnt = (int)*s_count;
    if (!FINAL) {
        for (int i = cnt + tid; i < KW; i += nt) store_key(dst + i, kSentinel);
        return;
    }
    // Order by (distance, id).  Up to one result per thread: the results that sort before a result are counted (the
    // pairs are all different, so the counts are the places) and it is written there - short loops over LDS reads
    // that all lanes make at the same address (a bitonic network, over lane exchanges or in LDS, took 7 us for
    // 100 results).  More results than threads: bitonic network in LDS.
    if (k2 <= nt) {                                              // uniform
        // nt / k2 threads share the count of one result (each takes a part of the slots, 16 reads at a time so that
        // they overlap; unused slots hold the largest distance bits and count for nobody) and add their parts up
        // in LDS; ids are looked at only by a thread that sees the result's distance a second time
        const int parts = min(nt / k2, k2), span = k2 / parts;   // powers of two; span >= 1
        const int mine = tid & (k2 - 1), part = tid / k2, j0 = part * span;
        if (tid < k2) s_hist[tid] = 0;
        __syncthreads();
        if (mine < cnt && part < parts) {
            const uint32_t d_mine = s_d[mine];
            int before = 0;
            bool tie = false;
            int j = j0;
            for (; j + 16 <= j0 + span; j += 16) {
                uint32_t dj[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) dj[u] = s_d[j + u];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    before += dj[u] < d_mine ? 1 : 0;
                    tie |= dj[u] == d_mine && j + u != mine;
                }
            }
            for (; j < j0 + span; ++j) {
                before += s_d[j] < d_mine ? 1 : 0;
                tie |= s_d[j] == d_mine && j != mine;
            }
            if (tie) {
                const int64_t id_mine = s_id[mine];
                for (int jj = j0; jj < j0 + span; ++jj) before += (s_d[jj] == d_mine && s_id[jj] < id_mine) ? 1 : 0;
            }
            if (before) lds_add(&s_hist[mine], (unsigned)before);
        }
        __syncthreads();
        if (tid < cnt) {
            const int place = (int)s_hist[tid];
            out_d[place] = __uint_as_float(s_d[tid]);
            out_i[place] = s_id[tid];
        }
        for (int i = cnt + tid; i < k; i += nt) { out_d[i] = __builtin_inff(); out_i[i] = -1; }
        return;
    }
    for (int size = 2; size <= k2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int i = tid; i < (k2 >> 1); i += nt) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint32_t da = s_d[lo], db = s_d[hi];
                const int64_t ia = s_id[lo], ib = s_id[hi];
                const bool gt = da > db || (da == db && ia > ib);
                if (gt == up) { s_d[lo] = db; s_d[hi] = da; s_id[lo] = ib; s_id[hi] = ia; }
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < k; i += nt) {
        out_d[i] = i < cnt ? __uint_as_float(s_d[i]) : __builtin_inff();
        out_i[i] = i < cnt ? s_id[i] : -1;
    }
}

// Room for keys when the table and candidate areas of the scan kernel's LDS are reused for the final selection
// (after its s_id and s_d).
__host__ __device__ inline int reduce_room_keys(int Mp, int cap, int k) {
    const int k2 = k <= 2 ? 2 : 1 << (32 - __builtin_clz((unsigned)(k - 1)));
    return (1024 * Mp + 8 * cap - 12 * k2) / 8;
}

// ------------------------------------------------------------------------------------------------
// Stage 3: scan of the probed lists with candidate selection.
// The probed lists of a query, concatenated in probe order, form a sequence of 64-vector blocks; the plan
// gives every workgroup a query, and the waves of a query's workgroups take that sequence in chunks of
// 4 to 32 blocks (the plan fixes the length per query, and how many chunks have it: the last ones are 4 blocks) from shared counters.  A lane owns one vector of the block: it reads its Mp code bytes
// with Mp/16 16-byte loads (NSETS blocks are kept in flight per wave) and adds Mp table entries from LDS.
// Because of the rotated code layout (see common.h), at step t lane l looks up sub-quantiser (l + t) mod Mp,
// so with the table stored [j][Mp] the lanes of a half-wave hit different LDS banks when Mp is 32 or 64.
// Candidates (distance bits << 32 | slot) that pass the bound on the final k-th best distance are appended
// to one buffer per workgroup.  The waves run independently; a wave that sees the buffer nearly full (or has
// no blocks left) waits at a barrier, and once all four are there the buffer is pruned to about k keys and
// the bound tightened.  The bound is the smallest such value any workgroup of the query has reached
// (thr[q] in global memory, polled once per chunk).  At the end the workgroup's (at most KW) surviving keys
// go to the query's key list, unsorted, and the query's last workgroup to finish selects the k best among
// them, looks up the ids and writes the results (see the end of the kernel).  RES: residual index (see the
// comment in process below).
// STREAM: the code blocks are read with non-temporal loads.  That is faster when the codes come from HBM anyway
// (measured on 16 GiB of codes: 5.7 instead of 5.5 TB/s; on 64 GiB: 6.2 instead of 5.8) and slower when the
// batch's lists would otherwise be found again in the caches by the next query or the next call (1 GiB of codes,
// 64 queries: 5.5 instead of 6.3 TB/s), so the host chooses it by the shape of the index.
// ------------------------------------------------------------------------------------------------
template <int C, int NSETS, bool RES, bool STREAM>
__global__ __launch_bounds__(kScanThreads, 2) void adc_scan_kernel(ScanArgs a) {
    constexpr int MP = 16 * C;
    extern __shared__ __align__(16) unsigned char smem[];   // the kernel has no other LDS: smem starts at LDS address 0
    const int k = a.k, KW = a.KW, cap = a.cap;
    const ScanLds s = carve_lds(smem, MP, cap, a.nprobe);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // (Workgroups are dealt to the 8 XCDs in turn by their launch number, so the workgroups of a query, consecutive in
    // the plan, sit on different XCDs.  Taking them from one XCD instead, so that the query's table is fetched into
    // one L2 rather than eight, was measured: 6 % faster at 32 queries, 3 % slower at 64 queries x 256 probes, equal
    // elsewhere - not kept.)
    const int wg = blockIdx.x;
    const int4 desc = a.desc[wg];            // (query, number among its workgroups | their count << 16, full-length chunks, counters and chunk length)
    if (desc.x < 0) return;                                  // spare workgroup (uniform exit)
    const int qi = desc.x;
    const bool lut_at_zero =
        reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) unsigned char *)smem) == 0;
    // the query's table starts on its way to LDS first (it depends on nothing else), then the probe tables
    ProbeTableRegs<kScanThreads> tables;
    load_probe_tables(a, qi, tables);
    lut_copy_begin<kScanThreads, MP>(a.lut + (size_t)qi * kKsub * MP, s.lut);
    store_probe_tables(a, s, tables);
    __syncthreads();

    // Best known bound on the k-th best key: the workgroup's own (a key, from its last pruning) or the query's
    // (a distance, which admits every slot).  A bound with a slot part matters when many vectors share the
    // k-th best distance: without it all of them would pass and be pruned away again and again.
    uint64_t thr = ~0ull;
    const int trigger = cap - kScanThreads;
    const int lane_m = lane % MP;
    uint32_t off4[16];
    make_off4(off4, lane);

    // The query's blocks (numbered along its probed lists) are handed out in chunks of chunk_len blocks to the
    // waves of all its workgroups: the first chunk of a wave is the one of its own number, later ones come from
    // the query's counter, asked for one chunk ahead so that the answer is there when it is needed.  A slow
    // workgroup (pruning, a busy memory channel) simply takes fewer chunks.
    const int TB = s.pfx[a.nprobe];                          // blocks of this query
    // (the zero below is lane-dependent as far as the compiler can tell: an address it knows to be the same in
    // all lanes makes it combine the lanes' additions and fetch the answer at once, which would wait for every
    // load in flight)
    const int wave_of_query = (desc.y & 0xFFFF) * kScanWaves + wave, nctr = desc.w & 0xFF, my_ctr = wave_of_query % nctr;
    const int tpc = 1 << (desc.w >> 8), chunk_len = kChunkBlocks * tpc;   // a chunk is tpc turns of kChunkBlocks blocks ...
    const int full = desc.z;                                 // ... up to chunk number `full`; from there on, one turn
    // first block of chunk c, and its number of turns
    auto chunk_at = [&](int c, int &turns) -> int {
        turns = c < full ? tpc : 1;
        return c < full ? c * chunk_len : (int)((unsigned)full * (unsigned)chunk_len + (unsigned)(c - full) * kChunkBlocks);
    };
    uint32_t *ctr = a.ctr + ((size_t)qi * kCtrPerQuery + my_ctr) * kCtrStride + __builtin_amdgcn_mbcnt_lo(0u, 0u);
    int pi = 0;                     // probe whose list holds the block looked up last (chunks only move forward)
    auto ask_chunk = [&]() -> uint32_t {
        uint32_t c = 0;
        if (lane == 0) c = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return c;                   // lane 0 holds the answer once the load counter says so
    };

    // Every call issues the same number of loads, whether or not block b exists (beyond the end a wave re-reads
    // a few bytes of block 0, which always exists): the compiler can then count the loads in flight exactly
    // and lets NSETS - 1 later requests stay in flight while one block is worked on.
    // nvalid = 0 marks a request beyond the end.  tx, cl: residual indexes only (the vector's own term, loaded with
    // the block, and the constant of its list).
    struct Meta { uint32_t gblock; int nvalid; float tx, cl; };
    const uint4 *idle = reinterpret_cast<const uint4 *>(a.codes);
    auto issue = [&](uint4 (&w)[C], Meta &m, int b) {
        m.nvalid = 0;
        const uint4 *src = idle;
        size_t tx_at = 0;
        if (b < TB) {
            for (;;) {              // lanes look at the next 64 prefix sums at once; b < TB = pfx[nprobe] bounds pi
                const int32_t e = s.pfx[min(pi + 1 + lane, a.nprobe)];
                const int adv = __popcll(__ballot(b >= e));
                pi += adv;
                if (adv < kWave) break;
            }
            const int bl = b - s.pfx[pi];
            m.gblock = (uint32_t)(s.blk[pi] + bl);
            m.nvalid = s.len[pi] - bl * kBlockVecs;           // >= 1; lanes >= nvalid hold padding
            src = reinterpret_cast<const uint4 *>(a.codes + (size_t)m.gblock * kBlockVecs * MP) + lane;
            if (RES) {              // the list's constant is the same in all lanes: kept in a scalar register
                m.cl = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(s.cst[pi])));
                tx_at = (size_t)m.gblock * kBlockVecs;
            }
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if constexpr (STREAM) {
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + c * kWave));
                w[c] = make_uint4(v.x, v.y, v.z, v.w);
            } else {
                w[c] = src[c * kWave];
            }
        }
        if (RES) m.tx = a.tx[tx_at + lane];                  // one more load per request, block or not
    };
    auto process = [&](const uint4 (&w)[C], const Meta &m) {
        float dist;
        if (C == 4 && lut_at_zero) dist = block_dist_m64(reinterpret_cast<const uint4 (&)[4]>(w), off4);
        else dist = block_dist_generic<C>(w, s.lut, lane_m);
        // residual index: the table sum is |q - p|^2 for the decoded residual p; adding 2 <c, p> (stored per vector)
        // and |c|^2 - 2 <q, c> (per probed list) makes it |q - c - p|^2; clamped, since key order needs dist >= 0
        if (RES) dist = fmaxf(0.f, dist + m.tx + m.cl);
        const uint32_t dbits = __float_as_uint(dist);
        const uint32_t slot = m.gblock * kBlockVecs + lane;
        bool pass = (lane < m.nvalid) && ((((uint64_t)dbits << 32) | slot) <= thr);
        append_candidates(pass, dbits, slot, s.cand, &s.misc[0], cap, lane);
    };

    uint4 w[NSETS][C];
    Meta meta[NSETS];
    int turns;                                               // turns of the chunk being requested (the wave's own first chunk to begin with)
    int cb = chunk_at(wave_of_query, turns);                 // first block of the turn being requested
    int turn = 0;                                            // which turn of its chunk that is
    uint32_t pending = ask_chunk();
    // the query's bound is polled once per chunk, with the chunk request, and used one turn later
    uint32_t tg = __hip_atomic_load(&a.thr[qi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int i = 0; i < NSETS; ++i) issue(w[i], meta[i], cb + i);
    lut_copy_end<kScanThreads, MP>(a.lut + (size_t)qi * kKsub * MP, s.lut);
    __syncthreads();
    // An episode is a meeting of all waves of the workgroup: every wave joins every episode (from wherever it
    // is in its loop), the two counters are read between two barriers (nobody appends in between), and the
    // buffer is pruned if it is nearly full.  A wave asks for an episode by waiting in one: when the buffer is
    // nearly full (the others notice at their next block) or when it has run out of blocks.  Returns the
    // number of waves that are out of blocks.
    auto episode = [&]() -> int {
        __syncthreads();
        const int n = (int)lds_peek(&s.misc[0]);
        const int ndone = (int)lds_peek(&s.misc[3]);
        __syncthreads();            // nobody appends again before everybody has read the two counters
        if (n > trigger) {          // uniform: all threads read the same values between the barriers
            const uint64_t T = wg_prune(s, min(n, cap), k);
            thr = min(thr, T);
            if (tid == 0) atomicMin(&a.thr[qi], (uint32_t)(T >> 32));
        }
        return ndone;
    };
    // One turn of the loop works through kChunkBlocks blocks; request number NSETS + j (counted from the wave's
    // first) is made at step j, so the step at which the next turn's blocks begin - and, every tpc turns, the next
    // chunk - is the same in every turn.
    static_assert(kChunkBlocks % NSETS == 0, "a chunk is a whole number of rounds over the register sets");
    for (;;) {
        bool any = false;           // this wave still holds a requested block
#pragma unroll
        for (int i = 0; i < NSETS; ++i) any |= meta[i].nvalid > 0;
        if (!any) break;            // chunks only move forward: nothing valid in flight means nothing is left
#pragma unroll
        for (int j = 0; j < kChunkBlocks; ++j) {
            const int i = j % NSETS, pos = (NSETS + j) % kChunkBlocks;   // position of the request within its chunk
            if (pos == 0) {
                if (++turn == turns) {                       // uniform: the chunk is used up, on to the one asked for
                    turn = 0;
                    const uint32_t v = min(__builtin_amdgcn_readfirstlane(pending), 0x7FFFFFFFu / (kChunkBlocks * 8 * kCtrPerQuery) - 1u);
                    cb = chunk_at((int)(v * nctr + my_ctr), turns);
                    pending = ask_chunk();
                    thr = min(thr, ((uint64_t)tg << 32) | 0xFFFFFFFFull);
                    tg = __hip_atomic_load(&a.thr[qi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    cb += kChunkBlocks;                      // the chunk's next turn
                }
            }
            if (meta[i].nvalid > 0) {
                // the count is looked at before every block; a wave appends at most 64 keys per block
                while ((int)lds_peek(&s.misc[0]) > trigger) episode();
                process(w[i], meta[i]);
            }
            issue(w[i], meta[i], cb + pos);
        }
    }
    // out of blocks: tell the others, and keep joining their episodes until every wave is out of blocks
    if (lane == 0) atomicAdd(&s.misc[3], 1u);
    while (episode() != kScanWaves) {}
    int n = min((int)lds_peek(&s.misc[0]), cap);
    if (n > KW) {                   // uniform
        const uint64_t T = wg_prune(s, n, k);
        if (tid == 0) atomicMin(&a.thr[qi], (uint32_t)(T >> 32));
        n = (int)lds_peek(&s.misc[0]);
    }
    // What the workgroup still holds goes to its KW slots (padded with kSentinel) of a key list: the query's, or,
    // when the query has more workgroups than one selection can take in LDS (fan), the list of its group of fan
    // consecutive workgroups.  The keys are written before the workgroup adds itself to the count of finished
    // workgroups; whoever sees that count complete may read the whole list.  The last workgroup of a group passes
    // the group's k best on to the query's list in the same way, and the last group of the query (or its last
    // workgroup, without groups) selects the results.  (With local bounds only, a query spread over S workgroups
    // ends with about k keys per workgroup that none of them can rule out; that is what the two levels are for.)
    const int seg = desc.y & 0xFFFF, S = desc.y >> 16, wg0 = wg - seg;   // the query's workgroups: wg0 .. wg0 + S - 1
    // Groups: none if one selection takes the keys of all S workgroups (a.fan of them fit its LDS); else groups of about
    // sqrt(S) workgroups, so that the two levels see about as many keys each - a selection is the work of one compute
    // unit, a few us per pass over 8,000 keys, and the groups' selections run side by side (512 workgroups in 9 groups
    // of 58: 20 to 30 us for the first level and 15 for the second; in 23 groups of 23: 10 to 13 and 16 to 21) - but no
    // smaller than it takes for the groups' own keys to fit the second selection.
    int fan = a.fan;
    if (S > fan) {                                               // uniform; a.fan * a.fan >= S (the host sees to that)
        int f = 1;
        while (f * f < S) ++f;
        fan = min(fan, max(f, (S + fan - 1) / fan));
    }
    const int R = (S + fan - 1) / fan;                           // R groups (R = 1: no groups)
    const int r = R == 1 ? 0 : seg / fan, gsize = R == 1 ? S : min(fan, S - r * fan);
    uint64_t *list = a.part + (size_t)(wg0 + r * fan) * KW;      // of the group (of the query, without groups)
    uint32_t *ldone = R == 1 ? &a.qdone[qi] : &a.gdone[wg0 + r];
    uint64_t *mine = list + (size_t)(seg - r * fan) * KW;
    for (int i = tid; i < KW; i += kScanThreads) store_key(mine + i, i < n ? s.cand[i] : kSentinel);
    publish_keys();
    if (tid == 0) s.misc[4] = atomicAdd(ldone, 1u);
    __syncthreads();
    if (s.misc[4] != (unsigned)(gsize - 1)) return;              // uniform
    // the last workgroup of the list: selection in the LDS that held table and candidates
    const int k2 = max(2, 1 << (32 - __clz(k - 1)));
    int64_t *s_id = reinterpret_cast<int64_t *>(smem);
    uint32_t *s_d = reinterpret_cast<uint32_t *>(s_id + k2);
    uint64_t *s_keys = reinterpret_cast<uint64_t *>(smem + 12 * (size_t)k2);
    float *res_d = a.out_d + (size_t)qi * k;
    int64_t *res_i = a.out_i + (size_t)qi * k;
    uint32_t bound = __hip_atomic_load(&a.thr[qi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (R == 1) {
        select_from_list<true>(list, S * KW, a.room, k, bound, s_keys, s.hist, s.state, &s.misc[0], a.ids, s_d, s_id, res_d, res_i,
                               nullptr, KW);
        return;
    }
    uint64_t *list2 = a.part2 + (size_t)wg0 * KW;                // the query's list: KW slots per group
    select_from_list<false>(list, gsize * KW, a.room, k, bound, s_keys, s.hist, s.state, &s.misc[0], nullptr, nullptr, nullptr,
                            nullptr, nullptr, list2 + (size_t)r * KW, KW);
    publish_keys();
    if (tid == 0) s.misc[4] = atomicAdd(&a.qdone[qi], 1u);
    __syncthreads();
    if (s.misc[4] != (unsigned)(R - 1)) return;                  // uniform
    bound = __hip_atomic_load(&a.thr[qi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    select_from_list<true>(list2, R * KW, a.room, k, bound, s_keys, s.hist, s.state, &s.misc[0], a.ids, s_d, s_id, res_d, res_i,
                           nullptr, KW);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
template <int DSUB>
void launch_lut_build_d(const piperag_index *ix, const float *q, int nq, float *lut, hipStream_t st) {
    const int per_query = nq >= 64 ? 4 : (nq >= 16 ? 8 : 16);     // workgroups per query: enough of them for small batches
    hipLaunchKernelGGL((lut_build_kernel<DSUB>), dim3(per_query, nq), dim3(256), 0, st, q, ix->pqT, ix->p.d, ix->p.M, ix->dsub,
                       ix->Mp, lut);
}

void launch_lut_build(const piperag_index *ix, const float *q, int nq, float *lut, hipStream_t st) {
    switch (ix->dsub) {                      // common slice widths get their loads unrolled at compile time
        case 4: launch_lut_build_d<4>(ix, q, nq, lut, st); break;
        case 6: launch_lut_build_d<6>(ix, q, nq, lut, st); break;
        case 8: launch_lut_build_d<8>(ix, q, nq, lut, st); break;
        case 12: launch_lut_build_d<12>(ix, q, nq, lut, st); break;
        case 16: launch_lut_build_d<16>(ix, q, nq, lut, st); break;
        default: launch_lut_build_d<0>(ix, q, nq, lut, st); break;
    }
}

// code blocks in flight per wave: as many as fit without register spills (the residual variant holds one more
// value per lane and block)
template <int C, bool RES>
constexpr int scan_nsets() { return C <= (RES ? 3 : 4) ? 4 : (C <= 6 ? 2 : 1); }

template <int C, bool RES, bool STREAM>
int launch_scan_rs(const ScanArgs &a, int G, size_t lds, hipStream_t st) {
    hipLaunchKernelGGL((adc_scan_kernel<C, scan_nsets<C, RES>(), RES, STREAM>), dim3(G), dim3(kScanThreads), lds, st, a);
    return PIPERAG_OK;
}
template <int C>
int launch_scan(const ScanArgs &a, bool stream, int G, size_t lds, hipStream_t st) {
    if (a.tx) return stream ? launch_scan_rs<C, true, true>(a, G, lds, st) : launch_scan_rs<C, true, false>(a, G, lds, st);
    return stream ? launch_scan_rs<C, false, true>(a, G, lds, st) : launch_scan_rs<C, false, false>(a, G, lds, st);
}

#define PR_DISPATCH_C(expr_prefix, ...)                                         \
    switch (ix->Mp / 16) {                                                      \
        case 1: rc = expr_prefix<1>(__VA_ARGS__); break;                        \
        case 2: rc = expr_prefix<2>(__VA_ARGS__); break;                        \
        case 3: rc = expr_prefix<3>(__VA_ARGS__); break;                        \
        case 4: rc = expr_prefix<4>(__VA_ARGS__); break;                        \
        case 5: rc = expr_prefix<5>(__VA_ARGS__); break;                        \
        case 6: rc = expr_prefix<6>(__VA_ARGS__); break;                        \
        case 7: rc = expr_prefix<7>(__VA_ARGS__); break;                        \
        case 8: rc = expr_prefix<8>(__VA_ARGS__); break;                        \
        default: PR_REQUIRE(false, PIPERAG_ERR_ARG, "unsupported M");           \
    }

// Kernels that may need more dynamic LDS than the default limit get the device's whole 160 KiB allowed.
constexpr int kMaxLds = 160 * 1024;
template <class K>
hipError_t allow_lds(K kernel) {            // whatever the kernel's static LDS leaves of the 160 KiB
    hipFuncAttributes fa;
    const hipError_t e = hipFuncGetAttributes(&fa, reinterpret_cast<const void *>(kernel));
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kMaxLds - (int)fa.sharedSizeBytes);
}
template <int C>
hipError_t allow_lds_scan() {
    hipError_t e = allow_lds(&adc_scan_kernel<C, scan_nsets<C, false>(), false, false>);
    if (e == hipSuccess) e = allow_lds(&adc_scan_kernel<C, scan_nsets<C, false>(), false, true>);
    if (e == hipSuccess) e = allow_lds(&adc_scan_kernel<C, scan_nsets<C, true>(), true, false>);
    if (e == hipSuccess) e = allow_lds(&adc_scan_kernel<C, scan_nsets<C, true>(), true, true>);
    return e;
}

PlanOut plan_bufs(const piperag_index *ix, const SearchWs &ws) {
    return PlanOut{ws.pfx, ws.pblk, ws.plen, ws.scanned, ws.thr, ix->p.residual ? ws.pcst : nullptr, ws.done};
}

ShareOut share_bufs(const SearchWs &ws, int fan) { return ShareOut{ws.seg0, ws.desc, ws.ctr, ws.done + ws.max_nq, fan}; }

// Parts of the depth the matrix-core coarse quantiser is split into for this shape (0: the row-wise kernel
// runs instead and writes finished distances).
int coarse_parts(const piperag_index *ix, const float *q, int nq) {
    const int d = ix->p.d, nlist = ix->p.nlist;
    if (!(nq > 4 && d % 4 == 0 && d >= 64 && reinterpret_cast<uintptr_t>(q) % 16 == 0)) return 0;
    const int tiles = ((nlist + CoarseTile::kRowsB - 1) / CoarseTile::kRowsB) * ((nq + CoarseTile::kRowsA - 1) / CoarseTile::kRowsA);
    int parts = 1;
    if (nlist <= kCoarseSplitMaxLists)
        while (parts < kCoarseMaxParts && tiles * parts < 256 && d / (parts * 2) >= 64) parts *= 2;
    return parts;
}

int launch_select(const piperag_index *ix, const SearchWs &ws, const float *q, int nq, int nprobe, int target, int max_wg, int fan,
                  hipStream_t st) {
    const int nlist = ix->p.nlist;
    const int G = select_groups(nlist, nq, nprobe, ix->ncu);
    const int slice_len = ((nlist + G - 1) / G + 3) / 4 * 4;
    const int np2 = next_pow2(std::max(2, nprobe));
    // the candidates of a query's slices are selected in LDS when they fit (they do, unless the row is so long that
    // the slices LDS allows, times nprobe, exceed it: more than half a million lists with nprobe 1024)
    const size_t cand_bytes = G > 1 ? sizeof(uint64_t) * (size_t)G * nprobe : 0;
    const int cand_in_lds = cand_bytes <= sizeof(float) * kSelMaxLdsRow;
    const size_t lds = std::max(std::max(sizeof(float) * (size_t)slice_len, cand_in_lds ? cand_bytes : 0), sizeof(uint64_t) * (size_t)np2);
    PR_REQUIRE(slice_len <= kSelMaxLdsRow && np2 <= kMaxNprobe, PIPERAG_ERR_LIMIT,
               "probe selection does not fit: nlist = %d, nprobe = %d", nlist, nprobe);
    uint32_t *arrived = ws.tb + ws.max_nq, *qticket = ws.tb + ws.max_nq + 1;
    if (slice_len <= kSelSmallRow)
        hipLaunchKernelGGL(select_probes_kernel<kSelThreads>, dim3(nq * G), dim3(kSelThreads), lds, st, ws.D, coarse_parts(ix, q, nq),
                           nq, G, slice_len, cand_in_lds, q, ix->p.d, ix->cnorm, nlist, nprobe, ws.probe, ws.probe_d, ws.max_nprobe,
                           ix->list_blk, ix->list_len, plan_bufs(ix, ws), ws.selcand, qticket, ws.tb, arrived, target, max_wg,
                           share_bufs(ws, fan));
    else
        hipLaunchKernelGGL(select_probes_kernel<kSelThreadsLong>, dim3(nq * G), dim3(kSelThreadsLong), lds, st, ws.D,
                           coarse_parts(ix, q, nq), nq, G, slice_len, cand_in_lds, q, ix->p.d, ix->cnorm, nlist, nprobe, ws.probe, ws.probe_d,
                           ws.max_nprobe, ix->list_blk, ix->list_len, plan_bufs(ix, ws), ws.selcand, qticket, ws.tb, arrived,
                           target, max_wg, share_bufs(ws, fan));
    return PIPERAG_OK;
}

int launch_coarse(const piperag_index *ix, const SearchWs &ws, const float *q, int nq, hipStream_t st) {
    constexpr int QT = 4;
    const int d = ix->p.d, nlist = ix->p.nlist;
    const int parts = coarse_parts(ix, q, nq);
    if (parts > 0) {                                         // batches: matrix cores
        const int dper = (d / parts + 31) / 32 * 32;
        hipLaunchKernelGGL(coarse_mfma_kernel, dim3((nlist + CoarseTile::kRowsB - 1) / CoarseTile::kRowsB,
                                                    (nq + CoarseTile::kRowsA - 1) / CoarseTile::kRowsA, parts),
                           dim3(256), 0, st, q, nq, ix->centroids, nlist, d, dper, ws.D);
        return PIPERAG_OK;
    }
    // one query (the serving case) gets a kernel of its own: a quarter of the lookups and lane reductions
    const int QTr = nq == 1 ? 1 : QT;
    const int groups = std::min((nlist + 15) / 16, 2048);   // a workgroup's 4 waves take 4 centres each per turn
    const dim3 grid(groups, (nq + QTr - 1) / QTr);
    const size_t lds = sizeof(float) * QTr * d;
    if (d % 4 == 0 && QTr == 1)
        hipLaunchKernelGGL((coarse_rowwise_kernel<1, 4, 4>), grid, dim3(256), lds, st, q, ix->centroids, ws.D, nq, nlist, d);
    else if (d % 4 == 0)
        hipLaunchKernelGGL((coarse_rowwise_kernel<QT, 4, 4>), grid, dim3(256), lds, st, q, ix->centroids, ws.D, nq, nlist, d);
    else if (QTr == 1)
        hipLaunchKernelGGL((coarse_rowwise_kernel<1, 1, 4>), grid, dim3(256), lds, st, q, ix->centroids, ws.D, nq, nlist, d);
    else
        hipLaunchKernelGGL((coarse_rowwise_kernel<QT, 1, 4>), grid, dim3(256), lds, st, q, ix->centroids, ws.D, nq, nlist, d);
    return PIPERAG_OK;
}

int check_search_args(const piperag_index *ix, const void *q, int32_t nq, int32_t nprobe, int32_t k, const void *od,
                      const void *oi) {
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(ix->finalized, PIPERAG_ERR_ARG, "index is not finalized");
    PR_REQUIRE(nq >= 0, PIPERAG_ERR_ARG, "nq = %d is negative", nq);
    if (nq == 0) return PIPERAG_OK;
    PR_REQUIRE(q && od && oi, PIPERAG_ERR_ARG, "queries / output pointer is NULL");
    PR_REQUIRE(nprobe >= 1 && k >= 1, PIPERAG_ERR_ARG, "nprobe = %d and k = %d must be >= 1", nprobe, k);
    PR_REQUIRE(nprobe <= ix->p.nlist, PIPERAG_ERR_ARG, "nprobe = %d exceeds nlist = %d", nprobe, ix->p.nlist);
    return PIPERAG_OK;
}
int check_search_limits(const piperag_index *ix, int32_t nq, int32_t nprobe, int32_t k) {
    PR_REQUIRE(nq <= ix->p.max_nq, PIPERAG_ERR_LIMIT, "nq = %d exceeds max_nq = %d", nq, ix->p.max_nq);
    PR_REQUIRE(nprobe <= ix->p.max_nprobe, PIPERAG_ERR_LIMIT, "nprobe = %d exceeds max_nprobe = %d", nprobe, ix->p.max_nprobe);
    PR_REQUIRE(k <= ix->p.max_k, PIPERAG_ERR_LIMIT, "k = %d exceeds max_k = %d", k, ix->p.max_k);
    return PIPERAG_OK;
}

// Scan workgroups a search call asks the plan for: two per compute unit the search may use (the whole chip unless
// piperag_set_compute_units says otherwise), or for large batches about 8 per query.
int scan_target_wgs(int nq, int ncu) { return std::min(kMaxScanWGs, std::max(std::min(kTargetScanWGs, 2 * ncu), 8 * nq)); }

// Enqueues one search on st, with `ws` as its scratch (kernel launches and event records only: it can be captured
// into a graph).  stages: record the index's stage events (not for searches that use a workspace other than the
// index's own).  Everything runs on st, in the order coarse quantiser, selection, tables, scan.  (The tables need
// only the queries and were once built on a side stream beside the first two stages; the two cross-stream waits
// cost more than the overlap gave: a waited-for single query took 111 instead of 90 us, 16 queries 158 instead
// of 139, and back-to-back batches of 64 or 256 ran no faster.  Building them by workgroups appended to the coarse
// quantiser's grid instead of a launch of their own was measured too: 1 us less for one query, 4 us for four -
// launches queued on one stream follow each other within a microsecond or two - and was not kept.)
int enqueue_search(const piperag_index *ix, const SearchWs &ws, bool stages, const float *q, int32_t nq, const int32_t *probes,
                   int32_t nprobe, int32_t k, float *out_d, int64_t *out_i, hipStream_t st) {
    int rc = PIPERAG_OK;
    const int pstride = ws.max_nprobe;
    const bool tm = ix->timing && stages;
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[0], st));
    if (!probes && (rc = launch_coarse(ix, ws, q, nq, st)) != PIPERAG_OK) return rc;
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[1], st));
    const int target_wgs = scan_target_wgs(nq, ix->ncu);
    const int G = std::max(target_wgs, nq);                 // upper bound of the workgroups the plan hands out
    const int KW = k + kKeepSlack;                          // key slots per scan workgroup in the partial buffer
    // Candidate slots of a scan workgroup: as many as kCandRoom beyond the keys kept, but fewer if that lets two
    // workgroups share a compute unit's 160 KiB of LDS (long probe tables would otherwise push the second one out).
    int cand_room = kCandRoom;
    {
        const size_t half = 80 * 1024, fixed = scan_lds_bytes(ix->Mp, KW, nprobe);
        if (fixed + 8 * (size_t)kCandRoom > half && fixed + 8 * (size_t)kCandRoomMin <= half) cand_room = (int)((half - fixed) / 8);
    }
    const int cap = KW + cand_room;
    // the query's last workgroup selects the results in the LDS that held its table and candidates: `room` keys,
    // i.e. the keys of `fan` workgroups; more workgroups per query are merged in groups of fan first; if two levels
    // do not cover a query's workgroups (very large k with short codes), there are no groups and a long list is
    // selected in global memory
    const int room = reduce_room_keys(ix->Mp, cap, k);
    int fan = std::max(1, room / KW);
    if ((long long)fan * fan < G) fan = G;
    if (!probes) {
        if ((rc = launch_select(ix, ws, q, nq, nprobe, target_wgs, G, fan, st)) != PIPERAG_OK) return rc;
    } else {
        hipLaunchKernelGGL(copy_probes_kernel, dim3(nq), dim3(64), 0, st, probes, nprobe, ix->p.nlist, ws.probe, pstride,
                           ix->list_blk, ix->list_len, plan_bufs(ix, ws));
        hipLaunchKernelGGL(share_kernel, dim3(1), dim3(256), 0, st, ws.pfx, pstride, nprobe, nq, target_wgs, G, share_bufs(ws, fan));
        if (ix->p.residual)
            hipLaunchKernelGGL(probe_const_kernel, dim3(nprobe, nq), dim3(64), 0, st, q, ix->centroids, ix->cnorm, ix->p.d,
                               ws.probe, pstride, ws.pcst);
    }
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[2], st));
    ScanArgs a{ix->codes, ws.lut, ws.pfx, ws.pblk, ws.plen, ix->p.residual ? ws.pcst : nullptr,
               ix->p.residual ? ix->tx : nullptr, ws.part, ws.thr, ws.desc, ws.ctr, nprobe, pstride, k, KW};
    launch_lut_build(ix, q, nq, ws.lut, st);
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[3], st));
    a.cap = cap;
    a.qdone = ws.done;
    a.room = room;
    a.fan = fan;
    a.gdone = ws.done + ws.max_nq;
    a.part2 = ws.part2;
    a.ids = ix->ids; a.out_d = out_d; a.out_i = out_i;
    const size_t lds = scan_lds_bytes(ix->Mp, a.cap, nprobe);
    PR_REQUIRE(lds <= (size_t)kMaxLds, PIPERAG_ERR_LIMIT, "scan needs %zu bytes of LDS (M, k, nprobe too large together)", lds);
    // Indexes far larger than the last-level cache are streamed: nothing read now is still cached when it is needed
    // again.  Measured with 64-byte codes: +4 % to +6 % at 16 GiB and 64 GiB of codes in 65,536 lists (0.25 and 1 MiB
    // per list on average) for 1 to 256 queries; but -4 % for batches of 8 and 64 queries on 192 GB of codes in 16,384
    // lists (11.7 MiB per list), hence the second condition.
    const size_t code_bytes = (size_t)ix->nblocks * kBlockVecs * ix->Mp;
    const bool streaming = ix->streaming < 0 ? code_bytes >= kStreamingCodeBytes && code_bytes / ix->p.nlist < kStreamingListBytes
                                             : ix->streaming > 0;
    PR_DISPATCH_C(launch_scan, a, streaming, G, lds, st)
    if (rc != PIPERAG_OK) return rc;
    if (tm) { PR_CHECK_HIP(hipEventRecord(ix->ev[4], st)); ix->ev_valid = true; }
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

// A search is four launches on one stream.  With replay enabled (piperag_set_graph_replay), a call that repeats an
// earlier one (same buffers, same sizes: a serving loop that refills its query buffer) is captured into a graph
// the second time it is seen and replayed with one launch from then on: one host call per search instead of four.
// It does not shorten a search (measured on this GPU: a waited-for single query takes 93 us replayed against 89 us
// launched plainly, and back-to-back calls lose 10 us each), so it is opt-in, for callers whose host thread is the
// scarce resource.  The graph holds only kernel nodes.  Stage timing keeps the plain path.
// The index is const for the caller: what a search changes is its workspace in device memory and the members
// declared mutable (statistics, event state, graph cache).
int search_impl(const piperag_index *ix, const float *q, int32_t nq, const int32_t *probes, int32_t nprobe, int32_t k,
                float *out_d, int64_t *out_i, hipStream_t st) {
    int rc = check_search_args(ix, q, nq, nprobe, k, out_d, out_i);
    if (rc != PIPERAG_OK || nq == 0) return rc;
    if ((rc = check_search_limits(ix, nq, nprobe, k)) != PIPERAG_OK) return rc;
    PR_CHECK_HIP(hipSetDevice(ix->device));
    ix->last_nq = nq;
    ix->last_scanned = ix->ws.scanned;
    if (ix->timing || !ix->replay) return enqueue_search(ix, ix->ws, true, q, nq, probes, nprobe, k, out_d, out_i, st);
    SearchGraph *slot = nullptr, *oldest = &ix->graphs[0];
    for (SearchGraph &g : ix->graphs) {
        if (g.seen && g.q == q && g.probes == probes && g.nq == nq && g.nprobe == nprobe && g.k == k && g.out_d == out_d &&
            g.out_i == out_i)
            slot = &g;
        if (g.stamp < oldest->stamp) oldest = &g;
    }
    if (!slot) {                                            // first time: remember the call, run it plainly
        if (oldest->exec) { (void)hipGraphExecDestroy(oldest->exec); }
        *oldest = SearchGraph{q, probes, nq, nprobe, k, out_d, out_i, nullptr, ++ix->graph_clock, 1};
        return enqueue_search(ix, ix->ws, true, q, nq, probes, nprobe, k, out_d, out_i, st);
    }
    slot->stamp = ++ix->graph_clock;
    if (!slot->exec) {                                      // second time: capture
        hipGraph_t graph = nullptr;
        PR_CHECK_HIP(hipStreamBeginCapture(ix->cap_stream, hipStreamCaptureModeRelaxed));
        rc = enqueue_search(ix, ix->ws, true, q, nq, probes, nprobe, k, out_d, out_i, ix->cap_stream);
        const hipError_t e = hipStreamEndCapture(ix->cap_stream, &graph);
        if (rc != PIPERAG_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
        if (e != hipSuccess || !graph) { set_error("graph capture failed: %s", hipGetErrorString(e)); return PIPERAG_ERR_HIP; }
        const hipError_t e2 = hipGraphInstantiate(&slot->exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e2 != hipSuccess) { slot->exec = nullptr; set_error("graph instantiation failed: %s", hipGetErrorString(e2)); return PIPERAG_ERR_HIP; }
    }
    PR_CHECK_HIP(hipGraphLaunch(slot->exec, st));
    return PIPERAG_OK;
}

// lut[q][j][Mp] (the scan's layout) -> out[q][m][j] (canonical), m < M.
__global__ __launch_bounds__(256) void lut_canonical_kernel(const float *__restrict__ lut, int M, int Mp, float *__restrict__ out) {
    const int qi = blockIdx.y, m = blockIdx.x, j = threadIdx.x;
    out[((size_t)qi * M + m) * kKsub + j] = lut[((size_t)qi * kKsub + j) * Mp + m];
}

__global__ void clear_u32_kernel(uint32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

constexpr int kMaxDevices = 64;
std::mutex g_dev_mutex;
bool g_search_configured[kMaxDevices];
void *g_scratch_ptr[kMaxDevices];           // per device: address of its copy of the static scratch array

}  // namespace

// ---- scratch for callers that cannot allocate ---------------------------------------------------
// One array per GPU, in the code object's own device memory, held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the address that call returns (one per device, kept in
// g_scratch_ptr) is what kernels and host calls are given.
static __device__ __align__(256) unsigned char scratch[PIPERAG_STATIC_SCRATCH_BYTES];

namespace piperag {

size_t search_ws_layout(SearchWs *ws, void *base, int nlist, int Mp, int max_nq, int max_nprobe, int max_k, int max_wgs) {
    unsigned char *b = static_cast<unsigned char *>(base);
    size_t off = 0;
    const size_t nq = (size_t)max_nq, np = (size_t)max_nprobe, wgs = (size_t)max_wgs;
    auto take = [&](auto **field, size_t count) {            // every array starts on a 256-byte boundary
        using T = std::remove_reference_t<decltype(**field)>;
        *field = b ? reinterpret_cast<T *>(b + off) : nullptr;
        off = (off + count * sizeof(T) + 255) / 256 * 256;
    };
    take(&ws->D, nq * nlist * (nlist <= kCoarseSplitMaxLists ? kCoarseMaxParts : 1));
    take(&ws->probe, nq * np);
    take(&ws->probe_d, nq * np);
    take(&ws->pfx, nq * (np + 1));
    take(&ws->scanned, nq);
    take(&ws->seg0, nq + 1);
    take(&ws->desc, wgs + nq);
    take(&ws->done, wgs + 2 * nq);
    take(&ws->tb, 2 * nq + 1);
    // selection workgroups of a batch: at most 64 per query and kSelTargetWGs in all, unless long rows need more
    take(&ws->selcand, std::max(nq * (size_t)((nlist + kSelMaxLdsRow - 1) / kSelMaxLdsRow), std::min((size_t)kSelTargetWGs, nq * 64)) * np);
    take(&ws->ctr, nq * kCtrPerQuery * kCtrStride);
    take(&ws->pcst, nq * np);
    take(&ws->pblk, nq * np);
    take(&ws->plen, nq * np);
    take(&ws->thr, nq);
    take(&ws->lut, nq * kKsub * Mp);
    take(&ws->part, (wgs + 2 * nq) * ((size_t)max_k + kKeepSlack));
    take(&ws->part2, (wgs + 2 * nq) * ((size_t)max_k + kKeepSlack));
    ws->max_nq = max_nq; ws->max_nprobe = max_nprobe; ws->max_k = max_k;
    return off;
}

int configure_search_kernels(int device) {
    PR_REQUIRE(device >= 0 && device < kMaxDevices, PIPERAG_ERR_ARG, "device %d out of range", device);
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (g_search_configured[device]) return PIPERAG_OK;
    int cur = -1;
    PR_CHECK_HIP(hipGetDevice(&cur));
    if (cur != device) PR_CHECK_HIP(hipSetDevice(device));
    PR_CHECK_HIP(allow_lds_scan<1>()); PR_CHECK_HIP(allow_lds_scan<2>()); PR_CHECK_HIP(allow_lds_scan<3>());
    PR_CHECK_HIP(allow_lds_scan<4>()); PR_CHECK_HIP(allow_lds_scan<5>()); PR_CHECK_HIP(allow_lds_scan<6>());
    PR_CHECK_HIP(allow_lds_scan<7>()); PR_CHECK_HIP(allow_lds_scan<8>());
    PR_CHECK_HIP(allow_lds(&select_probes_kernel<kSelThreads>));
    PR_CHECK_HIP(allow_lds(&select_probes_kernel<kSelThreadsLong>));
    PR_CHECK_HIP(allow_lds(&coarse_rowwise_kernel<4, 4, 4>)); PR_CHECK_HIP(allow_lds(&coarse_rowwise_kernel<4, 1, 4>));
    PR_CHECK_HIP(allow_lds(&coarse_rowwise_kernel<1, 4, 4>)); PR_CHECK_HIP(allow_lds(&coarse_rowwise_kernel<1, 1, 4>));
    // this device's copy of the static scratch array
    void *ptr = nullptr;
    PR_CHECK_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    PR_REQUIRE(ptr != nullptr && reinterpret_cast<uintptr_t>(ptr) % 256 == 0, PIPERAG_ERR_HIP, "static scratch array has no usable device address");
    g_scratch_ptr[device] = ptr;
    g_search_configured[device] = true;
    if (cur != device && cur >= 0) PR_CHECK_HIP(hipSetDevice(cur));
    return PIPERAG_OK;
}

}  // namespace piperag

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
extern "C" {

int piperag_ivfpq_search(const piperag_index *index, const float *queries_dev, int32_t nq, int32_t nprobe, int32_t k,
                         float *out_dist_dev, int64_t *out_ids_dev, void *stream) {
    return search_impl(index, queries_dev, nq, nullptr, nprobe, k, out_dist_dev, out_ids_dev, (hipStream_t)stream);
}

int piperag_ivfpq_search_probes(const piperag_index *index, const float *queries_dev, int32_t nq, const int32_t *probes_dev,
                                int32_t nprobe, int32_t k, float *out_dist_dev, int64_t *out_ids_dev, void *stream) {
    PR_REQUIRE(probes_dev != nullptr || nq == 0, PIPERAG_ERR_ARG, "probes_dev is NULL");
    return search_impl(index, queries_dev, nq, probes_dev, nprobe, k, out_dist_dev, out_ids_dev, (hipStream_t)stream);
}

int piperag_ivfpq_search_static(const piperag_index *index, const float *queries_dev, int32_t nq, int32_t nprobe, int32_t k,
                                float *out_dist_dev, int64_t *out_ids_dev, void *stream) {
    int rc = check_search_args(index, queries_dev, nq, nprobe, k, out_dist_dev, out_ids_dev);
    if (rc != PIPERAG_OK || nq == 0) return rc;
    PR_REQUIRE(nq <= 65535 && nprobe <= kMaxNprobe && k <= kMaxK, PIPERAG_ERR_LIMIT,
               "nq = %d, nprobe = %d, k = %d: beyond 65535 / %d / %d", nq, nprobe, k, kMaxNprobe, kMaxK);
    PR_CHECK_HIP(hipSetDevice(index->device));
    // the scratch is carved for exactly this call's sizes; what does not fit the static array is refused
    SearchWs ws;
    const int wgs = std::max(scan_target_wgs(nq, index->ncu), (int)nq);
    const size_t need = search_ws_layout(&ws, nullptr, index->p.nlist, index->Mp, nq, nprobe, k, wgs);
    PR_REQUIRE(need <= (size_t)PIPERAG_STATIC_SCRATCH_BYTES, PIPERAG_ERR_LIMIT,
               "this search needs %zu bytes of scratch; the static scratch array holds %zu (smaller nq, nprobe or k)", need,
               (size_t)PIPERAG_STATIC_SCRATCH_BYTES);
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_dev_mutex);
        ptr = index->device >= 0 && index->device < kMaxDevices ? g_scratch_ptr[index->device] : nullptr;
    }
    PR_REQUIRE(ptr != nullptr, PIPERAG_ERR_HIP, "the static scratch array was not set up on device %d", index->device);
    search_ws_layout(&ws, ptr, index->p.nlist, index->Mp, nq, nprobe, k, wgs);
    hipStream_t st = (hipStream_t)stream;
    // the array keeps the last call's contents, laid out for that call's sizes: the count of finished selections
    // and the per-query tickets behind it must start at zero (everything else is written before it is read)
    hipLaunchKernelGGL(clear_u32_kernel, dim3((nq + 1 + 255) / 256), dim3(256), 0, st, ws.tb + nq, nq + 1);
    index->last_nq = nq;
    index->last_scanned = ws.scanned;
    return enqueue_search(index, ws, false, queries_dev, nq, nullptr, nprobe, k, out_dist_dev, out_ids_dev, st);
}

int piperag_ivf_coarse(const piperag_index *index, const float *queries_dev, int32_t nq, int32_t nprobe,
                       int32_t *out_lists_dev, float *out_dist_dev, void *stream) {
    const piperag_index *ix = index;
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(nq >= 0, PIPERAG_ERR_ARG, "nq = %d is negative", nq);
    if (nq == 0) return PIPERAG_OK;
    PR_REQUIRE(queries_dev && out_lists_dev, PIPERAG_ERR_ARG, "queries / output pointer is NULL");
    PR_REQUIRE(nq <= ix->p.max_nq, PIPERAG_ERR_LIMIT, "nq = %d exceeds max_nq = %d", nq, ix->p.max_nq);
    PR_REQUIRE(nprobe >= 1 && nprobe <= ix->p.nlist, PIPERAG_ERR_ARG, "nprobe = %d out of range", nprobe);
    PR_REQUIRE(nprobe <= ix->p.max_nprobe, PIPERAG_ERR_LIMIT, "nprobe = %d exceeds max_nprobe = %d", nprobe, ix->p.max_nprobe);
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(ix->device));
    const SearchWs &ws = ix->ws;
    const int rc = launch_coarse(ix, ws, queries_dev, nq, st);
    if (rc != PIPERAG_OK) return rc;
    const int rc2 = launch_select(ix, ws, queries_dev, nq, nprobe, kTargetScanWGs, std::max(kTargetScanWGs, (int)nq), kMaxScanWGs, st);
    if (rc2 != PIPERAG_OK) return rc2;
    PR_CHECK_HIP(hipMemcpy2DAsync(out_lists_dev, sizeof(int32_t) * nprobe, ws.probe, sizeof(int32_t) * ws.max_nprobe,
                                  sizeof(int32_t) * nprobe, nq, hipMemcpyDeviceToDevice, st));
    if (out_dist_dev)
        PR_CHECK_HIP(hipMemcpy2DAsync(out_dist_dev, sizeof(float) * nprobe, ws.probe_d, sizeof(float) * ws.max_nprobe,
                                      sizeof(float) * nprobe, nq, hipMemcpyDeviceToDevice, st));
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

int piperag_ivf_lut(const piperag_index *index, const float *queries_dev, int32_t nq, float *out_lut_dev, void *stream) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(nq >= 0, PIPERAG_ERR_ARG, "nq = %d is negative", nq);
    if (nq == 0) return PIPERAG_OK;
    PR_REQUIRE(queries_dev && out_lut_dev, PIPERAG_ERR_ARG, "queries / output pointer is NULL");
    PR_REQUIRE(nq <= index->p.max_nq, PIPERAG_ERR_LIMIT, "nq = %d exceeds max_nq = %d", nq, index->p.max_nq);
    PR_CHECK_HIP(hipSetDevice(index->device));
    // the tables exactly as a search builds them (same kernel, same workspace), then rearranged for the caller
    launch_lut_build(index, queries_dev, nq, index->ws.lut, (hipStream_t)stream);
    hipLaunchKernelGGL(lut_canonical_kernel, dim3(index->p.M, nq), dim3(kKsub), 0, (hipStream_t)stream, index->ws.lut, index->p.M,
                       index->Mp, out_lut_dev);
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

int piperag_search_stats(const piperag_index *index, int64_t *scanned_vectors, int64_t *scanned_code_bytes) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    int64_t total = 0;
    if (index->last_nq > 0 && index->last_scanned) {
        std::vector<int64_t> h(index->last_nq);
        PR_CHECK_HIP(hipMemcpy(h.data(), index->last_scanned, sizeof(int64_t) * h.size(), hipMemcpyDeviceToHost));
        for (int64_t v : h) total += v;
    }
    if (scanned_vectors) *scanned_vectors = total;
    if (scanned_code_bytes) *scanned_code_bytes = total * index->p.M;
    return PIPERAG_OK;
}

int piperag_set_stage_timing(piperag_index *index, int enable) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    index->timing = enable != 0;
    index->ev_valid = false;
    return PIPERAG_OK;
}

static void drop_graphs(piperag_index *index) {
    for (SearchGraph &g : index->graphs) {
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
        g = SearchGraph{};
    }
}

int piperag_set_graph_replay(piperag_index *index, int enable) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    index->replay = enable != 0;
    if (!index->replay) drop_graphs(index);
    return PIPERAG_OK;
}

int piperag_set_compute_units(piperag_index *index, int32_t ncu) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    int total = 0;
    PR_CHECK_HIP(hipDeviceGetAttribute(&total, hipDeviceAttributeMultiprocessorCount, index->device));
    PR_REQUIRE(ncu <= total, PIPERAG_ERR_ARG, "ncu = %d exceeds the device's %d compute units", ncu, total);
    index->ncu = ncu <= 0 ? total : ncu;
    drop_graphs(index);              // a captured search holds the launch shapes of the time it was captured
    return PIPERAG_OK;
}

int piperag_set_scan_streaming(piperag_index *index, int mode) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    index->streaming = mode < 0 ? -1 : (mode > 0 ? 1 : 0);
    drop_graphs(index);              // a captured search holds the kernel that was chosen when it was captured
    return PIPERAG_OK;
}

int piperag_stage_times(const piperag_index *index, float *out_ms_host) {
    PR_REQUIRE(index != nullptr && out_ms_host != nullptr, PIPERAG_ERR_ARG, "NULL argument");
    PR_REQUIRE(index->timing && index->ev_valid, PIPERAG_ERR_ARG, "no timed search has run (enable stage timing first)");
    PR_CHECK_HIP(hipEventSynchronize(index->ev[PIPERAG_NSTAGES]));
    for (int s = 0; s < PIPERAG_NSTAGES; ++s)
        PR_CHECK_HIP(hipEventElapsedTime(&out_ms_host[s], index->ev[s], index->ev[s + 1]));
    return PIPERAG_OK;
}

int piperag_latency_profile(const piperag_index *index, const float *queries_dev, int32_t nq, const int32_t *nprobes_host,
                            int32_t n_nprobes, int32_t k, int32_t reps, float *out_p50_ms_host, float *out_fit_host,
                            void *stream) {
    PR_REQUIRE(index && queries_dev && nprobes_host && out_p50_ms_host, PIPERAG_ERR_ARG, "NULL argument");
    PR_REQUIRE(n_nprobes >= 1 && reps >= 1 && nq >= 1, PIPERAG_ERR_ARG, "n_nprobes, reps and nq must be >= 1");
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(index->device));
    hipEvent_t e0, e1;
    PR_CHECK_HIP(hipEventCreate(&e0));
    PR_CHECK_HIP(hipEventCreate(&e1));
    std::vector<float> t(reps);
    int rc = PIPERAG_OK;
    for (int i = 0; i < n_nprobes && rc == PIPERAG_OK; ++i) {
        for (int r = -2; r < reps && rc == PIPERAG_OK; ++r) {
            if (hipEventRecord(e0, st) != hipSuccess) { rc = PIPERAG_ERR_HIP; break; }
            rc = piperag_ivfpq_search(index, queries_dev, nq, nprobes_host[i], k, index->ws_out_d, index->ws_out_i, stream);
            if (rc != PIPERAG_OK) break;
            if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) { rc = PIPERAG_ERR_HIP; break; }
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = PIPERAG_ERR_HIP; break; }
            if (r >= 0) t[r] = ms;
        }
        if (rc != PIPERAG_OK) break;
        std::sort(t.begin(), t.end());
        out_p50_ms_host[i] = (reps & 1) ? t[reps / 2] : 0.5f * (t[reps / 2 - 1] + t[reps / 2]);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == PIPERAG_ERR_HIP) set_error("HIP event call failed in piperag_latency_profile");
    if (rc != PIPERAG_OK) return rc;
    if (out_fit_host) {
        // least squares of latency on nprobe
        double sx = 0, sy = 0, sxx = 0, sxy = 0;
        for (int i = 0; i < n_nprobes; ++i) {
            const double x = nprobes_host[i], y = out_p50_ms_host[i];
            sx += x; sy += y; sxx += x * x; sxy += x * y;
        }
        const double den = n_nprobes * sxx - sx * sx;
        const double b = den != 0.0 ? (n_nprobes * sxy - sx * sy) / den : 0.0;
        out_fit_host[0] = (float)((sy - b * sx) / n_nprobes);
        out_fit_host[1] = (float)b;
    }
    return PIPERAG_OK;
}

}  // extern "C"
