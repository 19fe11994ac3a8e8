// Search path of libpiperag: coarse quantiser, top-nprobe selection, scan plan, lookup-table build,
// list scan with k-selection, merge + id gather.  All kernels are written for gfx950 (wave64).
//
// Method: Section 3.2 (S3) of the paper - nprobe of the nlist inverted lists are selected per query and
// the product-quantised vectors inside them are compared with the query; Section 2 - the k closest are
// returned.  The retrieval latency model of S3 splits the time into an index-scan term (stages 0-1 here)
// and a vector-scan term proportional to nprobe (stages 2-4).
#include <stdlib.h>

#include <algorithm>
#include <vector>

#include "common.h"

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

// Largest key of the kth (1-based) smallest among n distinct 64-bit keys - i.e. a threshold T such that exactly
// kth keys are <= T - by most-significant-digit radix selection with the whole workgroup (blockDim >= 256,
// a multiple of 64).  key_at(i) may be evaluated several times.  Requires 1 <= kth <= n.  Stops as soon as
// the digits fixed so far isolate exactly the keys that are needed, which for float-derived keys is
// usually after the 32 distance bits.
template <class KeyFn>
__device__ uint64_t block_radix_select(KeyFn key_at, int n, int kth, unsigned *s_hist /*[256]*/,
                                       unsigned long long *s_state /*[4]*/) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6;
    uint64_t prefix = 0;
    for (int shift = 56; shift >= 0; shift -= 8) {
        for (int i = tid; i < 256; i += nt) s_hist[i] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += nt) {
            const uint64_t key = key_at(i);
            const bool in = (shift == 56) || ((key >> (shift + 8)) == (prefix >> (shift + 8)));
            if (in) atomicAdd(&s_hist[(unsigned)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        // inclusive prefix sum of the 256 digit counts: within each of the first 4 waves, then across them
        unsigned h = 0, incl = 0;
        if (tid < 256) {
            h = s_hist[tid];
            incl = h;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned o = __shfl_up(incl, off, 64);
                if (lane >= off) incl += o;
            }
            if (lane == 63) s_state[wave] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            for (int w = 0; w < wave; ++w) incl += (unsigned)s_state[w];
        }
        __syncthreads();
        if (tid < 256 && incl - h < (unsigned)kth && (unsigned)kth <= incl) {   // exactly one digit qualifies
            s_state[0] = prefix | ((uint64_t)tid << shift);
            s_state[1] = (unsigned long long)((unsigned)kth - (incl - h));
            s_state[2] = h;
        }
        __syncthreads();
        prefix = s_state[0];
        kth = (int)s_state[1];
        const bool whole_bucket = (unsigned long long)kth == s_state[2];
        __syncthreads();
        if (whole_bucket) return prefix | (shift > 0 ? ((1ull << shift) - 1ull) : 0ull);
    }
    return prefix;
}

// In-place ascending bitonic sort of n (power of two) 64-bit keys in LDS by the whole workgroup.
__device__ void block_bitonic_sort_u64(uint64_t *keys, int n) {
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int size = 2; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int i = tid; i < (n >> 1); i += nt) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const uint64_t a = keys[lo], b = keys[hi];
                if ((a > b) == up) { keys[lo] = b; keys[hi] = a; }
            }
        }
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// Stage 0: coarse distances  D[q][j] = || query_q - centre_j ||^2  (direct form, fp32)
// One wavefront per centre at a time; the lanes split the coordinates (VEC floats per lane per 64*VEC
// chunk, so a centre row is read with contiguous wavefront loads); QT queries of the batch are kept in
// LDS and share each centre read.  grid = (centre groups, ceil(nq / QT)).
// ------------------------------------------------------------------------------------------------
template <int QT, int VEC>
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
    for (int j = blockIdx.x * (blockDim.x >> 6) + wave; j < nlist; j += nwaves) {
        const float *row = cent + (size_t)j * d;
        float acc[QT];
#pragma unroll
        for (int qi = 0; qi < QT; ++qi) acc[qi] = 0.f;
        for (int t0 = lane * VEC; t0 < d; t0 += 64 * VEC) {
            float c[VEC];
            if (VEC == 4) {
                const float4 v = *reinterpret_cast<const float4 *>(row + t0);
                c[0] = v.x; c[1 % VEC] = v.y; c[2 % VEC] = v.z; c[3 % VEC] = v.w;
            } else {
                c[0] = row[t0];
            }
#pragma unroll
            for (int qi = 0; qi < QT; ++qi) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const float diff = s_q[qi * d + t0 + v] - c[v];
                    acc[qi] += diff * diff;
                }
            }
        }
#pragma unroll
        for (int qi = 0; qi < QT; ++qi) {
            const float s = wave_sum(acc[qi]);
            if (lane == 0 && qi < nqt) D[(size_t)(q0 + qi) * nlist + j] = s;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Stage 1a: per query, the nprobe smallest D[q][.] ordered by (distance, list).  One workgroup per query:
// radix selection of the nprobe-th smallest key (distance bits << 32 | list; distances are >= 0 so their
// bit patterns order like the values), compaction, bitonic sort.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void select_probes_kernel(const float *__restrict__ D, int nlist, int nprobe,
                                                            int32_t *__restrict__ probe, float *__restrict__ probe_d,
                                                            int probe_stride) {
    __shared__ unsigned s_hist[256];
    __shared__ unsigned long long s_state[4];
    __shared__ uint64_t s_keys[kMaxNprobe];
    __shared__ unsigned s_count;
    const int qi = blockIdx.x;
    const float *row = D + (size_t)qi * nlist;
    auto key_at = [&](int i) { return ((uint64_t)__float_as_uint(row[i]) << 32) | (uint32_t)i; };
    const uint64_t T = block_radix_select(key_at, nlist, nprobe, s_hist, s_state);
    const int np2 = max(2, 1 << (32 - __clz(nprobe - 1)));   // next power of two >= nprobe (>= 2)
    for (int i = threadIdx.x; i < np2; i += blockDim.x) s_keys[i] = kSentinel;
    if (threadIdx.x == 0) s_count = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < nlist; i += blockDim.x) {
        const uint64_t key = key_at(i);
        if (key <= T) {                                    // exactly nprobe keys qualify (keys are distinct)
            const unsigned slot = atomicAdd(&s_count, 1u);
            if (slot < (unsigned)np2) s_keys[slot] = key;
        }
    }
    __syncthreads();
    block_bitonic_sort_u64(s_keys, np2);
    for (int i = threadIdx.x; i < nprobe; i += blockDim.x) {
        probe[(size_t)qi * probe_stride + i] = (int32_t)(s_keys[i] & 0xFFFFFFFFu);
        probe_d[(size_t)qi * probe_stride + i] = __uint_as_float((uint32_t)(s_keys[i] >> 32));
    }
}

// Probe lists given by the caller: entries outside 0..nlist-1 and repeats of an earlier entry become -1
// (skipped), so that no list is scanned twice.
__global__ void copy_probes_kernel(const int32_t *__restrict__ src, int nprobe, int nlist, int32_t *__restrict__ dst,
                                   int probe_stride) {
    const int qi = blockIdx.x;
    const int32_t *row = src + (size_t)qi * nprobe;
    for (int i = threadIdx.x; i < nprobe; i += blockDim.x) {
        int32_t l = row[i];
        if (l < 0 || l >= nlist) l = -1;
        for (int e = 0; e < i && l >= 0; ++e)
            if (row[e] == l) l = -1;
        dst[(size_t)qi * probe_stride + i] = l;
    }
}

// Stage 1b: scan plan.  pfx[q][i] = number of 64-vector blocks in the first i probed lists of query q;
// scanned[q] = number of vectors in its probed lists; thr[q] = "no bound yet" for the scan's shared threshold.
__global__ void plan_kernel(const int32_t *__restrict__ probe, int probe_stride, int nprobe,
                            const int32_t *__restrict__ list_blk, const int32_t *__restrict__ list_len,
                            int32_t *__restrict__ pfx, int64_t *__restrict__ scanned, uint32_t *__restrict__ thr) {
    const int qi = blockIdx.x;
    if (threadIdx.x != 0) return;
    thr[qi] = 0xFFFFFFFFu;
    int32_t blocks = 0;
    int64_t vecs = 0;
    int32_t *out = pfx + (size_t)qi * (probe_stride + 1);
    for (int i = 0; i < nprobe; ++i) {
        out[i] = blocks;
        const int32_t l = probe[(size_t)qi * probe_stride + i];
        if (l >= 0) {
            blocks += list_blk[l + 1] - list_blk[l];
            vecs += list_len[l];
        }
    }
    out[nprobe] = blocks;
    scanned[qi] = vecs;
}

// ------------------------------------------------------------------------------------------------
// Stage 2: lookup tables.  entry(q, m, j) = sum_t (query_q[m*dsub+t] - pq[m][j][t])^2.
// Scan layout: lut[(q*256 + j)*Mp + m] (rows of padding sub-quantisers m >= M are zero);
// canonical layout (tap): out[(q*M + m)*256 + j].
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lut_kernel(const float *__restrict__ q, const float *__restrict__ pq, int d, int M,
                                                  int dsub, int Mp, float *__restrict__ out, int canonical) {
    const int qi = blockIdx.y, m = blockIdx.x, j = threadIdx.x;
    float acc = 0.f;
    if (m < M) {
        const float *qs = q + (size_t)qi * d + m * dsub;
        const float *c = pq + ((size_t)m * kKsub + j) * dsub;
        for (int t = 0; t < dsub; ++t) {
            const float diff = qs[t] - c[t];
            acc += diff * diff;
        }
    }
    if (canonical) {
        if (m < M) out[((size_t)qi * M + m) * kKsub + j] = acc;
    } else {
        out[((size_t)qi * kKsub + j) * Mp + m] = acc;
    }
}

// ------------------------------------------------------------------------------------------------
// Stage 3: scan of the probed lists with k-selection.
// grid = (S segments, nq).  The probed lists of a query, concatenated in probe order, form a sequence of
// 64-vector blocks; segment s takes an equal share of it, and the 4 waves of the workgroup take its blocks
// round-robin.  A lane owns one vector of the block: it reads its Mp code bytes with Mp/16 16-byte loads
// (NSETS blocks are kept in flight per wave) and adds Mp table entries from LDS.  Because of the rotated
// code layout (see common.h), at step t lane l looks up sub-quantiser (l + t) mod Mp, so with the table
// stored [j][Mp] the lanes of a half-wave hit different LDS banks when Mp is 32 or 64.
// For Mp = 64 the LDS byte address of a lookup is (code byte << 8) | (((l + t) mod 64) << 2): one byte
// permute of the code word with a per-step lane constant held in a register.
// k-selection: candidates (distance bits << 32 | slot) that pass a bound on the final k-th best distance
// are appended to one candidate buffer per workgroup.  Once per round of NSETS blocks per wave the
// workgroup meets at a barrier; when the buffer is nearly full it keeps only its k smallest keys (radix
// selection in LDS, no sorting) and tightens the bound.  The bound is the smallest k-th best any workgroup
// of the query has reached so far (thr[q] in global memory, polled with every block load); a candidate
// above it cannot be in the result.  At the end the workgroup's (at most k) keys go to the
// partial-result buffer, unsorted.
// ------------------------------------------------------------------------------------------------
struct ScanArgs {
    const uint8_t *codes;
    const float *lut;
    const int32_t *probe;
    const int32_t *pfx;
    const int32_t *list_blk;
    const int32_t *list_len;
    uint64_t *part;
    uint32_t *thr;
    int nprobe, probe_stride, k, KP;
#ifdef PIPERAG_TRACE
    unsigned long long *trace;   // [workgroups][8] timestamps
#endif
};

typedef const __attribute__((address_space(3))) float *lds_cfptr;

constexpr int kCandRoom = 1536;                       // candidate slots beyond KP
constexpr int kCandPerThread = (kMaxK + kCandRoom) / kScanThreads;

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

// Keeps the k smallest of the n (> k, distinct) keys in s_cand[0..n) at the front (any order) and returns
// the largest key kept.  Whole workgroup, called at a barrier-synchronised point; *s_count becomes k.
__device__ uint64_t wg_keep_k_smallest(uint64_t *s_cand, int n, int k, unsigned *s_hist, unsigned long long *s_state,
                                       unsigned *s_count) {
    const int tid = threadIdx.x;
    auto key_at = [&](int i) { return s_cand[i]; };
    const uint64_t T = block_radix_select(key_at, n, k, s_hist, s_state);
    uint64_t mine[kCandPerThread];
#pragma unroll
    for (int e = 0; e < kCandPerThread; ++e) {
        const int i = tid + e * kScanThreads;
        mine[e] = i < n ? s_cand[i] : kSentinel;
    }
    if (tid == 0) *s_count = 0;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kCandPerThread; ++e)
        if (mine[e] <= T && mine[e] != kSentinel) s_cand[atomicAdd(s_count, 1u)] = mine[e];
    __syncthreads();
    return T;
}

template <int C, int NSETS>
__global__ __launch_bounds__(kScanThreads, 2) void adc_scan_kernel(ScanArgs a) {
    constexpr int MP = 16 * C;
    extern __shared__ __align__(16) unsigned char smem[];   // the kernel has no other LDS: smem starts at LDS address 0
    const int k = a.k, KP = a.KP;
    const int cap = KP + kCandRoom;
    float *s_lut = reinterpret_cast<float *>(smem);                                  // [256*MP]
    uint64_t *s_cand = reinterpret_cast<uint64_t *>(smem + (size_t)1024 * MP);       // [cap]
    unsigned long long *s_state = reinterpret_cast<unsigned long long *>(s_cand + cap);   // [4]
    unsigned *s_hist = reinterpret_cast<unsigned *>(s_state + 4);                    // [256]
    unsigned *s_count = s_hist + 256;                                                // [1] (+1 pad)
    int32_t *s_pfx = reinterpret_cast<int32_t *>(s_count + 2);                       // [nprobe+1]
    int32_t *s_blk = s_pfx + (a.nprobe + 1);                                         // [nprobe]
    int32_t *s_len = s_blk + a.nprobe;                                               // [nprobe]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = blockIdx.y, seg = blockIdx.x, S = gridDim.x;
    const bool lut_at_zero =
        reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) unsigned char *)smem) == 0;

#ifdef PIPERAG_TRACE
    unsigned long long *tr = a.trace + ((size_t)qi * S + seg) * 8;
    unsigned nflush = 0;
    if (tid == 0) tr[0] = wall_clock64();
#endif
    {   // stage the query's table and probe tables
        const float4 *src = reinterpret_cast<const float4 *>(a.lut + (size_t)qi * kKsub * MP);
        float4 *dst = reinterpret_cast<float4 *>(s_lut);
        constexpr int kPer = kKsub * MP / 4 / kScanThreads;     // 16-byte pieces per thread (4*C)
        float4 tmp[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) tmp[i] = src[tid + i * kScanThreads];
#pragma unroll
        for (int i = 0; i < kPer; ++i) dst[tid + i * kScanThreads] = tmp[i];
        const int32_t *pf = a.pfx + (size_t)qi * (a.probe_stride + 1);
        for (int i = tid; i <= a.nprobe; i += kScanThreads) s_pfx[i] = pf[i];
        for (int i = tid; i < a.nprobe; i += kScanThreads) {
            const int32_t l = a.probe[(size_t)qi * a.probe_stride + i];
            s_blk[i] = l >= 0 ? a.list_blk[l] : 0;
            s_len[i] = l >= 0 ? a.list_len[l] : 0;
        }
        if (tid == 0) *s_count = 0;
    }
    __syncthreads();

#ifdef PIPERAG_TRACE
    if (tid == 0) tr[1] = wall_clock64();
#endif
    uint32_t thr = 0xFFFFFFFFu;     // best known bound on the k-th best distance (bits)
    const int TB = s_pfx[a.nprobe];
    const int b_begin = (int)((int64_t)TB * seg / S), b_end = (int)((int64_t)TB * (seg + 1) / S);
    const int rounds = (b_end - b_begin + kScanWaves * NSETS - 1) / (kScanWaves * NSETS);   // same for all waves
    const int trigger = cap - kScanThreads * NSETS;      // a round appends at most 256*NSETS keys; trigger >= KP >= k
    const int lane_m = lane % MP;
    uint32_t off4[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        off4[i] = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) off4[i] |= ((uint32_t)((lane + 4 * i + j) & 63) << 2) << (8 * j);
    }

    int b_next = b_begin + wave;    // next block this wave will request
    int pi = 0;                     // probe whose list holds b_next (advanced monotonically)

    struct Meta { uint32_t gblock; int nvalid; uint32_t tg; bool valid; };
    auto issue = [&](uint4 (&w)[C], Meta &m) {
        m.valid = b_next < b_end;
        if (!m.valid) return;
        while (b_next >= s_pfx[pi + 1]) ++pi;                 // b_next < TB = s_pfx[nprobe], so pi stays < nprobe
        const int bl = b_next - s_pfx[pi];
        m.gblock = (uint32_t)(s_blk[pi] + bl);
        m.nvalid = s_len[pi] - bl * kBlockVecs;               // >= 1; lanes >= nvalid hold padding
        const uint4 *blk = reinterpret_cast<const uint4 *>(a.codes + (size_t)m.gblock * kBlockVecs * MP);
#pragma unroll
        for (int c = 0; c < C; ++c) w[c] = blk[c * kWave + lane];
        m.tg = __hip_atomic_load(&a.thr[qi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        b_next += kScanWaves;
    };
    auto process = [&](const uint4 (&w)[C], const Meta &m) {
        float dist;
        if (C == 4 && lut_at_zero) dist = block_dist_m64(reinterpret_cast<const uint4 (&)[4]>(w), off4);
        else dist = block_dist_generic<C>(w, s_lut, lane_m);
        const uint32_t dbits = __float_as_uint(dist);
        thr = min(thr, m.tg);
        const bool pass = (lane < m.nvalid) && (dbits <= thr);
        const uint64_t mask = __ballot(pass);
        if (mask != 0) {
            unsigned base = 0;
            if (lane == 0) base = atomicAdd(s_count, (unsigned)__popcll(mask));
            base = __builtin_amdgcn_readfirstlane(base);
            if (pass) {
                const unsigned slot = base + (unsigned)__popcll(mask & ((1ull << lane) - 1ull));
                if (slot < (unsigned)cap)     // always true (see trigger); keeps a logic error from writing out of bounds
                    s_cand[slot] = ((uint64_t)dbits << 32) | (uint64_t)(m.gblock * kBlockVecs + lane);
            }
        }
    };

    uint4 w[NSETS][C];
    Meta meta[NSETS];
#pragma unroll
    for (int s = 0; s < NSETS; ++s) issue(w[s], meta[s]);
    for (int r = 0; r < rounds; ++r) {
#pragma unroll
        for (int s = 0; s < NSETS; ++s) {
            if (meta[s].valid) process(w[s], meta[s]);
            issue(w[s], meta[s]);
        }
        __syncthreads();
        const int n = (int)*reinterpret_cast<volatile unsigned *>(s_count);
        if (n > trigger) {          // uniform: every thread reads the same value after the barrier
            const uint64_t T = wg_keep_k_smallest(s_cand, min(n, cap), k, s_hist, s_state, s_count);
            const uint32_t kth = (uint32_t)(T >> 32);
            thr = min(thr, kth);
            if (tid == 0) atomicMin(&a.thr[qi], kth);
#ifdef PIPERAG_TRACE
            ++nflush;
#endif
        }
    }
#ifdef PIPERAG_TRACE
    if (tid == 0) { tr[2] = wall_clock64(); tr[5] = nflush; tr[6] = (unsigned long long)(b_end - b_begin); }
#endif
    __syncthreads();
    int n = min((int)*reinterpret_cast<volatile unsigned *>(s_count), cap);
    if (n > k) {
        const uint64_t T = wg_keep_k_smallest(s_cand, n, k, s_hist, s_state, s_count);
        if (tid == 0) atomicMin(&a.thr[qi], (uint32_t)(T >> 32));
        n = k;
    }
#ifdef PIPERAG_TRACE
    if (tid == 0) tr[3] = wall_clock64();
#endif
    uint64_t *out = a.part + ((size_t)qi * S + seg) * k;
    for (int i = tid; i < k; i += kScanThreads) out[i] = i < n ? s_cand[i] : kSentinel;
#ifdef PIPERAG_TRACE
    if (tid == 0) tr[4] = wall_clock64();
#endif
}

// ------------------------------------------------------------------------------------------------
// Stage 4: merge of the partial results of one query + id gather.  One workgroup of 1024 threads per
// query.  Only keys within the query's final bound thr[q] can be among the k best; they are compacted into
// LDS, the k smallest are selected there by radix selection.  If more than kMergeCap keys survive the
// bound (e.g. no workgroup ever collected k candidates, so there is no bound), the selection runs over the
// partial keys in global memory instead.  Then ids are looked up and the k results are sorted by
// (distance, id).
// ------------------------------------------------------------------------------------------------
constexpr int kMergeThreads = 1024;

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(const uint64_t *__restrict__ part, int S, int k,
                                                              const int64_t *__restrict__ ids,
                                                              const uint32_t *__restrict__ thr, float *__restrict__ out_d,
                                                              int64_t *__restrict__ out_i) {
    __shared__ uint64_t s_keys[kMergeCap];
    __shared__ unsigned s_hist[256];
    __shared__ unsigned long long s_state[4];
    __shared__ uint32_t s_d[kMaxK];
    __shared__ int64_t s_id[kMaxK];
    __shared__ unsigned s_count;
    const int qi = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
    const int n = S * k;
    const uint64_t *keys = part + (size_t)qi * n;
    const uint32_t bound = thr[qi];
    const int k2 = max(2, 1 << (32 - __clz(k - 1)));
    for (int i = tid; i < k2; i += nt) { s_d[i] = 0xFFFFFFFFu; s_id[i] = 0x7FFFFFFFFFFFFFFFll; }
    if (tid == 0) s_count = 0;
    __syncthreads();
    for (int i = tid; i < n; i += nt) {
        const uint64_t key = keys[i];
        if (key != kSentinel && (uint32_t)(key >> 32) <= bound) {
            const unsigned slot = atomicAdd(&s_count, 1u);
            if (slot < (unsigned)kMergeCap) s_keys[slot] = key;
        }
    }
    __syncthreads();
    const int found = (int)s_count;
    __syncthreads();
    if (found <= kMergeCap) {
        uint64_t T = kSentinel - 1;                              // fewer than k candidates: keep them all
        if (found > k) {
            auto key_at = [&](int i) { return s_keys[i]; };
            T = block_radix_select(key_at, found, k, s_hist, s_state);
        }
        if (tid == 0) s_count = 0;
        __syncthreads();
        for (int i = tid; i < found; i += nt) {
            const uint64_t key = s_keys[i];
            if (key <= T) {
                const unsigned slot = atomicAdd(&s_count, 1u);   // min(found, k) keys qualify (keys are distinct)
                if (slot < (unsigned)k) {
                    s_d[slot] = (uint32_t)(key >> 32);
                    s_id[slot] = ids[(uint32_t)key];
                }
            }
        }
    } else {
        auto key_at = [&](int i) { return keys[i]; };
        const uint64_t T = block_radix_select(key_at, n, k, s_hist, s_state);
        if (tid == 0) s_count = 0;
        __syncthreads();
        for (int i = tid; i < n; i += nt) {
            const uint64_t key = keys[i];
            if (key <= T && key != kSentinel) {
                const unsigned slot = atomicAdd(&s_count, 1u);   // exactly k keys are <= T (keys are distinct)
                if (slot < (unsigned)k) {
                    s_d[slot] = (uint32_t)(key >> 32);
                    s_id[slot] = ids[(uint32_t)key];
                }
            }
        }
    }
    __syncthreads();
    const int cnt = min((int)s_count, k);
    // bitonic sort of (distance bits, id) pairs
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
        out_d[(size_t)qi * k + i] = i < cnt ? __uint_as_float(s_d[i]) : __builtin_inff();
        out_i[(size_t)qi * k + i] = i < cnt ? s_id[i] : -1;
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
size_t scan_lds_bytes(int Mp, int KP, int nprobe) {
    return (size_t)1024 * Mp + sizeof(uint64_t) * ((size_t)KP + kCandRoom + 4) + sizeof(unsigned) * (256 + 2) +
           sizeof(int32_t) * (3 * (size_t)nprobe + 1);
}

template <int C>
int launch_scan(const ScanArgs &a, int S, int nq, size_t lds, hipStream_t st) {
    constexpr int NSETS = C <= 4 ? 4 : (C <= 6 ? 2 : 1);   // code blocks in flight per wave: as many as fit without register spills
    static size_t configured = 0;
    if (lds > configured) {
        PR_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&adc_scan_kernel<C, NSETS>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = lds;
    }
    hipLaunchKernelGGL((adc_scan_kernel<C, NSETS>), dim3(S, nq), dim3(kScanThreads), lds, st, a);
    return PIPERAG_OK;
}

int launch_coarse(const piperag_index *ix, const float *q, int nq, hipStream_t st) {
    constexpr int QT = 4;
    const int d = ix->p.d, nlist = ix->p.nlist;
    const int groups = std::min((nlist + 3) / 4, 2048);
    const dim3 grid(groups, (nq + QT - 1) / QT);
    const size_t lds = sizeof(float) * QT * d;
    static size_t configured = 48 * 1024;
    if (lds > configured) {
        PR_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&coarse_rowwise_kernel<QT, 4>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        PR_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&coarse_rowwise_kernel<QT, 1>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = lds;
    }
    if (d % 4 == 0)
        hipLaunchKernelGGL((coarse_rowwise_kernel<QT, 4>), grid, dim3(256), lds, st, q, ix->centroids, ix->ws_D, nq, nlist, d);
    else
        hipLaunchKernelGGL((coarse_rowwise_kernel<QT, 1>), grid, dim3(256), lds, st, q, ix->centroids, ix->ws_D, nq, nlist, d);
    return PIPERAG_OK;
}

#ifdef PIPERAG_TRACE
unsigned long long *g_trace_buf = nullptr;
int g_trace_n = 0;
#endif

int check_search_args(const piperag_index *ix, const void *q, int32_t nq, int32_t nprobe, int32_t k, const void *od,
                      const void *oi) {
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(ix->finalized, PIPERAG_ERR_ARG, "index is not finalized");
    PR_REQUIRE(nq >= 0, PIPERAG_ERR_ARG, "nq = %d is negative", nq);
    if (nq == 0) return PIPERAG_OK;
    PR_REQUIRE(q && od && oi, PIPERAG_ERR_ARG, "queries / output pointer is NULL");
    PR_REQUIRE(nq <= ix->p.max_nq, PIPERAG_ERR_LIMIT, "nq = %d exceeds max_nq = %d", nq, ix->p.max_nq);
    PR_REQUIRE(nprobe >= 1 && k >= 1, PIPERAG_ERR_ARG, "nprobe = %d and k = %d must be >= 1", nprobe, k);
    PR_REQUIRE(nprobe <= ix->p.nlist, PIPERAG_ERR_ARG, "nprobe = %d exceeds nlist = %d", nprobe, ix->p.nlist);
    PR_REQUIRE(nprobe <= ix->p.max_nprobe, PIPERAG_ERR_LIMIT, "nprobe = %d exceeds max_nprobe = %d", nprobe, ix->p.max_nprobe);
    PR_REQUIRE(k <= ix->p.max_k, PIPERAG_ERR_LIMIT, "k = %d exceeds max_k = %d", k, ix->p.max_k);
    return PIPERAG_OK;
}

int search_impl(const piperag_index *cix, const float *q, int32_t nq, const int32_t *probes, int32_t nprobe, int32_t k,
                float *out_d, int64_t *out_i, hipStream_t st) {
    piperag_index *ix = const_cast<piperag_index *>(cix);   // workspace and timing state are mutable
    int rc = check_search_args(ix, q, nq, nprobe, k, out_d, out_i);
    if (rc != PIPERAG_OK || nq == 0) return rc;
    PR_CHECK_HIP(hipSetDevice(ix->device));
    const int pstride = ix->p.max_nprobe;
    const bool tm = ix->timing;
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[0], st));
    if (!probes && (rc = launch_coarse(ix, q, nq, st)) != PIPERAG_OK) return rc;
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[1], st));
    if (!probes)
        hipLaunchKernelGGL(select_probes_kernel, dim3(nq), dim3(256), 0, st, ix->ws_D, ix->p.nlist, nprobe, ix->ws_probe,
                           ix->ws_probe_d, pstride);
    else
        hipLaunchKernelGGL(copy_probes_kernel, dim3(nq), dim3(64), 0, st, probes, nprobe, ix->p.nlist, ix->ws_probe, pstride);
    hipLaunchKernelGGL(plan_kernel, dim3(nq), dim3(64), 0, st, ix->ws_probe, pstride, nprobe, ix->list_blk, ix->list_len,
                       ix->ws_pfx, ix->ws_scanned, ix->ws_thr);
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[2], st));
    hipLaunchKernelGGL(lut_kernel, dim3(ix->Mp, nq), dim3(256), 0, st, q, ix->pq, ix->p.d, ix->p.M, ix->dsub, ix->Mp,
                       ix->ws_lut, 0);
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[3], st));

    const int KP = std::max(kWave, next_pow2(k));
    static const int target_wgs = [] {                      // tuning override, read once
        const char *e = getenv("PIPERAG_SCAN_WGS");
        const int v = e ? atoi(e) : 0;
        return v > 0 && v <= 2 * kTargetScanWGs ? v : kTargetScanWGs;
    }();
    int S = (target_wgs + nq - 1) / nq;
    S = std::max(1, std::min(S, kMaxSegments));
    ScanArgs a{ix->codes, ix->ws_lut, ix->ws_probe, ix->ws_pfx, ix->list_blk, ix->list_len, ix->ws_part, ix->ws_thr, nprobe, pstride, k, KP};
#ifdef PIPERAG_TRACE
    static unsigned long long *trace_buf = nullptr;
    if (!trace_buf) PR_CHECK_HIP(hipMalloc((void **)&trace_buf, 8 * sizeof(unsigned long long) * 8192));
    a.trace = trace_buf;
    g_trace_buf = trace_buf; g_trace_n = S * nq;
#endif
    const size_t lds = scan_lds_bytes(ix->Mp, KP, nprobe);
    PR_REQUIRE(lds <= 160 * 1024, PIPERAG_ERR_LIMIT, "scan needs %zu bytes of LDS (M, k, nprobe too large together)", lds);
    switch (ix->Mp / 16) {
        case 1: rc = launch_scan<1>(a, S, nq, lds, st); break;
        case 2: rc = launch_scan<2>(a, S, nq, lds, st); break;
        case 3: rc = launch_scan<3>(a, S, nq, lds, st); break;
        case 4: rc = launch_scan<4>(a, S, nq, lds, st); break;
        case 5: rc = launch_scan<5>(a, S, nq, lds, st); break;
        case 6: rc = launch_scan<6>(a, S, nq, lds, st); break;
        case 7: rc = launch_scan<7>(a, S, nq, lds, st); break;
        case 8: rc = launch_scan<8>(a, S, nq, lds, st); break;
        default: PR_REQUIRE(false, PIPERAG_ERR_ARG, "unsupported M");
    }
    if (rc != PIPERAG_OK) return rc;
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[4], st));
    hipLaunchKernelGGL(merge_kernel, dim3(nq), dim3(kMergeThreads), 0, st, ix->ws_part, S, k, ix->ids, ix->ws_thr, out_d, out_i);
    if (tm) { PR_CHECK_HIP(hipEventRecord(ix->ev[5], st)); ix->ev_valid = true; }
    ix->last_nq = nq;
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

}  // namespace

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

int piperag_ivf_coarse(const piperag_index *index, const float *queries_dev, int32_t nq, int32_t nprobe,
                       int32_t *out_lists_dev, float *out_dist_dev, void *stream) {
    piperag_index *ix = const_cast<piperag_index *>(index);
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(nq >= 0, PIPERAG_ERR_ARG, "nq = %d is negative", nq);
    if (nq == 0) return PIPERAG_OK;
    PR_REQUIRE(queries_dev && out_lists_dev, PIPERAG_ERR_ARG, "queries / output pointer is NULL");
    PR_REQUIRE(nq <= ix->p.max_nq, PIPERAG_ERR_LIMIT, "nq = %d exceeds max_nq = %d", nq, ix->p.max_nq);
    PR_REQUIRE(nprobe >= 1 && nprobe <= ix->p.nlist, PIPERAG_ERR_ARG, "nprobe = %d out of range", nprobe);
    PR_REQUIRE(nprobe <= ix->p.max_nprobe, PIPERAG_ERR_LIMIT, "nprobe = %d exceeds max_nprobe = %d", nprobe, ix->p.max_nprobe);
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(ix->device));
    const int rc = launch_coarse(ix, queries_dev, nq, st);
    if (rc != PIPERAG_OK) return rc;
    hipLaunchKernelGGL(select_probes_kernel, dim3(nq), dim3(256), 0, st, ix->ws_D, ix->p.nlist, nprobe, ix->ws_probe,
                       ix->ws_probe_d, ix->p.max_nprobe);
    PR_CHECK_HIP(hipMemcpy2DAsync(out_lists_dev, sizeof(int32_t) * nprobe, ix->ws_probe, sizeof(int32_t) * ix->p.max_nprobe,
                                  sizeof(int32_t) * nprobe, nq, hipMemcpyDeviceToDevice, st));
    if (out_dist_dev)
        PR_CHECK_HIP(hipMemcpy2DAsync(out_dist_dev, sizeof(float) * nprobe, ix->ws_probe_d, sizeof(float) * ix->p.max_nprobe,
                                      sizeof(float) * nprobe, nq, hipMemcpyDeviceToDevice, st));
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

int piperag_ivf_lut(const piperag_index *index, const float *queries_dev, int32_t nq, float *out_lut_dev, void *stream) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(nq >= 0, PIPERAG_ERR_ARG, "nq = %d is negative", nq);
    if (nq == 0) return PIPERAG_OK;
    PR_REQUIRE(queries_dev && out_lut_dev, PIPERAG_ERR_ARG, "queries / output pointer is NULL");
    PR_CHECK_HIP(hipSetDevice(index->device));
    hipLaunchKernelGGL(lut_kernel, dim3(index->p.M, nq), dim3(256), 0, (hipStream_t)stream, queries_dev, index->pq, index->p.d,
                       index->p.M, index->dsub, index->Mp, out_lut_dev, 1);
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

#ifdef PIPERAG_TRACE
__attribute__((visibility("default"))) int piperag_debug_trace(unsigned long long *out_host, int max_wg) {
    const int n = g_trace_n < max_wg ? g_trace_n : max_wg;
    if (hipMemcpy(out_host, g_trace_buf, sizeof(unsigned long long) * 8 * n, hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return n;
}
#endif

int piperag_search_stats(const piperag_index *index, int64_t *scanned_vectors, int64_t *scanned_code_bytes) {
    PR_REQUIRE(index != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    int64_t total = 0;
    if (index->last_nq > 0) {
        std::vector<int64_t> h(index->last_nq);
        PR_CHECK_HIP(hipMemcpy(h.data(), index->ws_scanned, sizeof(int64_t) * h.size(), hipMemcpyDeviceToHost));
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
