// Search path of libpiperag: coarse quantiser, top-nprobe selection, scan plan, lookup-table build,
// list scan with k-selection, merge + id gather.  All kernels are written for gfx950 (wave64).
//
// Method: Section 3.2 (S3) of the paper - nprobe of the nlist inverted lists are selected per query and
// the product-quantised vectors inside them are compared with the query; Section 2 - the k closest are
// returned.  The retrieval latency model of S3 splits the time into an index-scan term (stages 0-1 here)
// and a vector-scan term proportional to nprobe (stages 2-4).
#include <algorithm>
#include <vector>

#include "common.h"

using namespace piperag;

namespace {

// ------------------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void wave_sync() {
    // Orders LDS traffic between the lanes of one wavefront (no s_barrier needed: a wave runs in lock-step).
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// k-th smallest (1-based `kth`) of n 64-bit keys, by most-significant-digit radix selection with the whole
// workgroup.  key_at(i) may be evaluated several times.  Requires 1 <= kth <= n.
template <class KeyFn>
__device__ uint64_t block_radix_select(KeyFn key_at, int n, int kth, unsigned *s_hist /*[256]*/,
                                       unsigned long long *s_state /*[2]*/) {
    const int tid = threadIdx.x, nt = blockDim.x;
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
        if (tid == 0) {
            unsigned cum = 0;
            int dgt = 0;
            for (; dgt < 255; ++dgt) {
                const unsigned c = s_hist[dgt];
                if (cum + c >= (unsigned)kth) break;
                cum += c;
            }
            s_state[0] = prefix | ((uint64_t)dgt << shift);
            s_state[1] = (unsigned long long)(kth - (int)cum);
        }
        __syncthreads();
        prefix = s_state[0];
        kth = (int)s_state[1];
        __syncthreads();
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
    __shared__ unsigned long long s_state[2];
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
// scanned[q] = number of vectors in its probed lists.
__global__ void plan_kernel(const int32_t *__restrict__ probe, int probe_stride, int nprobe,
                            const int32_t *__restrict__ list_blk, const int32_t *__restrict__ list_len,
                            int32_t *__restrict__ pfx, int64_t *__restrict__ scanned) {
    const int qi = blockIdx.x;
    if (threadIdx.x != 0) return;
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
// and adds Mp table entries from LDS.  Because of the rotated code layout (see common.h), at step t lane l
// looks up sub-quantiser (l + t) mod Mp, so with the table stored [j][Mp] the lanes of a half-wave hit
// different LDS banks when Mp is 32 or 64.
// k-selection: each wave keeps its k best (distance bits << 32 | slot) sorted in LDS, filters candidates
// against the current k-th best, queues the survivors and merges the queue when it fills up.  At the end
// the 4 wave lists are merged and written to the partial-result buffer.
// ------------------------------------------------------------------------------------------------
struct ScanArgs {
    const uint8_t *codes;
    const float *lut;
    const int32_t *probe;
    const int32_t *pfx;
    const int32_t *list_blk;
    const int32_t *list_len;
    uint64_t *part;
    int nprobe, probe_stride, k, KP;
};

// Number of keys in sorted[0..n) that are smaller than key.
__device__ __forceinline__ int lower_bound_u64(const uint64_t *sorted, int n, uint64_t key) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (sorted[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Merges the wave's pending queue into its sorted best list (double-buffered: cur -> alt, then swapped).
__device__ void wave_flush(uint64_t *&cur, uint64_t *&alt, const uint64_t *queue, int qn, int k, int KP, int lane) {
    wave_sync();
    for (int i = lane; i < KP; i += kWave) alt[i] = kSentinel;
    wave_sync();
    for (int i = lane; i < qn; i += kWave) {
        const uint64_t key = queue[i];
        int r = lower_bound_u64(cur, KP, key);
        for (int j = 0; j < qn; ++j) r += (queue[j] < key) ? 1 : 0;
        if (r < k) alt[r] = key;
    }
    for (int i = lane; i < KP; i += kWave) {
        const uint64_t key = cur[i];
        if (key != kSentinel) {
            int r = i;
            for (int j = 0; j < qn; ++j) r += (queue[j] < key) ? 1 : 0;
            if (r < k) alt[r] = key;
        }
    }
    wave_sync();
    uint64_t *t = cur; cur = alt; alt = t;
}

template <int C>
__global__ __launch_bounds__(kScanThreads) void adc_scan_kernel(ScanArgs a) {
    constexpr int MP = 16 * C;
    extern __shared__ __align__(16) unsigned char smem[];
    float *s_lut = reinterpret_cast<float *>(smem);                                  // [256*MP]
    uint64_t *s_best = reinterpret_cast<uint64_t *>(smem + (size_t)1024 * MP);       // [4 waves][2][KP]
    uint64_t *s_queue = s_best + kScanWaves * 2 * a.KP;                              // [4][kQueueCap]
    uint64_t *s_wg = s_queue + kScanWaves * kQueueCap;                               // [KP]
    int32_t *s_pfx = reinterpret_cast<int32_t *>(s_wg + a.KP);                       // [nprobe+1]
    int32_t *s_blk = s_pfx + (a.nprobe + 1);                                         // [nprobe]
    int32_t *s_len = s_blk + a.nprobe;                                               // [nprobe]
    __shared__ int s_sel[kScanWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = blockIdx.y, seg = blockIdx.x, S = gridDim.x;
    const int k = a.k, KP = a.KP;

    {   // stage the query's table and probe tables
        const float4 *src = reinterpret_cast<const float4 *>(a.lut + (size_t)qi * kKsub * MP);
        float4 *dst = reinterpret_cast<float4 *>(s_lut);
        for (int i = tid; i < kKsub * MP / 4; i += kScanThreads) dst[i] = src[i];
        const int32_t *pf = a.pfx + (size_t)qi * (a.probe_stride + 1);
        for (int i = tid; i <= a.nprobe; i += kScanThreads) s_pfx[i] = pf[i];
        for (int i = tid; i < a.nprobe; i += kScanThreads) {
            const int32_t l = a.probe[(size_t)qi * a.probe_stride + i];
            s_blk[i] = l >= 0 ? a.list_blk[l] : 0;
            s_len[i] = l >= 0 ? a.list_len[l] : 0;
        }
        for (int i = tid; i < kScanWaves * 2 * KP; i += kScanThreads) s_best[i] = kSentinel;
    }
    __syncthreads();

    uint64_t *cur = s_best + (size_t)wave * 2 * KP, *alt = cur + KP;
    uint64_t *queue = s_queue + (size_t)wave * kQueueCap;
    int qn = 0;
    uint32_t thr = 0xFFFFFFFFu;     // distance bits of the wave's current k-th best

    const int TB = s_pfx[a.nprobe];
    const int b_begin = (int)((int64_t)TB * seg / S), b_end = (int)((int64_t)TB * (seg + 1) / S);
    const int lane_m = lane % MP;
    int pi = 0;

    for (int b = b_begin + wave; b < b_end; b += kScanWaves) {
        while (b >= s_pfx[pi + 1]) ++pi;                     // b < TB = s_pfx[nprobe], so pi stays < nprobe
        const int bl = b - s_pfx[pi];
        const uint32_t gblock = (uint32_t)(s_blk[pi] + bl);
        const int nvalid = s_len[pi] - bl * kBlockVecs;      // >= 1; lanes >= nvalid hold padding
        const uint4 *blk = reinterpret_cast<const uint4 *>(a.codes + (size_t)gblock * kBlockVecs * MP);
        uint4 w[C];
#pragma unroll
        for (int c = 0; c < C; ++c) w[c] = blk[c * kWave + lane];

        float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const uint32_t ww[4] = {w[c].x, w[c].y, w[c].z, w[c].w};
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int t = c * 16 + u;
                int m = lane_m + t;
                if (m >= MP) m -= MP;
                const uint32_t byte = (ww[u >> 2] >> (8 * (u & 3))) & 0xFFu;
                const float v = s_lut[byte * MP + m];
                if ((u & 3) == 0) acc0 += v; else if ((u & 3) == 1) acc1 += v; else if ((u & 3) == 2) acc2 += v; else acc3 += v;
            }
        }
        const float dist = (acc0 + acc1) + (acc2 + acc3);
        const uint32_t dbits = __float_as_uint(dist);
        const bool pass = (lane < nvalid) && (dbits <= thr);
        const uint64_t mask = __ballot(pass);
        if (mask != 0) {
            if (pass) {
                const int off = __popcll(mask & ((1ull << lane) - 1ull));
                queue[qn + off] = ((uint64_t)dbits << 32) | (uint64_t)(gblock * kBlockVecs + lane);
            }
            qn += __popcll(mask);
            if (qn > kQueueCap - kWave) {
                wave_flush(cur, alt, queue, qn, k, KP, lane);
                qn = 0;
                thr = (uint32_t)(cur[k - 1] >> 32);
            }
        }
    }
    if (qn > 0) wave_flush(cur, alt, queue, qn, k, KP, lane);
    if (lane == 0) s_sel[wave] = (cur == s_best + (size_t)wave * 2 * KP) ? 0 : 1;
    for (int i = tid; i < KP; i += kScanThreads) s_wg[i] = kSentinel;
    __syncthreads();

    // merge the four sorted wave lists: rank of a key = its index + number of smaller keys in the other lists
    for (int e = tid; e < kScanWaves * KP; e += kScanThreads) {
        const int w = e / KP, i = e - w * KP;
        const uint64_t *mine = s_best + ((size_t)w * 2 + s_sel[w]) * KP;
        const uint64_t key = mine[i];
        if (key == kSentinel) continue;
        int r = i;
        for (int o = 0; o < kScanWaves; ++o) {
            if (o == w) continue;
            r += lower_bound_u64(s_best + ((size_t)o * 2 + s_sel[o]) * KP, KP, key);
        }
        if (r < k) s_wg[r] = key;
    }
    __syncthreads();
    uint64_t *out = a.part + ((size_t)qi * S + seg) * k;
    for (int i = tid; i < k; i += kScanThreads) out[i] = s_wg[i];
}

// ------------------------------------------------------------------------------------------------
// Stage 4: merge of the partial results of one query + id gather.  One workgroup per query: radix
// selection of the k-th smallest key over the S*k partial keys, compaction, id lookup, bitonic sort by
// (distance, id), padded output.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void merge_kernel(const uint64_t *__restrict__ part, int S, int k,
                                                    const int64_t *__restrict__ ids, float *__restrict__ out_d,
                                                    int64_t *__restrict__ out_i) {
    __shared__ unsigned s_hist[256];
    __shared__ unsigned long long s_state[2];
    __shared__ uint32_t s_d[kMaxK];
    __shared__ int64_t s_id[kMaxK];
    __shared__ unsigned s_count;
    const int qi = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
    const int n = S * k;
    const uint64_t *keys = part + (size_t)qi * n;
    auto key_at = [&](int i) { return keys[i]; };
    const uint64_t T = block_radix_select(key_at, n, k, s_hist, s_state);
    const int k2 = max(2, 1 << (32 - __clz(k - 1)));
    for (int i = tid; i < k2; i += nt) { s_d[i] = 0xFFFFFFFFu; s_id[i] = 0x7FFFFFFFFFFFFFFFll; }
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
    return (size_t)1024 * Mp + sizeof(uint64_t) * ((size_t)kScanWaves * 2 * KP + kScanWaves * kQueueCap + KP) +
           sizeof(int32_t) * (3 * (size_t)nprobe + 1);
}

template <int C>
int launch_scan(const ScanArgs &a, int S, int nq, size_t lds, hipStream_t st) {
    static size_t configured = 0;
    if (lds > configured) {
        PR_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&adc_scan_kernel<C>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = lds;
    }
    hipLaunchKernelGGL(adc_scan_kernel<C>, dim3(S, nq), dim3(kScanThreads), lds, st, a);
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
                       ix->ws_pfx, ix->ws_scanned);
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[2], st));
    hipLaunchKernelGGL(lut_kernel, dim3(ix->Mp, nq), dim3(256), 0, st, q, ix->pq, ix->p.d, ix->p.M, ix->dsub, ix->Mp,
                       ix->ws_lut, 0);
    if (tm) PR_CHECK_HIP(hipEventRecord(ix->ev[3], st));

    const int KP = std::max(kWave, next_pow2(k));
    int S = (kTargetScanWGs + nq - 1) / nq;
    S = std::max(1, std::min(S, kMaxSegments));
    ScanArgs a{ix->codes, ix->ws_lut, ix->ws_probe, ix->ws_pfx, ix->list_blk, ix->list_len, ix->ws_part, nprobe, pstride, k, KP};
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
    hipLaunchKernelGGL(merge_kernel, dim3(nq), dim3(256), 0, st, ix->ws_part, S, k, ix->ids, out_d, out_i);
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
