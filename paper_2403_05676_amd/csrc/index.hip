// Index object of libpiperag: creation, staging of encoded vectors, grouping into inverted lists
// (Section 3.2, S3: the database is clustered into nlist lists) in the scan layout, file load / save and
// list read-back.
#include <stdarg.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "common.h"

using namespace piperag;

namespace piperag {
static thread_local char g_err[512] = "";
void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
}  // namespace piperag

namespace {

constexpr int kPlaceTile = 256;

// H[g][l] += 1 for every staged vector of chunk g (chunk = `chunk` consecutive staging entries).
__global__ void hist_kernel(const int32_t *__restrict__ st_list, int64_t n, int64_t chunk, int nlist,
                            uint32_t *__restrict__ H) {
    const int g = blockIdx.x;
    const int64_t a = (int64_t)g * chunk, b = min(n, a + chunk);
    for (int64_t i = a + threadIdx.x; i < b; i += blockDim.x) atomicAdd(&H[(size_t)g * nlist + st_list[i]], 1u);
}

// Turns H into exclusive prefix sums over the chunks (per list).  Without a cursor the sums start at 0 and the
// totals are written to list_len (the whole staging area at once); with a cursor they start at cursor[l], the
// number of entries of list l placed by earlier tiles, and the cursor moves on by the tile's total.
__global__ void colscan_kernel(uint32_t *__restrict__ H, int G, int nlist, int32_t *__restrict__ list_len,
                               uint32_t *__restrict__ cursor) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= nlist) return;
    uint32_t run = cursor ? cursor[l] : 0;
    for (int g = 0; g < G; ++g) {
        const uint32_t c = H[(size_t)g * nlist + l];
        H[(size_t)g * nlist + l] = run;
        run += c;
    }
    if (cursor) cursor[l] = run; else list_len[l] = (int32_t)run;
}

// counts[l] += number of entries with list l
__global__ void count_lists_kernel(const int32_t *__restrict__ lists, int64_t n, uint32_t *__restrict__ counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) atomicAdd(&counts[lists[i]], 1u);
}
__global__ void counts_to_len_kernel(const uint32_t *__restrict__ counts, int nlist, int32_t *__restrict__ list_len) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l < nlist) list_len[l] = (int32_t)counts[l];
}

// list_blk[l] = sum over l' < l of ceil(len[l'] / 64); one workgroup, sequential over tiles of 1024 lists.
__global__ __launch_bounds__(1024) void blockscan_kernel(const int32_t *__restrict__ list_len, int nlist,
                                                         int32_t *__restrict__ list_blk) {
    __shared__ int32_t s[1024];
    __shared__ int32_t s_base;
    if (threadIdx.x == 0) s_base = 0;
    __syncthreads();
    for (int l0 = 0; l0 < nlist; l0 += 1024) {
        const int l = l0 + threadIdx.x;
        const int32_t v = l < nlist ? (list_len[l] + kBlockVecs - 1) / kBlockVecs : 0;
        s[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {     // Hillis-Steele inclusive scan
            const int32_t add = threadIdx.x >= off ? s[threadIdx.x - off] : 0;
            __syncthreads();
            s[threadIdx.x] += add;
            __syncthreads();
        }
        const int32_t base = s_base;
        if (l < nlist) list_blk[l] = base + s[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 1023) s_base = base + s[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0) list_blk[nlist] = s_base;
}

// Byte address of code byte position t of slot `slot` in the scan layout.
__device__ __forceinline__ size_t scan_offset(uint32_t slot, int t, int Mp) {
    const uint32_t block = slot / kBlockVecs, lane = slot % kBlockVecs;
    return (size_t)block * kBlockVecs * Mp + (size_t)(t >> 4) * 1024 + lane * 16 + (t & 15);
}

// Stable placement: workgroup g walks its chunk of the staging area in order, 256 entries at a time.  The
// slot of an entry inside its list = running count of that list before the tile (H, owned by this
// workgroup) + number of earlier entries of the tile with the same list.
__global__ __launch_bounds__(kPlaceTile) void place_kernel(const int32_t *__restrict__ st_list,
                                                           const uint8_t *__restrict__ st_codes,
                                                           const int64_t *__restrict__ st_ids, int64_t n, int64_t chunk,
                                                           int nlist, int M, int Mp, uint32_t *H,
                                                           const int32_t *__restrict__ list_blk, uint8_t *__restrict__ codes,
                                                           int64_t *__restrict__ ids) {
    __shared__ int32_t s_l[kPlaceTile];
    const int g = blockIdx.x, tid = threadIdx.x;
    const int64_t a = (int64_t)g * chunk, b = min(n, a + chunk);
    uint32_t *Hg = H + (size_t)g * nlist;
    for (int64_t i0 = a; i0 < b; i0 += kPlaceTile) {
        const int64_t i = i0 + tid;
        const int32_t l = i < b ? st_list[i] : -1;
        s_l[tid] = l;
        __syncthreads();
        uint32_t slot = 0, in_list = 0;
        bool last = false;
        if (l >= 0) {
            int before = 0;
            last = true;
            for (int t = 0; t < kPlaceTile; ++t) {
                const bool same = s_l[t] == l;
                before += (same && t < tid) ? 1 : 0;
                last = last && !(same && t > tid);
            }
            in_list = Hg[l] + (uint32_t)before;
            slot = (uint32_t)list_blk[l] * kBlockVecs + in_list;
        }
        __syncthreads();                           // every read of Hg and s_l for this tile is done
        if (l >= 0 && last) Hg[l] = in_list + 1;
        __syncthreads();                           // counter updates visible to the next tile
        if (l >= 0) {
            ids[slot] = st_ids[i];
            const uint8_t *src = st_codes + (size_t)i * M;
            const int lane = slot % kBlockVecs;
            for (int t = 0; t < Mp; ++t) {
                const int m = (lane + t) % Mp;
                codes[scan_offset(slot, t, Mp)] = m < M ? src[m] : (uint8_t)0;
            }
        }
    }
}

// Inverse of the placement for one list: canonical rows out.
__global__ void gather_list_kernel(const uint8_t *__restrict__ codes, const int64_t *__restrict__ ids, uint32_t slot0,
                                   int64_t i0, int64_t count, int M, int Mp, uint8_t *__restrict__ out_codes,
                                   int64_t *__restrict__ out_ids) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const uint32_t slot = slot0 + (uint32_t)(i0 + i);
    const int lane = slot % kBlockVecs;
    if (out_ids) out_ids[i] = ids[slot];
    if (out_codes) {
        for (int m = 0; m < M; ++m) {
            const int t = ((m - lane) % Mp + Mp) % Mp;
            out_codes[(size_t)i * M + m] = codes[scan_offset(slot, t, Mp)];
        }
    }
}

// Residual indexes: tx[slot] = 2 <c_l, decode(code in slot)> for every slot of the scan layout (0 for padding).
// One wavefront per block of 64 slots; the block's list is found by bisection of list_blk.
__global__ __launch_bounds__(64) void residual_term_kernel(const uint8_t *__restrict__ codes, const int32_t *__restrict__ list_blk,
                                                           const int32_t *__restrict__ list_len, int nlist,
                                                           const float *__restrict__ cent, const float *__restrict__ pq, int d,
                                                           int M, int Mp, int dsub, float *__restrict__ tx) {
    const uint32_t block = blockIdx.x, lane = threadIdx.x;
    int lo = 0, hi = nlist;                                 // last list whose first block is <= block and that is not empty there
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((uint32_t)list_blk[mid] <= block) lo = mid; else hi = mid;
    }
    const int l = lo;
    const uint32_t slot = block * kBlockVecs + lane;
    const int in_list = (int)(slot - (uint32_t)list_blk[l] * kBlockVecs);
    float acc = 0.f;
    if (in_list < list_len[l]) {
        const float *c = cent + (size_t)l * d;
        for (int t = 0; t < Mp; ++t) {
            const int m = (int)((lane + t) % Mp);
            if (m >= M) continue;
            const int code = codes[(size_t)block * kBlockVecs * Mp + (size_t)(t >> 4) * 1024 + lane * 16 + (t & 15)];
            const float *pc = pq + ((size_t)m * kKsub + code) * dsub;
            for (int u = 0; u < dsub; ++u) acc += c[m * dsub + u] * pc[u];
        }
    }
    tx[slot] = 2.f * acc;
}

__global__ void fill_u32_kernel(uint32_t *__restrict__ dst, size_t n, uint32_t v) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}

__global__ void iota_ids_kernel(int64_t *__restrict__ dst, int64_t n, int64_t first) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = first + i;
}

__global__ void check_lists_kernel(const int32_t *__restrict__ lists, int64_t n, int nlist, int *__restrict__ bad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && (lists[i] < 0 || lists[i] >= nlist)) *bad = 1;
}

template <class T>
int dev_alloc(T **p, size_t count) {
    *p = nullptr;
    if (count == 0) count = 1;
    PR_CHECK_HIP(hipMalloc(reinterpret_cast<void **>(p), count * sizeof(T)));
    return PIPERAG_OK;
}

#define PR_TRY(expr)                      \
    do {                                  \
        int rc__ = (expr);                \
        if (rc__ != PIPERAG_OK) return rc__; \
    } while (0)

int check_params(const piperag_params *p) {
    PR_REQUIRE(p != nullptr, PIPERAG_ERR_ARG, "params is NULL");
    PR_REQUIRE(p->nbits == 8, PIPERAG_ERR_ARG, "nbits = %d: only 8-bit sub-quantisers are supported", p->nbits);
    PR_REQUIRE(p->residual == 0 || p->residual == 1, PIPERAG_ERR_ARG, "residual = %d must be 0 or 1", p->residual);
    PR_REQUIRE(p->M >= 1 && p->M <= 128, PIPERAG_ERR_ARG, "M = %d out of range 1..128", p->M);
    PR_REQUIRE(p->d >= 1 && p->d % p->M == 0, PIPERAG_ERR_ARG, "d = %d must be a positive multiple of M = %d", p->d, p->M);
    PR_REQUIRE(p->d <= 8192, PIPERAG_ERR_ARG, "d = %d exceeds 8192", p->d);
    PR_REQUIRE(p->nlist >= 1 && p->nlist <= (1 << 20), PIPERAG_ERR_ARG, "nlist = %d out of range 1..2^20", p->nlist);
    PR_REQUIRE(p->ntotal >= 0 && p->ntotal <= 0xFFF00000ll, PIPERAG_ERR_ARG, "ntotal = %lld out of range", (long long)p->ntotal);
    PR_REQUIRE(p->max_nq >= 1 && p->max_nq <= 65535, PIPERAG_ERR_ARG, "max_nq = %d out of range 1..65535", p->max_nq);
    PR_REQUIRE(p->max_nprobe >= 1 && p->max_nprobe <= kMaxNprobe, PIPERAG_ERR_ARG, "max_nprobe = %d out of range 1..%d",
               p->max_nprobe, kMaxNprobe);
    PR_REQUIRE(p->max_k >= 1 && p->max_k <= kMaxK, PIPERAG_ERR_ARG, "max_k = %d out of range 1..%d", p->max_k, kMaxK);
    return PIPERAG_OK;
}

void free_staging(piperag_index *ix) {
    (void)hipFree(ix->st_list); ix->st_list = nullptr;
    (void)hipFree(ix->st_codes); ix->st_codes = nullptr;
    (void)hipFree(ix->st_ids); ix->st_ids = nullptr;
    (void)hipFree(ix->bd_counts); ix->bd_counts = nullptr;
    (void)hipFree(ix->bd_cursor); ix->bd_cursor = nullptr;
}

int create_impl(const piperag_params *params, const float *cent_host, const float *pq_host, piperag_index **out) {
    PR_REQUIRE(out != nullptr, PIPERAG_ERR_ARG, "out is NULL");
    *out = nullptr;
    PR_TRY(check_params(params));
    PR_REQUIRE(cent_host && pq_host, PIPERAG_ERR_ARG, "centroids / codebook pointer is NULL");
    piperag_index *ix = new (std::nothrow) piperag_index();
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_OOM, "host allocation failed");
    memset(ix, 0, sizeof(*ix));
    ix->p = *params;
    ix->streaming = -1;
    ix->p.max_nprobe = std::min(ix->p.max_nprobe, ix->p.nlist);
    ix->dsub = params->d / params->M;
    ix->Mp = round_up(params->M, 16);
    ix->cap = params->ntotal;
    int rc = PIPERAG_OK;
    auto fail = [&](int code) { piperag_ivf_free(ix); return code; };
    if (hipGetDevice(&ix->device) != hipSuccess) { set_error("hipGetDevice failed"); return fail(PIPERAG_ERR_HIP); }
    if (hipDeviceGetAttribute(&ix->ncu, hipDeviceAttributeMultiprocessorCount, ix->device) != hipSuccess || ix->ncu < 1) {
        set_error("cannot read the number of compute units");
        return fail(PIPERAG_ERR_HIP);
    }
    const piperag_params &p = ix->p;
    const size_t ncent = (size_t)p.nlist * p.d, npq = (size_t)p.M * kKsub * ix->dsub;
    if ((rc = dev_alloc(&ix->centroids, ncent)) || (rc = dev_alloc(&ix->pq, npq)) ||
        (rc = dev_alloc(&ix->list_blk, (size_t)p.nlist + 1)) ||
        (rc = dev_alloc(&ix->list_len, (size_t)p.nlist)) ||
        (rc = dev_alloc(&ix->pqT, npq)) || (rc = dev_alloc(&ix->pqE, (size_t)p.M * pqe_rows(ix->dsub) * kKsub)) || (rc = dev_alloc(&ix->cnorm, (size_t)p.nlist)) ||
        (rc = dev_alloc(&ix->ws_out_d, (size_t)p.max_nq * p.max_k)) ||
        (rc = dev_alloc(&ix->ws_out_i, (size_t)p.max_nq * p.max_k)) || (rc = dev_alloc(&ix->flag, 1)))
        return fail(rc);
    if ((rc = configure_search_kernels(ix->device)) || (rc = configure_encode_kernels(ix->device))) return fail(rc);
    {   // the search workspace: one block, carved up by search_ws_layout
        const size_t ws_bytes = search_ws_layout(&ix->ws, nullptr, p.nlist, ix->Mp, p.max_nq, p.max_nprobe, p.max_k, kMaxScanWGs);
        if (hipMalloc(&ix->ws_mem, ws_bytes) != hipSuccess) { set_error("out of device memory for %zu bytes of search workspace", ws_bytes); return fail(PIPERAG_ERR_OOM); }
        search_ws_layout(&ix->ws, ix->ws_mem, p.nlist, ix->Mp, p.max_nq, p.max_nprobe, p.max_k, kMaxScanWGs);
    }
    if (hipMemset(ix->ws.tb, 0, sizeof(uint32_t) * (2 * (size_t)p.max_nq + 1)) != hipSuccess ||   // arrival counter starts at zero
        hipMemcpy(ix->centroids, cent_host, ncent * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(ix->pq, pq_host, npq * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) {
        set_error("upload of trained parameters failed");
        return fail(PIPERAG_ERR_HIP);
    }
    if (p.nlist >= 128 && p.d >= 64) {
        const size_t nsplit = split_f16_elems(p.nlist, p.d);
        if ((rc = dev_alloc(&ix->cent_hi, nsplit)) || (rc = dev_alloc(&ix->cent_lo, nsplit)) || (rc = dev_alloc(&ix->cent_amax, 64))) return fail(rc);
        split_f16(ix->centroids, p.nlist, p.d, ix->cent_amax, ix->cent_hi, ix->cent_lo, nullptr);
    }
    rownorm(ix->centroids, p.nlist, p.d, p.d, ix->cnorm, nullptr);
    if (hipStreamSynchronize(nullptr) != hipSuccess) { set_error("centre norms failed"); return fail(PIPERAG_ERR_HIP); }
    {   // centre-major copy of the codebook
        std::vector<float> t(npq);
        for (int m = 0; m < p.M; ++m)
            for (int j = 0; j < kKsub; ++j)
                memcpy(&t[((size_t)j * p.M + m) * ix->dsub], &pq_host[((size_t)m * kKsub + j) * ix->dsub], sizeof(float) * ix->dsub);
        if (hipMemcpy(ix->pqT, t.data(), npq * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) {
            set_error("upload of trained parameters failed");
            return fail(PIPERAG_ERR_HIP);
        }
    }
    {   // the encoder's copy of the codebook: depth-major, with the centres' squared norms as one more depth row
        const int T = pqe_rows(ix->dsub);
        std::vector<float> t((size_t)p.M * T * kKsub, 0.f);
        for (int m = 0; m < p.M; ++m)
            for (int j = 0; j < kKsub; ++j) {
                const float *c = &pq_host[((size_t)m * kKsub + j) * ix->dsub];
                float nn = 0.f;
                for (int u = 0; u < ix->dsub; ++u) {
                    t[((size_t)m * T + u) * kKsub + j] = c[u];
                    nn += c[u] * c[u];
                }
                t[((size_t)m * T + ix->dsub) * kKsub + j] = nn;
            }
        if (hipMemcpy(ix->pqE, t.data(), t.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) {
            set_error("upload of trained parameters failed");
            return fail(PIPERAG_ERR_HIP);
        }
    }
    for (int e = 0; e <= PIPERAG_NSTAGES; ++e)
        if (hipEventCreate(&ix->ev[e]) != hipSuccess) { set_error("hipEventCreate failed"); return fail(PIPERAG_ERR_HIP); }
    if (hipStreamCreateWithFlags(&ix->cap_stream, hipStreamNonBlocking) != hipSuccess) {
        set_error("creating the capture stream failed");
        return fail(PIPERAG_ERR_HIP);
    }
    *out = ix;
    return PIPERAG_OK;
}

int append_common(piperag_index *ix, int64_t n, const int64_t *ids_dev, hipStream_t st) {
    // ids of the n entries being appended at position ix->nadded
    if (ids_dev) {
        PR_CHECK_HIP(hipMemcpyAsync(ix->st_ids + ix->nadded, ids_dev, sizeof(int64_t) * n, hipMemcpyDeviceToDevice, st));
    } else {
        hipLaunchKernelGGL(iota_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ix->st_ids + ix->nadded, n,
                           ix->nadded);
    }
    return PIPERAG_OK;
}

}  // namespace

namespace piperag {
int begin_build(piperag_index *ix, int mode) {
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(!ix->finalized, PIPERAG_ERR_ARG, "index is finalized; no more vectors can be added");
    if (ix->build_mode == mode) return PIPERAG_OK;
    PR_REQUIRE(ix->build_mode == 0, PIPERAG_ERR_ARG, "one-pass (add) and two-pass (count / place) builds cannot be mixed");
    PR_CHECK_HIP(hipSetDevice(ix->device));
    int rc = dev_alloc(&ix->st_list, (size_t)ix->cap);
    if (rc == PIPERAG_OK && mode == 1) rc = dev_alloc(&ix->st_codes, (size_t)ix->cap * ix->p.M);
    if (rc == PIPERAG_OK && mode == 1) rc = dev_alloc(&ix->st_ids, (size_t)ix->cap);
    if (rc == PIPERAG_OK && mode == 2) rc = dev_alloc(&ix->bd_counts, (size_t)ix->p.nlist);
    if (rc == PIPERAG_OK && mode == 2) rc = dev_alloc(&ix->bd_cursor, (size_t)ix->p.nlist);
    if (rc == PIPERAG_OK && mode == 2 &&
        (hipMemset(ix->bd_counts, 0, sizeof(uint32_t) * ix->p.nlist) != hipSuccess ||
         hipMemset(ix->bd_cursor, 0, sizeof(uint32_t) * ix->p.nlist) != hipSuccess)) {
        set_error("clearing the list counters failed");
        rc = PIPERAG_ERR_HIP;
    }
    if (rc != PIPERAG_OK) { free_staging(ix); return rc; }
    ix->build_mode = mode;
    return PIPERAG_OK;
}

// used by encode.hip
int check_can_add(piperag_index *ix, int64_t n) {
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(!ix->finalized, PIPERAG_ERR_ARG, "index is finalized; no more vectors can be added");
    PR_REQUIRE(n >= 0, PIPERAG_ERR_ARG, "n = %lld is negative", (long long)n);
    PR_REQUIRE(ix->nadded + n <= ix->cap, PIPERAG_ERR_LIMIT, "adding %lld vectors to %lld exceeds the capacity %lld",
               (long long)n, (long long)ix->nadded, (long long)ix->cap);
    return n > 0 ? begin_build(ix, 1) : PIPERAG_OK;
}

// Places one tile of encoded vectors (two-pass build): lists_dev[i], codes_dev[i*M..], ids_dev[i] for i < n go to
// the next free slots of their lists, in order (a stable counting sort of the tile on top of the per-list
// cursors).  Scratch is taken and returned in stream order.
int place_tile(piperag_index *ix, const int32_t *lists_dev, const uint8_t *codes_dev, const int64_t *ids_dev, int64_t n,
               hipStream_t st) {
    const int nlist = ix->p.nlist;
    const int64_t chunk = round_up64(std::max<int64_t>((n + 1023) / 1024, 4096), kPlaceTile);
    const int G = (int)std::max<int64_t>(1, (n + chunk - 1) / chunk);
    uint32_t *H = nullptr;
    PR_CHECK_HIP(hipMallocAsync(reinterpret_cast<void **>(&H), sizeof(uint32_t) * (size_t)G * nlist, st));
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)(((size_t)G * nlist + 255) / 256)), dim3(256), 0, st, H, (size_t)G * nlist, 0u);
    hipLaunchKernelGGL(hist_kernel, dim3(G), dim3(256), 0, st, lists_dev, n, chunk, nlist, H);
    hipLaunchKernelGGL(colscan_kernel, dim3((nlist + 255) / 256), dim3(256), 0, st, H, G, nlist, (int32_t *)nullptr, ix->bd_cursor);
    hipLaunchKernelGGL(place_kernel, dim3(G), dim3(kPlaceTile), 0, st, lists_dev, codes_dev, ids_dev, n, chunk, nlist, ix->p.M,
                       ix->Mp, H, ix->list_blk, ix->codes, ix->ids);
    PR_CHECK_HIP(hipFreeAsync(H, st));
    return PIPERAG_OK;
}
void fill_iota(int64_t *dst, int64_t n, int64_t first, hipStream_t st) {
    hipLaunchKernelGGL(iota_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dst, n, first);
}
void count_lists(const int32_t *lists, int64_t n, uint32_t *counts, hipStream_t st) {
    hipLaunchKernelGGL(count_lists_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, lists, n, counts);
}
int append_ids(piperag_index *ix, int64_t n, const int64_t *ids_dev, hipStream_t st) { return append_common(ix, n, ids_dev, st); }
}  // namespace piperag

extern "C" {

const char *piperag_last_error(void) { return piperag::g_err; }

int piperag_ivf_create(const piperag_params *params, const float *centroids_host, const float *pq_codebook_host,
                       piperag_index **out) {
    return create_impl(params, centroids_host, pq_codebook_host, out);
}

void piperag_ivf_free(piperag_index *ix) {
    if (!ix) return;
    free_staging(ix);
    void *ptrs[] = {ix->centroids, ix->cnorm, ix->cent_hi, ix->cent_lo, ix->cent_amax, ix->rb_codes, ix->rb_ids, ix->pq, ix->pqT, ix->pqE, ix->codes, ix->ids, ix->list_blk, ix->list_len, ix->tx, ix->ws_mem, ix->ws_out_d, ix->ws_out_i, ix->flag};
    for (void *p : ptrs) (void)hipFree(p);
    for (int e = 0; e <= PIPERAG_NSTAGES; ++e)
        if (ix->ev[e]) (void)hipEventDestroy(ix->ev[e]);
    if (ix->cap_stream) (void)hipStreamDestroy(ix->cap_stream);
    for (SearchGraph &g : ix->graphs)
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
    delete ix;
}

int64_t piperag_ivf_ntotal(const piperag_index *ix) { return ix ? (ix->finalized ? ix->ntotal : ix->nadded) : -1; }

int piperag_ivf_add_encoded(piperag_index *ix, const int32_t *lists_dev, const uint8_t *codes_dev, const int64_t *ids_dev,
                            int64_t n, void *stream) {
    PR_TRY(check_can_add(ix, n));
    if (n == 0) return PIPERAG_OK;
    PR_REQUIRE(lists_dev && codes_dev, PIPERAG_ERR_ARG, "lists / codes pointer is NULL");
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(ix->device));
    // list numbers are used as array indices later: validate them now
    int *bad = ix->flag;
    PR_CHECK_HIP(hipMemsetAsync(bad, 0, sizeof(int), st));
    hipLaunchKernelGGL(check_lists_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, lists_dev, n, ix->p.nlist, bad);
    int h_bad = 0;
    PR_CHECK_HIP(hipMemcpyAsync(&h_bad, bad, sizeof(int), hipMemcpyDeviceToHost, st));
    PR_CHECK_HIP(hipStreamSynchronize(st));
    PR_REQUIRE(h_bad == 0, PIPERAG_ERR_ARG, "a list number is outside 0..nlist-1");
    PR_CHECK_HIP(hipMemcpyAsync(ix->st_list + ix->nadded, lists_dev, sizeof(int32_t) * n, hipMemcpyDeviceToDevice, st));
    PR_CHECK_HIP(hipMemcpyAsync(ix->st_codes + (size_t)ix->nadded * ix->p.M, codes_dev, (size_t)n * ix->p.M,
                                hipMemcpyDeviceToDevice, st));
    PR_TRY(append_common(ix, n, ids_dev, st));
    ix->nadded += n;
    PR_CHECK_HIP(hipGetLastError());
    return PIPERAG_OK;
}

// Sizes the lists (list_len is set), lays out the blocks and allocates the scan layout, cleared to "no vector".
static int allocate_lists(piperag_index *ix, hipStream_t st) {
    const int nlist = ix->p.nlist;
    hipLaunchKernelGGL(blockscan_kernel, dim3(1), dim3(1024), 0, st, ix->list_len, nlist, ix->list_blk);
    int32_t nblocks = 0;
    hipError_t e = hipMemcpyAsync(&nblocks, ix->list_blk + nlist, sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { set_error("sizing the lists failed: %s", hipGetErrorString(e)); return PIPERAG_ERR_HIP; }
    ix->nblocks = nblocks;
    PR_REQUIRE((int64_t)nblocks * kBlockVecs < 0xFFFFFFFFll, PIPERAG_ERR_LIMIT, "too many slots for 32-bit positions");
    const size_t code_bytes = (size_t)std::max<int64_t>(nblocks, 1) * kBlockVecs * ix->Mp;
    const size_t nslots = (size_t)std::max<int64_t>(nblocks, 1) * kBlockVecs;
    if (hipMalloc(reinterpret_cast<void **>(&ix->codes), code_bytes) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&ix->ids), nslots * sizeof(int64_t)) != hipSuccess) {
        set_error("out of device memory for %zu bytes of codes", code_bytes);
        return PIPERAG_ERR_OOM;
    }
    e = hipMemsetAsync(ix->codes, 0, code_bytes, st);
    if (e == hipSuccess) e = hipMemsetAsync(ix->ids, 0xFF, nslots * sizeof(int64_t), st);
    if (e != hipSuccess) { set_error("hipMemsetAsync failed: %s", hipGetErrorString(e)); return PIPERAG_ERR_HIP; }
    return PIPERAG_OK;
}

static int finish_build(piperag_index *ix, int64_t n) {
    if (ix->p.residual) {
        const size_t nslots = (size_t)std::max<int64_t>(ix->nblocks, 1) * kBlockVecs;
        PR_TRY(dev_alloc(&ix->tx, nslots));
        if (ix->nblocks > 0)
            hipLaunchKernelGGL(residual_term_kernel, dim3((unsigned)ix->nblocks), dim3(64), 0, nullptr, ix->codes, ix->list_blk,
                               ix->list_len, ix->p.nlist, ix->centroids, ix->pq, ix->p.d, ix->p.M, ix->Mp, ix->dsub, ix->tx);
        else
            PR_CHECK_HIP(hipMemset(ix->tx, 0, nslots * sizeof(float)));
        PR_CHECK_HIP(hipStreamSynchronize(nullptr));
    }
    std::vector<int32_t> hl(ix->p.nlist);
    if (hipMemcpy(hl.data(), ix->list_len, sizeof(int32_t) * ix->p.nlist, hipMemcpyDeviceToHost) != hipSuccess) {
        set_error("finalize (list lengths) failed");
        return PIPERAG_ERR_HIP;
    }
    ix->max_list_len = 0;
    for (int32_t v : hl) ix->max_list_len = std::max<int64_t>(ix->max_list_len, v);
    free_staging(ix);
    ix->ntotal = n;
    ix->finalized = true;
    return PIPERAG_OK;
}

int piperag_ivf_reserve(piperag_index *ix, void *stream) {
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(!ix->finalized && ix->build_mode == 2 && !ix->reserved, PIPERAG_ERR_ARG,
               "reserve follows the count calls of a two-pass build, once");
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(ix->device));
    hipLaunchKernelGGL(counts_to_len_kernel, dim3((ix->p.nlist + 255) / 256), dim3(256), 0, st, ix->bd_counts, ix->p.nlist,
                       ix->list_len);
    PR_TRY(allocate_lists(ix, st));
    PR_CHECK_HIP(hipStreamSynchronize(st));
    ix->reserved = true;
    return PIPERAG_OK;
}

int piperag_ivf_finalize(piperag_index *ix, void *stream) {
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(!ix->finalized, PIPERAG_ERR_ARG, "index is already finalized");
    hipStream_t st = (hipStream_t)stream;
    PR_CHECK_HIP(hipSetDevice(ix->device));
    if (ix->build_mode == 2) {
        PR_REQUIRE(ix->reserved && ix->nplaced == ix->nadded, PIPERAG_ERR_ARG,
                   "two-pass build incomplete: %lld vectors counted, %lld placed", (long long)ix->nadded, (long long)ix->nplaced);
        hipError_t e2 = hipStreamSynchronize(st);
        if (e2 == hipSuccess) e2 = hipGetLastError();
        if (e2 != hipSuccess) { set_error("finalize (placement) failed: %s", hipGetErrorString(e2)); return PIPERAG_ERR_HIP; }
        return finish_build(ix, ix->nadded);
    }
    const int64_t n = ix->nadded;
    const int nlist = ix->p.nlist, M = ix->p.M, Mp = ix->Mp;
    // chunks of the staging area, one placement workgroup each
    int64_t chunk = round_up64(std::max<int64_t>((n + 1023) / 1024, 4096), kPlaceTile);
    const int G = (int)std::max<int64_t>(1, (n + chunk - 1) / chunk);
    uint32_t *H = nullptr;
    PR_CHECK_HIP(hipMalloc(reinterpret_cast<void **>(&H), sizeof(uint32_t) * (size_t)G * nlist));
    auto cleanup = [&](int code) { (void)hipFree(H); return code; };
    hipError_t e = hipMemsetAsync(H, 0, sizeof(uint32_t) * (size_t)G * nlist, st);
    if (e != hipSuccess) { set_error("hipMemsetAsync failed: %s", hipGetErrorString(e)); return cleanup(PIPERAG_ERR_HIP); }
    if (n > 0) hipLaunchKernelGGL(hist_kernel, dim3(G), dim3(256), 0, st, ix->st_list, n, chunk, nlist, H);
    hipLaunchKernelGGL(colscan_kernel, dim3((nlist + 255) / 256), dim3(256), 0, st, H, G, nlist, ix->list_len, (uint32_t *)nullptr);
    {
        const int rca = allocate_lists(ix, st);
        if (rca != PIPERAG_OK) return cleanup(rca);
    }
    if (n > 0)
        hipLaunchKernelGGL(place_kernel, dim3(G), dim3(kPlaceTile), 0, st, ix->st_list, ix->st_codes, ix->st_ids, n, chunk,
                           nlist, M, Mp, H, ix->list_blk, ix->codes, ix->ids);
    e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { set_error("finalize (placement) failed: %s", hipGetErrorString(e)); return cleanup(PIPERAG_ERR_HIP); }
    return cleanup(finish_build(ix, n));
}

int piperag_ivf_list_lengths(const piperag_index *ix, int64_t *out_host) {
    PR_REQUIRE(ix && out_host, PIPERAG_ERR_ARG, "NULL argument");
    PR_REQUIRE(ix->finalized, PIPERAG_ERR_ARG, "index is not finalized");
    std::vector<int32_t> h(ix->p.nlist);
    PR_CHECK_HIP(hipMemcpy(h.data(), ix->list_len, sizeof(int32_t) * h.size(), hipMemcpyDeviceToHost));
    for (size_t l = 0; l < h.size(); ++l) out_host[l] = h[l];
    return PIPERAG_OK;
}

int piperag_ivf_get_list(const piperag_index *ix, int32_t list, int64_t *len_out, uint8_t *codes_host, int64_t *ids_host) {
    PR_REQUIRE(ix != nullptr, PIPERAG_ERR_ARG, "index is NULL");
    PR_REQUIRE(ix->finalized, PIPERAG_ERR_ARG, "index is not finalized");
    PR_REQUIRE(list >= 0 && list < ix->p.nlist, PIPERAG_ERR_ARG, "list = %d out of range", list);
    PR_CHECK_HIP(hipSetDevice(ix->device));
    int32_t len = 0, blk = 0;
    PR_CHECK_HIP(hipMemcpy(&len, ix->list_len + list, sizeof(int32_t), hipMemcpyDeviceToHost));
    PR_CHECK_HIP(hipMemcpy(&blk, ix->list_blk + list, sizeof(int32_t), hipMemcpyDeviceToHost));
    if (len_out) *len_out = len;
    if (len == 0 || (!codes_host && !ids_host)) return PIPERAG_OK;
    // read-back scratch sized for the longest list, allocated on first use and kept with the index
    const piperag_index *mix = ix;           // the read-back buffers are mutable members
    if (!mix->rb_codes) {
        const size_t cap = (size_t)std::max<int64_t>(ix->max_list_len, 1);
        if (hipMalloc(reinterpret_cast<void **>(&mix->rb_codes), cap * ix->p.M) != hipSuccess ||
            hipMalloc(reinterpret_cast<void **>(&mix->rb_ids), cap * sizeof(int64_t)) != hipSuccess) {
            (void)hipFree(mix->rb_codes); mix->rb_codes = nullptr;
            set_error("out of device memory for the list read-back buffer");
            return PIPERAG_ERR_OOM;
        }
    }
    PR_REQUIRE(len <= ix->max_list_len, PIPERAG_ERR_HIP, "list length %d exceeds the recorded maximum", len);
    hipLaunchKernelGGL(gather_list_kernel, dim3((len + 255) / 256), dim3(256), 0, 0, ix->codes, ix->ids,
                       (uint32_t)blk * kBlockVecs, (int64_t)0, (int64_t)len, ix->p.M, ix->Mp, codes_host ? mix->rb_codes : nullptr,
                       ids_host ? mix->rb_ids : nullptr);
    if (codes_host) PR_CHECK_HIP(hipMemcpy(codes_host, mix->rb_codes, (size_t)len * ix->p.M, hipMemcpyDeviceToHost));
    if (ids_host) PR_CHECK_HIP(hipMemcpy(ids_host, mix->rb_ids, (size_t)len * sizeof(int64_t), hipMemcpyDeviceToHost));
    return PIPERAG_OK;
}

// ---- file I/O ---------------------------------------------------------------------------------
namespace {
struct FileHeader {
    char magic[8];
    uint32_t version, d, nlist, M, nbits, zero;      // zero: flags (bit 0: residual codes)
    uint64_t ntotal;
    char pad[64 - 8 - 24 - 8];
};
static_assert(sizeof(FileHeader) == 64, "header is 64 bytes");
constexpr int64_t kIoVecs = 1 << 20;   // vectors per transfer
}  // namespace

int piperag_ivf_save(const piperag_index *ix, const char *path) {
    PR_REQUIRE(ix && path, PIPERAG_ERR_ARG, "NULL argument");
    PR_REQUIRE(ix->finalized, PIPERAG_ERR_ARG, "index is not finalized");
    PR_CHECK_HIP(hipSetDevice(ix->device));
    const piperag_params &p = ix->p;
    FILE *f = fopen(path, "wb");
    PR_REQUIRE(f != nullptr, PIPERAG_ERR_FILE, "cannot open %s for writing", path);
    FileHeader h;
    memset(&h, 0, sizeof(h));
    memcpy(h.magic, "PRAGIVF1", 8);
    h.version = 1; h.d = p.d; h.nlist = p.nlist; h.M = p.M; h.nbits = 8; h.zero = p.residual ? 1u : 0u; h.ntotal = (uint64_t)ix->ntotal;
    int rc = PIPERAG_OK;
    uint8_t *dc = nullptr;
    int64_t *di = nullptr;
    auto done = [&](int code) { fclose(f); (void)hipFree(dc); (void)hipFree(di); return code; };
    auto put = [&](const void *src, size_t bytes) { return fwrite(src, 1, bytes, f) == bytes; };
    std::vector<float> buf((size_t)p.nlist * p.d);
    std::vector<float> pqb((size_t)p.M * kKsub * ix->dsub);
    std::vector<int32_t> len(p.nlist), blk(p.nlist + 1);
    if (hipMemcpy(buf.data(), ix->centroids, buf.size() * 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(pqb.data(), ix->pq, pqb.size() * 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(len.data(), ix->list_len, len.size() * 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(blk.data(), ix->list_blk, blk.size() * 4, hipMemcpyDeviceToHost) != hipSuccess) {
        set_error("device read failed in save");
        return done(PIPERAG_ERR_HIP);
    }
    std::vector<int64_t> len64(len.begin(), len.end());
    if (!put(&h, sizeof(h)) || !put(buf.data(), buf.size() * 4) || !put(pqb.data(), pqb.size() * 4) ||
        !put(len64.data(), len64.size() * 8)) {
        set_error("write to %s failed", path);
        return done(PIPERAG_ERR_FILE);
    }
    if (hipMalloc(reinterpret_cast<void **>(&dc), (size_t)kIoVecs * p.M) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&di), (size_t)kIoVecs * 8) != hipSuccess) {
        set_error("out of device memory in save");
        return done(PIPERAG_ERR_OOM);
    }
    std::vector<uint8_t> hc((size_t)kIoVecs * p.M);
    std::vector<int64_t> hi((size_t)kIoVecs);
    for (int pass = 0; pass < 2 && rc == PIPERAG_OK; ++pass) {      // pass 0: all codes, pass 1: all ids
        for (int l = 0; l < p.nlist && rc == PIPERAG_OK; ++l) {
            for (int64_t i0 = 0; i0 < len[l]; i0 += kIoVecs) {
                const int64_t cnt = std::min<int64_t>(kIoVecs, len[l] - i0);
                hipLaunchKernelGGL(gather_list_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, 0, ix->codes, ix->ids,
                                   (uint32_t)blk[l] * kBlockVecs, i0, cnt, p.M, ix->Mp, pass == 0 ? dc : nullptr,
                                   pass == 1 ? di : nullptr);
                hipError_t e = pass == 0 ? hipMemcpy(hc.data(), dc, (size_t)cnt * p.M, hipMemcpyDeviceToHost)
                                         : hipMemcpy(hi.data(), di, (size_t)cnt * 8, hipMemcpyDeviceToHost);
                if (e != hipSuccess) { set_error("device read failed in save"); rc = PIPERAG_ERR_HIP; break; }
                if (!(pass == 0 ? put(hc.data(), (size_t)cnt * p.M) : put(hi.data(), (size_t)cnt * 8))) {
                    set_error("write to %s failed", path);
                    rc = PIPERAG_ERR_FILE;
                    break;
                }
            }
        }
    }
    return done(rc);
}

int piperag_ivf_load(const char *path, const piperag_params *limits, piperag_index **out) {
    PR_REQUIRE(path && limits && out, PIPERAG_ERR_ARG, "NULL argument");
    *out = nullptr;
    FILE *f = fopen(path, "rb");
    PR_REQUIRE(f != nullptr, PIPERAG_ERR_FILE, "cannot open %s", path);
    piperag_index *ix = nullptr;
    int32_t *dl = nullptr;
    uint8_t *dc = nullptr;
    int64_t *di = nullptr;
    auto done = [&](int code) {
        fclose(f);
        (void)hipFree(dl); (void)hipFree(dc); (void)hipFree(di);
        if (code != PIPERAG_OK && ix) piperag_ivf_free(ix);
        return code;
    };
    auto get = [&](void *dst, size_t bytes) { return fread(dst, 1, bytes, f) == bytes; };
    FileHeader h;
    if (!get(&h, sizeof(h)) || memcmp(h.magic, "PRAGIVF1", 8) != 0 || h.version != 1) {
        set_error("%s is not a version-1 index file", path);
        return done(PIPERAG_ERR_FILE);
    }
    piperag_params p = *limits;
    p.d = (int32_t)h.d; p.nlist = (int32_t)h.nlist; p.M = (int32_t)h.M; p.nbits = (int32_t)h.nbits;
    p.ntotal = (int64_t)h.ntotal;
    p.residual = (int32_t)(h.zero & 1u);
    if (h.zero > 1u || h.d > 8192 || h.nlist > (1u << 20) || h.M > 128 || h.M == 0 || h.d % h.M != 0 || h.ntotal > 0xFFF00000ull) {
        set_error("%s: header fields out of range", path);
        return done(PIPERAG_ERR_FILE);
    }
    std::vector<float> cent((size_t)p.nlist * p.d), pqb((size_t)p.M * kKsub * (p.d / p.M));
    std::vector<int64_t> len((size_t)p.nlist);
    if (!get(cent.data(), cent.size() * 4) || !get(pqb.data(), pqb.size() * 4) || !get(len.data(), len.size() * 8)) {
        set_error("%s is truncated (parameters)", path);
        return done(PIPERAG_ERR_FILE);
    }
    int64_t sum = 0;
    for (int64_t v : len) {
        if (v < 0 || v > p.ntotal) { set_error("%s: negative or oversized list length", path); return done(PIPERAG_ERR_FILE); }
        sum += v;
    }
    if (sum != p.ntotal) { set_error("%s: list lengths sum to %lld, header says %lld", path, (long long)sum, (long long)p.ntotal); return done(PIPERAG_ERR_FILE); }
    int rc = create_impl(&p, cent.data(), pqb.data(), &ix);
    if (rc != PIPERAG_OK) return done(rc);
    const int64_t n = p.ntotal;
    const long codes_pos = ftell(f);
    if (hipMalloc(reinterpret_cast<void **>(&dl), (size_t)kIoVecs * 4) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&dc), (size_t)kIoVecs * p.M) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&di), (size_t)kIoVecs * 8) != hipSuccess) {
        set_error("out of device memory in load");
        return done(PIPERAG_ERR_OOM);
    }
    std::vector<int32_t> hl((size_t)kIoVecs);
    std::vector<uint8_t> hc((size_t)kIoVecs * p.M);
    std::vector<int64_t> hi((size_t)kIoVecs);
    int list = 0;
    int64_t left_in_list = p.nlist > 0 ? len[0] : 0;
    for (int64_t i0 = 0; i0 < n; i0 += kIoVecs) {
        const int64_t cnt = std::min<int64_t>(kIoVecs, n - i0);
        for (int64_t i = 0; i < cnt; ++i) {
            while (left_in_list == 0) left_in_list = len[++list];
            hl[i] = list;
            --left_in_list;
        }
        if (fseek(f, codes_pos + i0 * p.M, SEEK_SET) != 0 || !get(hc.data(), (size_t)cnt * p.M) ||
            fseek(f, codes_pos + n * p.M + i0 * 8, SEEK_SET) != 0 || !get(hi.data(), (size_t)cnt * 8)) {
            set_error("%s is truncated (codes / ids)", path);
            return done(PIPERAG_ERR_FILE);
        }
        if (hipMemcpy(dl, hl.data(), (size_t)cnt * 4, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(dc, hc.data(), (size_t)cnt * p.M, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(di, hi.data(), (size_t)cnt * 8, hipMemcpyHostToDevice) != hipSuccess) {
            set_error("upload failed in load");
            return done(PIPERAG_ERR_HIP);
        }
        rc = piperag_ivf_add_encoded(ix, dl, dc, di, cnt, nullptr);
        if (rc == PIPERAG_OK && hipStreamSynchronize(nullptr) != hipSuccess) { set_error("sync failed in load"); rc = PIPERAG_ERR_HIP; }
        if (rc != PIPERAG_OK) return done(rc);
    }
    rc = piperag_ivf_finalize(ix, nullptr);
    if (rc != PIPERAG_OK) return done(rc);
    *out = ix;
    return done(PIPERAG_OK);
}

}  // extern "C"
