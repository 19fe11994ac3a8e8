// Internal definitions shared by the translation units of libpiperag (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#pragma GCC visibility push(default)
#include "../../include/piperag.h"
#pragma GCC visibility pop

namespace piperag {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kBlockVecs = 64;     // vectors per code block (one per lane)
constexpr int kKsub = 256;         // centres per sub-quantiser (8-bit codes)
constexpr int kMaxK = 1024;
constexpr int kMaxNprobe = 1024;
constexpr int kScanThreads = 256;  // 4 waves per scan workgroup
constexpr int kScanWaves = kScanThreads / kWave;
constexpr int kTargetScanWGs = 512;    // scan workgroups per search call: two per compute unit, all resident at once ...
constexpr int kMaxScanWGs = 2048;      // ... or, for large batches, about 8 per query up to this many: a query then has enough
                                       // workgroups to share its blocks evenly, and late workgroups fill in behind early finishers
constexpr int kMaxSegments = 1024;
constexpr int kCoarseMaxParts = 4;     // parts the coarse quantiser's depth may be split into
constexpr int kCoarseSplitMaxLists = 8192;   // ... for indexes of up to this many lists (the workspace holds that many partial rows)
constexpr int kCtrStride = 32;         // chunk counters sit 128 bytes apart
constexpr int kCtrPerQuery = 16;       // at most this many chunk counters share out one query's blocks
constexpr int kMinBlocksPerWG = 16;    // one round of the scan loop: 4 waves x 4 blocks
constexpr size_t kStreamingCodeBytes = (size_t)4 << 30;   // indexes with at least this many code bytes are scanned with non-temporal loads ...
constexpr size_t kStreamingListBytes = (size_t)4 << 20;   // ... unless their lists average this many code bytes or more
constexpr uint64_t kSentinel = 0xFFFFFFFFFFFFFFFFull;

void set_error(const char *fmt, ...);
void rownorm(const float *a, int64_t n, int d, int64_t lda, float *out, hipStream_t st);   // squared row norms
// scaled fp16 hi / lo parts of n rows of d values in the encoder's chunk-major layout; each part holds
// split_f16_elems(n, d) elements; *amax (device) receives the bits of the largest magnitude, which fixes the scale
void split_f16(const float *src, int64_t n, int d, uint32_t *amax, uint16_t *hi, uint16_t *lo, hipStream_t st);
size_t split_f16_elems(int64_t n, int d);

#define PR_CHECK_HIP(expr)                                                                     \
    do {                                                                                       \
        hipError_t e__ = (expr);                                                               \
        if (e__ != hipSuccess) {                                                               \
            piperag::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
            return e__ == hipErrorOutOfMemory ? PIPERAG_ERR_OOM : PIPERAG_ERR_HIP;             \
        }                                                                                      \
    } while (0)

#define PR_REQUIRE(cond, code, ...)          \
    do {                                     \
        if (!(cond)) {                       \
            piperag::set_error(__VA_ARGS__); \
            return (code);                   \
        }                                    \
    } while (0)

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline int64_t round_up64(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline int next_pow2(int v) { int p = 1; while (p < v) p <<= 1; return p; }

}  // namespace piperag

// The index object.  Code storage ("scan layout"): vectors are grouped list after list into blocks of 64
// slots (a list starts on a block boundary; unused slots of its last block have id -1 and zero codes).
// With Mp = M rounded up to a multiple of 16, block b occupies bytes [b*64*Mp, (b+1)*64*Mp) laid out as
// [chunk c < Mp/16][lane < 64][16 bytes]; byte t = 16*c + u of lane l is code byte (l + t) mod Mp of the
// vector in slot 64*b + l (zero when that index is >= M).  One 16-byte load per lane per chunk is thus a
// contiguous 1 KiB wavefront access, and at step t the 64 lanes look up 64 different sub-quantisers.
// A search call seen before, and its captured graph once it has been seen twice.
// depth rows of the encoder's codebook copy: the coordinates, one row of squared norms, rounded up to even
inline int pqe_rows(int dsub) { return (dsub + 2) / 2 * 2; }

// Device scratch of one search call.  Sized for (nlist, Mp, max_nq, max_nprobe, max_k) by search_ws_layout, which
// carves it out of one block of memory: the index owns one (allocated at creation), the entry point for callers
// that cannot allocate carves another out of a static device array.
struct SearchWs {
    float *D;             // [parts][max_nq*nlist] coarse distances, or partial inner products (parts = kCoarseMaxParts up to kCoarseSplitMaxLists lists, else 1)
    int32_t *probe;       // [max_nq*max_nprobe]
    float *probe_d;       // [max_nq*max_nprobe]
    int32_t *pfx;         // [max_nq*(max_nprobe+1)] block prefix sums of the probed lists
    int64_t *scanned;     // [max_nq]
    int32_t *seg0;        // [max_nq+1] first scan workgroup of each query
    int4 *desc;           // [kMaxScanWGs+max_nq] (query, number among the query's workgroups, their count, chunk counters in use) of each scan workgroup
    uint32_t *done;       // [max_nq + kMaxScanWGs + max_nq] finished scan workgroups (or groups of them) per query, then finished workgroups per group
    uint64_t *part2;      // same shape as part: the queries' lists when a query's workgroups are grouped
    uint32_t *tb;         // [2*max_nq+1] blocks of each query as published by the selection; then the count of finished selections and a ticket
                          // per query for its selection workgroups (both zero between searches)
    uint64_t *selcand;    // [max(max_nq * slices a long row needs, 512) * max_nprobe] candidate probes of the queries' selection workgroups
    uint32_t *ctr;        // [max_nq*kCtrPerQuery*kCtrStride] chunk counters of each query (one per 128 bytes)
    float *pcst;          // [max_nq*max_nprobe] residual indexes: |c_l|^2 - 2 <q, c_l> of each probed list
    int32_t *pblk;        // [max_nq*max_nprobe] first block of each probed list
    int32_t *plen;        // [max_nq*max_nprobe] length of each probed list
    uint32_t *thr;        // [max_nq] per-query bound on the k-th best distance (bits), shared by the scan workgroups
    float *lut;           // [max_nq*256*Mp], entry [q][j][m]
    uint64_t *part;       // [(kMaxScanWGs+2*max_nq)*(max_k+64)] key lists of the queries (or of their groups of workgroups): room for max_k+64 keys per scan workgroup
    int32_t max_nq, max_nprobe, max_k;   // what it is sized for; max_nprobe is the row stride of the probe tables
};

struct SearchGraph {
    const float *q;
    const int32_t *probes;
    int32_t nq, nprobe, k;
    float *out_d;
    int64_t *out_i;
    hipGraphExec_t exec;
    uint64_t stamp;
    int seen;
};

struct piperag_index {
    piperag_params p;
    int dsub, Mp, device;
    // trained parameters (device)
    float *centroids;  // [nlist*d]
    float *cnorm;      // [nlist] squared norms of the centres
    uint16_t *cent_hi, *cent_lo;   // scaled fp16 split of the centres for the encoder, chunk-major (NULL when the shape rules it out)
    uint32_t *cent_amax;           // [1] bits of the centres' largest magnitude (fixes the scale of the split)
    float *pq;         // [M*256*dsub] sub-quantiser-major (as given)
    float *pqE;        // [M][pqe_rows(dsub)][256] the encoder's copy: pqE[m][t][j] = pq[m][j][t], row dsub = squared norms, then zeros
    float *pqT;        // [256*M*dsub] centre-major copy for the table build: pqT[j][m][t] = pq[m][j][t]
    // Build state.  One-pass build (add / add_encoded, then finalize): a staging area of list number, canonical
    // code row and id per vector, allocated at the first add.  Two-pass build (count, reserve, place, finalize)
    // for databases whose staging area would not fit beside the index: pass 1 keeps only the list numbers and
    // counts the lists, reserve sizes the lists, pass 2 places every tile straight into the scan layout.
    int build_mode;     // 0 nothing added yet, 1 one-pass, 2 two-pass
    int64_t cap, nadded;
    int32_t *st_list;   // [cap] (both modes)
    uint8_t *st_codes;  // [cap*M] canonical rows (one-pass)
    int64_t *st_ids;    // [cap] (one-pass)
    uint32_t *bd_counts;   // [nlist] list sizes counted in pass 1 (two-pass)
    uint32_t *bd_cursor;   // [nlist] entries of each list placed so far (two-pass)
    int64_t nplaced;       // vectors placed in pass 2
    bool reserved;         // lists are sized, codes / ids allocated (two-pass)
    bool finalized;
    // residual indexes only: tx[slot] = 2 <c_l, decode(code)> of the vector in the slot (l its list), so that the
    // distance to it is the raw-table sum + tx[slot] + (|c_l|^2 - 2 <q, c_l>); computed at finalize
    float *tx;
    // scan layout (after finalize)
    int64_t ntotal, nblocks;
    uint8_t *codes;     // [nblocks*64*Mp]
    int64_t *ids;       // [nblocks*64]
    int32_t *list_blk;  // [nlist+1] first block of each list
    int32_t *list_len;  // [nlist]
    int64_t max_list_len;
    mutable uint8_t *rb_codes;  // read-back scratch for piperag_ivf_get_list (allocated on first use)
    mutable int64_t *rb_ids;
    // search workspace (one allocation, carved by search_ws_layout)
    SearchWs ws;
    void *ws_mem;
    float *ws_out_d;      // [max_nq*max_k] scratch outputs (latency profile)
    int64_t *ws_out_i;    // [max_nq*max_k]
    int *flag;            // [1] device flag for argument checks
    // state that searches (which take the index as const) update
    mutable int32_t last_nq;
    mutable const int64_t *last_scanned;   // the scanned-vector counts of the most recent search (in the workspace it used)
    // stage timing
    bool timing;
    hipEvent_t ev[PIPERAG_NSTAGES + 1];
    hipStream_t cap_stream;       // capture stream for the search graphs
    bool replay;                  // graph replay of repeated calls is enabled
    int streaming;                // scan loads: < 0 by index size, 0 ordinary, > 0 non-temporal
    int ncu;                      // compute units the searches may use (sizes the selection and scan launches)
    mutable SearchGraph graphs[8];
    mutable uint64_t graph_clock;
    mutable bool ev_valid;
};

namespace piperag {
// build plumbing shared by index.hip and encode.hip
// Carves a search workspace for the given shape out of `base` (256-byte aligned; NULL: only the size is wanted)
// and returns the bytes it takes.
size_t search_ws_layout(SearchWs *ws, void *base, int nlist, int Mp, int max_nq, int max_nprobe, int max_k, int max_wgs);
// Per-device set-up of the search and encode kernels (dynamic LDS limits, the static scratch array's address);
// called at index creation and by entry points that take no index.  Thread-safe.
int configure_search_kernels(int device);
int configure_encode_kernels(int device);
int begin_build(piperag_index *ix, int mode);     // allocates what the build mode needs at its first call; rejects mixing modes
int place_tile(piperag_index *ix, const int32_t *lists_dev, const uint8_t *codes_dev, const int64_t *ids_dev, int64_t n, hipStream_t st);
void fill_iota(int64_t *dst, int64_t n, int64_t first, hipStream_t st);
void count_lists(const int32_t *lists, int64_t n, uint32_t *counts, hipStream_t st);
}  // namespace piperag

