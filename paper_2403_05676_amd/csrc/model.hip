// Host-side arithmetic of the paper's performance models: the choice of the search space under a latency
// budget (Section 3.2, S3) and the projection of end-to-end latency onto faster hardware (Appendix "Performance
// Modeling for Future Hardware").  No GPU work - except the two calls at the end, which create and destroy a
// stream that owns a slice of the compute units, so that a search can run beside a generation step on one GPU
// the way the paper runs it on a server of its own (Section 3.2, S1).
#include "common.h"

#include <cmath>

using namespace piperag;

extern "C" {

int piperag_max_nprobe(const float *fit_host, float overhead_ms, float budget_ms, int32_t nprobe_cap, int32_t *out_nprobe,
                       int32_t *out_fits, float *out_predicted_ms) {
    PR_REQUIRE(fit_host && out_nprobe && out_fits, PIPERAG_ERR_ARG, "NULL argument");
    PR_REQUIRE(nprobe_cap >= 1, PIPERAG_ERR_ARG, "nprobe_cap = %d must be >= 1", nprobe_cap);
    const double a = fit_host[0], b = fit_host[1], o = overhead_ms, T = budget_ms;
    PR_REQUIRE(std::isfinite(a) && std::isfinite(b) && std::isfinite(o) && std::isfinite(T) && o >= 0.0, PIPERAG_ERR_ARG,
               "fit, overhead and budget must be finite, overhead >= 0");
    auto predicted = [&](int64_t p) { return o + a + b * (double)p; };
    int64_t best = 1;
    int fits = predicted(1) <= T;
    if (fits) {
        if (b <= 0.0) {
            best = nprobe_cap;
        } else {
            // largest p with o + a + b p <= T, then corrected by one step either way for the rounding of the division
            best = (int64_t)std::floor((T - o - a) / b);
            best = std::max<int64_t>(1, std::min<int64_t>(best, nprobe_cap));
            while (best < nprobe_cap && predicted(best + 1) <= T) ++best;
            while (best > 1 && predicted(best) > T) --best;
        }
    }
    *out_nprobe = (int32_t)best;
    *out_fits = fits;
    if (out_predicted_ms) *out_predicted_ms = (float)predicted(best);
    return PIPERAG_OK;
}

int piperag_project_latency(const float *inference_ms_host, const float *retrieval_ms_host, int32_t nchunks,
                            float inference_speedup, float retrieval_speedup, double *out_sequential_ms,
                            double *out_pipelined_ms) {
    PR_REQUIRE(inference_ms_host && retrieval_ms_host && out_sequential_ms && out_pipelined_ms, PIPERAG_ERR_ARG, "NULL argument");
    PR_REQUIRE(nchunks >= 1, PIPERAG_ERR_ARG, "nchunks = %d must be >= 1", nchunks);
    PR_REQUIRE(inference_speedup > 0.f && retrieval_speedup > 0.f && std::isfinite(inference_speedup) &&
                   std::isfinite(retrieval_speedup),
               PIPERAG_ERR_ARG, "speed-up factors must be positive and finite");
    double seq = 0.0, pipe = 0.0;
    for (int32_t c = 0; c < nchunks; ++c) {
        const double ti = (double)inference_ms_host[c] / (double)inference_speedup;
        const double tr = (double)retrieval_ms_host[c] / (double)retrieval_speedup;
        seq += ti + tr;
        pipe += c == 0 ? ti + tr : std::max(ti, tr);
    }
    *out_sequential_ms = seq;
    *out_pipelined_ms = pipe;
    return PIPERAG_OK;
}

int piperag_stream_create_cu_slice(int32_t first_cu, int32_t ncu, void **out_stream) {
    PR_REQUIRE(out_stream != nullptr, PIPERAG_ERR_ARG, "out_stream is NULL");
    *out_stream = nullptr;
    int device = 0, total = 0;
    PR_CHECK_HIP(hipGetDevice(&device));
    PR_CHECK_HIP(hipDeviceGetAttribute(&total, hipDeviceAttributeMultiprocessorCount, device));
    PR_REQUIRE(first_cu >= 0 && ncu >= 1 && first_cu + ncu <= total, PIPERAG_ERR_ARG,
               "compute units %d..%d are not within the device's %d", first_cu, first_cu + ncu - 1, total);
    uint32_t mask[32] = {0};
    PR_REQUIRE(total <= 32 * 32, PIPERAG_ERR_LIMIT, "more compute units than the mask holds");
    for (int cu = first_cu; cu < first_cu + ncu; ++cu) mask[cu >> 5] |= 1u << (cu & 31);
    hipStream_t st = nullptr;
    PR_CHECK_HIP(hipExtStreamCreateWithCUMask(&st, (uint32_t)((total + 31) / 32), mask));
    *out_stream = st;
    return PIPERAG_OK;
}

int piperag_stream_destroy(void *stream) {
    PR_REQUIRE(stream != nullptr, PIPERAG_ERR_ARG, "stream is NULL");
    PR_CHECK_HIP(hipStreamDestroy((hipStream_t)stream));
    return PIPERAG_OK;
}

}  // extern "C"
