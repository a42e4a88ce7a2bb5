// Diagnostics and tuning knobs (include/longlive_diag.h): the process-wide attention-kernel variant and the probe
// that measures what the matrix pipe sustains.  Not part of the method.
#include "../../include/longlive_diag.h"

#include "api_common.h"

using namespace ll;
using namespace ll_api;

extern "C" {

ll_status ll_set_attn_variant(int variant) {
    if (variant != 0 && !attn_variant_name(variant)) return fail(LL_ERR_INVALID_ARG, "no attention variant %d", variant);
    g_variant = variant;
    return LL_OK;
}
const char* ll_attn_variant_name(int variant) { return attn_variant_name(variant); }

ll_status ll_probe_mfma_rate(void* dev_scratch, size_t scratch_bytes, int workgroups, int iters, int random_operands,
                             double* tflops, double* clock_ghz, void* stream) {
    return ll_probe_mfma_mix(dev_scratch, scratch_bytes, workgroups, iters, random_operands, 0, 1, tflops, clock_ghz, stream);
}

ll_status ll_probe_mfma_mix(void* dev_scratch, size_t scratch_bytes, int workgroups, int iters, int random_operands,
                            int companion, int per_mfma, double* tflops, double* clock_ghz, void* stream) {
    if (!dev_scratch || !tflops || !clock_ghz) return fail(LL_ERR_INVALID_ARG, "null pointer");
    if (workgroups < 1 || workgroups > 4096 || iters < 1 || iters > (1 << 22))
        return fail(LL_ERR_INVALID_ARG, "workgroups %d or iters %d out of range", workgroups, iters);
    if (companion < PROBE_NONE || companion > PROBE_FP8_LDS || per_mfma < 1 || per_mfma > 2)
        return fail(LL_ERR_INVALID_ARG, "companion %d (0..11) or per_mfma %d (1, 2) out of range", companion, per_mfma);
    const size_t sink_bytes = size_t(workgroups) * 512 * sizeof(float);
    if (scratch_bytes < sink_bytes + 16) return fail(LL_ERR_BUFFER_TOO_SMALL, "scratch has %zu bytes, %zu needed", scratch_bytes, sink_bytes + 16);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* sink = static_cast<float*>(dev_scratch);
    unsigned long long* counters = reinterpret_cast<unsigned long long*>(static_cast<char*>(dev_scratch) + sink_bytes);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) e = launch_probe_mfma(sink, counters, workgroups, iters, random_operands, companion, per_mfma, s);   // clocks settle
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = launch_probe_mfma(sink, counters, workgroups, iters, random_operands, companion, per_mfma, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    unsigned long long host[2] = {0, 0};
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipMemcpy(host, counters, sizeof host, hipMemcpyDeviceToHost);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) return hip_fail(e, "ll_probe_mfma_mix");
    // 8 waves per workgroup, 16 MFMAs of 32x32x16 (2 * 32 * 32 * 16 flops; 32x32x64 for the fp8 kinds) per iteration and wave
    *tflops = double(workgroups) * 8 * iters * 16 * (companion >= PROBE_FP8_NONE ? 131072.0 : 32768.0) / (double(ms) * 1e9);
    *clock_ghz = host[1] ? double(host[0]) / (double(host[1]) * 10.0) : 0.0;
    return LL_OK;
}

}  // extern "C"
