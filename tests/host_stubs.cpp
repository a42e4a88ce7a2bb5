// Stand-ins for the kernel launchers, so that the library's host code (argument checks, bookkeeping, launch
// preparation) can be built and run under the host sanitizers with no device code at all.  Every launcher reports
// success; the kernel-variant queries describe one 256-query variant per head_dim and cache kind.
#include "../paper_2509_22622_amd/csrc/kernels.h"

namespace ll {
int attn_variant_count() { return 4; }
const char* attn_variant_name(int v) { return v >= 1 && v <= 4 ? "stub" : nullptr; }
int attn_variant_default(int D, int kblock) { return (kblock == KBLOCK8 ? 2 : 0) + (D == 128 ? 1 : 2); }
int attn_variant_qtile(int) { return 256; }
bool attn_variant_supports(int v, int D, int kblock) { return v == attn_variant_default(D, kblock); }
bool attn_variant_sink_shift(int v) { return v <= 2; }
int attn_variant_lse(int D) { return D == 128 ? 1 : 2; }
int attn_variant_qscale(int D) { return D == 128 ? 1 : 2; }
int attn_variant_qrope(int D) { return D == 128 ? 1 : 2; }
int attn_variant_short_keys(int D) { return D == 128 ? 1 : 2; }
bool attn_variant_applies_scale(int) { return true; }
bool attn_variant_out_frag(int) { return true; }
int bwd_tile_cols(int) { return 256; }
hipError_t launch_append(const AppendParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_append8(const AppendParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_read_frame(const ReadFrameParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_read_frame8(const ReadFrameParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_attn(const AttnParams&, int, hipStream_t) { return hipSuccess; }
hipError_t launch_out_proj(const OutProjParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_pack_out_weight(const uint16_t*, uint16_t*, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_bwd_dq(const BwdParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_bwd_dkv(const BwdParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_bwd_delta(const float*, const uint16_t*, float*, int, int, int, int64_t, hipStream_t) { return hipSuccess; }
hipError_t launch_bwd_finish(const BwdFinishParams&, hipStream_t) { return hipSuccess; }
hipError_t launch_probe_mfma(float*, unsigned long long*, int, int, int, int, int, hipStream_t) { return hipSuccess; }
}  // namespace ll
