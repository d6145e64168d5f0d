// temporary: context entry points land with the decoder kernels
#include "psd_host.h"
extern "C" {
int psd_create(const psd_model_desc*, const psd_model_desc*, const psd_model_desc*, const psd_params*, psd_ctx** out) { if (out) *out = nullptr; return PSD_EINVAL; }
void psd_destroy(psd_ctx*) {}
size_t psd_pool_bytes_needed(const psd_model_desc*, const psd_model_desc*, const psd_model_desc*, const psd_params*) { return 0; }
int psd_set_decoding(psd_ctx*, float, float, int32_t, int32_t, float) { return PSD_EINVAL; }
int psd_generate(psd_ctx*, const int32_t*, int32_t, int32_t, uint64_t, int32_t*, psd_stats*) { return PSD_EINVAL; }
int psd_generate_plain(psd_ctx*, int32_t, const int32_t*, int32_t, int32_t, uint64_t, int32_t*, psd_stats*) { return PSD_EINVAL; }
int psd_forward(psd_ctx*, int32_t, const int32_t*, int32_t, int32_t, float*) { return PSD_EINVAL; }
int psd_set_trace(psd_ctx*, psd_trace_fn, void*) { return PSD_EINVAL; }
int psd_profile(psd_ctx*, int32_t) { return PSD_EINVAL; }
int psd_kernel_stats(psd_ctx*, psd_kernel_stat*, int32_t) { return PSD_EINVAL; }
const char* psd_last_error(const psd_ctx*) { return psd::tls_error(); }
}
