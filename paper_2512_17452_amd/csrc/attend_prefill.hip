// Chunked-prefill attention under the vertical-slash mask (Sec. 4.2).
#include "wgkv_dev.h"

namespace wgkv {

size_t attend_prefill_ws_bytes(const View &pv, int n_seqs, int64_t total_q) {
    (void)pv; (void)n_seqs; (void)total_q;
    return 256;
}

hipError_t launch_attend_prefill(const View &pv, const CallSeqs &cs, int layer, const void *q,
                                 const void *k, const void *v, const float *g, float tau,
                                 float scale, float *out, void *ws, hipStream_t st) {
    (void)pv; (void)cs; (void)layer; (void)q; (void)k; (void)v; (void)g; (void)tau; (void)scale;
    (void)out; (void)ws; (void)st;
    return hipErrorNotSupported;
}

}  // namespace wgkv
