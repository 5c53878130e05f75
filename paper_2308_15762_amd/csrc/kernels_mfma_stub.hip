#include "kernels.h"
namespace hanayo { namespace k {
bool gemm_mfma_supported(const GemmArgs&) { return false; }
int gemm_mfma(const GemmArgs&, hipStream_t) { return set_error(HANAYO_EUNSUPPORTED, "no mfma gemm"); }
bool attn_mfma_supported(const AttnArgs&) { return false; }
int attn_forward_mfma(const AttnArgs&, hipStream_t) { return set_error(HANAYO_EUNSUPPORTED, "no mfma attention"); }
int attn_backward_mfma(const AttnArgs&, hipStream_t) { return set_error(HANAYO_EUNSUPPORTED, "no mfma attention"); }
}}
