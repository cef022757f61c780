#include "common.hpp"
namespace vista {
bool mfma_sglu_ffn_supported(const vista_ffn_desc&) { return false; }
vista_status mfma_sglu_ffn(const vista_ffn_desc&, float, const void*, const void*, const void*, const void*, void*, hipStream_t) { return VISTA_ERR_UNSUPPORTED; }
}
