#include "common.hpp"
namespace vista {
bool mfma_target_attend_supported(const vista_attend_desc&) { return false; }
vista_status mfma_target_attend(const vista_attend_desc&, float, const void*, const void*, void*, hipStream_t) { return VISTA_ERR_UNSUPPORTED; }
}
