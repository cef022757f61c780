#include "common.hpp"
namespace vista {
bool mfma_summarize_supported(const vista_summarize_desc&) { return false; }
size_t mfma_summarize_workspace(const vista_summarize_desc&, int) { return 0; }
vista_status mfma_summarize(const SummarizeArgs&) { return VISTA_ERR_UNSUPPORTED; }
}
