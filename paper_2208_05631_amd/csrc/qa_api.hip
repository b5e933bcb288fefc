// Entry points of libqadagrad that launch nothing: version, error strings, workspace sizes.
#include "qa_common.h"

namespace qa {
size_t quantize_workspace_bytes(const qa_layout* L);
size_t exact_sort_workspace_bytes(const qa_layout* L);
size_t step_workspace_bytes(const qa_layout* L);
size_t select_workspace_bytes(const qa_layout* L);
size_t step_selected_workspace_bytes(const qa_layout* L);
size_t grad_workspace_bytes(int64_t d, bool csr);
}  // namespace qa

extern "C" int qa_version(void) { return QA_VERSION; }

extern "C" const char* qa_strerror(int code) {
  switch (code) {
    case QA_OK: return "ok";
    case QA_ERR_INVALID_ARG: return "invalid argument (null pointer, size, stride or scalar out of range)";
    case QA_ERR_ALIGNMENT: return "buffer alignment requirement not met";
    case QA_ERR_WORKSPACE: return "workspace missing or too small (see qa_workspace_bytes)";
    case QA_ERR_LAUNCH: return "HIP kernel launch failed";
    case QA_ERR_UNSUPPORTED: return "request not supported by this build";
    case QA_ERR_TOO_LARGE: return "problem needs more scratch than the library's static array holds";
    default: return "unknown error code";
  }
}

extern "C" size_t qa_workspace_bytes(const qa_layout* layout, int op) {
  using namespace qa;
  if (!layout) return 0;
  if (op == QA_OP_GRAD_CSR || op == QA_OP_GRAD_DENSE) {
    if (layout->d < 1 || layout->M < 1) return 0;
    return (size_t)layout->M * grad_workspace_bytes(layout->d, op == QA_OP_GRAD_CSR);
  }
  if (check_layout(layout) != QA_OK) return 0;
  if (op == QA_OP_QUANTIZE) return quantize_workspace_bytes(layout);
  if (op == QA_OP_QUANTIZE_EXACT)
    return quantize_workspace_bytes(layout) + exact_sort_workspace_bytes(layout);
  if (op == QA_OP_STEP) return step_workspace_bytes(layout);
  if (op == QA_OP_SELECT) return select_workspace_bytes(layout);
  if (op == QA_OP_STEP_SELECTED) return step_selected_workspace_bytes(layout);
  return 0;
}
