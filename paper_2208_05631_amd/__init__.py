"""libqadagrad: MI355X-native hot path of QCMD adagrad / QRDA adagrad (arXiv 2208.05631).

The package is a thin binding over the C ABI declared in include/qadagrad.h.  Every step of
the path runs in the HIP kernels of libqadagrad.so; torch is used for device memory and
streams only.  Importing `binding` fails loudly if the shared library has not been built.
"""
from .binding import (  # noqa: F401
    QA_CSR, QA_DENSE, QA_METHOD_QCMD, QA_METHOD_QRDA, QA_OP_GRAD_CSR, QA_OP_GRAD_DENSE, QA_OP_QUANTIZE, QA_OP_STEP, QA_OP_SELECT, QA_OP_STEP_SELECTED, QA_OP_QUANTIZE_EXACT,
    QA_REQUANT_BUCKET, QA_REQUANT_GLOBAL, QA_REQUANT_NONE, QA_THRESH_GIVEN, QA_THRESH_EXACT, Layout, QaError,
    lib_path, qa_aggregate_unpack, qa_local_grad, qa_local_grad_batched, qa_quantize_pack, qa_step_qcmd, qa_step_qrda,
    qa_strerror, qa_version, qa_workspace_bytes, qa_indicator, qa_indicator_or,
    qa_quantize_pack_selected, qa_decode_selected, qa_quantize_pack_stochastic,
    SegmentPlan, qa_segment_plan_bytes, qa_segment_plan_init, qa_segment_workspace_bytes,
    qa_quantize_pack_segments, qa_step_qcmd_segments, qa_step_qrda_segments, qa_select_codes, qa_segment_plan_host,
    qa_step_qcmd_selected, qa_step_qrda_selected, qa_aggregate_quantize, qa_aggregate_quantize_selected,
    qa_quantize_pack_static,
)
from . import placement  # noqa: F401,E402  (where large arrays lie in device memory)
