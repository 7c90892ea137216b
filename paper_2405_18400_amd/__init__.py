"""Superposed Decoding hot path for MI355X: thin Python binding over the C-ABI library."""
from .binding import (  # noqa: F401
    SpdError, SpdDecodeCfg, SpdSampleCfg, SpdModelCfg, Session, lib, library_path,
    spd_workspace_bytes, spd_ngram_table_bytes, spd_strerror,
    spd_op_gemv, spd_op_swiglu, spd_op_attention, spd_op_attention_static,
    spd_test_state_layout, spd_test_state_status,
)
