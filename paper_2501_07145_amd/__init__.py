"""MI355X-native RFSF-TS feature map and feature Gram (C-ABI library + thin binding)."""
from .binding import (  # noqa: F401
    RfsfTsError, lib_path, load_library, rfsf_ts_features, rfsf_ts_features_static, rfsf_ts_gram,
    rfsf_ts_validate_tables, rfsf_ts_workspace_bytes, rfsf_ts_time_cut, rfsf_ts_profile_enable, rfsf_ts_profile_read, rfsf_ts_probe_peaks,
    feature_row_stride, rfsf_ts_normalize_features, rfsf_dp1d_features, rfsf_trp_features, rfsf_trp_workspace_bytes,
)
