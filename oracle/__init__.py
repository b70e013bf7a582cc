"""CPU oracle (test infrastructure only). See rfsf_ts_oracle.c for what it computes."""
from .rfsf_ts_oracle import (  # noqa: F401
    build, dp1d_features, features, features_order, features_ragged, gram, increments, normalize, threads, trp_features, lib_path,
)
