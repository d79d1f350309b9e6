"""MI355X-native Solon linear block code: encode / locate / decode behind a C ABI (libsolon.so)."""
from .solon import (  # noqa: F401
    EXPORTS, LIB_PATH, Plan, SolonError,
    SOLON_OK, SOLON_E_INVAL, SOLON_E_BOUND, SOLON_E_POINTS, SOLON_E_DECODE, SOLON_E_NUMERIC, SOLON_E_HIP,
    SOLON_F32, SOLON_BF16,
    SOLON_Q_GROUPS, SOLON_Q_REDUNDANCY, SOLON_Q_MESSAGE_LEN, SOLON_Q_MAX_GROUP, SOLON_Q_WORKSPACE, SOLON_Q_HAS_DEVICE,
    SOLON_Q_LAST_REDO, SOLON_Q_LIMIT_GROUP, SOLON_Q_LIMIT_M, SOLON_Q_LAST_ONE_PASS,
    lib, solon_decode, solon_decode_majority, solon_decode_update, solon_draw_projection, solon_decode_status, solon_default_points, solon_encode, solon_locate,
    solon_locate_decode, solon_locate_static, solon_tune,
)
