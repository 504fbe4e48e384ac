"""Python binding of libstrassen_tc (argument marshalling only; every step of the contraction runs in the
library's HIP kernels).  The functions mirror the C ABI declared in include/strassen_tc.h."""
from .binding import (  # noqa: F401
    TcError,
    Plan,
    VARIANTS,
    TC_LEVEL_AUTO,
    TC_VARIANT_AUTO,
    build,
    lib_path,
    load_library,
    tc_contract,
    tc_contract_timed,
    tc_destroy,
    tc_plan,
    tc_plan_info,
    tc_plan_predict,
    tc_model_defaults,
    tc_plan_schedule,
    tc_plan_vector,
    tc_plan_workspace_bytes,
    tc_strerror,
    contract,
)
