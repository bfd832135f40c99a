"""MI355X-native evaluator for property-annotated matrix chains (MOM: Matrix Operations in MLIR).

The product lives in libmom.so (csrc/, C ABI in include/mom.h); this package is its ctypes
binding, with the same function names.
"""
from .binding import (  # noqa: F401
    BoundEval, Equation, MOM_DIAGONAL, MOM_GENERAL, MOM_IDENTITY, MOM_LOWER_TRI, MOM_OUT_ZERO_FILL_TRIANGLE, MOM_PLAN_MIN_MULTS, MOM_PLAN_MIN_TIME, MOM_STATIC_WORKSPACE_BYTES, MOM_UPPER_TRI, MomError,
    Plan, bind_chain_eval, bind_chain_eval_batched, bind_equation_eval, library, mom_chain_eval, mom_chain_eval_batched, mom_chain_eval_static, mom_chain_plan, mom_chain_plan_ex, mom_equation_eval, mom_equation_plan, mom_init, mom_plan_cost_mults,
    mom_plan_from_splits, mom_plan_num_launches, mom_plan_num_products, mom_plan_product, mom_plan_result, mom_plan_splits, mom_plan_string,
    mom_plan_workspace_bytes, mom_probe_mfma_peak, mom_status_string,
)
