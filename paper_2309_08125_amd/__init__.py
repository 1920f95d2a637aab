"""MI355X-native pipeline-template planner (Oobleck, Section 4.1) -- Python binding."""
from .binding import (  # noqa: F401
    OOB_ECAPACITY, OOB_EHIP, OOB_EINVAL, OOB_EOVERFLOW, OOB_FORBIDDEN, OOB_OK, SYMBOLS,
    DeviceProfile, DeviceTemplates, Planner, load, oob_plan_create, oob_plan_destroy,
    oob_plan_layout_selftest, oob_plan_max_stages, oob_plan_templates, oob_plan_templates_batch, oob_plan_workspace_size,
    template_stages, OOB_OPT_PLAIN_SPLIT, OOB_OPT_XCD_ORDER, OOB_OPT_ONE_STREAM,
    OOB_OPT_SELECT8_FROM, OOB_OPT_FUSE_FROM,
    EXACT_SYMBOLS, ExactMinimum, oob_exact_minimum, oob_exact_workspace_size,
    OOB_EXACT_LIMIT_CAN_BIND, oob_exact_minimum_staged, oob_exact_staged_workspace_size,
    DIST_SYMBOLS, Distributor, oob_dist_choose, oob_dist_solve,
    OOB_DIST_OK, OOB_DIST_TOO_FEW_MICROBATCHES, OOB_DIST_TOO_MANY_TEMPLATES, OOB_DIST_BAD_TIME, OOB_DIST_NO_PIPELINE,
    RECONF_ROWS, RECONF_SYMBOLS, FailureSimulator, oob_reconf_simulate,
    INST_SYMBOLS, Instantiator, oob_inst_count, oob_inst_enumerate, oob_inst_workspace_size,
    OOB_INST_STATIC_BYTES, oob_inst_enumerate_static,
)
