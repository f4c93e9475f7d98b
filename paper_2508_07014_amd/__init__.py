"""MI355X-native phrase-boosting tree (GPU-PB shallow-fusion context biasing): Python binding of libpb.so."""
from .binding import (  # noqa: F401
    EXPORTS, PB_EHIP, PB_EINVAL, PB_ENOMEM, PB_ERANGE, PB_EUNSUPPORTED, PB_OK, PB_SELECT_FUSED, PB_SELECT_TWO_STAGE, PB_SELECT_TWO_STAGE_CTC, PB_W_LOGDEPTH, PB_W_UNIFORM, PB_W_UNIFORM_FINAL,
    Forest, PbError, Tree, library_path, load, pb_build, pb_forest_build, pb_forest_free, pb_free, pb_fuse_frames_forest, pb_fuse_step_beam_forest, pb_fuse_step_forest, pb_score_forest, pb_fuse_frames, pb_fuse_frames_select, pb_fuse_frames_plan, pb_fuse_frames_workspace_bytes, pb_fuse_frames_ws, pb_fuse_frames_static, pb_fuse_step, pb_fuse_step_select, pb_fuse_step_beam,
    pb_host_arrays, pb_info, pb_score, pb_state_prefix, pb_validate, pb_validate_states, strerror,
)
