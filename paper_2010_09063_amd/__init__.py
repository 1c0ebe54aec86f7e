"""MI355X-native private gradient step of DPSGD (arxiv 2010.09063): C-ABI HIP library + thin binding."""
from .dp_step import DpStep, DpStepError, dp_step_dense1_static, dp_step_sample_indices, dp_step_ceiling, load_library, LIB_PATH, EXPORTS  # noqa: F401
