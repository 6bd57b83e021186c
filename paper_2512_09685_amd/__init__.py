"""MI355X-native group-synchronous parameter update of STAR (arXiv 2512.09685).

The product is ``libstar.so`` (C ABI, declared in ``include/star.h``); this
package is its thin Python binding.  PyTorch only supplies device memory and
streams.
"""
from .binding import (  # noqa: F401
    MODE_ASGD, MODE_DYNAMIC_X, star_group_gram, star_noise_scale, MODE_SSGD, MODE_STATIC_X, star_select_mode_ar, star_select_mode_ps,
    GradRows, KERNEL_AFFINE, KERNEL_AFFINE_MFMA, KERNEL_AUTO, KERNEL_SEQ, OPT_DIRECT_NORMS, StarError, UpdateStream, last_error, library_path, load_library,
    star_group_norms, star_group_reduce, star_group_update, star_group_update_noalloc, star_group_update_publish, star_plan_affine, star_plan_choice, star_plan_claims, star_plan_even_split, star_shutdown,
    star_version, star_workspace_bytes,
)
