"""svb: singular values on one MI355X by two-stage reduction to bidiagonal form.

Thin Python binding over the C-ABI library libsvb.so (include/svb.h).  The
binding only marshals arguments; every step runs in the library.
"""
from .binding import (  # noqa: F401
    SVB_F64, SVB_F32, SVB_F16, SVB_BF16, SVB_OK, SvbError, library_path, load_library,
    svb_workspace_bytes, svb_svdvals, svb_ge2gb, svb_gb2bd, svb_gb2bd_workspace_bytes, svb_bdsvals, svb_bdsvals_dev,
    svb_bdsvals_dev_workspace_bytes, svb_last_timings,
    svb_status_string, svdvals, dtype_code, svb_profile_enable, svb_profile_collect,
    svb_profile_get, SVB_PROF_PANEL, SVB_PROF_UPDATE, SVB_PROF_UPDATE_UPPER, SVB_PROF_BAND_REDUCE,
    SVB_PROF_NARROW, SVB_PROF_STAGE3, SVB_PROF_NAMES, svb_gb2bd_noalloc, svb_choose_nb,
)
