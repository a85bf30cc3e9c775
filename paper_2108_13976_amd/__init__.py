"""MI355X-native batched Tag roll-out path (sampler, step, reset) behind a C ABI.

``binding`` is a thin ctypes layer over ``libwd.so`` (built by ``build.py`` from
``csrc/``); PyTorch only allocates device memory and supplies the stream.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    WD_OBS_FULL, WD_OBS_PARTIAL, WD_RESET_ALL, WD_RESET_DONE, TagEnvs, WdError, load_library,
    wd_create, wd_destroy, wd_get_step, wd_invalidate_obs, wd_iterate, wd_iterate_static, wd_last_error, wd_query_layout, wd_reset, wd_rollout,
    wd_sample, wd_set_step, wd_step, wd_strerror,
    CTagEnvs, wdc_create, wdc_destroy, wdc_get_step, wdc_iterate, wdc_query_layout, wdc_reset, wdc_rollout, wdc_sample,
    wdc_set_step, wdc_step,
)
