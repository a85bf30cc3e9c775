"""ctypes binding of libwd's C ABI (``include/wd.h``, ``include/wdc.h``): same names, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing, ``load_library`` raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(HERE, "libwd.so")

WD_OK = 0
WD_E_NULL, WD_E_CONFIG, WD_E_ALIGN, WD_E_STATE, WD_E_HIP, WD_E_UNSUPPORTED, WD_E_SCRATCH = -1, -2, -3, -4, -5, -6, -7
WD_STATIC_SCRATCH_BYTES = 8 << 20
WD_RESET_ALL, WD_RESET_DONE = 0, 1
WD_OBS_PARTIAL, WD_OBS_FULL = 0, 1

_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)


class wd_config(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("num_envs", ctypes.c_int32),
        ("env_offset", ctypes.c_int32),
        ("num_agents", ctypes.c_int32),
        ("num_taggers", ctypes.c_int32),
        ("grid_size", ctypes.c_int32),
        ("num_actions", ctypes.c_int32),
        ("episode_length", ctypes.c_int32),
        ("tag_r2", ctypes.c_int32),
        ("obs_mode", ctypes.c_int32),
        ("obs_k", ctypes.c_int32),
        ("tag_reward", ctypes.c_float),
        ("tag_penalty", ctypes.c_float),
        ("seed", ctypes.c_uint64),
        ("stream", ctypes.c_void_p),
    ]


BUFFER_NAMES = ("pos_x", "pos_y", "pos_x0", "pos_y0", "live", "action", "reward", "obs",
                "t", "done", "n_live_runners", "tags_step")


class wd_buffers(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in BUFFER_NAMES]


class wd_rollout_buffers(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("action", "reward", "done", "obs")]


class wd_layout(ctypes.Structure):
    _fields_ = [
        ("obs_dim", ctypes.c_int32),
        ("per_agent_elems", ctypes.c_int64),
        ("obs_elems", ctypes.c_int64),
        ("per_env_elems", ctypes.c_int64),
        ("probs_elems", ctypes.c_int64),
        ("bytes_per_iteration", ctypes.c_int64),
    ]


class WdError(RuntimeError):
    def __init__(self, status, what, detail=""):
        self.status = status
        msg = f"{what}: {wd_strerror(status)} ({status})"
        super().__init__(msg + (f" [{detail}]" if detail else ""))


_lib = None


def load_library(path=LIBRARY):
    """Load libwd.so.  Raises if it has not been built (``python -m paper_2108_13976_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2108_13976_amd.build`")
        # PyTorch allocates the buffers and supplies the stream, so libwd has to bind to the HIP
        # runtime that PyTorch brings: load that first (two runtimes in one process do not share
        # a device context, and the second one loaded may not find the GPU at all)
        import torch  # noqa: F401

        lib = ctypes.CDLL(path)
        H = ctypes.c_void_p
        lib.wd_query_layout.argtypes = [ctypes.POINTER(wd_config), ctypes.POINTER(wd_layout)]
        lib.wd_create.argtypes = [ctypes.POINTER(wd_config), ctypes.POINTER(wd_buffers), ctypes.POINTER(H)]
        lib.wd_reset.argtypes = [H, ctypes.c_int]
        lib.wd_sample.argtypes = [H, ctypes.c_void_p]
        lib.wd_step.argtypes = [H]
        lib.wd_iterate.argtypes = [H, ctypes.c_void_p]
        lib.wd_iterate_static.argtypes = [ctypes.POINTER(wd_config), ctypes.POINTER(wd_buffers), ctypes.c_void_p,
                                          ctypes.c_uint64]
        lib.wd_rollout.argtypes = [H, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.POINTER(wd_rollout_buffers)]
        lib.wd_get_step.argtypes = [H, ctypes.POINTER(ctypes.c_uint64)]
        lib.wd_set_step.argtypes = [H, ctypes.c_uint64]
        lib.wd_invalidate_obs.argtypes = [H]
        lib.wd_destroy.argtypes = [H]
        lib.wd_strerror.argtypes = [ctypes.c_int]
        lib.wd_strerror.restype = ctypes.c_char_p
        lib.wd_last_error.argtypes = [H]
        lib.wd_last_error.restype = ctypes.c_char_p
        for name in ("wd_query_layout", "wd_create", "wd_reset", "wd_sample", "wd_step", "wd_iterate", "wd_rollout",
                     "wd_get_step", "wd_set_step", "wd_destroy", "wd_iterate_static", "wd_invalidate_obs"):
            getattr(lib, name).restype = ctypes.c_int
        _declare_continuous(lib)
        _lib = lib
    return _lib


# ---- the C ABI, one Python function per entry point -------------------------------------------
def make_config(num_envs, num_agents, num_taggers, grid_size, episode_length, seed=0, tag_r2=2,
                obs_mode=WD_OBS_PARTIAL, obs_k=4, tag_reward=1.0, tag_penalty=-1.0, env_offset=0,
                num_actions=5, stream=None):
    return wd_config(ctypes.sizeof(wd_config), num_envs, env_offset, num_agents, num_taggers, grid_size,
                     num_actions, episode_length, tag_r2, obs_mode, obs_k, tag_reward, tag_penalty, seed,
                     stream)


def wd_query_layout(cfg):
    out = wd_layout()
    rc = load_library().wd_query_layout(ctypes.byref(cfg), ctypes.byref(out))
    if rc != WD_OK:
        raise WdError(rc, "wd_query_layout")
    return out


def wd_create(cfg, bufs):
    handle = ctypes.c_void_p()
    rc = load_library().wd_create(ctypes.byref(cfg), ctypes.byref(bufs), ctypes.byref(handle))
    if rc != WD_OK:
        raise WdError(rc, "wd_create")
    return handle


def _call(handle, name, *args):
    rc = getattr(load_library(), name)(handle, *args)
    if rc != WD_OK:
        raise WdError(rc, name, wd_last_error(handle) if rc == WD_E_HIP else "")


def wd_reset(handle, mode):
    _call(handle, "wd_reset", int(mode))


def wd_sample(handle, probs_ptr):
    _call(handle, "wd_sample", ctypes.c_void_p(probs_ptr))


def wd_step(handle):
    _call(handle, "wd_step")


def wd_iterate(handle, probs_ptr):
    _call(handle, "wd_iterate", ctypes.c_void_p(probs_ptr))


def wd_iterate_static(cfg, bufs, probs_ptr, g):
    rc = load_library().wd_iterate_static(ctypes.byref(cfg), ctypes.byref(bufs), ctypes.c_void_p(probs_ptr), int(g))
    if rc != WD_OK:
        raise WdError(rc, "wd_iterate_static")


def wd_invalidate_obs(handle):
    _call(handle, "wd_invalidate_obs")


def wd_rollout(handle, probs_ring_ptr, ring_len, k, out=None):
    _call(handle, "wd_rollout", ctypes.c_void_p(probs_ring_ptr), int(ring_len), int(k),
          ctypes.byref(out) if out is not None else None)


def wd_get_step(handle):
    g = ctypes.c_uint64()
    _call(handle, "wd_get_step", ctypes.byref(g))
    return int(g.value)


def wd_set_step(handle, g):
    _call(handle, "wd_set_step", ctypes.c_uint64(int(g)))


def wd_destroy(handle):
    _call(handle, "wd_destroy")


def wd_strerror(status):
    return load_library().wd_strerror(int(status)).decode()


def wd_last_error(handle):
    return load_library().wd_last_error(handle).decode()


# ---- convenience: buffers allocated by PyTorch on the device ------------------------------------
class TagEnvs:
    """E Tag environments resident on one GPU.  PyTorch allocates the state tensors and supplies
    the stream; every call forwards to the C ABI."""

    def __init__(self, num_envs, num_agents, num_taggers, grid_size, episode_length, seed=0, tag_r2=2,
                 obs_mode=WD_OBS_PARTIAL, obs_k=4, tag_reward=1.0, tag_penalty=-1.0, env_offset=0,
                 device="cuda:0", stream=None):
        import torch

        load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("TagEnvs needs a GPU: the HIP path has no CPU fallback")
        self.device = torch.device(device)
        self.torch_stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.cfg = make_config(num_envs, num_agents, num_taggers, grid_size, episode_length, seed, tag_r2,
                               obs_mode, obs_k, tag_reward, tag_penalty, env_offset,
                               stream=self.torch_stream.cuda_stream)
        self.layout = wd_query_layout(self.cfg)
        E, N, D = num_envs, num_agents, self.layout.obs_dim
        self.E, self.N, self.D = E, N, D
        i32, f32 = torch.int32, torch.float32
        with torch.cuda.device(self.device):
            self.tensors = {n: torch.zeros((E, N), dtype=i32, device=self.device)
                            for n in ("pos_x", "pos_y", "pos_x0", "pos_y0", "live", "action")}
            self.tensors["reward"] = torch.zeros((E, N), dtype=f32, device=self.device)
            self.tensors["obs"] = torch.zeros((E, N, D), dtype=f32, device=self.device)
            self.tensors.update({n: torch.zeros((E,), dtype=i32, device=self.device)
                                 for n in ("t", "done", "n_live_runners", "tags_step")})
        for n, ten in self.tensors.items():
            setattr(self, n, ten)
        self.bufs = wd_buffers(*[self.tensors[n].data_ptr() for n in BUFFER_NAMES])
        self.handle = wd_create(self.cfg, self.bufs)

    def reset(self, mode=WD_RESET_ALL):
        wd_reset(self.handle, mode)

    def sample(self, probs):
        self._check_probs(probs)
        wd_sample(self.handle, probs.data_ptr())

    def step(self):
        wd_step(self.handle)

    def iterate(self, probs):
        self._check_probs(probs)
        wd_iterate(self.handle, probs.data_ptr())

    def rollout(self, probs_ring, k, record=("action", "reward", "done", "obs")):
        """k iterations in one launch; returns a dict of [k, ...] device tensors for the recorded outputs."""
        import torch

        ring_len = probs_ring.shape[0]
        if (probs_ring.dtype != torch.float32 or not probs_ring.is_contiguous() or probs_ring.device != self.device
                or probs_ring.numel() != ring_len * self.layout.probs_elems):
            raise ValueError("probs_ring must be a contiguous float32 device tensor of shape [R, E, N, 5]")
        E, N, D = self.E, self.N, self.D
        shapes = {"action": ((k, E, N), torch.int32), "reward": ((k, E, N), torch.float32),
                  "done": ((k, E), torch.int32), "obs": ((k, E, N, D), torch.float32)}
        out = {n: torch.empty(shapes[n][0], dtype=shapes[n][1], device=self.device) for n in record}
        bufs = wd_rollout_buffers(*[out[n].data_ptr() if n in out else None for n in ("action", "reward", "done", "obs")])
        wd_rollout(self.handle, probs_ring.data_ptr(), ring_len, k, bufs)
        return out

    def _check_probs(self, probs):
        import torch

        if (probs.dtype != torch.float32 or not probs.is_contiguous() or probs.device != self.device
                or probs.numel() != self.layout.probs_elems):
            raise ValueError("probs must be a contiguous float32 device tensor of shape [E, N, 5]")

    @property
    def global_step(self):
        return wd_get_step(self.handle)

    @global_step.setter
    def global_step(self, g):
        wd_set_step(self.handle, g)

    def to_host(self):
        """Synchronise the stream and copy every state array to numpy."""
        self.torch_stream.synchronize()
        return {n: t.cpu().numpy() for n, t in self.tensors.items()}

    def close(self):
        if self.handle is not None:
            wd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ================================================================================================
# continuous Tag (include/wdc.h)
# ================================================================================================
class wdc_config(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("num_envs", ctypes.c_int32),
        ("env_offset", ctypes.c_int32),
        ("num_agents", ctypes.c_int32),
        ("num_taggers", ctypes.c_int32),
        ("num_headings", ctypes.c_int32),
        ("episode_length", ctypes.c_int32),
        ("obs_k", ctypes.c_int32),
        ("world_size", ctypes.c_float),
        ("accel", ctypes.c_float),
        ("max_speed_tagger", ctypes.c_float),
        ("max_speed_runner", ctypes.c_float),
        ("tag_r2", ctypes.c_float),
        ("tag_reward", ctypes.c_float),
        ("tag_penalty", ctypes.c_float),
        ("seed", ctypes.c_uint64),
        ("stream", ctypes.c_void_p),
    ]


CBUFFER_NAMES = ("x", "y", "v", "h", "x0", "y0", "h0", "live", "action", "reward", "obs",
                 "t", "done", "n_live_runners", "tags_step")


class wdc_buffers(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in CBUFFER_NAMES]


class wdc_layout(ctypes.Structure):
    _fields_ = [
        ("obs_dim", ctypes.c_int32),
        ("agent_elems", ctypes.c_int64),
        ("action_elems", ctypes.c_int64),
        ("obs_elems", ctypes.c_int64),
        ("env_elems", ctypes.c_int64),
        ("probs_elems", ctypes.c_int64),
        ("bytes_per_iteration", ctypes.c_int64),
    ]


class wdc_rollout_buffers(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("action", "reward", "done", "obs")]


def _declare_continuous(lib):
    H = ctypes.c_void_p
    lib.wdc_rollout.argtypes = [H, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.POINTER(wdc_rollout_buffers)]
    lib.wdc_rollout.restype = ctypes.c_int
    lib.wdc_query_layout.argtypes = [ctypes.POINTER(wdc_config), ctypes.POINTER(wdc_layout)]
    lib.wdc_create.argtypes = [ctypes.POINTER(wdc_config), ctypes.POINTER(wdc_buffers), ctypes.POINTER(H)]
    lib.wdc_reset.argtypes = [H, ctypes.c_int]
    lib.wdc_sample.argtypes = [H, ctypes.c_void_p]
    lib.wdc_step.argtypes = [H]
    lib.wdc_iterate.argtypes = [H, ctypes.c_void_p]
    lib.wdc_get_step.argtypes = [H, ctypes.POINTER(ctypes.c_uint64)]
    lib.wdc_set_step.argtypes = [H, ctypes.c_uint64]
    lib.wdc_destroy.argtypes = [H]
    lib.wdc_last_error.argtypes = [H]
    lib.wdc_last_error.restype = ctypes.c_char_p
    for name in ("wdc_query_layout", "wdc_create", "wdc_reset", "wdc_sample", "wdc_step", "wdc_iterate",
                 "wdc_get_step", "wdc_set_step", "wdc_destroy"):
        getattr(lib, name).restype = ctypes.c_int


def make_cconfig(num_envs, num_agents, num_taggers, episode_length, seed=0, world_size=20.0, num_headings=16,
                 accel=0.25, max_speed_tagger=1.0, max_speed_runner=0.75, tag_r2=1.0, obs_k=4, tag_reward=1.0,
                 tag_penalty=-1.0, env_offset=0, stream=None):
    return wdc_config(ctypes.sizeof(wdc_config), num_envs, env_offset, num_agents, num_taggers, num_headings,
                      episode_length, obs_k, world_size, accel, max_speed_tagger, max_speed_runner, tag_r2,
                      tag_reward, tag_penalty, seed, stream)


def wdc_query_layout(cfg):
    out = wdc_layout()
    rc = load_library().wdc_query_layout(ctypes.byref(cfg), ctypes.byref(out))
    if rc != WD_OK:
        raise WdError(rc, "wdc_query_layout")
    return out


def wdc_create(cfg, bufs):
    handle = ctypes.c_void_p()
    rc = load_library().wdc_create(ctypes.byref(cfg), ctypes.byref(bufs), ctypes.byref(handle))
    if rc != WD_OK:
        raise WdError(rc, "wdc_create")
    return handle


def _ccall(handle, name, *args):
    rc = getattr(load_library(), name)(handle, *args)
    if rc != WD_OK:
        raise WdError(rc, name, wdc_last_error(handle) if rc == WD_E_HIP else "")


def wdc_reset(handle, mode):
    _ccall(handle, "wdc_reset", int(mode))


def wdc_sample(handle, probs_ptr):
    _ccall(handle, "wdc_sample", ctypes.c_void_p(probs_ptr))


def wdc_step(handle):
    _ccall(handle, "wdc_step")


def wdc_iterate(handle, probs_ptr):
    _ccall(handle, "wdc_iterate", ctypes.c_void_p(probs_ptr))


def wdc_rollout(handle, probs_ring_ptr, ring_len, k, out=None):
    _ccall(handle, "wdc_rollout", ctypes.c_void_p(probs_ring_ptr), int(ring_len), int(k),
           ctypes.byref(out) if out is not None else None)


def wdc_get_step(handle):
    g = ctypes.c_uint64()
    _ccall(handle, "wdc_get_step", ctypes.byref(g))
    return int(g.value)


def wdc_set_step(handle, g):
    _ccall(handle, "wdc_set_step", ctypes.c_uint64(int(g)))


def wdc_destroy(handle):
    _ccall(handle, "wdc_destroy")


def wdc_last_error(handle):
    return load_library().wdc_last_error(handle).decode()


class CTagEnvs:
    """E continuous-Tag environments resident on one GPU.  PyTorch allocates the state tensors and
    supplies the stream; every call forwards to the C ABI."""

    FLOAT_ARRAYS = ("x", "y", "v", "x0", "y0", "reward")

    def __init__(self, num_envs, num_agents, num_taggers, episode_length, seed=0, world_size=20.0,
                 num_headings=16, accel=0.25, max_speed_tagger=1.0, max_speed_runner=0.75, tag_r2=1.0, obs_k=4,
                 tag_reward=1.0, tag_penalty=-1.0, env_offset=0, device="cuda:0", stream=None):
        import torch

        load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("CTagEnvs needs a GPU: the HIP path has no CPU fallback")
        self.device = torch.device(device)
        self.torch_stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.cfg = make_cconfig(num_envs, num_agents, num_taggers, episode_length, seed, world_size, num_headings,
                                accel, max_speed_tagger, max_speed_runner, tag_r2, obs_k, tag_reward, tag_penalty,
                                env_offset, stream=self.torch_stream.cuda_stream)
        self.layout = wdc_query_layout(self.cfg)
        E, N, D = num_envs, num_agents, self.layout.obs_dim
        self.E, self.N, self.D = E, N, D
        i32, f32 = torch.int32, torch.float32
        with torch.cuda.device(self.device):
            self.tensors = {n: torch.zeros((E, N), dtype=f32 if n in self.FLOAT_ARRAYS else i32, device=self.device)
                            for n in ("x", "y", "v", "h", "x0", "y0", "h0", "live", "reward")}
            self.tensors["action"] = torch.zeros((E, N, 2), dtype=i32, device=self.device)
            self.tensors["obs"] = torch.zeros((E, N, D), dtype=f32, device=self.device)
            self.tensors.update({n: torch.zeros((E,), dtype=i32, device=self.device)
                                 for n in ("t", "done", "n_live_runners", "tags_step")})
        for n, ten in self.tensors.items():
            setattr(self, n, ten)
        self.bufs = wdc_buffers(*[self.tensors[n].data_ptr() for n in CBUFFER_NAMES])
        self.handle = wdc_create(self.cfg, self.bufs)

    def _check_probs(self, probs):
        import torch

        if (probs.dtype != torch.float32 or not probs.is_contiguous() or probs.device != self.device
                or probs.numel() != self.layout.probs_elems):
            raise ValueError("probs must be a contiguous float32 device tensor of shape [E, N, 2, 5]")

    def reset(self, mode=WD_RESET_ALL):
        wdc_reset(self.handle, mode)

    def sample(self, probs):
        self._check_probs(probs)
        wdc_sample(self.handle, probs.data_ptr())

    def step(self):
        wdc_step(self.handle)

    def iterate(self, probs):
        self._check_probs(probs)
        wdc_iterate(self.handle, probs.data_ptr())

    def rollout(self, probs_ring, k, record=("action", "reward", "done", "obs")):
        """k iterations in one launch; returns a dict of [k, ...] device tensors for the recorded outputs."""
        import torch

        ring_len = probs_ring.shape[0]
        if (probs_ring.dtype != torch.float32 or not probs_ring.is_contiguous() or probs_ring.device != self.device
                or probs_ring.numel() != ring_len * self.layout.probs_elems):
            raise ValueError("probs_ring must be a contiguous float32 device tensor of shape [R, E, N, 2, 5]")
        E, N, D = self.E, self.N, self.D
        shapes = {"action": ((k, E, N, 2), torch.int32), "reward": ((k, E, N), torch.float32),
                  "done": ((k, E), torch.int32), "obs": ((k, E, N, D), torch.float32)}
        out = {n: torch.empty(shapes[n][0], dtype=shapes[n][1], device=self.device) for n in record}
        bufs = wdc_rollout_buffers(*[out[n].data_ptr() if n in out else None for n in ("action", "reward", "done", "obs")])
        wdc_rollout(self.handle, probs_ring.data_ptr(), ring_len, k, bufs if out else None)
        return out

    def to_host(self):
        """Synchronise the stream and copy every state array to numpy."""
        self.torch_stream.synchronize()
        return {n: t.cpu().numpy() for n, t in self.tensors.items()}

    def close(self):
        if self.handle is not None:
            wdc_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
