"""ctypes binding of libmaze_cdna4.so (argument marshalling only).

Every function here checks tensor device / dtype / shape / contiguity, then
passes raw device pointers and the current HIP stream to the C ABI declared in
include/maze_cdna4.h.  There is no CPU fallback: if the library is missing or a
tensor is not on the GPU the call raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, byref, c_char_p, c_double, c_int, c_size_t, c_uint64, c_void_p)

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmaze_cdna4.so")

# name -> (restype, argtypes); the same list is what the header declares.
SIGNATURES = {
    "maze_strerror": (c_char_p, [c_int]),
    "maze_workspace_bytes": (c_int, [c_int, c_int, c_int, c_int, POINTER(c_size_t)]),
    "maze_create": (c_int, [POINTER(c_void_p), c_int, c_int, c_int, c_int, c_int, c_void_p,
                            c_size_t]),
    "maze_destroy": (c_int, [c_void_p]),
    "maze_reset_to_levels": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "maze_step": (c_int, [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_void_p]),
    "maze_rollout_plan": (c_int, [c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_size_t, POINTER(c_int),
                                  POINTER(c_size_t)]),
    "maze_rollout_static": (c_int, [c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p,
                                    c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_void_p]),
    "maze_render_obs": (c_int, [c_void_p, c_void_p, c_void_p]),
    "maze_get_state": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "maze_set_state": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "maze_get_levels": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "maze_level_metrics": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p]),
    "maze_set_kernel_variant": (c_int, [c_void_p, c_int]),
    "maze_set_obs_mode": (c_int, [c_void_p, c_int, c_int]),
    "editor_workspace_bytes": (c_int, [c_int, c_int, c_int, POINTER(c_size_t)]),
    "editor_create": (c_int, [POINTER(c_void_p), c_int, c_int, c_int, c_int, c_void_p, c_size_t]),
    "editor_destroy": (c_int, [c_void_p]),
    "editor_reset": (c_int, [c_void_p, c_void_p, c_void_p]),
    "editor_step": (c_int, [c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_void_p]),
    "editor_get_levels": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "editor_set_levels": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "editor_random_levels": (c_int, [c_void_p, c_uint64, c_uint64, c_void_p]),
    "editor_mutate_levels": (c_int, [c_void_p, c_uint64, c_uint64, c_int, c_void_p]),
    "compute_gae": (c_int, [c_void_p, c_void_p, c_void_p, c_int, c_int, c_double, c_double,
                            c_void_p, c_void_p, c_void_p]),
    "replay_scores": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_double, c_void_p,
                              c_void_p, c_void_p, c_void_p, c_void_p]),
    "replay_distribution": (c_int, [c_void_p, c_void_p, c_int, c_int, c_int, c_double, c_double, c_void_p,
                                    c_void_p]),
}

_lib = None


class MazeError(RuntimeError):
    pass


def load_library():
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MazeError(f"{LIB_PATH} is missing: run __graft_entry__.build() "
                            "(python -m paper_2311_12716_amd.build) first")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        msg = load_library().maze_strerror(rc).decode()
        raise MazeError(f"{what} failed: {msg} ({rc})")


def _launch(device: torch.device, what: str, fn, *args):
    """Call an entry point that takes the stream as its last argument, with `device` current
    (the C side refuses a context used under another device) and that device's current stream."""
    index = device.index if device.index is not None else torch.cuda.current_device()
    if torch.cuda.current_device() == index:
        rc = fn(*args, torch.cuda.current_stream(index).cuda_stream)
    else:
        with torch.cuda.device(index):
            rc = fn(*args, torch.cuda.current_stream(index).cuda_stream)
    _check(rc, what)


def _ptr(t: torch.Tensor | None, dtype, shape, name: str):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise MazeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise MazeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise MazeError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise MazeError(f"{name} must be contiguous")
    return t.data_ptr()


class MazeEnv:
    """Batched student maze on one GPU (handle + workspace owner)."""

    def __init__(self, N: int, H: int, W: int, view: int, max_steps: int, device="cuda:0"):
        lib = load_library()
        self.N, self.H, self.W, self.view, self.max_steps = N, H, W, view, max_steps
        self.device = torch.device(device)
        nbytes = c_size_t(0)
        _check(lib.maze_workspace_bytes(N, H, W, view, byref(nbytes)), "maze_workspace_bytes")
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes.value, dtype=torch.uint8, device=self.device)
            h = c_void_p()
            _check(lib.maze_create(byref(h), N, H, W, view, max_steps,
                                   self.workspace.data_ptr(), nbytes.value), "maze_create")
        self._h = h
        self._destroy = lib.maze_destroy

    def close(self):
        # (the destroy function is kept on the object: at interpreter shutdown module globals
        # may already be gone when __del__ runs)
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    __del__ = close

    def set_kernel_variant(self, variant: int):
        _check(load_library().maze_set_kernel_variant(self._h, variant), "maze_set_kernel_variant")

    def set_obs_mode(self, encoding: int, occlusion: int):
        """encoding 0 one-hot / 1 (type, colour, state); occlusion 0 off / 1 on."""
        _check(load_library().maze_set_obs_mode(self._h, int(encoding), int(occlusion)),
               "maze_set_obs_mode")

    def reset_to_levels(self, walls, agent_xy, agent_dir, goal_xy):
        N, H, W = self.N, self.H, self.W
        _launch(self.device, "maze_reset_to_levels", load_library().maze_reset_to_levels,
                self._h, _ptr(walls, torch.int8, (N, H, W), "walls"),
                _ptr(agent_xy, torch.int32, (N, 2), "agent_xy"),
                _ptr(agent_dir, torch.int8, (N,), "agent_dir"),
                _ptr(goal_xy, torch.int32, (N, 2), "goal_xy"))

    def step(self, actions, reward=None, done=None, obs=None, want_obs=True):
        """actions int8 [n_steps,N]; returns (reward, done, obs) with obs after each step."""
        if actions.dim() != 2:
            raise MazeError("actions must be [n_steps, N]")
        n_steps, N, k = actions.shape[0], self.N, self.view
        dev = self.device
        if reward is None:
            reward = torch.empty((n_steps, N), dtype=torch.float32, device=dev)
        if done is None:
            done = torch.empty((n_steps, N), dtype=torch.uint8, device=dev)
        if obs is None and want_obs:
            obs = torch.empty((n_steps, N, k, k, 3), dtype=torch.int8, device=dev)
        _launch(self.device, "maze_step", load_library().maze_step,
            self._h, _ptr(actions, torch.int8, (n_steps, N), "actions"), n_steps,
            _ptr(reward, torch.float32, (n_steps, N), "reward"),
            _ptr(done, torch.uint8, (n_steps, N), "done"),
            _ptr(obs, torch.int8, (n_steps, N, k, k, 3), "obs"))
        return reward, done, obs

    def render_obs(self, obs=None):
        N, k = self.N, self.view
        if obs is None:
            obs = torch.empty((N, k, k, 3), dtype=torch.int8, device=self.device)
        _launch(self.device, "maze_render_obs", load_library().maze_render_obs, self._h,
                _ptr(obs, torch.int8, (N, k, k, 3), "obs"))
        return obs

    def get_state(self):
        N, dev = self.N, self.device
        xy = torch.empty((N, 2), dtype=torch.int32, device=dev)
        d = torch.empty((N,), dtype=torch.int8, device=dev)
        t = torch.empty((N,), dtype=torch.int32, device=dev)
        _launch(self.device, "maze_get_state", load_library().maze_get_state, self._h, xy.data_ptr(),
                d.data_ptr(), t.data_ptr())
        return xy, d, t

    def set_state(self, xy=None, direction=None, t=None):
        """Overwrite position int32 [N,2], heading int8 [N], step count int32 [N]; None keeps a part."""
        N = self.N
        _launch(self.device, "maze_set_state", load_library().maze_set_state,
            self._h, _ptr(xy, torch.int32, (N, 2), "xy"), _ptr(direction, torch.int8, (N,), "direction"),
            _ptr(t, torch.int32, (N,), "t"))

    def get_levels(self):
        N, H, W, dev = self.N, self.H, self.W, self.device
        walls = torch.empty((N, H, W), dtype=torch.int8, device=dev)
        axy = torch.empty((N, 2), dtype=torch.int32, device=dev)
        ad = torch.empty((N,), dtype=torch.int8, device=dev)
        gxy = torch.empty((N, 2), dtype=torch.int32, device=dev)
        _launch(self.device, "maze_get_levels", load_library().maze_get_levels, self._h,
                walls.data_ptr(), axy.data_ptr(), ad.data_ptr(), gxy.data_ptr())
        return walls, axy, ad, gxy


    def level_metrics(self, n_walls=None, path_len=None):
        """(n_walls, path_len) int32 [N] of the current levels; path_len -1 = unreachable."""
        N, dev = self.N, self.device
        if n_walls is None:
            n_walls = torch.empty((N,), dtype=torch.int32, device=dev)
        if path_len is None:
            path_len = torch.empty((N,), dtype=torch.int32, device=dev)
        _launch(self.device, "maze_level_metrics", load_library().maze_level_metrics, self._h,
                n_walls.data_ptr(), path_len.data_ptr())
        return n_walls, path_len


class EditorEnv:
    """Batched teacher design env on one GPU."""

    def __init__(self, N: int, H: int, W: int, n_walls: int, device="cuda:0"):
        lib = load_library()
        self.N, self.H, self.W, self.n_walls = N, H, W, n_walls
        self.device = torch.device(device)
        nbytes = c_size_t(0)
        _check(lib.editor_workspace_bytes(N, H, W, byref(nbytes)), "editor_workspace_bytes")
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes.value, dtype=torch.uint8, device=self.device)
            h = c_void_p()
            _check(lib.editor_create(byref(h), N, H, W, n_walls, self.workspace.data_ptr(),
                                     nbytes.value), "editor_create")
        self._h = h
        self._destroy = lib.editor_destroy

    def close(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    __del__ = close

    def reset(self, agent_dir_init):
        _launch(self.device, "editor_reset", load_library().editor_reset,
            self._h, _ptr(agent_dir_init, torch.int8, (self.N,), "agent_dir_init"))

    def step(self, actions, obs=None, t=None, done=None, want_obs=True):
        if actions.dim() != 2:
            raise MazeError("actions must be [n_steps, N]")
        n_steps, N, H, W, dev = actions.shape[0], self.N, self.H, self.W, self.device
        if obs is None and want_obs:
            obs = torch.empty((n_steps, N, H, W, 3), dtype=torch.int8, device=dev)
        if t is None:
            t = torch.empty((n_steps, N), dtype=torch.int32, device=dev)
        if done is None:
            done = torch.empty((n_steps, N), dtype=torch.uint8, device=dev)
        _launch(self.device, "editor_step", load_library().editor_step,
            self._h, _ptr(actions, torch.int32, (n_steps, N), "actions"), n_steps,
            _ptr(obs, torch.int8, (n_steps, N, H, W, 3), "obs"),
            _ptr(t, torch.int32, (n_steps, N), "t"),
            _ptr(done, torch.uint8, (n_steps, N), "done"))
        return obs, t, done

    def get_levels(self):
        N, H, W, dev = self.N, self.H, self.W, self.device
        walls = torch.empty((N, H, W), dtype=torch.int8, device=dev)
        axy = torch.empty((N, 2), dtype=torch.int32, device=dev)
        ad = torch.empty((N,), dtype=torch.int8, device=dev)
        gxy = torch.empty((N, 2), dtype=torch.int32, device=dev)
        _launch(self.device, "editor_get_levels", load_library().editor_get_levels, self._h,
                walls.data_ptr(), axy.data_ptr(), ad.data_ptr(), gxy.data_ptr())
        return walls, axy, ad, gxy

    def set_levels(self, walls, agent_xy, agent_dir, goal_xy):
        N, H, W = self.N, self.H, self.W
        _launch(self.device, "editor_set_levels", load_library().editor_set_levels,
            self._h, _ptr(walls, torch.int8, (N, H, W), "walls"),
            _ptr(agent_xy, torch.int32, (N, 2), "agent_xy"),
            _ptr(agent_dir, torch.int8, (N,), "agent_dir"),
            _ptr(goal_xy, torch.int32, (N, 2), "goal_xy"))

    def random_levels(self, seed: int, first_level_id: int = 0):
        """Replace every env by a level of the counter-based random generator."""
        _launch(self.device, "editor_random_levels", load_library().editor_random_levels, self._h,
                int(seed), int(first_level_id))

    def mutate_levels(self, seed: int, first_level_id: int, n_edits: int):
        _launch(self.device, "editor_mutate_levels", load_library().editor_mutate_levels, self._h,
                int(seed), int(first_level_id), int(n_edits))


def maze_rollout_static(H: int, W: int, view: int, max_steps: int, walls, agent_xy, agent_dir, goal_xy,
                        actions, reward, done, obs=None):
    """Reset to the given levels and roll out `actions` with no env object and no workspace (the
    library's static device array holds the state); every tensor, outputs included, is the caller's."""
    if actions.dim() != 2:
        raise MazeError("actions must be [n_steps, N]")
    n_steps, N = actions.shape
    _launch(actions.device, "maze_rollout_static", load_library().maze_rollout_static,
            N, H, W, view, max_steps, _ptr(walls, torch.int8, (N, H, W), "walls"),
            _ptr(agent_xy, torch.int32, (N, 2), "agent_xy"), _ptr(agent_dir, torch.int8, (N,), "agent_dir"),
            _ptr(goal_xy, torch.int32, (N, 2), "goal_xy"), _ptr(actions, torch.int8, (n_steps, N), "actions"),
            n_steps, _ptr(reward, torch.float32, (n_steps, N), "reward"),
            _ptr(done, torch.uint8, (n_steps, N), "done"),
            _ptr(obs, torch.int8, (n_steps, N, view, view, 3), "obs"))
    return reward, done, obs


def compute_gae(rewards, values, dones, gamma: float, lam: float, adv=None, returns=None,
                want_returns=True):
    """rewards f32 [T,N], values f32 [T+1,N], dones u8 [T,N] -> (adv, returns) f32 [T,N]."""
    if rewards.dim() != 2:
        raise MazeError("rewards must be [T, N]")
    T, N = rewards.shape
    if adv is None:
        adv = torch.empty((T, N), dtype=torch.float32, device=rewards.device)
    if returns is None and want_returns:
        returns = torch.empty((T, N), dtype=torch.float32, device=rewards.device)
    _launch(rewards.device, "compute_gae", load_library().compute_gae,
        _ptr(rewards, torch.float32, (T, N), "rewards"),
        _ptr(values, torch.float32, (T + 1, N), "values"),
        _ptr(dones, torch.uint8, (T, N), "dones"), T, N, float(gamma), float(lam),
        _ptr(adv, torch.float32, (T, N), "adv"),
        _ptr(returns, torch.float32, (T, N), "returns"))
    return adv, returns


def replay_scores(rewards, values, dones, adv, gamma: float, rmax=None):
    """Per-level replay scores -> (rmax, maxmc, pvl) f32 [N]; rmax (f32 [N]) is updated in place
    when given, else a new tensor holds the rollout's best return."""
    if rewards.dim() != 2:
        raise MazeError("rewards must be [T, N]")
    T, N = rewards.shape
    dev = rewards.device
    rmax_in = None if rmax is None else _ptr(rmax, torch.float32, (N,), "rmax")
    if rmax is None:
        rmax = torch.empty((N,), dtype=torch.float32, device=dev)
    maxmc = torch.empty((N,), dtype=torch.float32, device=dev)
    pvl = torch.empty((N,), dtype=torch.float32, device=dev)
    _launch(rewards.device, "replay_scores", load_library().replay_scores,
        _ptr(rewards, torch.float32, (T, N), "rewards"),
        _ptr(values, torch.float32, (T + 1, N), "values"),
        _ptr(dones, torch.uint8, (T, N), "dones"),
        _ptr(adv, torch.float32, (T, N), "adv"), T, N, float(gamma), rmax_in,
        rmax.data_ptr(), maxmc.data_ptr(), pvl.data_ptr())
    return rmax, maxmc, pvl


def replay_distribution(scores, last_seen, now: int, rank: bool, temperature: float,
                        staleness_coef: float, prob=None):
    """scores f32 [K], last_seen i32 [K] -> replay probabilities f32 [K]."""
    if scores.dim() != 1:
        raise MazeError("scores must be [K]")
    K = scores.shape[0]
    if prob is None:
        prob = torch.empty((K,), dtype=torch.float32, device=scores.device)
    _launch(scores.device, "replay_distribution", load_library().replay_distribution,
        _ptr(scores, torch.float32, (K,), "scores"), _ptr(last_seen, torch.int32, (K,), "last_seen"),
        K, int(now), 1 if rank else 0, float(temperature), float(staleness_coef),
        _ptr(prob, torch.float32, (K,), "prob"))
    return prob
