"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol
the header declares, the binding covers them, and host-side validation returns
error codes without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "maze_cdna4.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int|const char \*)\s*\*?\s*([a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    from paper_2311_12716_amd import binding
    return binding.load_library()


def test_header_declares_the_five_named_calls():
    names = declared_functions()
    for n in ("maze_reset_to_levels", "maze_step", "maze_render_obs", "editor_step", "compute_gae"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2311_12716_amd import binding
    names = declared_functions()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    assert sorted(binding.SIGNATURES) == names


def test_workspace_size_validation(lib):
    n = ctypes.c_size_t(0)
    assert lib.maze_workspace_bytes(32768, 13, 13, 5, ctypes.byref(n)) == 0 and n.value > 0
    assert n.value % 256 == 0
    assert lib.maze_workspace_bytes(8, 13, 13, 4, ctypes.byref(n)) == -1      # even view
    # a 1 x 1 view would leave the grid without the ring of wall that bounds the moves
    assert lib.maze_workspace_bytes(8, 13, 13, 1, ctypes.byref(n)) == -1
    assert lib.maze_workspace_bytes(8, 13, 13, -3, ctypes.byref(n)) == -1
    h = ctypes.c_void_p()
    assert lib.maze_create(ctypes.byref(h), 8, 13, 13, 1, 250, 256, 1 << 20) == -1 and h.value is None
    assert lib.maze_workspace_bytes(0, 13, 13, 5, ctypes.byref(n)) == -1
    assert lib.maze_workspace_bytes(8, 13, 0, 5, ctypes.byref(n)) == -1
    assert lib.maze_workspace_bytes(8, 60, 60, 7, ctypes.byref(n)) == -3     # padded rows > 64 bits
    # the limit itself: side + 2 (view - 1) = 64
    for side, view in ((60, 3), (56, 5), (52, 7), (48, 9)):
        assert lib.maze_workspace_bytes(8, side, side, view, ctypes.byref(n)) == 0
        assert lib.maze_workspace_bytes(8, side + 1, side, view, ctypes.byref(n)) == -3
        assert lib.maze_workspace_bytes(8, side, side + 1, view, ctypes.byref(n)) == -3
    assert lib.maze_workspace_bytes(8, 13, 13, 5, None) == -2
    assert lib.editor_workspace_bytes(8, 13, 13, ctypes.byref(n)) == 0 and n.value > 0
    assert lib.editor_workspace_bytes(8, 1, 1, ctypes.byref(n)) == -1
    assert lib.editor_workspace_bytes(8, 100, 100, ctypes.byref(n)) == -3
    assert lib.editor_workspace_bytes(-1, 13, 13, ctypes.byref(n)) == -1


def test_create_rejects_bad_arguments_before_touching_the_gpu(lib):
    h = ctypes.c_void_p()
    assert lib.maze_create(ctypes.byref(h), 8, 13, 13, 5, 250, None, 1 << 20) == -2
    assert lib.maze_create(None, 8, 13, 13, 5, 250, 256, 1 << 20) == -2
    assert lib.maze_create(ctypes.byref(h), 8, 13, 13, 5, 0, 256, 1 << 20) == -1     # max_steps
    assert lib.maze_create(ctypes.byref(h), 8, 13, 13, 5, 250, 257, 1 << 20) == -1   # alignment
    assert lib.maze_create(ctypes.byref(h), 8, 13, 13, 5, 250, 256, 16) == -3        # too small
    assert h.value is None
    assert lib.editor_create(ctypes.byref(h), 8, 13, 13, 50, None, 1 << 20) == -2
    assert lib.editor_create(ctypes.byref(h), 8, 13, 13, -1, 256, 1 << 20) == -1
    assert lib.editor_create(ctypes.byref(h), 8, 13, 13, 50, 256, 16) == -3
    assert lib.maze_destroy(None) == -2 and lib.editor_destroy(None) == -2
    assert lib.maze_step(None, None, 1, None, None, None, None) == -2
    assert lib.compute_gae(None, None, None, 1, 1, 0.9, 0.9, None, None, None) == -2
    assert lib.compute_gae(256, 256, 256, 0, 1, 0.9, 0.9, 256, None, None) == -1


def test_level_tools_reject_bad_arguments_before_touching_the_gpu(lib):
    u64 = ctypes.c_uint64
    assert lib.maze_level_metrics(None, 256, 256, None) == -2
    assert lib.maze_set_obs_mode(None, 0, 0) == -2
    assert lib.editor_set_levels(None, 256, 256, 256, 256, None) == -2
    assert lib.editor_random_levels(None, u64(1), u64(0), None) == -2
    assert lib.editor_mutate_levels(None, u64(1), u64(0), 3, None) == -2
    assert lib.replay_scores(None, 256, 256, 256, 4, 4, 0.99, None, 256, 256, 256, None) == -2
    assert lib.replay_scores(256, 256, 256, 256, 0, 4, 0.99, None, 256, 256, 256, None) == -1
    assert lib.replay_distribution(None, 256, 8, 0, 1, 0.3, 0.3, 256, None) == -2
    assert lib.replay_distribution(256, 256, 0, 0, 1, 0.3, 0.3, 256, None) == -1       # K
    assert lib.replay_distribution(256, 256, 8, 0, 1, 0.0, 0.3, 256, None) == -1       # temperature
    assert lib.replay_distribution(256, 256, 8, 0, 1, 0.3, 1.5, 256, None) == -1       # staleness
    assert lib.replay_distribution(256, 256, 1 << 20, 0, 1, 0.3, 0.3, 256, None) == -3  # K too large


def test_rollout_plan_and_the_lds_error_path(lib):
    """Which workgroup size a rollout takes, from the device's unit count and LDS size; a device
    whose LDS cannot hold 32 envs gets MAZE_EHIP (what maze_step then returns), never a
    silent switch to the slow kernel."""
    epw, lds = ctypes.c_int(-1), ctypes.c_size_t(0)

    def plan(N, H, W, k, enc=0, occ=0, cus=256, per_cu=160 * 1024):
        rc = lib.maze_rollout_plan(N, H, W, k, enc, occ, cus, per_cu, ctypes.byref(epw), ctypes.byref(lds))
        return rc, epw.value, lds.value

    # the benchmark configurations on a 256-unit device with 160 KB per unit
    rc, e, b = plan(32768, 13, 13, 5)
    assert (rc, e) == (0, 128) and 100 * 1024 < b <= 159 * 1024
    assert plan(32768, 13, 13, 5, enc=1)[:2] == (0, 128)
    # the occluded view alone: 32 envs per workgroup (two records waves); with typed bytes: 64
    assert plan(32768, 13, 13, 5, occ=1)[:2] == (0, 32)
    assert plan(32768, 13, 13, 5, enc=1, occ=1)[:2] == (0, 64)
    assert plan(16384, 13, 13, 5)[:2] == (0, 64)
    assert plan(8192, 13, 13, 5)[:2] == (0, 32)
    # a batch that would leave compute units idle with 32 envs per workgroup takes 16
    assert plan(4096, 13, 13, 5)[:2] == (0, 16)
    assert plan(4097, 13, 13, 5)[:2] == (0, 32)
    assert plan(32, 13, 13, 5)[:2] == (0, 16)
    assert plan(15, 13, 13, 5)[:2] == (0, 32)
    assert plan(8192, 51, 51, 7)[:2] == (0, 32)
    # fewer units: large workgroups from smaller batches on
    assert plan(8192, 13, 13, 5, cus=64)[:2] == (0, 128)
    # the same shapes with the 64 KB of an older part: smaller workgroups, still the fast kernel
    rc, e, b = plan(32768, 13, 13, 5, per_cu=64 * 1024)
    assert rc == 0 and e < 128 and b <= 63 * 1024
    # the largest grids with view 7 and both variants on need 128 KB for 32 envs
    rc, e, b = plan(8192, 52, 52, 7, enc=1, occ=1)
    assert (rc, e) == (0, 32) and 120 * 1024 < b <= 129 * 1024
    rc, e, b = plan(64, 52, 52, 7, enc=1, occ=1)
    assert (rc, e) == (0, 16) and b < 100 * 1024
    assert plan(64, 52, 52, 7, enc=1, occ=1, per_cu=64 * 1024)[0] == -4      # MAZE_EHIP
    assert plan(8192, 51, 51, 7, per_cu=64 * 1024)[0] == -4
    # view sizes the store-layout kernels do not take: no error, no workgroup size
    assert plan(64, 13, 13, 9)[:2] == (0, 0)
    # argument errors
    assert plan(64, 13, 13, 4)[0] == -1 and plan(64, 13, 13, 5, enc=2)[0] == -1
    assert plan(64, 13, 13, 5, cus=0)[0] == -1 and plan(64, 60, 60, 7)[0] == -3
    assert lib.maze_rollout_plan(64, 13, 13, 5, 0, 0, 256, 160 * 1024, None, ctypes.byref(lds)) == -2


def test_strerror_names_every_code(lib):
    seen = {lib.maze_strerror(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and all(s for s in seen)
    assert b"unknown" in lib.maze_strerror(-99)


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2311_12716_amd import binding
    with pytest.raises(binding.MazeError):
        binding.compute_gae(torch.zeros(4, 2), torch.zeros(5, 2), torch.zeros(4, 2, dtype=torch.uint8),
                            0.99, 0.95)
