"""The library's calls inside a captured HIP graph: they take the stream they are given,
allocate nothing and clear nothing with memset, so a policy loop can capture them.  Every
replay is checked against the oracle, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_12716_amd import binding, workloads as wl
from parity_util import DEV, cpu_student, gpu_student, note, to_gpu

pytestmark = pytest.mark.gpu


def test_replayed_step_and_rollout_match_the_oracle():
    w = wl.student_random("graph", 71, N=4096, T=40, n_walls=40, max_steps=30)
    env, o = gpu_student(w), cpu_student(w)
    acts = to_gpu(w.actions)
    N, k = w.N, w.view
    a1 = torch.zeros((1, N), dtype=torch.int8, device=DEV)
    r1 = torch.empty((1, N), dtype=torch.float32, device=DEV)
    d1 = torch.empty((1, N), dtype=torch.uint8, device=DEV)
    o1 = torch.empty((1, N, k, k, 3), dtype=torch.int8, device=DEV)
    a8 = torch.zeros((8, N), dtype=torch.int8, device=DEV)
    r8 = torch.empty((8, N), dtype=torch.float32, device=DEV)
    d8 = torch.empty((8, N), dtype=torch.uint8, device=DEV)
    o8 = torch.empty((8, N, k, k, 3), dtype=torch.int8, device=DEV)
    v8 = to_gpu(np.random.default_rng(0).random((9, N), dtype=np.float32))
    adv = torch.empty((8, N), dtype=torch.float32, device=DEV)
    nwalls = torch.empty((N,), dtype=torch.int32, device=DEV)
    plen = torch.empty((N,), dtype=torch.int32, device=DEV)

    # eager warm-up on a side stream, as capture requires (also sets the kernels' LDS limits)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        env.step(a1, r1, d1, o1)
        env.step(a8, r8, d8, o8)
        binding.compute_gae(r8, v8, d8, 0.995, 0.98, adv, None, want_returns=False)
        env.level_metrics(nwalls, plen)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    env.reset_to_levels(to_gpu(w.walls), to_gpu(w.agent_xy), to_gpu(w.agent_dir), to_gpu(w.goal_xy))

    g1, g8 = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g1):
        env.step(a1, r1, d1, o1)
    with torch.cuda.graph(g8):
        env.step(a8, r8, d8, o8)
        binding.compute_gae(r8, v8, d8, 0.995, 0.98, adv, None, want_returns=False)
        env.level_metrics(nwalls, plen)
    # capture only records: the env has not moved
    env.reset_to_levels(to_gpu(w.walls), to_gpu(w.agent_xy), to_gpu(w.agent_dir), to_gpu(w.goal_xy))

    onw, opl = oracle.level_metrics(w.walls, w.agent_xy, w.goal_xy)
    t = 0
    for rep in range(4):
        note(f"graph replay {rep}")
        a1.copy_(acts[t:t + 1])
        g1.replay()
        torch.cuda.synchronize()
        orr, od, oo = o.step(w.actions[t:t + 1], 1)
        assert (o1.cpu().numpy() == oo).all() and (d1.cpu().numpy() == od).all()
        assert np.abs(r1.cpu().numpy() - orr).max() <= 1e-6
        t += 1
        scratch = torch.rand((1 << 20,), device=DEV).sum().item()        # unrelated eager work
        a8.copy_(acts[t:t + 8])
        g8.replay()
        torch.cuda.synchronize()
        orr, od, oo = o.step(w.actions[t:t + 8], 8)
        assert (o8.cpu().numpy() == oo).all() and (d8.cpu().numpy() == od).all()
        assert np.abs(r8.cpu().numpy() - orr).max() <= 1e-6
        oadv, _ = oracle.compute_gae(orr, v8.cpu().numpy(), od, 0.995, 0.98)
        assert np.abs(adv.cpu().numpy() - oadv).max() <= 1e-6
        assert (nwalls.cpu().numpy() == onw).all() and (plen.cpu().numpy() == opl).all()
        t += 8
        assert scratch > 0


def test_replayed_pass_of_the_throughput_configuration():
    """Reset to levels + first render + the 256-step rollout of config 3 -- the launch whose store
    waves keep a clock schedule -- captured once and replayed; every replay against the oracle."""
    w = wl.config(3)
    env = gpu_student(w)
    lv = (to_gpu(w.walls), to_gpu(w.agent_xy), to_gpu(w.agent_dir), to_gpu(w.goal_xy))
    acts = to_gpu(w.actions)
    N, T, k = w.N, w.T, w.view
    obs0 = torch.empty((N, k, k, 3), dtype=torch.int8, device=DEV)
    r = torch.empty((T, N), dtype=torch.float32, device=DEV)
    d = torch.empty((T, N), dtype=torch.uint8, device=DEV)
    obs = torch.empty((T, N, k, k, 3), dtype=torch.int8, device=DEV)

    def one_pass():
        env.reset_to_levels(*lv)
        env.render_obs(obs0)
        env.step(acts, r, d, obs)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_pass()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_pass()
    o = cpu_student(w)
    want_obs0 = o.render_obs()
    orr, od, oobs = o.step(w.actions, T)
    for rep in range(3):
        note(f"pass replay {rep}")
        obs.zero_()
        r.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        assert (obs0.cpu().numpy() == want_obs0).all()
        assert (d.cpu().numpy() == od).all() and np.abs(r.cpu().numpy() - orr).max() <= 1e-6
        assert (obs.cpu().numpy() == oobs).all()
        assert torch.rand((1 << 20,), device=DEV).sum().item() > 0       # unrelated eager work
