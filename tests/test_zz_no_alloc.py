"""The allocation-free multi-tensor Adam step (q8_multi_adam8bit_step_noalloc) against the
plan-based entry point it is a variant of: same lists, separate buffers, every output bit for
bit (codes, block maxima, 32-bit states, weights), on two calls in a row, the second with a
smaller list (the static workspace keeps the first call's tables), then a third with the
first list again; and against the CPU oracle on the first list."""
import ctypes as C

import numpy as np
import pytest

import oracle
from paper_2412_01195_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def q8():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2412_01195_amd import q8opt
    q8opt.lib()
    return q8opt


@pytest.fixture(scope="module")
def tabs(q8):
    return (q8.upload_qtable(q8.build_qtable(q8.build_codebook(True))),
            q8.upload_qtable(q8.build_qtable(q8.build_codebook(False))))


def make_list(sizes, B, seed, min_8bit=4096):
    """Two identical device copies of a list (for the two entry points) plus the host original."""
    host, a, b = [], [], []
    for i, n in enumerate(sizes):
        w = synth.uniform_weights(seed, i, n)
        g = synth.normal_grad(seed, i, 1, n, 1e-3)
        nb = oracle.nblocks(n, B)
        if n >= min_8bit:
            st = dict(m_q=np.full(n, 127, np.uint8), r_q=np.zeros(n, np.uint8), N_m=np.zeros(nb, np.float32), N_r=np.zeros(nb, np.float32))
        else:
            st = dict(m_f32=np.zeros(n, np.float32), r_f32=np.zeros(n, np.float32))
        host.append(dict(w=w, g=g, **st))
        for dst in (a, b):
            dst.append({k: torch.from_numpy(v.copy()).cuda() for k, v in host[-1].items()})
    return host, a, b


def same(tag, xs, ys):
    for i, (x, y) in enumerate(zip(xs, ys)):
        for k in x:
            if k == "g":
                continue
            assert torch.equal(x[k].view(torch.uint8), y[k].view(torch.uint8)), "%s: tensor %d, %s differs" % (tag, i, k)


@pytest.mark.parametrize("B", [2048, 256])
def test_noalloc_equals_plan_on_two_calls_in_a_row(q8, tabs, B):
    big = [1, 63, 300, 4096, 4097, 5 * 4096 + 3, 3 * B + 1, 7 * B - 1, 100_003, 1_000_000 + 7, 2048, 33]
    big = big + [1000 + 37 * k for k in range(60)]              # 72 tensors: two chunks of descriptors
    small = [50_001, 7, 4096 * 3]
    lists = {}
    for name, sizes, seed in (("big", big, 11), ("small", small, 12)):
        host, a, b = make_list(sizes, B, seed)
        lists[name] = (host, a, b, q8.Plan(b, B))
    torch.cuda.synchronize()
    t = {"big": 0, "small": 0}
    for name in ("big", "small", "big", "small", "small", "big"):
        host, a, b, plan = lists[name]
        t[name] += 1
        q8.multi_adam8bit_step_noalloc(a, B, tabs[0], tabs[1], **H.ADAM, weight_decay=0.01, t=t[name],
                                       flags=q8.FLAG_DECOUPLED_WD | q8.FLAG_BIAS_CORRECTION)
        plan.multi_adam8bit_step(tabs[0], tabs[1], **H.ADAM, weight_decay=0.01, t=t[name],
                                 flags=q8.FLAG_DECOUPLED_WD | q8.FLAG_BIAS_CORRECTION)
        torch.cuda.synchronize()
        same("%s list, call %d" % (name, t[name]), a, b)
    # and the oracle, on the big list
    host, a, b, plan = lists["big"]
    qs, qu = H.codebooks()
    flags = oracle.FLAG_DECOUPLED_WD | oracle.FLAG_BIAS_CORRECTION
    for step in range(1, t["big"] + 1):
        for h in host:
            if "m_q" in h:
                oracle.adam8bit_step(h["w"], h["g"], h["m_q"], h["r_q"], h["N_m"], h["N_r"], qs, qu, B, **H.ADAM, wd=0.01, t=step, flags=flags)
            else:
                oracle.adam32_step(h["w"], h["g"], h["m_f32"], h["r_f32"], **H.ADAM, wd=0.01, t=step, flags=flags)
    for i, (h, d) in enumerate(zip(host, a)):
        for k in h:
            if k in ("g", "w"):
                continue
            assert np.array_equal(d[k].cpu().numpy().view(np.uint8), h[k].view(np.uint8)), "oracle: tensor %d, %s" % (i, k)
        assert H.rel_err(d["w"].cpu().numpy(), h["w"]) <= H.PARAM_RTOL
    for name in lists:
        lists[name][3].destroy()


def test_noalloc_recorded_by_stream_capture(q8, tabs):
    """The call enqueues kernels only (no allocation, memset or copy), so stream capture can
    record it: a graph holding one call over 50 tensors (two table-fill launches and the step)
    is replayed four times with eager gradient updates in between; after every replay the
    result equals the plan-based entry point run eagerly on a copy."""
    B = 2048
    sizes = [3 * B + 1, 100_003, 33, 4096, 5 * 4096 + 3] + [900 + 41 * k for k in range(45)]
    host, a, b = make_list(sizes, B, 13)
    plan = q8.Plan(b, B)
    hp = dict(H.ADAM, weight_decay=0.01, flags=q8.FLAG_DECOUPLED_WD)
    # eager first calls on a side stream, as torch asks before a capture (they also fill the
    # library's per-device caches: workspace address, occupancy)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        q8.multi_adam8bit_step_noalloc(a, B, tabs[0], tabs[1], **hp)
    torch.cuda.current_stream().wait_stream(s)
    plan.multi_adam8bit_step(tabs[0], tabs[1], **hp)
    torch.cuda.synchronize()
    same("eager call before the capture", a, b)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        q8.multi_adam8bit_step_noalloc(a, B, tabs[0], tabs[1], **hp)
    for rep in range(1, 5):
        for i, (x, y) in enumerate(zip(a, b)):                    # eager work between replays: fresh gradients
            g = torch.from_numpy(synth.normal_grad(13, i, 1 + rep, x["g"].numel(), 1e-3)).cuda()
            x["g"].copy_(g); y["g"].copy_(g)
        graph.replay()
        plan.multi_adam8bit_step(tabs[0], tabs[1], **hp)
        torch.cuda.synchronize()
        same("replay %d" % rep, a, b)
    plan.destroy()


def test_noalloc_limits_and_arguments(q8, tabs):
    L = q8.lib()
    w = torch.zeros(4096, device="cuda"); g = torch.zeros(4096, device="cuda")
    mq = torch.zeros(4096, dtype=torch.uint8, device="cuda"); N = torch.zeros(2, device="cuda")
    one = dict(w=w, g=g, m_q=mq, r_q=mq, N_m=N, N_r=N)
    with pytest.raises(q8.Q8Error) as err:
        q8.multi_adam8bit_step_noalloc([one] * 1025, 2048, tabs[0], tabs[1], **H.ADAM)
    assert err.value.status == q8.ELIMIT
    # more units than the workspace holds: described, never touched (n is only a number here)
    arr = q8._tensor_array([one], "float32", 2048)
    arr[0].n = (1 << 17) * 2048 + 1
    st = L.q8_multi_adam8bit_step_noalloc(arr, 1, 2048, tabs[0].data_ptr(), tabs[1].data_ptr(), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 0, None)
    assert st == q8.ELIMIT
    arr[0].n = 4096
    assert L.q8_multi_adam8bit_step_noalloc(arr, 1, 100, tabs[0].data_ptr(), tabs[1].data_ptr(), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 0, None) == q8.EBLOCK
    assert L.q8_multi_adam8bit_step_noalloc(None, 1, 2048, tabs[0].data_ptr(), tabs[1].data_ptr(), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 0, None) == q8.EINVAL
    assert L.q8_multi_adam8bit_step_noalloc(arr, 1, 2048, tabs[0].data_ptr(), tabs[1].data_ptr(), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 8, None) == q8.EINVAL
    sgd_only = dict(w=w, g=g, m_q=mq, N_m=N)                    # no second state: not usable with Adam
    with pytest.raises(q8.Q8Error) as err:
        q8.multi_adam8bit_step_noalloc([sgd_only], 2048, tabs[0], tabs[1], **H.ADAM)
    assert err.value.status == q8.EINVAL
    torch.cuda.synchronize()
