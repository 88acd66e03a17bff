"""Seeded random sweep over sizes, block sizes, storage types, optimizers, flags and gradient
scales (a fixed list of cases, so every run checks the same ones): stored weights, codes and
absmax must equal the oracle's bit for bit after every step."""
import os

import numpy as np
import pytest

import oracle
from paper_2412_01195_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

BLOCKS = (64, 128, 256, 512, 1024, 2048, 4096)
TORCH_DT = {"f32": "float32", "bf16": "bfloat16", "f16": "float16"}


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


def to_store(x, store):
    if store == "bf16":
        return synth.bf16_bits(x)
    if store == "f16":
        return synth.f16_bits(x)
    return np.ascontiguousarray(x, np.float32)


def to_dev(a, store):
    if store == "f32":
        return torch.from_numpy(a.copy()).cuda()
    return torch.from_numpy(a.view(np.int16).copy()).cuda().view(getattr(torch, TORCH_DT[store]))


def from_dev(t, store):
    if store == "f32":
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def make_grad(rng, n, scale):
    g = rng.standard_normal(n) * scale
    kind = rng.integers(0, 4)
    if kind == 1:
        g[rng.random(n) < 0.3] = 0.0                              # sparse gradient: exact zeros
    elif kind == 2:
        g = np.round(g / scale * 4) / 4 * scale                   # few distinct values: many equal quotients
    elif kind == 3:
        g *= 10.0 ** rng.uniform(-6, 0, n)                        # wide dynamic range inside blocks
    return g.astype(np.float32)


N_CASES = int(os.environ.get("Q8_FUZZ_CASES", "120"))      # a longer hunt: Q8_FUZZ_CASES=5000 pytest ...


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_case(q8, tabs, case):
    rng = np.random.default_rng(9000 + case)
    n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 6000), rng.integers(6000, 40000)]))
    B = int(rng.choice(BLOCKS))
    store = str(rng.choice(["f32", "bf16", "f16"]))
    adam = bool(rng.integers(0, 2))
    wd = float(rng.choice([0.0, 10.0 ** rng.uniform(-5, -1)]))
    flags = int(rng.integers(0, 4)) if adam else 0
    gmax = 3.0 if store == "f16" else 4.0                          # keep binary16 gradients finite
    scale = 10.0 ** rng.uniform(-12, gmax)
    steps = int(rng.integers(1, 5))
    tag = "case %d: n=%d B=%d %s %s wd=%g flags=%d scale=%.2g" % (case, n, B, store, "adam" if adam else "sgd", wd, flags, scale)

    w = to_store((rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 0)).astype(np.float32), store)
    st = H.zero_state(n, B, adam=adam)
    w_d = to_dev(w, store)
    st_d = {k: torch.from_numpy(v.copy()).cuda() for k, v in st.items()}
    hp_a = dict(alpha=float(10.0 ** rng.uniform(-4, -2)), beta1=float(rng.choice([0.9, 0.8, 0.0])),
                beta2=float(rng.choice([0.999, 0.99, 0.9])), eps=float(rng.choice([1e-8, 1e-6, 0.0 if scale > 1e-3 else 1e-8])))
    hp_s = dict(alpha=float(10.0 ** rng.uniform(-3, -1)), beta=float(rng.choice([0.9, 0.5, 0.0])))
    for t in range(1, steps + 1):
        g32 = make_grad(rng, n, scale)
        g = to_store(g32, store)
        if adam and hp_a["eps"] == 0.0:                            # 0/0 is outside the method: no stored zero
            stored_zero = (g32 == 0) if store == "f32" else ((g & 0x7fff) == 0)
            g32[stored_zero] = np.float32(scale)
            g = to_store(g32, store)
        g_d = to_dev(g, store)
        kw = dict(bf16=store == "bf16", f16=store == "f16")
        if adam:
            H.oracle_adam8(w, g, st, B, wd=wd, t=t, flags=flags, hp=hp_a, **kw)
            fn = {"f32": q8.adam8bit_step, "bf16": q8.adam8bit_step_bf16, "f16": q8.adam8bit_step_f16}[store]
            fn(w_d, g_d, st_d["m_q"], st_d["r_q"], st_d["N_m"], st_d["N_r"], tabs[0], tabs[1], B,
               weight_decay=wd, t=t, flags=flags, **hp_a)
        else:
            H.oracle_sgd8(w, g, st, B, wd=wd, hp=hp_s, **kw)
            fn = {"f32": q8.sgd8bit_step, "bf16": q8.sgd8bit_step_bf16, "f16": q8.sgd8bit_step_f16}[store]
            fn(w_d, g_d, st_d["m_q"], st_d["N_m"], tabs[0], B, hp_s["alpha"], hp_s["beta"], weight_decay=wd)
        got = from_dev(w_d, store)
        ref = w.view(got.dtype)
        same = (got == ref)
        if store == "f32":
            same |= (w_d.cpu().numpy() == 0) & (w == 0)            # the sign of an exact zero is not compared
        assert same.all(), "%s step %d: %d weights differ" % (tag, t, int((~same).sum()))
        for k, v in st.items():
            a = st_d[k].cpu().numpy()
            assert np.array_equal(a.view(np.uint8), v.view(np.uint8)), "%s step %d: %s differs" % (tag, t, k)


N_LISTS = int(os.environ.get("Q8_FUZZ_LISTS", "40"))


@pytest.mark.parametrize("case", range(N_LISTS))
def test_random_list(q8, tabs, case):
    """Multi-tensor plans over random lists: empty, tiny and ragged tensors, 8-bit or 32-bit states
    per tensor, any storage type, Adam or SGD; one launch per step, compared tensor by tensor."""
    rng = np.random.default_rng(70000 + case)
    B = int(rng.choice(BLOCKS))
    store = str(rng.choice(["f32", "bf16", "f16"]))
    adam = bool(rng.integers(0, 2))
    wd = float(rng.choice([0.0, 10.0 ** rng.uniform(-4, -1)]))
    flags = int(rng.integers(0, 4)) if adam else 0
    hp_a = dict(alpha=float(10.0 ** rng.uniform(-4, -2)), beta1=0.9, beta2=float(rng.choice([0.999, 0.99])), eps=1e-8)
    hp_s = dict(alpha=float(10.0 ** rng.uniform(-3, -1)), beta=0.9)
    count = int(rng.integers(1, 14))
    sizes = [int(rng.choice([0, rng.integers(1, 50), rng.integers(50, 3000), rng.integers(3000, 20000)])) for _ in range(count)]
    if sum(sizes) == 0:
        sizes[0] = 77
    kw = dict(bf16=store == "bf16", f16=store == "f16")
    tdt = getattr(torch, TORCH_DT[store])
    tens, refs = [], []
    for n in sizes:
        small = bool(rng.integers(0, 2)) and n > 0
        w = to_store((rng.standard_normal(n) * 0.1).astype(np.float32), store)
        ref = dict(w=w, n=n, small=small, scale=10.0 ** rng.uniform(-8, 1))
        d = dict(w=to_dev(w, store) if n else torch.empty(0, dtype=tdt, device="cuda"),
                 g=torch.zeros(n, dtype=tdt, device="cuda"))
        if small:
            ref["m"] = np.zeros(n, np.float32); ref["r"] = np.zeros(n, np.float32)
            d["m_f32"] = torch.zeros(n, device="cuda")
            if adam:
                d["r_f32"] = torch.zeros(n, device="cuda")
        else:
            ref["st"] = H.zero_state(n, B, adam=adam)
            d.update({k: torch.from_numpy(v.copy()).cuda() for k, v in ref["st"].items()})
        tens.append(d); refs.append(ref)
    plan = q8.Plan(tens, B, wg_dtype=TORCH_DT[store])
    widen = {"f32": lambda a: a, "bf16": lambda a: (a.astype(np.uint32) << 16).view(np.float32),
             "f16": lambda a: a.view(np.float16).astype(np.float32)}[store]
    narrow = {"bf16": oracle.f32_to_bf16, "f16": oracle.f32_to_f16}.get(store)
    try:
        for t in range(1, 4):
            for d, ref in zip(tens, refs):
                n = ref["n"]
                if n == 0:
                    continue
                g = to_store(make_grad(rng, n, ref["scale"]), store)
                d["g"].copy_(to_dev(g, store))
                if ref["small"]:
                    w32, g32 = widen(ref["w"]), widen(g)
                    if store != "f32":
                        w32 = w32.copy()
                    if adam:
                        oracle.adam32_step(w32, g32, ref["m"], ref["r"], hp_a["alpha"], hp_a["beta1"], hp_a["beta2"],
                                           hp_a["eps"], wd, t, flags)
                    else:
                        oracle.sgd32_step(w32, g32, ref["m"], hp_s["alpha"], hp_s["beta"], wd)
                    if store != "f32":
                        ref["w"][:] = np.array([narrow(v) for v in w32], np.uint16)
                elif adam:
                    H.oracle_adam8(ref["w"], g, ref["st"], B, wd=wd, t=t, flags=flags, hp=hp_a, **kw)
                else:
                    H.oracle_sgd8(ref["w"], g, ref["st"], B, wd=wd, hp=hp_s, **kw)
            if adam:
                plan.multi_adam8bit_step(tabs[0], tabs[1], weight_decay=wd, t=t, flags=flags, **hp_a)
            else:
                plan.multi_sgd8bit_step(tabs[0], hp_s["alpha"], hp_s["beta"], weight_decay=wd)
            for i, (d, ref) in enumerate(zip(tens, refs)):
                if ref["n"] == 0:
                    continue
                tag = "list %d tensor %d (n=%d, %s, B=%d) step %d" % (case, i, ref["n"], store, B, t)
                got = from_dev(d["w"], store)
                want = ref["w"].view(got.dtype)
                same = got == want
                if store == "f32":
                    same |= (d["w"].cpu().numpy() == 0) & (ref["w"] == 0)
                assert same.all(), tag
                if ref["small"]:
                    assert np.array_equal(d["m_f32"].cpu().numpy().view(np.uint32), ref["m"].view(np.uint32)), tag
                    if adam:
                        assert np.array_equal(d["r_f32"].cpu().numpy().view(np.uint32), ref["r"].view(np.uint32)), tag
                else:
                    for k, v in ref["st"].items():
                        assert np.array_equal(d[k].cpu().numpy().view(np.uint8), v.view(np.uint8)), (tag, k)
    finally:
        plan.destroy()


@pytest.mark.parametrize("kind", ["linear", "cubic", "jittered-tree"])
def test_other_codebooks(q8, kind):
    """The kernels search whatever strictly increasing codebook the table was built from (nothing
    about the dynamic-tree values is compiled in): quantize, dequantize and an Adam step with
    other signed / unsigned maps equal the oracle run with the same maps."""
    rng = np.random.default_rng(5)
    j = np.arange(256, dtype=np.float64)
    if kind == "linear":
        qs = ((j - 127.0) / 128.0); qs[255] = 1.0
        qu = j / 255.0
    elif kind == "cubic":
        x = (j - 127.0) / 128.0; x[255] = 1.0
        qs = np.sign(x) * np.abs(x) ** 3
        qu = (j / 255.0) ** 3
    else:
        qs0, qu0 = H.codebooks()
        def jitter(q):
            q = q.astype(np.float64).copy()
            gap = np.diff(q)
            step = rng.uniform(-0.2, 0.2, 254) * np.minimum(gap[:-1], gap[1:])
            step[q[1:-1] == 0] = 0.0                     # the map keeps its exact 0.0
            q[1:-1] += step
            return q
        qs, qu = jitter(qs0), jitter(qu0)
    qs, qu = qs.astype(np.float32), qu.astype(np.float32)
    assert np.all(np.diff(qs) > 0) and np.all(np.diff(qu) > 0)
    ts = q8.upload_qtable(q8.build_qtable(qs)); tu = q8.upload_qtable(q8.build_qtable(qu))
    n, B = 50000 + 37, 256
    T = (rng.standard_normal(n) * 10.0 ** rng.uniform(-4, 1, n)).astype(np.float32)
    for q, tab, x in ((qs, ts, T), (qu, tu, np.abs(T))):
        TQ_ref, N_ref = oracle.quantize_blockwise(q, x, B)
        TQ = torch.empty(n, dtype=torch.uint8, device="cuda"); N = torch.empty(oracle.nblocks(n, B), device="cuda")
        q8.quantize_blockwise(tab, torch.from_numpy(x).cuda(), B, TQ, N)
        assert np.array_equal(TQ.cpu().numpy(), TQ_ref) and np.array_equal(N.cpu().numpy().view(np.uint32), N_ref.view(np.uint32))
        TD = torch.empty(n, device="cuda")
        q8.dequantize_blockwise(tab, TQ, N, B, TD)
        assert np.array_equal(TD.cpu().numpy().view(np.uint32), oracle.dequantize_blockwise(q, TQ_ref, N_ref, B).view(np.uint32))
    # Adam with these maps: zero codes are those of 0.0 in each map
    zs, zu = int(np.flatnonzero(qs == 0)[0]), int(np.flatnonzero(qu == 0)[0])
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    st = dict(m_q=np.full(n, zs, np.uint8), r_q=np.full(n, zu, np.uint8),
              N_m=np.zeros(oracle.nblocks(n, B), np.float32), N_r=np.zeros(oracle.nblocks(n, B), np.float32))
    w_d = torch.from_numpy(w.copy()).cuda(); st_d = {k: torch.from_numpy(v.copy()).cuda() for k, v in st.items()}
    for t in range(1, 4):
        g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
        oracle.adam8bit_step(w, g, st["m_q"], st["r_q"], st["N_m"], st["N_r"], qs, qu, B, wd=1e-3, t=t, **H.ADAM)
        q8.adam8bit_step(w_d, torch.from_numpy(g).cuda(), st_d["m_q"], st_d["r_q"], st_d["N_m"], st_d["N_r"], ts, tu, B,
                         weight_decay=1e-3, t=t, **H.ADAM)
        assert np.array_equal(w_d.cpu().numpy().view(np.uint32), w.view(np.uint32)), (kind, t)
        for k, v in st.items():
            assert np.array_equal(st_d[k].cpu().numpy().view(np.uint8), v.view(np.uint8)), (kind, t, k)
