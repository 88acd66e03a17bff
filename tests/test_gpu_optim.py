"""torch.optim front ends (Adam8bit, SGD8bit) on a small network: after every step the
parameters and the optimizer states equal what the CPU oracle computes tensor by tensor from
the same gradients -- bit for bit -- including across a state_dict round trip."""
import copy

import numpy as np
import pytest

import oracle
from tests import harness as H

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def optim():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2412_01195_amd import optim, q8opt
    q8opt.lib()
    return optim


def make_model(dtype):
    torch.manual_seed(3)
    m = torch.nn.Sequential(torch.nn.Linear(64, 300), torch.nn.Tanh(), torch.nn.Linear(300, 40),
                            torch.nn.Tanh(), torch.nn.Linear(40, 130))
    return m.cuda().to(dtype)


def bits(t):
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16).ravel()
    return t.detach().cpu().numpy().ravel()


class Ref:
    """Per-tensor oracle state mirroring the optimizer's choices (8-bit from min8 elements on)."""

    def __init__(self, model, B, adam, min8, store):
        self.B, self.adam, self.store = B, adam, store          # store: "f32", "bf16" or "f16"
        self.bf16, self.f16 = store == "bf16", store == "f16"
        self.t = []
        for p in model.parameters():
            n = p.numel()
            e = dict(w=bits(p).copy(), n=n, small=n < min8)
            if e["small"]:
                e["m"] = np.zeros(n, np.float32); e["r"] = np.zeros(n, np.float32)
            else:
                e["st"] = H.zero_state(n, B, adam=adam)
            self.t.append(e)

    def step(self, grads, t, hp):
        for e, g in zip(self.t, grads):
            if e["small"]:
                w32, g32 = self.widen(e["w"]), self.widen(g)
                if self.adam:
                    oracle.adam32_step(w32, g32, e["m"], e["r"], hp["alpha"], hp["beta1"], hp["beta2"], hp["eps"],
                                       hp["wd"], t, hp["flags"])
                else:
                    oracle.sgd32_step(w32, g32, e["m"], hp["alpha"], hp["beta"], hp["wd"])
                if self.store != "f32":
                    narrow = oracle.f32_to_bf16 if self.bf16 else oracle.f32_to_f16
                    e["w"][:] = np.array([narrow(v) for v in w32], np.uint16)
            elif self.adam:
                H.oracle_adam8(e["w"], g, e["st"], self.B, wd=hp["wd"], t=t, flags=hp["flags"],
                               hp=dict(alpha=hp["alpha"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["eps"]),
                               bf16=self.bf16, f16=self.f16)
            else:
                H.oracle_sgd8(e["w"], g, e["st"], self.B, wd=hp["wd"], hp=dict(alpha=hp["alpha"], beta=hp["beta"]),
                              bf16=self.bf16, f16=self.f16)

    def widen(self, a):
        if self.bf16:
            return (a.astype(np.uint32) << 16).view(np.float32)
        if self.f16:
            return a.view(np.float16).astype(np.float32)
        return a

    def check(self, model, opt, tag):
        for i, (e, p) in enumerate(zip(self.t, model.parameters())):
            got = bits(p)
            u = np.uint32 if self.store == "f32" else np.uint16
            same = got.view(u) == e["w"].view(u)
            assert same.all(), "%s tensor %d: %d weights differ" % (tag, i, int((~same).sum()))
            st = opt.state[p]
            if e["small"]:
                assert np.array_equal(st["m_f32"].cpu().numpy().view(np.uint32), e["m"].view(np.uint32)), (tag, i)
                if self.adam:
                    assert np.array_equal(st["r_f32"].cpu().numpy().view(np.uint32), e["r"].view(np.uint32)), (tag, i)
            else:
                for k, v in e["st"].items():
                    a = st[k].cpu().numpy()
                    assert a.dtype == v.dtype, (tag, i, k, a.dtype)
                    assert np.array_equal(a.view(np.uint8), v.view(np.uint8)), (tag, i, k)


def train_step(model, opt, x):
    opt.zero_grad(set_to_none=True)
    loss = model(x).float().pow(2).mean()
    loss.backward()
    grads = [bits(p.grad).copy() for p in model.parameters()]
    opt.step()
    return grads


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16], ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("kind", ["adam", "adamw", "sgd"])
def test_optimizer_matches_oracle_and_survives_checkpoint(optim, dtype, kind):
    B, min8 = 256, 4096
    store = {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}[dtype]
    model = make_model(dtype)
    if kind == "sgd":
        opt = optim.SGD8bit(model.parameters(), lr=0.05, momentum=0.9, weight_decay=1e-4, block_size=B, min_8bit_size=min8)
        hp = dict(alpha=0.05, beta=0.9, wd=1e-4)
    elif kind == "adam":
        opt = optim.Adam8bit(model.parameters(), lr=1e-3, block_size=B, min_8bit_size=min8)
        hp = dict(alpha=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0, flags=0)
    else:
        opt = optim.Adam8bit(model.parameters(), lr=1e-3, weight_decay=0.05, bias_correction=True,
                             decoupled_weight_decay=True, block_size=B, min_8bit_size=min8)
        hp = dict(alpha=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.05,
                  flags=oracle.FLAG_BIAS_CORRECTION | oracle.FLAG_DECOUPLED_WD)
    ref = Ref(model, B, kind != "sgd", min8, store)
    gen = torch.Generator(device="cuda"); gen.manual_seed(11)
    for t in range(1, 5):
        x = torch.randn(32, 64, device="cuda", generator=gen).to(dtype)
        grads = train_step(model, opt, x)
        ref.step(grads, t, hp)
        ref.check(model, opt, "%s step %d" % (kind, t))

    # checkpoint: a fresh model + optimizer resumed from the state dicts continues identically
    model2 = make_model(dtype)
    model2.load_state_dict(copy.deepcopy(model.state_dict()))
    opt2 = type(opt)(model2.parameters(), **{k: v for k, v in opt.defaults.items() if k != "step"})
    opt2.load_state_dict(copy.deepcopy(opt.state_dict()))
    for p in model2.parameters():
        for k, v in opt2.state[p].items():
            assert v.dtype == (torch.uint8 if k in ("m_q", "r_q") else torch.float32), (k, v.dtype)
    for t in range(5, 7):
        x = torch.randn(32, 64, device="cuda", generator=gen).to(dtype)
        grads = train_step(model, opt, x)
        grads2 = train_step(model2, opt2, x)
        for a, b in zip(grads, grads2):
            assert np.array_equal(a, b)
        ref.step(grads, t, hp)
        ref.check(model, opt, "%s step %d" % (kind, t))
        ref.check(model2, opt2, "%s resumed step %d" % (kind, t))


def test_optimizer_rejects_what_it_cannot_run(optim):
    p = torch.nn.Parameter(torch.zeros(100, dtype=torch.float64, device="cuda"))
    opt = optim.Adam8bit([p])
    p.grad = torch.zeros_like(p)
    with pytest.raises(RuntimeError):
        opt.step()
    with pytest.raises(ValueError):
        optim.Adam8bit([torch.nn.Parameter(torch.zeros(8, device="cuda"))], block_size=100)
