"""GPU parity on the five benchmark configurations.

Small configurations (1-3 and a reduced 5) are compared element by element after every
step with host-generated inputs.  The full-size configurations 4 (10^9 parameters) and 5
(64 x 1 562 500, B = 256, heavy-tailed gradients) use device-generated seeded inputs and are
compared with the oracle over EVERY entry after EVERY step (the oracle's block ranges run on
all host threads), with the mismatch count reported; a quicker tier follows a sample of
blocks (blocks are independent, so a block's trajectory needs only its own weights,
gradients and state)."""
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


class FlatList:
    """A list of tensors carved out of flat host/device buffers (every tensor starts on a
    256-byte boundary), with 8-bit or 32-bit optimizer state per tensor."""

    def __init__(self, sizes, B, adam, min_8bit=0):
        self.sizes, self.B, self.adam = list(sizes), B, adam
        self.off, self.boff, self.is8 = [], [], []
        o = bo = 0
        for n in self.sizes:
            self.off.append(o); self.boff.append(bo)
            self.is8.append(n >= min_8bit)
            o += -(-n // 64) * 64
            bo += -(-oracle.nblocks(n, B) // 64) * 64
        self.total, self.btotal = o, bo
        z = lambda dt, k=self.total: np.zeros(k, dt)
        self.h = dict(w=z(np.float32), g=z(np.float32), m_q=np.full(self.total, 127, np.uint8), r_q=z(np.uint8),
                      N_m=z(np.float32, self.btotal), N_r=z(np.float32, self.btotal),
                      m_f32=z(np.float32), r_f32=z(np.float32))
        self.d = None

    def view(self, arrs, i, key):
        n = self.sizes[i]
        if key in ("N_m", "N_r"):
            return arrs[key][self.boff[i]: self.boff[i] + oracle.nblocks(n, self.B)]
        return arrs[key][self.off[i]: self.off[i] + n]

    def upload(self):
        self.d = {k: torch.from_numpy(v).cuda() for k, v in self.h.items()}

    def plan(self, q8):
        ts = []
        for i in range(len(self.sizes)):
            t = dict(w=self.view(self.d, i, "w"), g=self.view(self.d, i, "g"))
            if self.is8[i]:
                t.update(m_q=self.view(self.d, i, "m_q"), N_m=self.view(self.d, i, "N_m"))
                if self.adam:
                    t.update(r_q=self.view(self.d, i, "r_q"), N_r=self.view(self.d, i, "N_r"))
            else:
                t.update(m_f32=self.view(self.d, i, "m_f32"))
                if self.adam:
                    t.update(r_f32=self.view(self.d, i, "r_f32"))
            ts.append(t)
        return q8.Plan(ts, self.B)

    def oracle_step(self, t, wd=0.0, flags=0):
        qs, qu = H.codebooks()
        B = self.B

        def one(i):
            v = lambda k: self.view(self.h, i, k)
            if self.adam and self.is8[i]:
                oracle.adam8bit_step(v("w"), v("g"), v("m_q"), v("r_q"), v("N_m"), v("N_r"), qs, qu, B,
                                     H.ADAM["alpha"], H.ADAM["beta1"], H.ADAM["beta2"], H.ADAM["eps"], wd, t, flags)
            elif self.adam:
                oracle.adam32_step(v("w"), v("g"), v("m_f32"), v("r_f32"), H.ADAM["alpha"], H.ADAM["beta1"],
                                   H.ADAM["beta2"], H.ADAM["eps"], wd, t, flags)
            elif self.is8[i]:
                oracle.sgd8bit_step(v("w"), v("g"), v("m_q"), v("N_m"), qs, B, H.SGD["alpha"], H.SGD["beta"], wd)
            else:
                oracle.sgd32_step(v("w"), v("g"), v("m_f32"), H.SGD["alpha"], H.SGD["beta"], wd)
        list(H.pool().map(one, range(len(self.sizes))))

    def compare(self, tag):
        worst = 0.0
        keys = ["m_q", "N_m", "m_f32"] + (["r_q", "N_r", "r_f32"] if self.adam else [])
        for k in keys:
            a, b = self.d[k].cpu().numpy(), self.h[k]
            if a.dtype == np.float32:
                a, b = a.view(np.uint32), b.view(np.uint32)
            if not np.array_equal(a, b):
                bad = np.flatnonzero(a != b)
                raise AssertionError("%s: %s differs at %d entries, first flat index %d" % (tag, k, bad.size, bad[0]))
        worst = H.rel_err(self.d["w"].cpu().numpy(), self.h["w"])
        assert worst <= H.PARAM_RTOL, "%s: parameter relative error %.3g" % (tag, worst)
        return worst


def test_config2_sgd_resnet34_list(q8, tabs):
    """Config 2: 8-bit SGD (momentum 0.9, lr 0.1, wd 1e-4), B = 2048, ResNet34-shaped list
    (111 tensors, 8 168 800 parameters, all with 8-bit state), 20 steps."""
    specs = synth.resnet34_specs()
    assert len(specs) == 111 and sum(s.numel for s in specs) == 8168800
    L = FlatList([s.numel for s in specs], 2048, adam=False)
    for i, s in enumerate(specs):
        L.view(L.h, i, "w")[:] = synth.uniform_weights(2, i, s.numel)
    L.upload()
    plan = L.plan(q8)
    for t in range(1, 21):
        for i, s in enumerate(specs):
            L.view(L.h, i, "g")[:] = synth.normal_grad(2, i, t, s.numel, synth.fan_in_std(s, 1e-2))
        L.d["g"].copy_(torch.from_numpy(L.h["g"]))
        plan.multi_sgd8bit_step(tabs[0], **H.SGD, weight_decay=1e-4)
        L.oracle_step(t, wd=1e-4)
        L.compare("config 2 step %d" % t)
    plan.destroy()


def test_config3_adam_resnet293_list(q8, tabs):
    """Config 3: 8-bit Adam, B = 2048, ResNet293-shaped list (891 tensors, 30 160 480
    parameters); tensors under 4096 elements keep 32-bit states; 20 steps."""
    specs = synth.resnet293_specs()
    assert len(specs) == 891 and sum(s.numel for s in specs) == 30160480
    L = FlatList([s.numel for s in specs], 2048, adam=True, min_8bit=4096)
    assert sum(L.is8) == 296
    for i, s in enumerate(specs):
        L.view(L.h, i, "w")[:] = synth.uniform_weights(3, i, s.numel)
    L.upload()
    plan = L.plan(q8)
    for t in range(1, 21):
        for i, s in enumerate(specs):
            L.view(L.h, i, "g")[:] = synth.normal_grad(3, i, t, s.numel, 1e-3)
        L.d["g"].copy_(torch.from_numpy(L.h["g"]))
        plan.multi_adam8bit_step(tabs[0], tabs[1], **H.ADAM, t=t)
        L.oracle_step(t)
        L.compare("config 3 step %d" % t)
    plan.destroy()


def test_config5_reduced_heavy_tail(q8, tabs):
    """Config 5 at 1/100 size: 64 tensors x 15 625 parameters, B = 256 (61 blocks + a tail of
    9), Student-t gradients with per-tensor scales 1e-6..1e-1 and 1 % outliers, 50 steps."""
    sizes = [15625] * 64
    L = FlatList(sizes, 256, adam=True)
    scales = [synth.heavy_tail_scale(5, i) for i in range(64)]
    assert min(scales) < 1e-4 and max(scales) > 1e-3
    for i, n in enumerate(sizes):
        L.view(L.h, i, "w")[:] = synth.uniform_weights(5, i, n)
    L.upload()
    plan = L.plan(q8)
    for t in range(1, 51):
        for i, n in enumerate(sizes):
            L.view(L.h, i, "g")[:] = synth.heavy_tail_grad(5, i, t, n, scales[i], 256)
        L.d["g"].copy_(torch.from_numpy(L.h["g"]))
        plan.multi_adam8bit_step(tabs[0], tabs[1], **H.ADAM, t=t)
        L.oracle_step(t)
        L.compare("config 5 (reduced) step %d" % t)
    plan.destroy()


def test_dfresnet_adamw_list(q8, tabs):
    """Second architecture family of the paper (Sec. III-C, V): a DF-ResNet-shaped list in its
    deepest reversible form (638 tensors, 14.1 M parameters, many depth-wise 3x3 and 1x1
    tensors), trained as in the paper with AdamW (decoupled weight decay 0.05), here with the
    bias-correction extension as well; tensors under 4096 elements keep 32-bit states."""
    specs = synth.df_resnet_specs()
    assert len(specs) == 638 and sum(s.numel for s in specs) == 14060656
    small = synth.df_resnet_specs((2, 2, 4, 2))
    assert sum(s.numel for s in small[:-1]) == 4801840          # the 4.8 M of the DF-RevNet66 table
    L = FlatList([s.numel for s in specs], 2048, adam=True, min_8bit=4096)
    for i, s in enumerate(specs):
        L.view(L.h, i, "w")[:] = synth.uniform_weights(7, i, s.numel)
    L.upload()
    plan = L.plan(q8)
    flags = q8.FLAG_DECOUPLED_WD | q8.FLAG_BIAS_CORRECTION
    for t in range(1, 11):
        for i, s in enumerate(specs):
            L.view(L.h, i, "g")[:] = synth.normal_grad(7, i, t, s.numel, synth.fan_in_std(s, 1e-2))
        L.d["g"].copy_(torch.from_numpy(L.h["g"]))
        plan.multi_adam8bit_step(tabs[0], tabs[1], **H.ADAM, weight_decay=0.05, t=t, flags=flags)
        L.oracle_step(t, wd=0.05, flags=flags)
        L.compare("DF-ResNet list step %d" % t)
    plan.destroy()


@pytest.mark.parametrize("B", [64, 128, 256, 512, 1024, 2048, 4096])
def test_block_size_sweep_mixed_list(q8, tabs, B):
    """Every supported block size on a small list whose tensors start and end inside jobs,
    units and blocks (sizes around multiples of 1024 and of B)."""
    sizes = [1, 63, 1023, 1024, 1025, 4096, 4097, 5 * 4096 + 3, 3 * B, 3 * B + 1, 7 * B - 1, 100_003]
    L = FlatList(sizes, B, adam=True)
    for i, n in enumerate(sizes):
        L.view(L.h, i, "w")[:] = synth.uniform_weights(8, i, n)
    L.upload()
    plan = L.plan(q8)
    for t in range(1, 5):
        for i, n in enumerate(sizes):
            L.view(L.h, i, "g")[:] = synth.normal_grad(8, i, t, n, 1e-3)
        L.d["g"].copy_(torch.from_numpy(L.h["g"]))
        plan.multi_adam8bit_step(tabs[0], tabs[1], **H.ADAM, t=t)
        L.oracle_step(t)
        L.compare("B=%d step %d" % (B, t))
    plan.destroy()


# ------------------------------------------------------------------ full-size, sampled blocks
def sample_blocks(n, B, k, seed):
    nb = oracle.nblocks(n, B)
    rng = np.random.default_rng(seed)
    full = nb - 1 if n % B else nb                       # number of full blocks
    pick = np.unique(np.concatenate([[0, full - 1], rng.integers(0, full, k)]))
    return pick, (nb - 1 if n % B else None)


class SampledOracle:
    """Follows `pick` full blocks (treated as one contiguous pseudo-tensor: blocks are
    independent) and, if present, the short last block of a device tensor."""

    def __init__(self, n, B, pick, tail_block, w_dev):
        self.n, self.B, self.pick, self.tail = n, B, pick, tail_block
        idx = (torch.from_numpy(pick).cuda()[:, None] * B + torch.arange(B, device="cuda")[None, :]).reshape(-1)
        self.idx = idx
        self.bidx = torch.from_numpy(pick).cuda()
        self.w = w_dev[idx].cpu().numpy()
        self.st = H.zero_state(self.w.size, B)
        if tail_block is not None:
            self.tsl = slice(tail_block * B, n)
            self.tw = w_dev[self.tsl].cpu().numpy()
            self.tst = H.zero_state(self.tw.size, B)

    def step(self, g_dev, t):
        g = g_dev[self.idx].cpu().numpy()
        H.oracle_adam8(self.w, g, self.st, self.B, t=t)
        if self.tail is not None:
            H.oracle_adam8(self.tw, g_dev[self.tsl].cpu().numpy(), self.tst, self.B, t=t, split=False)

    def compare(self, tag, w_dev, d):
        got = dict(m_q=d["m_q"][self.idx], r_q=d["r_q"][self.idx], N_m=d["N_m"][self.bidx], N_r=d["N_r"][self.bidx])
        e = H.assert_state_equal(tag, got, self.st, w_dev[self.idx], self.w)
        if self.tail is not None:
            got = dict(m_q=d["m_q"][self.tsl], r_q=d["r_q"][self.tsl],
                       N_m=d["N_m"][self.tail:self.tail + 1], N_r=d["N_r"][self.tail:self.tail + 1])
            e = max(e, H.assert_state_equal(tag + " (short last block)", got, self.tst, w_dev[self.tsl], self.tw))
        return e


def device_state(n, B):
    nb = oracle.nblocks(n, B)
    return dict(m_q=torch.full((n,), 127, dtype=torch.uint8, device="cuda"),
                r_q=torch.zeros(n, dtype=torch.uint8, device="cuda"),
                N_m=torch.zeros(nb, device="cuda"), N_r=torch.zeros(nb, device="cuda"))


def check_block_properties(tag, d, n, B):
    """Whole-tensor invariants of Eq. quant1/quant2: the element that attains the block
    maximum is stored as the code of +1 (255) or, for a negative maximum of m, as code 0;
    maxima are finite and non-negative; r codes of a non-zero block include 255."""
    nb = oracle.nblocks(n, B)
    full = n // B
    for key, nkey in (("m_q", "N_m"), ("r_q", "N_r")):
        N = d[nkey]
        assert torch.isfinite(N).all() and (N >= 0).all(), tag
        c = d[key][: full * B].view(full, B)
        has_top = (c == 255).any(dim=1)
        if key == "m_q":
            has_top |= (c == 0).any(dim=1)
        assert bool((has_top | (N[:full] == 0)).all()), "%s: %s block without its maximum code" % (tag, key)
    assert nb == d["N_m"].numel()


def test_config4_one_billion_parameters_sampled(q8, tabs):
    """Config 4: one flat tensor of 10^9 parameters (last block 512 long), Adam, B = 2048,
    5 steps; launch configuration identical to the benchmark's."""
    n, B = 1_000_000_000, 2048
    gen = torch.Generator(device="cuda"); gen.manual_seed(4)
    w = torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen)
    g = torch.empty(n, device="cuda")
    d = device_state(n, B)
    pick, tail = sample_blocks(n, B, 3000, 44)
    assert tail == 488281 and n - tail * B == 512
    so = SampledOracle(n, B, pick, tail, w)
    for t in range(1, 6):
        g.normal_(0.0, 1e-3, generator=gen)
        so.step(g, t)
        q8.adam8bit_step(w, g, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        e = so.compare("config 4 step %d" % t, w, d)
        check_block_properties("config 4 step %d" % t, d, n, B)
    print("config 4: %d sampled blocks, max parameter relative error %.3g" % (pick.size + 1, e))


def test_more_than_2_31_elements(q8, tabs):
    """One tensor of 2^31 + 2^20 + 777 elements (21.5 GB of device memory for w, g and both
    states): element indices beyond 32 bits, sampled blocks on both sides of 2^31 and the
    short last block."""
    n, B = (1 << 31) + (1 << 20) + 777, 2048
    gen = torch.Generator(device="cuda"); gen.manual_seed(31)
    w = torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen)
    g = torch.empty(n, device="cuda")
    d = device_state(n, B)
    nb = oracle.nblocks(n, B)
    pick, tail = sample_blocks(n, B, 600, 45)
    edge = np.array([(1 << 31) // B - 2, (1 << 31) // B - 1, (1 << 31) // B, (1 << 31) // B + 1, nb - 3, nb - 2])
    pick = np.unique(np.concatenate([pick, edge]))
    assert tail == nb - 1 and n - tail * B == 777
    so = SampledOracle(n, B, pick, tail, w)
    for t in range(1, 3):
        g.normal_(0.0, 1e-3, generator=gen)
        so.step(g, t)
        q8.adam8bit_step(w, g, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        so.compare("2^31+ elements step %d" % t, w, d)
    check_block_properties("2^31+ elements", d, n, B)


def test_more_than_2_31_elements_every_entry(q8, tabs):
    """The same tensor of 2^31 + 2^20 + 777 elements, one Adam step, every entry against the
    oracle (the host threads split the blocks): no element index is lost beyond 32 bits."""
    n, B = (1 << 31) + (1 << 20) + 777, 2048
    gen = torch.Generator(device="cuda"); gen.manual_seed(32)
    w = torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen)
    g = torch.empty(n, device="cuda").normal_(0.0, 1e-3, generator=gen)
    d = device_state(n, B)
    chk = H.WholeTensorParity("2^31+ elements", w, B)
    chk.oracle_step(g, 1)
    q8.adam8bit_step(w, g, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=1)
    chk.compare(w, d, "2^31+ elements")
    H.report_parity("2^31 + 2^20 + 777 parameters, B=2048, 1 step, every entry", [chk])


def heavy_tail_grad_device(n, B, scale, gen):
    z = torch.randn(n, device="cuda", generator=gen)
    chi = torch.randn(3, n, device="cuda", generator=gen).pow_(2).sum(0).div_(3.0).sqrt_()
    g = z.div_(chi).mul_(scale)
    nb = -(-n // B)
    start = torch.arange(nb, device="cuda") * B
    length = torch.clamp(n - start, max=B)
    k = torch.clamp(torch.round(0.01 * length.float()), min=1).long()
    first = (torch.rand(nb, device="cuda", generator=gen) * length).long().clamp_(max=B - 1) % length
    for j in range(3):                                   # up to 3 distinct entries per block, evenly spaced
        pos = (first + j * (length // 3 + 1)) % length
        sel = k > j
        g[(start + pos)[sel]] *= 100.0
    return g


def test_config5_full_size_sampled(q8, tabs):
    """Config 5: 64 tensors x 1 562 500 parameters (100 M), Adam, B = 256 (last block 132
    long), Student-t gradients, per-tensor scales 1e-6..1e-1, 1 % outliers x100, 50 steps."""
    nt, n, B = 64, 1_562_500, 256
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    ws = [torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen) for _ in range(nt)]
    gs = [torch.empty(n, device="cuda") for _ in range(nt)]
    ds = [device_state(n, B) for _ in range(nt)]
    scales = [synth.heavy_tail_scale(5, i) for i in range(nt)]
    plan = q8.Plan([dict(w=ws[i], g=gs[i], **ds[i]) for i in range(nt)], B)
    sos = []
    for i in range(nt):
        pick, tail = sample_blocks(n, B, 150, 500 + i)
        assert tail == 6103 and n - tail * B == 132
        sos.append(SampledOracle(n, B, pick, tail, ws[i]))
    worst = 0.0
    for t in range(1, 51):
        for i in range(nt):
            gs[i].copy_(heavy_tail_grad_device(n, B, scales[i], gen))
            sos[i].step(gs[i], t)
        plan.multi_adam8bit_step(tabs[0], tabs[1], **H.ADAM, t=t)
        if t <= 3 or t % 10 == 0:
            for i in range(nt):
                worst = max(worst, sos[i].compare("config 5 tensor %d step %d" % (i, t), ws[i], ds[i]))
    for i in range(nt):
        worst = max(worst, sos[i].compare("config 5 tensor %d final" % i, ws[i], ds[i]))
        check_block_properties("config 5 tensor %d" % i, ds[i], n, B)
    plan.destroy()
    print("config 5: max parameter relative error %.3g" % worst)


# ------------------------------------------------------------------ full size, every entry, every step
def test_config4_one_billion_parameters_every_entry(q8, tabs):
    """Config 4 in the benchmark's launch configuration: one flat tensor of 10^9 parameters
    (488 282 blocks, the last 512 long), Adam, B = 2048, 5 steps.  The oracle advances all
    blocks; codes, block maxima and weights of the whole tensor are compared after each step."""
    n, B = 1_000_000_000, 2048
    gen = torch.Generator(device="cuda"); gen.manual_seed(4)
    w = torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen)
    g = torch.empty(n, device="cuda")
    d = device_state(n, B)
    chk = H.WholeTensorParity("config 4", w, B)
    for t in range(1, 6):
        g.normal_(0.0, 1e-3, generator=gen)
        chk.oracle_step(g, t)
        q8.adam8bit_step(w, g, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        bad = chk.compare(w, d, "config 4 step %d" % t)
        print("config 4 step %d: %d mismatching codes" % (t, bad), flush=True)
    H.report_parity("config 4 (1e9 parameters, B=2048, 5 steps, every entry after every step)", [chk])


def test_config5_full_size_every_entry(q8, tabs):
    """Config 5 at full size in one multi-tensor launch per step: 64 tensors x 1 562 500
    parameters, Adam, B = 256 (last block 132 long), Student-t gradients with per-tensor scales
    1e-6..1e-1 and 1 % outliers x100, 50 steps; every entry compared after every step."""
    nt, n, B = 64, 1_562_500, 256
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    ws = [torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen) for _ in range(nt)]
    gs = [torch.empty(n, device="cuda") for _ in range(nt)]
    ds = [device_state(n, B) for _ in range(nt)]
    scales = [synth.heavy_tail_scale(5, i) for i in range(nt)]
    plan = q8.Plan([dict(w=ws[i], g=gs[i], **ds[i]) for i in range(nt)], B)
    chks = [H.WholeTensorParity("config 5 tensor %d" % i, ws[i], B) for i in range(nt)]
    for t in range(1, 51):
        for i in range(nt):
            gs[i].copy_(heavy_tail_grad_device(n, B, scales[i], gen))
        list(H.pool().map(lambda i: chks[i].oracle_step(gs[i], t, split=False), range(nt)))
        plan.multi_adam8bit_step(tabs[0], tabs[1], **H.ADAM, t=t)
        bad = sum(chks[i].compare(ws[i], ds[i], "config 5 tensor %d step %d" % (i, t)) for i in range(nt))
        if t % 10 == 0 or bad:
            print("config 5 step %d: %d mismatching codes" % (t, bad), flush=True)
    plan.destroy()
    H.report_parity("config 5 (64 x 1 562 500 parameters, B=256, 50 steps, every entry after every step)", chks)


def _by_block_ranges(n, B, fn):
    """fn(element slice, block slice) over disjoint block ranges on the host threads (blocks
    are independent, so the split changes nothing)."""
    nb = oracle.nblocks(n, B)
    nthr = H.host_threads()
    per = -(-nb // nthr)
    parts = [(k * per, min(nb, (k + 1) * per)) for k in range(nthr) if k * per < nb]
    list(H.pool().map(lambda p: fn(slice(p[0] * B, min(n, p[1] * B)), slice(p[0], p[1])), parts))


def test_sgd_quantize_dequantize_one_billion_every_entry(q8, tabs):
    """The other 10^9-element workloads of bench.py (sgd1b, quant1b, dequant1b) in their launch
    configuration, every entry against the oracle: two SGD-momentum steps with coupled decay on
    10^9 parameters, then that tensor quantized stand-alone with both codebooks' rules (signed map,
    and the unsigned map on its absolute values) and dequantized again."""
    n, B, chunk = 1_000_000_000, 2048, 1 << 27
    qs, qu = H.codebooks()
    gen = torch.Generator(device="cuda"); gen.manual_seed(33)
    w_d = torch.empty(n, device="cuda"); g_d = torch.empty(n, device="cuda")
    w_d.uniform_(-0.1, 0.1, generator=gen)
    st_d = {k: torch.from_numpy(v).cuda() for k, v in H.zero_state(n, B, adam=False).items()}
    w_h = w_d.cpu().numpy()
    st_h = H.zero_state(n, B, adam=False)
    g_h = torch.empty(n, dtype=torch.float32, pin_memory=True)

    def same_bits(dev_t, host_a, what):
        for lo in range(0, host_a.size, chunk):
            hi = min(host_a.size, lo + chunk)
            ref = torch.from_numpy(host_a[lo:hi]).cuda()
            a, b = dev_t[lo:hi], ref
            if a.dtype == torch.float32:
                a, b = a.view(torch.int32), b.view(torch.int32)
            bad = int((a != b).sum())
            assert bad == 0, "%s differs in %d entries of [%d, %d)" % (what, bad, lo, hi)

    for t in (1, 2):
        g_d.normal_(0.0, 1e-2, generator=gen)
        q8.sgd8bit_step(w_d, g_d, st_d["m_q"], st_d["N_m"], tabs[0], B, weight_decay=1e-4, **H.SGD)
        g_h.copy_(g_d); torch.cuda.synchronize()
        g_np = g_h.numpy()
        _by_block_ranges(n, B, lambda e, b: oracle.sgd8bit_step(w_h[e], g_np[e], st_h["m_q"][e], st_h["N_m"][b], qs, B,
                                                                H.SGD["alpha"], H.SGD["beta"], 1e-4))
        same_bits(st_d["N_m"], st_h["N_m"], "SGD step %d: block maxima" % t)
        same_bits(st_d["m_q"], st_h["m_q"], "SGD step %d: codes" % t)
        same_bits(w_d, w_h, "SGD step %d: weights" % t)
    del g_d, g_h
    nb = oracle.nblocks(n, B)
    TQ = torch.empty(n, dtype=torch.uint8, device="cuda"); N = torch.empty(nb, device="cuda"); TD = torch.empty(n, device="cuda")
    for signed, q, tab in ((True, qs, tabs[0]), (False, qu, tabs[1])):
        T_h = w_h if signed else np.abs(w_h)
        T_d = w_d if signed else w_d.abs()
        TQ_ref = np.empty(n, np.uint8); N_ref = np.empty(nb, np.float32); TD_ref = np.empty(n, np.float32)

        def one(e, b):
            TQ_ref[e], N_ref[b] = oracle.quantize_blockwise(q, T_h[e], B)
            TD_ref[e] = oracle.dequantize_blockwise(q, TQ_ref[e], N_ref[b], B)
        _by_block_ranges(n, B, one)
        q8.quantize_blockwise(tab, T_d, B, TQ, N)
        q8.dequantize_blockwise(tab, TQ, N, B, TD)
        which = "signed" if signed else "unsigned"
        same_bits(N, N_ref, "quantize (%s map): block maxima" % which)
        same_bits(TQ, TQ_ref, "quantize (%s map): codes" % which)
        same_bits(TD, TD_ref, "dequantize (%s map)" % which)
        del T_d
    H.report("SGD (2 steps), quantize and dequantize (both maps) on 1e9 elements, B=2048: every weight, code, "
             "block maximum and dequantized value identical to the oracle's")


@pytest.mark.parametrize("B", [64, 256, 4096])
def test_block_size_sweep_one_billion_parameters_every_entry(q8, tabs, B):
    """The block-size sweep of bench.py (--block-size on 10^9 parameters) at its two ends and at
    the paper's alternative B = 256: Adam, two steps, every entry against the oracle."""
    n = 1_000_000_000
    gen = torch.Generator(device="cuda"); gen.manual_seed(64 + B)
    w = torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen)
    g = torch.empty(n, device="cuda")
    d = device_state(n, B)
    chk = H.WholeTensorParity("B=%d" % B, w, B)
    for t in (1, 2):
        g.normal_(0.0, 1e-3, generator=gen)
        chk.oracle_step(g, t)
        q8.adam8bit_step(w, g, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
        chk.compare(w, d, "B=%d step %d" % (B, t))
    H.report_parity("1e9 parameters, B=%d, 2 steps, every entry after every step" % B, [chk])
