"""Job counters of the dynamic scheduler are never shared by kernels that can run at the same
time: one long launch overlapped by many short ones on another stream, more streams than the
library has counters, more captured launches than it reserves counters for (the surplus runs
with the fixed assignment of work) -- every result is compared with the CPU oracle."""
import ctypes

import numpy as np
import pytest

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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class Small:
    """A small tensor with its oracle twin."""

    def __init__(self, seed, n, B):
        self.n, self.B, self.seed = n, B, seed
        self.w_ref = synth.uniform_weights(seed, 0, n)
        self.st = H.zero_state(n, B)
        self.g = synth.normal_grad(seed, 0, 1, n, 1e-3)
        self.w, self.gd = dev(self.w_ref), dev(self.g)
        self.d = {k: dev(v) for k, v in self.st.items()}
        self.t = 0

    def launch(self, q8, tabs):
        self.t += 1
        q8.adam8bit_step(self.w, self.gd, self.d["m_q"], self.d["r_q"], self.d["N_m"], self.d["N_r"],
                         tabs[0], tabs[1], self.B, **H.ADAM, t=self.t)

    def check(self, tag):
        for t in range(1, self.t + 1):
            H.oracle_adam8(self.w_ref, self.g, self.st, self.B, t=t)
        H.assert_state_equal(tag, self.d, self.st, self.w, self.w_ref)


def test_long_launch_overlapped_by_many_short_launches(q8, tabs):
    """One launch over 10^9 parameters on stream A (about 2.5 ms of kernel time) while 150
    launches over small tensors are issued on stream B: the long kernel keeps its counter
    to itself however many launches pass on other streams.  All results oracle-exact, the
    big tensor over every entry."""
    n, B = 1_000_000_000, 2048
    gen = torch.Generator(device="cuda"); gen.manual_seed(41)
    w = torch.empty(n, device="cuda").uniform_(-0.1, 0.1, generator=gen)
    g = torch.empty(n, device="cuda").normal_(0.0, 1e-3, generator=gen)
    d = dict(m_q=torch.full((n,), 127, dtype=torch.uint8, device="cuda"), r_q=torch.zeros(n, dtype=torch.uint8, device="cuda"),
             N_m=torch.zeros(-(-n // B), device="cuda"), N_r=torch.zeros(-(-n // B), device="cuda"))
    chk = H.WholeTensorParity("long launch", w, B)
    smalls = [Small(1000 + k, 20_000 + 777 * k, 2048 if k % 2 else 256) for k in range(3)]
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    # first launches of a process load code and query occupancy: keep them out of the overlap
    warm = [Small(1100 + k, 5_000, 2048 if k % 2 else 256) for k in range(2)]
    for s in warm:
        s.launch(q8, tabs)
    torch.cuda.synchronize()
    overlapped = 0
    for t in range(1, 3):
        chk.oracle_step(g, t)
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(sa):
            start.record()
            q8.adam8bit_step(w, g, d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM, t=t)
            end.record()
        first_b, last_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(sb):
            first_b.record()
            for k in range(150):
                smalls[k % 3].launch(q8, tabs)
            last_b.record()
        torch.cuda.synchronize()
        overlapped += start.elapsed_time(first_b) < start.elapsed_time(end)      # stream B started before the long kernel ended
        bad = chk.compare(w, d, "long launch step %d" % t)
        assert bad == 0
    for k, s in enumerate(smalls):
        s.check("small tensor %d after %d launches" % (k, s.t))
    assert overlapped >= 1, "stream B never overlapped the long launch: the test did not exercise what it is for"
    H.report_parity("long launch overlapped by 300 short launches (1e9 parameters, every entry)", [chk])


def test_more_streams_than_counters(q8, tabs):
    """260 streams created through the HIP runtime, more than the 192 per-stream counters: the
    library synchronizes the device once and starts its stream table afresh; results stay exact."""
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipStreamCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipStreamDestroy.argtypes = [ctypes.c_void_p]
    handles = []
    for _ in range(260):
        h = ctypes.c_void_p()
        assert hip.hipStreamCreate(ctypes.byref(h)) == 0
        handles.append(h.value)
    assert len(set(handles)) == 260
    smalls = [Small(2000 + k, 9_000 + 1111 * k, 2048) for k in range(4)]
    torch.cuda.synchronize()
    try:
        for i, h in enumerate(handles):
            s = torch.cuda.ExternalStream(h)
            with torch.cuda.stream(s):
                smalls[i % 4].launch(q8, tabs)
            if i % 4 == 3:
                torch.cuda.synchronize()             # the four tensors are stepped from different streams in turn
        torch.cuda.synchronize()
        for k, s in enumerate(smalls):
            s.check("tensor %d stepped from 65 different streams" % k)
    finally:
        torch.cuda.synchronize()
        for h in handles:
            hip.hipStreamDestroy(ctypes.c_void_p(h))


def test_more_captures_than_reserved_counters(q8, tabs):
    """80 separately captured launches, more than the 64 (capture, stream) counters the library
    reserves: the surplus launches run with the fixed assignment of work.  Replayed three times
    on alternating streams next to eager launches; every tensor oracle-exact.  The tensors are
    large enough (6 M parameters, 740 jobs for at most 512 workgroups) for several rounds."""
    n, B = 6_000_000 + 333, 2048
    ntens = 4
    ws, gds, ds, refs = [], [], [], []
    for k in range(ntens):
        w_ref = synth.uniform_weights(3000 + k, 0, n)
        st = H.zero_state(n, B)
        g = synth.normal_grad(3000 + k, 0, 1, n, 1e-3)
        ws.append(dev(w_ref)); gds.append(dev(g)); ds.append({kk: dev(v) for kk, v in st.items()})
        refs.append((w_ref, st, g))
    steps = [0] * ntens

    def launch(k):
        steps[k] += 1
        d = ds[k]
        q8.adam8bit_step(ws[k], gds[k], d["m_q"], d["r_q"], d["N_m"], d["N_r"], tabs[0], tabs[1], B, **H.ADAM)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch(0)                                     # eager warm-up fills the library's per-kernel caches
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graphs = []
    for i in range(80):
        gph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gph):
            q8.adam8bit_step(ws[i % ntens], gds[i % ntens], ds[i % ntens]["m_q"], ds[i % ntens]["r_q"],
                             ds[i % ntens]["N_m"], ds[i % ntens]["N_r"], tabs[0], tabs[1], B, **H.ADAM)
        graphs.append(gph)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        # graphs that touch different tensors run at the same time on two streams; graphs of one
        # tensor are kept in order by the synchronization after each group of four
        for i0 in range(0, 80, ntens):
            for j in range(ntens):
                with torch.cuda.stream(s1 if j % 2 else s2):
                    graphs[i0 + j].replay()
                steps[(i0 + j) % ntens] += 1
            torch.cuda.synchronize()
        launch(rep % ntens)                            # eager work between the rounds of replays
        torch.cuda.synchronize()
    for k in range(ntens):
        w_ref, st, g = refs[k]
        for _ in range(steps[k]):
            H.oracle_adam8(w_ref, g, st, B)
        H.assert_state_equal("tensor %d after %d steps" % (k, steps[k]), ds[k], st, ws[k], w_ref)


def test_fixed_order_fallback_for_every_kernel(q8, tabs):
    """After test_more_captures_than_reserved_counters every reserved counter is taken, so each
    further captured launch runs with the fixed assignment of work: SGD, the stand-alone
    quantizer and the bfloat16 Adam step, replayed twice, against the oracle."""
    import oracle
    n, B = 5_000_000 + 1234, 2048
    qs, _ = H.codebooks()
    # make sure the reserved counters are used up even when this test runs alone
    side = torch.cuda.Stream()
    dummy = Small(4100, 50_000, 2048)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dummy.launch(q8, tabs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for _ in range(70):
        gph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gph):
            q8.adam8bit_step(dummy.w, dummy.gd, dummy.d["m_q"], dummy.d["r_q"], dummy.d["N_m"], dummy.d["N_r"],
                             tabs[0], tabs[1], dummy.B, **H.ADAM)
        del gph
    # SGD
    w_ref = synth.uniform_weights(4000, 0, n); g = synth.normal_grad(4000, 0, 1, n, 1e-2)
    st = H.zero_state(n, B, adam=False)
    w, gd = dev(w_ref), dev(g)
    d = {k: dev(v) for k, v in st.items()}
    # quantizer
    T = synth.normal_grad(4001, 0, 1, n, 1.0)
    Td = dev(T); TQ = torch.empty(n, dtype=torch.uint8, device="cuda"); N = torch.empty(oracle.nblocks(n, B), device="cuda")
    # bfloat16 Adam
    wb_ref = synth.bf16_bits(synth.uniform_weights(4002, 0, n)); gb = synth.bf16_bits(synth.normal_grad(4002, 0, 1, n, 1e-3))
    stb = H.zero_state(n, B)
    wb = torch.from_numpy(wb_ref.view(np.int16).copy()).cuda().view(torch.bfloat16)
    gbd = torch.from_numpy(gb.view(np.int16).copy()).cuda().view(torch.bfloat16)
    db = {k: dev(v) for k, v in stb.items()}
    with torch.cuda.stream(side):                    # eager warm-up of the three kernels (they are not in any cache yet)
        q8.sgd8bit_step(w, gd, d["m_q"], d["N_m"], tabs[0], B, **H.SGD, weight_decay=1e-4)
        q8.quantize_blockwise(tabs[0], Td, B, TQ, N)
        q8.adam8bit_step_bf16(wb, gbd, db["m_q"], db["r_q"], db["N_m"], db["N_r"], tabs[0], tabs[1], B, **H.ADAM)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    H.oracle_sgd8(w_ref, g, st, B, wd=1e-4)
    H.oracle_adam8(wb_ref, gb, stb, B, bf16=True)
    gph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gph):
        q8.sgd8bit_step(w, gd, d["m_q"], d["N_m"], tabs[0], B, **H.SGD, weight_decay=1e-4)
        q8.quantize_blockwise(tabs[0], Td, B, TQ, N)
        q8.adam8bit_step_bf16(wb, gbd, db["m_q"], db["r_q"], db["N_m"], db["N_r"], tabs[0], tabs[1], B, **H.ADAM)
    for rep in range(2):
        TQ.fill_(3); N.fill_(-1.0)
        gph.replay()
        torch.cuda.synchronize()
        H.oracle_sgd8(w_ref, g, st, B, wd=1e-4)
        H.oracle_adam8(wb_ref, gb, stb, B, bf16=True)
        H.assert_state_equal("sgd replay %d" % rep, d, st, w, w_ref)
        TQ_ref, N_ref = oracle.quantize_blockwise(qs, T, B)
        assert np.array_equal(TQ.cpu().numpy(), TQ_ref) and np.array_equal(N.cpu().numpy().view(np.uint32), N_ref.view(np.uint32))
        for k in stb:
            a, b = db[k].cpu().numpy(), stb[k]
            if a.dtype == np.float32:
                a, b = a.view(np.uint32), b.view(np.uint32)
            assert np.array_equal(a, b), (rep, k)
        assert np.array_equal(wb.view(torch.int16).cpu().numpy().view(np.uint16), wb_ref)


def test_per_thread_default_stream_counts_once_per_thread(q8, tabs):
    """Two host threads launch on the per-thread default stream (the same handle value, two
    different streams): each thread gets its own counter.  Called through the C ABI directly."""
    import threading
    L = q8.lib()
    PER_THREAD = 2                                     # hipStreamPerThread
    n, B, steps = (1 << 20) + 555, 2048, 12
    items = [Small(5000 + k, n, B) for k in range(2)]
    torch.cuda.synchronize()
    errors = []

    def worker(k):
        try:
            s = items[k]
            for t in range(1, steps + 1):
                rc = L.q8_adam8bit_step(s.w.data_ptr(), s.gd.data_ptr(), s.d["m_q"].data_ptr(), s.d["r_q"].data_ptr(),
                                        s.d["N_m"].data_ptr(), s.d["N_r"].data_ptr(), tabs[0].data_ptr(), tabs[1].data_ptr(),
                                        n, B, H.ADAM["alpha"], H.ADAM["beta1"], H.ADAM["beta2"], H.ADAM["eps"], 0.0, t, 0, PER_THREAD)
                assert rc == 0, rc
            s.t = steps
        except Exception as e:
            errors.append(e)
    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for k, s in enumerate(items):
        s.check("thread %d on its per-thread default stream" % k)
