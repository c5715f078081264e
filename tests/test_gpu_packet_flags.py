"""mc_reduce_update_packets: one resident kernel sums packets in their order of arrival, each when
its device-memory flag says it has landed (Section 4.2, pipelined reductions).  Three situations,
each compared bit for bit with the oracle's whole step: every flag already set; a producer on a
second stream delivering and signalling packets while the reducer runs; and flags that never come,
where the kernel must give up after its bounded number of polls, return normally, leave every
packet either untouched or complete, and finish on a later call once the flags are set.
No kernel here can wait for ever: every poll loop is bounded by spin_limit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_1711_00705_amd import mc  # noqa: E402
from paper_1711_00705_amd import workloads as wl  # noqa: E402
import gpu_harness as gh  # noqa: E402

SIZES = [700_000, 36, 1_500_000, 4097, 800_001]      # 3,004,135 elements, ragged end
K, P = 4, 4
LR, MU, WD = 0.1, 0.9, 1e-4
# twice the compute units is the most the entry point accepts (512 on a whole MI355X)
N_BLOCKS = min(512, 2 * torch.cuda.get_device_properties(0).multi_processor_count) if torch.cuda.is_available() else 512


def _packets(bounds, packet_elems):
    """Per colour, ranges of packet_elems elements; arrival order interleaves the colours."""
    per_colour = []
    for c in range(len(bounds) - 1):
        lo, hi = int(bounds[c]), int(bounds[c + 1])
        per_colour.append([(b, min(hi, b + packet_elems)) for b in range(lo, hi, packet_elems)])
    out = []
    for j in range(max(len(p) for p in per_colour)):
        for p in per_colour:
            if j < len(p):
                out.append(p[j])
    return out


class Case:
    def __init__(self, packet_elems=256 * 300):
        self.L = mc.Layout(SIZES, K)
        self.O = oracle.Layout(SIZES, K)
        N = self.L.N
        self.order = wl.rotation_order(K, P)
        self.x_host = [oracle.pack(self.O, wl.contribution_tensors(SIZES, p)) for p in range(P)]
        self.w_host = oracle.pack(self.O, wl.weight_tensors(SIZES))
        rng = np.random.Generator(np.random.PCG64(3))
        self.v_host = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
        self.pk = _packets(self.L.colour_bounds(), packet_elems)
        self.n = len(self.pk)
        self.pk_dev = torch.tensor(np.array(self.pk, dtype=np.int64).reshape(-1), device="cuda")
        self.ready = torch.full((self.n,), 0xDEAD, dtype=torch.int32, device="cuda")
        self.progress = torch.full((N_BLOCKS + mc.PACKETS_STATUS_WORDS,), 77, dtype=torch.int32, device="cuda")
        self.spec = mc.update_spec(LR, MU, WD)
        w, v = self.w_host.copy(), self.v_host.copy()
        self.g_ref = oracle.reduce_update(self.O, self.x_host, w, v, LR, MU, WD, order=self.order)
        self.w_ref, self.v_ref = w, v

    def fresh_state(self):
        self.w = gh.to_dev(self.w_host)
        self.v = gh.to_dev(self.v_host)
        self.g = gh.dev_empty(self.L.N)

    def reduce(self, x_dev, spin_limit, stream, arrivals=1):
        mc.reduce_update_packets(self.L, [x.data_ptr() for x in x_dev], self.order, self.g.data_ptr(),
                                 self.w.data_ptr(), self.v.data_ptr(), self.spec, self.pk_dev.data_ptr(), self.n,
                                 self.ready.data_ptr(), arrivals, spin_limit, self.progress.data_ptr(), N_BLOCKS, stream)

    def signal(self, j, stream, arrivals=1):
        """The flag of packet j counts the elements that have landed: set it to its final value."""
        b, e = self.pk[j]
        mc.packet_signal(self.ready.data_ptr(), j, arrivals * (e - b), stream)

    def check_complete(self, what):
        pr = self.progress.cpu().numpy()
        assert np.all(pr[:N_BLOCKS] == self.n), f"{what}: some workgroup did not finish: {pr[:N_BLOCKS].min()} of {self.n}"
        assert pr[N_BLOCKS + 1] == 0, f"{what}: a packet descriptor was rejected"
        gh.assert_bits(self.g[:self.L.N].cpu().numpy(), self.g_ref, f"{what}: g")
        gh.assert_bits(self.w.cpu().numpy(), self.w_ref, f"{what}: w")
        gh.assert_bits(self.v.cpu().numpy(), self.v_ref, f"{what}: v")


def test_all_flags_already_set():
    c = Case()
    c.fresh_state()
    s = gh.stream_handle()
    x_dev = [gh.to_dev(x) for x in c.x_host]
    print(f"packets: {c.n} packets, all flags set beforehand", flush=True)
    mc.packets_reset(c.ready.data_ptr(), c.n, c.progress.data_ptr(), N_BLOCKS, s)
    for j in range(c.n):
        c.signal(j, s)
    c.reduce(x_dev, 1000, s)
    torch.cuda.synchronize()
    assert c.progress.cpu().numpy()[N_BLOCKS] == 0, "no workgroup should have had to give up"
    c.check_complete("flags pre-set")


def test_flags_that_never_come_then_resume():
    c = Case()
    c.fresh_state()
    s = gh.stream_handle()
    x_dev = [gh.to_dev(x) for x in c.x_host]
    print(f"packets: {c.n} packets, no flag set, spin limit 5", flush=True)
    mc.packets_reset(c.ready.data_ptr(), c.n, c.progress.data_ptr(), N_BLOCKS, s)
    c.reduce(x_dev, 5, s)
    torch.cuda.synchronize()                       # must return: the wait is bounded
    pr = c.progress.cpu().numpy()
    assert np.all(pr[:N_BLOCKS] == 0) and pr[N_BLOCKS] == N_BLOCKS, "every workgroup gives up before packet 0"
    gh.assert_bits(c.w.cpu().numpy(), c.w_host, "weights untouched after giving up")
    gh.assert_bits(c.v.cpu().numpy(), c.v_host, "momentum untouched after giving up")
    # half of the packets arrive: a second call gets exactly that far
    half = c.n // 2
    for j in range(half):
        c.signal(j, s)
    c.reduce(x_dev, 5, s)
    torch.cuda.synchronize()
    pr = c.progress.cpu().numpy()
    assert np.all(pr[:N_BLOCKS] == half), "every workgroup stops at the first packet without a flag"
    done = np.zeros(c.L.N, bool)
    for (b, e) in c.pk[:half]:
        done[b:e] = True
    w_now = c.w.cpu().numpy()
    gh.assert_bits(w_now[done], c.w_ref[done], "packets that arrived are complete")
    gh.assert_bits(w_now[~done], c.w_host[~done], "packets that did not arrive are untouched")
    # the rest arrives
    for j in range(half, c.n):
        c.signal(j, s)
    c.reduce(x_dev, 5, s)
    torch.cuda.synchronize()
    c.check_complete("resumed after giving up twice")


def test_producer_on_a_second_stream():
    c = Case()
    c.fresh_state()
    main = torch.cuda.current_stream()
    prod = torch.cuda.Stream()
    s, ps = int(main.cuda_stream), int(prod.cuda_stream)
    arriving = [2, 3]
    src = {p: gh.to_dev(c.x_host[p]) for p in arriving}
    x_dev = [gh.to_dev(c.x_host[p]) if p not in arriving else gh.dev_empty(c.L.N) for p in range(P)]   # NaN canaries
    print(f"packets: {c.n} packets delivered by copies on a second stream", flush=True)
    mc.packets_reset(c.ready.data_ptr(), c.n, c.progress.data_ptr(), N_BLOCKS, s)
    prod.wait_stream(main)
    c.reduce(x_dev, 20000, s, arrivals=len(arriving))     # about 20 ms of patience in total per workgroup
    for j, (b, e) in enumerate(c.pk):
        for p in arriving:                          # each delivery adds the elements it wrote to the packet's flag
            mc.packet_deliver(x_dev[p].data_ptr() + 4 * b, src[p].data_ptr() + 4 * b, e - b,
                              c.ready.data_ptr() + 4 * j, ps)
    done = torch.cuda.Event()
    done.record(prod)
    main.wait_event(done)
    c.reduce(x_dev, 20000, s, arrivals=len(arriving))     # finishes whatever the first launch gave up on
    torch.cuda.synchronize()
    print(f"workgroups that gave up in the first launch: {int(c.progress.cpu().numpy()[N_BLOCKS])} of {N_BLOCKS}", flush=True)
    c.check_complete("producer on a second stream")


def test_rejects_before_launch():
    c = Case()
    c.fresh_state()
    x = [gh.to_dev(xh) for xh in c.x_host]
    ptrs = [t.data_ptr() for t in x]
    args = dict(packets_ptr=c.pk_dev.data_ptr(), n_packets=c.n, ready_ptr=c.ready.data_ptr(), arrivals=1,
                spin_limit=1, progress_ptr=c.progress.data_ptr())

    def code(**kw):
        a = dict(args, n_blocks=N_BLOCKS)
        a.update(kw)
        try:
            mc.reduce_update_packets(c.L, ptrs, None, None, c.w.data_ptr(), c.v.data_ptr(), c.spec, **a)
        except mc.McError as e:
            return e.code
        return mc.OK
    assert code(n_blocks=0) == mc.ERR_INVALID_ARG
    assert code(arrivals=0) == mc.ERR_INVALID_ARG
    assert code(n_blocks=mc.PACKETS_MAX_BLOCKS + 1) == mc.ERR_INVALID_ARG
    assert code(packets_ptr=None) == mc.ERR_INVALID_ARG
    assert code(ready_ptr=None) == mc.ERR_INVALID_ARG
    assert code(progress_ptr=None) == mc.ERR_INVALID_ARG
    # a grid that could not be resident beside the producer's kernels is refused, not left to time out
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    room = torch.zeros(2 * cus + 1 + mc.PACKETS_STATUS_WORDS, dtype=torch.int32, device="cuda")
    assert code(n_blocks=2 * cus, progress_ptr=room.data_ptr()) == mc.OK
    assert code(n_blocks=2 * cus + 1, progress_ptr=room.data_ptr()) == mc.ERR_LIMIT
    big = mc.Layout([1000] * 40, 40)
    with pytest.raises(mc.McError) as e:
        mc.reduce_update_packets(big, ptrs, None, None, c.w.data_ptr(), c.v.data_ptr(), c.spec, n_blocks=8, **args)
    assert e.value.code == mc.ERR_LIMIT
    torch.cuda.synchronize()


def test_deliver_counts_elements_and_delay_returns():
    n = 5 * 1024 + 3                               # ragged: the last workgroup copies 3 words one by one
    src = gh.to_dev(np.arange(n, dtype=np.float32))
    dst = gh.dev_empty(n + 8)
    flag = torch.zeros(2, dtype=torch.int32, device="cuda")
    s = gh.stream_handle()
    mc.delay(200, s)
    mc.packet_deliver(dst.data_ptr(), src.data_ptr(), n, flag.data_ptr() + 4, s)
    torch.cuda.synchronize()
    assert flag.cpu().tolist() == [0, n]
    out = dst.cpu().numpy()
    gh.assert_bits(out[:n], np.arange(n, dtype=np.float32), "delivered words")
    assert np.all(out[n:].view(np.uint32) == 0xFFFFFFFF), "wrote past the packet"
